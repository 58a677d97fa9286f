"""Builds tests/c_caller/kvb_c_caller, the plain-C caller of the kvb ABI (test infrastructure).

gcc only: the program is C99, includes the HIP runtime's C API for hipMalloc / hipMemcpy, and
links libkvb.so, the oracle's libgdn_oracle.so and libamdhip64.  Library paths are recorded
relative to the executable, so the built tree can be moved as a whole."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
SRC = os.path.join(HERE, "kvb_c_caller.c")
EXE = os.path.join(HERE, "kvb_c_caller")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build(force=False):
    sys.path.insert(0, ROOT)
    from oracle import gdn
    from paper_2605_19049_amd import build as kvb_build
    if not os.path.exists(kvb_build.LIB):
        kvb_build.build_lib()
    gdn.build_lib()
    deps = [SRC, os.path.join(ROOT, "include", "kvb.h")]
    if not force and os.path.exists(EXE) and all(os.path.getmtime(EXE) >= os.path.getmtime(d) for d in deps):
        return EXE
    tmp = EXE + ".%d.tmp" % os.getpid()
    subprocess.check_call([
        "gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-Wno-unused-parameter",
        "-I", os.path.join(ROOT, "include"), "-isystem", os.path.join(ROCM, "include"),
        "-o", tmp, SRC,
        "-L", os.path.join(ROOT, "paper_2605_19049_amd"), "-lkvb",
        "-L", os.path.join(ROOT, "oracle"), "-lgdn_oracle",
        "-L", os.path.join(ROCM, "lib"), "-lamdhip64", "-lm",
        "-Wl,-rpath,$ORIGIN/../../paper_2605_19049_amd", "-Wl,-rpath,$ORIGIN/../../oracle",
        "-Wl,-rpath," + os.path.join(ROCM, "lib"),
    ])
    os.replace(tmp, EXE)
    return EXE


if __name__ == "__main__":
    print(build(force=True))
