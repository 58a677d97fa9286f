"""Build step: compile csrc/kvb.hip for gfx950 into libkvb.so next to this file.

hipcc cross-compiles without a GPU.  Run as ``python -m paper_2605_19049_amd.build``.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "kvb.hip")
LIB = os.path.join(HERE, "libkvb.so")

HIPCC_FLAGS = [
    "-std=c++20", "-O3", "--offload-arch=gfx950",
    # hipcc must not emit packed-fp32 VALU instructions on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # keep the single-lane ticket atomics as written: the wave-aggregating rewrite reads
    # the result back at once, which would make the wave wait for its whole state tile
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
    "-shared", "-fPIC", "-I" + os.path.join(ROOT, "include"),
]


def build_lib(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".%d.tmp" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + os.environ.get("KVB_EXTRA_HIPCC_FLAGS", "").split() + ["-o", tmp, SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose="-v" in sys.argv))
