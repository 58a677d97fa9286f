"""Build step: compile csrc/*.hip for gfx950 into libkvb.so next to this file.

One object per translation unit, compiled side by side, then one link.  hipcc cross-compiles
without a GPU.  Run as ``python -m paper_2605_19049_amd.build``.
"""
import os
import shutil
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
SOURCES = ["kvb_api.hip", "kvb_step_bf16.hip", "kvb_step_bf16_r16.hip", "kvb_step_f16.hip", "kvb_step_f16_r16.hip",
           "kvb_step_f32.hip", "kvb_verify_bf16.hip", "kvb_verify_f16.hip", "kvb_flush.hip", "kvb_direct.hip"]
LIB = os.path.join(HERE, "libkvb.so")

HIPCC_FLAGS = [
    "-std=c++20", "-O3", "--offload-arch=gfx950",
    # hipcc must not emit packed-fp32 VALU instructions on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # keep the single-lane ticket atomics as written: the wave-aggregating rewrite reads
    # the result back at once, which would make the wave wait for its whole state tile
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
    # leading scalar kernel arguments arrive in SGPRs at wave launch (kvb_step_kernel uses it)
    "-mllvm", "-amdgpu-kernarg-preload-count=4",
    "-fPIC", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def _clean(text):
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    return "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l)


def build_lib(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra = os.environ.get("KVB_EXTRA_HIPCC_FLAGS", "").split()
    # objects go to a scratch folder inside the package (ignored by git), removed afterwards
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    work = tempfile.mkdtemp(prefix="obj_", dir=os.path.join(HERE, "_build"))
    try:
        procs = []
        for src in SOURCES:
            obj = os.path.join(work, src + ".o")
            cmd = [hipcc] + HIPCC_FLAGS + extra + ["-c", "-o", obj, os.path.join(CSRC, src)]
            if verbose:
                print(" ".join(cmd), flush=True)
            procs.append((src, obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs, failed = [], []
        for src, obj, proc in procs:
            out = _clean(proc.communicate()[0])
            if proc.returncode != 0:
                failed.append("%s:\n%s" % (src, out))
            elif verbose and out.strip():
                print(out)
            objs.append(obj)
        if failed:
            raise RuntimeError("hipcc failed:\n" + "\n".join(failed))
        tmp = os.path.join(work, "libkvb.so")
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
        if verbose:
            print(" ".join(link), flush=True)
        proc = subprocess.run(link, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if proc.returncode != 0:
            raise RuntimeError("link failed:\n" + _clean(proc.stdout))
        final_tmp = LIB + ".%d.tmp" % os.getpid()
        shutil.copyfile(tmp, final_tmp)
        os.replace(final_tmp, LIB)
    finally:
        shutil.rmtree(work, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose="-v" in sys.argv))
