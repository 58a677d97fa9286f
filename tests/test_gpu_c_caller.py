"""The C ABI driven from a plain C99 program (tests/c_caller/kvb_c_caller.c): hipMalloc'ed
buffers, kvb_decode_flush / kvb_verify / kvb_flush on the default stream, results compared
inside the program with the fp64 oracle.  No Python and no PyTorch on that path."""
import importlib.util
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def _builder():
    spec = importlib.util.spec_from_file_location("c_caller_build", os.path.join(HERE, "c_caller", "build.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_c_caller_compiles_as_c99_and_links():
    exe = _builder().build()
    assert os.access(exe, os.X_OK)


@pytest.mark.gpu
def test_c_caller_matches_the_oracle():
    exe = _builder().build()   # (built beforehand by __graft_entry__.build(); compiled here only if missing)
    run = subprocess.run([exe], capture_output=True, text=True, timeout=110)
    print(run.stdout, run.stderr)
    assert run.returncode == 0, (run.returncode, run.stdout, run.stderr)
    assert "fill/status clean: yes" in run.stdout
