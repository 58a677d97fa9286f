"""CPU-side checks of the C ABI: the library loads, exports every symbol the header
declares, and rejects bad arguments before touching the GPU (no compute calls here)."""
import ctypes
import os
import re
import subprocess

import pytest

from paper_2605_19049_amd import kvb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "kvb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvb_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = header_functions()
    assert set(names) == set(kvb.EXPORTS)
    L = kvb.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_version_and_error_strings():
    assert kvb.version() == 120
    assert kvb.strerror(kvb.OK) == "ok"
    assert "invalid" in kvb.strerror(kvb.EINVAL)
    assert "unsupported" in kvb.strerror(kvb.EUNSUPPORTED)
    assert "unknown" in kvb.strerror(-99)


def test_struct_layout_matches_header():
    assert ctypes.sizeof(kvb.KvbShape) == 10 * 4
    assert kvb.KvbShape.rec_dtype.offset == 8 * 4 and kvb.KvbShape.scale.offset == 9 * 4
    assert kvb.KvbStore.n_slots.offset == 6 * 8 and kvb.KvbStore.flags.offset == 6 * 8 + 4
    assert kvb.KvbStore.block_table.offset == 7 * 8 and kvb.KvbStore.block_size.offset == 8 * 8
    assert kvb.KvbStore.n_blocks.offset == 8 * 8 + 8
    assert ctypes.sizeof(kvb.KvbStore) == 10 * 8


A = 0x1000  # a fake, well-aligned "device address": validation must fail before it is used


def _store(**kw):
    d = dict(state=A, buf_k=A, buf_u=A, buf_G=A, fill=A, status=A, n_slots=4)
    d.update(kw)
    return kvb.store(**d)


def _decode(sh, st, **kw):
    d = dict(slot=A, q=A, k=A, v=A, g=A, beta=A, out=A)
    d.update(kw)
    return kvb.kvb_decode(sh, st, d["slot"], d["q"], d["k"], d["v"], d["g"], d["beta"], d["out"],
                          stream=0, check=False)


GOOD = dict(B=2, Hk=2, Hv=4, dk=128, dv=128, cap=16, in_dtype=kvb.BF16)


@pytest.mark.parametrize("bad, code", [
    (dict(B=-1), kvb.EINVAL), (dict(Hk=0), kvb.EINVAL), (dict(Hk=3), kvb.EINVAL),
    (dict(cap=0), kvb.EINVAL), (dict(cap=129), kvb.EINVAL), (dict(dk=0), kvb.EINVAL),
    (dict(dk=96, dv=96), kvb.EUNSUPPORTED), (dict(dk=128, dv=64), kvb.EUNSUPPORTED),
    (dict(in_dtype=3), kvb.EUNSUPPORTED), (dict(out_dtype=3), kvb.EUNSUPPORTED), (dict(rec_dtype=3), kvb.EUNSUPPORTED),
    # 16-bit records and outputs take the inputs' own 16-bit type
    (dict(in_dtype=kvb.BF16, out_dtype=kvb.F16), kvb.EUNSUPPORTED),
    (dict(in_dtype=kvb.BF16, rec_dtype=kvb.F16), kvb.EUNSUPPORTED),
    (dict(in_dtype=kvb.F16, rec_dtype=kvb.BF16), kvb.EUNSUPPORTED),
    (dict(in_dtype=kvb.F32, out_dtype=kvb.BF16), kvb.EUNSUPPORTED),
    (dict(in_dtype=kvb.F32, rec_dtype=kvb.F16), kvb.EUNSUPPORTED),
])
def test_bad_shapes_are_rejected(bad, code):
    sh = kvb.shape(**{**GOOD, **bad})
    assert _decode(sh, _store()) == code


def test_bad_pointers_are_rejected():
    sh = kvb.shape(**GOOD)
    assert _decode(sh, _store(buf_u=None)) == kvb.EINVAL
    assert _decode(sh, _store(fill=None)) == kvb.EINVAL
    assert _decode(sh, _store(n_slots=0)) == kvb.EINVAL
    assert _decode(sh, _store(state=A + 4)) == kvb.EINVAL      # misaligned
    assert _decode(sh, _store(), q=None) == kvb.EINVAL
    assert _decode(sh, _store(), out=A + 8) == kvb.EINVAL
    assert _decode(sh, _store(), slot=None) == kvb.EINVAL
    assert _decode(sh, _store(), g=A + 2) == kvb.EINVAL


def test_empty_batch_is_a_noop_everywhere():
    sh = kvb.shape(**{**GOOD, "B": 0})
    st = _store()
    assert _decode(sh, st) == kvb.OK
    assert kvb.kvb_flush(sh, st, A, None, 1, stream=0, check=False) == kvb.OK
    assert kvb.kvb_verify(sh, st, A, 4, A, A, A, A, A, A, stream=0, check=False) == kvb.OK
    assert kvb.kvb_direct(sh, st, A, A, 8, A, A, A, A, A, A, stream=0, check=False) == kvb.OK


def test_flush_verify_direct_argument_ranges():
    sh = kvb.shape(**GOOD)
    st = _store()
    assert kvb.kvb_flush(sh, st, A, None, 0, stream=0, check=False) == kvb.EINVAL
    assert kvb.kvb_flush(sh, st, A, None, 17, stream=0, check=False) == kvb.EINVAL
    assert kvb.kvb_flush(sh, _store(state=None), A, None, 1, stream=0, check=False) == kvb.EINVAL
    assert kvb.kvb_flush(kvb.shape(**{**GOOD, "B": 0}), _store(state=None), A, A, 1, stream=0, check=False) == kvb.OK
    for T in (0, 9, 17):
        assert kvb.kvb_verify(sh, st, A, T, A, A, A, A, A, A, stream=0, check=False) == kvb.EINVAL
    for Lmax in (0, 17, 129):
        assert kvb.kvb_direct(sh, st, A, A, Lmax, A, A, A, A, A, A, stream=0, check=False) == kvb.EINVAL
    assert kvb.kvb_direct(sh, st, A, None, 8, A, A, A, A, A, A, stream=0, check=False) == kvb.EINVAL


def test_paged_store_argument_ranges():
    sh = kvb.shape(**GOOD)   # cap = 16
    ok = dict(block_table=A, block_size=8, max_blocks=2, n_blocks=64)
    assert _decode(kvb.shape(**{**GOOD, "B": 0}), _store(**ok)) == kvb.OK
    for bad in (dict(block_size=12), dict(block_size=4), dict(block_size=256), dict(max_blocks=1),
                dict(max_blocks=0), dict(max_blocks=17), dict(n_blocks=0), dict(block_table=A + 2)):
        assert _decode(sh, _store(**{**ok, **bad})) == kvb.EINVAL, bad
    # without a table the three sizes are ignored
    assert _decode(kvb.shape(**{**GOOD, "B": 0}), _store(block_size=3, max_blocks=99, n_blocks=-1)) == kvb.OK


def test_tree_verify_and_compact_argument_ranges():
    sh = kvb.shape(**GOOD)
    st = _store()
    tok = (A, A, A, A, A, A)
    assert kvb.kvb_verify_tree(sh, st, A, 4, None, *tok, stream=0, check=False) == kvb.EINVAL
    assert kvb.kvb_verify_tree(sh, st, A, 4, A + 2, *tok, stream=0, check=False) == kvb.EINVAL
    for T in (0, 9, 17):
        assert kvb.kvb_verify_tree(sh, st, A, T, A, *tok, stream=0, check=False) == kvb.EINVAL
        assert kvb.kvb_compact(sh, st, A, T, A, A, stream=0, check=False) == kvb.EINVAL
    assert kvb.kvb_compact(sh, st, A, 4, None, A, stream=0, check=False) == kvb.EINVAL
    assert kvb.kvb_compact(sh, st, A, 4, A, None, stream=0, check=False) == kvb.EINVAL
    empty = kvb.shape(**{**GOOD, "B": 0})
    assert kvb.kvb_verify_tree(empty, st, A, 4, A, *tok, stream=0, check=False) == kvb.OK
    assert kvb.kvb_compact(empty, st, A, 4, A, A, stream=0, check=False) == kvb.OK


def test_decode_flush_argument_ranges():
    sh = kvb.shape(**GOOD)
    args = (A, A, A, A, A, A, A)
    assert kvb.kvb_decode_flush(sh, _store(), *args, 0, stream=0, check=False) == kvb.EINVAL
    assert kvb.kvb_decode_flush(sh, _store(), *args, 17, stream=0, check=False) == kvb.EINVAL
    assert kvb.kvb_decode_flush(sh, _store(state=None), *args, 4, stream=0, check=False) == kvb.EINVAL
    assert kvb.kvb_decode_flush(kvb.shape(**{**GOOD, "B": 0}), _store(), *args, 4, stream=0, check=False) == kvb.OK


def test_check_flag_raises():
    sh = kvb.shape(**{**GOOD, "cap": 0})
    with pytest.raises(kvb.KvbError) as e:
        kvb.kvb_flush(sh, _store(), A, None, 1, stream=0)
    assert e.value.code == kvb.EINVAL


C_PROBE = r"""
#include <stdio.h>
#include <stddef.h>
#include "kvb.h"
int main(void)
{
    printf("%zu %zu %zu %zu\n", sizeof(kvb_shape), offsetof(kvb_shape, out_dtype), offsetof(kvb_shape, rec_dtype),
           offsetof(kvb_shape, scale));
    printf("%zu %zu %zu %zu %zu %zu %zu\n", sizeof(kvb_store), offsetof(kvb_store, buf_u), offsetof(kvb_store, fill),
           offsetof(kvb_store, n_slots), offsetof(kvb_store, flags), offsetof(kvb_store, block_table),
           offsetof(kvb_store, n_blocks));
    printf("%d %d %d %d %d %d\n", KVB_VERSION, KVB_F32, KVB_BF16, KVB_F16, KVB_STORE_STREAM, KVB_STORE_RESIDENT);
    return 0;
}
"""


def test_header_is_plain_c_and_agrees_with_the_binding(tmp_path):
    """include/kvb.h compiles as strict C99 (it is the boundary: no C++ in it), and the struct
    layout a C caller sees is the one the ctypes binding marshals."""
    src = tmp_path / "probe.c"
    src.write_text(C_PROBE)
    exe = tmp_path / "probe"
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror",
                           "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src)])
    lines = subprocess.check_output([str(exe)], text=True).splitlines()
    sh = [int(x) for x in lines[0].split()]
    st = [int(x) for x in lines[1].split()]
    co = [int(x) for x in lines[2].split()]
    assert sh == [ctypes.sizeof(kvb.KvbShape), kvb.KvbShape.out_dtype.offset, kvb.KvbShape.rec_dtype.offset,
                  kvb.KvbShape.scale.offset]
    assert st == [ctypes.sizeof(kvb.KvbStore), kvb.KvbStore.buf_u.offset, kvb.KvbStore.fill.offset,
                  kvb.KvbStore.n_slots.offset, kvb.KvbStore.flags.offset, kvb.KvbStore.block_table.offset,
                  kvb.KvbStore.n_blocks.offset]
    assert co == [kvb.version(), kvb.F32, kvb.BF16, kvb.F16, kvb.STORE_STREAM, kvb.STORE_RESIDENT]
