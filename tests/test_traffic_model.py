"""The byte counter behind the roofline numbers, pinned to the paper's Table 2 and
Eq. 6 / 9 / 17-19 (fp16 vectors, fp32 state, one head, as the table's caption states)."""
import math
import os

import pytest

from paper_2605_19049_amd import traffic as tr

GOLD = {}
for _l in open(os.path.join(os.path.dirname(__file__), "golden", "paper_memory_model.txt")):
    if _l.strip() and not _l.startswith("#"):
        GOLD[_l.split()[0]] = float(_l.split()[1])


@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("m", [4, 16, 32, 64])
def test_table2_chunkwise_and_recurrent_rows(d, m):
    lay = tr.Layout(dk=d, dv=d, r=1, in_bytes=2, u_bytes=2, G_bytes=2, out_bytes=2, gate_bytes=2)
    rd, wr = tr.chunk_cycle_rw(lay, m)
    assert rd == pytest.approx(4 * (1 + 1 / m) * d * d + 2 * (m + 4) * d + m + 5)   # Table 2, Chunkwise, Read
    assert wr == pytest.approx(4 * d * d / m + 6 * d + 2)                           # Table 2, Chunkwise, Write
    rrd, rwr = tr.recurrent_rw(lay)
    assert rrd == 4 * d * d + 6 * d + 4 and rwr == 4 * d * d + 2 * d                 # Table 2, Recurrent
    exact = (rrd + rwr) / (rd + wr)                                                 # Eq. 17, first line
    assert exact == pytest.approx((8 * d * d + 8 * d + 4) /
                                  (4 * d * d + 8 * d * d / m + 2 * m * d + 14 * d + m + 7))
    assert exact == pytest.approx(tr.paper_speedup_chunkwise(d, m), rel=2e-2)       # its approximation


def test_flush_cost_matches_section_3_2():
    d, m = 128, 16
    lay = tr.Layout(dk=d, dv=d, r=1, in_bytes=2, u_bytes=2, G_bytes=0, out_bytes=2, gate_bytes=2)
    assert tr.total(tr.flush_rw(lay, m)) == 8 * d * d + 4 * m * d                   # "8d^2 + 4md"


def test_eq6_peaks_at_two_sqrt_d():
    d = 128
    best = max(range(1, 200), key=lambda m: tr.paper_speedup_chunkwise(d, m))
    assert abs(best - 2 * math.sqrt(d)) < 1
    assert 2 * math.sqrt(d) == pytest.approx(GOLD["opt_buffer_d128"], abs=5e-3)


def test_verify_model_and_state_size():
    assert tr.paper_speedup_verify(128, 8) == pytest.approx(GOLD["verify_speedup_8_drafts_approx"], rel=0.1)
    assert tr.paper_speedup_verify(10 ** 6, 8) == pytest.approx(3.0, rel=1e-3)     # (m+1)/3 limit
    assert 32 * tr.KVB.state == GOLD["state_MB_per_request_layer"] * 2 ** 20


def test_kvb_layout_numbers_used_by_the_bench():
    """bf16 tokens, fp32 state / u / G / out, two v-heads per qk-head, d = 128."""
    rd, wr = tr.decode_rw(tr.KVB, 0)
    assert rd + wr == 65536 + 520 + 1156
    assert tr.KVB.record == 644
    assert tr.total(tr.flush_rw(tr.KVB, 16)) == 2 * 65536 + 16 * 644
    assert tr.total(tr.chunk_cycle_rw(tr.KVB, 16)) == pytest.approx(67212 + 644 * 7.5 + (131072 + 10304) / 16)


def test_16bit_storage_regime_layout():
    """fp16 (or bf16) inputs, records and outputs, two v-heads per qk-head, d = 128: a record is
    128 B of shared key + 256 B of delta value + 4 B of G; with r = 1 and 2-byte gates and G it is
    the layout of the paper's Table 2 (checked above through the same counter)."""
    lay = tr.layout("f16", "f16", "f16")
    assert lay.record == 128 + 256 + 4
    assert lay.token_in == 2 * 128 + 256 + 8 and lay.token_out == 256 + 388
    assert tr.layout("bf16", "f32", "f32") == tr.KVB and tr.KVB.record == 644
    paper = tr.Layout(r=1, in_bytes=2, u_bytes=2, G_bytes=2, out_bytes=2, gate_bytes=2)
    d, m = 128, 16
    rd, wr = tr.chunk_cycle_rw(paper, m)
    assert rd == pytest.approx(4 * (1 + 1 / m) * d * d + 2 * (m + 4) * d + m + 5)       # Table 2, Chunkwise
    # the same regime in this library's format (fp32 gates and G, keys shared by two heads) moves
    # fewer bytes per token than the table's single-head count, and 2-3 % fewer than fp32 records
    assert tr.total(tr.fused_cycle_rw(lay, 16)) < rd + wr
    assert 0.96 < tr.total(tr.fused_cycle_rw(lay, 16)) / tr.total(tr.fused_cycle_rw(tr.KVB, 16)) < 0.98
