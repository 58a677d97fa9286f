"""GPU parity of the 16-bit storage regimes against the (unchanged) fp64 recurrence oracle.

The paper's implementation keeps a fp32 state and fp16 vectors and records (Sec. 4.1; the
caption of the GDN memory-profile table in App. A.2).  Three things are selectable here:
  * fp16 inputs (q, k, v and the buffered keys) with fp32 records and outputs: held to the
    same bound as bf16 inputs, 2e-3 of the oracle's RMS, plus the regression guard;
  * 16-bit delta-value records: held to harness.TOL_REC (derived from the rounding of a stored
    u, see tests/test_record_precision.py, which emulates exactly that on the CPU);
  * 16-bit outputs: the fp32 result rounded once, so an element may be off by one unit
    roundoff of its own magnitude on top of the bound of the rest of the configuration.
"""
import numpy as np
import pytest
import torch

import harness as H
from harness import oracle
from paper_2605_19049_amd import kvb, synth
from test_gpu_parity import _direct_case, _tree_case, _verify_case, say
from test_record_precision import chunkwise_one_head

pytestmark = pytest.mark.gpu


def _decode_errs(d, in_dtype, rec_dtype, out_dtype, B, Hk, Hv, C, steps, fused, seed, block_size=None):
    rng = np.random.default_rng(seed)
    S0 = H.prefix_state(rng, B, Hk, Hv, d, d, in_dtype, 16)
    tok = synth.token_stream(rng, B, steps, Hk, Hv, d, d, in_dtype)
    lay = H.Layer(B, Hk, Hv, d, d, cap=C, in_dtype=in_dtype, rec_dtype=rec_dtype, out_dtype=out_dtype,
                  block_size=block_size)
    o, u, S, _ = H.run_decode(lay, S0, tok, C, fused=fused)
    o_ref, u_ref, S_ref = oracle.kvb_decode_expected(S0, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"])
    assert lay.spare_clean() and not lay.status().any()
    return H.rel_err(o, o_ref, lay.out_unit), H.rel_err(u, u_ref), H.rel_err(S, S_ref)


# --------------------------------------------------------------------------- fp16 inputs, fp32 records
@pytest.mark.parametrize("d, B, Hk, Hv, C, steps", [
    (128, 5, 2, 4, 16, 40), (128, 2, 1, 2, 32, 70), (128, 2, 1, 1, 64, 70), (128, 2, 2, 4, 128, 130),
    (64, 3, 2, 2, 8, 20), (32, 3, 1, 3, 8, 20), (64, 2, 1, 2, 100, 110)])
@pytest.mark.parametrize("fused", [False, True])
def test_fp16_inputs_decode_flush(d, B, Hk, Hv, C, steps, fused):
    e = _decode_errs(d, "f16", "f32", "f32", B, Hk, Hv, C, steps, fused, seed=300 + d + C)
    say("fp16 d=%d C=%d fused=%s rel err out/u/state: %.2e %.2e %.2e" % ((d, C, fused) + e))
    H.check(e, "f16")


@pytest.mark.parametrize("T", [1, 4, 8])
def test_fp16_inputs_verify_and_trees(T):
    e = _verify_case(B=6, Hk=2, Hv=4, d=128, C=16, cap=16 + T - 1, T=T, in_dtype="f16", seed=330 + T)
    say("fp16 verify T=%d rel err out/u/state: %.2e %.2e %.2e" % ((T,) + e))
    H.check(e, "f16")
    if T > 1:
        e = _tree_case(B=6, Hk=2, Hv=4, d=128, C=16, cap=16 + T - 1, T=T, in_dtype="f16", seed=340 + T)
        say("fp16 verify_tree T=%d rel err out/u/state: %.2e %.2e %.2e" % ((T,) + e))
        H.check(e, "f16")


def test_fp16_inputs_verify_other_kernels():
    """The 64-record window, no state, paged records, and the vector-ALU kernel (d = 64)."""
    H.check(_verify_case(B=4, Hk=1, Hv=2, d=128, C=64, cap=72, T=8, in_dtype="f16", seed=351), "f16")
    H.check(_verify_case(B=4, Hk=2, Hv=4, d=128, C=16, cap=20, T=4, in_dtype="f16", seed=352, kv_only=True), "f16")
    H.check(_tree_case(B=4, Hk=2, Hv=4, d=128, C=16, cap=24, T=8, in_dtype="f16", seed=353, block_size=8), "f16")
    H.check(_verify_case(B=3, Hk=2, Hv=2, d=64, C=8, cap=12, T=4, in_dtype="f16", seed=354), "f16")


@pytest.mark.parametrize("d, Lmax", [(128, 64), (128, 7), (128, 128), (128, 100), (64, 33), (32, 16)])
def test_fp16_inputs_direct(d, Lmax):
    e = _direct_case(B=5, Hk=2, Hv=4, d=d, Lmax=Lmax, cap=max(Lmax, 8), in_dtype="f16", seed=360 + Lmax)
    say("fp16 direct d=%d Lmax=%d rel err out/u/decode/state: %.2e %.2e %.2e %.2e" % ((d, Lmax) + e))
    H.check(e, "f16")


def test_fp16_flush_split_is_exact_to_fp32_rounding():
    """kvb_flush with fp16 keys multiplies them with a two-way fp16 split of the fp32 factor
    (22 significand bits).  One record per request on a zero state, v scaled over the range fp16
    values cover: every element of S = k^T u must match the oracle to a few fp32 roundings."""
    rng = np.random.default_rng(371)
    scales = np.array([2.0 ** -6, 2.0 ** -3, 1.0, 8.0, 64.0])
    B, Hk, Hv, d = len(scales), 1, 2, 128
    tok = synth.token_stream(rng, B, 1, Hk, Hv, d, d, "f16")
    tok["v"] = synth.round_to_fp16((tok["v"] * scales[:, None, None, None]).astype(np.float32))
    tok["g"][:] = -0.125
    S0 = np.zeros((B, Hv, d, d), np.float32)
    for cap in (16, 64):
        lay = H.Layer(B, Hk, Hv, d, d, cap=cap, in_dtype="f16")
        _, _, S, _ = H.run_decode(lay, S0, tok, cap, final_flush=True)
        _, _, S_ref = oracle.kvb_decode_expected(S0, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"])
        # a piece below 2^-14 is held with the absolute spacing 2^-24 of the fp16 subnormals: large
        # elements keep 22 bits, small ones an absolute accuracy at the level of a fp32 rounding of
        # values of order one (a dropped second piece would be 2^-12 of the element: 500 times the bound)
        err = np.abs(S - S_ref)
        excess = err - (2.0 ** -21 * np.abs(S_ref) + 2.0 ** -24)
        say("fp16 flush, one record, cap %d: worst error %.2e (element %.2e), bound 2^-21 |x| + 2^-24"
            % (cap, err.max(), np.abs(S_ref).reshape(-1)[err.argmax()]))
        assert excess.max() <= 0.0


# --------------------------------------------------------------------------- 16-bit records
@pytest.mark.parametrize("in_dtype", ["f16", "bf16"])
@pytest.mark.parametrize("d, B, Hk, Hv, C, steps, fused", [
    (128, 5, 2, 4, 16, 40, True), (128, 5, 2, 4, 16, 40, False), (128, 2, 1, 2, 64, 70, True),
    (128, 2, 2, 4, 128, 130, False), (64, 3, 2, 2, 8, 20, True), (32, 3, 1, 3, 8, 20, False)])
def test_16bit_records_decode_flush(in_dtype, d, B, Hk, Hv, C, steps, fused):
    e = _decode_errs(d, in_dtype, in_dtype, "f32", B, Hk, Hv, C, steps, fused, seed=400 + d + C)
    say("%s records d=%d C=%d fused=%s rel err out/u/state: %.2e %.2e %.2e" % ((in_dtype, d, C, fused) + e))
    H.check(e, in_dtype, in_dtype)


@pytest.mark.parametrize("in_dtype", ["f16", "bf16"])
def test_16bit_records_verify_tree_direct(in_dtype):
    t = dict(in_dtype=in_dtype, rec_dtype=in_dtype)
    H.check(_verify_case(B=6, Hk=2, Hv=4, d=128, C=16, cap=19, T=4, seed=431, **t), in_dtype, in_dtype, "verify")
    H.check(_verify_case(B=4, Hk=1, Hv=2, d=128, C=64, cap=72, T=8, seed=432, **t), in_dtype, in_dtype, "verify, long buffer")
    H.check(_tree_case(B=6, Hk=2, Hv=4, d=128, C=16, cap=23, T=8, seed=433, **t), in_dtype, in_dtype, "tree")
    H.check(_tree_case(B=4, Hk=2, Hv=4, d=128, C=16, cap=20, T=4, seed=434, kv_only=True, block_size=8, **t),
            in_dtype, in_dtype, "tree, no state, paged")
    H.check(_verify_case(B=3, Hk=2, Hv=2, d=64, C=8, cap=12, T=4, seed=435, **t), in_dtype, in_dtype, "verify d=64")
    for Lmax in (64, 128, 20):
        e = _direct_case(B=5, Hk=2, Hv=4, d=128, Lmax=Lmax, cap=max(Lmax, 8), seed=440 + Lmax, **t)
        say("%s records direct Lmax=%d rel err out/u/decode/state: %.2e %.2e %.2e %.2e" % ((in_dtype, Lmax) + e))
        H.check(e, in_dtype, in_dtype, "direct")
    H.check(_direct_case(B=4, Hk=1, Hv=2, d=32, Lmax=16, cap=16, seed=445, **t), in_dtype, in_dtype, "direct d=32")


@pytest.mark.parametrize("in_dtype", ["f16", "bf16"])
def test_16bit_records_are_what_later_steps_read(in_dtype):
    """The rule of include/kvb.h: a 16-bit record holds the delta value rounded to nearest, and
    every later use -- the token's own output, the following tokens, the state update -- reads
    that rounded value.  The CPU emulation of exactly this rule (fp64 otherwise) must then agree
    with the GPU far better than the bound that is held against the unrounded oracle: all but a
    few outputs to fp32 accuracy (a delta value that sits on a rounding boundary may fall the
    other way in fp32 than in fp64; such a flip moves what follows by one unit of that record)."""
    rng = np.random.default_rng(450)
    B, Hk, Hv, d, C, steps = 2, 1, 2, 128, 16, 48
    tok = synth.token_stream(rng, B, steps, Hk, Hv, d, d, in_dtype)
    S0 = np.zeros((B, Hv, d, d), np.float32)
    lay = H.Layer(B, Hk, Hv, d, d, cap=C, in_dtype=in_dtype, rec_dtype=in_dtype)
    o, u, S, _ = H.run_decode(lay, S0, tok, C, fused=True)
    f = lambda x: x.astype(np.float64)
    emu = np.stack([np.stack([chunkwise_one_head(f(tok["q"][b, :, h // (Hv // Hk)]), f(tok["k"][b, :, h // (Hv // Hk)]),
                                                 f(tok["v"][b, :, h]), f(tok["g"][b, :, h]), f(tok["beta"][b, :, h]),
                                                 C, in_dtype) for h in range(Hv)], axis=1) for b in range(B)])
    rms = np.sqrt((emu ** 2).mean())
    diff = np.abs(o - emu) / rms
    say("%s records vs their CPU emulation: median %.1e, 99th percentile %.1e, max %.1e of the output RMS"
        % (in_dtype, np.median(diff), np.quantile(diff, 0.99), diff.max()))
    assert np.quantile(diff, 0.9) < 1e-5
    assert diff.max() < H.TOL_REC[in_dtype]


# --------------------------------------------------------------------------- 16-bit outputs
@pytest.mark.parametrize("in_dtype", ["f16", "bf16"])
def test_16bit_outputs_are_the_fp32_outputs_rounded_once(in_dtype):
    """Same inputs with fp32 and with 16-bit outputs: the 16-bit output must be the fp32 output
    rounded to nearest even, bit for bit, in every call."""
    rng = np.random.default_rng(460)
    B, Hk, Hv, d, C, T = 4, 2, 4, 128, 16, 4
    S0 = H.prefix_state(rng, B, Hk, Hv, d, d, in_dtype, 8)
    tok = synth.token_stream(rng, B, 20, Hk, Hv, d, d, in_dtype)
    vtok = synth.token_stream(rng, B, T, Hk, Hv, d, d, in_dtype)
    dtok = synth.token_stream(rng, B, 40, Hk, Hv, d, d, in_dtype)
    lens = synth.context_lengths(rng, B, 1, 40)
    got = {}
    for out_dtype in ("f32", in_dtype):
        lay = H.Layer(B, Hk, Hv, d, d, cap=C + T, in_dtype=in_dtype, out_dtype=out_dtype, scale=0.25)
        o, _, _, _ = H.run_decode(lay, S0, tok, C, fused=True, final_flush=False)
        vo = lay.new_out(B, T, Hv, d)
        lay.verify(T, H.upload_tokens(vtok, in_dtype), vo)
        lay2 = H.Layer(B, Hk, Hv, d, d, cap=40, in_dtype=in_dtype, out_dtype=out_dtype, with_state=False)
        do = lay2.new_out(B, 40, Hv, d, fill=0.0)
        lay2.direct(H.dev(lens), 40, H.upload_tokens(dtok, in_dtype), do)
        torch.cuda.synchronize()
        got[out_dtype] = (torch.from_numpy(o), vo.cpu(), do.cpu())
    for wide, narrow, name in zip(got["f32"], got[in_dtype], ("decode", "verify", "direct")):
        want = wide.to(H.TORCH_DT[in_dtype]).float()
        assert torch.equal(narrow.float(), want), name
    # and against the oracle, with the one rounding allowed for
    o_ref, _, _ = oracle.kvb_decode_expected(S0, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"], scale=0.25)
    e = H.rel_err(got[in_dtype][0].numpy(), o_ref, H.UNIT[in_dtype])
    say("%s outputs: rel err beyond one rounding %.2e" % (in_dtype, e))
    H.check(e, in_dtype)


# --------------------------------------------------------------------------- the paper's regime at full size
@pytest.mark.parametrize("in_dtype", ["f16", "bf16"])
def test_paper_storage_regime_qwen3next_full(in_dtype):
    """The decode workload at full size (B=64, 16/32 heads, d=128, C=16, 256 steps) with 16-bit
    inputs, records and outputs and a fp32 state: fp16 is the paper's own configuration."""
    w = synth.WORKLOADS["qwen3next_decode"]
    rng = np.random.default_rng(w.seed)
    S0 = H.prefix_state(rng, w.B, w.Hk, w.Hv, w.dk, w.dv, in_dtype, w.prefix)
    tok = synth.token_stream(rng, w.B, w.steps, w.Hk, w.Hv, w.dk, w.dv, in_dtype)
    lay = H.Layer(w.B, w.Hk, w.Hv, w.dk, w.dv, cap=w.cap, in_dtype=in_dtype, rec_dtype=in_dtype, out_dtype=in_dtype)
    o, u, S, fills = H.run_decode(lay, S0, tok, w.C, fused=True)
    o_ref, u_ref, S_ref = oracle.kvb_decode_expected(S0, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"])
    e = (H.rel_err(o, o_ref, lay.out_unit), H.rel_err(u, u_ref), H.rel_err(S, S_ref))
    say("qwen3next_decode, %s inputs / records / outputs: rel err out/u/state: %.2e %.2e %.2e" % ((in_dtype,) + e))
    H.check(e, in_dtype, in_dtype)
    assert fills == [(t + 1) % w.C for t in range(w.steps)]


def test_fp16_inputs_full_size_verify_and_direct():
    """The speculative-verification and short-context workloads at full size with fp16 inputs."""
    w = synth.WORKLOADS["spec_verify"]
    e = _verify_case(w.B, w.Hk, w.Hv, w.dk, w.C, w.cap, w.T, "f16", w.seed)
    say("spec_verify fp16 rel err out/u/state: %.2e %.2e %.2e" % e)
    H.check(e, "f16")
    w = synth.WORKLOADS["short_direct"]
    e = _direct_case(w.B, w.Hk, w.Hv, w.dk, w.Lmax, w.cap + 1, "f16", w.seed, rec_dtype="f16", out_dtype="f16")
    say("short_direct fp16 inputs / records / outputs rel err out/u/decode/state: %.2e %.2e %.2e %.2e" % e)
    H.check(e, "f16", "f16")


# --------------------------------------------------------------------------- the kernel timer
def test_a_call_that_does_not_launch_disarms_its_timer():
    """An armed timer belongs to the very next call: if that call returns before launching (bad
    arguments, an empty batch), the timer is disarmed and does not attach itself to a later one."""
    lay = H.Layer(2, 1, 2, 128, 128, cap=4, in_dtype="bf16")
    rng = np.random.default_rng(470)
    tok = H.step_view(H.upload_tokens(synth.token_stream(rng, 2, 1, 1, 2, 128, 128, "bf16"), "bf16"), 0)
    out = lay.new_out(2, 2, 128)
    tm = kvb.Timer()
    tm.arm()
    st = lay.ds.c(True)
    rc = kvb.kvb_decode(lay.shape(B=0), st, lay.slot, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"], out)
    assert rc == kvb.OK
    lay.decode(tok, out)            # must not carry the timer
    torch.cuda.synchronize()
    with pytest.raises(kvb.KvbError):
        tm.us()                     # its events were never recorded
    tm.arm()
    lay.decode(tok, out)
    assert 0.0 < tm.us() < 1e5
    tm.close()
