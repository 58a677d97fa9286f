"""GPU parity: every kvb call against the fp64 recurrence oracle, through the C ABI.

Metric: max |gpu - oracle| / RMS(oracle) over all compared values; bound 1e-5 for the
all-fp32 workload and 2e-3 for bf16 inputs with fp32 state.
"""
import numpy as np
import pytest
import torch

import harness as H
from harness import oracle
from paper_2605_19049_amd import kvb, synth

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def ragged_warmup(layer, fills, wtok):
    """Bring request b's buffer to fills[b] records by decoding its first fills[b] warm-up
    tokens; step j only carries the requests that still need a record (slot subsets)."""
    dt = H.upload_tokens(wtok, layer.in_dtype)
    for j in range(int(fills.max(initial=0))):
        idx = np.nonzero(fills > j)[0]
        ii = torch.from_numpy(idx).to(layer.device)
        tok = {n: x[ii, j].contiguous() for n, x in dt.items()}
        out = layer.new_out(len(idx), layer.Hv, layer.dv)
        layer.decode(tok, out, slot=layer.slot[ii].contiguous(), B=len(idx))
    torch.cuda.synchronize()
    assert np.array_equal(layer.fill(), fills)


# --------------------------------------------------------------------------- decode + flush
@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("C", [8, 1, 2, 4, 32])
def test_tiny_fp32_decode_flush(C, fused):
    """Workload 1: all fp32, B=1, 2 heads, d=32, 64-token prefix, 32 steps; any chunk size
    gives the same outputs (chunk-size invariance)."""
    w = synth.WORKLOADS["tiny_fp32"]
    rng = np.random.default_rng(w.seed)
    S0 = H.prefix_state(rng, w.B, w.Hk, w.Hv, w.dk, w.dv, "f32", w.prefix)
    tok = synth.token_stream(rng, w.B, w.steps, w.Hk, w.Hv, w.dk, w.dv, "f32")
    lay = H.Layer(w.B, w.Hk, w.Hv, w.dk, w.dv, cap=C, in_dtype="f32")
    o, u, S, fills = H.run_decode(lay, S0, tok, C, fused=fused)
    o_ref, u_ref, S_ref = oracle.kvb_decode_expected(S0, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"])
    e = (H.rel_err(o, o_ref), H.rel_err(u, u_ref), H.rel_err(S, S_ref))
    say("tiny_fp32 C=%d fused=%s rel err out/u/state: %.2e %.2e %.2e" % ((C, fused) + e))
    H.check(e, "f32")
    assert fills == [(t + 1) % C for t in range(w.steps)]
    assert not lay.status().any()


@pytest.mark.parametrize("d, in_dtype, B, Hk, Hv, C, steps", [
    (128, "bf16", 5, 2, 4, 16, 40),
    (128, "f32", 2, 1, 2, 16, 20),
    (64, "bf16", 3, 2, 2, 8, 20),
    (64, "f32", 2, 1, 1, 8, 12),
    (32, "bf16", 3, 1, 3, 8, 20),
    (128, "bf16", 2, 1, 1, 64, 70),
    (128, "bf16", 2, 2, 4, 128, 130),
    (64, "bf16", 2, 1, 2, 100, 110),     # records beyond the 64-record window at the smaller head sizes
    (32, "f32", 2, 1, 1, 128, 130),
])
@pytest.mark.parametrize("fused", [False, True])
def test_decode_flush_shapes(d, in_dtype, B, Hk, Hv, C, steps, fused):
    rng = np.random.default_rng(100 + d + C)
    S0 = H.prefix_state(rng, B, Hk, Hv, d, d, in_dtype, 16)
    tok = synth.token_stream(rng, B, steps, Hk, Hv, d, d, in_dtype)
    lay = H.Layer(B, Hk, Hv, d, d, cap=C, in_dtype=in_dtype, scale=d ** -0.5)
    o, u, S, _ = H.run_decode(lay, S0, tok, C, fused=fused)
    o_ref, u_ref, S_ref = oracle.kvb_decode_expected(S0, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"],
                                                     scale=d ** -0.5)
    e = (H.rel_err(o, o_ref), H.rel_err(u, u_ref), H.rel_err(S, S_ref))
    say("d=%d %s C=%d fused=%s rel err out/u/state: %.2e %.2e %.2e" % ((d, in_dtype, C, fused) + e))
    H.check(e, in_dtype)


@pytest.mark.parametrize("fused", [False, True])
def test_qwen3next_decode_full(fused):
    """Workload 2 at full size: B=64, 16/32 heads, d=128, bf16, C=16, 256 steps; as
    kvb_decode + kvb_flush and as the single-kernel kvb_decode_flush."""
    w = synth.WORKLOADS["qwen3next_decode"]
    rng = np.random.default_rng(w.seed)
    S0 = H.prefix_state(rng, w.B, w.Hk, w.Hv, w.dk, w.dv, w.in_dtype, w.prefix)
    tok = synth.token_stream(rng, w.B, w.steps, w.Hk, w.Hv, w.dk, w.dv, w.in_dtype)
    lay = H.Layer(w.B, w.Hk, w.Hv, w.dk, w.dv, cap=w.cap, in_dtype=w.in_dtype)
    o, u, S, fills = H.run_decode(lay, S0, tok, w.C, fused=fused)
    o_ref, u_ref, S_ref = oracle.kvb_decode_expected(S0, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"])
    e = (H.rel_err(o, o_ref), H.rel_err(u, u_ref), H.rel_err(S, S_ref))
    say("qwen3next_decode fused=%s rel err out/u/state: %.2e %.2e %.2e" % ((fused,) + e))
    H.check(e, "bf16")
    assert fills == [(t + 1) % w.C for t in range(w.steps)]


def _scattered(B, seed):
    """Layer keyword arguments that put the B requests into random slots of a larger store."""
    n_slots = B + 3
    slots = np.random.default_rng(seed).permutation(n_slots)[:B].astype(np.int32)
    return dict(n_slots=n_slots, slots=slots)


# --------------------------------------------------------------------------- verify
def _verify_case(B, Hk, Hv, d, C, cap, T, in_dtype, seed, fill_hi=None, kv_only=False, block_size=None,
                 scatter=False, rec_dtype="f32", out_dtype="f32"):
    rng = np.random.default_rng(seed)
    fill_hi = C - 1 if fill_hi is None else fill_hi
    S0 = np.zeros((B, Hv, d, d), np.float32) if kv_only else H.prefix_state(rng, B, Hk, Hv, d, d, in_dtype, 16)
    fills = synth.buffer_fills(rng, B, 0, fill_hi)
    wtok = synth.token_stream(rng, B, max(1, fill_hi), Hk, Hv, d, d, in_dtype)
    vtok = synth.token_stream(rng, B, T, Hk, Hv, d, d, in_dtype)
    acc = synth.accepted_lengths(rng, B, T)
    lay = H.Layer(B, Hk, Hv, d, d, cap=cap, in_dtype=in_dtype, block_size=block_size, rec_dtype=rec_dtype,
                  out_dtype=out_dtype, **(_scattered(B, seed) if scatter else {}))
    lay.set_state(S0)
    ragged_warmup(lay, fills, wtok)
    # oracle: true state after the warm-up tokens
    _, _, S_true, _ = oracle.gdn_sequence(S0, wtok["q"], wtok["k"], wtok["v"], wtok["g"], wtok["beta"], lens=fills)
    o_ref, u_ref, S_acc = oracle.kvb_verify_expected(S_true, vtok["q"], vtok["k"], vtok["v"], vtok["g"],
                                                     vtok["beta"], acc)
    state_before = lay.ds.state.clone()
    out = lay.new_out(B, T, Hv, d, fill=float("nan"))
    lay.verify(T, H.upload_tokens(vtok, in_dtype), out, use_state=not kv_only)
    torch.cuda.synchronize()
    assert torch.equal(lay.ds.state, state_before), "kvb_verify wrote the state"
    assert np.array_equal(lay.fill(), fills), "kvb_verify changed fill"
    e_out = H.rel_err(H.host(out), o_ref, lay.out_unit)
    # draft records sit at f..f+T-1
    u_got = np.stack([lay.u_records(b, fills[b], fills[b] + T) for b in range(B)])  # [B,Hv,T,d]
    e_u = H.rel_err(u_got.transpose(0, 2, 1, 3), u_ref)
    # commit accepted prefix; flush the requests that reached C; then fold everything
    lay.flush(C, accepted=H.dev(acc))
    torch.cuda.synchronize()
    m = fills + acc
    assert np.array_equal(lay.fill(), np.where(m >= C, 0, m))
    lay.flush(1)
    torch.cuda.synchronize()
    e_S = H.rel_err(lay.get_state(), S_acc)
    assert not lay.status().any()
    assert lay.spare_clean()
    return e_out, e_u, e_S


def _tree_case(B, Hk, Hv, d, C, cap, T, in_dtype, seed, kind="random", kv_only=False, block_size=None,
               scatter=False, rec_dtype="f32", out_dtype="f32"):
    """kvb_verify_tree + kvb_compact + kvb_flush against the oracle run along every root path."""
    rng = np.random.default_rng(seed)
    fill_hi = min(C - 1, cap - T)
    S0 = np.zeros((B, Hv, d, d), np.float32) if kv_only else H.prefix_state(rng, B, Hk, Hv, d, d, in_dtype, 16)
    fills = synth.buffer_fills(rng, B, 0, fill_hi)
    wtok = synth.token_stream(rng, B, max(1, fill_hi), Hk, Hv, d, d, in_dtype)
    vtok = synth.token_stream(rng, B, T, Hk, Hv, d, d, in_dtype)
    parent = synth.draft_trees(rng, B, T, kind)
    leaf, path, plen = synth.accepted_paths(rng, parent)
    lay = H.Layer(B, Hk, Hv, d, d, cap=cap, in_dtype=in_dtype, block_size=block_size, rec_dtype=rec_dtype,
                  out_dtype=out_dtype, **(_scattered(B, seed) if scatter else {}))
    lay.set_state(S0)
    ragged_warmup(lay, fills, wtok)
    _, _, S_true, _ = oracle.gdn_sequence(S0, wtok["q"], wtok["k"], wtok["v"], wtok["g"], wtok["beta"], lens=fills)
    o_ref, u_ref, S_acc = oracle.kvb_verify_tree_expected(S_true, vtok["q"], vtok["k"], vtok["v"], vtok["g"],
                                                          vtok["beta"], parent, accepted_leaf=leaf)
    state_before = lay.ds.state.clone()
    out = lay.new_out(B, T, Hv, d, fill=float("nan"))
    lay.verify_tree(T, H.dev(parent), H.upload_tokens(vtok, in_dtype), out, use_state=not kv_only)
    torch.cuda.synchronize()
    assert torch.equal(lay.ds.state, state_before), "kvb_verify_tree wrote the state"
    assert np.array_equal(lay.fill(), fills), "kvb_verify_tree changed fill"
    e_out = H.rel_err(H.host(out), o_ref, lay.out_unit)
    u_got = np.stack([lay.u_records(b, fills[b], fills[b] + T) for b in range(B)])
    e_u = H.rel_err(u_got.transpose(0, 2, 1, 3), u_ref)
    # accepted root path to the front, commit it, fold everything
    lay.compact(T, H.dev(path), H.dev(plen))
    lay.flush(C, accepted=H.dev(plen))
    torch.cuda.synchronize()
    m = fills + plen
    assert np.array_equal(lay.fill(), np.where(m >= C, 0, m))
    lay.flush(1)
    torch.cuda.synchronize()
    e_S = H.rel_err(lay.get_state(), S_acc)
    assert not lay.status().any()
    assert lay.spare_clean()
    return e_out, e_u, e_S


@pytest.mark.parametrize("T, kind", [(2, "random"), (4, "random"), (5, "random"), (8, "random"), (8, "binary"),
                                     (6, "star"), (7, "chain")])
def test_verify_tree_small(T, kind):
    e = _tree_case(B=6, Hk=2, Hv=4, d=128, C=16, cap=16 + T - 1, T=T, in_dtype="bf16", seed=130 + T, kind=kind)
    say("verify_tree T=%d %s rel err out/u/state-after-commit: %.2e %.2e %.2e" % ((T, kind) + e))
    H.check(e, "bf16")


def test_verify_tree_fp32_d64_long_buffer_and_kv_only():
    """The vector-ALU kernel (fp32 inputs, d != 128), the 64-record window, and no state at all."""
    e = _tree_case(B=3, Hk=1, Hv=2, d=32, C=8, cap=12, T=4, in_dtype="f32", seed=141)
    H.check(e, "f32")
    e = _tree_case(B=3, Hk=2, Hv=2, d=64, C=8, cap=16, T=8, in_dtype="bf16", seed=142)
    H.check(e, "bf16")
    e = _tree_case(B=3, Hk=2, Hv=4, d=128, C=64, cap=72, T=8, in_dtype="bf16", seed=143)
    H.check(e, "bf16")
    e = _tree_case(B=4, Hk=2, Hv=4, d=128, C=16, cap=20, T=4, in_dtype="bf16", seed=144, kv_only=True)
    H.check(e, "bf16")


def test_verify_tree_chain_is_kvb_verify_bit_for_bit():
    """parent[i] = i - 1 must give exactly what kvb_verify gives (same kernel, same arithmetic)."""
    rng = np.random.default_rng(150)
    B, Hk, Hv, d, T, cap = 5, 2, 4, 128, 4, 20
    S0 = H.prefix_state(rng, B, Hk, Hv, d, d, "bf16", 8)
    fills = synth.buffer_fills(rng, B, 0, 15)
    wtok = synth.token_stream(rng, B, 15, Hk, Hv, d, d, "bf16")
    vtok = H.upload_tokens(synth.token_stream(rng, B, T, Hk, Hv, d, d, "bf16"), "bf16")
    outs = []
    for tree in (False, True):
        lay = H.Layer(B, Hk, Hv, d, d, cap=cap, in_dtype="bf16")
        lay.set_state(S0)
        ragged_warmup(lay, fills, wtok)
        out = torch.empty((B, T, Hv, d), dtype=torch.float32, device="cuda")
        if tree:
            lay.verify_tree(T, H.dev(synth.draft_trees(rng, B, T, "chain")), vtok, out)
        else:
            lay.verify(T, vtok, out)
        torch.cuda.synchronize()
        outs.append((out.cpu().numpy(), lay.ds.buf_u.cpu().numpy(), lay.ds.buf_G.cpu().numpy()))
    for x, y in zip(*outs):
        assert np.array_equal(x, y)


def test_bad_trees_and_paths_are_flagged_not_followed():
    rng = np.random.default_rng(151)
    B, Hk, Hv, d, T, cap = 3, 1, 2, 128, 4, 8
    lay = H.Layer(B, Hk, Hv, d, d, cap=cap, in_dtype="bf16")
    lay.set_state(np.zeros((B, Hv, d, d), np.float32))
    vtok = H.upload_tokens(synth.token_stream(rng, B, T, Hk, Hv, d, d, "bf16"), "bf16")
    parent = np.array([[-1, 0, 1, 2], [-1, 1, 0, 0], [-1, 0, 0, -7]], np.int32)   # rows 1, 2: not well formed
    out = torch.empty((B, T, Hv, d), dtype=torch.float32, device="cuda")
    lay.verify_tree(T, H.dev(parent), vtok, out)
    torch.cuda.synchronize()
    assert list(lay.status()) == [0, kvb.STATUS_BADPATH, kvb.STATUS_BADPATH]
    assert torch.isfinite(out).all()
    lay.ds.status.zero_()
    u_before = lay.ds.buf_u.clone()
    path = np.array([[0, 1, 3, 0], [2, 1, 0, 0], [0, 5, 0, 0]], np.int32)
    plen = np.array([3, 2, 2], np.int32)    # row 0 fine; row 1 decreasing; row 2 out of range
    lay.compact(T, H.dev(path), H.dev(plen))
    torch.cuda.synchronize()
    assert list(lay.status()) == [0, kvb.STATUS_BADPATH, kvb.STATUS_BADPATH]
    assert torch.equal(lay.ds.buf_u[1:], u_before[1:])
    assert torch.equal(lay.ds.buf_u[0, :, 2], u_before[0, :, 3])


@pytest.mark.parametrize("T", [1, 2, 3, 4, 5, 8])
def test_verify_small(T):
    e = _verify_case(B=6, Hk=2, Hv=4, d=128, C=16, cap=16 + T - 1, T=T, in_dtype="bf16", seed=30 + T)
    say("verify T=%d rel err out/u/state: %.2e %.2e %.2e" % ((T,) + e))
    H.check(e, "bf16")


def test_verify_tiny_fp32_and_d64():
    e = _verify_case(B=3, Hk=1, Hv=2, d=32, C=8, cap=12, T=4, in_dtype="f32", seed=41)
    say("verify fp32 d=32 rel err: %.2e %.2e %.2e" % e)
    H.check(e, "f32")
    e = _verify_case(B=3, Hk=2, Hv=2, d=64, C=8, cap=12, T=4, in_dtype="bf16", seed=42)
    H.check(e, "bf16")


def test_verify_long_buffer():
    e = _verify_case(B=4, Hk=1, Hv=2, d=128, C=64, cap=72, T=8, in_dtype="bf16", seed=43)
    say("verify C=64 T=8 rel err: %.2e %.2e %.2e" % e)
    H.check(e, "bf16")


def test_spec_verify_full():
    """Workload 3 at full size: B=128, fill ~U(0,15), 4 drafts, accepted ~U(0,4)."""
    w = synth.WORKLOADS["spec_verify"]
    e = _verify_case(w.B, w.Hk, w.Hv, w.dk, w.C, w.cap, w.T, w.in_dtype, w.seed)
    say("spec_verify rel err out/u/state: %.2e %.2e %.2e" % e)
    H.check(e, "bf16")


def test_spec_verify_tree_full():
    """Workload 3's size with tree-shaped drafts: B=128, fill ~U(0,15), a random 8-node tree per
    request, a random accepted root path; every draft checked along its own path."""
    w = synth.WORKLOADS["spec_verify"]
    e = _tree_case(w.B, w.Hk, w.Hv, w.dk, w.C, 24, 8, w.in_dtype, w.seed + 1)
    say("spec_verify (trees of 8) rel err out/u/state: %.2e %.2e %.2e" % e)
    H.check(e, "bf16")


# --------------------------------------------------------------------------- direct
def _direct_case(B, Hk, Hv, d, Lmax, cap, in_dtype, seed, lens=None, then_decode=True, block_size=None,
                 scatter=False, rec_dtype="f32", out_dtype="f32", poison=False):
    rng = np.random.default_rng(seed)
    if lens is None:
        lens = synth.context_lengths(rng, B, 1, Lmax)
    tok = synth.token_stream(rng, B, Lmax, Hk, Hv, d, d, in_dtype)
    if poison:   # whatever lies past a request's context must not reach its results
        for b in range(B):
            for x in tok.values():
                x[b, lens[b]:] = np.nan
    lay = H.Layer(B, Hk, Hv, d, d, cap=cap, in_dtype=in_dtype, with_state=False, block_size=block_size,
                  rec_dtype=rec_dtype, out_dtype=out_dtype, **(_scattered(B, seed) if scatter else {}))
    lay.ds.fill.fill_(3)          # stale fill must be discarded
    out = lay.new_out(B, Lmax, Hv, d, fill=float("nan"))
    lay.direct(H.dev(lens), Lmax, H.upload_tokens(tok, in_dtype), out)
    torch.cuda.synchronize()
    o_ref, u_ref, S_ref = oracle.kvb_direct_expected(tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"], lens)
    got = H.host(out)
    valid = ~np.isnan(o_ref)
    assert np.all(np.isnan(got[~valid])), "rows >= len were written"
    e_out = H.rel_err(got[valid], o_ref[valid], lay.out_unit)
    u_got = np.stack([lay.u_records(b, 0, Lmax) for b in range(B)]).transpose(0, 2, 1, 3)
    e_u = H.rel_err(u_got[valid], u_ref[valid])
    assert np.array_equal(lay.fill(), lens)
    e_dec = 0.0
    if then_decode:
        # one KV-only decode step for the requests that still have room, then fold into a zero state
        room = np.nonzero(lens < cap)[0]
        nt = synth.token_stream(rng, B, 1, Hk, Hv, d, d, in_dtype)
        ii = torch.from_numpy(room).cuda()
        dt = H.upload_tokens(nt, in_dtype)
        o1 = lay.new_out(len(room), Hv, d)
        lay.decode({n: x[ii, 0].contiguous() for n, x in dt.items()}, o1, slot=lay.slot[ii].contiguous(),
                   B=len(room), use_state=False)
        o1_ref, _, S_ref = oracle.gdn_sequence(S_ref, nt["q"], nt["k"], nt["v"], nt["g"], nt["beta"],
                                               lens=(lens < cap).astype(np.int32))[:3]
        e_dec = H.rel_err(H.host(o1), o1_ref[room, 0], lay.out_unit)
    lay.ds.state = torch.zeros((lay.n_slots, Hv, d, d), dtype=torch.float32, device="cuda")
    lay.flush(1)
    torch.cuda.synchronize()
    e_S = H.rel_err(lay.get_state(), S_ref)
    assert not lay.fill().any()
    assert lay.spare_clean()
    return e_out, e_u, e_dec, e_S


@pytest.mark.parametrize("d, in_dtype, Lmax", [(128, "bf16", 64), (128, "bf16", 7), (32, "f32", 16),
                                               (64, "bf16", 33), (128, "f32", 20), (128, "bf16", 128),
                                               (128, "bf16", 65), (128, "bf16", 100)])
def test_direct_small(d, in_dtype, Lmax):
    e = _direct_case(B=5, Hk=2, Hv=4, d=d, Lmax=Lmax, cap=max(Lmax, 8), in_dtype=in_dtype, seed=50 + Lmax)
    say("direct d=%d %s Lmax=%d rel err out/u/decode/state: %.2e %.2e %.2e %.2e" % ((d, in_dtype, Lmax) + e))
    H.check(e, in_dtype)


def test_direct_ignores_rows_beyond_the_context():
    """q, k, v, g, beta rows past len[b] hold NaN: outputs, records and the folded state of the valid
    rows are unaffected (every kernel of kvb_direct: 4 blocks, 8 blocks, the plain one)."""
    for d, in_dtype, Lmax in ((128, "bf16", 64), (128, "bf16", 128), (128, "f16", 40), (32, "f32", 16)):
        e = _direct_case(B=6, Hk=2, Hv=4, d=d, Lmax=Lmax, cap=Lmax, in_dtype=in_dtype, seed=70 + Lmax, poison=True,
                         then_decode=False)
        say("direct with NaN beyond the context, d=%d %s Lmax=%d: rel err out/u/decode/state %.2e %.2e %.2e %.2e"
            % ((d, in_dtype, Lmax) + e))
        H.check(e, in_dtype)


def test_direct_len_zero_and_one():
    e = _direct_case(B=4, Hk=1, Hv=2, d=128, Lmax=8, cap=8, in_dtype="bf16", seed=60,
                     lens=np.array([0, 1, 8, 2], np.int32))
    H.check(e, "bf16")


def test_short_direct_full():
    """Workload 4 at full size: B=256, context ~U(1,64), then one KV-only decode step."""
    w = synth.WORKLOADS["short_direct"]
    e = _direct_case(w.B, w.Hk, w.Hv, w.dk, w.Lmax, w.cap + 1, w.in_dtype, w.seed)
    say("short_direct rel err out/u/decode/state: %.2e %.2e %.2e %.2e" % e)
    H.check(e, "bf16")


# --------------------------------------------------------------------------- mixed batches
def test_mixed_fill_batch_reduced():
    """Workload 5 reduced (B=24, 2 layers, C=64): every request starts at its own fill, so a few
    requests flush at each step; the flush call runs every step with a device-side predicate."""
    B, Hk, Hv, d, C, steps, layers = 24, 2, 4, 128, 64, 80, 2
    rng = np.random.default_rng(5)
    for layer_i in range(layers):
        S0 = H.prefix_state(rng, B, Hk, Hv, d, d, "bf16", 8)
        fills = synth.buffer_fills(rng, B, 0, C - 1)
        wtok = synth.token_stream(rng, B, C - 1, Hk, Hv, d, d, "bf16")
        tok = synth.token_stream(rng, B, steps, Hk, Hv, d, d, "bf16")
        lay = H.Layer(B, Hk, Hv, d, d, cap=C, in_dtype="bf16")
        lay.set_state(S0)
        ragged_warmup(lay, fills, wtok)
        _, _, S_true, _ = oracle.gdn_sequence(S0, wtok["q"], wtok["k"], wtok["v"], wtok["g"], wtok["beta"],
                                              lens=fills)
        dt = H.upload_tokens(tok, "bf16")
        out = torch.empty((B, steps, Hv, d), dtype=torch.float32, device="cuda")
        for t in range(steps):
            o_t = torch.empty((B, Hv, d), dtype=torch.float32, device="cuda")
            if layer_i % 2:
                lay.decode_flush(H.step_view(dt, t), o_t, C)
            else:
                lay.decode(H.step_view(dt, t), o_t)
                lay.flush(C)
            out[:, t] = o_t
        torch.cuda.synchronize()
        assert np.array_equal(lay.fill(), (fills + steps) % C)
        lay.flush(1)
        o_ref, _, S_ref = oracle.kvb_decode_expected(S_true, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"])
        e = (H.rel_err(out.cpu().numpy(), o_ref), H.rel_err(lay.get_state(), S_ref))
        say("mixed layer %d rel err out/state: %.2e %.2e" % ((layer_i,) + e))
        H.check(e, "bf16")
        assert not lay.status().any()


# --------------------------------------------------------------------------- edge cases
def _small_layer(in_dtype="bf16", B=3, Hk=1, Hv=2, d=128, cap=4, **kw):
    return H.Layer(B, Hk, Hv, d, d, cap=cap, in_dtype=in_dtype, **kw)


def test_decode_and_verify_never_write_state_and_overflow_is_flagged():
    rng = np.random.default_rng(70)
    lay = _small_layer()
    S0 = synth.random_state(rng, 3, 2, 128, 128)
    lay.set_state(S0)
    tok = H.upload_tokens(synth.token_stream(rng, 3, 6, 1, 2, 128, 128, "bf16"), "bf16")
    before = lay.ds.state.clone()
    out = torch.full((3, 2, 128), 7.0, dtype=torch.float32, device="cuda")
    for t in range(4):
        lay.decode(H.step_view(tok, t), out)
    torch.cuda.synchronize()
    assert torch.equal(lay.ds.state, before)
    assert np.array_equal(lay.fill(), [4, 4, 4]) and not lay.status().any()
    # buffer full: the 5th token is refused, nothing is written
    u_before, out[:] = lay.ds.buf_u.clone(), 7.0
    lay.decode(H.step_view(tok, 4), out)
    vout = torch.full((3, 2, 2, 128), 7.0, dtype=torch.float32, device="cuda")
    lay.verify(2, {n: x[:, :2].contiguous() for n, x in tok.items()}, vout)
    torch.cuda.synchronize()
    assert np.array_equal(lay.fill(), [4, 4, 4])
    assert np.array_equal(lay.status(), [kvb.STATUS_OVERFLOW] * 3)
    assert torch.equal(lay.ds.buf_u, u_before) and torch.all(out == 7.0) and torch.all(vout == 7.0)
    assert torch.equal(lay.ds.state, before)


def test_slot_indirection_leaves_other_slots_alone():
    """Requests live in scattered slots of a larger store; unused slots hold poison that must
    survive; a slot index outside the store is skipped."""
    rng = np.random.default_rng(71)
    B, n_slots = 3, 7
    slots = np.array([5, 0, 3], np.int32)
    lay = H.Layer(B, 1, 2, 128, 128, cap=4, in_dtype="bf16", n_slots=n_slots, slots=slots)
    lay.ds.state.fill_(123.0)
    lay.ds.buf_u.fill_(-55.0)
    lay.ds.fill.fill_(2)
    lay.ds.fill[lay.slot.long()] = 0
    S0 = synth.random_state(rng, B, 2, 128, 128)
    tok = synth.token_stream(rng, B, 6, 1, 2, 128, 128, "bf16")
    o, u, S, _ = H.run_decode(lay, S0, tok, 4)
    o_ref, u_ref, S_ref = oracle.kvb_decode_expected(S0, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"])
    H.check((H.rel_err(o, o_ref), H.rel_err(S, S_ref)), "bf16")
    others = torch.tensor([1, 2, 4, 6], device="cuda")
    assert torch.all(lay.ds.state[others] == 123.0) and torch.all(lay.ds.buf_u[others] == -55.0)
    assert torch.all(lay.ds.fill[others] == 2)
    # out-of-range slots: the call succeeds and touches nothing
    bad = H.dev(np.array([7, -1, 100], np.int32))
    snap = (lay.ds.state.clone(), lay.ds.buf_u.clone(), lay.ds.fill.clone())
    out = torch.full((B, 2, 128), 9.0, dtype=torch.float32, device="cuda")
    lay.decode(H.step_view(H.upload_tokens(tok, "bf16"), 0), out, slot=bad)
    lay.flush(1, slot=bad)
    torch.cuda.synchronize()
    assert torch.equal(lay.ds.state, snap[0]) and torch.equal(lay.ds.buf_u, snap[1])
    assert torch.equal(lay.ds.fill, snap[2]) and torch.all(out == 9.0)


def test_closed_forms_on_the_gpu():
    """beta = 0: outputs are prod(alpha) q S0 and flushing scales the state by prod(alpha);
    beta = 0 and g = 0: flushing leaves the state bit-identical."""
    rng = np.random.default_rng(72)
    B, Hv, d = 2, 2, 128
    S0 = synth.random_state(rng, B, Hv, d, d)
    tok = synth.token_stream(rng, B, 4, 1, Hv, d, d, "bf16")
    tok["beta"][:] = 0
    lay = _small_layer(B=B)
    o, u, S, _ = H.run_decode(lay, S0, tok, 4, flush_every_step=False)
    gam = np.exp(np.cumsum(tok["g"].astype(np.float64), axis=1))
    want = gam[..., None] * np.einsum("bti,bhij->bthj", tok["q"][:, :, 0].astype(np.float64), S0.astype(np.float64))
    assert H.rel_err(o, want) < 1e-5 and not u.any()
    assert H.rel_err(S, gam[:, -1, :, None, None] * S0) < 1e-6
    tok["g"][:] = 0
    lay = _small_layer(B=B)
    o, u, S, _ = H.run_decode(lay, S0, tok, 4, flush_every_step=False)
    assert np.array_equal(S, S0)


@pytest.mark.parametrize("B, Hk, Hv, C", [(2, 1, 2, 16), (3, 2, 4, 32), (40, 16, 32, 16), (2, 1, 2, 64)])
def test_decode_ignores_whatever_lies_beyond_the_fill(B, Hk, Hv, C):
    """The record buffers start out full of NaN: a record past the fill may be read (a small launch
    requests the whole window before it knows the fill) but must never reach a result.  Small and
    large launches (the latter wait for the fill), windows of 16, 32 and 64 records."""
    rng = np.random.default_rng(74 + C)
    d = 128
    S0 = H.prefix_state(rng, B, Hk, Hv, d, d, "bf16", 4)
    tok = synth.token_stream(rng, B, C + 5, Hk, Hv, d, d, "bf16")
    for fused in (True, False):
        lay = H.Layer(B, Hk, Hv, d, d, cap=C, in_dtype="bf16")
        lay.ds.buf_u.fill_(float("nan"))
        lay.ds.buf_k.fill_(float("nan"))
        lay.ds.buf_G.fill_(float("nan"))
        o, u, S, _ = H.run_decode(lay, S0, tok, C, fused=fused)
        o_ref, u_ref, S_ref = oracle.kvb_decode_expected(S0, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"])
        assert np.isfinite(o).all() and np.isfinite(S).all()
        H.check((H.rel_err(o, o_ref), H.rel_err(u, u_ref), H.rel_err(S, S_ref)), "bf16")


def test_strong_decay_neither_overflows_nor_underflows_to_nan():
    """g = -20 per token over a 64-record chunk: gamma ratios are never formed."""
    rng = np.random.default_rng(73)
    B, Hk, Hv, d, C = 2, 1, 2, 128, 64
    S0 = synth.random_state(rng, B, Hv, d, d)
    tok = synth.token_stream(rng, B, C + 3, Hk, Hv, d, d, "bf16")
    tok["g"][:] = -20.0
    lay = H.Layer(B, Hk, Hv, d, d, cap=C, in_dtype="bf16")
    o, u, S, _ = H.run_decode(lay, S0, tok, C)
    o_ref, u_ref, S_ref = oracle.kvb_decode_expected(S0, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"])
    assert np.isfinite(o).all() and np.isfinite(S).all()
    H.check((H.rel_err(o, o_ref), H.rel_err(S, S_ref)), "bf16")


@pytest.mark.parametrize("cap", [16, 64])
def test_flush_products_keep_fp32_accuracy_over_a_wide_range(cap):
    """kvb_flush (bf16, d = 128) multiplies bf16 keys with a three-way bf16 split of the fp32
    factor; the split has to be exact whatever the magnitude.  One record per request on a zero
    state, v scaled by 1e-30 .. 1e30: every element of S = k^T u must match the oracle to fp32
    rounding of u and of the product (a dropped third piece would show as 1.5e-5)."""
    rng = np.random.default_rng(171)
    scales = np.array([1e-30, 1e-15, 1.0, 1e15, 1e30])
    B, Hk, Hv, d = len(scales), 1, 2, 128
    tok = synth.token_stream(rng, B, 1, Hk, Hv, d, d, "bf16")
    tok["v"] = synth.round_to_bf16((tok["v"] * scales[:, None, None, None]).astype(np.float32))
    tok["g"][:] = -0.125
    S0 = np.zeros((B, Hv, d, d), np.float32)
    lay = H.Layer(B, Hk, Hv, d, d, cap=cap, in_dtype="bf16")
    _, _, S, _ = H.run_decode(lay, S0, tok, cap, final_flush=True)
    _, _, S_ref = oracle.kvb_decode_expected(S0, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"])
    assert np.isfinite(S).all()
    nz = np.abs(S_ref) > 0
    rel = np.abs(S - S_ref)[nz] / np.abs(S_ref)[nz]
    say("flush, one record, scales 1e-30..1e30: max elementwise rel err %.2e" % rel.max())
    assert rel.max() < 4e-7
    # several records of mixed magnitude per request: the usual bound, per request
    tok = synth.token_stream(rng, B, cap, Hk, Hv, d, d, "bf16")
    mags = 10.0 ** rng.uniform(-3, 3, size=(B, cap))
    tok["v"] = synth.round_to_bf16((tok["v"] * mags[:, :, None, None]).astype(np.float32))
    lay = H.Layer(B, Hk, Hv, d, d, cap=cap, in_dtype="bf16")
    _, _, S, _ = H.run_decode(lay, S0, tok, cap, final_flush=True)
    _, _, S_ref = oracle.kvb_decode_expected(S0, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"])
    e = max(H.rel_err(S[b], S_ref[b]) for b in range(B))
    say("flush, %d records of mixed magnitude: rel err %.2e" % (cap, e))
    H.check(e, "bf16")


def test_accepting_nothing_appends_nothing():
    rng = np.random.default_rng(74)
    lay = _small_layer(cap=8)
    S0 = synth.random_state(rng, 3, 2, 128, 128)
    lay.set_state(S0)
    vt = H.upload_tokens(synth.token_stream(rng, 3, 4, 1, 2, 128, 128, "bf16"), "bf16")
    out = torch.empty((3, 4, 2, 128), dtype=torch.float32, device="cuda")
    lay.verify(4, vt, out)
    lay.flush(1, accepted=H.dev(np.zeros(3, np.int32)))
    torch.cuda.synchronize()
    assert not lay.fill().any()
    assert np.array_equal(lay.get_state(), S0)


def test_snapshot_restore_mid_chunk():
    """State, buffer and fill are plain caller-owned arrays: copying them is a checkpoint."""
    rng = np.random.default_rng(75)
    B, Hk, Hv, d, C = 2, 1, 2, 128, 8
    S0 = synth.random_state(rng, B, Hv, d, d)
    tok = synth.token_stream(rng, B, 12, Hk, Hv, d, d, "bf16")
    dt = H.upload_tokens(tok, "bf16")
    lay = H.Layer(B, Hk, Hv, d, d, cap=C, in_dtype="bf16")
    lay.set_state(S0)
    out = torch.empty((B, 12, Hv, d), dtype=torch.float32, device="cuda")

    def steps(lo, hi, dst):
        for t in range(lo, hi):
            o_t = torch.empty((B, Hv, d), dtype=torch.float32, device="cuda")
            lay.decode(H.step_view(dt, t), o_t)
            lay.flush(C)
            dst[:, t] = o_t

    steps(0, 5, out)
    snap = [x.clone() for x in (lay.ds.state, lay.ds.buf_k, lay.ds.buf_u, lay.ds.buf_G, lay.ds.fill)]
    steps(5, 12, out)
    for dst, src in zip((lay.ds.state, lay.ds.buf_k, lay.ds.buf_u, lay.ds.buf_G, lay.ds.fill), snap):
        dst.copy_(src)
    out2 = out.clone()
    steps(5, 12, out2)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


def test_hip_graph_replays_match_eager():
    """The decode + flush loop captured in a HIP graph: every replay, with eager work and
    synchronisation in between, gives the eager loop's outputs and state bit for bit."""
    rng = np.random.default_rng(76)
    B, Hk, Hv, d, C, n = 4, 2, 4, 128, 4, 10
    S0 = synth.random_state(rng, B, Hv, d, d)
    dt = H.upload_tokens(synth.token_stream(rng, B, n, Hk, Hv, d, d, "bf16"), "bf16")
    toks = [H.step_view(dt, t) for t in range(n)]
    lay = H.Layer(B, Hk, Hv, d, d, cap=C, in_dtype="bf16")
    outs = torch.zeros((n, B, Hv, d), dtype=torch.float32, device="cuda")
    bufs = (lay.ds.state, lay.ds.buf_k, lay.ds.buf_u, lay.ds.buf_G, lay.ds.fill)

    def loop():
        for t in range(n):
            lay.decode(toks[t], outs[t])
            lay.flush(C)

    def reset():
        lay.ds.buf_k.zero_(); lay.ds.buf_u.zero_(); lay.ds.buf_G.zero_(); lay.ds.fill.zero_()
        lay.set_state(S0)
        outs.zero_()

    reset()
    loop()
    torch.cuda.synchronize()
    want = [x.clone() for x in bufs + (outs,)]
    reset()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        loop()
    for rep in range(4):
        reset()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, ref in zip(bufs + (outs,), want):
            assert torch.equal(got, ref), "replay %d differs from eager" % rep
        loop()                       # eager work between replays
        torch.cuda.synchronize()


def test_kernel_timer_reports_the_armed_launch():
    rng = np.random.default_rng(77)
    lay = _small_layer(cap=4)
    lay.set_state(synth.random_state(rng, 3, 2, 128, 128))
    tok = H.upload_tokens(synth.token_stream(rng, 3, 2, 1, 2, 128, 128, "bf16"), "bf16")
    out = torch.empty((3, 2, 128), dtype=torch.float32, device="cuda")
    t = kvb.Timer()
    t.arm()
    lay.decode(H.step_view(tok, 0), out)
    lay.decode(H.step_view(tok, 1), out)      # not timed: the arm covers one launch
    us = t.us()
    t.close()
    torch.cuda.synchronize()
    assert 0.5 < us < 5000.0
    assert np.array_equal(lay.fill(), [2, 2, 2])


def test_long_mixed_full_size_sampled():
    """Workload 5 at full size: B=512, 36 stacked layers of the Qwen3-Next shape (36 GiB of fp32
    state), C=64, every (layer, request) starting at its own fill ~U(0,63), 128 decode steps per
    layer with the state update folded in when a buffer fills.  The fp64 oracle for all 589 824
    (request, layer, head) units would take hours, so outputs (all 128 steps) and final states are
    compared on a stated sample: the first 4 requests of layers 0 and 35 plus 24 (layer, request)
    pairs drawn from the workload's generator; every other unit is checked for finiteness."""
    w = synth.WORKLOADS["long_mixed"]
    B, Lyr, Hk, Hv, d, C, steps = w.B, w.layers, w.Hk, w.Hv, w.dk, w.C, w.steps
    free, _ = torch.cuda.mem_get_info()
    if free < 80 * 2 ** 30:
        pytest.skip("needs 80 GiB of free device memory")
    rng = np.random.default_rng(w.seed)
    n_slots = Lyr * B
    ds = kvb.DeviceStore(n_slots, Hk, Hv, d, d, w.cap, kvb.BF16)
    gen = torch.Generator(device="cuda").manual_seed(w.seed)
    for l in range(Lyr):                       # synthetic committed states, seeded, layer by layer
        ds.state[l * B:(l + 1) * B].normal_(0.0, 0.5, generator=gen)
    fills = np.stack([synth.buffer_fills(rng, B, 0, C - 1) for _ in range(Lyr)])        # [Lyr, B]
    wtok = synth.token_stream(rng, B, C - 1, Hk, Hv, d, d, "bf16")     # warm-up tokens (shared by layers)
    tok = synth.token_stream(rng, B, steps, Hk, Hv, d, d, "bf16")      # decode tokens (shared by layers)
    pairs = [(l, b) for l in (0, Lyr - 1) for b in range(4)]
    pairs += [(int(rng.integers(Lyr)), int(rng.integers(B))) for _ in range(24)]
    pairs = sorted(set(pairs))
    say("long_mixed: %d sampled (layer, request) pairs of %d" % (len(pairs), Lyr * B))
    S0 = {p: ds.state[p[0] * B + p[1]].cpu().numpy() for p in pairs}

    sh = lambda n: kvb.shape(n, Hk, Hv, d, d, w.cap, kvb.BF16)
    st = ds.c(flags=kvb.STORE_STREAM)
    dw = H.upload_tokens(wtok, "bf16")
    # ragged warm-up: step j of layer l carries the requests with fills[l, b] > j
    for l in range(Lyr):
        for j in range(int(fills[l].max())):
            idx = np.nonzero(fills[l] > j)[0]
            ii = torch.from_numpy(idx).cuda()
            t_ = {n: x[ii, j].contiguous() for n, x in dw.items()}
            out = torch.empty((len(idx), Hv, d), dtype=torch.float32, device="cuda")
            slot = (ii + l * B).to(torch.int32).contiguous()
            kvb.kvb_decode(sh(len(idx)), st, slot, t_["q"], t_["k"], t_["v"], t_["g"], t_["beta"], out)
    torch.cuda.synchronize()
    assert np.array_equal(ds.fill.cpu().numpy().reshape(Lyr, B), fills)
    say("long_mixed: warm-up done")

    dt = H.upload_tokens(tok, "bf16")
    slots = [torch.arange(l * B, (l + 1) * B, dtype=torch.int32, device="cuda") for l in range(Lyr)]
    samp_rows = {l: torch.tensor([b for (ll, b) in pairs if ll == l], device="cuda") for l in {p[0] for p in pairs}}
    got = {p: np.empty((steps, Hv, d), np.float32) for p in pairs}
    out = torch.empty((B, Hv, d), dtype=torch.float32, device="cuda")
    finite = torch.ones((), dtype=torch.bool, device="cuda")
    for t in range(steps):
        tk = H.step_view(dt, t)
        for l in range(Lyr):
            kvb.kvb_decode_flush(sh(B), st, slots[l], tk["q"], tk["k"], tk["v"], tk["g"], tk["beta"], out, C)
            finite &= torch.isfinite(out).all()
            if l in samp_rows:
                rows = out[samp_rows[l]].cpu().numpy()
                for r_, b in zip(rows, samp_rows[l].tolist()):
                    got[(l, b)][t] = r_
        if t % 32 == 31:
            say("long_mixed: step %d" % (t + 1))
    torch.cuda.synchronize()
    assert bool(finite), "a non-finite output somewhere in the batch"
    assert np.array_equal(ds.fill.cpu().numpy().reshape(Lyr, B), (fills + steps) % C)
    assert int(ds.status.sum().item()) == 0
    for l in range(Lyr):
        kvb.kvb_flush(sh(B), st, slots[l], None, 1)
    torch.cuda.synchronize()

    # oracle on the sample: one "request" per pair
    P = len(pairs)
    fl = np.array([fills[l, b] for l, b in pairs], np.int32)
    bi = np.array([b for _, b in pairs])
    S = np.stack([S0[p] for p in pairs])
    _, _, S_true, _ = oracle.gdn_sequence(S, wtok["q"][bi], wtok["k"][bi], wtok["v"][bi], wtok["g"][bi],
                                          wtok["beta"][bi], lens=fl)
    o_ref, _, S_ref = oracle.kvb_decode_expected(S_true, tok["q"][bi], tok["k"][bi], tok["v"][bi], tok["g"][bi],
                                                 tok["beta"][bi])
    o_got = np.stack([got[p] for p in pairs])                       # [P, steps, Hv, d]
    S_got = np.stack([ds.state[l * B + b].cpu().numpy() for l, b in pairs])
    e = (H.rel_err(o_got, o_ref), H.rel_err(S_got, S_ref))
    say("long_mixed full size: rel err out/state on %d sampled pairs: %.2e %.2e" % (P, e[0], e[1]))
    H.check(e, "bf16")
    assert bool(torch.isfinite(ds.state).all())


@pytest.mark.parametrize("Hk, Hv", [(3, 3), (1, 4), (2, 8)])
def test_head_grouping_ratios(Hk, Hv):
    """One, four and (again) four v-heads per qk-head, through decode, flush, verify and direct."""
    d, C, B = 128, 8, 3
    rng = np.random.default_rng(80 + Hv)
    S0 = H.prefix_state(rng, B, Hk, Hv, d, d, "bf16", 8)
    tok = synth.token_stream(rng, B, 19, Hk, Hv, d, d, "bf16")
    lay = H.Layer(B, Hk, Hv, d, d, cap=C, in_dtype="bf16")
    o, u, S, _ = H.run_decode(lay, S0, tok, C, fused=True)
    o_ref, u_ref, S_ref = oracle.kvb_decode_expected(S0, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"])
    H.check((H.rel_err(o, o_ref), H.rel_err(u, u_ref), H.rel_err(S, S_ref)), "bf16")
    e = _verify_case(B=B, Hk=Hk, Hv=Hv, d=d, C=C, cap=C + 3, T=4, in_dtype="bf16", seed=90 + Hv)
    H.check(e, "bf16")
    e = _direct_case(B=B, Hk=Hk, Hv=Hv, d=d, Lmax=40, cap=48, in_dtype="bf16", seed=95 + Hv)
    H.check(e, "bf16")


def test_largest_buffer_and_most_drafts():
    """cap = 128 (the paper's upper end, d records) with 8 drafts on nearly full buffers: the
    record windows' tail paths of both the decode and the verify kernel."""
    e = _verify_case(B=5, Hk=1, Hv=2, d=128, C=120, cap=128, T=8, in_dtype="bf16", seed=97, fill_hi=119)
    say("cap=128 T=8 rel err out/u/state: %.2e %.2e %.2e" % e)
    H.check(e, "bf16")
    e = _verify_case(B=3, Hk=1, Hv=2, d=128, C=40, cap=48, T=8, in_dtype="f32", seed=98, fill_hi=39)
    say("cap=48 T=8 fp32 rel err out/u/state: %.2e %.2e %.2e" % e)
    H.check(e, "f32")
    # the vector-ALU verify path (head size 64) with more than 64 buffered records
    e = _verify_case(B=3, Hk=1, Hv=2, d=64, C=96, cap=100, T=4, in_dtype="bf16", seed=100, fill_hi=95)   # fills 95, 88, 55
    say("cap=100 T=4 d=64 rel err out/u/state: %.2e %.2e %.2e" % e)
    H.check(e, "bf16")
    e = _verify_case(B=2, Hk=1, Hv=1, d=128, C=100, cap=104, T=4, in_dtype="f32", seed=108, fill_hi=99)    # fills 99, 61
    say("cap=104 T=4 d=128 fp32 rel err out/u/state: %.2e %.2e %.2e" % e)
    H.check(e, "f32")


def test_kv_only_verify_and_stream_hint_do_not_change_results():
    """kvb_verify with no state (KV-only contexts, Sec. 3.4) and the non-temporal state loads
    (a cache hint) against the same oracle / against the default path bit for bit."""
    e = _verify_case(B=4, Hk=2, Hv=4, d=128, C=16, cap=20, T=4, in_dtype="bf16", seed=99, kv_only=True)
    H.check(e, "bf16")
    rng = np.random.default_rng(101)
    B, Hk, Hv, d, C = 3, 2, 4, 128, 8
    S0 = synth.random_state(rng, B, Hv, d, d)
    tok = H.upload_tokens(synth.token_stream(rng, B, 11, Hk, Hv, d, d, "bf16"), "bf16")
    res = []
    for flags in (kvb.STORE_RESIDENT, kvb.STORE_STREAM):
        lay = H.Layer(B, Hk, Hv, d, d, cap=C, in_dtype="bf16")
        lay.set_state(S0)
        outs = torch.empty((11, B, Hv, d), dtype=torch.float32, device="cuda")
        for t in range(11):
            kvb.kvb_decode_flush(lay.shape(), lay.ds.c(flags=flags), lay.slot, *[H.step_view(tok, t)[n] for n in
                                 ("q", "k", "v", "g", "beta")], outs[t], C)
        vout = torch.empty((B, 3, Hv, d), dtype=torch.float32, device="cuda")
        vt = {n: x[:, :3].contiguous() for n, x in tok.items()}
        kvb.kvb_verify(lay.shape(), lay.ds.c(flags=flags), lay.slot, 3, vt["q"], vt["k"], vt["v"], vt["g"],
                       vt["beta"], vout)
        torch.cuda.synchronize()
        res.append((outs.clone(), vout.clone(), lay.ds.state.clone(), lay.ds.buf_u.clone()))
    for x, y in zip(*res):
        assert torch.equal(x, y)


@pytest.mark.parametrize("in_dtype, rec_dtype, cap, block_size", [
    ("bf16", "f32", 8, None), ("bf16", "f32", 40, None), ("f16", "f16", 40, None), ("bf16", "bf16", 16, None),
    ("f32", "f32", 12, None), ("bf16", "f32", 16, 8), ("f16", "f32", 48, 16)])
def test_stream_hint_does_not_change_kvb_flush(in_dtype, rec_dtype, cap, block_size):
    """kvb_flush with the state streamed past the caches (non-temporal loads and stores, what the
    library chooses by itself for large batches) against the default path, bit for bit."""
    rng = np.random.default_rng(1200 + cap)
    B, Hk, Hv, d = 3, 2, 4, 128
    S0 = synth.random_state(rng, B, Hv, d, d)
    tok = H.upload_tokens(synth.token_stream(rng, B, cap, Hk, Hv, d, d, in_dtype), in_dtype)
    res = []
    for flags in (kvb.STORE_RESIDENT, kvb.STORE_STREAM):
        lay = H.Layer(B, Hk, Hv, d, d, cap=cap, in_dtype=in_dtype, rec_dtype=rec_dtype, block_size=block_size)
        lay.set_state(S0)
        out = lay.new_out(B, Hv, d)
        for t in range(cap - 1):
            kvb.kvb_decode(lay.shape(), lay.ds.c(flags=flags), lay.slot, *[H.step_view(tok, t)[n] for n in
                           ("q", "k", "v", "g", "beta")], out)
        kvb.kvb_flush(lay.shape(), lay.ds.c(flags=flags), lay.slot, None, 1)
        torch.cuda.synchronize()
        assert not lay.ds.fill[lay.slot.long()].any()
        res.append(lay.get_state())
    assert np.array_equal(res[0], res[1])
    assert np.isfinite(res[0]).all() and not np.array_equal(res[0], np.asarray(S0, dtype=np.float32))


# --------------------------------------------------------------------------- paged record buffers
@pytest.mark.parametrize("d, in_dtype, C, block_size, fused", [
    (128, "bf16", 16, 16, True), (128, "bf16", 16, 8, True), (128, "bf16", 16, 8, False),
    (128, "bf16", 64, 16, True), (128, "bf16", 40, 8, False), (64, "bf16", 24, 8, True),
    (32, "f32", 16, 8, True), (128, "f32", 12, 16, False),
])
def test_paged_decode_flush(d, in_dtype, C, block_size, fused):
    """Blocks of 8 or 16 records dealt at random from a shared pool (Sec. 3.1): same results as the
    contiguous layout, nothing written outside the request's own blocks."""
    rng = np.random.default_rng(700 + d + C + block_size)
    B, Hk, Hv, steps = 3, 1, 2, 2 * C + 3
    S0 = H.prefix_state(rng, B, Hk, Hv, d, d, in_dtype, 8)
    tok = synth.token_stream(rng, B, steps, Hk, Hv, d, d, in_dtype)
    lay = H.Layer(B, Hk, Hv, d, d, cap=C, in_dtype=in_dtype, block_size=block_size)
    o, u, S, _ = H.run_decode(lay, S0, tok, C, fused=fused)
    o_ref, u_ref, S_ref = oracle.kvb_decode_expected(S0, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"])
    e = (H.rel_err(o, o_ref), H.rel_err(u, u_ref), H.rel_err(S, S_ref))
    say("paged d=%d %s C=%d block=%d fused=%s rel err out/u/state: %.2e %.2e %.2e" % ((d, in_dtype, C, block_size, fused) + e))
    H.check(e, in_dtype)
    assert lay.spare_clean() and not lay.status().any()


def test_paged_verify_tree_and_direct():
    e = _verify_case(B=6, Hk=2, Hv=4, d=128, C=16, cap=19, T=4, in_dtype="bf16", seed=710, block_size=8)
    H.check(e, "bf16")
    e = _verify_case(B=3, Hk=2, Hv=4, d=128, C=64, cap=71, T=8, in_dtype="bf16", seed=711, fill_hi=63, block_size=16)
    H.check(e, "bf16")
    e = _verify_case(B=2, Hk=1, Hv=2, d=32, C=8, cap=11, T=4, in_dtype="f32", seed=712, block_size=8)
    H.check(e, "f32")
    e = _tree_case(B=5, Hk=2, Hv=4, d=128, C=16, cap=23, T=8, in_dtype="bf16", seed=713, block_size=8)
    H.check(e, "bf16")
    e = _tree_case(B=3, Hk=2, Hv=2, d=64, C=8, cap=16, T=8, in_dtype="bf16", seed=714, block_size=16)
    H.check(e, "bf16")
    e = _direct_case(B=5, Hk=2, Hv=4, d=128, Lmax=64, cap=80, in_dtype="bf16", seed=715, block_size=16)
    H.check(e, "bf16")
    e = _direct_case(B=4, Hk=1, Hv=2, d=128, Lmax=37, cap=40, in_dtype="bf16", seed=716, block_size=8)
    H.check(e, "bf16")
    e = _direct_case(B=3, Hk=1, Hv=2, d=32, Lmax=16, cap=24, in_dtype="f32", seed=717, block_size=8)
    H.check(e, "f32")


def test_paged_qwen3next_decode_full():
    """Workload 2 at full size with 16-record blocks from a shuffled pool, fused step."""
    w = synth.WORKLOADS["qwen3next_decode"]
    rng = np.random.default_rng(w.seed)
    S0 = H.prefix_state(rng, w.B, w.Hk, w.Hv, w.dk, w.dv, w.in_dtype, w.prefix)
    tok = synth.token_stream(rng, w.B, 64, w.Hk, w.Hv, w.dk, w.dv, w.in_dtype)
    lay = H.Layer(w.B, w.Hk, w.Hv, w.dk, w.dv, cap=w.cap, in_dtype=w.in_dtype, block_size=16)
    o, u, S, _ = H.run_decode(lay, S0, tok, w.C, fused=True)
    o_ref, u_ref, S_ref = oracle.kvb_decode_expected(S0, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"])
    e = (H.rel_err(o, o_ref), H.rel_err(u, u_ref), H.rel_err(S, S_ref))
    say("paged qwen3next_decode rel err out/u/state: %.2e %.2e %.2e" % e)
    H.check(e, "bf16")
    assert lay.spare_clean()


def test_kv_only_speculative_decoding_commits_without_a_state():
    """A KV-only context (no state at all) verified in chunks of drafts: kvb_verify with a NULL
    state, then kvb_flush with a NULL state, which only commits the accepted prefix (Sec. 3.3 on
    top of Sec. 3.4).  Outputs against the recurrence from a zero state."""
    rng = np.random.default_rng(160)
    B, Hk, Hv, d, T, rounds, cap = 4, 2, 4, 128, 4, 5, 32
    tok = synth.token_stream(rng, B, T * rounds, Hk, Hv, d, d, "bf16")
    lay = H.Layer(B, Hk, Hv, d, d, cap=cap, in_dtype="bf16", with_state=False)
    S = np.zeros((B, Hv, d, d))
    pos = np.zeros(B, np.int64)          # tokens committed so far per request
    worst = 0.0
    for r_ in range(rounds):
        idx = pos[:, None] + np.arange(T)[None, :]
        chunk = {n: np.take_along_axis(x, idx.reshape((B, T) + (1,) * (x.ndim - 2)), axis=1) for n, x in tok.items()}
        acc = synth.accepted_lengths(rng, B, T)
        o_ref, _, S = oracle.kvb_verify_expected(S, chunk["q"], chunk["k"], chunk["v"], chunk["g"], chunk["beta"], acc)
        out = torch.empty((B, T, Hv, d), dtype=torch.float32, device="cuda")
        lay.verify(T, H.upload_tokens(chunk, "bf16"), out, use_state=False)
        kvb.kvb_flush(lay.shape(), lay.ds.c(False), lay.slot, H.dev(acc), 1)
        torch.cuda.synchronize()
        worst = max(worst, H.rel_err(out.cpu().numpy(), o_ref))
        pos += acc
        assert np.array_equal(lay.fill(), pos)
    H.check(worst, "bf16")
    assert not lay.status().any()


def test_direct_long_contexts_full_heads_and_paged():
    """Contexts up to d = 128 tokens (Sec. 3.4) at the model's head counts, ragged lengths that
    cover every block count, then paged records; each followed by the fold into a zero state."""
    lens = np.array([128, 127, 113, 112, 97, 96, 81, 80, 65, 64, 33, 1], np.int32)
    e = _direct_case(B=len(lens), Hk=16, Hv=32, d=128, Lmax=128, cap=128, in_dtype="bf16", seed=720, lens=lens,
                     then_decode=False)
    say("direct L<=128 rel err out/u/decode/state: %.2e %.2e %.2e %.2e" % e)
    H.check(e, "bf16")
    e = _direct_case(B=4, Hk=1, Hv=2, d=128, Lmax=120, cap=128, in_dtype="bf16", seed=721, block_size=16)
    H.check(e, "bf16")


def test_direct_beyond_64_needs_bf16_d128():
    lay = H.Layer(2, 1, 2, 32, 32, cap=128, in_dtype="f32", with_state=False)
    z = torch.zeros(1, device="cuda")
    rc = kvb.kvb_direct(lay.shape(), lay.ds.c(False), lay.slot, lay.slot, 100, z, z, z, z, z, z, check=False)
    assert rc == kvb.EUNSUPPORTED


# --------------------------------------------------------------------------- seeded random configurations
@pytest.mark.parametrize("seed", range(16))
def test_random_configurations(seed):
    """Every call at a seeded random shape: head counts and grouping, head size, input type, chunk
    and capacity (not multiples of anything), drafts, tree shape, contiguous or paged records."""
    rng = np.random.default_rng(9000 + seed)
    d = int(rng.choice([32, 64, 128, 128]))
    in_dtype = str(rng.choice(["bf16", "bf16", "f32"]))
    Hk = int(rng.integers(1, 4))
    Hv = Hk * int(rng.integers(1, 4))
    B = int(rng.integers(1, 6))
    T = int(rng.integers(1, 9))
    C = int(rng.integers(1, 41))
    block = [None, 8, 16, 32][int(rng.integers(0, 4))]
    scatter = bool(rng.integers(0, 2))
    # the storage regime, from a generator of its own (the shapes above stay as they were): half of the
    # 16-bit cases take fp16, a third of them 16-bit records, half of them 16-bit outputs
    rng2 = np.random.default_rng(9500 + seed)
    rec_dtype = out_dtype = "f32"
    if in_dtype == "bf16":
        in_dtype = str(rng2.choice(["bf16", "f16"]))
        rec_dtype = str(rng2.choice(["f32", "f32", in_dtype]))
        out_dtype = str(rng2.choice(["f32", in_dtype]))
    types = dict(rec_dtype=rec_dtype, out_dtype=out_dtype)
    tag = "seed %d: d=%d %s rec=%s out=%s Hk=%d Hv=%d B=%d T=%d C=%d block=%s" % (
        seed, d, in_dtype, rec_dtype, out_dtype, Hk, Hv, B, T, C, block)
    say(tag)
    # decode + flush over two and a half chunks
    steps = 2 * C + C // 2 + 1
    S0 = H.prefix_state(rng, B, Hk, Hv, d, d, in_dtype, 6)
    tok = synth.token_stream(rng, B, steps, Hk, Hv, d, d, in_dtype)
    lay = H.Layer(B, Hk, Hv, d, d, cap=C, in_dtype=in_dtype, block_size=block, **types,
                  **(_scattered(B, seed) if scatter else {}))
    o, u, S, _ = H.run_decode(lay, S0, tok, C, fused=bool(rng.integers(0, 2)))
    o_ref, u_ref, S_ref = oracle.kvb_decode_expected(S0, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"])
    e = (H.rel_err(o, o_ref, lay.out_unit), H.rel_err(u, u_ref), H.rel_err(S, S_ref))
    H.check(e, in_dtype, rec_dtype, (tag, "decode"))
    assert lay.spare_clean() and not lay.status().any()
    # verification (a chain or a tree) on top of a ragged buffer
    cap = C - 1 + T
    if bool(rng.integers(0, 2)):
        e = _verify_case(B, Hk, Hv, d, C, cap, T, in_dtype, 9100 + seed, block_size=block, scatter=scatter, **types)
    else:
        e = _tree_case(B, Hk, Hv, d, C, cap, T, in_dtype, 9100 + seed, block_size=block, scatter=scatter, **types)
    H.check(e, in_dtype, rec_dtype, (tag, "verify"))
    # a short context from the buffer alone
    Lmax = int(rng.integers(1, 65))
    e = _direct_case(B, Hk, Hv, d, Lmax, max(Lmax + int(rng.integers(0, 9)), 1), in_dtype, 9200 + seed,
                     block_size=block, scatter=scatter, **types)
    H.check(e, in_dtype, rec_dtype, (tag, "direct"))


@pytest.mark.parametrize("pattern", ["same", "alternating", "anticorrelated"])
def test_repeated_keys_and_no_decay_stay_within_tolerance(pattern):
    """Strongly correlated keys, beta close to 1 and no decay at all: the coefficients
    Gamma (k_i.k_l) are all +-1 (one key; one key with alternating sign) or +-0.9 (two keys with
    k1.k2 = -0.9 taking turns), the hardest cases for the forward substitution and for the block
    inverse of kvb_direct.  Decode over several chunks, 8 drafts, contexts of 64 and 128 tokens."""
    rng = np.random.default_rng(170)
    B, Hk, Hv, d, C = 3, 1, 2, 128, 16
    def same_key_tokens(T):
        tok = synth.token_stream(rng, B, T, Hk, Hv, d, d, "bf16")
        k1 = tok["k"][:, :1].copy()
        if pattern == "same":
            tok["k"][:] = k1
        elif pattern == "alternating":
            tok["k"][:] = k1 * ((-1.0) ** np.arange(T))[None, :, None, None]
        else:
            r = tok["k"][:, 1:2]
            r = r - (r * k1).sum(-1, keepdims=True) * k1 / (k1 * k1).sum(-1, keepdims=True)
            k2 = -0.9 * k1 + np.sqrt(1.0 - 0.81) * r / np.linalg.norm(r, axis=-1, keepdims=True)
            k2 = synth.round_to_bf16(k2.astype(np.float32)).astype(tok["k"].dtype)
            for t in range(T):
                tok["k"][:, t:t + 1] = k1 if t % 2 == 0 else k2
        tok["g"][:] = 0.0
        tok["beta"][:] = 0.96875          # exactly representable
        return tok
    tok = same_key_tokens(40)
    S0 = H.prefix_state(rng, B, Hk, Hv, d, d, "bf16", 8)
    lay = H.Layer(B, Hk, Hv, d, d, cap=C, in_dtype="bf16")
    o, u, S, _ = H.run_decode(lay, S0, tok, C, fused=True)
    o_ref, u_ref, S_ref = oracle.kvb_decode_expected(S0, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"])
    e = (H.rel_err(o, o_ref), H.rel_err(u, u_ref), H.rel_err(S, S_ref))
    say(pattern + " key, decode rel err out/u/state: %.2e %.2e %.2e" % e)
    H.check(e, "bf16")
    # drafts
    vt = same_key_tokens(8)
    lay = H.Layer(B, Hk, Hv, d, d, cap=8, in_dtype="bf16")
    lay.set_state(S0)
    out = torch.empty((B, 8, Hv, d), dtype=torch.float32, device="cuda")
    lay.verify(8, H.upload_tokens(vt, "bf16"), out)
    o_ref, _, _ = oracle.kvb_verify_expected(S0, vt["q"], vt["k"], vt["v"], vt["g"], vt["beta"], np.zeros(B, np.int32))
    e = H.rel_err(out.cpu().numpy(), o_ref)
    say(pattern + " key, verify rel err: %.2e" % e)
    H.check(e, "bf16")
    # a whole context
    dt_ = same_key_tokens(64)
    lay = H.Layer(B, Hk, Hv, d, d, cap=64, in_dtype="bf16", with_state=False)
    out = torch.empty((B, 64, Hv, d), dtype=torch.float32, device="cuda")
    lay.direct(H.dev(np.full(B, 64, np.int32)), 64, H.upload_tokens(dt_, "bf16"), out)
    o_ref, _, _ = oracle.kvb_direct_expected(dt_["q"], dt_["k"], dt_["v"], dt_["g"], dt_["beta"], np.full(B, 64, np.int32))
    e = H.rel_err(out.cpu().numpy(), o_ref)
    say(pattern + " key, direct rel err: %.2e" % e)
    H.check(e, "bf16")
    # ... and one of 128 tokens (the 8-block kernel)
    dt_ = same_key_tokens(128)
    lay = H.Layer(B, Hk, Hv, d, d, cap=128, in_dtype="bf16", with_state=False)
    out = torch.empty((B, 128, Hv, d), dtype=torch.float32, device="cuda")
    lay.direct(H.dev(np.full(B, 128, np.int32)), 128, H.upload_tokens(dt_, "bf16"), out)
    o_ref, _, _ = oracle.kvb_direct_expected(dt_["q"], dt_["k"], dt_["v"], dt_["g"], dt_["beta"], np.full(B, 128, np.int32))
    e = H.rel_err(out.cpu().numpy(), o_ref)
    say(pattern + " key, direct (128 tokens) rel err: %.2e" % e)
    H.check(e, "bf16")
