"""CPU pins of the parity oracle (oracle/gdn_oracle.c).

Each test fixes the oracle against something other than itself: a hand-worked
example, closed forms that follow from App. A.1 Eq. 11-12, the dense-inverse
matrix forms of Eq. 13 / Eq. 15, and the reduction to plain linear attention
(Sec. 2.1, Eq. 1).  Shapes use dk != dv so a transposed operand cannot pass.
"""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _inputs(seed, B, T, Hk, Hv, dk, dv, normalise=True):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, T, Hk, dk))
    k = rng.standard_normal((B, T, Hk, dk))
    if normalise:
        q /= np.linalg.norm(q, axis=-1, keepdims=True)
        k /= np.linalg.norm(k, axis=-1, keepdims=True)
    v = rng.standard_normal((B, T, Hv, dv))
    g = rng.uniform(-0.5, 0.0, (B, T, Hv))
    beta = 1 / (1 + np.exp(-rng.standard_normal((B, T, Hv))))
    S0 = rng.standard_normal((B, Hv, dk, dv))
    return S0, q, k, v, g, beta


# ---------------------------------------------------------------- hand example
def _read_golden(path):
    out = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        out[key] = np.array([float(x) for x in vals])
    return out


def test_hand_worked_example(oracle):
    gold = _read_golden(os.path.join(GOLDEN, "gdn_hand_example.txt"))
    S0 = gold["S0"].reshape(1, 1, 2, 2)
    q = gold["q"].reshape(1, 2, 1, 2)
    k = gold["k"].reshape(1, 2, 1, 2)
    v = gold["v"].reshape(1, 2, 1, 2)
    g = np.log(gold["alpha"]).reshape(1, 2, 1)
    beta = gold["beta"].reshape(1, 2, 1)
    o, u, S, _ = oracle.gdn_sequence(S0, q, k, v, g, beta)
    np.testing.assert_allclose(u.reshape(-1), gold["u"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(o.reshape(-1), gold["o"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(S.reshape(-1), gold["S2"], rtol=0, atol=1e-14)


# ---------------------------------------------------------------- closed forms
def test_beta_zero_is_pure_decay(oracle):
    """beta = 0 in Eq. 12 leaves S_t = alpha_t S_{t-1}: S_T = prod(alpha) S0 and
    o_t = prod_{i<=t}(alpha_i) q_t S0."""
    S0, q, k, v, g, beta = _inputs(1, 2, 6, 1, 2, 5, 3)
    beta[:] = 0
    o, u, S, _ = oracle.gdn_sequence(S0, q, k, v, g, beta)
    gam = np.exp(np.cumsum(g, axis=1))                      # [B,T,Hv]
    np.testing.assert_allclose(S, gam[:, -1, :, None, None] * S0, rtol=1e-13)
    qh = np.repeat(q, 2, axis=2)                            # Hk=1 -> both v heads
    want = gam[..., None] * np.einsum("bthi,bhij->bthj", qh, S0)
    np.testing.assert_allclose(o, want, rtol=1e-12, atol=1e-13)
    assert np.all(u == 0)


def test_no_gate_no_write_leaves_state_bit_identical(oracle):
    S0, q, k, v, g, beta = _inputs(2, 2, 5, 2, 2, 4, 6)
    g[:] = 0
    beta[:] = 0
    _, _, S, _ = oracle.gdn_sequence(S0, q, k, v, g, beta)
    assert np.array_equal(S, S0)


def test_orthonormal_keys_form_an_associative_memory(oracle):
    """alpha = beta = 1, orthonormal keys, zero start: the delta term vanishes,
    S = sum_i k_i^T v_i, and querying with k_i returns v_i exactly."""
    rng = np.random.default_rng(3)
    dk, dv, T = 6, 4, 6
    Q, _ = np.linalg.qr(rng.standard_normal((dk, dk)))
    k = Q[:T].reshape(1, T, 1, dk)
    v = rng.standard_normal((1, T, 1, dv))
    g = np.zeros((1, T, 1))
    beta = np.ones((1, T, 1))
    S0 = np.zeros((1, 1, dk, dv))
    o, u, S, _ = oracle.gdn_sequence(S0, k, k, v, g, beta)   # q_t = k_t
    np.testing.assert_allclose(S[0, 0], Q[:T].T @ v[0, :, 0], atol=1e-13)
    np.testing.assert_allclose(o, v, atol=1e-13)             # reads its own write
    # after all writes every key still retrieves its value
    o2, _, _, _ = oracle.gdn_sequence(S, k, k, np.zeros_like(v), g, np.zeros_like(beta))
    np.testing.assert_allclose(o2, v, atol=1e-13)


def test_same_key_twice_overwrites(oracle):
    """Delta rule with beta = 1: writing v2 under a key that holds v1 erases v1."""
    rng = np.random.default_rng(4)
    dk, dv = 5, 3
    key = rng.standard_normal(dk)
    key /= np.linalg.norm(key)
    k = np.tile(key, (1, 2, 1, 1))
    v = rng.standard_normal((1, 2, 1, dv))
    S0 = np.zeros((1, 1, dk, dv))
    o, u, S, _ = oracle.gdn_sequence(S0, k, k, v, np.zeros((1, 2, 1)), np.ones((1, 2, 1)))
    np.testing.assert_allclose(o[0, 1, 0], v[0, 1, 0], atol=1e-13)
    np.testing.assert_allclose(S[0, 0], np.outer(key, v[0, 1, 0]), atol=1e-13)
    # with beta = 1/2 the stored value moves half way (the (1-beta) mix of Eq. 12)
    o, _, _, _ = oracle.gdn_sequence(S0, k, k, v, np.zeros((1, 2, 1)),
                                     np.array([1.0, 0.5]).reshape(1, 2, 1))
    np.testing.assert_allclose(o[0, 1, 0], 0.5 * (v[0, 0, 0] + v[0, 1, 0]), atol=1e-13)


def test_orthogonal_keys_reduce_to_linear_attention(oracle):
    """alpha = 1 and mutually orthogonal unit keys: k_t S~ = 0 for every new key, so
    GDN equals Eq. 1 with values beta_t v_t: O = tril(Q K^T) (Diag(beta) V)."""
    rng = np.random.default_rng(5)
    dk, dv, T = 8, 5, 7
    Qm, _ = np.linalg.qr(rng.standard_normal((dk, dk)))
    K = Qm[:T]
    Qr = rng.standard_normal((T, dk))
    V = rng.standard_normal((T, dv))
    beta = rng.random(T)
    want = np.tril(Qr @ K.T) @ (beta[:, None] * V)
    o, _, _, _ = oracle.gdn_sequence(np.zeros((1, 1, dk, dv)), Qr.reshape(1, T, 1, dk),
                                     K.reshape(1, T, 1, dk), V.reshape(1, T, 1, dv),
                                     np.zeros((1, T, 1)), beta.reshape(1, T, 1))
    np.testing.assert_allclose(o[0, :, 0], want, atol=1e-13)


# ------------------------------------------------- dense-inverse matrix forms
def chunk_matrix_form(S0, Q, K, V, g, beta):
    """Eq. 15 for one head, one chunk, by explicit dense inverse.  Readings: the
    Gram matrix is K K^T (m x m); the state term of U carries Diag(gamma) next
    to K (as the single-token form Eq. 16 has it); gamma includes the token's own gate.
    Returns O, U and the end-of-chunk state (last line of Eq. 16)."""
    m = Q.shape[0]
    gam = np.exp(np.cumsum(g))
    Gam = np.tril(gam[:, None] / gam[None, :])
    A = np.linalg.inv(np.eye(m) + np.tril(beta[:, None] * (Gam * (K @ K.T)), -1))
    Vt = A @ (beta[:, None] * V)
    Kt = A @ (beta[:, None] * gam[:, None] * K)
    U = Vt - Kt @ S0
    O = gam[:, None] * (Q @ S0) + ((Q @ K.T) * Gam) @ U
    S_end = gam[-1] * S0 + (K * (gam[-1] / gam)[:, None]).T @ U
    return O, U, S_end


@pytest.mark.parametrize("chunk", [1, 2, 3, 7, 12])
def test_chunkwise_matrix_form_equals_recurrence(oracle, chunk):
    B, T, Hk, Hv, dk, dv = 2, 12, 2, 4, 6, 5
    S0, q, k, v, g, beta = _inputs(6, B, T, Hk, Hv, dk, dv)
    o, u, S, _ = oracle.gdn_sequence(S0, q, k, v, g, beta)
    for b in range(B):
        for h in range(Hv):
            hk = h // (Hv // Hk)
            Sc = S0[b, h]
            for s in range(0, T, chunk):
                e = min(T, s + chunk)
                O, U, Sc = chunk_matrix_form(Sc, q[b, s:e, hk], k[b, s:e, hk], v[b, s:e, h],
                                             g[b, s:e, h], beta[b, s:e, h])
                np.testing.assert_allclose(O, o[b, s:e, h], rtol=1e-10, atol=1e-11)
                np.testing.assert_allclose(U, u[b, s:e, h], rtol=1e-10, atol=1e-11)
            np.testing.assert_allclose(Sc, S[b, h], rtol=1e-10, atol=1e-11)


def test_parallel_matrix_form_equals_recurrence_from_zero_state(oracle):
    """Eq. 13: no state at all; also the ragged-length rule of the direct path."""
    B, T, Hk, Hv, dk, dv = 3, 9, 1, 2, 7, 4
    _, q, k, v, g, beta = _inputs(7, B, T, Hk, Hv, dk, dv)
    lens = np.array([9, 4, 1], dtype=np.int32)
    o, u, S = oracle.kvb_direct_expected(q, k, v, g, beta, lens)
    for b in range(B):
        L = lens[b]
        for h in range(Hv):
            gam = np.exp(np.cumsum(g[b, :L, h]))
            Gam = np.tril(gam[:, None] / gam[None, :])
            K, Q = k[b, :L, 0], q[b, :L, 0]
            A = np.linalg.inv(np.eye(L) + np.tril(beta[b, :L, h, None] * (Gam * (K @ K.T)), -1))
            Vt = A @ (beta[b, :L, h, None] * v[b, :L, h])
            O = ((Q @ K.T) * Gam) @ Vt
            np.testing.assert_allclose(O, o[b, :L, h], rtol=1e-10, atol=1e-11)
            np.testing.assert_allclose(Vt, u[b, :L, h], rtol=1e-10, atol=1e-11)
        assert np.all(np.isnan(o[b, L:]))


def test_literal_gamma_placement_is_not_the_recurrence(oracle):
    """The printed K~ = Diag(gamma) A Diag(beta) K differs from the recurrence once
    gates are not all 1; this documents why the other reading is used."""
    S0, q, k, v, g, beta = _inputs(8, 1, 7, 1, 1, 6, 5)
    o, _, _, _ = oracle.gdn_sequence(S0, q, k, v, g, beta)
    Q, K, V, gg, bb = q[0, :, 0], k[0, :, 0], v[0, :, 0], g[0, :, 0], beta[0, :, 0]
    gam = np.exp(np.cumsum(gg))
    Gam = np.tril(gam[:, None] / gam[None, :])
    A = np.linalg.inv(np.eye(7) + np.tril(bb[:, None] * (Gam * (K @ K.T)), -1))
    U_lit = A @ (bb[:, None] * V) - (gam[:, None] * (A @ (bb[:, None] * K))) @ S0[0, 0]
    O_lit = gam[:, None] * (Q @ S0[0, 0]) + ((Q @ K.T) * Gam) @ U_lit
    assert np.abs(O_lit - o[0, :, 0]).max() > 1e-3


# ------------------------------------------------------- driver-level behaviour
def test_sequence_can_be_split_anywhere(oracle):
    S0, q, k, v, g, beta = _inputs(9, 2, 10, 2, 4, 5, 3)
    o, u, S, _ = oracle.gdn_sequence(S0, q, k, v, g, beta)
    o1, u1, S1, _ = oracle.gdn_sequence(S0, q[:, :4], k[:, :4], v[:, :4], g[:, :4], beta[:, :4])
    o2, u2, S2, _ = oracle.gdn_sequence(S1, q[:, 4:], k[:, 4:], v[:, 4:], g[:, 4:], beta[:, 4:])
    assert np.array_equal(np.concatenate([o1, o2], 1), o)
    assert np.array_equal(np.concatenate([u1, u2], 1), u)
    assert np.array_equal(S2, S)


def test_grouped_heads_use_qk_head_h_div_r(oracle):
    B, T, Hk, Hv, dk, dv = 1, 4, 2, 6, 5, 3
    S0, q, k, v, g, beta = _inputs(10, B, T, Hk, Hv, dk, dv)
    o, _, S, _ = oracle.gdn_sequence(S0, q, k, v, g, beta)
    for h in range(Hv):
        hk = h // 3
        oh, _, Sh, _ = oracle.gdn_sequence(S0[:, h:h + 1], q[:, :, hk:hk + 1], k[:, :, hk:hk + 1],
                                           v[:, :, h:h + 1], g[:, :, h:h + 1], beta[:, :, h:h + 1])
        assert np.array_equal(oh[:, :, 0], o[:, :, h])
        assert np.array_equal(Sh[:, 0], S[:, h])


def test_scale_multiplies_outputs_only(oracle):
    S0, q, k, v, g, beta = _inputs(11, 1, 5, 1, 1, 4, 3)
    o1, u1, S1, _ = oracle.gdn_sequence(S0, q, k, v, g, beta, scale=1.0)
    o2, u2, S2, _ = oracle.gdn_sequence(S0, q, k, v, g, beta, scale=0.25)
    np.testing.assert_allclose(o2, 0.25 * o1, rtol=1e-15)
    assert np.array_equal(u1, u2) and np.array_equal(S1, S2)


def test_verify_equals_sequential_decode_and_commits_accepted_prefix(oracle):
    """Sec. 3.3: draft outputs are those of one-at-a-time decoding; the state moves
    by the accepted prefix only (accepted = 0 leaves it untouched)."""
    B, T, Hk, Hv, dk, dv = 4, 4, 1, 2, 6, 5
    S0, q, k, v, g, beta = _inputs(12, B, T, Hk, Hv, dk, dv)
    acc = np.array([0, 1, 3, 4], dtype=np.int32)
    o, u, S_acc = oracle.kvb_verify_expected(S0, q, k, v, g, beta, acc)
    S = S0.copy()
    for t in range(T):
        ot, ut, S = oracle.kvb_decode_expected(S, q[:, t:t + 1], k[:, t:t + 1], v[:, t:t + 1],
                                               g[:, t:t + 1], beta[:, t:t + 1])
        assert np.array_equal(ot[:, 0], o[:, t])
        for b in range(B):
            if acc[b] == t + 1:
                assert np.array_equal(S[b], S_acc[b])
    assert np.array_equal(S_acc[0], S0[0])


def test_planted_mistakes_are_caught(oracle):
    """A transposed write, a dropped gate or a pre-update read each break a pin:
    here checked directly against the dense-inverse form on one head."""
    S0, q, k, v, g, beta = _inputs(13, 1, 6, 1, 1, 5, 5)
    Q, K, V, gg, bb = q[0, :, 0], k[0, :, 0], v[0, :, 0], g[0, :, 0], beta[0, :, 0]
    O, U, S_end = chunk_matrix_form(S0[0, 0], Q, K, V, gg, bb)

    def recur(transpose=False, no_gate=False, pre_read=False):
        S = S0[0, 0].copy()
        out = []
        for t in range(6):
            if not no_gate:
                S = np.exp(gg[t]) * S
            if pre_read:
                out.append(Q[t] @ S)
            u = bb[t] * (V[t] - K[t] @ S)
            S = S + (np.outer(u, K[t]) if transpose else np.outer(K[t], u))
            if not pre_read:
                out.append(Q[t] @ S)
        return np.array(out)

    np.testing.assert_allclose(recur(), O, rtol=1e-10, atol=1e-11)
    for kw in ({"transpose": True}, {"no_gate": True}, {"pre_read": True}):
        assert np.abs(recur(**kw) - O).max() > 1e-3, kw


# ------------------------------------------------------------ tree-shaped drafts
def tree_matrix_form(S0, Q, K, V, g, beta, parent):
    """The masked matrix form for one head (App. A.1: M_ij != 0 iff j is a prefix token of i,
    gamma_t = product of alpha over Par(t)), on top of a committed state S0 as in Eq. 15.
    M is built from the parent pointers; everything else is the dense inverse as printed."""
    m = Q.shape[0]
    M = np.zeros((m, m))
    G = np.zeros(m)
    for i in range(m):
        n = i
        while n >= 0:
            M[i, n] = 1.0
            G[i] += g[n]
            n = parent[n]
    gam = np.exp(G)
    Gam = M * (gam[:, None] / gam[None, :])
    A = np.linalg.inv(np.eye(m) + np.tril(beta[:, None] * (Gam * (K @ K.T)), -1))
    U = A @ (beta[:, None] * (V - gam[:, None] * (K @ S0)))
    O = gam[:, None] * (Q @ S0) + ((Q @ K.T) * Gam) @ U
    return O, U, gam, Gam


@pytest.mark.parametrize("seed", [21, 22, 23])
def test_tree_drafts_equal_the_masked_matrix_form(oracle, seed):
    """Every draft of a random tree, against the dense-inverse form with the ancestor mask;
    the committed state after accepting a leaf, against S0 advanced by that root path."""
    B, T, Hk, Hv, dk, dv = 3, 7, 1, 2, 6, 5
    S0, q, k, v, g, beta = _inputs(seed, B, T, Hk, Hv, dk, dv)
    rng = np.random.default_rng(seed)
    parent = np.stack([[int(rng.integers(-1, i)) for i in range(T)] for _ in range(B)])
    leaf = np.array([T - 1, 2, -1])
    o, u, S_acc = oracle.kvb_verify_tree_expected(S0, q, k, v, g, beta, parent, accepted_leaf=leaf)
    for b in range(B):
        for h in range(Hv):
            O, U, gam, Gam = tree_matrix_form(S0[b, h], q[b, :, 0], k[b, :, 0], v[b, :, h], g[b, :, h],
                                              beta[b, :, h], parent[b])
            np.testing.assert_allclose(O, o[b, :, h], rtol=1e-10, atol=1e-11)
            np.testing.assert_allclose(U, u[b, :, h], rtol=1e-10, atol=1e-11)
            if leaf[b] >= 0:   # Eq. 8 / last line of Eq. 16 over the accepted path only
                L = leaf[b]
                want = gam[L] * S0[b, h] + (k[b, :, 0] * Gam[L][:, None]).T @ U
                np.testing.assert_allclose(want, S_acc[b, h], rtol=1e-10, atol=1e-11)
            else:
                assert np.array_equal(S_acc[b, h], S0[b, h])


def test_tree_special_cases(oracle):
    """A chain is sequential verification; a star is T independent single-token steps."""
    B, T, Hk, Hv, dk, dv = 2, 5, 1, 2, 6, 5
    S0, q, k, v, g, beta = _inputs(24, B, T, Hk, Hv, dk, dv)
    chain = np.tile(np.arange(T) - 1, (B, 1))
    o_c, u_c, S_c = oracle.kvb_verify_tree_expected(S0, q, k, v, g, beta, chain, accepted_leaf=np.array([3, 0]))
    o_s, u_s, S_s = oracle.kvb_verify_expected(S0, q, k, v, g, beta, np.array([4, 1], dtype=np.int32))
    assert np.array_equal(o_c, o_s) and np.array_equal(u_c, u_s) and np.array_equal(S_c, S_s)
    star = np.full((B, T), -1)
    o_t, u_t, _ = oracle.kvb_verify_tree_expected(S0, q, k, v, g, beta, star)
    for b in range(B):
        for h in range(Hv):
            for t in range(T):   # one step of Eq. 11-12 written out
                S = np.exp(g[b, t, h]) * S0[b, h]
                uu = beta[b, t, h] * (v[b, t, h] - k[b, t, 0] @ S)
                oo = q[b, t, 0] @ (S + np.outer(k[b, t, 0], uu))
                np.testing.assert_allclose(uu, u_t[b, t, h], rtol=1e-12, atol=1e-13)
                np.testing.assert_allclose(oo, o_t[b, t, h], rtol=1e-12, atol=1e-13)
