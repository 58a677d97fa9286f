"""TEST INFRASTRUCTURE: ctypes front end of the fp64 recurrence in gdn_oracle.c.

The four KVBuffer calls are regroupings of one recurrence (paper Sec. 2.1 and
App. A.1), so each ``*_expected`` helper below only decides which tokens are
fed to that recurrence and from which starting state.  No arithmetic of the
method lives in this file.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gdn_oracle.c")
_LIB = os.path.join(_HERE, "libgdn_oracle.so")
_lib = None


def build_lib(force=False):
    """Compile gdn_oracle.c with gcc (OpenMP) into libgdn_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".%d.tmp" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_lib())
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        lib.gdn_oracle_sequence.restype = ctypes.c_int
        lib.gdn_oracle_sequence.argtypes = [ctypes.c_int] * 6 + [
            ip, ctypes.c_double, dp, dp, dp, dp, dp, dp, dp, dp, ctypes.c_int]
        _lib = lib
    return _lib


def _f64(x):
    return np.ascontiguousarray(np.asarray(x), dtype=np.float64)


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def gdn_sequence(S0, q, k, v, g, beta, scale=1.0, lens=None, nthreads=0):
    """Run the recurrence (App. A.1, Eq. 11-12; output rule Eq. 3) over T tokens.

    S0 [B,Hv,dk,dv]; q,k [B,T,Hk,dk]; v [B,T,Hv,dv]; g (log decay), beta [B,T,Hv];
    lens [B] optional: request b consumes only its first lens[b] tokens.
    Returns (o [B,T,Hv,dv], u [B,T,Hv,dv], S_end [B,Hv,dk,dv], threads_used);
    rows t >= lens[b] of o and u are NaN.
    """
    lib = _load()
    S = _f64(S0).copy()
    q, k, v, g, beta = map(_f64, (q, k, v, g, beta))
    B, Hv, dk, dv = S.shape
    T, Hk = q.shape[1], q.shape[2]
    assert q.shape == (B, T, Hk, dk) and k.shape == q.shape, (q.shape, k.shape)
    assert v.shape == (B, T, Hv, dv), v.shape
    assert g.shape == (B, T, Hv) and beta.shape == g.shape
    o = np.full((B, T, Hv, dv), np.nan)
    u = np.full((B, T, Hv, dv), np.nan)
    lp = None
    if lens is not None:
        lens = np.ascontiguousarray(np.asarray(lens), dtype=np.int32)
        assert lens.shape == (B,)
        lp = lens.ctypes.data_as(ctypes.POINTER(ctypes.c_int))
    used = lib.gdn_oracle_sequence(B, T, Hk, Hv, dk, dv, lp, float(scale), _dptr(S),
                                   _dptr(q), _dptr(k), _dptr(v), _dptr(g), _dptr(beta),
                                   _dptr(o), _dptr(u), int(nthreads))
    if used < 0:
        raise ValueError("gdn_oracle_sequence: bad argument")
    return o, u, S, used


def kvb_decode_expected(S, q, k, v, g, beta, scale=1.0):
    """Chunkwise decoding (Sec. 3.2; Eq. 16) yields, token by token, exactly what
    the recurrence yields from the true (not the deferred) state S."""
    o, u, S_end, _ = gdn_sequence(S, q, k, v, g, beta, scale)
    return o, u, S_end


def kvb_verify_expected(S, q, k, v, g, beta, accepted, scale=1.0):
    """Parallel verification (Sec. 3.3, Eq. 7-8): outputs of all T sequential
    drafts as the recurrence gives them from a scratch copy of the true state;
    the state then advances by each request's accepted prefix only."""
    o, u, _, _ = gdn_sequence(S, q, k, v, g, beta, scale)
    _, _, S_acc, _ = gdn_sequence(S, q, k, v, g, beta, scale, lens=accepted)
    return o, u, S_acc


def kvb_direct_expected(q, k, v, g, beta, lens, scale=1.0):
    """KV-only path (Sec. 3.4; Eq. 13-14): the recurrence started from a zero
    state; request b has lens[b] tokens."""
    B, T, Hk, dk = np.asarray(q).shape
    Hv, dv = np.asarray(v).shape[2:]
    S0 = np.zeros((B, Hv, dk, dv))
    o, u, S_end, _ = gdn_sequence(S0, q, k, v, g, beta, scale, lens=lens)
    return o, u, S_end


def tree_paths(parent):
    """Root paths of a draft tree.  parent [B,T] with parent[b,i] in {-1, 0..i-1} (-1: the
    node follows the last committed token).  Returns (idx [B,T,T], plen [B,T]): the nodes of
    the path that ends in node i, oldest first, padded with node i itself."""
    parent = np.asarray(parent)
    B, T = parent.shape
    idx = np.zeros((B, T, T), np.int64)
    plen = np.zeros((B, T), np.int32)
    for b in range(B):
        for i in range(T):
            path, n = [], i
            while n >= 0:
                assert n < T and parent[b, n] < n, "parent indices must precede their children"
                path.append(n)
                n = int(parent[b, n])
            path.reverse()
            plen[b, i] = len(path)
            idx[b, i, :len(path)] = path
            idx[b, i, len(path):] = i
    return idx, plen


def kvb_verify_tree_expected(S, q, k, v, g, beta, parent, accepted_leaf=None, scale=1.0):
    """Verification of tree-shaped drafts (Sec. 3.3 with the mask M of App. A.1: a draft
    sees the committed context and its own ancestors only).  Node i's output and delta value
    are what the recurrence yields at the end of the root path of node i, started from a
    scratch copy of the true state S; every path is simply fed to the recurrence.
    accepted_leaf [B] (-1 = nothing accepted): the state then advances along the root path of
    that node only (Eq. 8).  Returns (o [B,T,Hv,dv], u [B,T,Hv,dv], S_acc)."""
    S = _f64(S)
    q, k, v, g, beta = map(_f64, (q, k, v, g, beta))
    B, T = g.shape[:2]
    idx, plen = tree_paths(parent)
    bb = np.arange(B)[:, None, None]
    # one "request" per (b, node): the tokens of its root path, in order
    def along(x):
        return x[bb, idx].reshape((B * T, T) + x.shape[2:])
    Sx = np.repeat(S, T, axis=0)
    o_p, u_p, _, _ = gdn_sequence(Sx, along(q), along(k), along(v), along(g), along(beta), scale,
                                  lens=plen.reshape(-1))
    last = (plen.reshape(-1) - 1)
    rows = np.arange(B * T)
    o = o_p[rows, last].reshape((B, T) + o_p.shape[2:])
    u = u_p[rows, last].reshape((B, T) + u_p.shape[2:])
    S_acc = S.copy()
    if accepted_leaf is not None:
        leaf = np.asarray(accepted_leaf)
        sel = np.where(leaf >= 0, leaf, 0)
        ib = idx[np.arange(B), sel]                         # [B,T] path of the accepted leaf
        ln = np.where(leaf >= 0, plen[np.arange(B), sel], 0).astype(np.int32)
        b1 = np.arange(B)[:, None]
        _, _, S_acc, _ = gdn_sequence(S, q[b1, ib], k[b1, ib], v[b1, ib], g[b1, ib], beta[b1, ib], scale, lens=ln)
    return o, u, S_acc
