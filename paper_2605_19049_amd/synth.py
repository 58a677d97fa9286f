"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module only draws random numbers, normalises / rounds them and names the
workload shapes.  It contains none of the method's arithmetic and imports
neither the HIP binding nor the CPU oracle.

Distributions (all workloads): q, k ~ N(0,1) then L2-normalised per head vector;
v ~ N(0,1); log decay g ~ U(-0.5, 0); beta = sigmoid(N(0,1)).  Values are drawn
in float64 with numpy's PCG64 ``default_rng(seed)`` in the order q, k, v, g,
beta, then rounded ONCE to the workload's input type, so that the fp64 oracle and
the GPU library receive bit-identical numbers.
"""
from dataclasses import dataclass

import numpy as np


def round_to_bf16(x):
    """Round float values to the nearest bfloat16 (ties to even); returns float32
    holding exactly representable values."""
    a = np.ascontiguousarray(x, dtype=np.float32)
    bits = a.view(np.uint32)
    out = (bits >> np.uint32(16)) & np.uint32(1)       # finite inputs: no uint32 wrap-around
    out += np.uint32(0x7FFF)
    out += bits
    out &= np.uint32(0xFFFF0000)
    return out.view(np.float32).reshape(a.shape)


def bf16_bits(x):
    """uint16 bit patterns of values that are already bf16-representable."""
    a = np.ascontiguousarray(x, dtype=np.float32)
    bits = a.view(np.uint32)
    assert not np.any(bits & 0xFFFF), "value is not bf16-representable"
    return (bits >> 16).astype(np.uint16).reshape(a.shape)


def round_to_fp16(x):
    return np.asarray(x, dtype=np.float32).astype(np.float16).astype(np.float32)


def round_input(x, in_dtype):
    """in_dtype: 'f32', 'bf16' or 'f16' -- the type q, k, v are handed over in."""
    if in_dtype == "f32":
        return np.asarray(x, dtype=np.float32)
    if in_dtype == "bf16":
        return round_to_bf16(x)
    if in_dtype == "f16":
        return round_to_fp16(x)
    raise ValueError(in_dtype)


@dataclass(frozen=True)
class Workload:
    """Shape of one synthetic workload (a GDN layer's decode-side problem)."""
    name: str
    B: int          # requests
    Hk: int         # q/k heads
    Hv: int         # v heads (Hv % Hk == 0)
    dk: int
    dv: int
    C: int          # chunk size: flush when the buffer holds C records
    cap: int        # records a request's buffer can hold
    in_dtype: str   # 'f32' | 'bf16'
    steps: int = 0  # decode steps
    T: int = 0      # draft tokens (verify)
    Lmax: int = 0   # longest context (direct)
    layers: int = 1
    seed: int = 0
    prefix: int = 64  # tokens folded into the initial state
    ragged: bool = False  # requests start at independent buffer fills ~U{0..C-1}


# The five workloads the build is measured / parity-checked on.
WORKLOADS = {
    "tiny_fp32": Workload("tiny_fp32", B=1, Hk=2, Hv=2, dk=32, dv=32, C=8, cap=8,
                          in_dtype="f32", steps=32, seed=0),
    "qwen3next_decode": Workload("qwen3next_decode", B=64, Hk=16, Hv=32, dk=128, dv=128,
                                 C=16, cap=16, in_dtype="bf16", steps=256, seed=2),
    "spec_verify": Workload("spec_verify", B=128, Hk=16, Hv=32, dk=128, dv=128, C=16,
                            cap=20, in_dtype="bf16", T=4, seed=3),
    "short_direct": Workload("short_direct", B=256, Hk=16, Hv=32, dk=128, dv=128, C=64,
                             cap=64, in_dtype="bf16", Lmax=64, seed=4, prefix=0),
    "long_mixed": Workload("long_mixed", B=512, Hk=16, Hv=32, dk=128, dv=128, C=64,
                           cap=64, in_dtype="bf16", steps=128, layers=36, seed=5, ragged=True),
}


def token_stream(rng, B, T, Hk, Hv, dk, dv, in_dtype):
    """T tokens for B requests.  Returns float32 arrays whose values are exactly
    representable in ``in_dtype``: q,k [B,T,Hk,dk]; v [B,T,Hv,dv]; g,beta [B,T,Hv]."""
    q = rng.standard_normal((B, T, Hk, dk))
    k = rng.standard_normal((B, T, Hk, dk))
    v = rng.standard_normal((B, T, Hv, dv))
    g = rng.uniform(-0.5, 0.0, (B, T, Hv))
    beta = 1.0 / (1.0 + np.exp(-rng.standard_normal((B, T, Hv))))
    q /= np.linalg.norm(q, axis=-1, keepdims=True)
    k /= np.linalg.norm(k, axis=-1, keepdims=True)
    return {
        "q": round_input(q, in_dtype), "k": round_input(k, in_dtype),
        "v": round_input(v, in_dtype),
        "g": g.astype(np.float32), "beta": beta.astype(np.float32),
    }


def random_state(rng, B, Hv, dk, dv, std=0.5):
    """A stand-in committed state (fp32) when no prefix is replayed."""
    return (std * rng.standard_normal((B, Hv, dk, dv))).astype(np.float32)


def buffer_fills(rng, B, lo, hi):
    """Per-request number of records already buffered, uniform on lo..hi inclusive."""
    return rng.integers(lo, hi + 1, size=B).astype(np.int32)


def accepted_lengths(rng, B, T):
    """Per-request accepted draft prefix, uniform on 0..T."""
    return rng.integers(0, T + 1, size=B).astype(np.int32)


def context_lengths(rng, B, lo, hi):
    """Per-request context length, uniform on lo..hi inclusive."""
    return rng.integers(lo, hi + 1, size=B).astype(np.int32)


def draft_trees(rng, B, T, kind="random"):
    """Parent pointers of B draft trees with T nodes each, parents before children
    (-1 = the node follows the last committed token).  kind: "random" (parent uniform over
    -1..i-1), "chain", "star", or "binary" (node i hangs under node (i-1)//2, the root under -1)."""
    par = np.empty((B, T), np.int32)
    for i in range(T):
        if kind == "chain":
            par[:, i] = i - 1
        elif kind == "star":
            par[:, i] = -1
        elif kind == "binary":
            par[:, i] = (i - 1) // 2 if i > 0 else -1
        else:
            par[:, i] = rng.integers(-1, i, size=B)
    return par


def accepted_paths(rng, parent):
    """For each tree a random accepted leaf (-1 = nothing accepted, probability 1/(T+1)) and the
    root path that ends there: (leaf [B], path [B,T] padded with 0, path_len [B])."""
    B, T = parent.shape
    leaf = rng.integers(-1, T, size=B).astype(np.int32)
    path = np.zeros((B, T), np.int32)
    plen = np.zeros(B, np.int32)
    for b in range(B):
        nodes, n = [], int(leaf[b])
        while n >= 0:
            nodes.append(n)
            n = int(parent[b, n])
        nodes.reverse()
        plen[b] = len(nodes)
        path[b, :len(nodes)] = nodes
    return leaf, path, plen
