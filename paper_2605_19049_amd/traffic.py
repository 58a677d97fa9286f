"""Algorithmic HBM bytes of each kvb call -- the numerators of the roofline figures.

"Algorithmic" means every array element the call has to read or write, counted
once, for the record layout of include/kvb.h.  The element sizes are parameters
so that the same counter, fed the paper's assumptions (fp16 q/k/v/o and records,
2-byte gates, no grouped heads), reproduces the paper's Table 2 and the speed-up
models Eq. 6 / 17-19; tests/test_traffic_model.py checks that.
"""
from dataclasses import dataclass


@dataclass(frozen=True)
class Layout:
    dk: int = 128
    dv: int = 128
    r: int = 2            # v-heads per qk-head (q, k and buffered keys are shared by r heads)
    in_bytes: int = 2     # q, k, v and buffered k
    u_bytes: int = 4      # buffered delta value
    G_bytes: int = 4      # buffered cumulative log decay
    out_bytes: int = 4
    gate_bytes: int = 4   # g and beta, each
    state_bytes: int = 4

    @property
    def state(self):
        return self.state_bytes * self.dk * self.dv

    @property
    def token_in(self):       # q, k (shared), v, g, beta of one new token, per v-head
        return 2 * self.in_bytes * self.dk / self.r + self.in_bytes * self.dv + 2 * self.gate_bytes

    @property
    def record(self):         # one buffered record (k share, u, G), per v-head
        return self.in_bytes * self.dk / self.r + self.u_bytes * self.dv + self.G_bytes

    @property
    def token_out(self):      # output + the appended record
        return self.out_bytes * self.dv + self.record


PAPER = Layout(r=1, in_bytes=2, u_bytes=2, G_bytes=2, out_bytes=2, gate_bytes=2)
KVB = Layout()

_BYTES = {"f32": 4, "bf16": 2, "f16": 2}


def layout(in_dtype="bf16", rec_dtype="f32", out_dtype="f32", r=2, dk=128, dv=128):
    """The layout of a kvb configuration: element types as the names of include/kvb.h's type
    codes.  The gates g, beta and the buffered cumulative log decay G are fp32 in every
    configuration; layout("f16", "f16", "f16") is the paper's storage regime (Sec. 4.1) in this
    library's record format."""
    return Layout(dk=dk, dv=dv, r=r, in_bytes=_BYTES[in_dtype], u_bytes=_BYTES[rec_dtype],
                  out_bytes=_BYTES[out_dtype])


def decode_rw(lay, fill, with_state=True):
    """(read, write) bytes per v-head of one kvb_decode at pre-append fill `fill`."""
    read = (lay.state if with_state else 0) + lay.token_in + fill * lay.record
    return read, lay.token_out


def flush_rw(lay, m):
    """(read, write) bytes per v-head of one kvb_flush of m records."""
    return lay.state + m * lay.record, lay.state


def decode_flush_rw(lay, fill, threshold):
    """(read, write) per v-head of one kvb_decode_flush at pre-append fill `fill`: the decode
    step, plus the state write-back when the append reaches `threshold` (the state and the
    records are read once, by the decode part)."""
    rd, wr = decode_rw(lay, fill)
    if fill + 1 >= threshold:
        wr += lay.state
    return rd, wr


def fused_cycle_rw(lay, C):
    """Average (read, write) per token per v-head over one cycle of kvb_decode_flush."""
    rd = wr = 0.0
    for j in range(C):
        a, b = decode_flush_rw(lay, j, C)
        rd, wr = rd + a, wr + b
    return rd / C, wr / C


def recurrent_rw(lay):
    """(read, write) per v-head of the fused recurrent step (Table 2, row 'Recurrent')."""
    return lay.state + lay.token_in, lay.state + lay.out_bytes * lay.dv


def verify_rw(lay, fill, T, with_state=True):
    read = (lay.state if with_state else 0) + T * lay.token_in + fill * lay.record
    return read, T * lay.token_out


def direct_rw(lay, L):
    """kvb_direct over a context of L tokens: every input once, every output and record once."""
    return L * lay.token_in, L * lay.token_out


def chunk_cycle_rw(lay, C):
    """Average (read, write) per token per v-head over one full cycle: decode at fills
    0..C-1 plus the flush of C records (the averaging rule of the paper's Fig. 3)."""
    rd = wr = 0.0
    for j in range(C):
        a, b = decode_rw(lay, j)
        rd, wr = rd + a, wr + b
    a, b = flush_rw(lay, C)
    return (rd + a) / C, (wr + b) / C


def total(rw):
    return rw[0] + rw[1]


# The paper's closed-form models, for reference next to measured ratios.
def paper_speedup_chunkwise(d, m):
    """Eq. 6 / Eq. 17 (approximate form)."""
    return 4 * (d + 1) / (2 * d + 4 * d / m + m + 7)


def paper_speedup_verify(d, m):
    """Eq. 9 / Eq. 18 (approximate form)."""
    return ((m + 1) * d + 2 * m) / (3 * d + 4 * m)


def paper_speedup_kv_only(d, m, L):
    """Eq. 10 / Eq. 19 (approximate form)."""
    return (d + 2 * d / m + m / 2 + 3.5) / (L + 2)
