// kvb_flush_kernel and kvb_flush_mfma_kernel (the deferred state update as its own launch), kvb_compact_kernel.
#include "kvb_device.h"

namespace kvb_impl {

// ---------------------------------------------------------------------------
// kvb_flush: S <- gamma_{m-1} S + sum_{l<m} Gamma_{m-1,l} k_l^T u_l   (Eq. 16, last line)
// The rank-m sum is accumulated apart from the state so that the state tile can
// stay in flight until the very end.
// ---------------------------------------------------------------------------
template <int D, typename TIn, typename TRec, bool PAGED>
__global__ __launch_bounds__(NT) void kvb_flush_kernel(const FlushArgs a)
{
    constexpr int LPR = D / 4;
    constexpr int RPP = NT / LPR;
    constexpr int NPASS = D / RPP;
    constexpr int LT = 16;                  // records staged per LDS tile
    constexpr int EPT = LT * D / NT;        // tile elements per thread

    __shared__ __attribute__((aligned(16))) float kh[LT][D];  // Gamma_{m-1,l} k_l
    __shared__ __attribute__((aligned(16))) float uu[LT][D];
    __shared__ int sBlk[NW][MAX_BLOCKS];

    const int tid = threadIdx.x;
    const int lb = logical_block();
    const int b = lb / a.Hv;
    const int h = lb % a.Hv;
    const int hk = h / (a.Hv / a.Hk);
    const int cap = a.cap;

    const int s = a.slot[b];
    if (s < 0 || s >= a.st.n_slots)
        return;
    const int f = a.st.fill[s] & FILL_MASK;
    int acc = a.accepted ? a.accepted[b] : 0;
    if (acc < 0)
        acc = 0;
    int m = f + acc;
    if (m > cap) {
        m = cap;
        if (tid == 0 && a.st.status)
            atomicOr(&a.st.status[s], KVB_STATUS_OVERFLOW);
    }
    // (no state: a KV-only context, Sec. 3.4 -- the call then only commits accepted drafts)
    const bool do_flush = a.st.state != nullptr && m >= a.threshold && m > 0;
    if (!do_flush) {
        if (m != f && tid == 0)   // fill only moves when something was accepted
            publish_fill(&a.st.fill[s], a.Hv, m);
        return;
    }
    int ticket = 0;
    if (tid == 0)
        ticket = take_ticket(&a.st.fill[s]);
    const int rg = tid / LPR, c4 = tid % LPR;
    const size_t unit = (size_t)s * a.Hv + h;
    const Pages<PAGED> pg = make_pages<PAGED>(a.st, s, cap, sBlk[tid / 64], tid % 64, load_block_id<PAGED>(a.st, s, tid % 64));
    auto ru = [&](int l) { return pg.row(l, a.Hv, h); };
    auto rk = [&](int l) { return pg.row(l, a.Hk, hk); };
    const float *Gbuf = a.st.buf_G;
    const TIn *kb = static_cast<const TIn *>(a.st.buf_k);
    const TRec *ub = static_cast<const TRec *>(a.st.buf_u);
    const float Glast = Gbuf[ru(m - 1)];

    // first record tile, then the state tile, so the tile's loads retire first
    float kt[EPT], ut[EPT];
    auto load_tile = [&](int l0) {
#pragma unroll
        for (int x = 0; x < EPT; ++x) {
            const int idx = tid + NT * x, l = l0 + idx / D, e = idx % D;
            if (l < m) {
                kt[x] = expf(Glast - Gbuf[ru(l)]) * to_f32(kb[rk(l) * D + e]);
                ut[x] = to_f32(ub[ru(l) * D + e]);
            } else {
                kt[x] = 0.0f;
                ut[x] = 0.0f;
            }
        }
    };
    load_tile(0);
    float4 *sp = reinterpret_cast<float4 *>(a.st.state + unit * D * D);
    float4 sreg[NPASS], dS[NPASS];
#pragma unroll
    for (int p = 0; p < NPASS; ++p) {
        sreg[p] = sp[(size_t)(rg + RPP * p) * LPR + c4];
        dS[p] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    for (int l0 = 0; l0 < m; l0 += LT) {
        if (l0 > 0) {
            __syncthreads();
            load_tile(l0);
        }
#pragma unroll
        for (int x = 0; x < EPT; ++x) {
            const int idx = tid + NT * x;
            kh[idx / D][idx % D] = kt[x];
            uu[idx / D][idx % D] = ut[x];
        }
        __syncthreads();
        const int nl = min(LT, m - l0);
        for (int l = 0; l < nl; ++l) {
            const float4 u = *reinterpret_cast<const float4 *>(&uu[l][4 * c4]);
#pragma unroll
            for (int p = 0; p < NPASS; ++p)
                fma4(dS[p], kh[l][rg + RPP * p], u);
        }
    }
    const float gam = expf(Glast);
#pragma unroll
    for (int p = 0; p < NPASS; ++p) {
        float4 o;
        o.x = fmaf(gam, sreg[p].x, dS[p].x);
        o.y = fmaf(gam, sreg[p].y, dS[p].y);
        o.z = fmaf(gam, sreg[p].z, dS[p].z);
        o.w = fmaf(gam, sreg[p].w, dS[p].w);
        sp[(size_t)(rg + RPP * p) * LPR + c4] = o;
    }
    if (tid == 0)
        publish_if_last(&a.st.fill[s], ticket, a.Hv, 0);
}

// ---------------------------------------------------------------------------
// kvb_flush for 16-bit keys and d = 128, on the matrix cores.
//
// The rank-m update is the dense contraction K^T (Diag(Gamma) U), dk x m by m x dv.  The keys
// are bf16 or fp16 as stored, so they are exact operands of v_mfma_f32_16x16x32_{bf16,f16}; the
// other factor x = Gamma_l u_l is fp32 (also when u_l itself is a 16-bit record: the decay
// weight is not) and is cut into pieces of the keys' type, x = x1 + x2 (+ x3), each piece the
// leading bits of what is left, taken off by an exact subtraction, so that k * x = sum k * x_p
// holds to the last piece and the sum is accumulated in fp32 as before.  bf16 pieces carry 8
// significand bits: three of them give all 24 bits of a fp32 record; two (16 bits, 2^-17
// relative) are far below the 2^-9 rounding a bf16 record already carries.  fp16 pieces carry
// 11 bits: two give 22 bits (2^-23 relative, the rounding of fp32 itself is 2^-24); a piece
// below the fp16 range (6e-8) is dropped, an absolute error that small against delta values
// of order one.  The 16-bit instruction runs at 16 times the rate of the fp32 matrix
// instruction, so even three products come at about 5 times that rate and 10 times the rate
// of plain vector-ALU FMAs, which is what bounds the vector-ALU kernel above from 16 records on.
//
// Operand layout (lane = 16 lq + lm): A holds A[lm][8 lq + j], B holds B[8 lq + j][lm],
// j = 0..7, the result D[4 lq + v][lm], v = 0..3.  The contraction index is the record,
// 32 records per instruction.  Which state row a tile row stands for, and which column a tile
// column, is free, and chosen so that every global access is a whole row segment:
//   tile row mi of row tile rt    = state row 8 mi + rt: one 16-byte load of k_l[8 lm .. 8 lm + 7]
//                                   holds the lane's element of all 8 row tiles of record l;
//   tile column ni of column tile t = column 32 wave + 2 ni + t: u and the state are accessed
//                                   as float2, 16 lanes to a 128-byte line.
// A lane ends up with rows 32 lq .. 32 lq + 31 of its column pair.  A wave owns 32 columns of
// all rows and needs nothing from the other waves: the kernel has no barrier.
// MULTI: more than one 32-record chunk (cap > 32); the sums then stay in registers across the
// chunks, otherwise each row tile is finished and stored as soon as its six products are done.
// STREAM: the state is read with non-temporal loads AND written back with non-temporal stores,
// for a state too large to be found in the last-level cache at its next use.  Only the two
// together pay: measured at 256 MiB of state and 64 records, 138 us with either or neither,
// 107 us with both (a state that passes through the cache in one direction still turns it
// over); at 128 MiB, which the cache keeps, they cost 10 %.
// ---------------------------------------------------------------------------
template <typename TIn, typename TRec, bool MULTI, bool STREAM, bool PAGED>
// (register budgets: 3 workgroups per CU, 2 where the sums persist)
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(MULTI ? 2 : 3)))
void kvb_flush_mfma_kernel(const int32_t *slot_arg, int32_t Hv_arg, int32_t nblocks_arg, const FlushArgs a)
{
    // (the three leading arguments repeat a.slot, a.Hv and the grid size: preloaded into scalar registers
    // at wave launch, so that the load of slot[b] does not wait for the fetch of the argument block)
    constexpr int D = 128;
    constexpr int CH = 32;   // records per chunk
    // pieces of the fp32 factor (see above)
    constexpr int NP = (__is_same(TIn, bf16_t) && sizeof(TRec) == 4) ? 3 : 2;
    __shared__ int sBlk[NW][MAX_BLOCKS];

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64;   // (a scalar)
    const int lm = lane % 16, lq = lane / 16;
    const int lb = logical_block(nblocks_arg);
    const int b = lb / Hv_arg;
    const int s = slot_arg[b];
    __builtin_amdgcn_sched_barrier(0);   // nothing that needs the argument block goes above this load
    const int h = lb % Hv_arg;
    const int hk = h / (a.Hv / a.Hk);
    const int cap = a.cap;

    if (s < 0 || s >= a.st.n_slots)
        return;
    const int f = a.st.fill[s] & FILL_MASK;
    int nacc = a.accepted ? a.accepted[b] : 0;
    if (nacc < 0)
        nacc = 0;
    int m = f + nacc;
    if (m > cap) {
        m = cap;
        if (tid == 0 && a.st.status)
            atomicOr(&a.st.status[s], KVB_STATUS_OVERFLOW);
    }
    const bool do_flush = a.st.state != nullptr && m >= a.threshold && m > 0;
    if (!do_flush) {
        if (m != f && tid == 0)
            publish_fill(&a.st.fill[s], a.Hv, m);
        return;
    }
    const size_t unit = (size_t)s * a.Hv + h;
    const Pages<PAGED> pg = make_pages<PAGED>(a.st, s, cap, sBlk[wave], lane, load_block_id<PAGED>(a.st, s, lane));
    auto ru = [&](int l) { return pg.row(l, a.Hv, h); };
    auto rk = [&](int l) { return pg.row(l, a.Hk, hk); };
    const float *Gbuf = a.st.buf_G;
    const TIn *kb = static_cast<const TIn *>(a.st.buf_k);
    const TRec *ub = static_cast<const TRec *>(a.st.buf_u);
    const float Glast = Gbuf[ru(m - 1)];
    const int col2 = 32 * wave + 2 * lm;

    // records 32 c + 8 lq + j of chunk c as raw bits; an index past m is clamped to record 0
    // (finite values that meet a zero weight)
    uint4 kraw[8];
    Raw2<TRec> uraw[8];
    float Graw[8];
    auto load_chunk = [&](int c) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int l = CH * c + 8 * lq + j;
            const int lc = l < m ? l : 0;
            kraw[j] = *reinterpret_cast<const uint4 *>(kb + rk(lc) * D + 8 * lm);
            uraw[j] = load_raw2(ub + ru(lc) * D + col2);
            Graw[j] = Gbuf[ru(lc)];
        }
    };
    // first chunk, then the state tile: loads retire in issue order, and the products of the
    // first chunk run while the state is in flight
    load_chunk(0);
    __builtin_amdgcn_sched_barrier(0);
    // State row tiles in flight: a window of 4 of the 8, refilled tile by tile as the results are
    // stored (all 8 in flight measured the same and cost a workgroup per CU).
    constexpr int WIN = 4;
    float *sp = a.st.state + unit * D * D + col2;
    float2 sreg[WIN][4];
    auto issue_state = [&](int rt) {
#pragma unroll
        for (int v = 0; v < 4; ++v)
            sreg[rt % WIN][v] = load_state2<STREAM>(sp + (size_t)(32 * lq + 8 * v + rt) * D);
        __builtin_amdgcn_sched_barrier(0);   // issue in the order they are consumed
    };
#pragma unroll
    for (int rt = 0; rt < WIN; ++rt)
        issue_state(rt);
    int ticket = 0;
    if (tid == 0)
        ticket = take_ticket(&a.st.fill[s]);

    // B operands of a chunk: piece p of Gamma_l u_l[col2 + t], 8 records to a lane
    uint4 bop[2][NP];
    auto build_b = [&](int c) {
        float w[8];
        float2 uf[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            w[j] = CH * c + 8 * lq + j < m ? expf(Glast - Graw[j]) : 0.0f;
            uf[j] = unpack2r(uraw[j]);
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            float r[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                r[j] = w[j] * (t ? uf[j].y : uf[j].x);
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                // the leading significand bits of what is left; the rest is exact in fp32
                uint32_t top[8];   // the piece, in the upper half of the word
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    if constexpr (__is_same(TIn, bf16_t)) {
                        top[j] = __builtin_bit_cast(uint32_t, r[j]) & 0xFFFF0000u;
                        r[j] -= __builtin_bit_cast(float, top[j]);
                    } else {
                        const f16_t hp = from_f32<f16_t>(r[j]);
                        top[j] = (uint32_t)hp.bits << 16;
                        r[j] -= to_f32(hp);
                    }
                }
                uint4 w4;
                w4.x = (top[0] >> 16) | top[1];
                w4.y = (top[2] >> 16) | top[3];
                w4.z = (top[4] >> 16) | top[5];
                w4.w = (top[6] >> 16) | top[7];
                bop[t][p] = w4;
            }
        }
    };
    // A operand of row tile rt: element rt of each record's 8-element slice
    auto build_a = [&](int rt) {
        uint32_t d[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t w = rt / 2 == 0 ? kraw[j].x : rt / 2 == 1 ? kraw[j].y : rt / 2 == 2 ? kraw[j].z : kraw[j].w;
            d[j] = rt % 2 ? (w >> 16) : (w & 0xFFFFu);
        }
        uint4 w4;
        w4.x = d[0] | (d[1] << 16);
        w4.y = d[2] | (d[3] << 16);
        w4.z = d[4] | (d[5] << 16);
        w4.w = d[6] | (d[7] << 16);
        return w4;
    };
    auto products = [&](int rt, f32x4_t &c0, f32x4_t &c1) {
        const uint4 aop = build_a(rt);
#pragma unroll
        for (int p = NP - 1; p >= 0; --p) {   // smallest pieces first
            c0 = mfma16x32<TIn>(aop, bop[0][p], c0);
            c1 = mfma16x32<TIn>(aop, bop[1][p], c1);
        }
    };
    const float gam = expf(Glast);
    auto finish = [&](int rt, const f32x4_t &c0, const f32x4_t &c1) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float2 o;
            o.x = fmaf(gam, sreg[rt % WIN][v].x, c0[v]);
            o.y = fmaf(gam, sreg[rt % WIN][v].y, c1[v]);
            if constexpr (STREAM)
                store2_nt(sp + (size_t)(32 * lq + 8 * v + rt) * D, o.x, o.y);
            else
                *reinterpret_cast<float2 *>(sp + (size_t)(32 * lq + 8 * v + rt) * D) = o;
        }
        if (rt + WIN < 8) {
            __builtin_amdgcn_sched_barrier(0);
            issue_state(rt + WIN);
        }
    };
    if constexpr (!MULTI) {
        build_b(0);
#pragma unroll
        for (int rt = 0; rt < 8; ++rt) {
            f32x4_t c0 = {0.f, 0.f, 0.f, 0.f}, c1 = {0.f, 0.f, 0.f, 0.f};
            products(rt, c0, c1);
            finish(rt, c0, c1);
        }
    } else {
        f32x4_t acc[8][2];
#pragma unroll
        for (int rt = 0; rt < 8; ++rt)
            acc[rt][0] = acc[rt][1] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        const int nchunk = (m + CH - 1) / CH;
        for (int c = 0; c < nchunk; ++c) {
            if (c > 0)
                load_chunk(c);
            build_b(c);
#pragma unroll
            for (int rt = 0; rt < 8; ++rt)
                products(rt, acc[rt][0], acc[rt][1]);
        }
#pragma unroll
        for (int rt = 0; rt < 8; ++rt)
            finish(rt, acc[rt][0], acc[rt][1]);
    }
    if (tid == 0)
        publish_if_last(&a.st.fill[s], ticket, a.Hv, 0);
}

// ---------------------------------------------------------------------------
// kvb_compact: after kvb_verify_tree, the records of the accepted root path
// (nodes path[0] < path[1] < ...) move from positions f + path[j] to f + j, so that
// the accepted drafts are a prefix of the T new records and kvb_flush(accepted)
// commits them (Sec. 3.3, Eq. 8: the state is updated from the accepted tokens
// only).  path[j] >= j, so a move never overwrites a record that a later move reads;
// every thread carries the same element of all records, in order, so no two threads
// touch the same word.
// ---------------------------------------------------------------------------
template <int D, typename TIn, typename TRec, bool PAGED>
__global__ __launch_bounds__(NT) void kvb_compact_kernel(const CompactArgs a)
{
    __shared__ int sBlk[NW][MAX_BLOCKS];
    const int tid = threadIdx.x;
    const int b = blockIdx.x / a.Hv;
    const int h = blockIdx.x % a.Hv;
    const int r = a.Hv / a.Hk;
    const int s = a.slot[b];
    if (s < 0 || s >= a.st.n_slots)
        return;
    const int f = a.st.fill[s] & FILL_MASK;
    const int n = a.path_len[b];
    bool bad = n < 0 || n > a.T || f + a.T > a.cap;
    int prev = -1;
    for (int j = 0; j < n && !bad; ++j) {   // uniform
        const int pj = a.path[(size_t)b * a.T + j];
        bad = pj <= prev || pj >= a.T;
        prev = pj;
    }
    if (bad) {
        if (tid == 0 && a.st.status)
            atomicOr(&a.st.status[s], KVB_STATUS_BADPATH);
        return;
    }
    const Pages<PAGED> pg = make_pages<PAGED>(a.st, s, a.cap, sBlk[tid / 64], tid % 64, load_block_id<PAGED>(a.st, s, tid % 64));
    auto ru = [&](int l) { return pg.row(l, a.Hv, h); };
    auto rk = [&](int l) { return pg.row(l, a.Hk, h / r); };
    TRec *ub = static_cast<TRec *>(a.st.buf_u);
    float *Gb = a.st.buf_G;
    TIn *kb = static_cast<TIn *>(a.st.buf_k);
    for (int j = 0; j < n; ++j) {
        const int src = f + a.path[(size_t)b * a.T + j], dst = f + j;
        if (src == dst)
            continue;
        for (int e = tid; e < D; e += NT)
            ub[ru(dst) * D + e] = ub[ru(src) * D + e];
        if (h % r == 0)
            for (int e = tid; e < D; e += NT)
                kb[rk(dst) * D + e] = kb[rk(src) * D + e];
        if (tid == 0)
            Gb[ru(dst)] = Gb[ru(src)];
    }
}

// ---------------------------------------------------------------------------
// launch
// ---------------------------------------------------------------------------
int launch_flush(int dk, int in_dtype, int rec_dtype, const FlushArgs &a, int blocks, hipStream_t stream)
{
    if (dk == 128 && in_dtype != KVB_F32)   // the matrix-core kernel
        return dispatch_types16(in_dtype, rec_dtype, [&]<typename TIn, typename TRec>() {
            if (a.cap <= 32) {
                if (a.stream)
                    LAUNCH_LEAD(blocks, stream, a, kvb_flush_mfma_kernel<TIn, TRec, false, true);
                else
                    LAUNCH_LEAD(blocks, stream, a, kvb_flush_mfma_kernel<TIn, TRec, false, false);
            } else {
                if (a.stream)
                    LAUNCH_LEAD(blocks, stream, a, kvb_flush_mfma_kernel<TIn, TRec, true, true);
                else
                    LAUNCH_LEAD(blocks, stream, a, kvb_flush_mfma_kernel<TIn, TRec, true, false);
            }
        });
    return dispatch(dk, in_dtype, rec_dtype, [&]<int D, typename TIn, typename TRec>() {
        if constexpr (!(D == 128 && sizeof(TIn) == 2))
            LAUNCH_PAGED(blocks, stream, a, kvb_flush_kernel<D, TIn, TRec);
    });
}

int launch_compact(int dk, int in_dtype, int rec_dtype, const CompactArgs &a, int blocks, hipStream_t stream)
{
    return dispatch(dk, in_dtype, rec_dtype,
                    [&]<int D, typename TIn, typename TRec>() { LAUNCH_PAGED(blocks, stream, a, kvb_compact_kernel<D, TIn, TRec); });
}

}  // namespace kvb_impl
