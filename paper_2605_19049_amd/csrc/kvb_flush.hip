// kvb_flush_kernel (the deferred state update as its own launch) and kvb_compact_kernel.
#include "kvb_device.h"

namespace kvb_impl {

// ---------------------------------------------------------------------------
// kvb_flush: S <- gamma_{m-1} S + sum_{l<m} Gamma_{m-1,l} k_l^T u_l   (Eq. 16, last line)
// The rank-m sum is accumulated apart from the state so that the state tile can
// stay in flight until the very end.
// ---------------------------------------------------------------------------
template <int D, typename TIn, bool PAGED>
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
    const float *ub = a.st.buf_u;
    const float Glast = Gbuf[ru(m - 1)];

    // first record tile, then the state tile, so the tile's loads retire first
    float kt[EPT], ut[EPT];
    auto load_tile = [&](int l0) {
#pragma unroll
        for (int x = 0; x < EPT; ++x) {
            const int idx = tid + NT * x, l = l0 + idx / D, e = idx % D;
            if (l < m) {
                kt[x] = expf(Glast - Gbuf[ru(l)]) * to_f32(kb[rk(l) * D + e]);
                ut[x] = ub[ru(l) * D + e];
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
// kvb_compact: after kvb_verify_tree, the records of the accepted root path
// (nodes path[0] < path[1] < ...) move from positions f + path[j] to f + j, so that
// the accepted drafts are a prefix of the T new records and kvb_flush(accepted)
// commits them (Sec. 3.3, Eq. 8: the state is updated from the accepted tokens
// only).  path[j] >= j, so a move never overwrites a record that a later move reads;
// every thread carries the same element of all records, in order, so no two threads
// touch the same word.
// ---------------------------------------------------------------------------
template <int D, typename TIn, bool PAGED>
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
    float *ub = a.st.buf_u;
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
int launch_flush(int dk, int in_dtype, const FlushArgs &a, int blocks, hipStream_t stream)
{
    return dispatch(dk, in_dtype, [&]<int D, typename TIn>() { LAUNCH_PAGED(blocks, stream, a, kvb_flush_kernel<D, TIn); });
}

int launch_compact(int dk, int in_dtype, const CompactArgs &a, int blocks, hipStream_t stream)
{
    return dispatch(dk, in_dtype, [&]<int D, typename TIn>() { LAUNCH_PAGED(blocks, stream, a, kvb_compact_kernel<D, TIn); });
}

}  // namespace kvb_impl
