// kvb -- KVBuffer-style Gated DeltaNet decoding, HIP kernels for gfx950 and the
// C-ABI entry points declared in include/kvb.h.
//
// Work decomposition (every kernel): one 256-thread workgroup per (request b,
// v-head h); the committed state S0[dk][dv] (fp32, dv contiguous, 64 KB at
// d = 128) is streamed exactly once per call.  Besides the state a unit needs
// its buffered keys k_l, delta values u_l and cumulative log decays G_l (paper
// App. A.1, the paragraph after Eq. 16), a few KB.
//   kvb_step_kernel         decode (T = 1) and generic verify: vector ALUs; a thread owns
//                           4 adjacent dv columns of 16 state rows (16-byte loads)
//   kvb_verify_mfma_kernel  verify, bf16 / d = 128: matrix cores; a wave owns 32 dv columns
//   kvb_flush_kernel        deferred state update as its own launch
//   kvb_direct_mfma_kernel  short contexts, bf16 / d = 128: matrix cores throughout
//   kvb_direct_kernel       short contexts, other types and head sizes
//
// Notation follows App. A.1: gamma_i = exp(G_i), Gamma_il = exp(G_i - G_l).

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "kvb.h"

struct kvb_timer {
    hipEvent_t start, stop;
};

namespace {

constexpr int NT = 256;      // threads per workgroup
constexpr int NW = NT / 64;  // wavefronts per workgroup
constexpr int FILL_MASK = 0xFFFF;
constexpr int TICKET_ONE = 1 << 16;

struct bf16_t {
    uint16_t bits;
};

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return __uint_as_float((uint32_t)x.bits << 16); }

// 8 consecutive elements starting at p (p is 16-byte aligned for bf16, 32 for fp32).
__device__ __forceinline__ void load8(const float *p, float (&o)[8])
{
    const float4 a = *reinterpret_cast<const float4 *>(p);
    const float4 b = *reinterpret_cast<const float4 *>(p + 4);
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
    o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t *p, float (&o)[8])
{
    const uint4 w = *reinterpret_cast<const uint4 *>(p);
    o[0] = __uint_as_float(w.x << 16); o[1] = __uint_as_float(w.x & 0xFFFF0000u);
    o[2] = __uint_as_float(w.y << 16); o[3] = __uint_as_float(w.y & 0xFFFF0000u);
    o[4] = __uint_as_float(w.z << 16); o[5] = __uint_as_float(w.z & 0xFFFF0000u);
    o[6] = __uint_as_float(w.w << 16); o[7] = __uint_as_float(w.w & 0xFFFF0000u);
}

// The same 8 elements as untouched bits: issuing a load and converting its result are
// kept apart so that no wait lands between two loads.
template <typename T>
struct Raw8;
template <>
struct Raw8<float> {
    float4 a, b;
};
template <>
struct Raw8<bf16_t> {
    uint4 w;
};
__device__ __forceinline__ Raw8<float> load_raw8(const float *p)
{
    return Raw8<float>{*reinterpret_cast<const float4 *>(p), *reinterpret_cast<const float4 *>(p + 4)};
}
__device__ __forceinline__ Raw8<bf16_t> load_raw8(const bf16_t *p)
{
    return Raw8<bf16_t>{*reinterpret_cast<const uint4 *>(p)};
}
__device__ __forceinline__ void unpack8(const Raw8<float> &r, float (&o)[8])
{
    o[0] = r.a.x; o[1] = r.a.y; o[2] = r.a.z; o[3] = r.a.w;
    o[4] = r.b.x; o[5] = r.b.y; o[6] = r.b.z; o[7] = r.b.w;
}
__device__ __forceinline__ void unpack8(const Raw8<bf16_t> &r, float (&o)[8])
{
    o[0] = __uint_as_float(r.w.x << 16); o[1] = __uint_as_float(r.w.x & 0xFFFF0000u);
    o[2] = __uint_as_float(r.w.y << 16); o[3] = __uint_as_float(r.w.y & 0xFFFF0000u);
    o[4] = __uint_as_float(r.w.z << 16); o[5] = __uint_as_float(r.w.z & 0xFFFF0000u);
    o[6] = __uint_as_float(r.w.w << 16); o[7] = __uint_as_float(r.w.w & 0xFFFF0000u);
}

// One 16-byte piece of the state tile.  STREAM: non-temporal load, for a state that will
// not be read again before the last-level cache has turned over (measured on MI355X:
// +14% at 1 GiB of state per call, -5% at 128 MiB, which the 256 MB cache keeps).
template <bool STREAM>
__device__ __forceinline__ float4 load_state4(const float4 *p)
{
    if constexpr (STREAM) {
        typedef float v4f __attribute__((ext_vector_type(4)));
        const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(p));
        return make_float4(t.x, t.y, t.z, t.w);
    } else {
        return *p;
    }
}

__device__ __forceinline__ void fma4(float4 &acc, float c, const float4 &x)
{
    acc.x = fmaf(c, x.x, acc.x);
    acc.y = fmaf(c, x.y, acc.y);
    acc.z = fmaf(c, x.z, acc.z);
    acc.w = fmaf(c, x.w, acc.w);
}

// The workgroups of one request share fill[slot].  Each reads it (low 16 bits)
// when it starts and takes a ticket (bits 16..) when it has finished; the
// workgroup holding the last ticket knows every other one has read the word and
// stores the new plain value.  Relaxed ordering is enough and matters: a
// workgroup's read of the word has long completed when it takes its ticket
// (its value fed address computations), the store depends on the ticket's
// return value, and nothing else is communicated through the word.  Acquire /
// release ordering at device scope would make every workgroup write back and
// invalidate its L2, which costs more than the kernel's whole memory traffic.
//
// The ticket is taken once the workgroup's loads are in flight (take_ticket), so that its
// round trip overlaps the streaming, and is looked at only at the very end.
__device__ __forceinline__ int take_ticket(int32_t *word)
{
    return __hip_atomic_fetch_add(word, TICKET_ONE, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void publish_if_last(int32_t *word, int ticket, int nwg, int new_fill)
{
    // Opaque to the optimiser: otherwise the shift below is hoisted next to the atomic and
    // the wave waits there for the ticket (and for every load it issued before it).
    asm volatile("" : "+v"(ticket));
    if ((ticket >> 16) == nwg - 1)
        __hip_atomic_store(word, new_fill, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void publish_fill(int32_t *word, int nwg, int new_fill)
{
    publish_if_last(word, take_ticket(word), nwg, new_fill);
}

__device__ __forceinline__ void store_raw8(float *p, const Raw8<float> &r)
{
    *reinterpret_cast<float4 *>(p) = r.a;
    *reinterpret_cast<float4 *>(p + 4) = r.b;
}
__device__ __forceinline__ void store_raw8(bf16_t *p, const Raw8<bf16_t> &r)
{
    *reinterpret_cast<uint4 *>(p) = r.w;
}

// Workgroup ids are dealt round-robin to the 8 XCDs (each with its own L2).  Map them so
// that XCD x works on one contiguous eighth of the (request, head) units: all heads of a
// request then share an L2, which keeps the per-request ticket atomics and the keys that
// grouped heads share inside one XCD.
__device__ __forceinline__ int logical_block()
{
    const int n = gridDim.x, x = blockIdx.x;
    return (n % 8 == 0) ? (x % 8) * (n / 8) + x / 8 : x;
}

struct Store {
    float *state;
    void *buf_k;
    float *buf_u;
    float *buf_G;
    int32_t *fill;
    int32_t *status;
    int32_t n_slots;
    // Paged record buffers (Sec. 3.1: blocks of 8 or 16 records from a pool shared by all requests).
    // block_table == nullptr: slot s owns the records s*cap .. s*cap+cap-1 of each head, as one block.
    const int32_t *block_table;   // [n_slots, max_blocks] block ids
    int32_t block_size;           // records per block, a power of two (cap when not paged)
    int32_t max_blocks;           // row length of block_table (1 when not paged)
    int32_t n_blocks;             // blocks in the pools; ids are clamped into 0..n_blocks-1
};

// Where record l of the request lives.  The record arrays are [blocks, heads, block_size, ...]:
// a head's records inside a block are contiguous.  Without a block table the block is the slot
// and block_size is cap, which is the contiguous layout.  Each wave keeps its own copy of the
// request's block-table row in LDS (written and read by the same wave, so no barrier), filled
// from one small vector load that is issued before the state loads and therefore never waits
// for them.
constexpr int MAX_BLOCKS = KVB_MAX_BLOCKS;   // cap <= 128, block_size >= 8
// PAGED is a compile-time switch of every kernel: the contiguous layout then costs nothing
// (measured: a run-time flag cost the decode step 2 %; and a dummy load from fill[s] in its
// place doubled the step time, every wave's first load queueing behind the ticket atomics
// that the other heads of the request issue on that word).
template <bool PAGED>
struct Pages {
    const int *tab;   // this wave's LDS copy of the row
    int s, bs, lg;
    __device__ __forceinline__ int blk(int l) const
    {
        if constexpr (PAGED)
            return tab[l >> lg];
        else
            return s;
    }
    __device__ __forceinline__ int off(int l) const { return PAGED ? (l & (bs - 1)) : l; }
    // row of record l of head `head` (H heads per block) in units of one record
    __device__ __forceinline__ size_t row(int l, int H, int head) const
    {
        return ((size_t)blk(l) * H + head) * bs + off(l);
    }
};
// The lane's entry of the block-table row (lanes >= max_blocks repeat the last entry).
template <bool PAGED>
__device__ __forceinline__ int load_block_id(const Store &st, int s, int lane)
{
    if constexpr (PAGED)
        return st.block_table[(size_t)s * st.max_blocks + min(lane, st.max_blocks - 1)];
    else
        return 0;
}
template <bool PAGED>
__device__ __forceinline__ Pages<PAGED> make_pages(const Store &st, int s, int cap, int *tab, int lane, int id)
{
    Pages<PAGED> pg;
    pg.tab = tab;
    pg.s = s;
    if constexpr (PAGED) {
        if (lane < MAX_BLOCKS)
            tab[lane] = min(max(id, 0), st.n_blocks - 1);
        pg.bs = st.block_size;
        pg.lg = 31 - __builtin_clz(st.block_size);
    } else {
        pg.bs = cap;
        pg.lg = 0;
    }
    return pg;
}

struct StepArgs {
    Store st;
    const int32_t *slot;
    const void *q, *k, *v;
    const float *g, *beta;
    float *out;
    int32_t Hk, Hv, cap, T;
    float scale;
    int32_t advance;    // 1: decode (fill += T after the step); 0: verify (fill untouched)
    int32_t threshold;  // fused decode + flush only: fold the buffer into the state once it holds this many
    int32_t stream_state;  // non-temporal state loads
    // kvb_verify_tree: parent[b][i] in {-1, 0..i-1} of draft i.  When `tree` is 0 the drafts are
    // a chain and `parent` points at some other readable array of at least B*T words (its
    // values are ignored), so that the kernels can load it without a branch.
    const int32_t *parent;
    int32_t tree;
};

// ---------------------------------------------------------------------------
// kvb_decode (TM == 1) and kvb_verify (TM >= T): rows f..f+T-1 of the chunkwise
// form, Eq. 15/16.  Per (b,h):
//   accU_i = -gamma_i k_i S0 - sum_{l<f} Gamma_il (k_i.k_l) u_l
//   accO_i =  gamma_i q_i S0 + sum_{l<f} Gamma_il (q_i.k_l) u_l
// are accumulated over state rows and buffered records alike (both are "rows"
// weighted by a per-row scalar), reduced across the workgroup, and the T new
// rows are then finished by forward substitution among themselves.
//
// Load order is the point of this kernel.  The memory counter retires loads
// in issue order, so the few small loads whose values are needed first (new
// q/k rows, the buffered records of a WREC-record window, v) are issued
// before the 64 KB state tile; the dot products and the LDS exchange then run
// while the state is still in flight.
// ---------------------------------------------------------------------------
template <int N>
__device__ __forceinline__ float group_sum(float x)
{
#pragma unroll
    for (int off = 1; off < N; off <<= 1)
        x += __shfl_xor(x, off);
    return x;
}

//
// FUSE (decode only): when the append brings the buffer to `threshold` records the same
// workgroup applies the deferred update S <- gamma_f S0 + sum_{l<=f} Gamma_fl k_l^T u_l to
// the state tile it already holds in registers and writes it back, which saves the second
// kernel's re-read of the state.
template <int D, typename TIn, int TM, int WREC, bool HAS_STATE, bool FUSE, bool STREAM, bool PAGED>
__global__ __launch_bounds__(NT) void kvb_step_kernel(const StepArgs a)
{
    constexpr int LPR = D / 4;       // lanes covering one state row with float4
    constexpr int RPP = NT / LPR;    // rows covered by the workgroup per pass
    constexpr int NPASS = D / RPP;   // state rows per thread
    constexpr int GL = D / 8;        // lanes sharing one key dot product (8 elements each)
    constexpr int NG = NT / GL;      // records handled per pass of the dot-product phase
    constexpr int KP = (WREC + NG - 1) / NG;    // key passes held in registers
    constexpr int UP = (WREC + RPP - 1) / RPP;  // delta-value passes held in registers
    constexpr int NC = KVB_MAX_CAP + TM;
    // the two smaller window tiers are only launched when the whole buffer fits the window
    constexpr bool TAIL = WREC >= 64;
    constexpr int LT = 16;                 // records per LDS tile of the fused state update
    constexpr int EPT = LT * D / NT;
    // state loads issued before the fill is known (the 64-record window keeps the records first:
    // holding it across the state pass costs a workgroup per CU)
    constexpr bool EARLY = TM == 1 && HAS_STATE && WREC <= 32;
    static_assert(!FUSE || (TM == 1 && HAS_STATE), "the fused update belongs to kvb_decode with a state");

    __shared__ __attribute__((aligned(16))) float sKs[TM][D];  // -gamma_i k_i (state-row weights for accU)
    __shared__ __attribute__((aligned(16))) float sQs[TM][D];  //  gamma_i q_i
    __shared__ __attribute__((aligned(16))) float rK[TM][D];   // raw new rows
    __shared__ __attribute__((aligned(16))) float rQ[TM][D];
    __shared__ float cK[TM][NC];     // Gamma_il (k_i.k_l), 0 for l >= f+i
    __shared__ float cQ[TM][NC];     // Gamma_il (q_i.k_l), 0 for l >  f+i
    __shared__ __attribute__((aligned(16))) float red[NW][TM][2][D];
    __shared__ __attribute__((aligned(16))) float kh[FUSE ? LT : 1][D];  // Gamma_fl k_l tile
    __shared__ int sBlk[NW][MAX_BLOCKS];
    __shared__ __attribute__((aligned(16))) float uu[FUSE ? LT : 1][D];  // u_l tile

    const int tid = threadIdx.x;
    const int lb = logical_block();
    const int b = lb / a.Hv;
    const int h = lb % a.Hv;
    const int r = a.Hv / a.Hk;
    const int hk = h / r;
    const int T = TM == 1 ? 1 : a.T;
    const int cap = a.cap;

    const int s = a.slot[b];
    if (s < 0 || s >= a.st.n_slots)
        return;

    const int rg = tid / LPR, c4 = tid % LPR;
    const int grp = tid / GL, sub = tid % GL;
    const size_t unit = (size_t)s * a.Hv + h;
    const TIn *qin = static_cast<const TIn *>(a.q);
    const TIn *kin = static_cast<const TIn *>(a.k);
    const TIn *vin = static_cast<const TIn *>(a.v);
    const float *Gbuf = a.st.buf_G;                              // record l of this head: Gbuf[ru(l)]
    const TIn *kb = static_cast<const TIn *>(a.st.buf_k);        //                        kb + rk(l) * D
    const float4 *up = reinterpret_cast<const float4 *>(a.st.buf_u);   //                  up + ru(l) * LPR
    const int blk_id = load_block_id<PAGED>(a.st, s, tid % 64);

    // ---- 1. loads that need only the request index --------------------------
    // All vector loads of this kernel are issued as raw bits from always-valid addresses (an
    // index past the fill is clamped to record 0 and its value ignored), with no branch and
    // no conversion in between, so nothing waits before the state tile is in flight.
    // new rows: each thread's 8-element slice of q_i, k_i (TM > 1: thread idx -> row idx / (D/8))
    const int nr_i = TM == 1 ? 0 : min(tid / (D / 8), T - 1);
    const int nr_e = TM == 1 ? sub : tid % (D / 8);
    const size_t nr_o = (((size_t)b * T + nr_i) * a.Hk + hk) * D + 8 * nr_e;
    const Raw8<TIn> q_raw = load_raw8(qin + nr_o);
    const Raw8<TIn> k_raw = load_raw8(kin + nr_o);
    TIn v_raw[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
        v_raw[i] = vin[(((size_t)b * T + min(i, T - 1)) * a.Hv + h) * D + tid % D];

    // ---- 2. the state tile goes in flight ------------------------------------
    // Decoding one token (EARLY): the state's address needs the slot only, so its loads go out
    // before the fill count is known.  Each dependent scalar load costs microseconds while the
    // chip is streaming, and this takes one of them off the path to the first state byte.  The
    // buffered records, whose addresses do need the fill, follow the state and are consumed
    // after it.  The multi-row variants keep the records ahead of the state, since their
    // dot-product phase is long enough to be worth hiding under the state's flight.
    // (scheduling fences: the instruction scheduler must not reorder loads across them; the
    // memory counter retires loads in issue order)
    float4 sreg[NPASS];
    auto issue_state = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        const float4 *sp = reinterpret_cast<const float4 *>(a.st.state + unit * D * D);
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            sreg[p] = load_state4<STREAM>(sp + (size_t)(rg + RPP * p) * LPR + c4);
            __builtin_amdgcn_sched_barrier(0);   // issue in the order they are consumed
        }
    };
    if constexpr (EARLY)
        issue_state();

    // per-row scalars (uniform); requested together with the fill, after the state loads,
    // so that no scalar wait stands between the slot and the first state byte
    float gnew[TM], bet[TM];
    int par[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const size_t o = ((size_t)b * T + min(i, T - 1)) * a.Hv + h;
        gnew[i] = i < T ? a.g[o] : 0.0f;
        bet[i] = i < T ? a.beta[o] : 0.0f;
        par[i] = i - 1;
        if constexpr (TM > 1) {
            const int pl = a.parent[(size_t)b * T + min(i, T - 1)];
            par[i] = a.tree ? pl : i - 1;
        }
    }
    const int f = a.st.fill[s] & FILL_MASK;
    if (f + T > cap) {
        if (tid == 0) {
            if (a.st.status)
                atomicOr(&a.st.status[s], KVB_STATUS_OVERFLOW);
            if (a.advance)
                publish_fill(&a.st.fill[s], a.Hv, f);
        }
        return;
    }
    const Pages<PAGED> pg = make_pages<PAGED>(a.st, s, cap, sBlk[tid / 64], tid % 64, blk_id);
    auto ru = [&](int l) { return pg.row(l, a.Hv, h); };    // row of record l in buf_u / buf_G
    auto rk = [&](int l) { return pg.row(l, a.Hk, hk); };   // row of record l in buf_k
    // cumulative log decay of the new rows (uniform)
    // Gc[i]: cumulative log decay of new row i along its own root path (a chain unless the
    // drafts form a tree); anc[i]: bit j set iff new row j is a strict ancestor of row i.
    // A parent index that does not precede its child is taken as -1 and flagged.
    float Gc[TM];
    int anc[TM];
    float G_prev = f > 0 ? Gbuf[ru(f - 1)] : 0.0f;
    auto finish_Gc = [&]() {
        bool bad = false;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            float base = G_prev;
            int am = 0;
            bad = bad || (i < T && (par[i] < -1 || par[i] >= i));
#pragma unroll
            for (int j = 0; j < i; ++j) {
                const bool is_parent = par[i] == j;
                base = is_parent ? Gc[j] : base;
                am = is_parent ? (anc[j] | (1 << j)) : am;
            }
            Gc[i] = base + gnew[i];
            anc[i] = am;
        }
        if (TM > 1 && bad && tid == 0 && a.st.status)
            atomicOr(&a.st.status[s], KVB_STATUS_BADPATH);
    };
    if constexpr (!EARLY)
        finish_Gc();
    // window of buffered records
    Raw8<TIn> kl_raw[KP];
    float Gl[KP];
#pragma unroll
    for (int p = 0; p < KP; ++p) {
        const int l = grp + NG * p;
        const int lc = l < f ? l : 0;
        kl_raw[p] = load_raw8(kb + rk(lc) * D + 8 * sub);
        Gl[p] = Gbuf[ru(lc)];
    }
    float4 ur[UP];
#pragma unroll
    for (int j = 0; j < UP; ++j) {
        const int l = rg + RPP * j;
        ur[j] = up[ru(l < f ? l : 0) * LPR + c4];
    }
    if constexpr (HAS_STATE && !EARLY)
        issue_state();
    __builtin_amdgcn_sched_barrier(0);
    // youngest memory operation of the wave: nothing waits for it before the very end
    int ticket = 0;
    if (a.advance && tid == 0)
        ticket = take_ticket(&a.st.fill[s]);

    // ---- 3. decayed dot products of the new rows with every earlier key ----
    float q8[8], k8[8];
    unpack8(q_raw, q8);
    unpack8(k_raw, k8);
    float4 accU[TM], accO[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        accU[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        accO[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if constexpr (TM == 1) {
        // EARLY applies gamma after the sum over state rows (Gc comes back behind the state)
        const float gw = EARLY ? 1.0f : expf(Gc[0]);
        if (grp == 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                sKs[0][8 * sub + e] = -gw * k8[e];
                sQs[0][8 * sub + e] = gw * q8[e];
            }
        }
        float dqk = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            dqk = fmaf(q8[e], k8[e], dqk);
        dqk = group_sum<GL>(dqk);
        if (tid == 0) {
            cK[0][f] = 0.0f;
            cQ[0][f] = dqk;
        }
        if constexpr (EARLY) {
            // the state rows are consumed first, in the order they were issued; the records
            // (younger loads) are not touched before the last state row has been used
            __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int p = 0; p < NPASS; ++p) {
                const int row = rg + RPP * p;
                fma4(accU[0], sKs[0][row], sreg[p]);
                fma4(accO[0], sQs[0][row], sreg[p]);
            }
            // pins the sums (and everything derived from G_prev, a load younger than the
            // state) to this point: pure arithmetic is otherwise free to drift across the fences
            asm volatile("" : "+v"(accU[0].x), "+v"(accU[0].y), "+v"(accU[0].z), "+v"(accU[0].w),
                              "+v"(accO[0].x), "+v"(accO[0].y), "+v"(accO[0].z), "+v"(accO[0].w),
                              "+v"(G_prev));
            __builtin_amdgcn_sched_barrier(0);
            finish_Gc();
            const float gam = expf(Gc[0]);
            accU[0].x *= gam; accU[0].y *= gam; accU[0].z *= gam; accU[0].w *= gam;
            accO[0].x *= gam; accO[0].y *= gam; accO[0].z *= gam; accO[0].w *= gam;
        }
#pragma unroll
        for (int p = 0; p < KP; ++p) {
            const int l = grp + NG * p;
            float kx[8];
            unpack8(kl_raw[p], kx);
            float dkk = 0.0f, dq = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                dkk = fmaf(kx[e], k8[e], dkk);
                dq = fmaf(kx[e], q8[e], dq);
            }
            dkk = group_sum<GL>(dkk);
            dq = group_sum<GL>(dq);
            if (sub == 0 && l < f) {
                const float w = expf(Gc[0] - Gl[p]);
                cK[0][l] = w * dkk;
                cQ[0][l] = w * dq;
            }
        }
        for (int l = KP * NG + grp; TAIL && l < f; l += NG) {   // records beyond the register window
            float kx[8];
            load8(kb + rk(l) * D + 8 * sub, kx);
            float dkk = 0.0f, dq = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                dkk = fmaf(kx[e], k8[e], dkk);
                dq = fmaf(kx[e], q8[e], dq);
            }
            dkk = group_sum<GL>(dkk);
            dq = group_sum<GL>(dq);
            if (sub == 0) {
                const float w = expf(Gc[0] - Gbuf[ru(l)]);
                cK[0][l] = w * dkk;
                cQ[0][l] = w * dq;
            }
        }
    } else {
        if (tid < T * (D / 8)) {
            float gam = 0.0f;
#pragma unroll
            for (int j = 0; j < TM; ++j)
                if (j == nr_i)
                    gam = expf(Gc[j]);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                rK[nr_i][8 * nr_e + e] = k8[e];
                rQ[nr_i][8 * nr_e + e] = q8[e];
                sKs[nr_i][8 * nr_e + e] = -gam * k8[e];
                sQs[nr_i][8 * nr_e + e] = gam * q8[e];
            }
        }
        __syncthreads();   // rK, rQ visible
        // buffered records, all T new rows at once
        auto rows_vs_record = [&](const float(&kx)[8], float Gx, int l) {
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if (i < T) {
                    float dkk = 0.0f, dq = 0.0f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        dkk = fmaf(kx[e], rK[i][8 * sub + e], dkk);
                        dq = fmaf(kx[e], rQ[i][8 * sub + e], dq);
                    }
                    dkk = group_sum<GL>(dkk);
                    dq = group_sum<GL>(dq);
                    if (sub == 0 && l < f) {
                        const float w = expf(Gc[i] - Gx);
                        cK[i][l] = w * dkk;
                        cQ[i][l] = w * dq;
                    }
                }
            }
        };
#pragma unroll
        for (int p = 0; p < KP; ++p) {
            float kx[8];
            unpack8(kl_raw[p], kx);
            rows_vs_record(kx, Gl[p], grp + NG * p);
        }
        for (int l0 = KP * NG; TAIL && l0 < f; l0 += NG) {
            const int l = l0 + grp;
            float kx[8];
            float Gx = 0.0f;
            if (l < f) {
                load8(kb + rk(l) * D + 8 * sub, kx);
                Gx = Gbuf[ru(l)];
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    kx[e] = 0.0f;
            }
            rows_vs_record(kx, Gx, l);
        }
        // new rows against each other: pair (i, j <= i) -> columns f+j of row i
        for (int pr = grp; pr < T * T; pr += NG) {
            const int i = pr / T, j = pr % T;
            float dkk = 0.0f, dq = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float kj = rK[j][8 * sub + e];
                dkk = fmaf(kj, rK[i][8 * sub + e], dkk);
                dq = fmaf(kj, rQ[i][8 * sub + e], dq);
            }
            dkk = group_sum<GL>(dkk);
            dq = group_sum<GL>(dq);
            if (sub == 0) {
                float Gi = 0.0f, Gj = 0.0f;
                int ai = 0;
#pragma unroll
                for (int x = 0; x < TM; ++x) {
                    if (x == i) { Gi = Gc[x]; ai = anc[x]; }
                    if (x == j) Gj = Gc[x];
                }
                const bool above = (ai >> j) & 1;   // row j is a strict ancestor of row i
                const float w = (above || j == i) ? expf(Gi - Gj) : 0.0f;
                cK[i][f + j] = above ? w * dkk : 0.0f;
                cQ[i][f + j] = w * dq;
            }
        }
    }
    __syncthreads();

    // ---- 4. accumulate over buffered records and state rows ----------------
#pragma unroll
    for (int j = 0; j < UP; ++j) {
        const int l = rg + RPP * j;
        if (l < f) {
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if (i < T) {
                    fma4(accU[i], -cK[i][l], ur[j]);
                    fma4(accO[i], cQ[i][l], ur[j]);
                }
            }
        }
    }
    for (int l = UP * RPP + rg; TAIL && l < f; l += RPP) {
        const float4 u = up[ru(l) * LPR + c4];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if (i < T) {
                fma4(accU[i], -cK[i][l], u);
                fma4(accO[i], cQ[i][l], u);
            }
        }
    }
    if constexpr (HAS_STATE && !EARLY) {
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            const int row = rg + RPP * p;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if (i < T) {
                    fma4(accU[i], sKs[i][row], sreg[p]);
                    fma4(accO[i], sQs[i][row], sreg[p]);
                }
            }
        }
    }

    // ---- 5. reduce over the row groups: shuffles inside the wave, LDS across waves
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        if (i < T) {
#pragma unroll
            for (int off = LPR; off < 64; off <<= 1) {
                accU[i].x += __shfl_xor(accU[i].x, off);
                accU[i].y += __shfl_xor(accU[i].y, off);
                accU[i].z += __shfl_xor(accU[i].z, off);
                accU[i].w += __shfl_xor(accU[i].w, off);
                accO[i].x += __shfl_xor(accO[i].x, off);
                accO[i].y += __shfl_xor(accO[i].y, off);
                accO[i].z += __shfl_xor(accO[i].z, off);
                accO[i].w += __shfl_xor(accO[i].w, off);
            }
        }
    }
    {
        const int wave = tid / 64, lane = tid % 64;
        if (lane < LPR) {
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if (i < T) {
                    *reinterpret_cast<float4 *>(&red[wave][i][0][4 * lane]) = accU[i];
                    *reinterpret_cast<float4 *>(&red[wave][i][1][4 * lane]) = accO[i];
                }
            }
        }
    }
    __syncthreads();

    // ---- 6. finish the T new rows (forward substitution), write results -----
    float u_new = 0.0f;
    if (tid < D) {
        float uprev[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if (i < T) {
                float au = 0.0f, ao = 0.0f;
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    au += red[w][i][0][tid];
                    ao += red[w][i][1][tid];
                }
                const size_t row = ((size_t)b * T + i) * a.Hv + h;
                float acc = to_f32(v_raw[i]) + au;
#pragma unroll
                for (int j = 0; j < TM; ++j)
                    if (j < i)
                        acc = fmaf(-cK[i][f + j], uprev[j], acc);
                const float ui = bet[i] * acc;
#pragma unroll
                for (int j = 0; j < TM; ++j)
                    if (j < i)
                        ao = fmaf(cQ[i][f + j], uprev[j], ao);
                ao = fmaf(cQ[i][f + i], ui, ao);
                uprev[i] = ui;
                u_new = ui;
                a.out[row * D + tid] = a.scale * ao;
                a.st.buf_u[ru(f + i) * D + tid] = ui;
            }
        }
    }
    if (tid < T) {
        float gv = 0.0f;
#pragma unroll
        for (int j = 0; j < TM; ++j)
            if (j == tid)
                gv = Gc[j];
        a.st.buf_G[ru(f + tid)] = gv;
    }
    if (h % r == 0 && tid < T * (D / 8)) {   // the threads that loaded the new k rows store them
        TIn *kw = static_cast<TIn *>(a.st.buf_k) + rk(f + nr_i) * D;
        store_raw8(kw + 8 * nr_e, k_raw);
    }
    int new_fill = f + T;
    if constexpr (FUSE) {
        const int m = f + 1;
        if (m >= a.threshold) {   // uniform over the workgroup (and over the request)
            const float gam = expf(Gc[0]);
#pragma unroll
            for (int p = 0; p < NPASS; ++p) {
                sreg[p].x *= gam; sreg[p].y *= gam; sreg[p].z *= gam; sreg[p].w *= gam;
            }
            const float *ub = a.st.buf_u;
            // one LDS tile of LT records: record f itself comes from this workgroup's registers
            auto inject_new = [&](int l0) {
                if (f >= l0 && f < l0 + LT) {
                    if (grp == 0) {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            kh[f - l0][8 * sub + e] = k8[e];
                    }
                    if (tid < D)
                        uu[f - l0][tid] = u_new;
                }
            };
            auto apply_tile = [&](int l0) {
                const int nl = min(LT, m - l0);
                for (int l = 0; l < nl; ++l) {
                    const float4 u = *reinterpret_cast<const float4 *>(&uu[l][4 * c4]);
#pragma unroll
                    for (int p = 0; p < NPASS; ++p)
                        fma4(sreg[p], kh[l][rg + RPP * p], u);
                }
            };
            int l_done = 0;
            if constexpr (NG == LT && 2 * RPP == LT && WREC <= 32) {
                // d = 128: a window pass of keys is exactly one tile, two passes of delta values
                // fill it, so the tiles inside the register window need no second trip to memory
                // (not for the 64-record window: keeping it alive this long costs a workgroup per CU)
#pragma unroll
                for (int p = 0; p < KP; ++p) {
                    if (LT * p < m) {   // uniform
                        __syncthreads();
                        const int l = LT * p + grp;
                        float kx[8];
                        unpack8(kl_raw[p], kx);
                        const float w = l < f ? expf(Gc[0] - Gl[p]) : 0.0f;
                        if (l != f) {   // row f of the tile belongs to inject_new
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                kh[grp][8 * sub + e] = l < f ? w * kx[e] : 0.0f;
                        }
#pragma unroll
                        for (int jj = 0; jj < 2; ++jj) {
                            const int lu = LT * p + RPP * jj + rg;
                            const float4 u = ur[2 * p + jj];
                            if (lu != f)
                                *reinterpret_cast<float4 *>(&uu[RPP * jj + rg][4 * c4]) =
                                    lu < f ? u : make_float4(0.f, 0.f, 0.f, 0.f);
                        }
                        inject_new(LT * p);
                        __syncthreads();
                        apply_tile(LT * p);
                    }
                }
                l_done = LT * KP;
            }
            for (int l0 = l_done; l0 < m; l0 += LT) {
                __syncthreads();
                // records before f come back from memory (written by earlier calls)
#pragma unroll
                for (int x = 0; x < EPT; ++x) {
                    const int idx = tid + NT * x, l = l0 + idx / D, e = idx % D;
                    if (l < f) {
                        kh[idx / D][e] = expf(Gc[0] - Gbuf[ru(l)]) * to_f32(kb[rk(l) * D + e]);
                        uu[idx / D][e] = ub[ru(l) * D + e];
                    } else if (l > f) {
                        kh[idx / D][e] = 0.0f;
                        uu[idx / D][e] = 0.0f;
                    }
                }
                inject_new(l0);
                __syncthreads();
                apply_tile(l0);
            }
            float4 *sw = reinterpret_cast<float4 *>(a.st.state + unit * D * D);
#pragma unroll
            for (int p = 0; p < NPASS; ++p)
                sw[(size_t)(rg + RPP * p) * LPR + c4] = sreg[p];
            new_fill = 0;
        }
    }
    if (a.advance && tid == 0)
        publish_if_last(&a.st.fill[s], ticket, a.Hv, new_fill);
}

// ---------------------------------------------------------------------------
// kvb_flush: S <- gamma_{m-1} S + sum_{l<m} Gamma_{m-1,l} k_l^T u_l   (Eq. 16, last line)
// The rank-m sum is accumulated apart from the state so that the state tile can
// stay in flight until the very end.
// ---------------------------------------------------------------------------
struct FlushArgs {
    Store st;
    const int32_t *slot;
    const int32_t *accepted;
    int32_t Hk, Hv, cap, threshold;
};

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
// kvb_direct: the parallel form, Eq. 13, from a zero state.
//   cK[i][l] = Gamma_il (k_i.k_l) (l < i)     cQ[i][l] = Gamma_il (q_i.k_l) (l <= i)
//   u_i = beta_i ( v_i - sum_{l<i} cK[i][l] u_l )       (row i of A Diag(beta) V)
//   o_i = scale * sum_{l<=i} cQ[i][l] u_l
// ---------------------------------------------------------------------------
struct DirectArgs {
    Store st;
    const int32_t *slot;
    const int32_t *len;
    const void *q, *k, *v;
    const float *g, *beta;
    float *out;
    int32_t Hk, Hv, cap, Lmax;
    float scale;
};

template <int D, typename TIn, bool PAGED>
__global__ __launch_bounds__(NT) void kvb_direct_kernel(const DirectArgs a)
{
    constexpr int LM = KVB_MAX_DIRECT_LEN;
    __shared__ float sK[LM][D + 1];
    __shared__ float sQ[LM][D + 1];
    __shared__ float cK[LM][LM + 1];
    __shared__ float cQ[LM][LM + 1];
    __shared__ float sU[LM][D];
    __shared__ float sG[LM];
    __shared__ float sB[LM];
    __shared__ int sBlk[NW][MAX_BLOCKS];

    const int tid = threadIdx.x;
    const int lb = logical_block();
    const int b = lb / a.Hv;
    const int h = lb % a.Hv;
    const int r = a.Hv / a.Hk;
    const int hk = h / r;
    const int Lmax = a.Lmax;

    const int s = a.slot[b];
    if (s < 0 || s >= a.st.n_slots)
        return;
    int L = a.len[b];
    if (L < 0 || L > Lmax) {
        L = Lmax;
        if (tid == 0 && a.st.status)
            atomicOr(&a.st.status[s], KVB_STATUS_OVERFLOW);
    }
    const Pages<PAGED> pg = make_pages<PAGED>(a.st, s, a.cap, sBlk[tid / 64], tid % 64, load_block_id<PAGED>(a.st, s, tid % 64));
    auto ru = [&](int l) { return pg.row(l, a.Hv, h); };
    auto rk = [&](int l) { return pg.row(l, a.Hk, hk); };
    const TIn *qin = static_cast<const TIn *>(a.q);
    const TIn *kin = static_cast<const TIn *>(a.k);
    const TIn *vin = static_cast<const TIn *>(a.v);

    for (int idx = tid; idx < L * D; idx += NT) {
        const int i = idx / D, e = idx % D;
        const size_t o = (((size_t)b * Lmax + i) * a.Hk + hk) * D + e;
        sK[i][e] = to_f32(kin[o]);
        sQ[i][e] = to_f32(qin[o]);
    }
    if (tid < L) {
        float run = 0.0f;
        for (int t = 0; t <= tid; ++t)
            run += a.g[((size_t)b * Lmax + t) * a.Hv + h];
        sG[tid] = run;
        sB[tid] = a.beta[((size_t)b * Lmax + tid) * a.Hv + h];
    }
    __syncthreads();

    for (int p = tid; p < L * L; p += NT) {
        const int i = p / L, l = p % L;
        if (l <= i) {
            float dkk = 0.0f, dqk = 0.0f;
#pragma unroll 8
            for (int e = 0; e < D; ++e) {
                const float kl = sK[l][e];
                dkk = fmaf(sK[i][e], kl, dkk);
                dqk = fmaf(sQ[i][e], kl, dqk);
            }
            const float gam = expf(sG[i] - sG[l]);
            cK[i][l] = gam * dkk;
            cQ[i][l] = gam * dqk;
        }
    }
    __syncthreads();

    if (tid < D) {
        for (int i = 0; i < L; ++i) {
            const size_t row = ((size_t)b * Lmax + i) * a.Hv + h;
            float acc = to_f32(vin[row * D + tid]);
            float o = 0.0f;
            for (int l = 0; l < i; ++l) {
                const float ul = sU[l][tid];
                acc = fmaf(-cK[i][l], ul, acc);
                o = fmaf(cQ[i][l], ul, o);
            }
            const float ui = sB[i] * acc;
            sU[i][tid] = ui;
            o = fmaf(cQ[i][i], ui, o);
            a.out[row * D + tid] = a.scale * o;
            a.st.buf_u[ru(i) * D + tid] = ui;
        }
    }
    if (tid < L)
        a.st.buf_G[ru(tid)] = sG[tid];
    if (h % r == 0) {
        TIn *kb = static_cast<TIn *>(a.st.buf_k);
        for (int idx = tid; idx < L * D; idx += NT) {
            const int i = idx / D, e = idx % D;
            kb[rk(i) * D + e] = kin[(((size_t)b * Lmax + i) * a.Hk + hk) * D + e];
        }
    }
    if (h == 0 && tid == 0)
        a.st.fill[s] = L;
}

// ---------------------------------------------------------------------------
// kvb_direct for bf16 inputs and d = 128, on the matrix cores throughout.
//
// The context is cut into blocks of 16 rows.  With N_il = beta_i Gamma_il (k_i.k_l) (l < i)
// and M_il = Gamma_il (q_i.k_l) (l <= i) the parallel form (Eq. 13) is
//     (I + N) U = Diag(beta) V,      O = M U,
// solved block row by block row:  U_d = T_d ( beta V_d - sum_{e<d} N_de U_e ),
// T_d = (I + N_dd)^-1 = (I - N)(I + N^2)(I + N^4)(I + N^8)   (N_dd is strictly lower, N^16 = 0),
// O_d = sum_{e<=d} M_de U_e.
//   * Gram tiles (k.k, q.k over dk = 128, bf16 operands): v_mfma_f32_16x16x32_bf16.
//   * everything after that has fp32 operands: v_mfma_f32_16x16x4_f32 (exact products).
//
// Register chaining.  Call "A-form" of a 16x16 matrix X the register layout in which lane l
// holds X[l%16][4*(l/16)+v], v = 0..3, and "B-form" the one with X[4*(l/16)+v][l%16].  An
// MFMA result is in B-form; feeding four k-steps with (a = xa[v], b = yb[v]) gives the
// B-form of X Y, and swapping the operands, (a = yb[v], b = xa[v]), gives the A-form of X Y.
// A Gram tile computed as (rows of block e) x (rows of block d) lands directly in A-form of
// the (d, e) tile, so no value ever needs to move between lanes: tiles shared between waves
// go through LDS as whole per-lane float4s.  Each wave owns 32 dv columns (two column tiles).
// ---------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

// B-form of X Y from X in A-form and Y in B-form (swap the arguments for the A-form of X Y).
__device__ __forceinline__ f32x4_t mm16(const f32x4_t &xa, const f32x4_t &yb, f32x4_t acc)
{
#pragma unroll
    for (int v = 0; v < 4; ++v)
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[v], yb[v], acc, 0, 0, 0);
    return acc;
}

// exp for arguments that are differences of cumulative log decays (<= 0, a few tens at
// most): one multiply and the hardware exp2; relative error about |x| * 2^-23, far inside
// the 2e-3 bound of the bf16 paths that use it.
__device__ __forceinline__ float fast_exp(float x) { return __expf(x); }

template <typename... Ts>
constexpr uint32_t pack2(Ts... xs)
{
    uint32_t r = 0;
    int sh = 0;
    ((r |= (uint32_t)xs << sh, sh += 2), ...);
    return r;
}

// Raw Gram tile from rows staged in LDS (row stride GS bf16 elements): lane l reads row l%16
// of the A-side block and of the B-side block at k = 8*(l/16) + 32*step.  acc[v] =
// (A-side row 4*(l/16)+v) . (B-side row l%16), i.e. the A-form of the (B-block, A-block) tile.
template <int GS>
__device__ __forceinline__ f32x4_t gram16(const bf16_t *arow, const bf16_t *brow, int lq)
{
    f32x4_t c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int st = 0; st < 4; ++st) {
        const uint4 av = *reinterpret_cast<const uint4 *>(arow + 8 * lq + 32 * st);
        const uint4 bv = *reinterpret_cast<const uint4 *>(brow + 8 * lq + 32 * st);
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av),
                                                    __builtin_bit_cast(bf16x8_t, bv), c, 0, 0, 0);
    }
    return c;
}

template <bool PAGED>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(5, 5))) void kvb_direct_mfma_kernel(
    const DirectArgs a)
{
    constexpr int D = 128;
    constexpr int LM = KVB_MAX_DIRECT_LEN;
    constexpr int NB = LM / 16;                 // blocks of 16 rows (4)
    constexpr int NLOW = NB * (NB + 1) / 2;     // lower-triangular block pairs (10)
    constexpr int GS = D + 8;                   // LDS row stride of the staged keys / queries (272 B:
                                                // consecutive rows start 4 banks apart)
    static_assert(NB == NW, "one diagonal block per wave");
    // One LDS region, used twice: first the staged K and Q rows (bf16), then, once every
    // raw Gram tile sits in registers, the weighted tiles in A-form (one float4 per lane):
    // -N_de (d > e), M_de (d >= e), T_d.
    constexpr int STAGE_BYTES = LM * GS * 2;
    constexpr int TILE_BYTES = (2 * NLOW + NB) * 64 * 16;
    __shared__ __attribute__((aligned(16))) unsigned char region[STAGE_BYTES > TILE_BYTES ? STAGE_BYTES : TILE_BYTES];
    __shared__ float sG[LM];
    __shared__ float sB[LM];
    __shared__ int sBlk[NW][MAX_BLOCKS];
    bf16_t *sK = reinterpret_cast<bf16_t *>(region);
    float4(*tN)[64] = reinterpret_cast<float4(*)[64]>(region);
    float4(*tM)[64] = tN + NLOW;
    float4(*tT)[64] = tM + NLOW;

    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
    const int c16 = lane % 16, lq = lane / 16;
    const int lb = logical_block();
    const int b = lb / a.Hv;
    const int h = lb % a.Hv;
    const int r = a.Hv / a.Hk;
    const int hk = h / r;
    const int Lmax = a.Lmax;

    const int s = a.slot[b];
    if (s < 0 || s >= a.st.n_slots)
        return;
    int L = a.len[b];
    if (L < 0 || L > Lmax) {
        L = Lmax;
        if (tid == 0 && a.st.status)
            atomicOr(&a.st.status[s], KVB_STATUS_OVERFLOW);
    }
    if (L == 0) {
        if (h == 0 && tid == 0)
            a.st.fill[s] = 0;
        return;
    }
    const Pages<PAGED> pg = make_pages<PAGED>(a.st, s, a.cap, sBlk[wave], lane, load_block_id<PAGED>(a.st, s, lane));
    auto ru = [&](int l) { return pg.row(l, a.Hv, h); };
    auto rk = [&](int l) { return pg.row(l, a.Hk, hk); };
    const bf16_t *qin = static_cast<const bf16_t *>(a.q);
    const bf16_t *kin = static_cast<const bf16_t *>(a.k);
    const bf16_t *vin = static_cast<const bf16_t *>(a.v);
    const int nb = (L + 15) / 16;
    auto tri = [](int d, int e) { return d * (d + 1) / 2 + e; };

    // ---- all global loads of the workgroup, issued together ---------------------
    // K and Q rows, 16 bytes per thread and pass (pass p = rows 16 p .. 16 p + 15)
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    u32x4_t kst[NB];
    const int srow = tid / 16, sc8 = tid % 16;
    // (uniform 64-bit base + 32-bit per-lane offset keeps the address arithmetic out of the VGPRs)
    const bf16_t *kbase = kin + ((size_t)b * Lmax * a.Hk + hk) * D;
    const bf16_t *qbase = qin + ((size_t)b * Lmax * a.Hk + hk) * D;
    const bf16_t *vbase = vin + ((size_t)b * Lmax * a.Hv + h) * D;
    const uint32_t qk_stride = (uint32_t)a.Hk * D, v_stride = (uint32_t)a.Hv * D;
#pragma unroll
    for (int p = 0; p < NB; ++p) {   // rows past the context re-read its last row (never used)
        const uint32_t o = (uint32_t)min(16 * p + srow, L - 1) * qk_stride + 8 * sc8;
        kst[p] = u32x4_t{0u, 0u, 0u, 0u};
        if (p < nb)   // uniform
            kst[p] = *reinterpret_cast<const u32x4_t *>(kbase + o);
    }
    // Q is not staged: the waves read the rows of their q.k tiles straight from memory in the
    // operand layout of the matrix instruction (row 16 d + c16, k = 8 lq + 32 step); a block of
    // 16 query rows is 4 KB and is shared by at most 4 tiles, so the repeats hit in the caches
    // and the LDS footprint is that of K alone (5 workgroups per CU instead of 4).
    // Tiles are dealt round-robin: t = wave + 4 n; t < 6 are k.k pairs, the rest q.k pairs.
    constexpr uint32_t PDB = pack2(1, 2, 2, 3, 3, 3, 0, 1, 1, 2, 2, 2, 3, 3, 3, 3);
    constexpr uint32_t PEB = pack2(0, 0, 1, 0, 1, 2, 0, 0, 1, 0, 1, 2, 0, 1, 2, 3);
    auto PD = [](int t) { return (int)((PDB >> (2 * t)) & 3u); };
    auto PE = [](int t) { return (int)((PEB >> (2 * t)) & 3u); };
    u32x4_t qop[3][4];   // n = 1 (waves 2, 3 only), 2, 3
#pragma unroll
    for (int n = 1; n < 4; ++n) {
        const int t = wave + NW * n, d = PD(t);
        const uint32_t o = (uint32_t)min(16 * d + c16, L - 1) * qk_stride + 8 * lq;
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            qop[n - 1][st] = u32x4_t{0u, 0u, 0u, 0u};
            if (t >= 6 && d < nb)   // uniform
                qop[n - 1][st] = *reinterpret_cast<const u32x4_t *>(qbase + o + 32 * st);
        }
    }
    const int col2 = 32 * wave + 2 * c16;
    // cumulative log decay (inclusive scan over the wave) and beta
    if (wave == 0) {
        float gv = lane < L ? a.g[((size_t)b * Lmax + lane) * a.Hv + h] : 0.0f;
        const float bv = lane < L ? a.beta[((size_t)b * Lmax + lane) * a.Hv + h] : 0.0f;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const float t = __shfl_up(gv, off);
            if (lane >= off)
                gv += t;
        }
        sG[lane] = gv;
        sB[lane] = bv;
        if (lane < L)
            a.st.buf_G[ru(lane)] = gv;
    }
    // stage K, Q; the thread that loaded a piece of K also appends it to the buffer
    bf16_t *kb = static_cast<bf16_t *>(a.st.buf_k);
#pragma unroll
    for (int p = 0; p < NB; ++p) {
        if (p < nb) {   // uniform
            *reinterpret_cast<u32x4_t *>(sK + (16 * p + srow) * GS + 8 * sc8) = kst[p];
            if (h % r == 0 && 16 * p + srow < L)
                *reinterpret_cast<u32x4_t *>(kb + rk(16 * p + srow) * D + 8 * sc8) = kst[p];
        }
    }
    __syncthreads();

    // ---- raw Gram tiles: this wave's diagonal k.k tile and its share of the others ----
    // off-diagonal k.k pairs (d > e): 6; q.k pairs (d >= e): 10
    // (two bits per entry, packed: a table indexed by the wave number would live in scratch)
    f32x4_t gdiag = {0.f, 0.f, 0.f, 0.f};
    if (wave < nb)
        gdiag = gram16<GS>(sK + (16 * wave + c16) * GS, sK + (16 * wave + c16) * GS, lq);
    f32x4_t gsh[4];
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        const int t = wave + NW * n, d = PD(t), e = PE(t);
        gsh[n] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        if (d < nb) {   // uniform
            if (t < 6) {
                gsh[n] = gram16<GS>(sK + (16 * e + c16) * GS, sK + (16 * d + c16) * GS, lq);
            } else if (n > 0) {   // t >= 6 implies n >= 1
                const bf16_t *arow = sK + (16 * e + c16) * GS;
#pragma unroll
                for (int st = 0; st < 4; ++st) {
                    const uint4 av = *reinterpret_cast<const uint4 *>(arow + 8 * lq + 32 * st);
                    gsh[n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8_t, av), __builtin_bit_cast(bf16x8_t, qop[n > 0 ? n - 1 : 0][st]),
                        gsh[n], 0, 0, 0);
                }
            }
        }
    }
    __syncthreads();   // every wave is done with the staged rows: the region now takes the tiles

    // v in B-form: rows 16 d + 4 lq + v, this lane's two adjacent columns 32 wave + 2 c16, + 1.
    // Requested only now, when the registers of the staged rows are free again; the values
    // are not needed before the substitution, two phases further down.
    uint32_t v_raw[NB][4];
#pragma unroll
    for (int d = 0; d < NB; ++d)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            v_raw[d][v] = 0u;
            if (d < nb)   // uniform
                v_raw[d][v] = *reinterpret_cast<const uint32_t *>(
                    vbase + (uint32_t)min(16 * d + 4 * lq + v, L - 1) * v_stride + col2);
        }

    // weights and masks.  A-form element of tile (d, e): row i = 16 d + c16, column l = 16 e + 4 lq + v.
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        const int t = wave + NW * n, d = PD(t), e = PE(t);
        if (d < nb) {
            const int i = 16 * d + c16;
            const bool isq = t >= 6;
            float o[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int l = 16 * e + 4 * lq + v;
                const bool ok = i < L && (isq ? l <= i : l < i);
                const float w = ok ? fast_exp(sG[i] - sG[l]) : 0.0f;
                o[v] = (isq ? w : -sB[i] * w) * gsh[n][v];
            }
            const float4 o4 = make_float4(o[0], o[1], o[2], o[3]);
            if (isq)
                tM[tri(d, e)][lane] = o4;
            else
                tN[tri(d, e)][lane] = o4;
        }
    }
    // T_d for d = wave.  The raw diagonal tile is symmetric, so the same registers give the
    // A-form (row 16 d + c16, column 16 d + 4 lq + v) and the B-form (row and column swapped).
    if (wave < nb) {
        const int d = wave;
        f32x4_t na, nbm, ia;   // N in both forms; identity mask (the same in both forms)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int ia_i = 16 * d + c16, ia_l = 16 * d + 4 * lq + v;    // A-form indices
            const int ib_i = ia_l, ib_l = ia_i;                            // B-form indices
            const float wa = (ia_i < L && ia_l < ia_i) ? sB[ia_i] * fast_exp(sG[ia_i] - sG[ia_l]) : 0.0f;
            const float wb = (ib_i < L && ib_l < ib_i) ? sB[ib_i] * fast_exp(sG[ib_i] - sG[ib_l]) : 0.0f;
            na[v] = wa * gdiag[v];
            nbm[v] = wb * gdiag[v];
            ia[v] = ia_i == ia_l ? 1.0f : 0.0f;
        }
        const f32x4_t z = {0.f, 0.f, 0.f, 0.f};
        const f32x4_t n2b = mm16(na, nbm, z), n2a = mm16(nbm, na, z);
        const f32x4_t n4b = mm16(n2a, n2b, z), n4a = mm16(n2b, n2a, z);
        const f32x4_t n8b = mm16(n4a, n4b, z);
        // A-form of (I - N)(I + N^2), then x (I + N^4), then x (I + N^8)
        f32x4_t p = mm16(ia + n2b, ia - na, z);
        p = mm16(ia + n4b, p, z);
        p = mm16(ia + n8b, p, z);
        tT[d][lane] = make_float4(p[0], p[1], p[2], p[3]);
    }
    __syncthreads();

    // ---- block forward substitution and outputs, this wave's 32 columns ----------
    // column tile c of the wave holds columns 32 wave + 2 n + c (n = 0..15): a lane's two
    // tiles are adjacent columns, so v arrives as one 4-byte load and results leave as float2
    f32x4_t U[NB][2];
    float *outp = a.out + (((size_t)b * Lmax) * a.Hv + h) * D;
    float *up = a.st.buf_u;
#pragma unroll
    for (int d = 0; d < NB; ++d) {
        if (d < nb) {   // uniform
            f32x4_t acc[2], o[2];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = 16 * d + 4 * lq + v;
                const float bi = i < L ? sB[i] : 0.0f;
                acc[0][v] = bi * __uint_as_float(v_raw[d][v] << 16);
                acc[1][v] = bi * __uint_as_float(v_raw[d][v] & 0xFFFF0000u);
            }
            o[0] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            o[1] = o[0];
#pragma unroll
            for (int e = 0; e < d; ++e) {
                const float4 n4 = tN[tri(d, e)][lane];
                const float4 m4 = tM[tri(d, e)][lane];
                const f32x4_t nn = {n4.x, n4.y, n4.z, n4.w}, mm = {m4.x, m4.y, m4.z, m4.w};
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    acc[c] = mm16(nn, U[e][c], acc[c]);
                    o[c] = mm16(mm, U[e][c], o[c]);
                }
            }
            const float4 t4 = tT[d][lane];
            const float4 m4 = tM[tri(d, d)][lane];
            const f32x4_t tt = {t4.x, t4.y, t4.z, t4.w}, mm = {m4.x, m4.y, m4.z, m4.w};
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                U[d][c] = mm16(tt, acc[c], f32x4_t{0.f, 0.f, 0.f, 0.f});
                o[c] = mm16(mm, U[d][c], o[c]);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = 16 * d + 4 * lq + v;
                if (i < L) {
                    *reinterpret_cast<float2 *>(outp + ((uint32_t)i * v_stride + col2)) =
                        make_float2(a.scale * o[0][v], a.scale * o[1][v]);
                    *reinterpret_cast<float2 *>(up + (ru(i) * D + col2)) = make_float2(U[d][0][v], U[d][1][v]);
                }
            }
        }
    }
    if (h == 0 && tid == 0)
        a.st.fill[s] = L;
}

// ---------------------------------------------------------------------------
// kvb_verify for bf16 inputs and d = 128, on the matrix cores.
//
// With T drafts the step is a pair of small dense contractions (Sec. 3.3, Eq. 7; Eq. 15):
//   stage 1   C1[m][l] = W[m] . k_l        W = [k_0..k_7 ; q_0..q_7] (16 x dk, bf16),
//             l over the buffered and the new keys  -> v_mfma_f32_16x16x32_bf16
//   stage 2   acc[m][:] = sum_rows sW[row][m] S0[row][:] + sum_{l<f} cW[l][m] u_l[:]
//             (16 x (dk + f)) . ((dk + f) x dv), fp32 operands -> v_mfma_f32_16x16x4_f32
// where sW[row][m] = -gamma_i k_i[row] (m = i) or gamma_i q_i[row] (m = 8 + i) and
// cW[l][m] = -/+ Gamma_il C1[m][l].  The cost of stage 2 does not depend on T <= 8.
// Each wave owns 32 dv columns for all rows, so no reduction across waves is needed; a
// lane loads 2 adjacent columns of 4 consecutive rows' worth of lanes (16 lanes x 8 B =
// one 128-byte line per row).  MFMA layouts: see kvb_direct_mfma_kernel; for 16x16x4 fp32
// lane l supplies A[l%16][l/16] and B[l/16][l%16] and receives C[4*(l/16)+v][l%16].
// ---------------------------------------------------------------------------
template <int WREC, bool HAS_STATE, bool STREAM, bool PAGED>
__global__ __launch_bounds__(NT) void kvb_verify_mfma_kernel(const StepArgs a)
{
    constexpr int D = 128;
    constexpr int TMX = KVB_MAX_DRAFTS;                       // 8
    constexpr int NTILE = (KVB_MAX_CAP + TMX + 15) / 16;      // key tiles of 16 (9)
    constexpr int NTW = ((WREC + TMX + 15) / 16 + NW - 1) / NW;  // tiles per wave held in registers
    constexpr int WQ = WREC / 4;                              // record quads held in registers
    constexpr bool TAIL = WREC >= 64;
    constexpr bool EARLY = HAS_STATE && WREC <= 32;   // state loads issued before the fill is known
    static_assert(TMX == 8, "row m of W is draft m % 8");

    __shared__ __attribute__((aligned(16))) float sW[D][16];
    __shared__ __attribute__((aligned(16))) float cW[NTILE * 16][16];
    __shared__ __attribute__((aligned(16))) float fin[16][D];
    __shared__ int sBlk[NW][MAX_BLOCKS];
    __shared__ float sGc[TAIL ? NW : 1][TMX];   // per-wave table for the keys beyond the register window

    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
    const int lb = logical_block();
    const int b = lb / a.Hv;
    const int h = lb % a.Hv;
    const int r = a.Hv / a.Hk;
    const int hk = h / r;
    const int T = a.T;
    const int cap = a.cap;

    const int s = a.slot[b];
    if (s < 0 || s >= a.st.n_slots)
        return;
    const size_t unit = (size_t)s * a.Hv + h;
    const bf16_t *qin = static_cast<const bf16_t *>(a.q);
    const bf16_t *kin = static_cast<const bf16_t *>(a.k);
    const bf16_t *vin = static_cast<const bf16_t *>(a.v);
    const float *Gbuf = a.st.buf_G;                               // record l of this head: Gbuf[ru(l)]
    const bf16_t *kb = static_cast<const bf16_t *>(a.st.buf_k);   //                        kb + rk(l) * D
    const float *ub = a.st.buf_u;                                 //                        ub + ru(l) * D
    const int blk_id = load_block_id<PAGED>(a.st, s, lane);

    const int lm = lane % 16, lq = lane / 16;   // MFMA row/column index and k index of this lane
    const int col2 = 32 * wave + 2 * lm;

    // ---- 1. loads that need only the request index: raw bits, clamped addresses, no branches
    // row lm of W (draft lm % 8; k for lm < 8, q above), k-chunk lq of each 32-wide step
    const int wi = min(lm % 8, T - 1);
    const bf16_t *wrow = (lm < 8 ? kin : qin) + (((size_t)b * T + wi) * a.Hk + hk) * D + 8 * lq;
    uint4 wa[4];
#pragma unroll
    for (int st = 0; st < 4; ++st)
        wa[st] = *reinterpret_cast<const uint4 *>(wrow + 32 * st);

    // ---- 2. the state: rows 4 st + lq, the wave's 32 columns -----------------
    // EARLY: the state's address needs the slot only, so its loads go out before the fill is
    // known and before the long scalar prologue; the records follow and are consumed after the
    // state (the decay gamma_i of row i is then applied to the finished sum over state rows).
    float2 sreg[D / 4];
    auto issue_state = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        const float *sp = a.st.state + unit * D * D + col2;
#pragma unroll
        for (int st = 0; st < D / 4; ++st) {
            const float2 *p = reinterpret_cast<const float2 *>(sp + (size_t)(4 * st + lq) * D);
            if constexpr (STREAM) {
                typedef float v2f __attribute__((ext_vector_type(2)));
                const v2f t = __builtin_nontemporal_load(reinterpret_cast<const v2f *>(p));
                sreg[st] = make_float2(t.x, t.y);
            } else {
                sreg[st] = *p;
            }
            __builtin_amdgcn_sched_barrier(0);   // issue in the order they are consumed
        }
    };
    if constexpr (EARLY)
        issue_state();

    const int f = a.st.fill[s] & FILL_MASK;
    if (f + T > cap) {
        if (tid == 0 && a.st.status)
            atomicOr(&a.st.status[s], KVB_STATUS_OVERFLOW);
        return;
    }
    const int nrec = f + T;
    const Pages<PAGED> pg = make_pages<PAGED>(a.st, s, cap, sBlk[wave], lane, blk_id);
    auto ru = [&](int l) { return pg.row(l, a.Hv, h); };
    auto rk = [&](int l) { return pg.row(l, a.Hk, hk); };
    const int ntile = (nrec + 15) / 16;

    // ---- 3. loads that need the fill ------------------------------------------
    // per-draft scalars of draft lane % 8, one vector load each (a scalar load per draft costs
    // a round trip each while the chip is streaming)
    const size_t go = ((size_t)b * T + min(lane % 8, T - 1)) * a.Hv + h;
    float g_raw = a.g[go];
    float beta_mine = a.beta[go];
    int par_raw = a.parent[(size_t)b * T + min(lane % 8, T - 1)];
    float G_prev = f > 0 ? Gbuf[ru(f - 1)] : 0.0f;
    // keys of this wave's tiles (buffered first, then the new ones)
    uint4 kt[NTW][4];
    float Gn[NTW];
#pragma unroll
    for (int x = 0; x < NTW; ++x) {
        const int n = 16 * (wave + NW * x) + lm;
        const bf16_t *kp = n < f ? kb + rk(n) * D
                                 : kin + (((size_t)b * T + min(max(n - f, 0), T - 1)) * a.Hk + hk) * D;
        Gn[x] = Gbuf[ru(n < f ? n : 0)];
#pragma unroll
        for (int st = 0; st < 4; ++st)
            kt[x][st] = *reinterpret_cast<const uint4 *>(kp + 8 * lq + 32 * st);
    }
    // buffered delta values: quad sq = records 4 sq .. 4 sq + 3, this lane: record 4 sq + lq,
    // columns 32 wave + 2 lm, + 1
    float2 uq[WQ];
#pragma unroll
    for (int sq = 0; sq < WQ; ++sq) {
        const int l = 4 * sq + lq;
        uq[sq] = *reinterpret_cast<const float2 *>(ub + ru(l < f ? l : 0) * D + col2);
    }
    // v of this wave's columns (used by lanes 0..31 in the last stage)
    const int colf = 32 * wave + lane % 32;
    bf16_t v_raw[TMX];
#pragma unroll
    for (int i = 0; i < TMX; ++i)
        v_raw[i] = vin[(((size_t)b * T + min(i, T - 1)) * a.Hv + h) * D + colf];
    if constexpr (HAS_STATE && !EARLY)
        issue_state();
    __builtin_amdgcn_sched_barrier(0);

    // Cumulative log decays and betas of the drafts as wave-uniform values read from the lanes
    // that loaded them.  Whatever a lane needs by a draft index of its own is selected here,
    // while the running sum is in a register: an array indexed at run time would live in
    // scratch memory, whose loads share the counter of the state loads.
    float bet[TMX];
    float GcRow[4];      // of the draft of accumulator row 4 lq + v: draft v (lq even) or 4 + v (lq odd)
    float GcLm = 0.0f;   // of draft lm % 8 (the row of W this lane loaded)
    float GcTid = 0.0f;  // of draft tid (the lane that stores it)
    float GcKey[NTW];    // of the new key this lane holds in window tile x, if it holds one
#pragma unroll
    for (int x = 0; x < NTW; ++x)
        GcKey[x] = 0.0f;
    // Drafts form a chain (kvb_verify) or a tree (kvb_verify_tree): the decay of draft i runs
    // along its own root path, and anc_i has bit j set iff draft j is a strict ancestor of i.
    // A parent index that does not precede its child is taken as -1 and flagged.
    int ancRow[4];       // ancestor bits of the draft of accumulator row 4 lq + v
    auto finish_Gc = [&]() {
        float Gi[TMX];   // wave-uniform; constant indices only
        int anc[TMX];
        bool bad = false;
        const bool tree = a.tree != 0;   // uniform; no load sits behind this branch
#pragma unroll
        for (int i = 0; i < TMX; ++i) {
            const float gi = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, g_raw), i));
            bet[i] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, beta_mine), i));
            float base = i > 0 ? Gi[i > 0 ? i - 1 : 0] : G_prev;   // chain: the previous draft
            int am = (1 << i) - 1;
            if (tree) {
                const int pi = __builtin_amdgcn_readlane(par_raw, i);
                bad = bad || (i < T && (pi < -1 || pi >= i));
                base = G_prev;
                am = 0;
#pragma unroll
                for (int j = 0; j < i; ++j) {
                    const bool is_parent = pi == j;
                    base = is_parent ? Gi[j] : base;
                    am = is_parent ? (anc[j] | (1 << j)) : am;
                }
            }
            const float run = base + (i < T ? gi : 0.0f);
            Gi[i] = run;
            anc[i] = am;
            if (i < 4) {
                GcRow[i] = run;
                ancRow[i] = am;
            } else {
                GcRow[i - 4] = lq % 2 ? run : GcRow[i - 4];
                ancRow[i - 4] = lq % 2 ? am : ancRow[i - 4];
            }
            GcLm = lm % 8 == i ? run : GcLm;
            GcTid = tid == i ? run : GcTid;
#pragma unroll
            for (int x = 0; x < NTW; ++x)
                GcKey[x] = 16 * (wave + NW * x) + lm - f == i ? run : GcKey[x];
            if (TAIL && lane == 0)
                sGc[wave][i] = run;
        }
        if (bad && tid == 0 && a.st.status)
            atomicOr(&a.st.status[s], KVB_STATUS_BADPATH);
    };
    if constexpr (!EARLY)
        finish_Gc();

    // ---- 4. weights of the state rows ------------------------------------------
    f32x4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    const bool live = lm % 8 < T;
    {
        // the chunk this lane holds for step == wave covers state rows 32 wave + 8 lq .. + 7
        float x[8];
        unpack8(Raw8<bf16_t>{wa[0]}, x);
#pragma unroll
        for (int st = 1; st < 4; ++st) {
            float y[8];
            unpack8(Raw8<bf16_t>{wa[st]}, y);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                x[e] = wave == st ? y[e] : x[e];
        }
        float gam;
        if constexpr (EARLY)
            gam = live ? 1.0f : 0.0f;
        else
            gam = live ? expf(GcLm) : 0.0f;
        const float sg = lm < 8 ? -gam : gam;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            sW[32 * wave + 8 * lq + e][lm] = sg * x[e];
    }
    auto state_rows = [&]() {
#pragma unroll
        for (int st = 0; st < D / 4; ++st) {
            const float aw = sW[4 * st + lq][lm];
            acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(aw, sreg[st].x, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(aw, sreg[st].y, acc1, 0, 0, 0);
        }
    };
    if constexpr (EARLY) {
        __syncthreads();   // sW complete
        __builtin_amdgcn_sched_barrier(0);
        state_rows();
        // pins the sums, and whatever derives from the loads younger than the state, to this
        // point: pure arithmetic is otherwise free to drift across the fences
        asm volatile("" : "+v"(acc0), "+v"(acc1), "+v"(G_prev), "+v"(g_raw), "+v"(beta_mine), "+v"(par_raw));
        __builtin_amdgcn_sched_barrier(0);
        finish_Gc();
        // acc*[v] is row m = 4 lq + v = draft m % 8: apply its gamma
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int i = (4 * lq + v) % 8;
            const float gam = i < T ? expf(GcRow[v]) : 0.0f;
            acc0[v] *= gam;
            acc1[v] *= gam;
        }
    }

    // ---- 5. stage 1: decayed dot products with every buffered and new key -------
    // Gkey: cumulative log decay of key n of the tile (a buffered one from memory, a new one from above)
    auto key_tile = [&](int tile, const uint4(&kk)[4], float Gkey) {
        f32x4_t c1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int st = 0; st < 4; ++st)
            c1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wa[st]),
                                                         __builtin_bit_cast(bf16x8_t, kk[st]), c1, 0, 0, 0);
        // this lane: rows m = 4 lq + v of W against key n
        const int n = 16 * tile + lm;
        float o[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int m = 4 * lq + v, i = m % 8;
            const bool isq = m >= 8;
            // a buffered key is seen by every draft; a new one by its descendants (q rows: and by itself)
            const bool above = n >= f && ((ancRow[v] >> min(n - f, 31)) & 1);
            const bool ok = i < T && n < nrec && (n < f || above || (isq && n - f == i));
            const float w = ok ? expf(GcRow[v] - Gkey) : 0.0f;
            o[v] = (isq ? w : -w) * c1[v];
        }
        *reinterpret_cast<float4 *>(&cW[n][4 * lq]) = make_float4(o[0], o[1], o[2], o[3]);
    };
#pragma unroll
    for (int x = 0; x < NTW; ++x) {
        const int tile = wave + NW * x;
        if (tile < ntile)
            key_tile(tile, kt[x], 16 * tile + lm < f ? Gn[x] : GcKey[x]);
    }
    for (int tile = wave + NW * NTW; TAIL && tile < ntile; tile += NW) {   // keys beyond the register window
        const int n = 16 * tile + lm;
        const bf16_t *kp = n < f ? kb + rk(min(n, cap - 1)) * D
                                 : kin + (((size_t)b * T + min(max(n - f, 0), T - 1)) * a.Hk + hk) * D;
        uint4 kk[4];
#pragma unroll
        for (int st = 0; st < 4; ++st)
            kk[st] = *reinterpret_cast<const uint4 *>(kp + 8 * lq + 32 * st);
        const float Gb = Gbuf[ru(n < f ? n : 0)];
        key_tile(tile, kk, n < f ? Gb : sGc[wave][min(max(n - f, 0), TMX - 1)]);
    }
    __syncthreads();

    // ---- 6. stage 2 on the fp32 matrix cores: records (and, if not yet done, state rows)
    const int nquad = (f + 3) / 4;
#pragma unroll
    for (int sq = 0; sq < WQ; ++sq) {
        if (sq < nquad) {   // uniform
            const bool ok = 4 * sq + lq < f;
            const float aw = cW[4 * sq + lq][lm];
            acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(aw, ok ? uq[sq].x : 0.0f, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(aw, ok ? uq[sq].y : 0.0f, acc1, 0, 0, 0);
        }
    }
    for (int sq = WQ; TAIL && sq < nquad; ++sq) {
        const int l = 4 * sq + lq;
        const float2 u = *reinterpret_cast<const float2 *>(ub + ru(l < f ? l : 0) * D + col2);
        const float aw = cW[l][lm];
        acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(aw, l < f ? u.x : 0.0f, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(aw, l < f ? u.y : 0.0f, acc1, 0, 0, 0);
    }
    if constexpr (HAS_STATE && !EARLY)
        state_rows();
    // acc*[v] = row m = 4 lq + v, column col2 (+1)
#pragma unroll
    for (int v = 0; v < 4; ++v)
        *reinterpret_cast<float2 *>(&fin[4 * lq + v][col2]) = make_float2(acc0[v], acc1[v]);
    __syncthreads();

    // ---- 5. the T new rows among themselves; results ---------------------------
    // (all loads are consumed before the first store: the memory counter also counts stores,
    // and a wait for a late load inside the loop would wait for the stores of earlier drafts)
    float vf[TMX];
#pragma unroll
    for (int i = 0; i < TMX; ++i) {
        vf[i] = to_f32(v_raw[i]);
        asm volatile("" : "+v"(vf[i]));
    }
    if (lane < 32) {
        // every LDS value of the substitution is fetched up front (independent reads, one
        // round trip for all) rather than one by one along the serial chain
        float fu[TMX], fo[TMX], ck[TMX][TMX], cq[TMX][TMX];
#pragma unroll
        for (int i = 0; i < TMX; ++i) {
            if (i < T) {   // uniform
                fu[i] = fin[i][colf];
                fo[i] = fin[8 + i][colf];
#pragma unroll
                for (int j = 0; j <= i; ++j) {
                    ck[i][j] = cW[f + j][i];       // K rows are stored negated
                    cq[i][j] = cW[f + j][8 + i];
                }
            } else {
                fu[i] = fo[i] = 0.0f;
#pragma unroll
                for (int j = 0; j <= i; ++j)
                    ck[i][j] = cq[i][j] = 0.0f;
            }
        }
#pragma unroll
        for (int i = 0; i < TMX; ++i) {
            asm volatile("" : "+v"(fu[i]), "+v"(fo[i]));
#pragma unroll
            for (int j = 0; j <= i; ++j)
                asm volatile("" : "+v"(ck[i][j]), "+v"(cq[i][j]));
        }
        float uprev[TMX];
#pragma unroll
        for (int i = 0; i < TMX; ++i) {
            if (i < T) {
                float acc = vf[i] + fu[i];
                float ao = fo[i];
#pragma unroll
                for (int j = 0; j < TMX; ++j) {
                    if (j < i) {
                        acc = fmaf(ck[i][j], uprev[j], acc);
                        ao = fmaf(cq[i][j], uprev[j], ao);
                    }
                }
                const float ui = bet[i] * acc;
                ao = fmaf(cq[i][i], ui, ao);
                uprev[i] = ui;
                fin[i][colf] = ui;                 // a lane overwrites only what it has read itself
                fin[8 + i][colf] = a.scale * ao;
            }
        }
    }
    __syncthreads();
    // results leave as whole 512-byte rows, 16 bytes per lane: T rows of u, then T rows of out
    for (int idx = tid; idx < 2 * T * (D / 4); idx += NT) {
        const int rr = idx / (D / 4), c4 = idx % (D / 4);
        const bool is_u = rr < T;
        const int i = is_u ? rr : rr - T;
        const float4 val = *reinterpret_cast<const float4 *>(&fin[is_u ? i : 8 + i][4 * c4]);
        float *dst = is_u ? a.st.buf_u + ru(f + i) * D : a.out + (((size_t)b * T + i) * a.Hv + h) * D;
        *reinterpret_cast<float4 *>(dst + 4 * c4) = val;
    }
    if (tid < T)
        a.st.buf_G[ru(f + tid)] = GcTid;
    if (h % r == 0 && wave == 0 && lm < T) {   // lanes holding k rows store them
        bf16_t *kw = static_cast<bf16_t *>(a.st.buf_k) + rk(f + lm) * D + 8 * lq;
#pragma unroll
        for (int st = 0; st < 4; ++st)
            *reinterpret_cast<uint4 *>(kw + 32 * st) = wa[st];
    }
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
struct CompactArgs {
    Store st;
    const int32_t *slot;
    const int32_t *path;
    const int32_t *path_len;
    int32_t Hk, Hv, cap, T;
};

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
// host side
// ---------------------------------------------------------------------------
thread_local hipError_t g_last_hip_error = hipSuccess;
thread_local kvb_timer *g_armed = nullptr;

bool aligned(const void *p, size_t n) { return (reinterpret_cast<uintptr_t>(p) % n) == 0; }

int check_common(const kvb_shape *sh, const kvb_store *st, const int32_t *slot)
{
    if (!sh || !st || !slot)
        return KVB_EINVAL;
    if (sh->B < 0 || sh->Hk <= 0 || sh->Hv <= 0 || sh->Hv % sh->Hk != 0)
        return KVB_EINVAL;
    if (sh->dk <= 0 || sh->dv <= 0)
        return KVB_EINVAL;
    if (sh->cap < 1 || sh->cap > KVB_MAX_CAP)
        return KVB_EINVAL;
    if (st->n_slots <= 0 || !st->buf_k || !st->buf_u || !st->buf_G || !st->fill)
        return KVB_EINVAL;
    if (st->block_table) {   // paged record buffers
        const int bs = st->block_size;
        if (bs < 8 || bs > KVB_MAX_CAP || (bs & (bs - 1)) != 0)
            return KVB_EINVAL;
        if (st->max_blocks < 1 || st->max_blocks > KVB_MAX_BLOCKS || st->n_blocks < 1)
            return KVB_EINVAL;
        if ((long long)bs * st->max_blocks < sh->cap || !aligned(st->block_table, 4))
            return KVB_EINVAL;
    }
    if (!aligned(st->state, 16) || !aligned(st->buf_k, 16) || !aligned(st->buf_u, 16) ||
        !aligned(st->buf_G, 4) || !aligned(st->fill, 4) || !aligned(st->status, 4) || !aligned(slot, 4))
        return KVB_EINVAL;
    if ((long long)sh->B * sh->Hv > 0x7FFFFFFFLL)
        return KVB_EINVAL;
    if (sh->in_dtype != KVB_F32 && sh->in_dtype != KVB_BF16)
        return KVB_EUNSUPPORTED;
    if (sh->out_dtype != KVB_F32)
        return KVB_EUNSUPPORTED;
    if (sh->dk != sh->dv || (sh->dk != 32 && sh->dk != 64 && sh->dk != 128))
        return KVB_EUNSUPPORTED;
    return KVB_OK;
}

int check_tokens(const void *q, const void *k, const void *v, const float *g, const float *beta, const void *out)
{
    if (!q || !k || !v || !g || !beta || !out)
        return KVB_EINVAL;
    if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(out, 16) || !aligned(g, 4) ||
        !aligned(beta, 4))
        return KVB_EINVAL;
    return KVB_OK;
}

// Whether the state should be streamed past the caches: the caller's hint, else by this
// call's own state footprint against the 256 MB last-level cache.
bool stream_state(const kvb_shape *sh, const kvb_store *st)
{
    if (st->flags & KVB_STORE_STREAM)
        return true;
    if (st->flags & KVB_STORE_RESIDENT)
        return false;
    const double bytes = 4.0 * sh->B * sh->Hv * sh->dk * sh->dv;
    return bytes > 384.0 * 1024 * 1024;
}

Store dev_store(const kvb_store *st)
{
    return Store{st->state, st->buf_k, st->buf_u, st->buf_G, st->fill, st->status, st->n_slots,
                 st->block_table, st->block_table ? st->block_size : 0, st->block_table ? st->max_blocks : 1,
                 st->block_table ? st->n_blocks : 0};
}

int finish_launch()
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        g_last_hip_error = e;
        return KVB_EHIP;
    }
    return KVB_OK;
}

// One kernel launch.  If this thread armed a timer, the launch carries its two events so
// that they hold the kernel's own begin / end timestamps.
template <typename Args>
void launch(void (*kernel)(Args), int blocks, hipStream_t stream, const Args &a)
{
    kvb_timer *t = g_armed;
    g_armed = nullptr;
    if (t)
        hipExtLaunchKernelGGL(kernel, dim3(blocks), dim3(NT), 0, stream, t->start, t->stop, 0, a);
    else
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(NT), 0, stream, a);
}

// Picks the paged or the contiguous instance of a kernel template whose last parameter is PAGED;
// the arguments after `a` are the kernel's name and its leading template arguments.
#define LAUNCH_PAGED(blocks, stream, a, ...)                          \
    do {                                                              \
        if ((a).st.block_table)                                       \
            launch(__VA_ARGS__, true>, blocks, stream, a);            \
        else                                                          \
            launch(__VA_ARGS__, false>, blocks, stream, a);           \
    } while (0)

template <int D, typename TIn, int TM, int WREC>
void launch_step_s(const StepArgs &a, int blocks, hipStream_t stream)
{
    // (a branch inside the kernel around the state loads would make the compiler's wait
    // counters conservative at the join, so these are compile-time variants)
    const bool st = a.stream_state != 0;
    if constexpr (TM == 1) {
        if (a.threshold > 0) {
            if (st)
                LAUNCH_PAGED(blocks, stream, a, kvb_step_kernel<D, TIn, 1, WREC, true, true, true);
            else
                LAUNCH_PAGED(blocks, stream, a, kvb_step_kernel<D, TIn, 1, WREC, true, true, false);
            return;
        }
    }
    if (!a.st.state)
        LAUNCH_PAGED(blocks, stream, a, kvb_step_kernel<D, TIn, TM, WREC, false, false, false);
    else if (st)
        LAUNCH_PAGED(blocks, stream, a, kvb_step_kernel<D, TIn, TM, WREC, true, false, true);
    else
        LAUNCH_PAGED(blocks, stream, a, kvb_step_kernel<D, TIn, TM, WREC, true, false, false);
}

template <int D, typename TIn, int TM>
void launch_step_w(const StepArgs &a, int blocks, hipStream_t stream)
{
    // Register window of buffered records.  For d = 128 the smallest tier that holds the
    // whole buffer is used; the smaller head sizes only carry the general (64 + tail) tier.
    if (D == 128 && a.cap <= 16)
        launch_step_s<D, TIn, TM, D == 128 ? 16 : 64>(a, blocks, stream);
    else if (D == 128 && a.cap <= 32)
        launch_step_s<D, TIn, TM, D == 128 ? 32 : 64>(a, blocks, stream);
    else
        launch_step_s<D, TIn, TM, 64>(a, blocks, stream);
}

template <int WREC>
void launch_verify_mfma(const StepArgs &a, int blocks, hipStream_t stream)
{
    if (!a.st.state)
        LAUNCH_PAGED(blocks, stream, a, kvb_verify_mfma_kernel<WREC, false, false);
    else if (a.stream_state)
        LAUNCH_PAGED(blocks, stream, a, kvb_verify_mfma_kernel<WREC, true, true);
    else
        LAUNCH_PAGED(blocks, stream, a, kvb_verify_mfma_kernel<WREC, true, false);
}

template <int D, typename TIn>
void launch_step(const StepArgs &a, int blocks, hipStream_t stream)
{
    if constexpr (D == 128 && sizeof(TIn) == 2) {
        if (a.T > 1) {   // several drafts: the matrix-core kernel; a request that fits has fill <= cap - T
            if (a.cap - a.T <= 16)
                launch_verify_mfma<16>(a, blocks, stream);
            else if (a.cap - a.T <= 32)
                launch_verify_mfma<32>(a, blocks, stream);
            else
                launch_verify_mfma<64>(a, blocks, stream);
            return;
        }
    }
    if (a.T == 1)
        launch_step_w<D, TIn, 1>(a, blocks, stream);
    else if (a.T <= 4)
        launch_step_w<D, TIn, 4>(a, blocks, stream);
    else
        launch_step_w<D, TIn, 8>(a, blocks, stream);
}

// Calls f.template operator()<D, TIn>() for the compiled (head size, dtype) pairs.
template <typename F>
int dispatch(const kvb_shape *sh, F &&f)
{
    const bool bf = sh->in_dtype == KVB_BF16;
    switch (sh->dk) {
    case 32:
        bf ? f.template operator()<32, bf16_t>() : f.template operator()<32, float>();
        return KVB_OK;
    case 64:
        bf ? f.template operator()<64, bf16_t>() : f.template operator()<64, float>();
        return KVB_OK;
    case 128:
        bf ? f.template operator()<128, bf16_t>() : f.template operator()<128, float>();
        return KVB_OK;
    }
    return KVB_EUNSUPPORTED;
}

int step_common(const kvb_shape *sh, const kvb_store *st, const int32_t *slot, int T, const void *q,
                const void *k, const void *v, const float *g, const float *beta, void *out, void *stream,
                int advance, int threshold = 0, const int32_t *parent = nullptr)
{
    int rc = check_common(sh, st, slot);
    if (rc != KVB_OK)
        return rc;
    rc = check_tokens(q, k, v, g, beta, out);
    if (rc != KVB_OK)
        return rc;
    if (T < 1 || T > KVB_MAX_DRAFTS || T > sh->cap)
        return KVB_EINVAL;
    if (sh->B == 0)
        return KVB_OK;
    StepArgs a{dev_store(st), slot, q, k, v, g, beta, static_cast<float *>(out), sh->Hk, sh->Hv, sh->cap, T,
               sh->scale, advance, threshold, stream_state(sh, st) ? 1 : 0,
               // chain: g stands in as a readable array of at least B*T words whose values are ignored
               parent ? parent : reinterpret_cast<const int32_t *>(g), parent ? 1 : 0};
    const int blocks = sh->B * sh->Hv;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    rc = dispatch(sh, [&]<int D, typename TIn>() { launch_step<D, TIn>(a, blocks, hs); });
    if (rc != KVB_OK)
        return rc;
    return finish_launch();
}

}  // namespace

extern "C" {

int kvb_decode(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, const void *q, const void *k,
               const void *v, const float *g, const float *beta, void *out, void *stream)
{
    return step_common(shape, store, slot, 1, q, k, v, g, beta, out, stream, 1);
}

int kvb_decode_flush(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, const void *q,
                     const void *k, const void *v, const float *g, const float *beta, void *out,
                     int32_t threshold, void *stream)
{
    if (!shape || !store)
        return KVB_EINVAL;
    if (!store->state || threshold < 1 || threshold > shape->cap)
        return KVB_EINVAL;
    return step_common(shape, store, slot, 1, q, k, v, g, beta, out, stream, 1, threshold);
}

int kvb_verify(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, int32_t T, const void *q,
               const void *k, const void *v, const float *g, const float *beta, void *out, void *stream)
{
    return step_common(shape, store, slot, T, q, k, v, g, beta, out, stream, 0);
}

int kvb_verify_tree(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, int32_t T,
                    const int32_t *parent, const void *q, const void *k, const void *v, const float *g,
                    const float *beta, void *out, void *stream)
{
    if (!parent || !aligned(parent, 4))
        return KVB_EINVAL;
    return step_common(shape, store, slot, T, q, k, v, g, beta, out, stream, 0, 0, parent);
}

int kvb_compact(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, int32_t T,
                const int32_t *path, const int32_t *path_len, void *stream)
{
    int rc = check_common(shape, store, slot);
    if (rc != KVB_OK)
        return rc;
    if (!path || !path_len || !aligned(path, 4) || !aligned(path_len, 4))
        return KVB_EINVAL;
    if (T < 1 || T > KVB_MAX_DRAFTS || T > shape->cap)
        return KVB_EINVAL;
    if (shape->B == 0)
        return KVB_OK;
    CompactArgs a{dev_store(store), slot, path, path_len, shape->Hk, shape->Hv, shape->cap, T};
    const int blocks = shape->B * shape->Hv;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    rc = dispatch(shape, [&]<int D, typename TIn>() { LAUNCH_PAGED(blocks, hs, a, kvb_compact_kernel<D, TIn); });
    if (rc != KVB_OK)
        return rc;
    return finish_launch();
}

int kvb_flush(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, const int32_t *accepted,
              int32_t threshold, void *stream)
{
    int rc = check_common(shape, store, slot);
    if (rc != KVB_OK)
        return rc;
    if (!aligned(accepted, 4))
        return KVB_EINVAL;
    if (!store->state && !accepted)   // nothing to fold into and nothing to commit
        return KVB_EINVAL;
    if (threshold < 1 || threshold > shape->cap)
        return KVB_EINVAL;
    if (shape->B == 0)
        return KVB_OK;
    FlushArgs a{dev_store(store), slot, accepted, shape->Hk, shape->Hv, shape->cap, threshold};
    const int blocks = shape->B * shape->Hv;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    rc = dispatch(shape, [&]<int D, typename TIn>() {
        LAUNCH_PAGED(blocks, hs, a, kvb_flush_kernel<D, TIn);
    });
    if (rc != KVB_OK)
        return rc;
    return finish_launch();
}

int kvb_direct(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, const int32_t *len,
               int32_t Lmax, const void *q, const void *k, const void *v, const float *g, const float *beta,
               void *out, void *stream)
{
    int rc = check_common(shape, store, slot);
    if (rc != KVB_OK)
        return rc;
    rc = check_tokens(q, k, v, g, beta, out);
    if (rc != KVB_OK)
        return rc;
    if (!len || !aligned(len, 4))
        return KVB_EINVAL;
    if (Lmax < 1 || Lmax > shape->cap || Lmax > KVB_MAX_DIRECT_LEN)
        return KVB_EINVAL;
    if (shape->B == 0)
        return KVB_OK;
    DirectArgs a{dev_store(store), slot, len, q, k, v, g, beta, static_cast<float *>(out), shape->Hk, shape->Hv,
                 shape->cap, Lmax, shape->scale};
    const int blocks = shape->B * shape->Hv;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    if (shape->dk == 128 && shape->in_dtype == KVB_BF16) {
        if (a.st.block_table)
            launch(kvb_direct_mfma_kernel<true>, blocks, hs, a);
        else
            launch(kvb_direct_mfma_kernel<false>, blocks, hs, a);
        return finish_launch();
    }
    rc = dispatch(shape, [&]<int D, typename TIn>() {
        LAUNCH_PAGED(blocks, hs, a, kvb_direct_kernel<D, TIn);
    });
    if (rc != KVB_OK)
        return rc;
    return finish_launch();
}

int kvb_timer_create(kvb_timer **timer)
{
    if (!timer)
        return KVB_EINVAL;
    kvb_timer *t = new kvb_timer{nullptr, nullptr};
    hipError_t e = hipEventCreate(&t->start);
    if (e == hipSuccess)
        e = hipEventCreate(&t->stop);
    if (e != hipSuccess) {
        g_last_hip_error = e;
        if (t->start)
            (void)hipEventDestroy(t->start);
        delete t;
        return KVB_EHIP;
    }
    *timer = t;
    return KVB_OK;
}

int kvb_timer_arm(kvb_timer *timer)
{
    g_armed = timer;
    return KVB_OK;
}

int kvb_timer_read(kvb_timer *timer, float *microseconds)
{
    if (!timer || !microseconds)
        return KVB_EINVAL;
    hipError_t e = hipEventSynchronize(timer->stop);
    float ms = 0.0f;
    if (e == hipSuccess)
        e = hipEventElapsedTime(&ms, timer->start, timer->stop);
    if (e != hipSuccess) {
        g_last_hip_error = e;
        return KVB_EHIP;
    }
    *microseconds = ms * 1000.0f;
    return KVB_OK;
}

void kvb_timer_destroy(kvb_timer *timer)
{
    if (!timer)
        return;
    if (g_armed == timer)
        g_armed = nullptr;
    (void)hipEventDestroy(timer->start);
    (void)hipEventDestroy(timer->stop);
    delete timer;
}

const char *kvb_strerror(int code)
{
    switch (code) {
    case KVB_OK:
        return "ok";
    case KVB_EINVAL:
        return "invalid argument (null or misaligned pointer, or a size out of range)";
    case KVB_EUNSUPPORTED:
        return "unsupported head size or dtype";
    case KVB_EHIP:
        return hipGetErrorString(g_last_hip_error);
    }
    return "unknown kvb error code";
}

int kvb_version(void) { return KVB_VERSION; }

}  // extern "C"
