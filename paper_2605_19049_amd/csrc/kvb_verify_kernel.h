// kvb_verify_mfma_kernel: kvb_verify / kvb_verify_tree for 16-bit inputs and d = 128.  Template code
// only; kvb_verify_bf16.hip and kvb_verify_f16.hip instantiate it for their input type.
#ifndef KVB_VERIFY_KERNEL_H
#define KVB_VERIFY_KERNEL_H

#include "kvb_device.h"

namespace kvb_impl {

// ---------------------------------------------------------------------------
// kvb_verify for 16-bit inputs (bf16 or fp16) and d = 128, on the matrix cores.
//
// With T drafts the step is a pair of small dense contractions (Sec. 3.3, Eq. 7; Eq. 15):
//   stage 1   C1[m][l] = W[m] . k_l        W = [k_0..k_7 ; q_0..q_7] (16 x dk, 16-bit),
//             l over the buffered and the new keys  -> v_mfma_f32_16x16x32_{bf16,f16}
//   stage 2   acc[m][:] = sum_rows sW[row][m] S0[row][:] + sum_{l<f} cW[l][m] u_l[:]
//             (16 x (dk + f)) . ((dk + f) x dv), fp32 operands -> v_mfma_f32_16x16x4_f32
// where sW[row][m] = -gamma_i k_i[row] (m = i) or gamma_i q_i[row] (m = 8 + i) and
// cW[l][m] = -/+ Gamma_il C1[m][l].  The cost of stage 2 does not depend on T <= 8.
// Each wave owns 32 dv columns for all rows, so no reduction across waves is needed; a
// lane loads 2 adjacent columns of 4 consecutive rows' worth of lanes (16 lanes x 8 B =
// one 128-byte line per row).  MFMA layouts: see kvb_direct_mfma_kernel; for 16x16x4 fp32
// lane l supplies A[l%16][l/16] and B[l/16][l%16] and receives C[4*(l/16)+v][l%16].
// ---------------------------------------------------------------------------
template <typename TIn, typename TRec, int WREC, bool HAS_STATE, bool STREAM, bool PAGED>
// (register budgets: 4 waves per SIMD with a record window of 16 or 32, 3 with the 64-record window)
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(!HAS_STATE ? 1 : WREC <= 32 ? 4 : 3)))
void kvb_verify_mfma_kernel(const int32_t *slot_arg, int32_t Hv_arg, int32_t nblocks_arg, const StepArgs a)
{
    // (the three leading arguments repeat a.slot, a.Hv and the grid size: preloaded into scalar registers
    // at wave launch, so that the load of slot[b] does not wait for the fetch of the argument block)
    constexpr int D = 128;
    constexpr int TMX = KVB_MAX_DRAFTS;                       // 8
    constexpr int NTILE = (KVB_MAX_CAP + TMX + 15) / 16;      // key tiles of 16 (9)
    constexpr int NTW = ((WREC + TMX + 15) / 16 + NW - 1) / NW;  // tiles per wave held in registers
    constexpr int WQ = WREC / 4;                              // record quads held in registers
    constexpr bool TAIL = WREC >= 64;
    constexpr bool EARLY = HAS_STATE;   // state loads issued before the fill is known
    static_assert(TMX == 8, "row m of W is draft m % 8");

    __shared__ __attribute__((aligned(16))) float sW[D][16];
    __shared__ __attribute__((aligned(16))) float cW[NTILE * 16][16];
    __shared__ __attribute__((aligned(16))) float fin[16][D];
    __shared__ int sBlk[NW][MAX_BLOCKS];
    __shared__ float sGc[TAIL ? NW : 1][TMX];   // per-wave table for the keys beyond the register window

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64;   // (a scalar)
    const int lb = logical_block(nblocks_arg);
    const int b = lb / Hv_arg;
    const int s = slot_arg[b];
    __builtin_amdgcn_sched_barrier(0);   // nothing that needs the argument block goes above this load
    const int h = lb % Hv_arg;
    const int r = a.Hv / a.Hk;
    const int hk = h / r;
    const int T = a.T;
    const int cap = a.cap;

    if (s < 0 || s >= a.st.n_slots)
        return;
    const size_t unit = (size_t)s * a.Hv + h;
    const TIn *qin = static_cast<const TIn *>(a.q);
    const TIn *kin = static_cast<const TIn *>(a.k);
    const TIn *vin = static_cast<const TIn *>(a.v);
    const float *Gbuf = a.st.buf_G;                          // record l of this head: Gbuf[ru(l)]
    const TIn *kb = static_cast<const TIn *>(a.st.buf_k);    //                        kb + rk(l) * D
    const TRec *ub = static_cast<const TRec *>(a.st.buf_u);  //                        ub + ru(l) * D
    const Out<TIn> out{a.out, a.out_wide != 0};
    const int blk_id = load_block_id<PAGED>(a.st, s, lane);

    const int lm = lane % 16, lq = lane / 16;   // MFMA row/column index and k index of this lane
    const int col2 = 32 * wave + 2 * lm;

    // ---- 1. loads that need only the request index: raw bits, clamped addresses, no branches
    // row lm of W (draft lm % 8; k for lm < 8, q above), k-chunk lq of each 32-wide step
    const int wi = min(lm % 8, T - 1);
    const TIn *wrow = (lm < 8 ? kin : qin) + (((size_t)b * T + wi) * a.Hk + hk) * D + 8 * lq;
    uint4 wa[4];
#pragma unroll
    for (int st = 0; st < 4; ++st)
        wa[st] = *reinterpret_cast<const uint4 *>(wrow + 32 * st);

    // ---- 2. the state: rows 4 st + lq, the wave's 32 columns -----------------
    // EARLY: the state's address needs the slot only, so its loads go out before the fill is
    // known and before the long scalar prologue; the records follow and are consumed after the
    // state (the decay gamma_i of row i is then applied to the finished sum over state rows).
    // State row-quads in flight per wave.  EARLY keeps half of the tile in registers and refills a
    // register pair as soon as its quad has gone through the matrix cores: 32 registers less, which
    // is what lets a fourth workgroup onto each CU (the kernel is bound by how well its waves hide
    // each other's waits, not by bytes in flight).
    constexpr int WIN = EARLY ? 16 : D / 4;
    float2 sreg[WIN];
    const float *sp = a.st.state + (HAS_STATE ? unit * D * D + col2 : 0);
    auto load_quad = [&](int st) {
        const float2 *p = reinterpret_cast<const float2 *>(sp + (size_t)(4 * st + lq) * D);
        if constexpr (STREAM) {
            typedef float v2f __attribute__((ext_vector_type(2)));
            const v2f t = __builtin_nontemporal_load(reinterpret_cast<const v2f *>(p));
            return make_float2(t.x, t.y);
        } else {
            return *p;
        }
    };
    auto issue_state = [&]() {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int st = 0; st < WIN; ++st) {
            sreg[st] = load_quad(st);
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
        const TIn *kp = n < f ? kb + rk(n) * D
                              : kin + (((size_t)b * T + min(max(n - f, 0), T - 1)) * a.Hk + hk) * D;
        Gn[x] = Gbuf[ru(n < f ? n : 0)];
#pragma unroll
        for (int st = 0; st < 4; ++st)
            kt[x][st] = *reinterpret_cast<const uint4 *>(kp + 8 * lq + 32 * st);
    }
    // buffered delta values: quad sq = records 4 sq .. 4 sq + 3, this lane: record 4 sq + lq,
    // columns 32 wave + 2 lm, + 1
    Raw2<TRec> uq[WQ];
#pragma unroll
    for (int sq = 0; sq < WQ; ++sq) {
        const int l = 4 * sq + lq;
        uq[sq] = load_raw2(ub + ru(l < f ? l : 0) * D + col2);
    }
    // v of this wave's columns (used by lanes 0..31 in the last stage)
    const int colf = 32 * wave + lane % 32;
    TIn v_raw[TMX];
#pragma unroll
    for (int i = 0; i < TMX; ++i)
        v_raw[i] = vin[(((size_t)b * T + min(i, T - 1)) * a.Hv + h) * D + colf];
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
        unpack8(Raw8<TIn>{wa[0]}, x);
#pragma unroll
        for (int st = 1; st < 4; ++st) {
            float y[8];
            unpack8(Raw8<TIn>{wa[st]}, y);
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
            const float2 sv = sreg[st % WIN];
            acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(aw, sv.x, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(aw, sv.y, acc1, 0, 0, 0);
            if (st + WIN < D / 4) {   // the freed registers take the quad WIN further on
                __builtin_amdgcn_sched_barrier(0);
                sreg[st % WIN] = load_quad(st + WIN);
                __builtin_amdgcn_sched_barrier(0);
            }
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
            c1 = mfma16x32<TIn>(wa[st], kk[st], c1);
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
        const TIn *kp = n < f ? kb + rk(min(n, cap - 1)) * D
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
            const float2 uv = unpack2r(uq[sq]);
            acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(aw, ok ? uv.x : 0.0f, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(aw, ok ? uv.y : 0.0f, acc1, 0, 0, 0);
        }
    }
    // records beyond the register window: four quads to a round trip (requested together, clamped)
    for (int s0 = WQ; TAIL && s0 < nquad; s0 += 4) {
        Raw2<TRec> u4r[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int l = 4 * (s0 + j) + lq;
            u4r[j] = load_raw2(ub + ru(l < f ? l : 0) * D + col2);
        }
        float2 u4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            u4[j] = unpack2r(u4r[j]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int l = 4 * (s0 + j) + lq;   // < 4 * 35 + 4 = 144 rows of cW
            if (s0 + j < nquad) {   // uniform
                const float aw = cW[l][lm];
                acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(aw, l < f ? u4[j].x : 0.0f, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(aw, l < f ? u4[j].y : 0.0f, acc1, 0, 0, 0);
            }
        }
    }
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
                // the record as it will be stored is what every later use reads
                const float ui = rounded_to<TRec>(bet[i] * acc);
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
        if (is_u)   // (already rounded to the record type: the conversion is exact)
            store4(static_cast<TRec *>(a.st.buf_u) + ru(f + i) * D + 4 * c4, val);
        else
            out.put4((((size_t)b * T + i) * a.Hv + h) * D + 4 * c4, val);
    }
    if (tid < T)
        a.st.buf_G[ru(f + tid)] = GcTid;
    if (h % r == 0 && wave == 0 && lm < T) {   // lanes holding k rows store them
        TIn *kw = static_cast<TIn *>(a.st.buf_k) + rk(f + lm) * D + 8 * lq;
#pragma unroll
        for (int st = 0; st < 4; ++st)
            *reinterpret_cast<uint4 *>(kw + 32 * st) = wa[st];
    }
}

// ---------------------------------------------------------------------------
// launch
// ---------------------------------------------------------------------------
template <typename TIn, typename TRec, int WREC>
void launch_verify_w(const StepArgs &a, int blocks, hipStream_t stream)
{
    if (!a.st.state)
        LAUNCH_LEAD(blocks, stream, a, kvb_verify_mfma_kernel<TIn, TRec, WREC, false, false);
    else if (a.stream_state)
        LAUNCH_LEAD(blocks, stream, a, kvb_verify_mfma_kernel<TIn, TRec, WREC, true, true);
    else
        LAUNCH_LEAD(blocks, stream, a, kvb_verify_mfma_kernel<TIn, TRec, WREC, true, false);
}

template <typename TIn, typename TRec>
void launch_verify_typed(const StepArgs &a, int blocks, hipStream_t stream)
{
    // record window: a request that fits has fill <= cap - T
    if (a.cap - a.T <= 16)
        launch_verify_w<TIn, TRec, 16>(a, blocks, stream);
    else if (a.cap - a.T <= 32)
        launch_verify_w<TIn, TRec, 32>(a, blocks, stream);
    else
        launch_verify_w<TIn, TRec, 64>(a, blocks, stream);
}

}  // namespace kvb_impl
#endif  // KVB_VERIFY_KERNEL_H
