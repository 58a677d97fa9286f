// kvb_step_kernel: kvb_decode, kvb_decode_flush and the vector-ALU kvb_verify / kvb_verify_tree, with its
// launch helpers.  Template code only; kvb_step_bf16.hip and kvb_step_f32.hip instantiate it for their
// input type (two translation units, so that they compile side by side).
#ifndef KVB_STEP_KERNEL_H
#define KVB_STEP_KERNEL_H

#include "kvb_device.h"

namespace kvb_impl {

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
template <int D, typename TIn, typename TRec, int TM, int WREC, bool HAS_STATE, bool FUSE, bool STREAM, bool PAGED>
// (register budget: the 64-record decode variants sit at the edge of three workgroups per CU; hold them there)
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(TM == 1 && WREC == 64 && HAS_STATE ? 3 : 1)))
void kvb_step_kernel(const int32_t *slot_arg, int32_t Hv_arg, int32_t nblocks_arg,
                                                      const StepArgs a)
{
    // The three leading arguments repeat a.slot, a.Hv and the grid size: as plain leading kernel
    // arguments they are preloaded into scalar registers at wave launch (the build asks for it), so
    // the load of slot[b] -- the head of the dependent chain to the first state byte -- goes out at
    // once instead of after the round trip that fetches the argument block.
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
    const int lb = logical_block(nblocks_arg);
    const int b = lb / Hv_arg;
    const int s = slot_arg[b];
    __builtin_amdgcn_sched_barrier(0);   // nothing that needs the argument block goes above this load
    const int h = lb % Hv_arg;
    const int r = a.Hv / a.Hk;
    const int hk = h / r;
    const int T = TM == 1 ? 1 : a.T;
    const int cap = a.cap;
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
    const TRec *ub = static_cast<const TRec *>(a.st.buf_u);      //                        ub + ru(l) * D
    const Out<TIn> out{a.out, a.out_wide != 0};
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
    Raw4<TRec> ur_raw[UP];
#pragma unroll
    for (int j = 0; j < UP; ++j) {
        const int l = rg + RPP * j;
        ur_raw[j] = load_raw4(ub + ru(l < f ? l : 0) * D + 4 * c4);
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
        if constexpr (TAIL) {
            // records beyond the register window: all their passes are requested together (clamped,
            // no branch around the loads), so a long buffer costs one more round trip, not one per pass
            constexpr int KT = (KVB_MAX_CAP - KP * NG + NG - 1) / NG;
            if (f > KP * NG) {   // uniform
                Raw8<TIn> kt_raw[KT];
                float Gt[KT];
#pragma unroll
                for (int x = 0; x < KT; ++x) {
                    const int l = (KP + x) * NG + grp;
                    const int lc = l < f ? l : 0;
                    kt_raw[x] = load_raw8(kb + rk(lc) * D + 8 * sub);
                    Gt[x] = Gbuf[ru(lc)];
                }
#pragma unroll
                for (int x = 0; x < KT; ++x) {
                    const int l = (KP + x) * NG + grp;
                    if ((KP + x) * NG < f) {   // uniform
                        float kx[8];
                        unpack8(kt_raw[x], kx);
                        float dkk = 0.0f, dq = 0.0f;
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            dkk = fmaf(kx[e], k8[e], dkk);
                            dq = fmaf(kx[e], q8[e], dq);
                        }
                        dkk = group_sum<GL>(dkk);
                        dq = group_sum<GL>(dq);
                        if (sub == 0 && l < f) {
                            const float w = expf(Gc[0] - Gt[x]);
                            cK[0][l] = w * dkk;
                            cQ[0][l] = w * dq;
                        }
                    }
                }
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
    float4 ur[UP];
#pragma unroll
    for (int j = 0; j < UP; ++j) {
        const int l = rg + RPP * j;
        ur[j] = unpack4(ur_raw[j]);
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
    if constexpr (TAIL) {
        // delta values beyond the register window, four passes to a round trip
        constexpr int UT = (KVB_MAX_CAP - UP * RPP + RPP - 1) / RPP;
#pragma unroll
        for (int x0 = 0; x0 < UT; x0 += 4) {
            if ((UP + x0) * RPP < f) {   // uniform
                Raw4<TRec> ut_raw[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int l = (UP + x0 + j) * RPP + rg;
                    ut_raw[j] = load_raw4(ub + ru(l < f ? l : 0) * D + 4 * c4);
                }
                float4 ut[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    ut[j] = unpack4(ut_raw[j]);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int l = (UP + x0 + j) * RPP + rg;
                    if (x0 + j < UT && l < f) {
#pragma unroll
                        for (int i = 0; i < TM; ++i) {
                            if (i < T) {
                                fma4(accU[i], -cK[i][l], ut[j]);
                                fma4(accO[i], cQ[i][l], ut[j]);
                            }
                        }
                    }
                }
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
                // the record as it is stored is what every later use reads, this token's output included
                const TRec ur_i = from_f32<TRec>(bet[i] * acc);
                const float ui = to_f32(ur_i);
#pragma unroll
                for (int j = 0; j < TM; ++j)
                    if (j < i)
                        ao = fmaf(cQ[i][f + j], uprev[j], ao);
                ao = fmaf(cQ[i][f + i], ui, ao);
                uprev[i] = ui;
                u_new = ui;
                out.put1(row * D + tid, a.scale * ao);
                static_cast<TRec *>(a.st.buf_u)[ru(f + i) * D + tid] = ur_i;
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
            if constexpr (NG == LT) {
              if (l_done < m) {   // uniform
                // records before f come back from memory (written by earlier calls): thread (grp, sub)
                // brings 8 elements of record l0 + grp, and the next tile is requested before this
                // one is applied, so its round trip hides under the multiply-adds
                const int lmax = f > 0 ? f - 1 : 0;   // requests are clamped; rows >= f are not used
                int lr = min(l_done + grp, lmax);
                size_t rowr = ru(lr);
                Raw8<TIn> kq = load_raw8(kb + rk(lr) * D + 8 * sub);
                Raw8<TRec> uq = load_raw8(ub + rowr * D + 8 * sub);
                float Gq = Gbuf[rowr];
                for (int l0 = l_done; l0 < m; l0 += LT) {
                    __syncthreads();
                    const int l = l0 + grp;
                    if (l != f) {   // row f of the tile belongs to inject_new
                        float kx[8];
                        unpack8(kq, kx);
                        const float w = l < f ? expf(Gc[0] - Gq) : 0.0f;
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            kh[grp][8 * sub + e] = l < f ? w * kx[e] : 0.0f;
                        // (component by component: a select between two float4 objects is compiled
                        // as a select between their addresses, which puts them in scratch memory)
                        const bool in = l < f;
                        float ux[8];
                        unpack8(uq, ux);
                        *reinterpret_cast<float4 *>(&uu[grp][8 * sub]) = make_float4(
                            in ? ux[0] : 0.0f, in ? ux[1] : 0.0f, in ? ux[2] : 0.0f, in ? ux[3] : 0.0f);
                        *reinterpret_cast<float4 *>(&uu[grp][8 * sub + 4]) = make_float4(
                            in ? ux[4] : 0.0f, in ? ux[5] : 0.0f, in ? ux[6] : 0.0f, in ? ux[7] : 0.0f);
                    }
                    inject_new(l0);
                    // (the request past the last tile re-reads a valid record and is dropped)
                    lr = min(l0 + LT + grp, lmax);
                    rowr = ru(lr);
                    kq = load_raw8(kb + rk(lr) * D + 8 * sub);
                    uq = load_raw8(ub + rowr * D + 8 * sub);
                    Gq = Gbuf[rowr];
                    __syncthreads();
                    apply_tile(l0);
                }
              }
            } else {
                for (int l0 = l_done; l0 < m; l0 += LT) {
                    __syncthreads();
                    // records before f come back from memory (written by earlier calls)
#pragma unroll
                    for (int x = 0; x < EPT; ++x) {
                        const int idx = tid + NT * x, l = l0 + idx / D, e = idx % D;
                        if (l < f) {
                            kh[idx / D][e] = expf(Gc[0] - Gbuf[ru(l)]) * to_f32(kb[rk(l) * D + e]);
                            uu[idx / D][e] = to_f32(ub[ru(l) * D + e]);
                        } else if (l > f) {
                            kh[idx / D][e] = 0.0f;
                            uu[idx / D][e] = 0.0f;
                        }
                    }
                    inject_new(l0);
                    __syncthreads();
                    apply_tile(l0);
                }
            }
            float4 *sw = reinterpret_cast<float4 *>(a.st.state + unit * D * D);
#pragma unroll
            for (int p = 0; p < NPASS; ++p) {
                if constexpr (STREAM) {   // a state that is streamed in is streamed out again (+1 % on 1 GiB of state)
                    typedef float v4f __attribute__((ext_vector_type(4)));
                    __builtin_nontemporal_store(v4f{sreg[p].x, sreg[p].y, sreg[p].z, sreg[p].w},
                                                reinterpret_cast<v4f *>(sw + (size_t)(rg + RPP * p) * LPR + c4));
                } else {
                    sw[(size_t)(rg + RPP * p) * LPR + c4] = sreg[p];
                }
            }
            new_fill = 0;
        }
    }
    if (a.advance && tid == 0)
        publish_if_last(&a.st.fill[s], ticket, a.Hv, new_fill);
}

// ---------------------------------------------------------------------------
// launch
// ---------------------------------------------------------------------------
template <int D, typename TIn, typename TRec, int TM, int WREC>
void launch_step_s(const StepArgs &a, int blocks, hipStream_t stream)
{
    // (a branch inside the kernel around the state loads would make the compiler's wait
    // counters conservative at the join, so these are compile-time variants)
    const bool st = a.stream_state != 0 && D == 128;   // the small head sizes are not tuned: no streaming variant
    if constexpr (TM == 1) {
        if (a.threshold > 0) {
            if constexpr (D == 128) {
                if (st) {
                    LAUNCH_LEAD(blocks, stream, a, kvb_step_kernel<D, TIn, TRec, 1, WREC, true, true, true);
                    return;
                }
            }
            LAUNCH_LEAD(blocks, stream, a, kvb_step_kernel<D, TIn, TRec, 1, WREC, true, true, false);
            return;
        }
    }
    if (!a.st.state) {
        LAUNCH_LEAD(blocks, stream, a, kvb_step_kernel<D, TIn, TRec, TM, WREC, false, false, false);
        return;
    }
    if constexpr (D == 128) {
        if (st) {
            LAUNCH_LEAD(blocks, stream, a, kvb_step_kernel<D, TIn, TRec, TM, WREC, true, false, true);
            return;
        }
    }
    LAUNCH_LEAD(blocks, stream, a, kvb_step_kernel<D, TIn, TRec, TM, WREC, true, false, false);
}

template <int D, typename TIn, typename TRec, int TM>
void launch_step_w(const StepArgs &a, int blocks, hipStream_t stream)
{
    // Register window of buffered records.  For d = 128 the smallest tier that holds the
    // whole buffer is used; the smaller head sizes only carry the general (64 + tail) tier.
    if constexpr (D == 128) {
        if (a.cap <= 16) {
            launch_step_s<D, TIn, TRec, TM, 16>(a, blocks, stream);
            return;
        }
        if (a.cap <= 32) {
            launch_step_s<D, TIn, TRec, TM, 32>(a, blocks, stream);
            return;
        }
    }
    launch_step_s<D, TIn, TRec, TM, 64>(a, blocks, stream);
}

template <int D, typename TIn, typename TRec>
void launch_step_t(const StepArgs &a, int blocks, hipStream_t stream)
{
    if (a.T == 1) {
        launch_step_w<D, TIn, TRec, 1>(a, blocks, stream);
        return;
    }
    // several drafts with 16-bit inputs and d = 128 belong to kvb_verify_mfma_kernel; the
    // vector-ALU variants are not compiled for that pair
    if constexpr (!(D == 128 && sizeof(TIn) == 2)) {
        if (a.T <= 4)
            launch_step_w<D, TIn, TRec, 4>(a, blocks, stream);
        else
            launch_step_w<D, TIn, TRec, 8>(a, blocks, stream);
    }
}

// All head sizes of one (input type, record type) pair.
template <typename TIn, typename TRec>
int launch_step_typed(int dk, const StepArgs &a, int blocks, hipStream_t stream)
{
    switch (dk) {
    case 32:
        launch_step_t<32, TIn, TRec>(a, blocks, stream);
        return KVB_OK;
    case 64:
        launch_step_t<64, TIn, TRec>(a, blocks, stream);
        return KVB_OK;
    case 128:
        launch_step_t<128, TIn, TRec>(a, blocks, stream);
        return KVB_OK;
    }
    return KVB_EUNSUPPORTED;
}

}  // namespace kvb_impl
#endif  // KVB_STEP_KERNEL_H
