// kvb -- KVBuffer-style Gated DeltaNet decoding, HIP kernels for gfx950 and the
// C-ABI entry points declared in include/kvb.h.
//
// Work decomposition (all four calls): one 256-thread workgroup per (request b,
// v-head h).  The committed state S0[dk][dv] (fp32, dv contiguous) is streamed
// once with 16-byte loads: a thread owns 4 adjacent dv columns of the rows
// rg, rg+RPP, rg+2*RPP, ... so a wave's load instruction covers whole
// contiguous rows.  Everything a (b,h) unit needs besides the state -- the
// buffered keys k_l, delta values u_l and cumulative log decays G_l (paper
// App. A.1, the paragraph after Eq. 16) -- is a few KB and is staged through LDS.
//
// Notation follows App. A.1: gamma_i = exp(G_i), Gamma_il = exp(G_i - G_l).

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvb.h"

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
// stores the new plain value.
__device__ __forceinline__ void publish_fill(int32_t *word, int nwg, int new_fill)
{
    const int old = __hip_atomic_fetch_add(word, TICKET_ONE, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    if ((old >> 16) == nwg - 1)
        __hip_atomic_store(word, new_fill, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

struct Store {
    float *state;
    void *buf_k;
    float *buf_u;
    float *buf_G;
    int32_t *fill;
    int32_t *status;
    int32_t n_slots;
};

struct StepArgs {
    Store st;
    const int32_t *slot;
    const void *q, *k, *v;
    const float *g, *beta;
    float *out;
    int32_t Hk, Hv, cap, T;
    float scale;
    int32_t advance;  // 1: decode (fill += T after the step); 0: verify (fill untouched)
};

// ---------------------------------------------------------------------------
// kvb_decode (TM == 1) and kvb_verify (TM >= T): rows f..f+T-1 of the chunkwise
// form, Eq. 15/16.  Per (b,h):
//   accU_i = -gamma_i k_i S0 - sum_{l<f} Gamma_il (k_i.k_l) u_l
//   accO_i =  gamma_i q_i S0 + sum_{l<f} Gamma_il (q_i.k_l) u_l
// are accumulated over state rows and buffered records alike (both are "rows"
// weighted by a per-row scalar), reduced across the workgroup, and the T drafts
// are then finished by forward substitution among themselves.
// ---------------------------------------------------------------------------
template <int D, typename TIn, int TM>
__global__ __launch_bounds__(NT) void kvb_step_kernel(const StepArgs a)
{
    constexpr int LPR = D / 4;       // lanes covering one state row with float4
    constexpr int RPP = NT / LPR;    // rows covered by the workgroup per pass
    constexpr int NPASS = D / RPP;   // rows per thread
    constexpr int GL = D / 8;        // lanes sharing one key dot product (8 elements each)
    constexpr int NG = NT / GL;      // records handled per pass of the dot-product phase
    constexpr int NC = KVB_MAX_CAP + TM;

    __shared__ float sKs[TM][D];     // -gamma_i * k_i   (weights of the state rows for accU)
    __shared__ float sQs[TM][D];     //  gamma_i * q_i
    __shared__ float rK[TM][D];      // raw k_i, q_i
    __shared__ float rQ[TM][D];
    __shared__ float cK[TM][NC];     // Gamma_il (k_i.k_l), 0 for l >= f+i
    __shared__ float cQ[TM][NC];     // Gamma_il (q_i.k_l), 0 for l >  f+i
    __shared__ float red[NW][TM][2][D];

    const int tid = threadIdx.x;
    const int b = blockIdx.x / a.Hv;
    const int h = blockIdx.x % a.Hv;
    const int r = a.Hv / a.Hk;
    const int hk = h / r;
    const int T = a.T;
    const int cap = a.cap;

    const int s = a.slot[b];
    if (s < 0 || s >= a.st.n_slots)
        return;
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

    const int rg = tid / LPR;
    const int c4 = tid % LPR;
    const size_t unit = (size_t)s * a.Hv + h;

    // 1. put the whole state tile in flight
    float4 sreg[NPASS];
    const bool has_state = a.st.state != nullptr;
    if (has_state) {
        const float4 *sp = reinterpret_cast<const float4 *>(a.st.state + unit * D * D);
#pragma unroll
        for (int p = 0; p < NPASS; ++p)
            sreg[p] = sp[(size_t)(rg + RPP * p) * LPR + c4];
    }

    // 2. per-draft scalars and the new q, k rows
    const float *Gbuf = a.st.buf_G + unit * cap;
    float Gc[TM], bet[TM];
    {
        float run = f > 0 ? Gbuf[f - 1] : 0.0f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if (i < T) {
                run += a.g[((size_t)b * T + i) * a.Hv + h];
                bet[i] = a.beta[((size_t)b * T + i) * a.Hv + h];
            } else {
                bet[i] = 0.0f;
            }
            Gc[i] = run;
        }
    }
    const TIn *qin = static_cast<const TIn *>(a.q);
    const TIn *kin = static_cast<const TIn *>(a.k);
    if (tid < D) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if (i < T) {
                const size_t o = (((size_t)b * T + i) * a.Hk + hk) * D + tid;
                const float kv = to_f32(kin[o]);
                const float qv = to_f32(qin[o]);
                const float gam = expf(Gc[i]);
                rK[i][tid] = kv;
                rQ[i][tid] = qv;
                sKs[i][tid] = -gam * kv;
                sQs[i][tid] = gam * qv;
            }
        }
    }
    __syncthreads();

    // 3. decayed dot products of the new rows with every earlier key
    {
        const int grp = tid / GL, sub = tid % GL;
        const int nrec = f + T;
        const TIn *kb = static_cast<const TIn *>(a.st.buf_k) + ((size_t)s * a.Hk + hk) * cap * D;
        for (int base = 0; base < nrec; base += NG) {
            const int l = base + grp;
            if (l < nrec) {
                float kl[8];
                float Gl;
                if (l < f) {
                    load8(kb + (size_t)l * D + 8 * sub, kl);
                    Gl = Gbuf[l];
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        kl[e] = rK[l - f][8 * sub + e];
                    Gl = 0.0f;  // set per draft below
                }
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    if (i < T) {
                        float dkk = 0.0f, dqk = 0.0f;
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            dkk = fmaf(kl[e], rK[i][8 * sub + e], dkk);
                            dqk = fmaf(kl[e], rQ[i][8 * sub + e], dqk);
                        }
#pragma unroll
                        for (int off = 1; off < GL; off <<= 1) {
                            dkk += __shfl_xor(dkk, off);
                            dqk += __shfl_xor(dqk, off);
                        }
                        if (sub == 0) {
                            const int li = f + i;
                            float gl = Gl;
                            if (l >= f) {
                                // G of draft l-f: Gc[] indexed statically
                                gl = 0.0f;
#pragma unroll
                                for (int j = 0; j < TM; ++j)
                                    if (j == l - f)
                                        gl = Gc[j];
                            }
                            const float gam = l <= li ? expf(Gc[i] - gl) : 0.0f;
                            cK[i][l] = l < li ? gam * dkk : 0.0f;
                            cQ[i][l] = gam * dqk;
                        }
                    }
                }
            }
        }
    }
    __syncthreads();

    // 4. accumulate over buffered records and state rows
    float4 accU[TM], accO[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        accU[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        accO[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    {
        const float4 *up = reinterpret_cast<const float4 *>(a.st.buf_u + unit * cap * D);
        for (int l = rg; l < f; l += RPP) {
            const float4 u = up[(size_t)l * LPR + c4];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if (i < T) {
                    fma4(accU[i], -cK[i][l], u);
                    fma4(accO[i], cQ[i][l], u);
                }
            }
        }
    }
    if (has_state) {
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

    // 5. reduce over the row groups: inside the wave by shuffles, across waves via LDS
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

    // 6. finish the T new rows (forward substitution among the drafts), write results
    if (tid < D) {
        const TIn *vin = static_cast<const TIn *>(a.v);
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
                float acc = to_f32(vin[row * D + tid]) + au;
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
                a.out[row * D + tid] = a.scale * ao;
                a.st.buf_u[(unit * cap + f + i) * D + tid] = ui;
            }
        }
    }
    if (tid < T) {
        float gv = 0.0f;
#pragma unroll
        for (int j = 0; j < TM; ++j)
            if (j == tid)
                gv = Gc[j];
        a.st.buf_G[unit * cap + f + tid] = gv;
    }
    if (h % r == 0) {
        TIn *kb = static_cast<TIn *>(a.st.buf_k) + (((size_t)s * a.Hk + hk) * cap + f) * D;
        for (int idx = tid; idx < T * D; idx += NT) {
            const int i = idx / D, e = idx % D;
            kb[(size_t)i * D + e] = kin[(((size_t)b * T + i) * a.Hk + hk) * D + e];
        }
    }
    if (a.advance && tid == 0)
        publish_fill(&a.st.fill[s], a.Hv, f + T);
}

// ---------------------------------------------------------------------------
// kvb_flush: S <- gamma_{m-1} S + sum_{l<m} Gamma_{m-1,l} k_l^T u_l   (Eq. 16, last line)
// ---------------------------------------------------------------------------
struct FlushArgs {
    Store st;
    const int32_t *slot;
    const int32_t *accepted;
    int32_t Hk, Hv, cap, threshold;
};

template <int D, typename TIn>
__global__ __launch_bounds__(NT) void kvb_flush_kernel(const FlushArgs a)
{
    constexpr int LPR = D / 4;
    constexpr int RPP = NT / LPR;
    constexpr int NPASS = D / RPP;
    constexpr int LT = 16;  // records staged per LDS tile

    __shared__ float kh[LT][D];  // Gamma_{m-1,l} k_l
    __shared__ float uu[LT][D];

    const int tid = threadIdx.x;
    const int b = blockIdx.x / a.Hv;
    const int h = blockIdx.x % a.Hv;
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
    const bool do_flush = m >= a.threshold && m > 0;
    if (do_flush) {
        const int rg = tid / LPR, c4 = tid % LPR;
        const size_t unit = (size_t)s * a.Hv + h;
        float4 *sp = reinterpret_cast<float4 *>(a.st.state + unit * D * D);
        float4 sreg[NPASS];
#pragma unroll
        for (int p = 0; p < NPASS; ++p)
            sreg[p] = sp[(size_t)(rg + RPP * p) * LPR + c4];

        const float *Gbuf = a.st.buf_G + unit * cap;
        const float Glast = Gbuf[m - 1];
        const float gam = expf(Glast);
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            sreg[p].x *= gam; sreg[p].y *= gam; sreg[p].z *= gam; sreg[p].w *= gam;
        }
        const TIn *kb = static_cast<const TIn *>(a.st.buf_k) + ((size_t)s * a.Hk + hk) * cap * D;
        const float *ub = a.st.buf_u + unit * cap * D;
        for (int l0 = 0; l0 < m; l0 += LT) {
            const int nl = min(LT, m - l0);
            for (int idx = tid; idx < nl * D; idx += NT) {
                const int l = idx / D, e = idx % D;
                kh[l][e] = expf(Glast - Gbuf[l0 + l]) * to_f32(kb[(size_t)(l0 + l) * D + e]);
                uu[l][e] = ub[(size_t)(l0 + l) * D + e];
            }
            __syncthreads();
            for (int l = 0; l < nl; ++l) {
                const float4 u = *reinterpret_cast<const float4 *>(&uu[l][4 * c4]);
#pragma unroll
                for (int p = 0; p < NPASS; ++p)
                    fma4(sreg[p], kh[l][rg + RPP * p], u);
            }
            __syncthreads();
        }
#pragma unroll
        for (int p = 0; p < NPASS; ++p)
            sp[(size_t)(rg + RPP * p) * LPR + c4] = sreg[p];
    }
    if (tid == 0)
        publish_fill(&a.st.fill[s], a.Hv, do_flush ? 0 : m);
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

template <int D, typename TIn>
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

    const int tid = threadIdx.x;
    const int b = blockIdx.x / a.Hv;
    const int h = blockIdx.x % a.Hv;
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
    const size_t unit = (size_t)s * a.Hv + h;
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
            a.st.buf_u[(unit * a.cap + i) * D + tid] = ui;
        }
    }
    if (tid < L)
        a.st.buf_G[unit * a.cap + tid] = sG[tid];
    if (h % r == 0) {
        TIn *kb = static_cast<TIn *>(a.st.buf_k) + ((size_t)s * a.Hk + hk) * a.cap * D;
        for (int idx = tid; idx < L * D; idx += NT) {
            const int i = idx / D, e = idx % D;
            kb[(size_t)i * D + e] = kin[(((size_t)b * Lmax + i) * a.Hk + hk) * D + e];
        }
    }
    if (h == 0 && tid == 0)
        a.st.fill[s] = L;
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
thread_local hipError_t g_last_hip_error = hipSuccess;

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

Store dev_store(const kvb_store *st)
{
    return Store{st->state, st->buf_k, st->buf_u, st->buf_G, st->fill, st->status, st->n_slots};
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

template <int D, typename TIn>
void launch_step(const StepArgs &a, int blocks, hipStream_t stream)
{
    if (a.T == 1)
        hipLaunchKernelGGL((kvb_step_kernel<D, TIn, 1>), dim3(blocks), dim3(NT), 0, stream, a);
    else if (a.T == 2)
        hipLaunchKernelGGL((kvb_step_kernel<D, TIn, 2>), dim3(blocks), dim3(NT), 0, stream, a);
    else if (a.T <= 4)
        hipLaunchKernelGGL((kvb_step_kernel<D, TIn, 4>), dim3(blocks), dim3(NT), 0, stream, a);
    else
        hipLaunchKernelGGL((kvb_step_kernel<D, TIn, 8>), dim3(blocks), dim3(NT), 0, stream, a);
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
                int advance)
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
               sh->scale, advance};
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

int kvb_verify(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, int32_t T, const void *q,
               const void *k, const void *v, const float *g, const float *beta, void *out, void *stream)
{
    return step_common(shape, store, slot, T, q, k, v, g, beta, out, stream, 0);
}

int kvb_flush(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, const int32_t *accepted,
              int32_t threshold, void *stream)
{
    int rc = check_common(shape, store, slot);
    if (rc != KVB_OK)
        return rc;
    if (!store->state || !aligned(accepted, 4))
        return KVB_EINVAL;
    if (threshold < 1 || threshold > shape->cap)
        return KVB_EINVAL;
    if (shape->B == 0)
        return KVB_OK;
    FlushArgs a{dev_store(store), slot, accepted, shape->Hk, shape->Hv, shape->cap, threshold};
    const int blocks = shape->B * shape->Hv;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    rc = dispatch(shape, [&]<int D, typename TIn>() {
        hipLaunchKernelGGL((kvb_flush_kernel<D, TIn>), dim3(blocks), dim3(NT), 0, hs, a);
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
    rc = dispatch(shape, [&]<int D, typename TIn>() {
        hipLaunchKernelGGL((kvb_direct_kernel<D, TIn>), dim3(blocks), dim3(NT), 0, hs, a);
    });
    if (rc != KVB_OK)
        return rc;
    return finish_launch();
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
