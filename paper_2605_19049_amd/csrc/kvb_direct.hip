// kvb_direct: kvb_direct_mfma_kernel, kvb_direct_mfma_long_kernel (16-bit inputs, d = 128) and kvb_direct_kernel
// (fp32 inputs and the other head sizes).
#include "kvb_device.h"

namespace kvb_impl {

// ---------------------------------------------------------------------------
// kvb_direct: the parallel form, Eq. 13, from a zero state.
//   cK[i][l] = Gamma_il (k_i.k_l) (l < i)     cQ[i][l] = Gamma_il (q_i.k_l) (l <= i)
//   u_i = beta_i ( v_i - sum_{l<i} cK[i][l] u_l )       (row i of A Diag(beta) V)
//   o_i = scale * sum_{l<=i} cQ[i][l] u_l
// ---------------------------------------------------------------------------
template <int D, typename TIn, typename TRec, bool PAGED>
__global__ __launch_bounds__(NT) void kvb_direct_kernel(const DirectArgs a)
{
    constexpr int LM = 64;   // longest context of this kernel
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
    const Out<TIn> out{a.out, a.out_wide != 0};

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
            // the record as it is stored is what every later use reads
            const TRec ur_i = from_f32<TRec>(sB[i] * acc);
            const float ui = to_f32(ur_i);
            sU[i][tid] = ui;
            o = fmaf(cQ[i][i], ui, o);
            out.put1(row * D + tid, a.scale * o);
            static_cast<TRec *>(a.st.buf_u)[ru(i) * D + tid] = ur_i;
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
// kvb_direct for 16-bit inputs (bf16 or fp16) and d = 128, on the matrix cores throughout.
// What the two kernels below share.
//
// The context is cut into blocks of 16 rows.  With N_il = beta_i Gamma_il (k_i.k_l) (l < i)
// and M_il = Gamma_il (q_i.k_l) (l <= i) the parallel form (Eq. 13) is
//     (I + N) U = Diag(beta) V,      O = M U.
// The kernel for up to 128 tokens solves it block row by block row,
//     U_d = T_d ( beta V_d - sum_{e<d} N_de U_e ),      O_d = sum_{e<=d} M_de U_e,
// T_d = (I + N_dd)^-1 by blocked inversion (unit_lower_inverse16 below; N_dd is strictly lower),
// with fp32 operands on v_mfma_f32_16x16x4_f32 (exact products) after the Gram tiles; the
// kernel for up to 64 tokens forms the whole inverse and multiplies (see its own header).
//   * Gram tiles (k.k, q.k over dk = 128, 16-bit operands): v_mfma_f32_16x16x32_{bf16,f16}.
//
// Register chaining.  Call "A-form" of a 16x16 matrix X the register layout in which lane l
// holds X[l%16][4*(l/16)+v], v = 0..3, and "B-form" the one with X[4*(l/16)+v][l%16].  An
// MFMA result is in B-form; feeding four k-steps with (a = xa[v], b = yb[v]) gives the
// B-form of X Y, and swapping the operands, (a = yb[v], b = xa[v]), gives the A-form of X Y.
// A Gram tile computed as (rows of block e) x (rows of block d) lands directly in A-form of
// the (d, e) tile, so no value ever needs to move between lanes: tiles shared between waves
// go through LDS as whole per-lane float4s.  Each wave owns 32 dv columns (two column tiles).
// ---------------------------------------------------------------------------

// B-form of X Y from X in A-form and Y in B-form (swap the arguments for the A-form of X Y).
__device__ __forceinline__ f32x4_t mm16(const f32x4_t &xa, const f32x4_t &yb, f32x4_t acc)
{
#pragma unroll
    for (int v = 0; v < 4; ++v)
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[v], yb[v], acc, 0, 0, 0);
    return acc;
}

// A-form of (I + N)^-1 for a strictly lower triangular 16 x 16 block N given in both forms
// (ia: the identity, which reads the same in both).  Blocked inversion, exact: with the
// diagonal blocks of a 2 x 2 block partition already inverted (T), [[A,0],[C,B]]^-1 =
// T - T C T.  Three levels: 4 x 4 diagonal blocks D0, where (I + D0)^-1 = (I - D0)(I + D0^2)
// since D0^4 = 0; then the 4 x 4 blocks C1 under them inside each 8 x 8; then the lower left
// 8 x 8 block C2.  Every intermediate stays of the size of the inverse itself.  (The plain
// Neumann product (I - N)(I + N^2)(I + N^4)(I + N^8) is also exact in exact arithmetic, but its
// powers grow like binomial coefficients when the keys of a block are strongly correlated, and
// the cancellation then costs four digits.)
__device__ __forceinline__ f32x4_t unit_lower_inverse16(const f32x4_t &na, const f32x4_t &nb, const f32x4_t &ia,
                                                        int c16, int lq)
{
    f32x4_t d0a, d0b, c1a, c2a;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int ai = c16, al = 4 * lq + v;   // A-form: row, column inside the block
        const int bi = al, bl = ai;            // B-form
        d0a[v] = ai / 4 == al / 4 ? na[v] : 0.0f;
        d0b[v] = bi / 4 == bl / 4 ? nb[v] : 0.0f;
        c1a[v] = (ai / 8 == al / 8 && ai / 4 == al / 4 + 1) ? na[v] : 0.0f;
        c2a[v] = (ai >= 8 && al < 8) ? na[v] : 0.0f;
    }
    const f32x4_t z = {0.f, 0.f, 0.f, 0.f};
    const f32x4_t d2b = mm16(d0a, d0b, z);                 // D0^2
    const f32x4_t t0a = mm16(ia + d2b, ia - d0a, z);       // (I - D0)(I + D0^2), A-form
    const f32x4_t t0b = mm16(ia - d0a, ia + d2b, z);       //                     B-form
    const f32x4_t p1b = mm16(c1a, t0b, z);                 // C1 T0
    const f32x4_t t1a = t0a - mm16(p1b, t0a, z);           // T0 - T0 C1 T0
    const f32x4_t t1b = t0b - mm16(t0a, p1b, z);
    const f32x4_t p2b = mm16(c2a, t1b, z);                 // C2 T1
    return t1a - mm16(p2b, t1a, z);                        // T1 - T1 C2 T1
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
template <typename TIn, int GS>
__device__ __forceinline__ f32x4_t gram16(const TIn *arow, const TIn *brow, int lq)
{
    f32x4_t c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int st = 0; st < 4; ++st) {
        const uint4 av = *reinterpret_cast<const uint4 *>(arow + 8 * lq + 32 * st);
        const uint4 bv = *reinterpret_cast<const uint4 *>(brow + 8 * lq + 32 * st);
        c = mfma16x32<TIn>(av, bv, c);
    }
    return c;
}

// ---------------------------------------------------------------------------
// Pieces.  A fp32 value x is cut into NP values of the 16-bit input type, x = x_1 + ... + x_NP
// (+ a remainder below 2^-24 |x| for three bf16 pieces, 2^-22 |x| for two fp16 pieces), each
// the leading bits of what is left, so that a product of two fp32 tiles becomes a few products
// of 16-bit tiles on v_mfma_f32_16x16x32, which runs at 16 times the rate of the fp32 matrix
// instruction.  take_piece handles two values at once and returns their pieces packed in one
// word (first value in the low half); the two arguments become the remainders.
// ---------------------------------------------------------------------------
template <typename T>
constexpr int pieces_of_f32() { return __is_same(T, bf16_t) ? 3 : 2; }

template <typename T>
__device__ __forceinline__ uint32_t take_piece(float &a, float &b)
{
    if constexpr (__is_same(T, bf16_t)) {
        const uint32_t ua = __builtin_bit_cast(uint32_t, a), ub = __builtin_bit_cast(uint32_t, b);
        a -= __builtin_bit_cast(float, ua & 0xFFFF0000u);   // exact
        b -= __builtin_bit_cast(float, ub & 0xFFFF0000u);
        return __builtin_amdgcn_perm(ub, ua, 0x07060302u);   // (ua >> 16) | (ub & 0xFFFF0000)
    } else {
        const f16_t ha = from_f32<f16_t>(a), hb = from_f32<f16_t>(b);
        a -= to_f32(ha);   // exact
        b -= to_f32(hb);
        return (uint32_t)ha.bits | ((uint32_t)hb.bits << 16);
    }
}

// The four values a lane holds of a 16 x 16 tile (either form), cut into NP pieces; piece p is
// two words: values (0, 1) and (2, 3), which is how an operand of the 16-bit matrix instruction
// holds four consecutive contraction indices.
template <typename T, int NP>
__device__ __forceinline__ void split_tile(const f32x4_t &x, uint2 (&p)[NP])
{
    float x0 = x[0], x1 = x[1], x2 = x[2], x3 = x[3];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        p[i].x = take_piece<T>(x0, x1);
        p[i].y = take_piece<T>(x2, x3);
    }
}

// acc += X Y for a 16 x 16 fp32 tile X given as NPX pieces in A-form and a tile Y given as NPY
// pieces in B-form (NPY = 1: Y is exactly representable in the 16-bit type).  One instruction
// contracts over 32 slots; a lane's 8 slots are its 4 contraction indices taken twice, so an
// instruction adds two piece products X_a Y_b + X_c Y_d.  Three instructions give the six
// products down to 2^-16 of the leading one (all that matter for a fp32 result).
template <typename T, int NPX, int NPY>
__device__ __forceinline__ f32x4_t mm16_pieces(const uint2 (&x)[NPX], const uint2 (&y)[NPY], f32x4_t acc)
{
    auto ins = [&](const uint2 &xa, const uint2 &xc, const uint2 &yb, const uint2 &yd) {
        acc = mfma16x32<T>(uint4{xa.x, xa.y, xc.x, xc.y}, uint4{yb.x, yb.y, yd.x, yd.y}, acc);
    };
    const uint2 zero = {0u, 0u};
    if constexpr (NPX == 3 && NPY == 3) {   // smallest terms first
        ins(x[2], x[0], y[0], y[2]);        // X3 Y1 + X1 Y3
        ins(x[1], x[1], y[1], y[0]);        // X2 Y2 + X2 Y1
        ins(x[0], x[0], y[0], y[1]);        // X1 Y1 + X1 Y2
    } else if constexpr (NPX == 3 && NPY == 1) {
        ins(x[2], zero, y[0], y[0]);        // X3 Y
        ins(x[0], x[1], y[0], y[0]);        // X1 Y + X2 Y
    } else if constexpr (NPX == 2 && NPY == 2) {
        ins(x[1], x[1], y[0], y[1]);        // X2 Y1 + X2 Y2
        ins(x[0], x[0], y[0], y[1]);        // X1 Y1 + X1 Y2
    } else {
        static_assert(NPX == 2 && NPY == 1, "piece counts");
        ins(x[0], x[1], y[0], y[0]);        // X1 Y + X2 Y
    }
    return acc;
}

// ---------------------------------------------------------------------------
// kvb_direct for 16-bit inputs, d = 128 and contexts of up to 64 tokens.
//
// With N_il = beta_i Gamma_il (k_i.k_l) (l < i) and M_il = Gamma_il (q_i.k_l) (l <= i) the
// parallel form (Eq. 13) is U = (I + N)^-1 Diag(beta) V, O = M U.  The kernel forms the inverse
// itself, A^ = (I + N)^-1 Diag(beta) (64 x 64, lower triangular, in 16 x 16 tiles), because then
//   * U = A^ V has the values -- exact 16-bit operands -- as its right factor: with A^ cut into
//     pieces the product runs on the 16-bit matrix instruction, one instruction per piece and per
//     two tiles of A^, and no block row waits for another (there is no substitution chain through
//     the 128 columns, which is where the time of a row-by-row solve goes);
//   * O = M U uses M in pieces (cut once, when the tile is weighted) and U in pieces.
// What is left in fp32 (v_mfma_f32_16x16x4_f32, exact products) is the small triangular
// work that produces A^: the four diagonal blocks T_d = (I + N_dd)^-1 (unit_lower_inverse16), and
// two levels of blocked inversion  [[P, 0], [C, R]]^-1 = [[P^-1, 0], [-R^-1 C P^-1, R^-1]]:
//     A_10 = -T_1 N_10 T_0                     A_32 = -T_3 N_32 T_2
//     W = C P^-1:  W_20 = (N_20 - N_21 T_1 N_10) T_0    W_21 = N_21 T_1      (same for row 3)
//     A_20 = -T_2 W_20   A_21 = -T_2 W_21   A_30 = -(A_32 W_20 + T_3 W_30)   A_31 = -(A_32 W_21 + T_3 W_31)
// Every entry of A is a key-to-key product through a chain of contractions (I - beta k^T k), so
// it is bounded by 1 whatever the keys: forming the inverse loses nothing here.  The four waves
// share this work tile by tile; tiles cross LDS row-major, so that a reader takes them in
// A-form (one 16-byte read) or in B-form (four 4-byte reads, the transposed access).
//
// LDS, one region X used three times -- the staged keys; then the fp32 tiles N_de (d > e), T_d,
// A_32, W_20, W_21; then the pieces of A^ -- and the pieces of M next to it: 36 KB for bf16,
// four workgroups per CU (28 KB and five for fp16).  A wave owns 32 dv columns: column tile c of wave w holds columns
// 32 w + 2 n + c (n = 0..15), so a lane's two tiles are adjacent columns.
// ---------------------------------------------------------------------------
// Workgroups per CU: the two fp16 pieces need 28 KB of LDS and 92 registers, which leaves room for
// five (6 % faster than four on ragged lengths); the three bf16 pieces need 36 KB and 124.
template <typename T>
constexpr int DIRECT_WG_PER_CU = __is_same(T, f16_t) ? 5 : 4;
template <typename TIn, typename TRec, bool PAGED>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(DIRECT_WG_PER_CU<TIn>, DIRECT_WG_PER_CU<TIn>))) void kvb_direct_mfma_kernel(
    const int32_t *len_arg, int32_t Hv_arg, int32_t nblocks_arg, const DirectArgs a)
{
    // The three leading arguments repeat a.len, a.Hv and the grid size: as plain leading kernel arguments
    // they are preloaded into scalar registers at wave launch (the build asks for it), so the load of
    // len[b] -- the head of the dependent chain to the first key byte -- goes out at once instead of after
    // the round trip that fetches the argument block.
    constexpr int D = 128;
    constexpr int LM = 64;   // longest context of this kernel
    constexpr int NB = LM / 16;                 // blocks of 16 rows (4)
    constexpr int NLOW = NB * (NB + 1) / 2;     // lower-triangular block pairs (10)
    constexpr int GS = D + 8;                   // LDS row stride of the staged keys (272 B:
                                                // consecutive rows start 4 banks apart)
    constexpr int NP = pieces_of_f32<TIn>();    // pieces of a fp32 tile
    constexpr int NPU = sizeof(TRec) == 2 ? 1 : NP;   // a 16-bit record is one piece as it stands
    static_assert(NB == NW, "one diagonal block per wave");
    constexpr int STAGE_BYTES = LM * GS * 2;
    constexpr int PIECE_BYTES = NLOW * NP * 512;        // pieces of A^ (and as much again for M)
    constexpr int F32_TILE = 1024;
    constexpr int OFF_N = 0;                            // N_de, d > e: 6 tiles, slot d (d - 1) / 2 + e
    constexpr int OFF_T01 = 6 * F32_TILE;               // T_0, T_1 (read before the pieces are written)
    constexpr int OFF_LATE = PIECE_BYTES;               // T_2, T_3, A_32, W_20, W_21 (read while they are)
    constexpr int X_BYTES = STAGE_BYTES > OFF_LATE + 5 * F32_TILE ? STAGE_BYTES : OFF_LATE + 5 * F32_TILE;
    static_assert(OFF_T01 + 2 * F32_TILE <= OFF_LATE, "the early tiles lie under the pieces only");
    __shared__ __attribute__((aligned(16))) unsigned char region[X_BYTES + PIECE_BYTES];
    __shared__ __attribute__((aligned(16))) float sG[LM];
    __shared__ __attribute__((aligned(16))) float sB[LM];
    __shared__ int sBlk[NW][MAX_BLOCKS];
    TIn *sK = reinterpret_cast<TIn *>(region);
    auto pieceA = [&](int tile, int p) { return reinterpret_cast<uint2 *>(region + (tile * NP + p) * 512); };
    auto pieceM = [&](int tile, int p) { return reinterpret_cast<uint2 *>(region + X_BYTES + (tile * NP + p) * 512); };

    // (the wave index as a scalar: conditions and tile numbers derived from it are then uniform for
    // the compiler, scalar branches instead of masked ones)
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64;
    const int c16 = lane % 16, lq = lane / 16;
    const int lb = logical_block(nblocks_arg);
    const int b = lb / Hv_arg;
    int L = len_arg[b];
    __builtin_amdgcn_sched_barrier(0);   // nothing that needs the argument block goes above this load
    const int h = lb % Hv_arg;
    const int r = a.Hv / a.Hk;
    const int hk = h / r;
    const int Lmax = a.Lmax;

    const int s = a.slot[b];
    if (s < 0 || s >= a.st.n_slots)
        return;
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
    // ---- every input of the workgroup is requested at once ------------------------
    // (no branch around a load: at a join the compiler waits for every load in flight, which would
    // make the passes take their round trips one after the other; a row past the context re-reads
    // the context's last row from the cache and is never used.  Reading the rows up to Lmax as they
    // are instead would cost a short context the traffic of a long one.)
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    u32x4_t kst[NB];
    const int srow = tid / 16, sc8 = tid % 16;
    const int col2 = 32 * wave + 2 * c16;
    // (uniform 64-bit base + 32-bit per-lane offset keeps the address arithmetic out of the VGPRs)
    const TIn *kbase = static_cast<const TIn *>(a.k) + ((size_t)b * Lmax * a.Hk + hk) * D;
    const TIn *qbase = static_cast<const TIn *>(a.q) + ((size_t)b * Lmax * a.Hk + hk) * D;
    const TIn *vbase = static_cast<const TIn *>(a.v) + ((size_t)b * Lmax * a.Hv + h) * D;
    const uint32_t qk_stride = (uint32_t)a.Hk * D, v_stride = (uint32_t)a.Hv * D;
#pragma unroll
    for (int p = 0; p < NB; ++p)   // pass p = rows 16 p .. 16 p + 15, 16 bytes per thread
        kst[p] = *reinterpret_cast<const u32x4_t *>(kbase + (uint32_t)min(16 * p + srow, L - 1) * qk_stride + 8 * sc8);
    // Q is not staged: the waves read the rows of their q.k tiles straight from memory in the
    // operand layout of the matrix instruction (row 16 d + c16, k = 8 lq + 32 step); a block of
    // 16 query rows is 4 KB and is shared by at most 4 tiles, so the repeats hit in the caches.
    // Tiles are dealt round-robin: t = wave + 4 n; t < 6 are k.k pairs, the rest q.k pairs.
    constexpr uint32_t PDB = pack2(1, 2, 2, 3, 3, 3, 0, 1, 1, 2, 2, 2, 3, 3, 3, 3);
    constexpr uint32_t PEB = pack2(0, 0, 1, 0, 1, 2, 0, 0, 1, 0, 1, 2, 0, 1, 2, 3);
    auto PD = [](int t) { return (int)((PDB >> (2 * t)) & 3u); };
    auto PE = [](int t) { return (int)((PEB >> (2 * t)) & 3u); };
    u32x4_t qop[3][4];   // n = 1 (waves 2, 3 only), 2, 3
#pragma unroll
    for (int n = 1; n < 4; ++n) {
        const uint32_t o = (uint32_t)min(16 * PD(wave + NW * n) + c16, L - 1) * qk_stride + 8 * lq;
#pragma unroll
        for (int st = 0; st < 4; ++st)
            qop[n - 1][st] = *reinterpret_cast<const u32x4_t *>(qbase + o + 32 * st);
    }
    const size_t gb_o = ((size_t)b * Lmax + min(lane, L - 1)) * a.Hv + h;
    float g_raw = a.g[gb_o], beta_raw = a.beta[gb_o];   // (every wave: a branch around a load costs more)

    const Pages<PAGED> pg = make_pages<PAGED>(a.st, s, a.cap, sBlk[wave], lane, load_block_id<PAGED>(a.st, s, lane));
    auto ru = [&](int l) { return pg.row(l, a.Hv, h); };
    auto rk = [&](int l) { return pg.row(l, a.Hk, hk); };
    const Out<TIn> out{a.out, a.out_wide != 0};
    const int nb = (L + 15) / 16;
    auto tri = [](int d, int e) { return d * (d + 1) / 2 + e; };    // slot of pair d >= e
    auto trn = [](int d, int e) { return d * (d - 1) / 2 + e; };    // slot of pair d > e
    // fp32 tiles in LDS are row-major 16 x 16: A-form is one 16-byte access, B-form four 4-byte ones
    auto lds_a = [&](int off) {
        const float4 t = *reinterpret_cast<const float4 *>(region + off + c16 * 64 + lq * 16);
        return f32x4_t{t.x, t.y, t.z, t.w};
    };
    auto lds_b = [&](int off) {
        const float *t = reinterpret_cast<const float *>(region + off) + 64 * lq + c16;
        return f32x4_t{t[0], t[16], t[32], t[48]};
    };
    auto put_a = [&](int off, const f32x4_t &x) {
        *reinterpret_cast<float4 *>(region + off + c16 * 64 + lq * 16) = make_float4(x[0], x[1], x[2], x[3]);
    };
    // (tiles that only ever travel in B-form keep their per-lane layout)
    auto put_lane = [&](int off, const f32x4_t &x) {
        *reinterpret_cast<float4 *>(region + off + lane * 16) = make_float4(x[0], x[1], x[2], x[3]);
    };
    auto lds_lane = [&](int off) {
        const float4 t = *reinterpret_cast<const float4 *>(region + off + lane * 16);
        return f32x4_t{t.x, t.y, t.z, t.w};
    };
    constexpr int OFF_T2 = OFF_LATE, OFF_T3 = OFF_LATE + F32_TILE, OFF_A32 = OFF_LATE + 2 * F32_TILE,
                  OFF_W20 = OFF_LATE + 3 * F32_TILE, OFF_W21 = OFF_LATE + 4 * F32_TILE;
    auto off_n = [&](int d, int e) { return OFF_N + trn(d, e) * F32_TILE; };
    auto off_t = [&](int d) { return d < 2 ? OFF_T01 + d * F32_TILE : OFF_LATE + (d - 2) * F32_TILE; };

    // cumulative log decay (inclusive scan over the wave) and beta
    if (wave == 0) {
        float gv = lane < L ? g_raw : 0.0f;
        const float bv = lane < L ? beta_raw : 0.0f;
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
    // stage K; the thread that loaded a piece of K also appends it to the buffer
    TIn *kb = static_cast<TIn *>(a.st.buf_k);
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
        gdiag = gram16<TIn, GS>(sK + (16 * wave + c16) * GS, sK + (16 * wave + c16) * GS, lq);
    f32x4_t gsh[4];
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        const int t = wave + NW * n, d = PD(t), e = PE(t);
        gsh[n] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        if (d < nb) {   // uniform
            if (t < 6) {
                gsh[n] = gram16<TIn, GS>(sK + (16 * e + c16) * GS, sK + (16 * d + c16) * GS, lq);
            } else if (n > 0) {   // t >= 6 implies n >= 1
                const TIn *arow = sK + (16 * e + c16) * GS;
#pragma unroll
                for (int st = 0; st < 4; ++st) {
                    const uint4 av = *reinterpret_cast<const uint4 *>(arow + 8 * lq + 32 * st);
                    gsh[n] = mfma16x32<TIn>(av, __builtin_bit_cast(uint4, qop[n > 0 ? n - 1 : 0][st]), gsh[n]);
                }
            }
        }
    }
    __syncthreads();   // every wave is done with the staged rows: the region now takes the tiles

    // v in B-form: rows 16 d + 4 lq + v, this lane's two adjacent columns 32 wave + 2 c16, + 1.
    // Requested only now, when the registers of the staged rows are free again; the values are not
    // needed before the last phase.
    uint32_t v_raw[NB][4];
#pragma unroll
    for (int d = 0; d < NB; ++d)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            v_raw[d][v] = *reinterpret_cast<const uint32_t *>(
                vbase + (uint32_t)min(16 * d + 4 * lq + v, L - 1) * v_stride + col2);
    // ---- weights and masks.  A-form element of tile (d, e): row i = 16 d + c16, column l = 16 e + 4 lq + v.
    // N tiles go to LDS in fp32 (they enter the inverse), M tiles are cut into pieces at once.
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        const int t = wave + NW * n, d = PD(t), e = PE(t);
        if (d < nb) {
            const int i = 16 * d + c16;
            const bool isq = t >= 6;
            // (LDS reads without a condition, then selects: a read under a condition becomes a
            // branch with a wait of its own, one round trip per element)
            const float gi = sG[i];
            const float si = isq ? 1.0f : sB[i];
            const float4 gl4 = *reinterpret_cast<const float4 *>(&sG[16 * e + 4 * lq]);
            const float gl[4] = {gl4.x, gl4.y, gl4.z, gl4.w};
            f32x4_t o;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int l = 16 * e + 4 * lq + v;
                const bool ok = i < L && (isq ? l <= i : l < i);
                o[v] = ok ? si * fast_exp(gi - gl[v]) * gsh[n][v] : 0.0f;
            }
            if (isq) {
                uint2 pc[NP];
                split_tile<TIn, NP>(o, pc);
#pragma unroll
                for (int p = 0; p < NP; ++p)
                    pieceM(tri(d, e), p)[lane] = pc[p];
            } else {
                put_a(off_n(d, e), o);
            }
        }
    }
    // T_d = (I + N_dd)^-1 for d = wave.  The raw diagonal tile is symmetric, so the same registers
    // give the A-form (row 16 d + c16, column 16 d + 4 lq + v) and the B-form (row and column swapped).
    f32x4_t t_own = {0.f, 0.f, 0.f, 0.f};   // T_wave, A-form
    if (wave < nb) {
        const int d = wave;
        f32x4_t na, nbm, ia;   // N in both forms; identity mask (the same in both forms)
        const float gc = sG[16 * d + c16], bc = sB[16 * d + c16];
        const float4 gq4 = *reinterpret_cast<const float4 *>(&sG[16 * d + 4 * lq]);
        const float4 bq4 = *reinterpret_cast<const float4 *>(&sB[16 * d + 4 * lq]);
        const float gq[4] = {gq4.x, gq4.y, gq4.z, gq4.w}, bq[4] = {bq4.x, bq4.y, bq4.z, bq4.w};
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int ia_i = 16 * d + c16, ia_l = 16 * d + 4 * lq + v;    // A-form indices
            const int ib_i = ia_l, ib_l = ia_i;                            // B-form indices
            na[v] = (ia_i < L && ia_l < ia_i) ? bc * fast_exp(gc - gq[v]) * gdiag[v] : 0.0f;
            nbm[v] = (ib_i < L && ib_l < ib_i) ? bq[v] * fast_exp(gq[v] - gc) * gdiag[v] : 0.0f;
            ia[v] = ia_i == ia_l ? 1.0f : 0.0f;
        }
        t_own = unit_lower_inverse16(na, nbm, ia, c16, lq);
        if (nb > 1)
            put_a(off_t(d), t_own);
    }
    __syncthreads();

    // ---- the off-diagonal tiles of A = (I + N)^-1, first half: A_10, A_32 and W = C P^-1 -------
    const f32x4_t z4 = {0.f, 0.f, 0.f, 0.f};
    f32x4_t w_own = z4;    // W_2w (waves 0, 1) or W_3,w-2 (waves 2, 3), B-form
    f32x4_t a_lvl2 = z4;   // A_10 (wave 1) or A_32 (wave 3), A-form
    if (nb > 1) {          // (uniform; mm16(x_a, y_b) = B-form of X Y, mm16(y_b, x_a) = its A-form)
        if (wave == 0 || wave == 2) {
            const int dr = wave == 0 ? 2 : 3;        // block row of C
            if (dr < nb) {
                const f32x4_t y1a = mm16(lds_b(off_t(1)), lds_a(off_n(dr, 1)), z4);   // N_d1 T_1
                const f32x4_t y2a = mm16(lds_b(off_n(1, 0)), y1a, z4);                // N_d1 T_1 N_10
                w_own = mm16(lds_a(off_n(dr, 0)) - y2a, lds_b(off_t(0)), z4);         // (N_d0 - ...) T_0
                if (wave == 0)
                    put_lane(OFF_W20, w_own);
            }
        } else if (wave == 1) {
            const f32x4_t pb = mm16(lds_a(off_n(1, 0)), lds_b(off_t(0)), z4);          // N_10 T_0
            a_lvl2 = -mm16(pb, t_own, z4);                                             // -T_1 (N_10 T_0)
            if (nb > 2) {
                w_own = mm16(lds_a(off_n(2, 1)), lds_b(off_t(1)), z4);                 // N_21 T_1
                put_lane(OFF_W21, w_own);
            }
        } else if (nb == 4) {   // wave 3
            w_own = mm16(lds_a(off_n(3, 1)), lds_b(off_t(1)), z4);                     // N_31 T_1
            const f32x4_t pb = mm16(lds_a(off_n(3, 2)), lds_b(off_t(2)), z4);          // N_32 T_2
            a_lvl2 = -mm16(pb, t_own, z4);                                             // -T_3 (N_32 T_2)
            put_a(OFF_A32, a_lvl2);
        }
    }
    __syncthreads();

    // ---- second half: A_2e = -T_2 W_2e, A_3e = -(A_32 W_2e + T_3 W_3e); then every tile of A,
    // its columns scaled by beta (A^ = A Diag(beta)), goes to LDS in pieces.  The pieces take the
    // place of the N tiles, T_0 and T_1, which nobody reads any more.
    auto put_pieces = [&](int d, int e, const f32x4_t &xa) {
        const float4 b4 = *reinterpret_cast<const float4 *>(&sB[16 * e + 4 * lq]);
        uint2 pc[NP];
        split_tile<TIn, NP>(f32x4_t{xa[0] * b4.x, xa[1] * b4.y, xa[2] * b4.z, xa[3] * b4.w}, pc);
#pragma unroll
        for (int p = 0; p < NP; ++p)
            pieceA(tri(d, e), p)[lane] = pc[p];
    };
    if (wave < nb)
        put_pieces(wave, wave, t_own);
    if (wave == 1 && nb > 1)
        put_pieces(1, 0, a_lvl2);
    if (wave == 3 && nb == 4)
        put_pieces(3, 2, a_lvl2);
    if (wave < 2) {
        if (nb > 2)
            put_pieces(2, wave, -mm16(w_own, lds_a(OFF_T2), z4));
    } else if (nb == 4) {
        const f32x4_t w2b = lds_lane(wave == 2 ? OFF_W20 : OFF_W21);
        f32x4_t x = mm16(w2b, lds_a(OFF_A32), z4);
        x = mm16(w_own, lds_a(OFF_T3), x);
        put_pieces(3, wave - 2, -x);
    }
    __syncthreads();

    // ---- U = A^ V and O = M U on the 16-bit matrix instruction, this wave's 32 columns ----------
    // Operand of the values for two row blocks (e, e + 1) and column tile c: the lane's 8 slots are
    // rows 16 e + 4 lq + 0..3 and 16 (e + 1) + 4 lq + 0..3; a word of v_raw holds both column tiles.
    uint4 vop[NB / 2][2];
#pragma unroll
    for (int e2 = 0; e2 < NB / 2; ++e2) {
        const uint32_t *w0 = v_raw[2 * e2], *w1 = v_raw[2 * e2 + 1];
        vop[e2][0] = uint4{__builtin_amdgcn_perm(w0[1], w0[0], 0x05040100u), __builtin_amdgcn_perm(w0[3], w0[2], 0x05040100u),
                           __builtin_amdgcn_perm(w1[1], w1[0], 0x05040100u), __builtin_amdgcn_perm(w1[3], w1[2], 0x05040100u)};
        vop[e2][1] = uint4{__builtin_amdgcn_perm(w0[1], w0[0], 0x07060302u), __builtin_amdgcn_perm(w0[3], w0[2], 0x07060302u),
                           __builtin_amdgcn_perm(w1[1], w1[0], 0x07060302u), __builtin_amdgcn_perm(w1[3], w1[2], 0x07060302u)};
    }
    uint2 upc[NB][2][NPU];   // the pieces of U_e, column tile c (B-form)
    const size_t outp = (((size_t)b * Lmax) * a.Hv + h) * D;
    TRec *up = static_cast<TRec *>(a.st.buf_u);
#pragma unroll
    for (int d = 0; d < NB; ++d) {
        if (d < nb) {   // uniform
            f32x4_t U[2] = {z4, z4}, o[2] = {z4, z4};
#pragma unroll
            for (int p = NP - 1; p >= 0; --p) {   // smallest pieces first
#pragma unroll
                for (int e2 = 0; e2 <= d / 2; ++e2) {
                    const uint2 lo = pieceA(tri(d, 2 * e2), p)[lane];
                    uint2 hi = {0u, 0u};
                    if (2 * e2 + 1 <= d)
                        hi = pieceA(tri(d, 2 * e2 + 1), p)[lane];
                    const uint4 aop = {lo.x, lo.y, hi.x, hi.y};
#pragma unroll
                    for (int c = 0; c < 2; ++c)
                        U[c] = mfma16x32<TIn>(aop, vop[e2][c], U[c]);
                }
            }
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                if constexpr (sizeof(TRec) == 2) {
                    // the outputs read the records as stored; a rounded value is one piece as it stands
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        U[c][v] = rounded_to<TRec>(U[c][v]);
                    upc[d][c][0] = uint2{pack_pair<TRec>(U[c][0], U[c][1]), pack_pair<TRec>(U[c][2], U[c][3])};
                } else {
                    split_tile<TIn, NPU>(U[c], upc[d][c]);
                }
            }
#pragma unroll
            for (int e = 0; e <= d; ++e) {
                uint2 mp[NP];
#pragma unroll
                for (int p = 0; p < NP; ++p)
                    mp[p] = pieceM(tri(d, e), p)[lane];
#pragma unroll
                for (int c = 0; c < 2; ++c)
                    o[c] = mm16_pieces<TIn, NP, NPU>(mp, upc[e][c], o[c]);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = 16 * d + 4 * lq + v;
                if (i < L) {
                    // (streaming stores: neither array is read again by this kernel, and lines that do not
                    // linger in the L2 leave it to the keys, queries and values that the heads of a request share)
                    out.put2_nt(outp + ((uint32_t)i * v_stride + col2), a.scale * o[0][v], a.scale * o[1][v]);
                    store2_nt(up + (ru(i) * D + col2), U[0][v], U[1][v]);
                }
            }
        }
    }
    if (h == 0 && tid == 0)
        a.st.fill[s] = L;
}

// ---------------------------------------------------------------------------
// kvb_direct for contexts of 65 .. 128 tokens (16-bit inputs, d = 128): the block-row method with 8
// blocks of 16 rows.  Kept apart from the kernel above, which is tuned around "4 blocks, one per wave" (its raw
// Gram tiles and query operands all fit in registers at once).  Here a wave owns two diagonal
// blocks and 16 of the 64 off-diagonal k.k and q.k tiles; the query rows of a tile are fetched
// one tile ahead; the tile region (80 tiles, 80 KB) again takes the place of the staged keys.
// ---------------------------------------------------------------------------
template <typename TIn, typename TRec, bool PAGED>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(2, 2))) void kvb_direct_mfma_long_kernel(
    const DirectArgs a)
{
    constexpr int D = 128;
    constexpr int NB = 8;                       // blocks of 16 rows
    constexpr int LM = 16 * NB;                 // 128
    constexpr int NLOW = NB * (NB + 1) / 2;     // block pairs d >= e (36)
    constexpr int NKK = NB * (NB - 1) / 2;      // off-diagonal k.k pairs (28)
    constexpr int NTPW = NB * NB / NW;          // off-diagonal k.k + all q.k tiles per wave (16)
    constexpr int DPW = NB / NW;                // diagonal blocks per wave (2)
    constexpr int GS = D + 8;
    constexpr int STAGE_BYTES = LM * GS * 2;
    constexpr int TILE_BYTES = (NKK + NLOW + NB) * 64 * 16;   // 72 KB: two workgroups per CU
    __shared__ __attribute__((aligned(16))) unsigned char region[STAGE_BYTES > TILE_BYTES ? STAGE_BYTES : TILE_BYTES];
    __shared__ __attribute__((aligned(16))) float sG[LM];
    __shared__ __attribute__((aligned(16))) float sB[LM];
    __shared__ int sBlk[NW][MAX_BLOCKS];
    TIn *sK = reinterpret_cast<TIn *>(region);
    float4(*tN)[64] = reinterpret_cast<float4(*)[64]>(region);
    float4(*tM)[64] = tN + NKK;
    float4(*tT)[64] = tM + NLOW;

    // (the wave index as a scalar: conditions and tile numbers derived from it are then uniform for
    // the compiler, scalar branches instead of masked ones)
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64;
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
    const TIn *qin = static_cast<const TIn *>(a.q);
    const TIn *kin = static_cast<const TIn *>(a.k);
    const TIn *vin = static_cast<const TIn *>(a.v);
    const Out<TIn> out{a.out, a.out_wide != 0};
    const int nb = (L + 15) / 16;
    auto tri = [](int d, int e) { return d * (d + 1) / 2 + e; };    // slot of pair d >= e
    auto trn = [](int d, int e) { return d * (d - 1) / 2 + e; };    // slot of pair d > e
    // tile t of the dealing order -> block pair: t < NKK are the k.k pairs (d > e), row by row,
    // then the q.k pairs (d >= e), row by row.  Uniform, a handful of scalar steps.
    auto pair_of = [&](int t, int &d, int &e, bool &isq) {
        isq = t >= NKK;
        if (!isq) {
            d = 1;
            while (t >= d) {
                t -= d;
                ++d;
            }
        } else {
            t -= NKK;
            d = 0;
            while (t > d) {
                t -= d + 1;
                ++d;
            }
        }
        e = t;
    };

    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    const int srow = tid / 16, sc8 = tid % 16;
    const TIn *kbase = kin + ((size_t)b * Lmax * a.Hk + hk) * D;
    const TIn *qbase = qin + ((size_t)b * Lmax * a.Hk + hk) * D;
    const TIn *vbase = vin + ((size_t)b * Lmax * a.Hv + h) * D;
    const uint32_t qk_stride = (uint32_t)a.Hk * D, v_stride = (uint32_t)a.Hv * D;
    const int col2 = 32 * wave + 2 * c16;

    // ---- keys: load, stage, append to the buffer --------------------------------
    u32x4_t kst[NB];
#pragma unroll
    for (int p = 0; p < NB; ++p) {   // rows past the context re-read its last row (never used)
        const uint32_t o = (uint32_t)min(16 * p + srow, L - 1) * qk_stride + 8 * sc8;
        kst[p] = *reinterpret_cast<const u32x4_t *>(kbase + o);   // (no branch around a load, as above)
    }
    // cumulative log decay and beta: wave 0 takes tokens 0..63, wave 1 tokens 64..127 (it adds
    // the sum of the first 64 decays, which it forms itself)
    if (wave < 2) {
        const int t0 = 64 * wave + lane;
        float gv = t0 < L ? a.g[((size_t)b * Lmax + t0) * a.Hv + h] : 0.0f;
        const float bv = t0 < L ? a.beta[((size_t)b * Lmax + t0) * a.Hv + h] : 0.0f;
        float base = 0.0f;
        if (wave == 1) {
            base = lane < L ? a.g[((size_t)b * Lmax + lane) * a.Hv + h] : 0.0f;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1)
                base += __shfl_xor(base, off);
        }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const float t = __shfl_up(gv, off);
            if (lane >= off)
                gv += t;
        }
        gv += base;
        sG[t0] = gv;
        sB[t0] = bv;
        if (t0 < L)
            a.st.buf_G[ru(t0)] = gv;
    }
    TIn *kb = static_cast<TIn *>(a.st.buf_k);
#pragma unroll
    for (int p = 0; p < NB; ++p) {
        if (p < nb) {   // uniform
            *reinterpret_cast<u32x4_t *>(sK + (16 * p + srow) * GS + 8 * sc8) = kst[p];
            if (h % r == 0 && 16 * p + srow < L)
                *reinterpret_cast<u32x4_t *>(kb + rk(16 * p + srow) * D + 8 * sc8) = kst[p];
        }
    }
    __syncthreads();

    // ---- raw Gram tiles ----------------------------------------------------------
    f32x4_t gdiag[DPW];
#pragma unroll
    for (int x = 0; x < DPW; ++x) {
        const int d = wave + NW * x;
        gdiag[x] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        if (d < nb)
            gdiag[x] = gram16<TIn, GS>(sK + (16 * d + c16) * GS, sK + (16 * d + c16) * GS, lq);
    }
    // query rows of a q.k tile, in the operand layout (row 16 d + c16, k = 8 lq + 32 step),
    // requested one tile ahead of their use
    auto load_q = [&](int t, u32x4_t(&qq)[4]) {
        int d, e;
        bool isq;
        pair_of(t, d, e, isq);
        const uint32_t o = (uint32_t)min(16 * d + c16, L - 1) * qk_stride + 8 * lq;
#pragma unroll
        for (int st = 0; st < 4; ++st)   // (also for k.k tiles and empty blocks: no branch around a load)
            qq[st] = *reinterpret_cast<const u32x4_t *>(qbase + o + 32 * st);
    };
    f32x4_t gsh[NTPW];
    u32x4_t qa[4], qb[4];
    load_q(wave, qa);
#pragma unroll
    for (int n = 0; n < NTPW; ++n) {
        const int t = wave + NW * n;
        if (n + 1 < NTPW) {
            if (n % 2 == 0)
                load_q(t + NW, qb);
            else
                load_q(t + NW, qa);
        }
        int d, e;
        bool isq;
        pair_of(t, d, e, isq);
        gsh[n] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        if (d < nb) {   // uniform
            if (!isq) {
                gsh[n] = gram16<TIn, GS>(sK + (16 * e + c16) * GS, sK + (16 * d + c16) * GS, lq);
            } else {
                const TIn *arow = sK + (16 * e + c16) * GS;
#pragma unroll
                for (int st = 0; st < 4; ++st) {
                    const uint4 av = *reinterpret_cast<const uint4 *>(arow + 8 * lq + 32 * st);
                    gsh[n] = mfma16x32<TIn>(av, __builtin_bit_cast(uint4, n % 2 == 0 ? qa[st] : qb[st]), gsh[n]);
                }
            }
        }
    }
    __syncthreads();   // every wave is done with the staged rows: the region now takes the tiles

    // v in B-form: rows 16 d + 4 lq + v, this lane's two adjacent columns
    uint32_t v_raw[NB][4];
#pragma unroll
    for (int d = 0; d < NB; ++d)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            v_raw[d][v] = *reinterpret_cast<const uint32_t *>(
                vbase + (uint32_t)min(16 * d + 4 * lq + v, L - 1) * v_stride + col2);
        }

    // weights and masks.  A-form element of tile (d, e): row i = 16 d + c16, column l = 16 e + 4 lq + v.
#pragma unroll
    for (int n = 0; n < NTPW; ++n) {
        int d, e;
        bool isq;
        pair_of(wave + NW * n, d, e, isq);
        if (d < nb) {
            const int i = 16 * d + c16;
            // (LDS reads without a condition, then selects: a read under a condition becomes a
            // branch with a wait of its own, one round trip per element)
            const float gi = sG[i];
            const float si = isq ? 1.0f : -sB[i];
            const float4 gl4 = *reinterpret_cast<const float4 *>(&sG[16 * e + 4 * lq]);
            const float gl[4] = {gl4.x, gl4.y, gl4.z, gl4.w};
            float o[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int l = 16 * e + 4 * lq + v;
                const bool ok = i < L && (isq ? l <= i : l < i);
                o[v] = ok ? si * fast_exp(gi - gl[v]) * gsh[n][v] : 0.0f;
            }
            const float4 o4 = make_float4(o[0], o[1], o[2], o[3]);
            if (isq)
                tM[tri(d, e)][lane] = o4;
            else
                tN[trn(d, e)][lane] = o4;
        }
    }
    // T_d = (I + N_dd)^-1 for this wave's diagonal blocks (see the kernel above)
#pragma unroll
    for (int x = 0; x < DPW; ++x) {
        const int d = wave + NW * x;
        if (d < nb) {
            f32x4_t na, nbm, ia;
            const float gc = sG[16 * d + c16], bc = sB[16 * d + c16];
            const float4 gq4 = *reinterpret_cast<const float4 *>(&sG[16 * d + 4 * lq]);
            const float4 bq4 = *reinterpret_cast<const float4 *>(&sB[16 * d + 4 * lq]);
            const float gq[4] = {gq4.x, gq4.y, gq4.z, gq4.w}, bq[4] = {bq4.x, bq4.y, bq4.z, bq4.w};
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int ia_i = 16 * d + c16, ia_l = 16 * d + 4 * lq + v;
                const int ib_i = ia_l, ib_l = ia_i;
                na[v] = (ia_i < L && ia_l < ia_i) ? bc * fast_exp(gc - gq[v]) * gdiag[x][v] : 0.0f;
                nbm[v] = (ib_i < L && ib_l < ib_i) ? bq[v] * fast_exp(gq[v] - gc) * gdiag[x][v] : 0.0f;
                ia[v] = ia_i == ia_l ? 1.0f : 0.0f;
            }
            const f32x4_t p = unit_lower_inverse16(na, nbm, ia, c16, lq);
            tT[d][lane] = make_float4(p[0], p[1], p[2], p[3]);
        }
    }
    __syncthreads();

    // ---- block forward substitution and outputs, this wave's 32 columns ----------
    f32x4_t U[NB][2];
    const size_t outp = (((size_t)b * Lmax) * a.Hv + h) * D;
    TRec *up = static_cast<TRec *>(a.st.buf_u);
#pragma unroll
    for (int d = 0; d < NB; ++d) {
        if (d < nb) {   // uniform
            f32x4_t acc[2], o[2];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = 16 * d + 4 * lq + v;
                const float bi = sB[i];   // zero beyond the context
                const float2 vv = unpack_pair<TIn>(v_raw[d][v]);
                acc[0][v] = bi * vv.x;
                acc[1][v] = bi * vv.y;
            }
            o[0] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            o[1] = o[0];
#pragma unroll
            for (int e = 0; e < d; ++e) {
                const float4 n4 = tN[trn(d, e)][lane];
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
                if constexpr (sizeof(TRec) == 2) {   // later blocks and this block's outputs read the records as stored
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        U[d][c][v] = rounded_to<TRec>(U[d][c][v]);
                }
                o[c] = mm16(mm, U[d][c], o[c]);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = 16 * d + 4 * lq + v;
                if (i < L) {
                    out.put2(outp + ((uint32_t)i * v_stride + col2), a.scale * o[0][v], a.scale * o[1][v]);
                    store2(up + (ru(i) * D + col2), U[d][0][v], U[d][1][v]);
                }
            }
        }
    }
    if (h == 0 && tid == 0)
        a.st.fill[s] = L;
}

// ---------------------------------------------------------------------------
// launch
// ---------------------------------------------------------------------------
int launch_direct(int dk, int in_dtype, int rec_dtype, const DirectArgs &a, int blocks, hipStream_t stream)
{
    if (dk == 128 && in_dtype != KVB_F32)
        return dispatch_types16(in_dtype, rec_dtype, [&]<typename TIn, typename TRec>() {
            if (a.Lmax > 64)   // 5 .. 8 blocks of 16 rows
                LAUNCH_PAGED(blocks, stream, a, kvb_direct_mfma_long_kernel<TIn, TRec);
            else if (a.st.block_table)
                launch(kvb_direct_mfma_kernel<TIn, TRec, true>, blocks, stream, a.len, a.Hv, blocks, a);
            else
                launch(kvb_direct_mfma_kernel<TIn, TRec, false>, blocks, stream, a.len, a.Hv, blocks, a);
        });
    if (a.Lmax > 64)   // the plain kernel holds a 64-token context in LDS
        return KVB_EUNSUPPORTED;
    return dispatch(dk, in_dtype, rec_dtype, [&]<int D, typename TIn, typename TRec>() {
        if constexpr (!(D == 128 && sizeof(TIn) == 2))
            LAUNCH_PAGED(blocks, stream, a, kvb_direct_kernel<D, TIn, TRec);
    });
}

}  // namespace kvb_impl
