// kvb -- KVBuffer-style Gated DeltaNet decoding, HIP kernels for gfx950 behind the C ABI of
// include/kvb.h.  This header holds what the translation units share: device helpers, the
// argument structs of the kernels, and the launch plumbing.
//   kvb_step_kernel.h    kvb_step_kernel (decode and the vector-ALU verify); instantiated per
//                        (input type, record type) by kvb_step_f32.hip, kvb_step_bf16.hip,
//                        kvb_step_bf16_r16.hip, kvb_step_f16.hip, kvb_step_f16_r16.hip
//   kvb_verify_kernel.h  kvb_verify_mfma_kernel; instantiated by kvb_verify_bf16.hip, kvb_verify_f16.hip
//   kvb_flush.hip        kvb_flush_mfma_kernel, kvb_flush_kernel, kvb_compact_kernel
//   kvb_direct.hip       kvb_direct_mfma_kernel, kvb_direct_mfma_long_kernel, kvb_direct_kernel
//   kvb_api.hip          argument checks, the extern "C" entry points, the kernel timer
//
// Element types (Sec. 4.1: 16-bit vectors and records beside a fp32 state): TIn is the type of
// q, k, v and of the buffered keys (float, bf16_t or f16_t), TRec that of the buffered delta
// values (float, or TIn when that is 16-bit); outputs are fp32 or TIn, chosen at run time at the
// final store.  All arithmetic is fp32.
//
// Work decomposition (every kernel): one 256-thread workgroup per (request b,
// v-head h); the committed state S0[dk][dv] (fp32, dv contiguous, 64 KB at
// d = 128) is streamed exactly once per call.  Besides the state a unit needs
// its buffered keys k_l, delta values u_l and cumulative log decays G_l (paper
// App. A.1, the paragraph after Eq. 16), a few KB.
//   kvb_step_kernel         decode (T = 1) and generic verify: vector ALUs; a thread owns
//                           4 adjacent dv columns of 16 state rows (16-byte loads)
//   kvb_verify_mfma_kernel  verify, 16-bit inputs / d = 128: matrix cores; a wave owns 32 dv columns
//   kvb_flush_mfma_kernel   deferred state update, 16-bit inputs / d = 128: matrix cores on exact
//                           16-bit pieces of the fp32 factor
//   kvb_flush_kernel        the same for the other types and head sizes: vector ALUs
//   kvb_direct_mfma_kernel  short contexts, 16-bit inputs / d = 128: matrix cores throughout
//   kvb_direct_kernel       short contexts, other types and head sizes
//
// Notation follows App. A.1: gamma_i = exp(G_i), Gamma_il = exp(G_i - G_l).

#ifndef KVB_DEVICE_H
#define KVB_DEVICE_H

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <tuple>
#include <type_traits>

#include "kvb.h"

struct kvb_timer {
    hipEvent_t start, stop;
};

namespace kvb_impl {

constexpr int NT = 256;      // threads per workgroup
constexpr int NW = NT / 64;  // wavefronts per workgroup
constexpr int FILL_MASK = 0xFFFF;
constexpr int TICKET_ONE = 1 << 16;

struct bf16_t {
    uint16_t bits;
};
struct f16_t {
    uint16_t bits;
};

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4_t;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return __uint_as_float((uint32_t)x.bits << 16); }
__device__ __forceinline__ float to_f32(f16_t x) { return (float)__builtin_bit_cast(_Float16, x.bits); }

// Rounding to a storage type, to nearest even (the hardware conversions of gfx950).
template <typename T>
__device__ __forceinline__ T from_f32(float x);
template <>
__device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <>
__device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { return bf16_t{__builtin_bit_cast(uint16_t, (__bf16)x)}; }
template <>
__device__ __forceinline__ f16_t from_f32<f16_t>(float x) { return f16_t{__builtin_bit_cast(uint16_t, (_Float16)x)}; }
// x as the storage type T will hold it
template <typename T>
__device__ __forceinline__ float rounded_to(float x) { return to_f32(from_f32<T>(x)); }

// The two 16-bit elements packed in one word, and two floats packed into one.
template <typename T>
__device__ __forceinline__ float2 unpack_pair(uint32_t w)
{
    if constexpr (__is_same(T, bf16_t)) {
        return make_float2(__uint_as_float(w << 16), __uint_as_float(w & 0xFFFF0000u));
    } else {
        const f16x2_t h = __builtin_bit_cast(f16x2_t, w);
        return make_float2((float)h[0], (float)h[1]);
    }
}
template <typename T>
__device__ __forceinline__ uint32_t pack_pair(float lo, float hi)
{
    return (uint32_t)from_f32<T>(lo).bits | ((uint32_t)from_f32<T>(hi).bits << 16);
}

// 8 consecutive elements starting at p (p is 16-byte aligned for the 16-bit types, 32 for fp32).
__device__ __forceinline__ void load8(const float *p, float (&o)[8])
{
    const float4 a = *reinterpret_cast<const float4 *>(p);
    const float4 b = *reinterpret_cast<const float4 *>(p + 4);
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
    o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}

// The same 8 elements as untouched bits: issuing a load and converting its result are
// kept apart so that no wait lands between two loads.
template <typename T>
struct Raw8 {
    uint4 w;
};
template <>
struct Raw8<float> {
    float4 a, b;
};
__device__ __forceinline__ Raw8<float> load_raw8(const float *p)
{
    return Raw8<float>{*reinterpret_cast<const float4 *>(p), *reinterpret_cast<const float4 *>(p + 4)};
}
template <typename T>
__device__ __forceinline__ Raw8<T> load_raw8(const T *p)
{
    return Raw8<T>{*reinterpret_cast<const uint4 *>(p)};
}
__device__ __forceinline__ void unpack8(const Raw8<float> &r, float (&o)[8])
{
    o[0] = r.a.x; o[1] = r.a.y; o[2] = r.a.z; o[3] = r.a.w;
    o[4] = r.b.x; o[5] = r.b.y; o[6] = r.b.z; o[7] = r.b.w;
}
template <typename T>
__device__ __forceinline__ void unpack8(const Raw8<T> &r, float (&o)[8])
{
    const float2 a = unpack_pair<T>(r.w.x), b = unpack_pair<T>(r.w.y), c = unpack_pair<T>(r.w.z), d = unpack_pair<T>(r.w.w);
    o[0] = a.x; o[1] = a.y; o[2] = b.x; o[3] = b.y;
    o[4] = c.x; o[5] = c.y; o[6] = d.x; o[7] = d.y;
}
template <typename T>
__device__ __forceinline__ void load8(const T *p, float (&o)[8])
{
    unpack8(load_raw8(p), o);
}

// 4 and 2 consecutive elements of a record array (delta values), raw and converted.
template <typename T>
struct Raw4 {
    uint2 w;
};
template <>
struct Raw4<float> {
    float4 a;
};
__device__ __forceinline__ Raw4<float> load_raw4(const float *p) { return Raw4<float>{*reinterpret_cast<const float4 *>(p)}; }
template <typename T>
__device__ __forceinline__ Raw4<T> load_raw4(const T *p) { return Raw4<T>{*reinterpret_cast<const uint2 *>(p)}; }
__device__ __forceinline__ float4 unpack4(const Raw4<float> &r) { return r.a; }
template <typename T>
__device__ __forceinline__ float4 unpack4(const Raw4<T> &r)
{
    const float2 a = unpack_pair<T>(r.w.x), b = unpack_pair<T>(r.w.y);
    return make_float4(a.x, a.y, b.x, b.y);
}
template <typename T>
struct Raw2 {
    uint32_t w;
};
template <>
struct Raw2<float> {
    float2 a;
};
__device__ __forceinline__ Raw2<float> load_raw2(const float *p) { return Raw2<float>{*reinterpret_cast<const float2 *>(p)}; }
template <typename T>
__device__ __forceinline__ Raw2<T> load_raw2(const T *p) { return Raw2<T>{*reinterpret_cast<const uint32_t *>(p)}; }
__device__ __forceinline__ float2 unpack2r(const Raw2<float> &r) { return r.a; }
template <typename T>
__device__ __forceinline__ float2 unpack2r(const Raw2<T> &r) { return unpack_pair<T>(r.w); }

// Stores of already-rounded or to-be-rounded values into an array of type T.
__device__ __forceinline__ void store2(float *p, float x, float y) { *reinterpret_cast<float2 *>(p) = make_float2(x, y); }
template <typename T>
__device__ __forceinline__ void store2(T *p, float x, float y) { *reinterpret_cast<uint32_t *>(p) = pack_pair<T>(x, y); }
// The same as streaming (non-temporal) stores, for results that this kernel does not read again.
__device__ __forceinline__ void store2_nt(float *p, float x, float y)
{
    typedef float v2f __attribute__((ext_vector_type(2)));
    __builtin_nontemporal_store(v2f{x, y}, reinterpret_cast<v2f *>(p));
}
template <typename T>
__device__ __forceinline__ void store2_nt(T *p, float x, float y)
{
    static_assert(sizeof(T) == 2, "a 16-bit storage type");
    __builtin_nontemporal_store(pack_pair<T>(x, y), reinterpret_cast<uint32_t *>(p));
}
__device__ __forceinline__ void store4(float *p, const float4 &v) { *reinterpret_cast<float4 *>(p) = v; }
template <typename T>
__device__ __forceinline__ void store4(T *p, const float4 &v)
{
    *reinterpret_cast<uint2 *>(p) = make_uint2(pack_pair<T>(v.x, v.y), pack_pair<T>(v.z, v.w));
}
__device__ __forceinline__ void store1(float *p, float x) { *p = x; }
template <typename T>
__device__ __forceinline__ void store1(T *p, float x) { *p = from_f32<T>(x); }

// The output array has a run-time element type (KVB_F32 or the 16-bit input type TIn): the
// stores sit at the end of every kernel, where a uniform branch costs nothing.
template <typename TIn>
struct Out {
    void *p;
    bool wide;   // fp32 elements
    __device__ __forceinline__ void put1(size_t i, float x) const
    {
        if constexpr (sizeof(TIn) == 4) {
            static_cast<float *>(p)[i] = x;
        } else {
            if (wide)
                static_cast<float *>(p)[i] = x;
            else
                store1(static_cast<TIn *>(p) + i, x);
        }
    }
    __device__ __forceinline__ void put2(size_t i, float x, float y) const
    {
        if constexpr (sizeof(TIn) == 4) {
            store2(static_cast<float *>(p) + i, x, y);
        } else {
            if (wide)
                store2(static_cast<float *>(p) + i, x, y);
            else
                store2(static_cast<TIn *>(p) + i, x, y);
        }
    }
    __device__ __forceinline__ void put2_nt(size_t i, float x, float y) const
    {
        if constexpr (sizeof(TIn) == 4) {
            store2_nt(static_cast<float *>(p) + i, x, y);
        } else {
            if (wide)
                store2_nt(static_cast<float *>(p) + i, x, y);
            else
                store2_nt(static_cast<TIn *>(p) + i, x, y);
        }
    }
    __device__ __forceinline__ void put4(size_t i, const float4 &v) const
    {
        if constexpr (sizeof(TIn) == 4) {
            store4(static_cast<float *>(p) + i, v);
        } else {
            if (wide)
                store4(static_cast<float *>(p) + i, v);
            else
                store4(static_cast<TIn *>(p) + i, v);
        }
    }
};

// v_mfma_f32_16x16x32 on 16-bit operands of type T given as raw bits (8 elements per lane).
template <typename T>
__device__ __forceinline__ f32x4_t mfma16x32(const uint4 &a, const uint4 &b, const f32x4_t &c)
{
    if constexpr (__is_same(T, bf16_t))
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b),
                                                       c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b),
                                                      c, 0, 0, 0);
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

// The same for an 8-byte piece.
template <bool STREAM>
__device__ __forceinline__ float2 load_state2(const float *p)
{
    if constexpr (STREAM) {
        typedef float v2f __attribute__((ext_vector_type(2)));
        const v2f t = __builtin_nontemporal_load(reinterpret_cast<const v2f *>(p));
        return make_float2(t.x, t.y);
    } else {
        return *reinterpret_cast<const float2 *>(p);
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
template <typename T>
__device__ __forceinline__ void store_raw8(T *p, const Raw8<T> &r)
{
    *reinterpret_cast<uint4 *>(p) = r.w;
}

// Workgroup ids are dealt round-robin to the 8 XCDs (each with its own L2).  Map them so
// that XCD x works on one contiguous eighth of the (request, head) units: all heads of a
// request then share an L2, which keeps the per-request ticket atomics and the keys that
// grouped heads share inside one XCD.
__device__ __forceinline__ int logical_block(int n)
{
    const int x = blockIdx.x;
    return (n % 8 == 0) ? (x % 8) * (n / 8) + x / 8 : x;
}
__device__ __forceinline__ int logical_block() { return logical_block(gridDim.x); }

struct Store {
    float *state;
    void *buf_k;   // input type
    void *buf_u;   // record type
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
        __builtin_amdgcn_wave_barrier();   // the lookups below stay behind this store (same wave, so no more is needed)
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
    void *out;
    int32_t out_wide;   // fp32 outputs (otherwise the 16-bit input type)
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

struct FlushArgs {
    Store st;
    const int32_t *slot;
    const int32_t *accepted;
    int32_t Hk, Hv, cap, threshold;
    int32_t stream;   // non-temporal state loads and stores
};

struct DirectArgs {
    Store st;
    const int32_t *slot;
    const int32_t *len;
    const void *q, *k, *v;
    const float *g, *beta;
    void *out;
    int32_t out_wide;   // fp32 outputs (otherwise the 16-bit input type)
    int32_t Hk, Hv, cap, Lmax;
    float scale;
};

struct CompactArgs {
    Store st;
    const int32_t *slot;
    const int32_t *path;
    const int32_t *path_len;
    int32_t Hk, Hv, cap, T;
};

// ---------------------------------------------------------------------------
// launch plumbing (host)
// ---------------------------------------------------------------------------
// The timer that the calling thread armed for its next launch, and what its last launch
// returned (kvb_api.hip).
extern thread_local kvb_timer *g_armed;
extern thread_local hipError_t g_launch_status;

// One kernel launch.  If this thread armed a timer, the launch carries its two events so
// that they hold the kernel's own begin / end timestamps.  The runtime's return code is kept
// in g_launch_status (the runtime's "last error" is left alone: it may hold some other
// library's error, which is neither ours to report nor ours to clear).
template <typename... Params, typename... Args>
void launch(void (*kernel)(Params...), int blocks, hipStream_t stream, const Args &...a)
{
    static_assert(sizeof...(Params) == sizeof...(Args), "one argument per kernel parameter");
    std::tuple<std::remove_cv_t<Params>...> params{a...};
    void *argv[sizeof...(Params)];
    std::apply([&](auto &...p) { int i = 0; ((argv[i++] = &p), ...); }, params);
    kvb_timer *t = g_armed;
    g_armed = nullptr;
    if (t)
        g_launch_status = hipExtLaunchKernel(reinterpret_cast<const void *>(kernel), dim3(blocks), dim3(NT), argv, 0,
                                             stream, t->start, t->stop, 0);
    else
        g_launch_status = hipLaunchKernel(reinterpret_cast<const void *>(kernel), dim3(blocks), dim3(NT), argv, 0, stream);
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

// The same for kernels that take (slot, Hv, grid size) as three plain leading arguments ahead of the
// argument struct: the build preloads the first kernel-argument words into scalar registers at wave
// launch, so the load of slot[b] -- the head of every dependent chain -- goes out at once.
#define LAUNCH_LEAD(blocks, stream, a, ...)                                            \
    do {                                                                               \
        if ((a).st.block_table)                                                        \
            launch(__VA_ARGS__, true>, blocks, stream, (a).slot, (a).Hv, blocks, a);   \
        else                                                                           \
            launch(__VA_ARGS__, false>, blocks, stream, (a).slot, (a).Hv, blocks, a);  \
    } while (0)

// The compiled (input type, record type) pairs: fp32 records with any input type, 16-bit records
// of the input's own 16-bit type.  Calls f.template operator()<TIn, TRec>().
template <typename F>
int dispatch_types(int in_dtype, int rec_dtype, F &&f)
{
    const bool wide = rec_dtype == KVB_F32;
    if (in_dtype == KVB_F32 && wide)
        f.template operator()<float, float>();
    else if (in_dtype == KVB_BF16 && wide)
        f.template operator()<bf16_t, float>();
    else if (in_dtype == KVB_BF16 && rec_dtype == KVB_BF16)
        f.template operator()<bf16_t, bf16_t>();
    else if (in_dtype == KVB_F16 && wide)
        f.template operator()<f16_t, float>();
    else if (in_dtype == KVB_F16 && rec_dtype == KVB_F16)
        f.template operator()<f16_t, f16_t>();
    else
        return KVB_EUNSUPPORTED;
    return KVB_OK;
}
// The same for the 16-bit input types alone (the matrix-core kernels).
template <typename F>
int dispatch_types16(int in_dtype, int rec_dtype, F &&f)
{
    const bool wide = rec_dtype == KVB_F32;
    if (in_dtype == KVB_BF16 && wide)
        f.template operator()<bf16_t, float>();
    else if (in_dtype == KVB_BF16 && rec_dtype == KVB_BF16)
        f.template operator()<bf16_t, bf16_t>();
    else if (in_dtype == KVB_F16 && wide)
        f.template operator()<f16_t, float>();
    else if (in_dtype == KVB_F16 && rec_dtype == KVB_F16)
        f.template operator()<f16_t, f16_t>();
    else
        return KVB_EUNSUPPORTED;
    return KVB_OK;
}

// Calls f.template operator()<D, TIn, TRec>() for the compiled head sizes and type pairs.
template <typename F>
int dispatch(int dk, int in_dtype, int rec_dtype, F &&f)
{
    if (dk != 32 && dk != 64 && dk != 128)
        return KVB_EUNSUPPORTED;
    return dispatch_types(in_dtype, rec_dtype, [&]<typename TIn, typename TRec>() {
        if (dk == 32)
            f.template operator()<32, TIn, TRec>();
        else if (dk == 64)
            f.template operator()<64, TIn, TRec>();
        else
            f.template operator()<128, TIn, TRec>();
    });
}

// One launcher per translation unit.  They return KVB_EUNSUPPORTED for a head size or type pair
// that is not compiled; none of them checks the launch (the caller does).
template <typename TIn, typename TRec>
int launch_step_typed(int dk, const StepArgs &a, int blocks, hipStream_t stream);   // kvb_step_*.hip, one unit per pair
template <typename TIn, typename TRec>
void launch_verify_typed(const StepArgs &a, int blocks, hipStream_t stream);        // kvb_verify_*.hip (16-bit inputs, d = 128)
int launch_flush(int dk, int in_dtype, int rec_dtype, const FlushArgs &a, int blocks, hipStream_t stream);    // kvb_flush.hip
int launch_compact(int dk, int in_dtype, int rec_dtype, const CompactArgs &a, int blocks, hipStream_t stream);
int launch_direct(int dk, int in_dtype, int rec_dtype, const DirectArgs &a, int blocks, hipStream_t stream);  // kvb_direct.hip

}  // namespace kvb_impl
#endif  // KVB_DEVICE_H
