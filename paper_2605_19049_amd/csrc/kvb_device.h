// kvb -- KVBuffer-style Gated DeltaNet decoding, HIP kernels for gfx950 behind the C ABI of
// include/kvb.h.  This header holds what the translation units share: device helpers, the
// argument structs of the kernels, and the launch plumbing.
//   kvb_step_kernel.h, kvb_step_bf16.hip, kvb_step_f32.hip
//                   kvb_step_kernel (decode and the vector-ALU verify), one unit per input type
//   kvb_verify.hip  kvb_verify_mfma_kernel
//   kvb_flush.hip   kvb_flush_kernel, kvb_compact_kernel
//   kvb_direct.hip  kvb_direct_mfma_kernel, kvb_direct_kernel
//   kvb_api.hip     argument checks, the extern "C" entry points, the kernel timer
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

#ifndef KVB_DEVICE_H
#define KVB_DEVICE_H

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

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
__device__ __forceinline__ int logical_block(int n)
{
    const int x = blockIdx.x;
    return (n % 8 == 0) ? (x % 8) * (n / 8) + x / 8 : x;
}
__device__ __forceinline__ int logical_block() { return logical_block(gridDim.x); }

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

struct FlushArgs {
    Store st;
    const int32_t *slot;
    const int32_t *accepted;
    int32_t Hk, Hv, cap, threshold;
};

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

struct CompactArgs {
    Store st;
    const int32_t *slot;
    const int32_t *path;
    const int32_t *path_len;
    int32_t Hk, Hv, cap, T;
};

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

// ---------------------------------------------------------------------------
// launch plumbing (host)
// ---------------------------------------------------------------------------
// The timer that the calling thread armed for its next launch (kvb_api.hip).
extern thread_local kvb_timer *g_armed;

// One kernel launch.  If this thread armed a timer, the launch carries its two events so
// that they hold the kernel's own begin / end timestamps.
template <typename... Params, typename... Args>
void launch(void (*kernel)(Params...), int blocks, hipStream_t stream, const Args &...a)
{
    kvb_timer *t = g_armed;
    g_armed = nullptr;
    if (t)
        hipExtLaunchKernelGGL(kernel, dim3(blocks), dim3(NT), 0, stream, t->start, t->stop, 0, a...);
    else
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(NT), 0, stream, a...);
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

// Calls f.template operator()<D, TIn>() for the compiled (head size, dtype) pairs.
template <typename F>
int dispatch(int dk, int in_dtype, F &&f)
{
    const bool bf = in_dtype == KVB_BF16;
    switch (dk) {
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

// One launcher per translation unit.  Those that take (dk, in_dtype) return KVB_EUNSUPPORTED
// for a pair that is not compiled; none of them checks the launch (the caller does).
int launch_step_bf16(int dk, const StepArgs &a, int blocks, hipStream_t stream);                // kvb_step_bf16.hip
int launch_step_f32(int dk, const StepArgs &a, int blocks, hipStream_t stream);                 // kvb_step_f32.hip
void launch_verify_mfma(const StepArgs &a, int blocks, hipStream_t stream);                    // kvb_verify.hip (bf16, d = 128)
int launch_flush(int dk, int in_dtype, const FlushArgs &a, int blocks, hipStream_t stream);    // kvb_flush.hip
int launch_compact(int dk, int in_dtype, const CompactArgs &a, int blocks, hipStream_t stream);
int launch_direct(int dk, int in_dtype, const DirectArgs &a, int blocks, hipStream_t stream);  // kvb_direct.hip

}  // namespace kvb_impl
#endif  // KVB_DEVICE_H
