// Host side of the library: argument checks (all before the first HIP call), the extern "C" entry
// points of include/kvb.h, the kernel timer.
#include "kvb_device.h"

namespace kvb_impl {

thread_local kvb_timer *g_armed = nullptr;
thread_local hipError_t g_launch_status = hipSuccess;

}  // namespace kvb_impl

using namespace kvb_impl;

namespace {

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
    if (sh->in_dtype != KVB_F32 && sh->in_dtype != KVB_BF16 && sh->in_dtype != KVB_F16)
        return KVB_EUNSUPPORTED;
    // records and outputs: fp32, or the 16-bit type of the inputs
    if (sh->out_dtype != KVB_F32 && (sh->in_dtype == KVB_F32 || sh->out_dtype != sh->in_dtype))
        return KVB_EUNSUPPORTED;
    if (sh->rec_dtype != KVB_F32 && (sh->in_dtype == KVB_F32 || sh->rec_dtype != sh->in_dtype))
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
// call's own state footprint against the 256 MB last-level cache.  For decoding and verification
// the switch sits at 288 MiB: a state of 256 MiB re-read every step still finds most of itself
// in the cache and runs faster with plain loads (kvb_decode_flush at C = 16: 49 against 53 us per
// step), at 288 MiB the two are level (59 us), at 320 MiB streaming wins (65 against 71).  kvb_flush
// reads and writes the state, twice the lines through the cache: measured, streaming wins from
// about 200 MiB of state on (16 records: 65 against 71 us at 192 MiB, 88 against 84 at 224 MiB;
// 64 records: 139 against 107 us at 256 MiB), so its switch sits at 192 MiB.
bool stream_state(const kvb_shape *sh, const kvb_store *st, double limit_mib = 288.0)
{
    if (st->flags & KVB_STORE_STREAM)
        return true;
    if (st->flags & KVB_STORE_RESIDENT)
        return false;
    const double bytes = 4.0 * sh->B * sh->Hv * sh->dk * sh->dv;
    return bytes > limit_mib * 1024 * 1024;
}

Store dev_store(const kvb_store *st)
{
    return Store{st->state, st->buf_k, st->buf_u, st->buf_G, st->fill, st->status, st->n_slots,
                 st->block_table, st->block_table ? st->block_size : 0, st->block_table ? st->max_blocks : 1,
                 st->block_table ? st->n_blocks : 0};
}

// The status of the launch this thread has just made (what the launch call itself returned:
// an error some other library left behind in the runtime is neither reported nor cleared).
int finish_launch()
{
    const hipError_t e = g_launch_status;
    if (e != hipSuccess) {
        g_last_hip_error = e;
        return KVB_EHIP;
    }
    return KVB_OK;
}

// Every compute entry point ends with no timer armed: a call that returns before it launches
// (bad arguments, B = 0) must not leave its timer to some later, unrelated launch.
struct DisarmOnExit {
    ~DisarmOnExit() { g_armed = nullptr; }
};

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
    StepArgs a{dev_store(st), slot, q, k, v, g, beta, out, sh->out_dtype == KVB_F32, sh->Hk, sh->Hv, sh->cap, T,
               sh->scale, advance, threshold, stream_state(sh, st) ? 1 : 0,
               // chain: g stands in as a readable array of at least B*T words whose values are ignored
               parent ? parent : reinterpret_cast<const int32_t *>(g), parent ? 1 : 0};
    const int blocks = sh->B * sh->Hv;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    g_launch_status = hipSuccess;
    if (sh->dk == 128 && sh->in_dtype != KVB_F32 && T > 1)   // several drafts: the matrix-core kernel
        rc = dispatch_types16(sh->in_dtype, sh->rec_dtype,
                              [&]<typename TIn, typename TRec>() { launch_verify_typed<TIn, TRec>(a, blocks, hs); });
    else
        rc = dispatch_types(sh->in_dtype, sh->rec_dtype, [&]<typename TIn, typename TRec>() {
            launch_step_typed<TIn, TRec>(sh->dk, a, blocks, hs);   // (the head size was checked above)
        });
    if (rc != KVB_OK)
        return rc;
    return finish_launch();
}

}  // namespace

extern "C" {

int kvb_decode(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, const void *q, const void *k,
               const void *v, const float *g, const float *beta, void *out, void *stream)
{
    DisarmOnExit disarm;
    return step_common(shape, store, slot, 1, q, k, v, g, beta, out, stream, 1);
}

int kvb_decode_flush(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, const void *q,
                     const void *k, const void *v, const float *g, const float *beta, void *out,
                     int32_t threshold, void *stream)
{
    DisarmOnExit disarm;
    if (!shape || !store)
        return KVB_EINVAL;
    if (!store->state || threshold < 1 || threshold > shape->cap)
        return KVB_EINVAL;
    return step_common(shape, store, slot, 1, q, k, v, g, beta, out, stream, 1, threshold);
}

int kvb_verify(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, int32_t T, const void *q,
               const void *k, const void *v, const float *g, const float *beta, void *out, void *stream)
{
    DisarmOnExit disarm;
    return step_common(shape, store, slot, T, q, k, v, g, beta, out, stream, 0);
}

int kvb_verify_tree(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, int32_t T,
                    const int32_t *parent, const void *q, const void *k, const void *v, const float *g,
                    const float *beta, void *out, void *stream)
{
    DisarmOnExit disarm;
    if (!parent || !aligned(parent, 4))
        return KVB_EINVAL;
    return step_common(shape, store, slot, T, q, k, v, g, beta, out, stream, 0, 0, parent);
}

int kvb_compact(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, int32_t T,
                const int32_t *path, const int32_t *path_len, void *stream)
{
    DisarmOnExit disarm;
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
    g_launch_status = hipSuccess;
    rc = launch_compact(shape->dk, shape->in_dtype, shape->rec_dtype, a, blocks, hs);
    if (rc != KVB_OK)
        return rc;
    return finish_launch();
}

int kvb_flush(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, const int32_t *accepted,
              int32_t threshold, void *stream)
{
    DisarmOnExit disarm;
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
    FlushArgs a{dev_store(store), slot, accepted, shape->Hk, shape->Hv, shape->cap, threshold,
                store->state && stream_state(shape, store, 192.0) ? 1 : 0};
    const int blocks = shape->B * shape->Hv;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    g_launch_status = hipSuccess;
    rc = launch_flush(shape->dk, shape->in_dtype, shape->rec_dtype, a, blocks, hs);
    if (rc != KVB_OK)
        return rc;
    return finish_launch();
}

int kvb_direct(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, const int32_t *len,
               int32_t Lmax, const void *q, const void *k, const void *v, const float *g, const float *beta,
               void *out, void *stream)
{
    DisarmOnExit disarm;
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
    DirectArgs a{dev_store(store), slot, len, q, k, v, g, beta, out, shape->out_dtype == KVB_F32, shape->Hk,
                 shape->Hv, shape->cap, Lmax, shape->scale};
    const int blocks = shape->B * shape->Hv;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    g_launch_status = hipSuccess;
    rc = launch_direct(shape->dk, shape->in_dtype, shape->rec_dtype, a, blocks, hs);
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
        (void)hipGetLastError();   // (as in kvb_timer_read)
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
        (void)hipGetLastError();   // this call's own error: not left behind for the caller's next HIP call
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
