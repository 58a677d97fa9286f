/*
 * kvb -- KVBuffer-style Gated DeltaNet decoding for AMD MI355X (gfx950).
 *
 * C ABI of the library.  Every pointer marked "device" is device memory owned
 * by the caller; the compute calls never allocate, free or synchronise, and
 * enqueue all work on the caller's HIP stream (`stream` is a hipStream_t passed
 * as void*; NULL = the default stream).  The two structs are host memory and are
 * read only during the call.  The only state the library keeps is two
 * thread-local words on the host: the timer armed for the calling thread's next
 * launch (kvb_timer_arm) and the HIP error code behind the last KVB_EHIP.
 *
 * Notation (paper Sec. 2.1, Sec. 3, App. A.1).  For one request and one v-head:
 *   S0    the committed state, dk x dv, fp32                (the "state slot", Sec. 2.2)
 *   f     number of records in the request's buffer         ("fill")
 *   record l (0 <= l < f) = ( k_l, u_l, G_l ):
 *         k_l  key of the l-th token since the last flush
 *         u_l  its delta value (the quantity the paper buffers instead of v)
 *         G_l  sum of the log decays g of tokens 0..l of the chunk, so that
 *              gamma_l = exp(G_l) and Gamma_{il} = exp(G_i - G_l) <= 1 for i >= l
 *   For a new token at chunk position i (App. A.1, Eq. 16):
 *         u_i = beta_i ( v_i - gamma_i k_i S0 - sum_{l<i}  Gamma_{il} (k_i.k_l) u_l )
 *         o_i = scale  ( gamma_i q_i S0       + sum_{l<=i} Gamma_{il} (q_i.k_l) u_l )
 *         S   = gamma_m-1 S0 + sum_{l<m} Gamma_{m-1,l} k_l^T u_l          (flush of m records)
 *   which is exactly the token-by-token recurrence of Eq. 11-12 regrouped.
 *
 * Grouped heads: v-head h uses the q and k of qk-head h / (Hv / Hk).
 * The gate is passed as a log decay g <= 0 (alpha = exp(g)); gamma ratios are
 * never formed, only exp of differences.
 */
#ifndef KVB_H
#define KVB_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KVB_VERSION 120 /* 120: fp16 inputs, 16-bit delta-value records and outputs (kvb_shape.rec_dtype) */

/* return codes */
#define KVB_OK            0
#define KVB_EINVAL       (-1) /* null / misaligned pointer, size out of range          */
#define KVB_EUNSUPPORTED (-2) /* head size or dtype combination that is not compiled    */
#define KVB_EHIP         (-3) /* the HIP runtime refused the launch                     */

/* element types: of q, k, v and the buffered keys (in_dtype), of the buffered delta values
 * (rec_dtype) and of the outputs (out_dtype).  The paper's implementation keeps a fp32 state
 * and fp16 vectors and records (Sec. 4.1; caption of the GDN memory-profile table, App. A.2):
 * that is in = rec = out = KVB_F16.  A 16-bit rec_dtype or out_dtype must equal in_dtype;
 * KVB_F32 is always allowed for both.  The state is fp32 throughout. */
#define KVB_F32  0
#define KVB_BF16 1
#define KVB_F16  2
/* Which (in_dtype, head size) pairs are tuned.  d = 128 with KVB_BF16 or KVB_F16 inputs (any
 * allowed rec_dtype / out_dtype) is the pair the kernels are built and measured for: matrix-
 * instruction kernels for kvb_verify, kvb_verify_tree, kvb_flush and kvb_direct, the streaming
 * decode kernel for kvb_decode / kvb_decode_flush.  KVB_F32 inputs at any head size, and
 * d = 32 or 64 with any input type, run plain vector-ALU kernels that exist for correctness
 * (the fp32 parity workload, small test shapes): same results, no performance claim, and
 * kvb_direct is limited to 64 tokens there. */

#define KVB_MAX_CAP        128 /* largest `cap` (the paper buffers at most d records, Sec. 3.4) */
#define KVB_MAX_DRAFTS       8 /* largest T of kvb_verify (Sec. 4.2 sweeps up to 8)             */
#define KVB_MAX_DIRECT_LEN 128 /* largest Lmax of kvb_direct (Sec. 3.4: contexts up to d tokens);
                                  16-bit inputs with d = 128; the other compiled pairs take 64   */
#define KVB_MAX_BLOCKS      16 /* longest block-table row (KVB_MAX_CAP / smallest block)        */

/* kvb_store.flags: how the state should travel through the caches.  With neither bit the
 * library streams (non-temporal loads, and non-temporal stores when the state is written
 * back) when the states one call touches, 4 * B * Hv * dk * dv bytes, exceed 288 MiB: a little
 * more than the 256 MB last-level cache, because a state of 256 MiB that is re-read every
 * step still finds most of itself there; kvb_flush, which passes the state through the cache
 * in both directions, switches at 192 MiB.  A model with many GDN layers should set
 * KVB_STORE_STREAM: each layer's state is next read one token later, after every other
 * layer's has passed through. */
#define KVB_STORE_STREAM   1
#define KVB_STORE_RESIDENT 2

/* bits set in status[slot]: a call would have overrun that request's buffer; a draft tree or
 * an accepted path handed to kvb_verify_tree / kvb_compact was not well formed */
#define KVB_STATUS_OVERFLOW 1
#define KVB_STATUS_BADPATH  2

typedef struct kvb_shape {
    int32_t B;         /* requests in this call (0 = no-op)                                */
    int32_t Hk;        /* q/k heads                                                        */
    int32_t Hv;        /* v heads, Hv % Hk == 0                                            */
    int32_t dk;        /* key/query head size;   compiled: dk == dv in {32, 64, 128}       */
    int32_t dv;        /* value head size                                                  */
    int32_t cap;       /* records one request's buffer can hold, 1..KVB_MAX_CAP            */
    int32_t in_dtype;  /* KVB_F32, KVB_BF16 or KVB_F16: type of q, k, v and of buf_k       */
    int32_t out_dtype; /* type of `out`: KVB_F32, or in_dtype if that is a 16-bit type     */
    int32_t rec_dtype; /* type of buf_u: KVB_F32, or in_dtype if that is a 16-bit type.    */
                       /* A 16-bit record holds the delta value rounded to nearest even;   */
                       /* every later use (the token's own output included) reads that     */
                       /* rounded value, so a record is all that later calls depend on.    */
    float   scale;     /* multiplies every output (1.0 = the paper's formulas)             */
} kvb_shape;

typedef struct kvb_store {
    float   *state;   /* device [n_slots, Hv, dk, dv] fp32, dv contiguous.  May be NULL for
                         kvb_decode / kvb_verify: KV-only mode, S0 taken as zero (Sec. 3.4). */
    void    *buf_k;   /* device [n_slots, Hk, cap, dk] in_dtype                             */
    void    *buf_u;   /* device [n_slots, Hv, cap, dv] rec_dtype                            */
    float   *buf_G;   /* device [n_slots, Hv, cap]     fp32                                 */
    int32_t *fill;    /* device [n_slots]; 0..cap between calls.  While a call that changes
                         fill runs, bits 16.. of the word count the workgroups that have
                         read it; the last one stores the new fill, so the word is a plain
                         count again when the call's kernel ends.                           */
    int32_t *status;  /* device [n_slots] sticky KVB_STATUS_* bits, or NULL                 */
    int32_t  n_slots; /* slots in the arrays above; requests whose slot is outside
                         0..n_slots-1 are skipped                                           */
    int32_t  flags;   /* KVB_STORE_* hints, 0 = let the library decide                      */
    /* Paged record buffers (Sec. 3.1: a request's buffer is made of blocks of 8 or 16 records
     * drawn from a pool shared by all requests).  block_table == NULL (and the three sizes 0):
     * the layout above, one block of cap records per slot.  Otherwise record l of slot s lives
     * in block block_table[s][l / block_size] at position l % block_size, and the record
     * arrays are pools of n_blocks blocks:
     *   buf_k [n_blocks, Hk, block_size, dk]   buf_u [n_blocks, Hv, block_size, dv]
     *   buf_G [n_blocks, Hv, block_size]
     * state, fill and status stay per slot.  Only the entries that cover records 0..cap-1 are
     * read; ids outside 0..n_blocks-1 are clamped into the pool.  Two requests of one call must
     * not share a block.                                                                     */
    const int32_t *block_table; /* device [n_slots, max_blocks] or NULL                       */
    int32_t  block_size;        /* 8, 16, 32, 64 or 128 records                               */
    int32_t  max_blocks;        /* 1..KVB_MAX_BLOCKS, block_size * max_blocks >= cap          */
    int32_t  n_blocks;          /* blocks in the pools                                        */
} kvb_store;

/*
 * All compute calls take `slot`: device int32 [B], the store slot of request b.
 * A slot must not appear twice in one call.  state, buf_k, buf_u, q, k, v and
 * out must be 16-byte aligned; the int32 / float vectors 4-byte aligned.
 */

/*
 * kvb_decode -- chunkwise decoding of ONE new token per request (Sec. 3.2; the
 * single-token chunkwise form, App. A.1 Eq. 16; with store->state == NULL the
 * single-token parallel form, Eq. 14).  Reads S0 and records 0..f-1, writes the
 * output and record f = (k, u, G_f), then fill = f + 1.  Never writes `state`.
 *   q, k  device [B, Hk, dk] in_dtype      v    device [B, Hv, dv] in_dtype
 *   g     device [B, Hv] fp32 log decay    beta device [B, Hv] fp32
 *   out   device [B, Hv, dv] out_dtype
 * A request with f == cap is skipped: its out row and buffer are left as they
 * are and status[slot] gets KVB_STATUS_OVERFLOW.
 */
int kvb_decode(const kvb_shape *shape, const kvb_store *store, const int32_t *slot,
               const void *q, const void *k, const void *v,
               const float *g, const float *beta, void *out, void *stream);

/*
 * kvb_decode_flush -- kvb_decode followed by kvb_flush(accepted = NULL, threshold), in one
 * pass (the paper launches the state update as a second kernel, Sec. 4.2; here a request
 * whose buffer reaches `threshold` records with this token has its state updated from the
 * tile the decode step has already read, which saves re-reading it).  Same arguments,
 * results and error behaviour as the two calls in sequence; state must not be NULL;
 * threshold 1..cap (threshold 1 is the fused recurrent step: every token is folded at once).
 */
int kvb_decode_flush(const kvb_shape *shape, const kvb_store *store, const int32_t *slot,
                     const void *q, const void *k, const void *v,
                     const float *g, const float *beta, void *out,
                     int32_t threshold, void *stream);

/*
 * kvb_flush -- the deferred, batched state update (Sec. 3.2, Eq. 5; for GDN the
 * last line of App. A.1 Eq. 16; with `accepted` the accepted-only update of
 * Sec. 3.3 Eq. 8).  For request b: m = fill + (accepted ? accepted[b] : 0); if
 * m >= threshold and m > 0:  S <- exp(G_{m-1}) S + sum_l exp(G_{m-1} - G_l) k_l^T u_l
 * and fill = 0; otherwise fill = m and the state is untouched.  Besides
 * kvb_decode_flush the only call that writes `state`.
 * On a zeroed state this is the KV-only -> state transition of Sec. 3.4.
 * state == NULL (a KV-only context): nothing is folded, the call only commits the accepted
 * drafts of a preceding kvb_verify (fill = m); `accepted` must then be given.
 *   accepted  device int32 [B] (each 0..T of the preceding kvb_verify) or NULL
 *   threshold 1..cap; 1 flushes every non-empty buffer
 * m > cap sets KVB_STATUS_OVERFLOW and is treated as cap.
 */
int kvb_flush(const kvb_shape *shape, const kvb_store *store, const int32_t *slot,
              const int32_t *accepted, int32_t threshold, void *stream);

/*
 * kvb_verify -- parallel verification of T sequential draft tokens per request
 * (Sec. 3.3, Eq. 7; for GDN the chunkwise matrix form App. A.1 Eq. 15 restricted
 * to rows f..f+T-1).  One pass over S0 serves all T drafts; no temporary state
 * is formed.  Writes T outputs and records f..f+T-1 but leaves `fill` (and
 * `state`) untouched: committing is kvb_flush(accepted, ...).
 *   T     1..KVB_MAX_DRAFTS
 *   q, k  device [B, T, Hk, dk]   v device [B, T, Hv, dv]   g, beta device [B, T, Hv]
 *   out   device [B, T, Hv, dv] out_dtype
 * A request with f + T > cap is skipped with KVB_STATUS_OVERFLOW.
 */
int kvb_verify(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, int32_t T,
               const void *q, const void *k, const void *v,
               const float *g, const float *beta, void *out, void *stream);

/*
 * kvb_verify_tree -- kvb_verify for drafts that form a tree (Sec. 3.3: the mask M and the
 * prefix set Par(t) of App. A.1 admit any draft structure; the figure of Sec. 3.3 accepts
 * drafts 0 and 2 of three).  Draft i continues the committed context and then exactly its
 * ancestors among the T drafts: its decay, its delta value and its output are those of the
 * root path that ends in i.  With parent[b][i] = i - 1 this is kvb_verify.
 *   parent  device int32 [B, T]: parent[b][i] in {-1, 0 .. i-1}; -1 = the draft follows the last
 *           committed token.  Parents precede their children.  An entry outside that range is
 *           taken as -1 and status[slot] gets KVB_STATUS_BADPATH.  T = 1: not read.
 * Everything else as kvb_verify: record f + i holds draft i (its G is cumulative along its own
 * path), fill and state are untouched.  Committing an accepted root path is kvb_compact followed
 * by kvb_flush(accepted = path_len).
 */
int kvb_verify_tree(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, int32_t T,
                    const int32_t *parent, const void *q, const void *k, const void *v,
                    const float *g, const float *beta, void *out, void *stream);

/*
 * kvb_compact -- makes the accepted drafts of a tree a prefix of the T new records (Sec. 3.3,
 * Eq. 8: only accepted tokens reach the state).  For request b the records at f + path[b][j]
 * move to f + j, j = 0 .. path_len[b]-1; the caller then commits them with
 * kvb_flush(accepted = path_len, ...).  Neither fill nor state changes here.
 *   T         the T of the preceding kvb_verify_tree
 *   path      device int32 [B, T]: the accepted root path, oldest draft first, strictly increasing
 *             node indices in 0 .. T-1 (the caller passes a path of the tree; only its order and
 *             range are checked)
 *   path_len  device int32 [B]: 0 .. T accepted drafts
 * A path that is not increasing, a length outside 0..T, or f + T > cap leaves the request's
 * records as they are and sets KVB_STATUS_BADPATH.
 */
int kvb_compact(const kvb_shape *shape, const kvb_store *store, const int32_t *slot, int32_t T,
                const int32_t *path, const int32_t *path_len, void *stream);

/*
 * kvb_direct -- state-free computation of a whole short context from its keys
 * and values (Sec. 3.4; the parallel form App. A.1 Eq. 13).  For request b the
 * first len[b] tokens are processed from a zero state: outputs for every
 * position, records 0..len[b]-1, fill = len[b] (whatever the buffer held before
 * is discarded).  `state` is neither read nor written.  Decoding then continues
 * with kvb_decode (state NULL), and kvb_flush on a zeroed state folds the
 * records into a state once the context outgrows the buffer.
 *   len   device int32 [B], 0..Lmax        Lmax 1..min(cap, KVB_MAX_DIRECT_LEN); above 64 only for
 *         16-bit inputs with d = 128 (KVB_EUNSUPPORTED otherwise)
 *   q, k  device [B, Lmax, Hk, dk]  v device [B, Lmax, Hv, dv]  g, beta device [B, Lmax, Hv]
 *   out   device [B, Lmax, Hv, dv] out_dtype; rows >= len[b] are not written
 * len[b] outside 0..Lmax is clamped to Lmax with KVB_STATUS_OVERFLOW.
 * With a 16-bit rec_dtype the outputs read the records as stored (rounded), like everywhere
 * else; the delta values themselves are solved for in fp32 before they are rounded -- all
 * rows at once up to 64 tokens, 16 rows at a time above that -- so a row's delta value does
 * not see the rounding of the rows solved with it.
 */
int kvb_direct(const kvb_shape *shape, const kvb_store *store, const int32_t *slot,
               const int32_t *len, int32_t Lmax,
               const void *q, const void *k, const void *v,
               const float *g, const float *beta, void *out, void *stream);

/*
 * Kernel timer (measurement aid, no part of the method).  A timer owns two HIP events.
 * kvb_timer_arm makes the NEXT kernel that the calling thread launches through this
 * library record its own begin and end timestamps into them; kvb_timer_read waits for that
 * kernel and returns its duration.  Timers are host objects: create / destroy allocate and
 * free them, the only allocation this library ever performs.  Do not arm during stream capture.
 */
typedef struct kvb_timer kvb_timer;
int  kvb_timer_create(kvb_timer **timer);
int  kvb_timer_arm(kvb_timer *timer);          /* NULL disarms */
int  kvb_timer_read(kvb_timer *timer, float *microseconds);
void kvb_timer_destroy(kvb_timer *timer);

/* Static text for a return code (for KVB_EHIP: the last HIP error string of this thread). */
const char *kvb_strerror(int code);

/* KVB_VERSION of the built library. */
int kvb_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVB_H */
