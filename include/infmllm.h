/*
 * infmllm.h -- C ABI of the MI355X-native streaming step of Inf-MLLM (arxiv 2409.09086).
 *
 * One stream object is one layer of one sequence: a KV cache held to a fixed budget
 * B = r + R (r relevant tokens chosen by attention weight, R most recent tokens).
 * Each call of infmllm_step is one prompt arrival of Sec. 3.2: the chunk's K/V are
 * appended to the t cached rows, the chunk's L queries attend all n = t + L keys, the
 * column-mean attention weight plus the attention bias of Sec. 3.3 ranks the n - R older
 * keys, and the cache is compressed to the r best of them plus the R newest (Alg. 1).
 *
 * Conventions that hold for every entry point:
 *   - "device" pointers address HIP device memory of the GPU that is current when
 *     infmllm_stream_attach is called; "host" pointers address ordinary host memory.
 *   - The library never allocates or frees device memory.  All device memory, including
 *     the workspace that holds the cache, is the caller's and must stay valid until the
 *     attached HIP stream has passed the last call that used it.
 *   - Calls only enqueue work on the attached HIP stream and return; none waits for the
 *     device except infmllm_stream_profile_read.
 *   - Every function that returns int returns INFMLLM_OK or a negative INFMLLM_E* code and
 *     never throws or aborts; infmllm_last_error() gives a message for the calling thread's
 *     last failure.  A call refused for its arguments or for the stream's state (EINVAL, ENOMEM,
 *     ECAPACITY, ESTATE) leaves the stream as it was.  EHIP means a HIP call or a kernel launch
 *     failed part-way through the call's launches: the host counters (length, tokens streamed) are
 *     not advanced, but cache rows may already have been written, so the stream's contents are
 *     undefined from then on and the only calls that make sense are infmllm_stream_import (which
 *     replaces the cache) and infmllm_stream_destroy.  infmllm_evict_batched commits its streams
 *     in groups of 16; after EHIP the groups before the failing one are complete.
 *   - A stream is not thread-safe; different streams may be used from different threads.
 *   - Tensors are dense, row-major, token-major: q and out are [chunk_len, heads, head_dim],
 *     k and v are [chunk_len, kv_heads, head_dim], in the stream's dtype.
 */
#ifndef INFMLLM_H
#define INFMLLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct infmllm_stream infmllm_stream_t; /* opaque, library-owned host object */

enum { INFMLLM_BF16 = 0, INFMLLM_FP32 = 1 };

enum {
    INFMLLM_OK = 0,
    INFMLLM_EINVAL = -1,    /* bad argument (range, null pointer, unsupported shape)        */
    INFMLLM_ENOMEM = -2,    /* workspace too small / host allocation failed                 */
    INFMLLM_ECAPACITY = -3, /* chunk_len exceeds the stream's max_chunk                     */
    INFMLLM_ESTATE = -4,    /* call not allowed in this state (step before attach, ...)     */
    INFMLLM_EHIP = -5       /* a HIP call or kernel launch failed                           */
};

enum {
    INFMLLM_PARAM_BIAS = 0,      /* b of Alg. 1 (attention bias, Sec. 3.3); default 1e-4, the
                                    value Sec. 4.2 uses                                      */
    INFMLLM_PARAM_SCALE = 1,     /* softmax scale on q.k; default 1/sqrt(head_dim)           */
    INFMLLM_PARAM_MAX_CHUNK = 2, /* largest chunk_len a step may carry; default = budget.
                                    Fixes the cache capacity at budget + max_chunk rows      */
    INFMLLM_PARAM_MAX_DECODE = 4,/* tokens that may be decoded (infmllm_decode) between two chunk
                                    steps; default 0.  The cache may then hold up to budget +
                                    max_decode rows and its capacity grows by as much              */
    INFMLLM_PARAM_POLICY = 5,    /* which score the selection (Alg. 1 l.5) ranks; the methods Inf-MLLM is
                                    compared with (Sec. 2, Sec. 4.1) as modes of the same kernels:
                                    0 (default) W' = S + D of Alg. 1;
                                    1 window: W'[j] = j, the cache is the newest `budget` tokens;
                                    2 initial + recent: W'[j] = -j, the budget - recent oldest cached
                                      tokens and the `recent` newest;
                                    3 cumulative: W'[j] = A[j] + S[j], A = the W' a row was retained
                                      with in earlier steps (0 if never ranked); b is not applied.
                                    Modes 1 and 2 launch no scoring kernel                         */
    INFMLLM_PARAM_ROPE_BASE = 6, /* cache-relative rotary position encoding (Sec. 3.4, length extrapolation):
                                    0 (default) off; a value > 1 is the base of the rotary angles.  q and k
                                    are then passed unrotated; for every attention the key in cache row j is
                                    turned to position j and the query of chunk row i to position t + i
                                    (pairs (x[i], x[i + head_dim/2]), angle p * base^(-2i/head_dim)), so
                                    relative distances never exceed the cache size.  Costs one extra pass over
                                    the cached keys per step and workspace for the turned copies     */
    INFMLLM_PARAM_IMPL = 3,      /* debug/test: 0 (default) = bf16 streams run attention and
                                    scoring on the matrix cores; 1 = every dtype runs the
                                    plain fp32-arithmetic kernels (fp32 streams always do)   */
    INFMLLM_PARAM_ATTN_TILE = 7  /* debug/test, head_dim 128 on the matrix cores: 0 (default) = the
                                    attention launch picks its workgroup shape from the chunk length;
                                    1 = 128 query rows x 2 key ways x 64 keys, 2 = 64 rows x 4 ways x 32,
                                    3 = 128 rows x 2 ways x 32, 4 = 128 rows x 1 way x 64, 5 = 256 rows with
                                    64 rows per wavefront.  Results are the same up to rounding order  */
};

/*
 * Creates a stream (Alg. 1 inputs: retrieval/recent window, number of relevant tokens,
 * given here as budget = r + recent).  Host-only: touches no device.
 *   budget   1..131072  rows kept after every step (B)
 *   recent   0..budget  newest rows that are always kept (R); r = budget - recent
 *   heads    query heads; kv_heads divides heads (grouped-query attention pools the
 *            heads/kv_heads query heads of a group by their mean before ranking)
 *   head_dim 64 or 128
 *   dtype    INFMLLM_BF16 or INFMLLM_FP32 (element type of q, k, v, out and of the cache)
 *   out      receives the handle; the caller releases it with infmllm_stream_destroy
 * Errors: EINVAL for any argument out of range, ENOMEM if the host object cannot be made.
 */
int infmllm_stream_create(int budget, int recent, int heads, int kv_heads, int head_dim,
                          int dtype, infmllm_stream_t** out);

/*
 * Sets b, the softmax scale, max_chunk, max_decode or the kernel family (Alg. 1 input b;
 * Sec. 3.3).  Only before infmllm_stream_attach (ESTATE afterwards: the parameters size the
 * workspace, so they are fixed earlier than the first step).  EINVAL for an unknown
 * parameter, a non-finite value, bias < 0, scale <= 0, max_chunk < 1, max_decode < 0 or impl
 * outside {0, 1}.  bias and scale are kept in double; a kernel receives the constant it needs
 * (scale * log2(e), the ramp step b / c of Alg. 1 l.2) formed in double and rounded once to float.
 */
int infmllm_stream_set_param(infmllm_stream_t* s, int which, double value);

/* Bytes of device workspace the stream needs with its current parameters (0 if s is null). */
size_t infmllm_stream_workspace_bytes(const infmllm_stream_t* s);

/*
 * Hands the stream its device workspace (256-byte aligned, at least
 * infmllm_stream_workspace_bytes(s) bytes, caller-owned) and the HIP stream (a
 * hipStream_t passed as void*, null for the default stream) all later work is enqueued
 * on.  The workspace holds the cache (one copy of K and V of budget + max_decode + max_chunk rows per
 * kv-head, stream positions, scores and the two tables that map physical rows to stream order and back:
 * an eviction leaves the retained rows where they are and only moves the chunk's survivors into the rows
 * it frees) and per-step temporaries; attach enqueues a clear of the whole workspace on that stream.
 * The cache starts empty.  Errors: EINVAL (null/misaligned workspace; budget + max_decode + max_chunk - recent
 * above 131072, the most candidates a step can rank), ENOMEM (too small), ESTATE (already attached), EHIP.
 */
int infmllm_stream_attach(infmllm_stream_t* s, void* dev_workspace, size_t bytes, void* hip_stream);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture, serving loops and
 * harnesses that forbid hipMalloc): infmllm_stream_attach with the workspace taken from an array of
 * INFMLLM_STATIC_WORKSPACE_BYTES bytes that the library's code object holds on every GPU it is loaded on,
 * for the life of the process.  The stream is attached on the device that is current at the call; the
 * call allocates nothing (no hipMalloc / hipFree, no allocating library routine) and clears the part of
 * the array it uses with a fill kernel on hip_stream.  At most one stream per device can hold the array:
 * a second infmllm_stream_attach_static on that device fails with ESTATE until the first stream has been
 * destroyed (infmllm_stream_destroy releases the array; work of the destroyed stream still in flight on
 * its HIP stream would race with the next holder, so the caller orders the two, e.g. by using one HIP
 * stream).  The array keeps its last contents between holders; everything a stream relies on is cleared
 * at attach.  Errors: EINVAL (null stream, rotary position table requested: its table is uploaded from a
 * host buffer), ENOMEM (infmllm_stream_workspace_bytes(s) exceeds INFMLLM_STATIC_WORKSPACE_BYTES),
 * ESTATE (already attached, array in use), EHIP.
 */
#define INFMLLM_STATIC_WORKSPACE_BYTES (64u << 20)
int infmllm_stream_attach_static(infmllm_stream_t* s, void* hip_stream);

/*
 * One streaming step (Sec. 3.2 and Alg. 1), enqueued on the attached HIP stream:
 *   append      the chunk's k, v become cache rows t .. t+L-1 (stream positions T .. T+L-1)
 *   attention   out[i] = softmax_j(scale * q[i].K[j]) V[j] over the t cached keys and the
 *               chunk's keys up to and including i (causal inside the chunk)
 *   score       S[j] = mean over the last min(recent, L) query rows (and over the query
 *               heads of a group) of the attention weight on key j, j < c = n - recent
 *               (Alg. 1 l.1);  W'[j] = S[j] - (c-1-j) * b / c  (Alg. 1 l.2-4)
 *   select      the r = budget - recent largest W' per kv-head, ties to the newer key
 *               (Alg. 1 l.5), in ascending order, followed by [c, n) (Alg. 1 l.6-7)
 *   compact     cache rows, positions and scores are gathered by that list (Alg. 1 l.8)
 * While n <= budget nothing is evicted and the list is 0 .. n-1.
 *
 *   q, k, v     device, read-only, layouts as stated above; chunk_len = L in 1..max_chunk
 *   out         device, [L, heads, head_dim], written
 *   retained    device, int32 [kv_heads, budget]; row h receives the kept indices into the
 *               n rows that were cached before compaction, ascending; entries from
 *               *n_retained on are left untouched.  May be null (nothing is reported)
 *   n_retained  device, int32 scalar = min(n, budget).  May be null
 * Errors: EINVAL (null q/k/v/out, chunk_len < 1), ECAPACITY (chunk_len > max_chunk),
 * ESTATE (not attached), EHIP (launch failure).
 */
int infmllm_step(infmllm_stream_t* s, const void* q, const void* k, const void* v, int chunk_len,
                 void* out, int32_t* retained, int32_t* n_retained);

/*
 * One decoding step (Sec. 3.2, last paragraph: the eviction runs when a prompt arrives, not
 * while tokens are decoded), enqueued on the attached HIP stream: the token's k, v become cache
 * row t (stream position T), out = softmax_j(scale * q.K[j]) V[j] over all t + 1 keys, nothing
 * is evicted.  The cache may so grow to budget + max_decode rows; the next infmllm_step brings
 * it back to the budget.
 *   q      device, [1, heads, head_dim];  k, v  device, [1, kv_heads, head_dim];  read-only
 *   out    device, [1, heads, head_dim], written
 * Errors: EINVAL (null pointer), ECAPACITY (the cache already holds budget + max_decode rows),
 * ESTATE (not attached), EHIP.
 */
int infmllm_decode(infmllm_stream_t* s, const void* q, const void* k, const void* v, void* out);

/*
 * n_tokens decoding steps (Sec. 3.2, last paragraph) enqueued by one call, for callers whose per-call host
 * cost would exceed a token's kernels (a drafted continuation being verified, teacher-forced decoding):
 * token i is decoded exactly as by the i-th of n_tokens calls of infmllm_decode, so it attends the rows
 * cached before the call and tokens 0 .. i of the call.
 *   q      device, [n_tokens, heads, head_dim];  k, v  device, [n_tokens, kv_heads, head_dim];  read-only
 *   out    device, [n_tokens, heads, head_dim], written
 * Errors: EINVAL (null pointer, n_tokens < 1), ECAPACITY (the cache would exceed budget + max_decode
 * rows: nothing is enqueued), ESTATE (not attached), EHIP.
 */
int infmllm_decode_n(infmllm_stream_t* s, const void* q, const void* k, const void* v, void* out, int n_tokens);

/*
 * Layer-batched eviction (Alg. 1, note under "Input": the method treats the caches of all
 * layers at once).  A model's layers attend one after the other, but their evictions do not
 * depend on each other, so they can share launches:
 *
 * infmllm_step_attend does what infmllm_step does up to and including the scores (append or
 * in-place read of the chunk, chunk attention, S and the attention bias).  If the chunk fits
 * into the budget the step is complete, exactly as with infmllm_step (retained / n_retained are
 * written).  Otherwise the eviction is left pending: retained / n_retained are not touched, the
 * stream accepts no call other than infmllm_evict_batched, infmllm_stream_pending,
 * infmllm_stream_len / _streamed / _max_len and infmllm_stream_destroy (ESTATE), and q, k, v must
 * stay valid and unchanged until the kernels of that infmllm_evict_batched have run (the chunk's
 * rows are gathered from k and v in place).  Arguments and errors as for infmllm_step.
 */
int infmllm_step_attend(infmllm_stream_t* s, const void* q, const void* k, const void* v, int chunk_len,
                        void* out, int32_t* retained, int32_t* n_retained);

/* 1 if an eviction is pending on s, 0 if not, -1 if s is null. */
int infmllm_stream_pending(const infmllm_stream_t* s);

/*
 * Selection, recent-window move and gather (Alg. 1 l.5-8) of `count` streams with a pending
 * eviction, as one selection launch and one gather launch per 16 streams, enqueued on their
 * common HIP stream.  The result for every stream is the one infmllm_step would have produced.
 *   streams     host array of `count` distinct streams that have the same budget, recent, heads,
 *               kv_heads, head_dim, dtype, max_chunk and max_decode and are attached to the same
 *               HIP stream (their chunk lengths and cached lengths may differ)
 *   retained    host array of `count` device pointers, each int32 [kv_heads, budget] as in
 *               infmllm_step, or null; the array itself may be null
 *   n_retained  host array of `count` device pointers to an int32, or null entries / null array
 * Errors: EINVAL (null or repeated stream, differing geometry or HIP stream), ESTATE (a stream
 * with no eviction pending; nothing is launched then), EHIP.
 */
int infmllm_evict_batched(infmllm_stream_t* const* streams, int count, int32_t* const* retained,
                          int32_t* const* n_retained);

/* Tokens now cached (host bookkeeping; at most budget after a step, up to budget + max_decode
 * after decoding steps); -1 if s is null. */
int infmllm_stream_len(const infmllm_stream_t* s);

/* Most rows the cache can hold between two steps: budget + max_decode; -1 if s is null. */
int infmllm_stream_max_len(const infmllm_stream_t* s);

/* Tokens streamed so far, i.e. the stream position the next chunk starts at; -1 if null. */
int64_t infmllm_stream_streamed(const infmllm_stream_t* s);

/*
 * Copies the stream position of every cached row to pos (device, int32 [kv_heads, max_len] with
 * max_len = infmllm_stream_max_len(s), i.e. [kv_heads, budget] unless max_decode was set; the
 * first infmllm_stream_len entries of each row are written).  These are Alg. 1's I
 * expressed as positions in the whole stream.  Errors: EINVAL, ESTATE, EHIP.
 */
int infmllm_stream_positions(infmllm_stream_t* s, int32_t* pos);

/*
 * Debug/test: copies the cache out.  K, V: device, [kv_heads, len, head_dim] in the stream's
 * dtype; pos: device int32 [kv_heads, len]; score: device float [kv_heads, len] (the biased
 * score W' that admitted a row at the last eviction, +inf for rows that have only ever been
 * inside the recent window).  len = infmllm_stream_len(s).  Any pointer may be null.
 */
int infmllm_stream_export(infmllm_stream_t* s, void* K, void* V, int32_t* pos, float* score);

/*
 * Debug/test: replaces the cache by len rows per kv-head (layouts as for export; pos must
 * be strictly ascending per head) and sets the number of tokens streamed so far.  Scores
 * are set to +inf.  Errors: EINVAL (len outside 0..max_len, null pointers with len > 0),
 * ESTATE (not attached), EHIP.
 */
int infmllm_stream_import(infmllm_stream_t* s, const void* K, const void* V, const int32_t* pos,
                          int len, int64_t streamed);

/*
 * Debug/test: copies the biased scores W' of the most recent evicting step to w (device,
 * float [kv_heads, c]) and returns c through n_candidates (host int); c = 0 if the last
 * step did not evict.  Errors: EINVAL, ESTATE, EHIP.
 */
int infmllm_stream_last_scores(infmllm_stream_t* s, float* w, int* n_candidates);

/* Kernels of one step, as indexed by the profiling calls below. */
enum {
    INFMLLM_K_APPEND = 0,
    INFMLLM_K_ATTN = 1,
    INFMLLM_K_SCORE = 2,
    INFMLLM_K_SELECT = 3,
    INFMLLM_K_COMPACT = 4,
    INFMLLM_K_DECODE = 5,
    INFMLLM_K_ROPE = 6,
    INFMLLM_K_EVICT = 7,  /* not a kernel: from the start of the selection launch to the end of the gather launch of
                             a step (Alg. 1 l.5-8 as a whole, one event pair instead of two) */
    INFMLLM_K_COUNT = 8
};

/*
 * Measurement: brackets every kernel of the next max_steps steps with HIP events on the
 * attached stream (max_steps = 0 switches this off and releases the events).  The events cost
 * a few microseconds per step, so whole-step throughput is measured with profiling off.
 * Errors: EINVAL (max_steps outside 0..4096), ESTATE (not attached), EHIP.
 */
int infmllm_stream_profile(infmllm_stream_t* s, int max_steps);

/*
 * Chooses which of the INFMLLM_K_* intervals get events in the steps recorded from now on: bit k of
 * `kernels` switches interval k on (default: all).  Every event pair delays the stream a little, so a
 * caller who wants the undisturbed duration of one interval records only that one; INFMLLM_K_EVICT
 * alone records two events per step, before the selection launch and after the gather launch.
 * Errors: EINVAL (null stream, empty mask or bits beyond INFMLLM_K_COUNT).
 */
int infmllm_stream_profile_select(infmllm_stream_t* s, unsigned kernels);

/*
 * Measurement: waits for the recorded events and returns, per kernel, the summed duration in
 * milliseconds (ms, host float[INFMLLM_K_COUNT]) and the number of launches that were timed
 * (launches, host int[INFMLLM_K_COUNT]); then starts over with the same capacity.  This is the
 * only call that blocks the host.  Errors: EINVAL, EHIP.
 */
int infmllm_stream_profile_read(infmllm_stream_t* s, float* ms, int* launches);

/* Message for the calling thread's most recent failure ("" if none).  Never null. */
const char* infmllm_last_error(void);

/* Releases the host object (not the workspace).  Null is a no-op. */
void infmllm_stream_destroy(infmllm_stream_t* s);

#ifdef __cplusplus
}
#endif
#endif /* INFMLLM_H */
