// Internal launch interface between the C-ABI host code and the gfx950 kernels.
// Everything here is asynchronous on the given HIP stream; nothing allocates.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace infmllm {

// Every K and V buffer of the cache is followed by this many rows of padding, and the whole
// workspace is zeroed when it is attached: the matrix-core attention kernel reads whole key
// tiles and may run this far past the last cached row (into finite data it then masks).
constexpr int CACHE_PAD_ROWS = 256;

// Geometry of one stream, fixed at attach time.
struct Geometry {
    int B;        // budget (rows kept after a step)
    int R;        // recent window (newest rows always kept)
    int Hq;       // query heads
    int Hkv;      // key/value heads
    int G;        // Hq / Hkv
    int d;        // head_dim (64 or 128)
    int cap;      // cache rows per kv-head = B + max_chunk
    int max_chunk;
    int max_decode;
    int elt;      // bytes per element (2 = bf16, 4 = fp32)
    double scale; // softmax scale (kernels take it, times log2(e) where they work in base 2, rounded once to float)
    double bias;  // b of Alg. 1 (the ramp step b / c is formed in double and rounded once to float)
    int policy;   // score ranked by the selection: 0 Alg. 1, 1 window, 2 initial + recent, 3 cumulative
    int attn_tile;// test hook: 0 = the matrix-core attention picks its tile shape, 1..4 = forces one
};
enum { POLICY_INFMLLM = 0, POLICY_WINDOW = 1, POLICY_INITIAL_RECENT = 2, POLICY_CUMULATIVE = 3 };

// One side of the double-buffered cache.
struct CacheView {
    void* K;        // [Hkv][cap][d]
    void* V;        // [Hkv][cap][d]
    int32_t* pos;   // [Hkv][cap]
    float* score;   // [Hkv][cap]
};

// a1: rows t..t+L-1 <- chunk; pos <- T..T+L-1; score <- +inf.
hipError_t launch_append(const Geometry& g, const CacheView& c, const void* k, const void* v,
                         int t, int L, int64_t T, hipStream_t st);

// a2 (plain fp32 arithmetic, any dtype): out and per-row log-sum-exp.
hipError_t launch_attn_simple(const Geometry& g, const CacheView& c, const void* q, int t, int L,
                              void* out, float* lse, hipStream_t st);

// a3+a4 (plain fp32 arithmetic, any dtype): W'[h][j] for j < cnd = n - R.
// With g.policy == POLICY_CUMULATIVE the score is S plus the score the row carries in c.score
// (a row never ranked carries +inf there and counts as 0) and no bias is applied.
hipError_t launch_score_simple(const Geometry& g, const CacheView& c, const void* q, const float* lse,
                               int t, int L, float* Wb, hipStream_t st);

// Scratch of the matrix-core scoring launch.
struct FwdScratch {
    // Row-split scoring: raw column sums of each split, [SCORE_SPLIT_WGS][256] fp32, followed by one
    // arrival counter per (kv-head, column block), [SCORE_SPLIT_WGS] int32, zero between launches.
    float* score_part;
};
// most workgroups a row-split scoring launch may have
constexpr int SCORE_SPLIT_WGS = 512;

// Where the keys and values of a step live.  Rows below `rows` come from the cache; rows from
// `rows` on are taken straight from the chunk tensors k, v ([L][Hkv][d]) as chunk row j - rows.
// With rows = n (after an append) the chunk pointers are never used.
struct KeySource {
    int rows;
    const void* k;
    const void* v;
};

// a2 on bf16 MFMA (bf16 streams only): out and the row log-sum-exp (base 2).
hipError_t launch_attn_mfma(const Geometry& g, const CacheView& c, const KeySource& ks, const void* q, int t, int L,
                            void* out, float* lse, hipStream_t st);

// a3+a4 on bf16 MFMA (bf16 streams only).
hipError_t launch_score_mfma(const Geometry& g, const CacheView& c, const KeySource& ks, const void* q,
                             const float* lse, const FwdScratch& sc, int t, int L, float* Wb, hipStream_t st);

// a5+a6: I[h] = sort_asc(top-r of W'[h][0..cnd)) ++ [cnd, n).  I has row stride B.
// user_I (row stride B) and user_count may be null.  The same launch also moves the recent
// window (rows cnd..n-1 of src / the chunk) to rows r..B-1 of dst, on workgroups of its own.
hipError_t launch_select(const Geometry& g, const float* Wb, int n, int32_t* I, int32_t* user_I,
                         int32_t* user_count, const CacheView& src, const KeySource& ks, int64_t T,
                         const CacheView& dst, hipStream_t st);

// One stream's share of a batched eviction (a5-a7 for the layers of a model in one launch each,
// Alg. 1 Input note).  All streams of a batch have the same geometry.
struct EvictJob {
    const float* Wb;          // [Hkv][cap] biased scores of this stream
    int32_t* I;               // [Hkv][B] index list (stream scratch)
    int32_t* user_I;          // [Hkv][B] or null
    int32_t* user_count;      // one int or null
    CacheView src, dst;       // live half, other half
    const void* kc;           // chunk tensors, rows >= tc of the key axis
    const void* vc;
    int tc, pos0, n, pad_;
};
constexpr int EVICT_MAX_JOBS = 16;
struct EvictBatch {
    int count, pad_;
    EvictJob job[EVICT_MAX_JOBS];
};
hipError_t launch_select_batch(const Geometry& g, const EvictBatch& eb, hipStream_t st);
hipError_t launch_compact_batch(const Geometry& g, const EvictBatch& eb, hipStream_t st);

// Comparison policies that rank by age: W'[h][j] = sign * j for j < cnd (sign +1 keeps the newest,
// -1 the oldest).
hipError_t launch_rank_scores(const Geometry& g, float* Wb, int cnd, float sign, hipStream_t st);

// Cache-relative rotary encoding pre-pass: Krot[h][j] <- K[h][j] turned to position j for j in [j0, j1);
// kcrot[i][h] <- kc[i][h] and qrot[i][h] <- q[i][h] turned to position t + i for i < L (kc and q may each
// be null).  tab = [cap][d/2] pairs (cos, sin) of doubles; within a position, the entry of pair 8a + e is at
// index e * (d/16) + a, so that the threads of a row (one per a) read consecutive entries.
hipError_t launch_rope(const Geometry& g, const void* K, void* Krot, int j0, int j1, const void* kc, void* kcrot,
                       const void* q, void* qrot, int t, int L, const double* tab, hipStream_t st);

// Clears `bytes` bytes (a multiple of 16) at p (16-byte aligned) with a fill kernel, which, unlike a
// memset node, may be recorded into a HIP graph.
hipError_t launch_zero(void* p, size_t bytes, hipStream_t st);

// warm-up: I[h][j] = j for j < n.
hipError_t launch_iota(const Geometry& g, int n, int32_t* user_I, int32_t* user_count, hipStream_t st);

// Decoding step: appends the token's k, v as cache row t and attends all t + 1 keys with q (one
// row per query head).  part is scratch of [Hq][max_split][d + 2] floats followed by Hkv ints that are zero
// between launches (ticket counters; the last workgroup of a kv-head to finish merges its splits).
constexpr int DECODE_MAX_SPLIT = 64;
hipError_t launch_decode(const Geometry& g, const CacheView& c, const void* q, const void* k, const void* v, int t,
                         int64_t T, void* out, float* part, int max_split, hipStream_t st);

// score[h][0..len) <- +inf (used when a cache is imported).
hipError_t launch_fill_inf(const Geometry& g, float* score, int len, hipStream_t st);

// a7: dst rows x < B - R <- src rows I[h][x], score <- W'[I] (the recent rows were moved by launch_select).
// Rows at or above ks.rows are gathered from the chunk tensors; their position is T + (row - ks.rows).
hipError_t launch_compact(const Geometry& g, const CacheView& src, const KeySource& ks, int64_t T,
                          const CacheView& dst, const int32_t* I, const float* Wb, int n, hipStream_t st);

}  // namespace infmllm
