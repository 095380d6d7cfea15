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
    int cap;      // physical cache rows per kv-head = B + max_decode + max_chunk
    int max_chunk;
    int max_decode;
    int elt;      // bytes per element (2 = bf16, 4 = fp32)
    double scale; // softmax scale (kernels take it, times log2(e) where they work in base 2, rounded once to float)
    double bias;  // b of Alg. 1 (the ramp step b / c is formed in double and rounded once to float)
    int policy;   // score ranked by the selection: 0 Alg. 1, 1 window, 2 initial + recent, 3 cumulative
    int attn_tile;// test hook: 0 = the matrix-core attention picks its tile shape, 1..4 = forces one
};
enum { POLICY_INFMLLM = 0, POLICY_WINDOW = 1, POLICY_INITIAL_RECENT = 2, POLICY_CUMULATIVE = 3 };

// The cache of one stream.  Rows are kept where they are: an eviction does not compact K and V, it
// frees the physical rows of the evicted tokens and hands them to the retained rows that lie outside
// rows 0..B-1 (the chunk's survivors, tokens decoded since the last chunk).  Softmax attention over the
// cached keys does not depend on their order, so the attention kernels sweep physical rows 0..len-1 as
// they are; what needs the stream order (Alg. 1's slot index: the bias ramp, the tie rule, the index
// list) goes through two small tables.  The cached rows always occupy physical rows 0..len-1.
struct CacheView {
    void* K;            // [Hkv][cap][d]   by physical row
    void* V;            // [Hkv][cap][d]
    int32_t* pos;       // [Hkv][cap]      stream position of the token in each physical row
    float* score;       // [Hkv][cap]      W' the row was last retained with (+inf: never ranked)
    int32_t* rank;      // [Hkv][cap]      stream-order index (0 = oldest cached token) of each physical row
    int32_t* row;       // [Hkv][cap]      physical row of each stream-order index (inverse of rank)
};

// Retained rows an eviction has to move, per kv-head: entry k says that the token in src[k] (physical
// cache row src[k] if src[k] < tc, the rows in the cache; else row src[k] - tc of the chunk tensors)
// becomes physical row dst[k] with the new stream-order index x[k] and the score entry score[k].
// Written by the selection launch, read by the placement launch.  max = max_chunk + max_decode entries
// per head.
struct MoveList {
    int32_t* src;       // [Hkv][max]
    int32_t* dst;       // [Hkv][max]
    int32_t* x;         // [Hkv][max]
    float* score;       // [Hkv][max]
    int32_t* count;     // [Hkv]
    int max;
};

// a1: physical rows t..t+L-1 <- chunk; pos <- T..T+L-1; score <- +inf; rank and row <- identity there.
hipError_t launch_append(const Geometry& g, const CacheView& c, const void* k, const void* v,
                         int t, int L, int64_t T, hipStream_t st);

// a2 (plain fp32 arithmetic, any dtype): out and per-row log-sum-exp.
hipError_t launch_attn_simple(const Geometry& g, const CacheView& c, const void* q, int t, int L,
                              void* out, float* lse, hipStream_t st);

// a3+a4 (plain fp32 arithmetic, any dtype): W'[h][j] for j < cnd = n - R, j = the stream-order index of a
// column (c.rank of its physical row); all n rows are in the cache here.
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

// The same for head_dim 128 with 64 query rows per wavefront (one wavefront per SIMD, 256-row workgroups):
// the shape for long key ranges and grids that fill the chip; launch_attn_mfma picks it by itself.
hipError_t launch_attn_mfma64(const Geometry& g, const CacheView& c, const KeySource& ks, const void* q, int t, int L,
                              void* out, float* lse, hipStream_t st);

// a3+a4 on bf16 MFMA (bf16 streams only).
hipError_t launch_score_mfma(const Geometry& g, const CacheView& c, const KeySource& ks, const void* q,
                             const float* lse, const FwdScratch& sc, int t, int L, float* Wb, hipStream_t st);

// a5+a6: I[h] = sort_asc(top-r of W'[h][0..cnd)) ++ [cnd, n), in stream-order indices.  I has row
// stride B.  user_I (row stride B) and user_count may be null.  The same workgroup then plans the
// placement (Alg. 1 l.8 without moving the rows that stay): a retained token whose physical row is
// below B keeps it and gets its new rank, row and score entries here; the others go into the move
// list, paired in order with the physical rows the eviction frees.  tc = rows in the cache (stream-order
// indices from tc on are chunk rows read in place).
hipError_t launch_select(const Geometry& g, const float* Wb, int n, int tc, int32_t* I, int32_t* user_I,
                         int32_t* user_count, const CacheView& c, const MoveList& mv, hipStream_t st);

// a7: copies the K and V rows of the move list to their new physical rows and writes their pos, rank,
// row and score entries.  nmax = most entries a head's list can hold in this step.
hipError_t launch_place(const Geometry& g, const CacheView& c, const KeySource& ks, int64_t T, const MoveList& mv,
                        int nmax, hipStream_t st);

// One stream's share of a batched eviction (a5-a7 for the layers of a model in one launch each,
// Alg. 1 Input note).  All streams of a batch have the same geometry.
struct EvictJob {
    const float* Wb;          // [Hkv][cap] biased scores of this stream
    int32_t* I;               // [Hkv][B] index list (stream scratch)
    int32_t* user_I;          // [Hkv][B] or null
    int32_t* user_count;      // one int or null
    CacheView c;
    MoveList mv;
    const void* kc;           // chunk tensors, stream-order indices >= tc
    const void* vc;
    int tc, pos0, n, pad_;
};
constexpr int EVICT_MAX_JOBS = 16;
struct EvictBatch {
    int count, pad_;
    EvictJob job[EVICT_MAX_JOBS];
};
hipError_t launch_select_batch(const Geometry& g, const EvictBatch& eb, hipStream_t st);
hipError_t launch_place_batch(const Geometry& g, const EvictBatch& eb, int nmax, hipStream_t st);

// Comparison policies that rank by age: W'[h][j] = sign * j for j < cnd (sign +1 keeps the newest,
// -1 the oldest).
hipError_t launch_rank_scores(const Geometry& g, float* Wb, int cnd, float sign, hipStream_t st);

// Cache-relative rotary encoding pre-pass: Krot[h][p] <- K[h][p] turned to position rank[h][p] (the row's
// stream-order index in the cache) for physical rows p in [j0, j1);
// kcrot[i][h] <- kc[i][h] and qrot[i][h] <- q[i][h] turned to position t + i for i < L (kc and q may each
// be null).  tab = [cap][d/2] pairs (cos, sin) of doubles; within a position, the entry of pair 8a + e is at
// index e * (d/16) + a, so that the threads of a row (one per a) read consecutive entries.
hipError_t launch_rope(const Geometry& g, const void* K, void* Krot, const int32_t* rank, int j0, int j1,
                       const void* kc, void* kcrot, const void* q, void* qrot, int t, int L, const double* tab,
                       hipStream_t st);

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

// After an import: score[h][0..len) <- +inf, rank and row <- identity.
hipError_t launch_reset_tables(const Geometry& g, const CacheView& c, int len, hipStream_t st);

// The cache in stream order (Alg. 1's K_s, V_s and their positions): out row j <- physical row c.row[h][j],
// j < len.  Kout / Vout [Hkv][len][d], pos_out / score_out [Hkv][pitch]; any of them may be null.
hipError_t launch_export(const Geometry& g, const CacheView& c, int len, void* Kout, void* Vout, int32_t* pos_out,
                         float* score_out, int pitch, hipStream_t st);

}  // namespace infmllm
