// Device code of the per-head top-r selection (Alg. 1 l.5-7) and of the placement plan that follows it
// (which retained rows stay where they are, which move where), templated on TPB, the threads of the
// calling workgroup.
#pragma once
#include "launch.h"

namespace infmllm {
namespace {

__device__ __forceinline__ uint32_t order_key(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);    // larger float <=> larger key
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// Adds 1 to hist[digit] for every active lane whose `on` is true, one LDS atomic per distinct
// digit per wavefront.
__device__ __forceinline__ void wave_histogram(uint32_t* hist, uint32_t digit, bool on)
{
    uint64_t todo = __ballot(on);
    while (todo) {
        const int leader = __ffsll((long long)todo) - 1;      // wavefront-uniform
        const uint32_t dl = (uint32_t)__builtin_amdgcn_readlane((int)digit, leader);
        const uint64_t same = __ballot(on && digit == dl);
        if (lane_id() == leader) atomicAdd(&hist[dl], (uint32_t)__popcll(same));
        todo &= ~same;
    }
}

// Inclusive prefix sum over the 64 lanes of a wavefront whose lanes are all active, through the
// data-parallel-primitive lane shifts (no LDS round trip): shifts by 1, 2, 4, 8 inside each row
// of 16 lanes, then the last lane of rows 0 and 2 added to rows 1 and 3, then lane 31 to rows 2, 3.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t x)
{
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, false);   // row_shr:1
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, false);   // row_shr:2
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, false);   // row_shr:4
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, false);   // row_shr:8
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false);   // row_bcast:15
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false);   // row_bcast:31
    return x;
}

// Exclusive prefix sums of tab[0 .. count) in place, by one whole wavefront.
__device__ __forceinline__ void wave_exclusive_table(uint32_t* tab, int count)
{
    const int l = lane_id();
    uint32_t run = 0;
    for (int base = 0; base < count; base += 64) {
        const int idx = base + l;
        const uint32_t v = idx < count ? tab[idx] : 0u;
        const uint32_t incl = wave_inclusive_sum(v);
        if (idx < count) tab[idx] = run + incl - v;
        run += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
    }
}

// Minimum / maximum over the 64 lanes of a wavefront whose lanes are all active; lane 63 holds the result.
template <bool MAX>
__device__ __forceinline__ uint32_t wave_extreme_to_last_lane(uint32_t x)
{
    constexpr int ID = MAX ? 0 : -1;                          // identity, read where a shift has no source lane
#define INFMLLM_STEP(ctrl, rows)                                                             \
    {                                                                                        \
        const uint32_t y = (uint32_t)__builtin_amdgcn_update_dpp(ID, (int)x, ctrl, rows, 0xf, false); \
        x = MAX ? (x > y ? x : y) : (x < y ? x : y);                                         \
    }
    INFMLLM_STEP(0x111, 0xf) INFMLLM_STEP(0x112, 0xf) INFMLLM_STEP(0x114, 0xf) INFMLLM_STEP(0x118, 0xf)
    INFMLLM_STEP(0x142, 0xa) INFMLLM_STEP(0x143, 0xc)
#undef INFMLLM_STEP
    return x;
}

// Largest budget the placement plan keeps its two bit maps for (one bit per retained slot, one per
// physical row below B) in LDS.
constexpr int PLAN_MAX_B = 131072;

// Exclusive prefix sum of v over the TPB threads of the workgroup (all of them call it); *total = the sum.
template <int TPB>
__device__ __forceinline__ uint32_t block_exclusive_sum(uint32_t v, uint32_t* wsum /* [TPB/64] in LDS */, uint32_t* total)
{
    constexpr int NW = TPB / 64;
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    const uint32_t incl = wave_inclusive_sum(v);
    if (l == 63) wsum[w] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int x = 0; x < NW; ++x) {
        const uint32_t s = wsum[x];
        before += x < w ? s : 0u;
        all += s;
    }
    __syncthreads();                                          // wsum may be reused by the next call
    *total = all;
    return before + incl - v;
}

// The tables of one kv-head that the placement plan reads and writes (see CacheView).
struct PlanTables {
    const int32_t* row_old;    // [cap] physical row of each stream-order index before the eviction
    int32_t* row_new;          // [cap] ... after it
    int32_t* rank;             // [cap] stream-order index of each physical row (rewritten for rows 0..B-1)
    float* score;              // [cap]
    int32_t* mv_src;           // [mv_max] move list of this head
    int32_t* mv_dst;
    int32_t* mv_x;
    int32_t* mv_count;         // one int
};

// Alg. 1 l.8 without moving the rows that stay.  Ih[0..B) is the retained list (stream-order indices,
// ascending).  A retained token that is cached in a physical row below B keeps that row: its new index x
// goes into rank / row_new, its score entry becomes W'[j] (+inf inside the recent window).  Every other
// retained token (a chunk row, or a cached row at or above B) is a mover; the physical rows below B
// that no retained token occupies are exactly as many, and the k-th mover (by x) is paired with the k-th
// free row (ascending), which makes the layout a function of the retained list alone.  The K/V copies and
// the movers' table entries are left to the placement launch.
template <int TPB>
__device__ __forceinline__ void plan_moves(const int32_t* __restrict__ Ih, const float* __restrict__ W, int tc, int B,
                                           int r, const PlanTables& pt)
{
    __shared__ uint32_t occ[PLAN_MAX_B / 32], mov[PLAN_MAX_B / 32];
    __shared__ uint32_t wsum[TPB / 64];
    const int tid = threadIdx.x;
    const int words = (B + 31) / 32;
    for (int w = tid; w < words; w += TPB) { occ[w] = 0u; mov[w] = 0u; }
    __syncthreads();                                          // also: Ih as written by this workgroup is visible
    for (int x = tid; x < B; x += TPB) {
        const int j = Ih[x];
        const int p = j < tc ? pt.row_old[j] : -1;
        if (p >= 0 && p < B) {
            atomicOr(&occ[p >> 5], 1u << (p & 31));
            pt.rank[p] = x;
            pt.row_new[x] = p;
            pt.score[p] = x < r ? W[j] : __builtin_inff();
        } else {
            atomicOr(&mov[x >> 5], 1u << (x & 31));
        }
    }
    __syncthreads();
    uint32_t fbase = 0, mbase = 0;                            // free rows / movers listed so far (uniform)
    for (int w0 = 0; w0 < words; w0 += TPB) {
        const int w = w0 + tid;
        uint32_t f = 0u, m = 0u;
        if (w < words) {
            f = ~occ[w];
            if (32 * w + 32 > B) f &= (1u << (B - 32 * w)) - 1u;   // only rows below B
            m = mov[w];
        }
        uint32_t ftot, mtot;
        uint32_t fo = fbase + block_exclusive_sum<TPB>((uint32_t)__popc(f), wsum, &ftot);
        uint32_t mo = mbase + block_exclusive_sum<TPB>((uint32_t)__popc(m), wsum, &mtot);
        while (f) {
            const int b = __ffs((int)f) - 1;
            f &= f - 1u;
            pt.mv_dst[fo++] = 32 * w + b;
        }
        while (m) {
            const int b = __ffs((int)m) - 1;
            m &= m - 1u;
            const int x = 32 * w + b;
            pt.mv_src[mo] = Ih[x];
            pt.mv_x[mo++] = x;
        }
        fbase += ftot;
        mbase += mtot;
    }
    if (tid == 0) *pt.mv_count = (int32_t)mbase;               // = fbase: B rows are retained, B rows lie below B
}

// Same selection with the candidates of a head held in registers (KPT keys per thread, key
// k*TPB + tid in slot k): the scores are read from memory once.  The leading bits that every key
// shares (sign and most of the exponent, as a rule) are found from the smallest and the largest
// key and skipped, so that the 8-bit digits that follow are spread over their bins and can be
// counted with plain LDS atomics, into one of two histograms: the other is cleared beside the
// bin search and a pass costs two barriers.  The digits stop as soon as the bin that holds the
// r-th largest key is wanted whole (as a rule after the second: few of a few thousand candidates
// share 16 bits), and the ordered write needs two more barriers.
template <int KPT, int TPB>
__device__ __forceinline__ void select_reg_body(const float* __restrict__ Wb, int32_t* __restrict__ I,
                                                int32_t* __restrict__ userI, int32_t* __restrict__ user_count,
                                                int h, int cnd, int r, int R, int B, int cap)
{
    constexpr int NW = TPB / 64;
    static_assert(TPB >= 512, "one wavefront searches the bins while four others clear the next histogram");
    __shared__ uint32_t hist[2][256];
    __shared__ uint32_t s_min, s_max, s_prefix, s_remaining, s_ties, s_done;
    __shared__ uint32_t tab_eq[KPT * NW], tab_gt[KPT * NW];

    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
    const float* W = Wb + (size_t)h * cap;
    int32_t* Ih = I + (size_t)h * B;
    int32_t* Uh = userI ? userI + (size_t)h * B : nullptr;

    if (r > 0) {
        if (tid == 0) { s_min = 0xffffffffu; s_max = 0u; s_remaining = (uint32_t)r; s_ties = (uint32_t)cnd; s_done = 0; }
        if (tid < 256) hist[0][tid] = 0;
        uint32_t key[KPT];
        uint32_t lo_key = 0xffffffffu, hi_key = 0u;
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            const int j = k * TPB + tid;
            key[k] = 0u;
            if (j < cnd) {
                key[k] = order_key(W[j]);
                lo_key = key[k] < lo_key ? key[k] : lo_key;
                hi_key = key[k] > hi_key ? key[k] : hi_key;
            }
        }
        lo_key = wave_extreme_to_last_lane<false>(lo_key);
        hi_key = wave_extreme_to_last_lane<true>(hi_key);
        __syncthreads();
        if (l == 63) { atomicMin(&s_min, lo_key); atomicMax(&s_max, hi_key); }
        __syncthreads();
        // bits [top, 32) are the same in every key; the digits cover bits [0, top) from the top down
        const uint32_t spread = s_min ^ s_max;
        int hi = spread ? 32 - __builtin_clz(spread) : 0;
        uint32_t T = hi >= 32 ? 0u : (s_min >> hi << hi);      // the r-th largest key, as far as it is known
        for (int pass = 0; hi > 0; ++pass) {
            const int lo = hi > 8 ? hi - 8 : 0;
            uint32_t* hp = hist[pass & 1];
            const uint32_t himask = hi >= 32 ? 0u : (0xffffffffu << hi), dmask = (1u << (hi - lo)) - 1u;
#pragma unroll
            for (int k = 0; k < KPT; ++k)
                if ((k * TPB + tid < cnd) && ((key[k] & himask) == T)) atomicAdd(&hp[(key[k] >> lo) & dmask], 1u);
            __syncthreads();
            if (tid < 64) {
                // wavefront 0 walks the bins from the top; lane l owns bins 255-4l .. 252-4l
                uint32_t c0 = hp[255 - 4 * l], c1 = hp[254 - 4 * l], c2 = hp[253 - 4 * l], c3 = hp[252 - 4 * l];
                const uint32_t mine = c0 + c1 + c2 + c3, incl = wave_inclusive_sum(mine);
                const uint32_t before = incl - mine, need = s_remaining;
                if (before < need && need <= incl) {          // the r-th largest falls in my bins
                    uint32_t acc = before;
                    int bin = 255 - 4 * l;
                    uint32_t cnt = c0;
                    if (acc + cnt < need) { acc += cnt; --bin; cnt = c1;
                        if (acc + cnt < need) { acc += cnt; --bin; cnt = c2;
                            if (acc + cnt < need) { acc += cnt; --bin; cnt = c3; } } }
                    s_prefix = T | ((uint32_t)bin << lo);
                    s_remaining = need - acc;                 // still to take inside that bin
                    s_ties = cnt;                             // keys in that bin
                    // the whole bin is wanted: every key >= the bin's lowest is kept, the later digits
                    // decide nothing (T = that lowest key, no tie dropped)
                    if (need - acc == cnt) s_done = 1;
                }
            } else if (tid >= 256 && tid < 512) {
                hist[(pass + 1) & 1][tid - 256] = 0;
            }
            __syncthreads();
            T = s_prefix;
            hi = s_done ? 0 : lo;
        }
        const uint32_t skip_eq = s_ties - s_remaining;        // oldest ties that are dropped
        const uint64_t below = (l == 0) ? 0ull : (~0ull >> (64 - l));

        // kept = {key > T} U {ties of rank >= skip_eq in index order}; a segment is the 64 keys of
        // slot k in wavefront w, and segments follow index order
        uint64_t beq[KPT], bgt[KPT];
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            const bool in = k * TPB + tid < cnd;
            beq[k] = __ballot(in && key[k] == T);
            bgt[k] = __ballot(in && key[k] > T);
            if (l == 0) {
                tab_eq[k * NW + w] = (uint32_t)__popcll(beq[k]);
                tab_gt[k * NW + w] = (uint32_t)__popcll(bgt[k]);
            }
        }
        __syncthreads();
        if (w == 0) wave_exclusive_table(tab_eq, KPT * NW);
        else if (w == 1) wave_exclusive_table(tab_gt, KPT * NW);
        __syncthreads();
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            const uint32_t eq_before = tab_eq[k * NW + w];
            const uint32_t eq_rank = eq_before + (uint32_t)__popcll(beq[k] & below);
            const bool keep_eq = ((beq[k] >> l) & 1ull) && eq_rank >= skip_eq;
            const uint64_t bke = __ballot(keep_eq);
            if (keep_eq || ((bgt[k] >> l) & 1ull)) {
                // kept before this segment: every greater key, and the ties past the dropped ones
                const uint32_t dst = tab_gt[k * NW + w] + (eq_before > skip_eq ? eq_before - skip_eq : 0u)
                                   + (uint32_t)__popcll((bgt[k] | bke) & below);
                const int j = k * TPB + tid;
                Ih[dst] = j;
                if (Uh) Uh[dst] = j;
            }
        }
    }
    for (int x = tid; x < R; x += TPB) {                      // recent window: [c, n)
        Ih[r + x] = cnd + x;
        if (Uh) Uh[r + x] = cnd + x;
    }
    if (user_count && h == 0 && tid == 0) *user_count = B;
}

}  // namespace
}  // namespace infmllm
