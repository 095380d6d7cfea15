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

// Workgroup barrier for data handed over through LDS only.  `__syncthreads` also waits for every global store
// and load of the wavefront to complete (about a microsecond for a store on its way to memory), which the
// selection and the plan never need: nothing they write to memory is read again before the kernel ends.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

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

// What the selection leaves in LDS for the placement plan: for every segment of 64 candidates (stream-order
// indices 64 s .. 64 s + 63) which of them are retained, and how many retained candidates precede the
// segment.  The new stream-order index of a retained candidate j is base[j / 64] plus the retained ones below
// it in its segment; a token of the recent window (j >= c) is retained with index r + (j - c).
constexpr int PLAN_MAX_C = 131072;                            // most candidates (n - R) a step may have
struct KeptMap {
    uint64_t bits[PLAN_MAX_C / 64];
    uint32_t base[PLAN_MAX_C / 64];
};

// The tables of one kv-head that the placement plan reads and writes (see CacheView, MoveList).
struct PlanTables {
    int32_t* rank;             // [cap] stream-order index of each physical row: read, and rewritten for the rows that stay
    int32_t* row;              // [cap] physical row of each stream-order index: written for the rows that stay
    float* score;              // [cap]
    int32_t* mv_src;           // [mv_max] move list of this head
    int32_t* mv_dst;
    int32_t* mv_x;
    float* mv_score;
    int32_t* mv_count;         // one int
};

// Alg. 1 l.8 without moving the rows that stay.  Every physical row below max(tc, B) and every chunk row is
// looked at once, 64 consecutive ones per wavefront, so that all table traffic is coalesced and the two lists
// are compacted with ballots: a cached row whose token is retained and that lies below B keeps its place (its
// new index goes into rank / row, its score entry becomes W'[j], +inf inside the recent window); a retained
// token in a row at or above B, or in the chunk, is a mover; a row below B whose token is evicted (or that is
// empty) is free.  There are exactly as many movers as free rows, and the k-th mover is paired with the k-th
// free row, both in ascending order, which makes the layout a function of the retained set alone.  The K/V
// copies and the movers' table entries are left to the placement launch.
// What the plan reads from memory does not depend on the selection: the stream-order index of every physical
// row and the score W' of that index.  The first PLAN_PRE items of every thread are therefore requested before
// the selection starts and have long arrived when the plan wants them; a plan with more items (more than
// PLAN_PRE * 1024 rows) loads the rest pass by pass.
constexpr int PLAN_PRE = 12;
struct PlanPre {
    int jj[PLAN_PRE];
    float w[PLAN_PRE];
};
// item q of the plan: a physical row below max(tc, B), then the chunk rows read in place; its token, or -1
__device__ __forceinline__ int plan_item_token(const int32_t* __restrict__ rank, int q, int tc, int P1, int nitems)
{
    return q < tc ? rank[q] : (q >= P1 && q < nitems ? tc + (q - P1) : -1);
}
// The two halves of the prefetch: the tokens of the items (table reads), and, once those have arrived, their scores.
// The selection requests its candidates between the two, so that it does not wait for the second trip to memory.
template <int TPB>
__device__ __forceinline__ void plan_prefetch_tokens(PlanPre& pre, const int32_t* __restrict__ rank, int n, int tc, int B)
{
    const int P1 = tc > B ? tc : B, nitems = P1 + (n - tc);
#pragma unroll
    for (int g = 0; g < PLAN_PRE; ++g) pre.jj[g] = plan_item_token(rank, g * TPB + (int)threadIdx.x, tc, P1, nitems);
}
template <int TPB>
__device__ __forceinline__ void plan_prefetch_scores(PlanPre& pre, const float* __restrict__ W, int cnd)
{
#pragma unroll
    for (int g = 0; g < PLAN_PRE; ++g) pre.w[g] = (pre.jj[g] >= 0 && pre.jj[g] < cnd) ? W[pre.jj[g]] : __builtin_inff();
}

template <int TPB>
__device__ __forceinline__ void plan_moves(const KeptMap& km, const float* __restrict__ W, int n, int tc, int cnd,
                                           int B, int r, const PlanTables& pt, const PlanPre& pre)
{
    constexpr int NW = TPB / 64, CH = 64 / NW;                 // CH passes of TPB items share one table of 64 counts
    __shared__ uint32_t cnt_free[64], cnt_mov[64];
    __shared__ uint32_t tot_free, tot_mov;
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
    const uint64_t below = (l == 0) ? 0ull : (~0ull >> (64 - l));
    const int P1 = tc > B ? tc : B;                           // physical rows looked at
    const int nitems = P1 + (n - tc);                         // ... then the chunk rows read in place
    // new index of token j, or -1 if it is evicted
    auto new_index = [&](int j) -> int {
        if (j >= cnd) return r + (j - cnd);
        const uint64_t bits = km.bits[j >> 6];
        if (!((bits >> (j & 63)) & 1ull)) return -1;
        return (int)km.base[j >> 6] + __popcll(bits & ((1ull << (j & 63)) - 1ull));
    };
    uint32_t fbase = 0, mbase = 0;                            // free rows / movers listed so far (uniform)
    lds_barrier();                                          // the kept map is complete
    static_assert(PLAN_PRE % CH == 0, "prefetched items are consumed in whole passes");
    auto pass = [&](int q0, const int (&jj)[CH], const float (&wv)[CH]) {
        int xs[CH], src[CH];
        uint64_t bfree[CH], bmov[CH];
        float sc[CH];
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            xs[u] = jj[u] >= 0 ? new_index(jj[u]) : -1;
            sc[u] = (xs[u] >= 0 && xs[u] < r) ? wv[u] : __builtin_inff();
        }
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int q = q0 + u * TPB + tid;
            const bool kept = xs[u] >= 0;
            const bool stays = kept && q < tc && q < B;
            const bool moves = kept && !stays;
            const bool is_free = !kept && q < B;
            src[u] = q < P1 ? q : jj[u];                      // a cache row below tc, or tc + chunk row
            if (stays) {
                pt.rank[q] = xs[u];
                pt.row[xs[u]] = q;
                pt.score[q] = sc[u];
            }
            bfree[u] = __ballot(is_free);
            bmov[u] = __ballot(moves);
            if (l == 0) {
                cnt_free[u * NW + w] = (uint32_t)__popcll(bfree[u]);
                cnt_mov[u * NW + w] = (uint32_t)__popcll(bmov[u]);
            }
        }
        lds_barrier();
        if (w == 0) {
            const uint32_t v = cnt_free[l], incl = wave_inclusive_sum(v);
            cnt_free[l] = incl - v;
            if (l == 63) tot_free = incl;
        } else if (w == 1) {
            const uint32_t v = cnt_mov[l], incl = wave_inclusive_sum(v);
            cnt_mov[l] = incl - v;
            if (l == 63) tot_mov = incl;
        }
        lds_barrier();
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int q = q0 + u * TPB + tid;
            if ((bfree[u] >> l) & 1ull) pt.mv_dst[fbase + cnt_free[u * NW + w] + (uint32_t)__popcll(bfree[u] & below)] = q;
            if ((bmov[u] >> l) & 1ull) {
                const uint32_t k = mbase + cnt_mov[u * NW + w] + (uint32_t)__popcll(bmov[u] & below);
                pt.mv_src[k] = src[u];
                pt.mv_x[k] = xs[u];
                pt.mv_score[k] = sc[u];
            }
        }
        fbase += tot_free;
        mbase += tot_mov;
        lds_barrier();                                      // the count tables are rewritten by the next pass
    };
#pragma unroll
    for (int p = 0; p < PLAN_PRE / CH; ++p) {                 // the passes whose loads were requested up front
        if (p * CH * TPB < nitems) {
            int jj[CH];
            float wv[CH];
#pragma unroll
            for (int u = 0; u < CH; ++u) { jj[u] = pre.jj[p * CH + u]; wv[u] = pre.w[p * CH + u]; }
            pass(p * CH * TPB, jj, wv);
        }
    }
    for (int q0 = PLAN_PRE * TPB; q0 < nitems; q0 += CH * TPB) {
        int jj[CH];
        float wv[CH];
#pragma unroll
        for (int u = 0; u < CH; ++u) jj[u] = plan_item_token(pt.rank, q0 + u * TPB + tid, tc, P1, nitems);
#pragma unroll
        for (int u = 0; u < CH; ++u) wv[u] = (jj[u] >= 0 && jj[u] < cnd) ? W[jj[u]] : __builtin_inff();
        pass(q0, jj, wv);
    }
    if (tid == 0) *pt.mv_count = (int32_t)mbase;               // = fbase: B tokens are retained, B rows lie below B
}

// Same selection with the candidates of a head held in registers (KPT keys per thread, key
// k*TPB + tid in slot k): the scores are read from memory once.  The leading bits that every key
// shares (sign and most of the exponent, as a rule) are found from the smallest and the largest
// key and skipped, so that the 8-bit digits that follow are spread over their bins and can be
// counted with plain LDS atomics, into one of two histograms: the other is cleared beside the
// bin search and a pass costs two barriers.  The digits stop as soon as the bin that holds the
// r-th largest key is wanted whole (as a rule after the second: few of a few thousand candidates
// share 16 bits), and the ordered write needs two more barriers.
template <int KPT, int TPB, typename AfterLoads>
__device__ __forceinline__ void select_reg_body(const float* __restrict__ Wb, int32_t* __restrict__ I,
                                                int32_t* __restrict__ userI, int32_t* __restrict__ user_count,
                                                int h, int cnd, int r, int R, int B, int cap, KeptMap& km,
                                                AfterLoads&& after_loads)
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
        float wj[KPT];
        uint32_t lo_key = 0xffffffffu, hi_key = 0u;
#pragma unroll
        for (int k = 0; k < KPT; ++k) wj[k] = W[k * TPB + tid < cnd ? k * TPB + tid : 0];   // cnd >= 1 here
        after_loads();                                        // further loads of the caller, behind the candidates
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            const int j = k * TPB + tid;
            key[k] = 0u;
            if (j < cnd) {
                key[k] = order_key(wj[k]);
                lo_key = key[k] < lo_key ? key[k] : lo_key;
                hi_key = key[k] > hi_key ? key[k] : hi_key;
            }
        }
        lo_key = wave_extreme_to_last_lane<false>(lo_key);
        hi_key = wave_extreme_to_last_lane<true>(hi_key);
        lds_barrier();
        if (l == 63) { atomicMin(&s_min, lo_key); atomicMax(&s_max, hi_key); }
        lds_barrier();
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
            lds_barrier();
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
            lds_barrier();
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
        lds_barrier();
        if (w == 0) wave_exclusive_table(tab_eq, KPT * NW);
        else if (w == 1) wave_exclusive_table(tab_gt, KPT * NW);
        lds_barrier();
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            const uint32_t eq_before = tab_eq[k * NW + w];
            const uint32_t eq_rank = eq_before + (uint32_t)__popcll(beq[k] & below);
            const bool keep_eq = ((beq[k] >> l) & 1ull) && eq_rank >= skip_eq;
            const uint64_t bke = __ballot(keep_eq);
            // kept before this segment: every greater key, and the ties past the dropped ones
            const uint32_t seg_base = tab_gt[k * NW + w] + (eq_before > skip_eq ? eq_before - skip_eq : 0u);
            if (l == 0) {                                     // for the placement plan
                km.bits[k * NW + w] = bgt[k] | bke;
                km.base[k * NW + w] = seg_base;
            }
            if (keep_eq || ((bgt[k] >> l) & 1ull)) {
                const uint32_t dst = seg_base + (uint32_t)__popcll((bgt[k] | bke) & below);
                const int j = k * TPB + tid;
                Ih[dst] = j;
                if (Uh) Uh[dst] = j;
            }
        }
    }
    else {
        after_loads();
        for (int sgm = tid; sgm < (cnd + 63) / 64; sgm += TPB) { km.bits[sgm] = 0ull; km.base[sgm] = 0u; }   // nothing ranked
    }
    for (int x = tid; x < R; x += TPB) {                      // recent window: [c, n)
        Ih[r + x] = cnd + x;
        if (Uh) Uh[r + x] = cnd + x;
    }
    if (user_count && h == 0 && tid == 0) *user_count = B;
}

}  // namespace
}  // namespace infmllm
