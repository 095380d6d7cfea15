// Per-head top-r selection for gfx950 (Alg. 1 l.5-7).
//
// One workgroup of 1024 threads per kv-head.  The r-th largest biased score is found with an
// MSB-first radix select over order-preserving 32-bit keys (8-bit digits).  With the candidates
// of a head in registers (select_body.h) the digits start below the bits all keys share and are
// counted with LDS atomics; with the candidates left in memory (more than 16 per thread) the
// histograms are built from wavefront ballots of the candidates that still match the prefix.
// The kept set {key > T} U {the newest ties of key == T} is then written in ascending index
// order through block-wide ballot/popcount scans, followed by the recent window [c, n), which
// is kept unconditionally.  Ties go to the larger index (the newer key).  The same workgroup then
// plans the placement of the retained rows (select_body.h: plan_moves).
#include "launch.h"
#include "select_body.h"

namespace infmllm {

namespace {

constexpr int TPB = 1024;
constexpr int NW = TPB / 64;

// Selection of kv-head h by one workgroup, candidates re-read from memory in every pass.
__device__ __forceinline__ void select_mem_body(const float* __restrict__ Wb, int32_t* __restrict__ I,
                                                int32_t* __restrict__ userI, int32_t* __restrict__ user_count,
                                                int h, int cnd, int r, int R, int B, int cap, KeptMap& km)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t s_prefix, s_remaining, s_ties;
    __shared__ uint32_t wave_eq[NW], wave_keep[NW];
    __shared__ uint32_t run_eq, run_keep;

    const float* W = Wb + (size_t)h * cap;
    int32_t* Ih = I + (size_t)h * B;
    int32_t* Uh = userI ? userI + (size_t)h * B : nullptr;

    if (r > 0) {
        // ---- radix select: key of the r-th largest -------------------------------------
        if (threadIdx.x == 0) { s_prefix = 0; s_remaining = (uint32_t)r; }
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            for (int x = threadIdx.x; x < 256; x += TPB) hist[x] = 0;
            __syncthreads();
            const uint32_t prefix = s_prefix;
            const uint32_t himask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
            for (int j0 = 0; j0 < cnd; j0 += TPB) {
                const int j = j0 + threadIdx.x;
                const bool in = j < cnd;
                const uint32_t key = in ? order_key(W[j]) : 0u;
                const bool on = in && ((key & himask) == prefix);
                wave_histogram(hist, (key >> shift) & 0xffu, on);
            }
            __syncthreads();
            if (threadIdx.x < 64) {
                // wavefront 0 walks the bins from the top; lane l owns bins 255-4l .. 252-4l
                const int l = threadIdx.x;
                uint32_t c0 = hist[255 - 4 * l], c1 = hist[254 - 4 * l], c2 = hist[253 - 4 * l], c3 = hist[252 - 4 * l];
                const uint32_t mine = c0 + c1 + c2 + c3, incl = wave_inclusive_sum(mine);
                const uint32_t before = incl - mine;          // keys in higher bins than my four
                const uint32_t need = s_remaining;
                if (before < need && need <= incl) {          // the r-th largest falls in my bins
                    uint32_t acc = before;
                    int bin = 255 - 4 * l;
                    uint32_t cnt = c0;
                    if (acc + cnt < need) { acc += cnt; --bin; cnt = c1;
                        if (acc + cnt < need) { acc += cnt; --bin; cnt = c2;
                            if (acc + cnt < need) { acc += cnt; --bin; cnt = c3; } } }
                    s_prefix = prefix | ((uint32_t)bin << shift);
                    s_remaining = need - acc;                 // still to take inside that bin
                    s_ties = cnt;                             // after the last pass: keys == T
                }
            }
            __syncthreads();
        }
        const uint32_t T = s_prefix;
        const uint32_t skip_eq = s_ties - s_remaining;        // oldest ties that are dropped
        if (threadIdx.x == 0) { run_eq = 0; run_keep = 0; }
        __syncthreads();

        // ---- ordered write of the kept candidates -----------------------------------------
        const int w = threadIdx.x >> 6, l = lane_id();
        const uint64_t below = (l == 0) ? 0ull : (~0ull >> (64 - l));
        for (int j0 = 0; j0 < cnd; j0 += TPB) {
            const int j = j0 + threadIdx.x;
            const uint32_t key = (j < cnd) ? order_key(W[j]) : 0u;
            const bool gt = (j < cnd) && key > T;
            const bool eq = (j < cnd) && key == T;
            const uint64_t beq = __ballot(eq);
            if (l == 0) wave_eq[w] = (uint32_t)__popcll(beq);
            __syncthreads();
            uint32_t eq_rank = run_eq + (uint32_t)__popcll(beq & below);
            for (int x = 0; x < w; ++x) eq_rank += wave_eq[x];
            const bool keep = gt || (eq && eq_rank >= skip_eq);
            const uint64_t bk = __ballot(keep);
            if (l == 0) wave_keep[w] = (uint32_t)__popcll(bk);
            __syncthreads();
            uint32_t seg_base = run_keep;
            for (int x = 0; x < w; ++x) seg_base += wave_keep[x];
            if (l == 0) {                                     // for the placement plan
                km.bits[j0 / 64 + w] = bk;
                km.base[j0 / 64 + w] = seg_base;
            }
            const uint32_t dst = seg_base + (uint32_t)__popcll(bk & below);
            if (keep) {
                Ih[dst] = j;
                if (Uh) Uh[dst] = j;
            }
            __syncthreads();
            if (threadIdx.x == 0) {
                uint32_t te = 0, tk = 0;
                for (int x = 0; x < NW; ++x) { te += wave_eq[x]; tk += wave_keep[x]; }
                run_eq += te;
                run_keep += tk;
            }
            __syncthreads();
        }
    }
    else {
        for (int sgm = threadIdx.x; sgm < (cnd + 63) / 64; sgm += TPB) { km.bits[sgm] = 0ull; km.base[sgm] = 0u; }
    }
    // ---- recent window: [c, n) -------------------------------------------------------------
    for (int x = threadIdx.x; x < R; x += TPB) {
        Ih[r + x] = cnd + x;
        if (Uh) Uh[r + x] = cnd + x;
    }
    if (user_count && h == 0 && threadIdx.x == 0) *user_count = B;
}


// KPT = 0: candidates stay in memory.
// after_loads is called once, when the selection has requested its candidates and not yet used them.
template <int KPT, typename AfterLoads>
__device__ __forceinline__ void select_body(const float* Wb, int32_t* I, int32_t* userI, int32_t* user_count, int h,
                                            int cnd, int r, int R, int B, int cap, KeptMap& km, AfterLoads&& after_loads)
{
    if constexpr (KPT == 0) {
        after_loads();
        select_mem_body(Wb, I, userI, user_count, h, cnd, r, R, B, cap, km);
    } else {
        select_reg_body<KPT, TPB>(Wb, I, userI, user_count, h, cnd, r, R, B, cap, km, after_loads);
    }
}

// One workgroup per kv-head: selection, then the placement plan.
template <int KPT>
__global__ void __launch_bounds__(TPB)
select_kernel(const float* __restrict__ Wb, int32_t* __restrict__ I, int32_t* __restrict__ userI,
              int32_t* __restrict__ user_count, int cnd, int r, int R, int B, int cap, int tc, CacheView c, MoveList mv)
{
    __shared__ KeptMap km;
    const int h = blockIdx.x;
    const size_t hb = (size_t)h * cap, mb = (size_t)h * mv.max;
    PlanPre pre;
    plan_prefetch_tokens<TPB>(pre, c.rank + hb, cnd + R, tc, B);
    select_body<KPT>(Wb, I, userI, user_count, h, cnd, r, R, B, cap, km,
                     [&]() __attribute__((always_inline)) { plan_prefetch_scores<TPB>(pre, Wb + hb, cnd); });
    const PlanTables pt{c.rank + hb, c.row + hb, c.score + hb, mv.src + mb, mv.dst + mb, mv.x + mb, mv.score + mb,
                        mv.count + h};
    plan_moves<TPB>(km, Wb + hb, cnd + R, tc, cnd, B, r, pt, pre);
}

// Several streams of one geometry (the layers of a model, Alg. 1 Input note): stream j owns
// workgroups [j * Hkv, (j + 1) * Hkv).
template <int KPT>
__global__ void __launch_bounds__(TPB)
select_batch_kernel(EvictBatch eb, int r, int R, int B, int cap, int Hkv)
{
    const int j = blockIdx.x / Hkv, h = blockIdx.x % Hkv;
    const EvictJob& job = eb.job[j];
    __shared__ KeptMap km;
    const int cnd = job.n - R;
    const size_t hb = (size_t)h * cap, mb = (size_t)h * job.mv.max;
    PlanPre pre;
    plan_prefetch_tokens<TPB>(pre, job.c.rank + hb, job.n, job.tc, B);
    select_body<KPT>(job.Wb, job.I, job.user_I, job.user_count, h, cnd, r, R, B, cap, km,
                     [&]() __attribute__((always_inline)) { plan_prefetch_scores<TPB>(pre, job.Wb + hb, cnd); });
    const PlanTables pt{job.c.rank + hb, job.c.row + hb, job.c.score + hb, job.mv.src + mb, job.mv.dst + mb,
                        job.mv.x + mb, job.mv.score + mb, job.mv.count + h};
    plan_moves<TPB>(km, job.Wb + hb, job.n, job.tc, cnd, B, r, pt, pre);
}

}  // namespace

hipError_t launch_select(const Geometry& g, const float* Wb, int n, int tc, int32_t* I, int32_t* user_I,
                         int32_t* user_count, const CacheView& c, const MoveList& mv, hipStream_t st)
{
    const int cnd = n - g.R, r = g.B - g.R;
    if (cnd > PLAN_MAX_C) return hipErrorInvalidValue;
    const dim3 grid(g.Hkv);
#define INFMLLM_SELECT(KPT)                                                                                \
    hipLaunchKernelGGL(select_kernel<KPT>, grid, dim3(TPB), 0, st, Wb, I, user_I, user_count, cnd, r, g.R, g.B, g.cap, \
                       tc, c, mv)
    if (cnd <= 2 * TPB) INFMLLM_SELECT(2);
    else if (cnd <= 4 * TPB) INFMLLM_SELECT(4);
    else if (cnd <= 8 * TPB) INFMLLM_SELECT(8);
    else if (cnd <= 16 * TPB) INFMLLM_SELECT(16);
    else INFMLLM_SELECT(0);                                  // candidates stay in memory
#undef INFMLLM_SELECT
    return hipGetLastError();
}

hipError_t launch_select_batch(const Geometry& g, const EvictBatch& eb, hipStream_t st)
{
    if (eb.count < 1 || eb.count > EVICT_MAX_JOBS) return hipErrorInvalidValue;
    const int r = g.B - g.R;
    int cnd = 0;
    for (int j = 0; j < eb.count; ++j) cnd = eb.job[j].n - g.R > cnd ? eb.job[j].n - g.R : cnd;
    if (cnd > PLAN_MAX_C) return hipErrorInvalidValue;
    const dim3 grid(g.Hkv * eb.count);
#define INFMLLM_SELECT(KPT) \
    hipLaunchKernelGGL(select_batch_kernel<KPT>, grid, dim3(TPB), 0, st, eb, r, g.R, g.B, g.cap, g.Hkv)
    if (cnd <= 2 * TPB) INFMLLM_SELECT(2);
    else if (cnd <= 4 * TPB) INFMLLM_SELECT(4);
    else if (cnd <= 8 * TPB) INFMLLM_SELECT(8);
    else if (cnd <= 16 * TPB) INFMLLM_SELECT(16);
    else INFMLLM_SELECT(0);
#undef INFMLLM_SELECT
    return hipGetLastError();
}

}  // namespace infmllm
