// Device code of the per-head top-r selection (Alg. 1 l.5-7) and of the recent-window move, shared by the
// selection kernels and by the scoring kernel, whose last workgroup of a kv-head can run the selection
// itself.  TPB = threads of the calling workgroup.
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
        const int leader = __ffsll((long long)todo) - 1;
        const uint32_t dl = __shfl(digit, leader);
        const uint64_t same = __ballot(on && digit == dl);
        if (lane_id() == leader) atomicAdd(&hist[dl], (uint32_t)__popcll(same));
        todo &= ~same;
    }
}

// The recent window [c, n) is kept whatever the scores say (Alg. 1 l.6), so its rows can move to
// their final place, rows r .. B-1 of the other cache half, while the selection is still being
// worked out.  The selection occupies one workgroup per kv-head; the workgroups with
// blockIdx.x >= Hkv of the same launch do this copy on the CUs the selection leaves idle.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
struct RecentCopy {
    const u32x4* Ks; const u32x4* Vs; const int32_t* ps;      // live cache half
    const u32x4* kc; const u32x4* vc;                         // chunk tensors (rows >= tc), may be null
    u32x4* Kd; u32x4* Vd; int32_t* pd; float* sd;             // other half
    int tc, pos0, vpr, ncopy;                                 // vpr = 16-byte vectors per row
};

template <int TPB>
__device__ __forceinline__ void copy_recent(const RecentCopy& rc, int wg, int Hkv, int cnd, int r, int R, int cap)
{
    const long total = (long)Hkv * R * rc.vpr;
    for (long idx = (long)wg * TPB + threadIdx.x; idx < total; idx += (long)rc.ncopy * TPB) {
        const int x = (int)(idx % rc.vpr);
        const long hr = idx / rc.vpr;
        const int row = (int)(hr % R), h = (int)(hr / R);
        const int src = cnd + row, dst = r + row;
        const bool cached = src < rc.tc;
        const long so = cached ? ((long)h * cap + src) * rc.vpr + x : ((long)(src - rc.tc) * Hkv + h) * rc.vpr + x;
        const long dof = ((long)h * cap + dst) * rc.vpr + x;
        const u32x4 kk = __builtin_nontemporal_load((cached ? rc.Ks : rc.kc) + so);
        const u32x4 vv = __builtin_nontemporal_load((cached ? rc.Vs : rc.vc) + so);
        __builtin_nontemporal_store(kk, rc.Kd + dof);
        __builtin_nontemporal_store(vv, rc.Vd + dof);
        if (x == 0) {
            rc.pd[(long)h * cap + dst] = cached ? rc.ps[(long)h * cap + src] : rc.pos0 + (src - rc.tc);
            rc.sd[(long)h * cap + dst] = __builtin_inff();
        }
    }
}

// Same selection with the candidates of a head held in registers (KPT keys per thread, key
// k*1024 + tid in slot k): the scores are read from memory once, the first digit (sign and
// exponent bits, a handful of distinct values) is counted through ballots, the later digits
// (spread evenly) through plain LDS atomics, and the ordered write needs four barriers in all.
template <int KPT, int TPB, bool THROUGH>
__device__ __forceinline__ void select_reg_body(const float* __restrict__ Wb, int32_t* __restrict__ I,
                                                int32_t* __restrict__ userI, int32_t* __restrict__ user_count,
                                                int h, int cnd, int r, int R, int B, int cap)
{
    constexpr int NW = TPB / 64;
    __shared__ uint32_t hist[256];
    __shared__ uint32_t s_prefix, s_remaining, s_ties;
    __shared__ uint32_t tab_eq[KPT * NW], tab_keep[KPT * NW];

    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
    const float* W = Wb + (size_t)h * cap;
    int32_t* Ih = I + (size_t)h * B;
    int32_t* Uh = userI ? userI + (size_t)h * B : nullptr;

    if (r > 0) {
        uint32_t key[KPT];
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            const int j = k * TPB + tid;
            key[k] = 0u;                                      // 0 is below every real key
            if (j < cnd)
                key[k] = order_key(THROUGH ? __hip_atomic_load(W + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : W[j]);
        }
        if (tid == 0) { s_prefix = 0; s_remaining = (uint32_t)r; }
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            const uint32_t prefix = s_prefix;
            const uint32_t himask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
#pragma unroll
            for (int k = 0; k < KPT; ++k) {
                const bool on = (k * TPB + tid < cnd) && ((key[k] & himask) == prefix);
                const uint32_t digit = (key[k] >> shift) & 0xffu;
                if (pass == 0) wave_histogram(hist, digit, on);
                else if (on) atomicAdd(&hist[digit], 1u);
            }
            __syncthreads();
            if (tid < 64) {
                uint32_t c0 = hist[255 - 4 * l], c1 = hist[254 - 4 * l], c2 = hist[253 - 4 * l], c3 = hist[252 - 4 * l];
                uint32_t mine = c0 + c1 + c2 + c3, incl = mine;
                for (int o = 1; o < 64; o <<= 1) {
                    const uint32_t up = __shfl_up(incl, o);
                    if (l >= o) incl += up;
                }
                const uint32_t before = incl - mine, need = s_remaining;
                if (before < need && need <= incl) {
                    uint32_t acc = before;
                    int bin = 255 - 4 * l;
                    uint32_t cnt = c0;
                    if (acc + cnt < need) { acc += cnt; --bin; cnt = c1;
                        if (acc + cnt < need) { acc += cnt; --bin; cnt = c2;
                            if (acc + cnt < need) { acc += cnt; --bin; cnt = c3; } } }
                    s_prefix = prefix | ((uint32_t)bin << shift);
                    s_remaining = need - acc;
                    s_ties = cnt;
                }
            }
            __syncthreads();
        }
        const uint32_t T = s_prefix;
        const uint32_t skip_eq = s_ties - s_remaining;        // oldest ties that are dropped
        const uint64_t below = (l == 0) ? 0ull : (~0ull >> (64 - l));

        // rank among the ties, in index order: slot k, wavefront w, lane
        uint64_t beq[KPT];
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            beq[k] = __ballot((k * TPB + tid < cnd) && key[k] == T);
            if (l == 0) tab_eq[k * NW + w] = (uint32_t)__popcll(beq[k]);
        }
        __syncthreads();
        if (tid < 64) {                                       // exclusive scan of the KPT*NW counts
            uint32_t run = 0;
            for (int base = 0; base < KPT * NW; base += 64) {
                const int idx = base + l;
                const uint32_t v = idx < KPT * NW ? tab_eq[idx] : 0u;
                uint32_t incl = v;
                for (int o = 1; o < 64; o <<= 1) {
                    const uint32_t up = __shfl_up(incl, o);
                    if (l >= o) incl += up;
                }
                if (idx < KPT * NW) tab_eq[idx] = run + incl - v;
                run += __shfl(incl, 63);
            }
        }
        __syncthreads();
        uint64_t bkeep[KPT];
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            const bool in = k * TPB + tid < cnd;
            const uint32_t eq_rank = tab_eq[k * NW + w] + (uint32_t)__popcll(beq[k] & below);
            const bool keep = in && (key[k] > T || (key[k] == T && eq_rank >= skip_eq));
            bkeep[k] = __ballot(keep);
            if (l == 0) tab_keep[k * NW + w] = (uint32_t)__popcll(bkeep[k]);
        }
        __syncthreads();
        if (tid < 64) {
            uint32_t run = 0;
            for (int base = 0; base < KPT * NW; base += 64) {
                const int idx = base + l;
                const uint32_t v = idx < KPT * NW ? tab_keep[idx] : 0u;
                uint32_t incl = v;
                for (int o = 1; o < 64; o <<= 1) {
                    const uint32_t up = __shfl_up(incl, o);
                    if (l >= o) incl += up;
                }
                if (idx < KPT * NW) tab_keep[idx] = run + incl - v;
                run += __shfl(incl, 63);
            }
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            if ((bkeep[k] >> l) & 1ull) {
                const uint32_t dst = tab_keep[k * NW + w] + (uint32_t)__popcll(bkeep[k] & below);
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
