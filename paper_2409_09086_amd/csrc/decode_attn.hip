// Decoding step for gfx950 (Sec. 3.2, last paragraph): one new token per call, its query attends
// all t cached keys plus its own, nothing is evicted.
//
// One query row against n keys is a matrix-vector product: every K and V byte is used once, so the
// step is HBM-bound and runs on the vector ALUs (no matrix cores).  The key range of a kv-head is cut
// into `nsplit` pieces so that the grid covers the chip; a workgroup streams its piece with 16-byte
// loads (consecutive lanes cover a row), keeps one online-softmax state per row slot and query head
// of the group, merges the row slots through LDS and writes an un-normalised partial.  The workgroup
// of a kv-head that finishes last (a ticket counter per kv-head) merges the partials of its heads,
// so the step is one launch; the partials travel through agent-scope stores and loads, which go
// through to memory, so no cache has to be flushed.  The token's own k, v are read from the
// caller's tensors and written to cache row t by the workgroup that owns the last piece.
#include "launch.h"

namespace infmllm {

namespace {

constexpr int DEC_THREADS = 512;            // eight wavefronts: enough rows in flight per CU to cover the memory latency
constexpr float DEC_TAU = 8.0f;             // the softmax reference moves only when a logit exceeds it by 2^8

// Sum over the LPR consecutive lanes that cover one row, result in every lane (DPP butterflies).
template <int LPR>
__device__ __forceinline__ float row_sum(float x)
{

    // quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));
    if (LPR >= 8) x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true));
    if (LPR >= 16) x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, true));
    if (LPR >= 32) x += __shfl_xor(x, 16);
    return x;
}

template <typename T> struct Vec16;
template <> struct Vec16<uint16_t> {        // bf16 as raw bits, 8 per 16 bytes
    static constexpr int N = 8;
    typedef uint32_t raw __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ void unpack(raw r, float* f)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(r[i] << 16);
            f[2 * i + 1] = __uint_as_float(r[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ uint16_t from_float(float x)
    {
        uint32_t u = __float_as_uint(x);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
        u += 0x7fffu + ((u >> 16) & 1u);
        return (uint16_t)(u >> 16);
    }
};
template <> struct Vec16<float> {
    static constexpr int N = 4;
    typedef uint32_t raw __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ void unpack(raw r, float* f)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) f[i] = __uint_as_float(r[i]);
    }
    static __device__ __forceinline__ float from_float(float x) { return x; }
};

// part layout: [query head][split][D + 2] = {reference maximum (base-2 logits), sum, un-normalised out[D]}
// NG = query heads of the group handled per sweep over the keys (1, 2 or 4)
template <typename T, int D, int NG>
__global__ void __launch_bounds__(DEC_THREADS)
decode_partial_kernel(const T* __restrict__ q, const T* __restrict__ knew, const T* __restrict__ vnew,
                      T* __restrict__ K, T* __restrict__ V, int32_t* __restrict__ pos, float* __restrict__ score,
                      int32_t* __restrict__ rank, int32_t* __restrict__ row, float* __restrict__ part, int* __restrict__ arrived, T* __restrict__ out, int t, int G, int cap,
                      int nsplit, int pos_new, float c)
{
    using VT = Vec16<T>;
    typedef typename VT::raw raw;
    constexpr int VEC = VT::N;
    constexpr int LPR = D / VEC;                       // lanes that cover one row
    constexpr int SLOTS = DEC_THREADS / LPR;           // rows in flight per workgroup pass
    __shared__ float s_m[SLOTS][NG], s_l[SLOTS][NG];
    __shared__ float s_o[SLOTS][NG][D];
    __shared__ int s_ticket;

    const int sp = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
    const int slot = tid / LPR, cc = tid % LPR;
    const int n = t + 1;
    const int j0 = (int)((long)n * sp / nsplit), j1 = (int)((long)n * (sp + 1) / nsplit);
    const T* Kh = K + (size_t)h * cap * D;
    const T* Vh = V + (size_t)h * cap * D;

    for (int g0 = 0; g0 < G; g0 += NG) {               // G is a multiple of NG
        float qv[NG][VEC];
#pragma unroll
        for (int gg = 0; gg < NG; ++gg) VT::unpack(*(const raw*)(q + (size_t)(h * G + g0 + gg) * D + cc * VEC), qv[gg]);
        float m[NG], mu[NG], l[NG], o[NG][VEC];
#pragma unroll
        for (int gg = 0; gg < NG; ++gg) {
            m[gg] = -__builtin_inff();
            mu[gg] = 0.f;
            l[gg] = 0.f;
#pragma unroll
            for (int e = 0; e < VEC; ++e) o[gg][e] = 0.f;
        }
        // UNR rows per thread are loaded before any is used, to keep enough bytes in flight
        constexpr int UNR = 4;
        for (int row0 = j0 + slot; row0 < j1; row0 += UNR * SLOTS) {
            raw kr[UNR], vr[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int row = min(row0 + u * SLOTS, j1 - 1);      // clamped rows are skipped below
                const bool cached = row < t;                        // row t is the token being decoded
                kr[u] = *(const raw*)((cached ? Kh + (size_t)row * D : knew + (size_t)h * D) + cc * VEC);
                vr[u] = *(const raw*)((cached ? Vh + (size_t)row * D : vnew + (size_t)h * D) + cc * VEC);
            }
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                if (row0 + u * SLOTS >= j1) break;
                float kf[VEC], vf[VEC];
                VT::unpack(kr[u], kf);
                VT::unpack(vr[u], vf);
#pragma unroll
                for (int gg = 0; gg < NG; ++gg) {
                    float dot = 0.f;
#pragma unroll
                    for (int e = 0; e < VEC; ++e) dot = __builtin_fmaf(qv[gg][e], kf[e], dot);
                    const float s2 = row_sum<LPR>(dot) * c;
                    if (s2 > m[gg] + DEC_TAU) {             // same decision in all lanes of the row
                        const float alpha = __builtin_amdgcn_exp2f(m[gg] - s2);   // first row: 2^-inf = 0
                        m[gg] = s2;
                        mu[gg] = s2;
                        l[gg] *= alpha;
#pragma unroll
                        for (int e = 0; e < VEC; ++e) o[gg][e] *= alpha;
                    }
                    const float p = __builtin_amdgcn_exp2f(s2 - mu[gg]);
                    l[gg] += p;
#pragma unroll
                    for (int e = 0; e < VEC; ++e) o[gg][e] = __builtin_fmaf(p, vf[e], o[gg][e]);
                }
            }
        }
        // merge the row slots of the workgroup
        __syncthreads();
#pragma unroll
        for (int gg = 0; gg < NG; ++gg) {
            if (cc == 0) { s_m[slot][gg] = m[gg]; s_l[slot][gg] = l[gg]; }
#pragma unroll
            for (int e = 0; e < VEC; ++e) s_o[slot][gg][cc * VEC + e] = o[gg][e];
        }
        __syncthreads();
        for (int idx = tid; idx < NG * D; idx += DEC_THREADS) {
            const int gg = idx / D, x = idx % D;
            float mt = -__builtin_inff();
            for (int s = 0; s < SLOTS; ++s) mt = fmaxf(mt, s_m[s][gg]);
            const float mz = (mt == -__builtin_inff()) ? 0.f : mt;   // an empty piece keeps m = -inf, l = 0
            float lt = 0.f, ot = 0.f;
            for (int s = 0; s < SLOTS; ++s) {
                const float w = __builtin_amdgcn_exp2f(s_m[s][gg] - mz);
                lt += w * s_l[s][gg];
                ot += w * s_o[s][gg][x];
            }
            // The partials are read by whichever workgroup of this kv-head finishes last, possibly on another
            // XCD with its own L2: they are written with agent-scope stores, which go through to memory.
            float* pp = part + ((size_t)(h * G + g0 + gg) * nsplit + sp) * (D + 2);
            __hip_atomic_store(pp + 2 + x, ot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (x == 0) {
                __hip_atomic_store(pp, mt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(pp + 1, lt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
    // the token's own row becomes cache row t
    if (sp == nsplit - 1) {
        if (tid < LPR) {
            *(raw*)(K + ((size_t)h * cap + t) * D + tid * VEC) = *(const raw*)(knew + (size_t)h * D + tid * VEC);
            *(raw*)(V + ((size_t)h * cap + t) * D + tid * VEC) = *(const raw*)(vnew + (size_t)h * D + tid * VEC);
        }
        if (tid == 0) {
            pos[(size_t)h * cap + t] = pos_new;
            score[(size_t)h * cap + t] = __builtin_inff();
            rank[(size_t)h * cap + t] = t;                     // the newest token, in the first free physical row
            row[(size_t)h * cap + t] = t;
        }
    }
    // The workgroup of this kv-head that arrives last merges the splits: every workgroup waits until its own
    // partials have been written through, then takes a ticket.  No workgroup waits for another one.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) s_ticket = __hip_atomic_fetch_add(arrived + h, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (s_ticket != nsplit - 1) return;
    if (tid == 0) __hip_atomic_store(arrived + h, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next launch
    // out[head][x] = sum_s w_s o_s[x] / sum_s w_s l_s, w_s = 2^(m_s - max m); sixteen splits are requested at a
    // time before any is used (a loop over the splits would serialise the trips to memory, about a microsecond each)
    constexpr int CH = 16;
    for (int idx = tid; idx < G * D; idx += DEC_THREADS) {
        const int gq = h * G + idx / D, x = idx % D;
        const float* pp = part + (size_t)gq * nsplit * (D + 2);
        float mt = -__builtin_inff(), lt = 0.f, ot = 0.f;
        for (int s0 = 0; s0 < nsplit; s0 += CH) {
            float mv[CH], lv[CH], ov[CH];
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                const int s = min(s0 + u, nsplit - 1);
                mv[u] = __hip_atomic_load(pp + (size_t)s * (D + 2), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                lv[u] = __hip_atomic_load(pp + (size_t)s * (D + 2) + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ov[u] = __hip_atomic_load(pp + (size_t)s * (D + 2) + 2 + x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            float mc = mt;
#pragma unroll
            for (int u = 0; u < CH; ++u) mc = fmaxf(mc, mv[u]);
            const float rescale = __builtin_amdgcn_exp2f(mt - mc);          // first chunk: 2^-inf = 0
            lt *= rescale;
            ot *= rescale;
            mt = mc;
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                if (s0 + u >= nsplit) break;
                const float w = __builtin_amdgcn_exp2f(mv[u] - mt);         // an empty piece has m = -inf
                lt += w * lv[u];
                ot += w * ov[u];
            }
        }
        out[(size_t)gq * D + x] = VT::from_float(ot / lt);
    }
}

}  // namespace

hipError_t launch_decode(const Geometry& g, const CacheView& c, const void* q, const void* k, const void* v, int t,
                         int64_t T, void* out, float* part, int max_split, hipStream_t st)
{
    const int n = t + 1;
    int nsplit = 256 / g.Hkv;                           // one workgroup per CU (more only add partials to merge) ...
    if (nsplit > n / 256) nsplit = n / 256;             // ... of at least 256 keys each: two passes of its row slots
    if (nsplit > max_split) nsplit = max_split;
    if (nsplit < 1) nsplit = 1;
    const float cc = (float)(g.scale * 1.4426950408889634);
    int* arrived = (int*)(part + (size_t)g.Hq * max_split * (g.d + 2));   // one ticket counter per kv-head, zero between launches
    const dim3 grid(nsplit, g.Hkv);
#define INFMLLM_DECODE_NG(TT, DD, NG)                                                                            \
    hipLaunchKernelGGL((decode_partial_kernel<TT, DD, NG>), grid, dim3(DEC_THREADS), 0, st, (const TT*)q,        \
                       (const TT*)k, (const TT*)v, (TT*)c.K, (TT*)c.V, c.pos, c.score, c.rank, c.row, part, arrived, (TT*)out, t, \
                       g.G, g.cap, nsplit, (int)T, cc)
#define INFMLLM_DECODE(TT, DD)                                                                                   \
    do {                                                                                                         \
        if (g.G % 4 == 0) INFMLLM_DECODE_NG(TT, DD, 4);                                                          \
        else if (g.G % 2 == 0) INFMLLM_DECODE_NG(TT, DD, 2);                                                     \
        else INFMLLM_DECODE_NG(TT, DD, 1);                                                                       \
    } while (0)
    if (g.elt == 2 && g.d == 128) INFMLLM_DECODE(uint16_t, 128);
    else if (g.elt == 2 && g.d == 64) INFMLLM_DECODE(uint16_t, 64);
    else if (g.elt == 4 && g.d == 128) INFMLLM_DECODE(float, 128);
    else if (g.elt == 4 && g.d == 64) INFMLLM_DECODE(float, 64);
    else return hipErrorInvalidValue;
#undef INFMLLM_DECODE_NG
#undef INFMLLM_DECODE
    return hipGetLastError();
}

}  // namespace infmllm
