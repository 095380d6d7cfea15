// Plain fp32-arithmetic chunk attention and column scoring for gfx950.
//
// This is the path of fp32 streams (an fp32 contraction cannot go through the bf16 matrix
// cores within the 1e-4 output tolerance); bf16 streams use the MFMA kernels instead and
// reach this file only when the stream was created with the plain-arithmetic override.
//
//   attn_simple  : Sec. 3.2 -- the L new queries attend the t cached keys and, causally, the
//                  chunk's own keys.  One workgroup per (query row, query head): logits into
//                  LDS, block softmax, then P.V with lanes along head_dim.  Also writes the
//                  row's log-sum-exp, which the scoring kernel needs.
//   score_simple : Alg. 1 l.1-4 -- a thread owns one candidate key column (its key row lives in
//                  registers) and a quarter of the scored query rows, and sums the exact softmax
//                  weights exp(s - lse); the four quarters are added in a fixed order, then mean
//                  over rows and group heads, plus the bias ramp.  Column sums are complete
//                  inside a workgroup, so the result does not depend on any order across
//                  workgroups.
#include "launch.h"

namespace infmllm {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <typename T> struct Elt;
template <> struct Elt<float> {
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ f32x4 load4(const float* p) { return *(const f32x4*)p; }   // p 16-byte aligned
    static __device__ __forceinline__ void store(float* p, float x) { *p = x; }
};
template <> struct Elt<uint16_t> {   // bf16 held as raw bits
    static __device__ __forceinline__ float load(const uint16_t* p) { return __uint_as_float((uint32_t)(*p) << 16); }
    static __device__ __forceinline__ f32x4 load4(const uint16_t* p)                              // p 8-byte aligned
    {
        const u32x2 w = *(const u32x2*)p;
        return f32x4{__uint_as_float(w[0] << 16), __uint_as_float(w[0] & 0xffff0000u), __uint_as_float(w[1] << 16),
                     __uint_as_float(w[1] & 0xffff0000u)};
    }
    static __device__ __forceinline__ void store(uint16_t* p, float x)
    {
        uint32_t u = __float_as_uint(x);
        if ((u & 0x7fffffffu) > 0x7f800000u) { *p = (uint16_t)((u >> 16) | 0x40); return; }   // NaN
        u += 0x7fffu + ((u >> 16) & 1u);                                                      // RNE
        *p = (uint16_t)(u >> 16);
    }
};

__device__ __forceinline__ float block_reduce_max(float x, float* red)
{
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = x;
    __syncthreads();
    float r = red[0];
    for (int i = 1; i < (int)(blockDim.x >> 6); ++i) r = fmaxf(r, red[i]);
    return r;
}

__device__ __forceinline__ float block_reduce_sum(float x, float* red)
{
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = x;
    __syncthreads();
    float r = red[0];
    for (int i = 1; i < (int)(blockDim.x >> 6); ++i) r += red[i];
    return r;
}

// grid (L, Hq), 256 threads, dynamic LDS: n floats of logits/weights.
template <typename T, int D>
__global__ void __launch_bounds__(256)
attn_simple_kernel(const T* __restrict__ q, const T* __restrict__ K, const T* __restrict__ V,
                   T* __restrict__ out, float* __restrict__ lse, int t, int L, int Hq, int G, int cap,
                   int max_chunk, float scale)
{
    extern __shared__ float p[];                 // [vis]
    __shared__ float qs[D];
    __shared__ float red[4];
    __shared__ __attribute__((aligned(16))) float part[1024];   // [256 / (D/4)][D]

    const int i = blockIdx.x, g = blockIdx.y, h = g / G;
    const int vis = t + i + 1;                   // columns 0 .. t+i are visible
    const T* Kh = K + (size_t)h * cap * D;
    const T* Vh = V + (size_t)h * cap * D;
    const T* qi = q + ((size_t)i * Hq + g) * D;
    for (int x = threadIdx.x; x < D; x += 256) qs[x] = Elt<T>::load(qi + x);
    __syncthreads();

    float mx = -__builtin_inff();
    for (int j = threadIdx.x; j < vis; j += 256) {
        const T* kj = Kh + (size_t)j * D;
        float acc = 0.f;
#pragma unroll 4
        for (int x = 0; x < D; x += 4) {
            const f32x4 kv = Elt<T>::load4(kj + x);
            acc = fmaf(qs[x], kv[0], acc);
            acc = fmaf(qs[x + 1], kv[1], acc);
            acc = fmaf(qs[x + 2], kv[2], acc);
            acc = fmaf(qs[x + 3], kv[3], acc);
        }
        acc *= scale;
        p[j] = acc;
        mx = fmaxf(mx, acc);
    }
    mx = block_reduce_max(mx, red);
    float sum = 0.f;
    for (int j = threadIdx.x; j < vis; j += 256) {
        const float e = expf(p[j] - mx);
        p[j] = e;
        sum += e;
    }
    sum = block_reduce_sum(sum, red);            // its barriers also publish p[]
    const float inv = 1.0f / sum;

    constexpr int LPR = D / 4, NG = 256 / LPR;   // lanes along a value row (four columns each), groups along the keys
    const int x4 = 4 * (threadIdx.x % LPR), grp = threadIdx.x / LPR;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int j = grp; j < vis; j += 4 * NG) {                 // four rows requested before the first is used
        f32x4 vv[4];
        float w[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int ju = j + u * NG;
            vv[u] = Elt<T>::load4(Vh + (size_t)(ju < vis ? ju : j) * D + x4);
            w[u] = ju < vis ? p[ju] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            acc[0] = fmaf(w[u], vv[u][0], acc[0]);
            acc[1] = fmaf(w[u], vv[u][1], acc[1]);
            acc[2] = fmaf(w[u], vv[u][2], acc[2]);
            acc[3] = fmaf(w[u], vv[u][3], acc[3]);
        }
    }
    *(f32x4*)(part + grp * D + x4) = acc;
    __syncthreads();
    if (threadIdx.x < D) {
        float o = 0.f;
#pragma unroll
        for (int u = 0; u < NG; ++u) o += part[u * D + threadIdx.x];
        Elt<T>::store(out + ((size_t)i * Hq + g) * D + threadIdx.x, o * inv);
    }
    if (threadIdx.x == 0) lse[(size_t)g * max_chunk + i] = mx + logf(sum);
}

// grid (ceil(n/64), Hkv), 256 threads = 64 columns x 4 slices of the scored rows (a slice is a
// wavefront).  Thread = (column, slice): a column is a physical cache row p (all n rows are cached on this
// path), a candidate if its stream-order index j = rank[p] is below cnd; the key row lives in registers, the
// thread sums the weights of every fourth scored row, and the four slices are added in slice order.
template <typename T, int D>
__global__ void __launch_bounds__(256)
score_simple_kernel(const T* __restrict__ q, const T* __restrict__ K, const float* __restrict__ lse,
                    const float* __restrict__ carry, const int32_t* __restrict__ rank, float* __restrict__ Wb, int L,
                    int lq, int Hq, int G, int cap, int max_chunk, int cnd, int n, float scale, float dstep /* b / c, Alg. 1 l.2 */)
{
    constexpr int RT = 16, NS = 4;               // query rows staged per round, row slices
    constexpr int CPT = (RT * D / 4 + 255) / 256; // 16-byte chunks of a round per thread
    __shared__ __attribute__((aligned(16))) float qs[2][RT][D];
    __shared__ float ls[2][RT];
    __shared__ float red[NS][64];

    const int h = blockIdx.y;
    const int col = threadIdx.x & 63, slice = threadIdx.x >> 6;
    const int p = blockIdx.x * 64 + col;                                   // physical row
    const int j = p < n ? rank[(size_t)h * cap + p] : cnd;                 // stream-order index
    const bool live = j < cnd;
    float kr[D];
    {
        const T* kj = K + ((size_t)h * cap + (live ? p : 0)) * D;
#pragma unroll
        for (int x = 0; x < D; x += 4) {
            const f32x4 kv = Elt<T>::load4(kj + x);
            kr[x] = kv[0]; kr[x + 1] = kv[1]; kr[x + 2] = kv[2]; kr[x + 3] = kv[3];
        }
    }
    // Rounds of RT scored rows, over the heads of the group one after the other.  The rows of round rd + 1 are
    // requested before round rd is used and go to the other LDS buffer afterwards: one barrier per round.
    const int rpg = (lq + RT - 1) / RT, nrounds = G * rpg;
    f32x4 nq[CPT];
    float nl = 0.f;
    auto request = [&](int rd) {
        const int g = h * G + rd / rpg, i0 = L - lq + (rd % rpg) * RT;
        const int rows = min(RT, L - i0);
#pragma unroll
        for (int u = 0; u < CPT; ++u) {
            const int e = threadIdx.x + u * 256, r = e / (D / 4), x = 4 * (e % (D / 4));
            nq[u] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (r < rows) nq[u] = Elt<T>::load4(q + ((size_t)(i0 + r) * Hq + g) * D + x);
        }
        if (threadIdx.x < rows) nl = lse[(size_t)g * max_chunk + i0 + threadIdx.x];
    };
    auto publish = [&](int buf) {
#pragma unroll
        for (int u = 0; u < CPT; ++u) {
            const int e = threadIdx.x + u * 256, r = e / (D / 4), x = 4 * (e % (D / 4));
            if (r < RT) *(f32x4*)&qs[buf][r][x] = nq[u];
        }
        if (threadIdx.x < RT) ls[buf][threadIdx.x] = nl;
    };
    float acc = 0.f;
    if (nrounds > 0) { request(0); publish(0); }
    for (int rd = 0; rd < nrounds; ++rd) {
        const int buf = rd & 1;
        if (rd + 1 < nrounds) request(rd + 1);
        __syncthreads();                         // round rd is complete in qs[buf]; qs[buf ^ 1] is no longer read
        const int rows = min(RT, lq - (rd % rpg) * RT);
        for (int r = slice; r < rows; r += NS) {
            float s = 0.f;
#pragma unroll
            for (int x = 0; x < D; ++x) s = fmaf(qs[buf][r][x], kr[x], s);
            acc += expf(s * scale - ls[buf][r]);
        }
        if (rd + 1 < nrounds) publish(buf ^ 1);
    }
    red[slice][col] = acc;
    __syncthreads();
    if (live && slice == 0) {
        const float tot = ((red[0][col] + red[1][col]) + red[2][col]) + red[3][col];
        const float S = (lq > 0) ? tot / (float)(G * lq) : 0.f;        // Alg. 1 l.1, pooled over the group
        float w = S - (float)(cnd - 1 - j) * dstep;                    // Alg. 1 l.3-4
        if (carry) {                                                   // cumulative policy: total so far, no bias
            const float a = carry[(size_t)h * cap + p];
            w = S + (a < __builtin_inff() ? a : 0.f);                  // +inf marks a row never ranked
        }
        Wb[(size_t)h * cap + j] = w;
    }
}

}  // namespace

hipError_t launch_attn_simple(const Geometry& g, const CacheView& c, const void* q, int t, int L, void* out,
                              float* lse, hipStream_t st)
{
    const dim3 grid(L, g.Hq), block(256);
    const size_t lds = (size_t)(t + L) * sizeof(float);
#define INFMLLM_ATTN(TT, DD)                                                                            \
    do {                                                                                                \
        if (lds > 48 * 1024) {                                                                          \
            hipError_t e = hipFuncSetAttribute((const void*)attn_simple_kernel<TT, DD>,                 \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);   \
            if (e != hipSuccess) return e;                                                              \
        }                                                                                               \
        hipLaunchKernelGGL((attn_simple_kernel<TT, DD>), grid, block, lds, st, (const TT*)q,            \
                           (const TT*)c.K, (const TT*)c.V, (TT*)out, lse, t, L, g.Hq, g.G, g.cap,       \
                           g.max_chunk, (float)g.scale);                                                       \
    } while (0)
    if (g.elt == 4 && g.d == 64) INFMLLM_ATTN(float, 64);
    else if (g.elt == 4 && g.d == 128) INFMLLM_ATTN(float, 128);
    else if (g.elt == 2 && g.d == 64) INFMLLM_ATTN(uint16_t, 64);
    else if (g.elt == 2 && g.d == 128) INFMLLM_ATTN(uint16_t, 128);
    else return hipErrorInvalidValue;
#undef INFMLLM_ATTN
    return hipGetLastError();
}

hipError_t launch_score_simple(const Geometry& g, const CacheView& c, const void* q, const float* lse, int t,
                               int L, float* Wb, hipStream_t st)
{
    const int n = t + L, cnd = n - g.R, lq = g.R < L ? g.R : L;
    if (cnd <= 0) return hipSuccess;
    const dim3 grid((n + 63) / 64, g.Hkv), block(256);
#define INFMLLM_SCORE(TT, DD)                                                                           \
    hipLaunchKernelGGL((score_simple_kernel<TT, DD>), grid, block, 0, st, (const TT*)q, (const TT*)c.K, \
                       lse, g.policy == POLICY_CUMULATIVE ? c.score : nullptr, c.rank, Wb, L, lq, g.Hq, g.G, g.cap, \
                       g.max_chunk, cnd, n, (float)g.scale, (float)(g.bias / (double)cnd))
    if (g.elt == 4 && g.d == 64) INFMLLM_SCORE(float, 64);
    else if (g.elt == 4 && g.d == 128) INFMLLM_SCORE(float, 128);
    else if (g.elt == 2 && g.d == 64) INFMLLM_SCORE(uint16_t, 64);
    else if (g.elt == 2 && g.d == 128) INFMLLM_SCORE(uint16_t, 128);
    else return hipErrorInvalidValue;
#undef INFMLLM_SCORE
    return hipGetLastError();
}

}  // namespace infmllm
