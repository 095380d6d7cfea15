// Cache maintenance kernels for gfx950: append (Sec. 3.2, first paragraph), the warm-up index
// list, and the gather that compresses the cache (Alg. 1 l.8).  All three are pure data
// movement and HBM-bound: every thread moves 16-byte vectors, a row of head_dim elements is
// covered by consecutive lanes so that each wavefront touches whole rows.
#include "launch.h"

namespace infmllm {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// chunk k/v [L][Hkv][d]  ->  cache rows [h][t+i][d]
__global__ void __launch_bounds__(256)
append_kernel(const u32x4* __restrict__ k, const u32x4* __restrict__ v, u32x4* __restrict__ K,
              u32x4* __restrict__ V, int32_t* __restrict__ pos, float* __restrict__ score, int t, int L,
              int Hkv, int cap, int vec_per_row, int pos0)
{
    const long total = (long)L * Hkv * vec_per_row;
    for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (long)gridDim.x * blockDim.x) {
        const int x = (int)(idx % vec_per_row);
        const long ih = idx / vec_per_row;
        const int h = (int)(ih % Hkv);
        const int i = (int)(ih / Hkv);
        const long dst = ((long)h * cap + t + i) * vec_per_row + x;
        K[dst] = k[idx];
        V[dst] = v[idx];
        if (x == 0) {
            pos[(long)h * cap + t + i] = pos0 + i;
            score[(long)h * cap + t + i] = __builtin_inff();
        }
    }
}

__global__ void __launch_bounds__(256)
zero_kernel(u32x4* __restrict__ p, size_t nvec)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += (size_t)gridDim.x * blockDim.x)
        p[i] = u32x4{0u, 0u, 0u, 0u};
}

__global__ void __launch_bounds__(256)
iota_kernel(int32_t* __restrict__ I, int32_t* __restrict__ count, int n, int Hkv, int B)
{
    const int total = n * Hkv;
    for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += gridDim.x * blockDim.x) {
        const int h = idx / n, j = idx - h * n;
        if (I) I[(long)h * B + j] = j;
    }
    if (count && blockIdx.x == 0 && threadIdx.x == 0) *count = n;
}

__global__ void __launch_bounds__(256)
rank_score_kernel(float* __restrict__ Wb, int cnd, int Hkv, int cap, float sign)
{
    const int total = cnd * Hkv;
    for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += gridDim.x * blockDim.x) {
        const int h = idx / cnd, j = idx - h * cnd;
        Wb[(long)h * cap + j] = sign * (float)j;
    }
}

__global__ void __launch_bounds__(256)
fill_inf_kernel(float* __restrict__ score, int len, int Hkv, int cap)
{
    const int total = len * Hkv;
    for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += gridDim.x * blockDim.x) {
        const int h = idx / len, j = idx - h * len;
        score[(long)h * cap + j] = __builtin_inff();
    }
}

// dst[h][x] <- src[h][I[h][x]] for x < rows (the relevant rows; I has row stride B).  One thread per
// 16-byte vector of a row of K and V.
template <int VPR>
__device__ __forceinline__ void compact_body(const u32x4* __restrict__ Ks, const u32x4* __restrict__ Vs,
                                             const int32_t* __restrict__ ps, const u32x4* __restrict__ kc,
                                             const u32x4* __restrict__ vc, int tc, int pos0, int Hkv,
                                             u32x4* __restrict__ Kd, u32x4* __restrict__ Vd,
                                             int32_t* __restrict__ pd, float* __restrict__ sd,
                                             const int32_t* __restrict__ I, const float* __restrict__ Wb, int B,
                                             int rows, int cap)
{
    constexpr int ROWS = 256 / VPR;               // rows per block pass
    const int h = blockIdx.y;
    const int lane_row = threadIdx.x / VPR, x = threadIdx.x % VPR;
    const long hb = (long)h * cap;
    for (int row0 = blockIdx.x * ROWS * 4; row0 < rows; row0 += gridDim.x * ROWS * 4) {
        int src[4];
        u32x4 kk[4], vv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = row0 + u * ROWS + lane_row;
            src[u] = (r < rows) ? I[(long)h * B + r] : -1;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (src[u] >= 0) {
                const bool cached = src[u] < tc;          // else the row is still in the chunk tensors
                const long off = cached ? (hb + src[u]) * VPR + x : ((long)(src[u] - tc) * Hkv + h) * VPR + x;
                kk[u] = __builtin_nontemporal_load((cached ? Ks : kc) + off);
                vv[u] = __builtin_nontemporal_load((cached ? Vs : vc) + off);
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = row0 + u * ROWS + lane_row;
            if (src[u] >= 0) {
                __builtin_nontemporal_store(kk[u], &Kd[(hb + r) * VPR + x]);
                __builtin_nontemporal_store(vv[u], &Vd[(hb + r) * VPR + x]);
                if (x == 0) {
                    pd[hb + r] = (src[u] < tc) ? ps[hb + src[u]] : pos0 + (src[u] - tc);
                    sd[hb + r] = Wb[(long)h * cap + src[u]];
                }
            }
        }
    }
}

template <int VPR>
__global__ void __launch_bounds__(256)
compact_kernel(const u32x4* __restrict__ Ks, const u32x4* __restrict__ Vs, const int32_t* __restrict__ ps,
               const u32x4* __restrict__ kc, const u32x4* __restrict__ vc, int tc, int pos0, int Hkv,
               u32x4* __restrict__ Kd, u32x4* __restrict__ Vd, int32_t* __restrict__ pd,
               float* __restrict__ sd, const int32_t* __restrict__ I, const float* __restrict__ Wb,
               int B, int rows, int cap)
{
    compact_body<VPR>(Ks, Vs, ps, kc, vc, tc, pos0, Hkv, Kd, Vd, pd, sd, I, Wb, B, rows, cap);
}

// blockIdx.z = stream of the batch
template <int VPR>
__global__ void __launch_bounds__(256)
compact_batch_kernel(EvictBatch eb, int Hkv, int B, int rows, int cap)
{
    const EvictJob& j = eb.job[blockIdx.z];
    compact_body<VPR>((const u32x4*)j.src.K, (const u32x4*)j.src.V, j.src.pos, (const u32x4*)j.kc, (const u32x4*)j.vc,
                      j.tc, j.pos0, Hkv, (u32x4*)j.dst.K, (u32x4*)j.dst.V, j.dst.pos, j.dst.score, j.I, j.Wb, B, rows,
                      cap);
}

}  // namespace

hipError_t launch_append(const Geometry& g, const CacheView& c, const void* k, const void* v, int t,
                         int L, int64_t T, hipStream_t st)
{
    const int vpr = g.d * g.elt / 16;
    const long total = (long)L * g.Hkv * vpr;
    int blocks = (int)((total + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(append_kernel, dim3(blocks), dim3(256), 0, st, (const u32x4*)k, (const u32x4*)v,
                       (u32x4*)c.K, (u32x4*)c.V, c.pos, c.score, t, L, g.Hkv, g.cap, vpr, (int)T);
    return hipGetLastError();
}

hipError_t launch_zero(void* p, size_t bytes, hipStream_t st)
{
    if (bytes == 0) return hipSuccess;
    if (((uintptr_t)p | bytes) & 15) return hipErrorInvalidValue;
    const size_t nvec = bytes / 16;
    size_t blocks = (nvec + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(zero_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (u32x4*)p, nvec);
    return hipGetLastError();
}

hipError_t launch_iota(const Geometry& g, int n, int32_t* user_I, int32_t* user_count, hipStream_t st)
{
    if (!user_I && !user_count) return hipSuccess;
    int blocks = (n * g.Hkv + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(iota_kernel, dim3(blocks), dim3(256), 0, st, user_I, user_count, n, g.Hkv, g.B);
    return hipGetLastError();
}

hipError_t launch_rank_scores(const Geometry& g, float* Wb, int cnd, float sign, hipStream_t st)
{
    if (cnd <= 0) return hipSuccess;
    int blocks = (cnd * g.Hkv + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(rank_score_kernel, dim3(blocks), dim3(256), 0, st, Wb, cnd, g.Hkv, g.cap, sign);
    return hipGetLastError();
}

hipError_t launch_fill_inf(const Geometry& g, float* score, int len, hipStream_t st)
{
    if (len <= 0) return hipSuccess;
    int blocks = (len * g.Hkv + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(fill_inf_kernel, dim3(blocks), dim3(256), 0, st, score, len, g.Hkv, g.cap);
    return hipGetLastError();
}

hipError_t launch_compact(const Geometry& g, const CacheView& src, const KeySource& ks, int64_t T,
                          const CacheView& dst, const int32_t* I, const float* Wb, int n, hipStream_t st)
{
    const int vpr = g.d * g.elt / 16;             // 8 (d=64 bf16), 16 (d=128 bf16 / d=64 fp32), 32 (d=128 fp32)
    const int rows_per_pass = (256 / vpr) * 4;
    const int rows = g.B - g.R;                   // the recent rows have been moved already
    (void)n;
    if (rows <= 0) return hipSuccess;
    int bx = (rows + rows_per_pass - 1) / rows_per_pass;
    const dim3 grid(bx, g.Hkv), block(256);
#define INFMLLM_COMPACT(VPR)                                                                          \
    hipLaunchKernelGGL(compact_kernel<VPR>, grid, block, 0, st, (const u32x4*)src.K, (const u32x4*)src.V, \
                       src.pos, (const u32x4*)ks.k, (const u32x4*)ks.v, ks.rows, (int)T, g.Hkv, (u32x4*)dst.K,  \
                       (u32x4*)dst.V, dst.pos, dst.score, I, Wb, g.B, rows, g.cap)
    switch (vpr) {
        case 8: INFMLLM_COMPACT(8); break;
        case 16: INFMLLM_COMPACT(16); break;
        case 32: INFMLLM_COMPACT(32); break;
        default: return hipErrorInvalidValue;
    }
#undef INFMLLM_COMPACT
    return hipGetLastError();
}

hipError_t launch_compact_batch(const Geometry& g, const EvictBatch& eb, hipStream_t st)
{
    if (eb.count < 1 || eb.count > EVICT_MAX_JOBS) return hipErrorInvalidValue;
    const int vpr = g.d * g.elt / 16;
    const int rows_per_pass = (256 / vpr) * 4;
    const int rows = g.B - g.R;
    if (rows <= 0) return hipSuccess;
    const dim3 grid((rows + rows_per_pass - 1) / rows_per_pass, g.Hkv, eb.count), block(256);
    switch (vpr) {
        case 8: hipLaunchKernelGGL(compact_batch_kernel<8>, grid, block, 0, st, eb, g.Hkv, g.B, rows, g.cap); break;
        case 16: hipLaunchKernelGGL(compact_batch_kernel<16>, grid, block, 0, st, eb, g.Hkv, g.B, rows, g.cap); break;
        case 32: hipLaunchKernelGGL(compact_batch_kernel<32>, grid, block, 0, st, eb, g.Hkv, g.B, rows, g.cap); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace infmllm
