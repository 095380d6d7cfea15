// Cache maintenance kernels for gfx950: append (Sec. 3.2, first paragraph), the warm-up index
// list, the placement that completes an eviction (Alg. 1 l.8: only the retained rows that are not
// already inside physical rows 0..B-1 are moved, into the rows the eviction frees) and the export of
// the cache in stream order.  All are pure data movement and HBM-bound: every thread moves 16-byte
// vectors, a row of head_dim elements is covered by consecutive lanes so that each wavefront touches
// whole rows.
#include "launch.h"

namespace infmllm {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// chunk k/v [L][Hkv][d]  ->  cache rows [h][t+i][d]
__global__ void __launch_bounds__(256)
append_kernel(const u32x4* __restrict__ k, const u32x4* __restrict__ v, u32x4* __restrict__ K,
              u32x4* __restrict__ V, int32_t* __restrict__ pos, float* __restrict__ score,
              int32_t* __restrict__ rank, int32_t* __restrict__ row, int t, int L, int Hkv, int cap, int vec_per_row,
              int pos0)
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
            rank[(long)h * cap + t + i] = t + i;          // the cached rows fill physical rows 0..t-1, so the
            row[(long)h * cap + t + i] = t + i;           // next stream-order index and the next free row agree
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
reset_tables_kernel(float* __restrict__ score, int32_t* __restrict__ rank, int32_t* __restrict__ row, int len, int Hkv,
                    int cap)
{
    const int total = len * Hkv;
    for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += gridDim.x * blockDim.x) {
        const int h = idx / len, j = idx - h * len;
        score[(long)h * cap + j] = __builtin_inff();
        rank[(long)h * cap + j] = j;
        row[(long)h * cap + j] = j;
    }
}

// Entry k of a head's move list: the token in src[k] (a physical cache row at or above B, or a row of the
// chunk tensors) goes to physical row dst[k] (below B) and has stream-order index x[k] from now on.  One
// thread per 16-byte vector of a row of K and V, two rows in flight per thread.  Sources lie at or above B,
// destinations below it, so no row is read after it has been overwritten.
template <int VPR>
__device__ __forceinline__ void place_body(u32x4* __restrict__ K, u32x4* __restrict__ V, int32_t* __restrict__ pos,
                                           float* __restrict__ score, int32_t* __restrict__ rank,
                                           int32_t* __restrict__ row, const u32x4* __restrict__ kc,
                                           const u32x4* __restrict__ vc, int tc, int pos0, int Hkv, int cap,
                                           const int32_t* __restrict__ mv_src, const int32_t* __restrict__ mv_dst,
                                           const int32_t* __restrict__ mv_x, const float* __restrict__ mv_score,
                                           const int32_t* __restrict__ mv_count, int mv_max)
{
    constexpr int ROWS = 256 / VPR, U = 2;        // rows per block pass, passes in flight
    const int h = blockIdx.y;
    const int lane_row = threadIdx.x / VPR, xv = threadIdx.x % VPR;
    const long hb = (long)h * cap, mb = (long)h * mv_max;
    const int count = mv_count[h];
    for (int k0 = blockIdx.x * ROWS * U; k0 < count; k0 += gridDim.x * ROWS * U) {
        int sp[U], p[U];
        u32x4 kk[U], vv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = k0 + u * ROWS + lane_row;
            sp[u] = (k < count) ? mv_src[mb + k] : -1;
            p[u] = (k < count) ? mv_dst[mb + k] : 0;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (sp[u] >= 0) {
                const bool cached = sp[u] < tc;
                const long off = cached ? (hb + sp[u]) * VPR + xv : ((long)(sp[u] - tc) * Hkv + h) * VPR + xv;
                kk[u] = __builtin_nontemporal_load((cached ? (const u32x4*)K : kc) + off);
                vv[u] = __builtin_nontemporal_load((cached ? (const u32x4*)V : vc) + off);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (sp[u] >= 0) {
                K[(hb + p[u]) * VPR + xv] = kk[u];
                V[(hb + p[u]) * VPR + xv] = vv[u];
                if (xv == 0) {
                    const int k = k0 + u * ROWS + lane_row;
                    const int x = mv_x[mb + k];
                    pos[hb + p[u]] = sp[u] < tc ? pos[hb + sp[u]] : pos0 + (sp[u] - tc);
                    rank[hb + p[u]] = x;
                    row[hb + x] = p[u];
                    score[hb + p[u]] = mv_score[mb + k];
                }
            }
        }
    }
}

template <int VPR>
__global__ void __launch_bounds__(256)
place_kernel(u32x4* __restrict__ K, u32x4* __restrict__ V, int32_t* __restrict__ pos, float* __restrict__ score,
             int32_t* __restrict__ rank, int32_t* __restrict__ row, const u32x4* __restrict__ kc,
             const u32x4* __restrict__ vc, int tc, int pos0, int Hkv, int cap, const int32_t* __restrict__ mv_src,
             const int32_t* __restrict__ mv_dst, const int32_t* __restrict__ mv_x, const float* __restrict__ mv_score,
             const int32_t* __restrict__ mv_count, int mv_max)
{
    place_body<VPR>(K, V, pos, score, rank, row, kc, vc, tc, pos0, Hkv, cap, mv_src, mv_dst, mv_x, mv_score, mv_count,
                    mv_max);
}

// blockIdx.z = stream of the batch
template <int VPR>
__global__ void __launch_bounds__(256)
place_batch_kernel(EvictBatch eb, int Hkv, int cap)
{
    const EvictJob& j = eb.job[blockIdx.z];
    place_body<VPR>((u32x4*)j.c.K, (u32x4*)j.c.V, j.c.pos, j.c.score, j.c.rank, j.c.row, (const u32x4*)j.kc,
                    (const u32x4*)j.vc, j.tc, j.pos0, Hkv, cap, j.mv.src, j.mv.dst, j.mv.x, j.mv.score, j.mv.count,
                    j.mv.max);
}

// out row j of head h <- physical row row[h][j]: the cache in stream order.
template <int VPR>
__global__ void __launch_bounds__(256)
export_rows_kernel(const u32x4* __restrict__ K, const u32x4* __restrict__ V, const int32_t* __restrict__ row,
                   u32x4* __restrict__ Kout, u32x4* __restrict__ Vout, int len, int cap)
{
    constexpr int ROWS = 256 / VPR;
    const int h = blockIdx.y, lane_row = threadIdx.x / VPR, xv = threadIdx.x % VPR;
    for (int j = blockIdx.x * ROWS + lane_row; j < len; j += gridDim.x * ROWS) {
        const long src = ((long)h * cap + row[(long)h * cap + j]) * VPR + xv, dst = ((long)h * len + j) * VPR + xv;
        if (Kout) Kout[dst] = K[src];
        if (Vout) Vout[dst] = V[src];
    }
}

__global__ void __launch_bounds__(256)
export_scalars_kernel(const int32_t* __restrict__ pos, const float* __restrict__ score, const int32_t* __restrict__ row,
                      int32_t* __restrict__ pos_out, float* __restrict__ score_out, int len, int Hkv, int cap, int pitch)
{
    const int total = len * Hkv;
    for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += gridDim.x * blockDim.x) {
        const int h = idx / len, j = idx - h * len;
        const long p = (long)h * cap + row[(long)h * cap + j];
        if (pos_out) pos_out[(long)h * pitch + j] = pos[p];
        if (score_out) score_out[(long)h * pitch + j] = score[p];
    }
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
                       (u32x4*)c.K, (u32x4*)c.V, c.pos, c.score, c.rank, c.row, t, L, g.Hkv, g.cap, vpr, (int)T);
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

hipError_t launch_reset_tables(const Geometry& g, const CacheView& c, int len, hipStream_t st)
{
    if (len <= 0) return hipSuccess;
    int blocks = (len * g.Hkv + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(reset_tables_kernel, dim3(blocks), dim3(256), 0, st, c.score, c.rank, c.row, len, g.Hkv, g.cap);
    return hipGetLastError();
}

hipError_t launch_place(const Geometry& g, const CacheView& c, const KeySource& ks, int64_t T, const MoveList& mv,
                        int nmax, hipStream_t st)
{
    const int vpr = g.d * g.elt / 16;             // 8 (d=64 bf16), 16 (d=128 bf16 / d=64 fp32), 32 (d=128 fp32)
    const int rows_per_pass = (256 / vpr) * 2;
    if (nmax <= 0) return hipSuccess;
    if (nmax > mv.max) return hipErrorInvalidValue;
    const dim3 grid((nmax + rows_per_pass - 1) / rows_per_pass, g.Hkv), block(256);
#define INFMLLM_PLACE(VPR)                                                                                      \
    hipLaunchKernelGGL(place_kernel<VPR>, grid, block, 0, st, (u32x4*)c.K, (u32x4*)c.V, c.pos, c.score, c.rank, c.row, \
                       (const u32x4*)ks.k, (const u32x4*)ks.v, ks.rows, (int)T, g.Hkv, g.cap, mv.src, mv.dst, mv.x,     \
                       mv.score, mv.count, mv.max)
    switch (vpr) {
        case 8: INFMLLM_PLACE(8); break;
        case 16: INFMLLM_PLACE(16); break;
        case 32: INFMLLM_PLACE(32); break;
        default: return hipErrorInvalidValue;
    }
#undef INFMLLM_PLACE
    return hipGetLastError();
}

hipError_t launch_place_batch(const Geometry& g, const EvictBatch& eb, int nmax, hipStream_t st)
{
    if (eb.count < 1 || eb.count > EVICT_MAX_JOBS) return hipErrorInvalidValue;
    const int vpr = g.d * g.elt / 16;
    const int rows_per_pass = (256 / vpr) * 2;
    if (nmax <= 0) return hipSuccess;
    const dim3 grid((nmax + rows_per_pass - 1) / rows_per_pass, g.Hkv, eb.count), block(256);
    switch (vpr) {
        case 8: hipLaunchKernelGGL(place_batch_kernel<8>, grid, block, 0, st, eb, g.Hkv, g.cap); break;
        case 16: hipLaunchKernelGGL(place_batch_kernel<16>, grid, block, 0, st, eb, g.Hkv, g.cap); break;
        case 32: hipLaunchKernelGGL(place_batch_kernel<32>, grid, block, 0, st, eb, g.Hkv, g.cap); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_export(const Geometry& g, const CacheView& c, int len, void* Kout, void* Vout, int32_t* pos_out,
                         float* score_out, int pitch, hipStream_t st)
{
    if (len <= 0) return hipSuccess;
    const int vpr = g.d * g.elt / 16;
    if (Kout || Vout) {
        const int rows = 256 / vpr;
        int bx = (len + rows - 1) / rows;
        if (bx > 2048) bx = 2048;
        const dim3 grid(bx, g.Hkv), block(256);
        switch (vpr) {
            case 8: hipLaunchKernelGGL(export_rows_kernel<8>, grid, block, 0, st, (const u32x4*)c.K, (const u32x4*)c.V, c.row, (u32x4*)Kout, (u32x4*)Vout, len, g.cap); break;
            case 16: hipLaunchKernelGGL(export_rows_kernel<16>, grid, block, 0, st, (const u32x4*)c.K, (const u32x4*)c.V, c.row, (u32x4*)Kout, (u32x4*)Vout, len, g.cap); break;
            case 32: hipLaunchKernelGGL(export_rows_kernel<32>, grid, block, 0, st, (const u32x4*)c.K, (const u32x4*)c.V, c.row, (u32x4*)Kout, (u32x4*)Vout, len, g.cap); break;
            default: return hipErrorInvalidValue;
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (pos_out || score_out) {
        int blocks = (len * g.Hkv + 255) / 256;
        if (blocks > 1024) blocks = 1024;
        hipLaunchKernelGGL(export_scalars_kernel, dim3(blocks), dim3(256), 0, st, c.pos, c.score, c.row, pos_out,
                           score_out, len, g.Hkv, g.cap, pitch);
    }
    return hipGetLastError();
}

}  // namespace infmllm
