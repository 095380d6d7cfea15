// Cache-relative rotary position encoding for gfx950 (Sec. 3.4: length extrapolation; Sec. 4.1: the
// models use rotary embeddings).  Keys are cached as given; before attention is computed the key in
// cache row j is turned to position j and the query of chunk row i to position t + i, so relative
// distances are distances inside the cache.  This pre-pass writes the turned copies (K_rot in the cache
// layout, the chunk's keys and the queries token-major) which the attention and scoring kernels then read
// in place of the originals; selection and compaction keep working on the unrotated rows.
//
// Pair (x[i], x[i + d/2]) is turned by p * base^(-2i/d).  The turned values are stored in the stream's
// element type, as a model stores its rotated q and k.  The arithmetic is fp64 on a (cos, sin) table
// computed on the host in fp64, so that each stored value is the correctly rounded one: an fp32 rotation
// lands on the other side of a bf16 rounding boundary about once in 10^5 values, and one such key can
// change which rows a step retains.  The pass is HBM-bound; the fp64 work hides behind the loads.
#include "launch.h"

namespace infmllm {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int ROPE_HPT = 4;                                   // heads per thread

template <typename T> struct Oct;                             // eight consecutive elements of a row
template <> struct Oct<uint16_t> {
    u32x4 raw;
    __device__ __forceinline__ void load(const uint16_t* p) { raw = *(const u32x4*)p; }
    __device__ __forceinline__ void store(uint16_t* p) const { *(u32x4*)p = raw; }
    __device__ __forceinline__ double get(int e) const
    {
        const uint32_t w = raw[e >> 1];
        return (double)__uint_as_float((e & 1) ? (w & 0xffff0000u) : (w << 16));
    }
    // elements 2w and 2w + 1 at once; each is rounded to nearest even twice: to fp32, then to bf16
    __device__ __forceinline__ void set2(int w, double v0, double v1)
    {
        uint32_t u0 = __float_as_uint((float)v0), u1 = __float_as_uint((float)v1);
        u0 += 0x7fffu + ((u0 >> 16) & 1u);
        u1 += 0x7fffu + ((u1 >> 16) & 1u);
        raw[w] = (u0 >> 16) | (u1 & 0xffff0000u);
    }
};
template <> struct Oct<float> {
    f32x4 lo, hi;
    __device__ __forceinline__ void load(const float* p) { lo = *(const f32x4*)p; hi = *(const f32x4*)(p + 4); }
    __device__ __forceinline__ void store(float* p) const { *(f32x4*)p = lo; *(f32x4*)(p + 4) = hi; }
    __device__ __forceinline__ double get(int e) const { return (double)(e < 4 ? lo[e & 3] : hi[e & 3]); }
    __device__ __forceinline__ void set2(int w, double v0, double v1)
    {
        if (w < 2) { lo[2 * w] = (float)v0; lo[2 * w + 1] = (float)v1; }
        else { hi[2 * w - 4] = (float)v0; hi[2 * w - 3] = (float)v1; }
    }
};

// One thread = one (row, group of 8 pairs, group of HPT heads): the table entries are loaded once and the
// HPT heads of that row are turned with them; blockIdx.y picks the group of heads.  Rows: physical cache rows
// [j0, j1) (position = the row's stream-order index rank[h][p], looked up per head), then the chunk's L key rows
// (position t + i, if kc is given), then the L query rows (position t + i).
template <typename T, int D>
__global__ void __launch_bounds__(256)
rope_kernel(const T* __restrict__ K, T* __restrict__ Krot, const int32_t* __restrict__ rank, int j0, int j1, int cap, int Hkv,
            const T* __restrict__ kc, T* __restrict__ kcrot, const T* __restrict__ q, T* __restrict__ qrot, int Hq,
            int t, int L, const double2* __restrict__ tab)
{
    constexpr int GPR = D / 16;                               // groups of 8 pairs per row
    const int nA = j1 - j0, nB = kc ? L : 0, nC = q ? L : 0;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)(nA + nB + nC) * GPR) return;
    const int item = (int)(idx / GPR), cc = (int)(idx % GPR);
    int pos = 0, heads;
    const T* src;
    T* dst;
    long hstride;                                             // elements between two heads of the same row
    const bool cache_row = item < nA;
    if (cache_row) {
        const int p = j0 + item;                              // physical row; its position differs from head to head
        heads = Hkv; hstride = (long)cap * D;
        src = K + (long)p * D; dst = Krot + (long)p * D;
        rank += p;
    } else if (item < nA + nB) {
        const int i = item - nA;
        pos = t + i; heads = Hkv; hstride = D;
        src = kc + (long)i * Hkv * D; dst = kcrot + (long)i * Hkv * D;
    } else {
        const int i = item - nA - nB;
        pos = t + i; heads = Hq; hstride = D;
        src = q + (long)i * Hq * D; dst = qrot + (long)i * Hq * D;
    }
    double cs[8], sn[8];
    auto table = [&](int at) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const double2 v = tab[(long)at * (D / 2) + e * GPR + cc];   // lanes of a row read consecutive entries
            cs[e] = v.x; sn[e] = v.y;
        }
    };
    const int h0 = blockIdx.y * ROPE_HPT, h1 = min(heads, h0 + ROPE_HPT);
    auto turn = [&](const Oct<T>& a, const Oct<T>& b, T* out) {
        Oct<T> ra, rb;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const double x0 = a.get(2 * w), y0 = b.get(2 * w), x1 = a.get(2 * w + 1), y1 = b.get(2 * w + 1);
            ra.set2(w, x0 * cs[2 * w] - y0 * sn[2 * w], x1 * cs[2 * w + 1] - y1 * sn[2 * w + 1]);
            rb.set2(w, y0 * cs[2 * w] + x0 * sn[2 * w], y1 * cs[2 * w + 1] + x1 * sn[2 * w + 1]);
        }
        ra.store(out + 8 * cc);
        rb.store(out + D / 2 + 8 * cc);
    };
    if (cache_row) {
        // a cached row's position is its stream-order index in its own head's cache
        for (int h = h0; h < h1; ++h) {
            Oct<T> a, b;
            a.load(src + h * hstride + 8 * cc);
            b.load(src + h * hstride + D / 2 + 8 * cc);
            table(rank[(long)h * cap]);
            turn(a, b, dst + h * hstride);
        }
        return;
    }
    table(pos);
    if (h1 - h0 == ROPE_HPT) {
        // a full group of heads: every load is requested before the first value is used
        Oct<T> a[ROPE_HPT], b[ROPE_HPT];                      // x[8cc .. 8cc+8) and x[d/2 + 8cc .. +8)
#pragma unroll
        for (int u = 0; u < ROPE_HPT; ++u) {
            a[u].load(src + (h0 + u) * hstride + 8 * cc);
            b[u].load(src + (h0 + u) * hstride + D / 2 + 8 * cc);
        }
#pragma unroll
        for (int u = 0; u < ROPE_HPT; ++u) turn(a[u], b[u], dst + (h0 + u) * hstride);
    } else {
        for (int h = h0; h < h1; ++h) {
            Oct<T> a, b;
            a.load(src + h * hstride + 8 * cc);
            b.load(src + h * hstride + D / 2 + 8 * cc);
            turn(a, b, dst + h * hstride);
        }
    }
}

}  // namespace

hipError_t launch_rope(const Geometry& g, const void* K, void* Krot, const int32_t* rank, int j0, int j1,
                       const void* kc, void* kcrot, const void* q, void* qrot, int t, int L, const double* tab,
                       hipStream_t st)
{
    if (j1 < j0) j1 = j0;
    const long items = (long)(j1 - j0) + (kc ? L : 0) + (q ? L : 0);
    if (items <= 0) return hipSuccess;
    const long threads = items * (g.d / 16);
    const int hmax = g.Hq > g.Hkv ? g.Hq : g.Hkv;
    const dim3 grid((unsigned)((threads + 255) / 256), (unsigned)((hmax + ROPE_HPT - 1) / ROPE_HPT)), block(256);
#define INFMLLM_ROPE(TT, DD)                                                                                  \
    hipLaunchKernelGGL((rope_kernel<TT, DD>), grid, block, 0, st, (const TT*)K, (TT*)Krot, rank, j0, j1, g.cap, g.Hkv, \
                       (const TT*)kc, (TT*)kcrot, (const TT*)q, (TT*)qrot, g.Hq, t, L, (const double2*)tab)
    if (g.elt == 2 && g.d == 128) INFMLLM_ROPE(uint16_t, 128);
    else if (g.elt == 2 && g.d == 64) INFMLLM_ROPE(uint16_t, 64);
    else if (g.elt == 4 && g.d == 128) INFMLLM_ROPE(float, 128);
    else if (g.elt == 4 && g.d == 64) INFMLLM_ROPE(float, 64);
    else return hipErrorInvalidValue;
#undef INFMLLM_ROPE
    return hipGetLastError();
}

}  // namespace infmllm
