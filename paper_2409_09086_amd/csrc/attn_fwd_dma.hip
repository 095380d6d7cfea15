// Chunk attention (Sec. 3.2) on bf16 matrix cores for head_dim 128, with K/V tiles brought from
// global memory straight into LDS (global_load_lds, 16 bytes per lane) instead of through
// registers.  Arithmetic, tile shapes, key ways and key split are those of the register-staged
// kernel; what changes is the staging:
//   * no staging registers, no LDS store instructions and no wait for the loads in the middle of
//     an iteration: the loads of tile i+1 are issued at the top of iteration i and are only waited
//     for at its end, right before the single barrier;
//   * LDS rows are unpadded (the hardware writes 64 consecutive 16-byte slots per load); bank
//     conflicts are avoided by permuting which source chunk each lane loads (see the kernel).
#include <type_traits>

#include "launch.h"
#include "mfma_common.h"

namespace infmllm {

namespace {

template <int RB, int KW, int KVB>
struct DmaCfg {
    static constexpr int D = 128;
    static constexpr int NW = RB * KW, NT = 64 * NW;
    static constexpr int SUB = KVB * 32, TILE = KW * SUB;
    static constexpr int NLD = TILE / 4 / NW;              // 1-KB (4-row) loads per wavefront per tensor per tile
    static constexpr int KBYTES = TILE * 256, VBYTES = TILE * 256;
    static constexpr int OREG = D / 2;                     // fp32 accumulators of O^T per lane
    static constexpr int MERGE = (KW - 1) * RB * 64 * (OREG + 2) * 4;
    static constexpr int TILES = 2 * (KBYTES + VBYTES);    // [K0 K1 V0 V1]
    static constexpr int LDS = TILES > MERGE ? TILES : MERGE;
    static_assert(TILE % (4 * NW) == 0, "tile must split evenly over the wavefronts");
    static_assert(TILE <= CACHE_PAD_ROWS, "workspace padding assumes smaller tiles");
    static_assert(KBYTES <= 32768, "buffer offsets must fit the LDS instruction offset field");
};

template <int RB, int KW, int KVB>
__global__ void __launch_bounds__(64 * RB * KW)
attn_fwd_dma_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
                uint16_t* __restrict__ out, float* __restrict__ lse2, int t, int L, int Hq, int G, int cap,
                int max_chunk, int hpw, int ntile, int ny, int nsplit, float* __restrict__ part_o,
                float* __restrict__ part_ml, float c /* scale * log2(e) */)
{
    using C = DmaCfg<RB, KW, KVB>;
    constexpr int D = 128;
    __shared__ __attribute__((aligned(16))) char smem[C::LDS];

    // Workgroup -> (row tile, head group).  Consecutive workgroup ids go round-robin over the 8
    // XCDs; all row tiles of one kv-head are given ids of one residue class so that they share
    // that XCD's L2 copy of the head's K and V.
    // With nsplit > 1 the key range of a row tile is cut into nsplit pieces handled by different
    // workgroups; each writes an un-normalised partial and a second kernel combines them.
    int bx, by, sp;
    {
        const int bid = blockIdx.x, per_y = ntile * nsplit;
        int rem;
        if ((ny & 7) == 0) {
            const int xcd = bid & 7, li = bid >> 3;
            by = xcd + 8 * (li / per_y);
            rem = li % per_y;
        } else {
            by = bid / per_y;
            rem = bid % per_y;
        }
        bx = ntile - 1 - rem / nsplit;                       // longest (most keys visible) tiles first
        sp = rem % nsplit;
    }
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, hh = lane >> 5;
    const int rb = wave % RB, kw = wave / RB;
    const int rbph = RB / hpw;                               // row blocks per head inside the workgroup
    const int ngrp = G / hpw;                                // head groups per kv-head
    const int h = by / ngrp, hgrp = by % ngrp;
    const int g = h * G + hgrp * hpw + rb % hpw;             // query head of this wavefront
    const int row0 = 32 * (bx * rbph + rb / hpw);            // first query row of this wavefront
    const int wg_rows_end = min(L, 32 * (bx + 1) * rbph);
    const int n_end = t + wg_rows_end;                       // keys any row of the workgroup can see
    const int my_row = row0 + l32;
    const int my_lim = t + min(my_row, L - 1);               // last visible key of my row
    const int wave_end = (row0 < L) ? t + min(L, row0 + 32) : 0;

    const uint16_t* Kh = K + (size_t)h * cap * D;
    const uint16_t* Vh = V + (size_t)h * cap * D;

    // query fragments: B operand of S^T = K.Q^T, lane (row l32, half hh) holds Q[row][16s + 8hh .. +8)
    bf16x8 qf[D / 16];
    {
        const bool ok = my_row < L;
        const uint16_t* qp = q + ((size_t)(ok ? my_row : 0) * Hq + g) * D + 8 * hh;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            u32x4 v = *(const u32x4*)(qp + 16 * s);
            if (!ok) v = u32x4{0u, 0u, 0u, 0u};
            qf[s] = as_bf16x8(v);
        }
    }

    f32x16 o[D / 32];
#pragma unroll
    for (int b = 0; b < D / 32; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[b][i] = 0.f;
    float m_ref = -__builtin_inff(), m_use = 0.f, lsum = 0.f;

    // Tiles go from global memory straight into LDS (no register staging): every wavefront issues
    // NLD 1-KB loads for K and for V per tile; lane l of a load fills 16-byte slot l of a 4-row block.
    // The slot a lane fills is fixed by the hardware, the source chunk it loads is ours to choose, so
    // the bank swizzle is applied on the source side: slot p of row r holds chunk p ^ swz(r).
    //   K: swz(r) = r & 15        (16 rows read the same logical chunk -> 16 different slots)
    //   V: swz(r) = (r & 3) << 2  (4 rows read the same 64-byte window -> 4 different windows)
    // A tile may run past the last cached row: the cache buffers are padded and hold only finite
    // values, the logits of such rows are masked, and a finite V row times a zero weight adds nothing.
    uint32_t dma_k[C::NLD], dma_v[C::NLD];                   // element offsets inside a tile, loop-invariant
#pragma unroll
    for (int u = 0; u < C::NLD; ++u) {
        const int r = 4 * (wave * C::NLD + u) + (lane >> 4), p = lane & 15;
        dma_k[u] = (uint32_t)(r * D + ((p ^ (r & 15)) << 3));
        dma_v[u] = (uint32_t)(r * D + ((p ^ ((r & 3) << 2)) << 3));
    }
    typedef const __attribute__((address_space(1))) void* gptr_t;
    typedef __attribute__((address_space(3))) void* lptr_t;
    auto dma = [&](int kv0, int buf) {
        const uint16_t* kt = Kh + (size_t)kv0 * D;
        const uint16_t* vt = Vh + (size_t)kv0 * D;
        char* kd = smem + buf * C::KBYTES + (wave * C::NLD) * 1024;
        char* vd = smem + 2 * C::KBYTES + buf * C::VBYTES + (wave * C::NLD) * 1024;
#pragma unroll
        for (int u = 0; u < C::NLD; ++u) {
            __builtin_amdgcn_global_load_lds((gptr_t)(kt + dma_k[u]), (lptr_t)(kd + u * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((gptr_t)(vt + dma_v[u]), (lptr_t)(vd + u * 1024), 16, 0, 0);
        }
    };
    // LDS byte offsets of this lane's fragments inside buffer 0 (buffers are selected by immediates)
    int kaddr[D / 16];
#pragma unroll
    for (int s = 0; s < D / 16; ++s) kaddr[s] = (kw * C::SUB + l32) * 256 + (((2 * s + hh) ^ (l32 & 15)) << 4);
    // transpose read: lane l of a 16-lane block supplies the address of key row l/4, 4 columns at 4*(l%4)
    int vaddr[D / 32];
#pragma unroll
    for (int b = 0; b < D / 32; ++b)
        vaddr[b] = 2 * C::KBYTES + (kw * C::SUB + 4 * hh + ((lane & 15) >> 2)) * 256 + 64 * (b ^ ((lane >> 2) & 3)) +
                   32 * ((lane >> 4) & 1) + 8 * (lane & 3);

    const int ntiles_all = (n_end + C::TILE - 1) / C::TILE;
    const int tile_lo = (int)((long)ntiles_all * sp / nsplit), ntiles = (int)((long)ntiles_all * (sp + 1) / nsplit);
    if (tile_lo < ntiles) dma(tile_lo * C::TILE, tile_lo & 1);
    __builtin_amdgcn_s_waitcnt(0);                           // my loads have landed ...
    __syncthreads();                                         // ... and so have everyone else's
    auto body = [&](auto buf_tag, int tile) {
        constexpr int BUF = decltype(buf_tag)::value;
        const int kv0 = tile * C::TILE;
        // the other buffer was last read one iteration ago, before the barrier that ended it
        if (tile + 1 < ntiles) dma(kv0 + C::TILE, BUF ^ 1);
        const int sub0 = kv0 + kw * C::SUB;                  // first key of my slice of the tile
        if (sub0 < wave_end) {                               // else nothing visible for this wavefront
            // ---- S^T = K . Q^T -----------------------------------------------------------------
            f32x16 acc[KVB];
#pragma unroll
            for (int kb = 0; kb < KVB; ++kb) {
                bf16x8 kf[D / 16];
#pragma unroll
                for (int s = 0; s < D / 16; ++s)
                    kf[s] = as_bf16x8(*(const u32x4*)(smem + kaddr[s] + BUF * C::KBYTES + 32 * kb * 256));
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[kb][i] = 0.f;
#pragma unroll
                for (int s = 0; s < D / 16; ++s)
                    acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[s], acc[kb], 0, 0, 0);
            }
            // ---- causal mask on tiles that reach past the first row's limit --------------------
            if (sub0 + C::SUB - 1 > t + row0) {
#pragma unroll
                for (int kb = 0; kb < KVB; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int kv = sub0 + 32 * kb + 8 * (i / 4) + 4 * hh + (i % 4);
                        if (kv > my_lim) acc[kb][i] = -__builtin_inff();
                    }
            }
            // ---- online softmax, in-lane along the key axis, lazily moved reference ------------
            float mx = acc[0][0];
#pragma unroll
            for (int kb = 0; kb < KVB; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, acc[kb][i]);
            mx = xhalf_max(mx) * c;
            if (__any(mx > m_ref + RESCALE_TAU)) {
                const float m_new = fmaxf(m_ref, mx);
                const float mu = (m_new == -__builtin_inff()) ? 0.f : m_new;
                const float alpha = fast_exp2(m_ref - mu);   // m_ref = -inf gives 0
                m_ref = m_new;
                m_use = mu;
                lsum *= alpha;
#pragma unroll
                for (int b = 0; b < D / 32; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[b][i] *= alpha;
            }
            // ---- P (fp32 -> bf16 for the product) and O^T += V^T . P^T -------------------------
#pragma unroll
            for (int kb = 0; kb < KVB; ++kb) {
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) {
                    bf16x4 vlo[D / 32], vhi[D / 32];
#pragma unroll
                    for (int b = 0; b < D / 32; ++b) {
                        const char* vp = smem + vaddr[b] + BUF * C::VBYTES + (32 * kb + 16 * tt) * 256;
                        vlo[b] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)vp);
                        vhi[b] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(vp + 8 * 256));
                    }
                    bf16x8 pf;
#pragma unroll
                    for (int p = 0; p < 8; ++p) {
                        const float e = fast_exp2(__builtin_fmaf(acc[kb][8 * tt + p], c, -m_use));
                        lsum += e;
                        pf[p] = (__bf16)e;
                    }
#pragma unroll
                    for (int b = 0; b < D / 32; ++b) {
                        const bf16x8 vf = __builtin_shufflevector(vlo[b], vhi[b], 0, 1, 2, 3, 4, 5, 6, 7);
                        o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, o[b], 0, 0, 0);
                    }
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(0);                       // the next tile's loads of this wavefront have landed
        __syncthreads();
    };
    for (int tile = tile_lo; tile < ntiles; ++tile) {
        if (tile & 1) body(std::integral_constant<int, 1>{}, tile);
        else body(std::integral_constant<int, 0>{}, tile);
    }

    // ---- merge the key ways of a query block ---------------------------------------------------
    if (KW > 1) {
        float* mg = (float*)smem;
        if (kw > 0) {
            float* w = mg + (size_t)((kw - 1) * RB + rb) * 64 * (C::OREG + 2);
            w[lane] = m_ref;
            w[64 + lane] = lsum;
#pragma unroll
            for (int b = 0; b < D / 32; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) w[(2 + b * 16 + i) * 64 + lane] = o[b][i];
        }
        __syncthreads();
        if (kw == 0) {
            for (int k2 = 1; k2 < KW; ++k2) {
                const float* w = mg + (size_t)((k2 - 1) * RB + rb) * 64 * (C::OREG + 2);
                const float m2 = w[lane], l2 = w[64 + lane];
                const float mt = fmaxf(m_ref, m2);
                const float mu = (mt == -__builtin_inff()) ? 0.f : mt;
                const float a1 = fast_exp2(m_ref - mu), a2 = fast_exp2(m2 - mu);
                lsum = lsum * a1 + l2 * a2;
#pragma unroll
                for (int b = 0; b < D / 32; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[b][i] = o[b][i] * a1 + w[(2 + b * 16 + i) * 64 + lane] * a2;
                m_ref = mt;
            }
        }
    }
    if (kw != 0 || my_row >= L) return;

    // ---- normalise and store: lane (row l32, half hh) holds O[row][32b + 8(i/4) + 4hh + i%4] -----
    const float ltot = lsum + xhalf(lsum);
    if (nsplit > 1) {
        // un-normalised partial of this key split: [split][row][head][D] fp32, (m, l) beside it
        const size_t rowi = ((size_t)sp * L + my_row) * Hq + g;
        float* pp = part_o + rowi * D;
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                f32x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = o[b][4 * a + e];
                *(f32x4*)(pp + 32 * b + 8 * a + 4 * hh) = w;
            }
        if (hh == 0) {
            part_ml[rowi * 2] = m_ref;
            part_ml[rowi * 2 + 1] = ltot;
        }
        return;
    }
    const float inv = 1.0f / ltot;
    uint16_t* op = out + ((size_t)my_row * Hq + g) * D;
#pragma unroll
    for (int b = 0; b < D / 32; ++b)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            bf16x4 w;
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o[b][4 * a + e] * inv);
            *(bf16x4*)(op + 32 * b + 8 * a + 4 * hh) = w;
        }
    if (hh == 0) lse2[(size_t)g * max_chunk + my_row] = m_ref + __builtin_log2f(ltot);
}


template <int RB, int KW, int KVB>
hipError_t launch_dma_cfg(const Geometry& g, const CacheView& c, const void* q, int t, int L, void* out, float* lse,
                          const FwdScratch& sc, int nsplit, hipStream_t st)
{
    const int hpw = (RB % g.G == 0) ? g.G : ((g.G % RB == 0) ? RB : 1);
    const int rbph = RB / hpw;
    const int ntile = (L + 32 * rbph - 1) / (32 * rbph), ny = g.Hkv * (g.G / hpw);
    if (nsplit > 1 && (size_t)nsplit * L > sc.part_rows) nsplit = 1;     // no scratch: no split
    hipLaunchKernelGGL((attn_fwd_dma_kernel<RB, KW, KVB>), dim3(ntile * ny * nsplit), dim3(64 * RB * KW), 0, st,
                       (const uint16_t*)q, (const uint16_t*)c.K, (const uint16_t*)c.V, (uint16_t*)out, lse, t, L,
                       g.Hq, g.G, g.cap, g.max_chunk, hpw, ntile, ny, nsplit, sc.part_o, sc.part_ml,
                       g.scale * LOG2E);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || nsplit == 1) return e;
    return launch_attn_combine(g, sc, L, nsplit, out, lse, st);
}

}  // namespace

hipError_t launch_attn_fwd_dma(const Geometry& g, const CacheView& c, const void* q, int t, int L, void* out,
                               float* lse, const FwdScratch& sc, int variant, int nsplit, hipStream_t st)
{
    if (g.d != 128) return hipErrorInvalidValue;
    switch (variant) {
        case 1: return launch_dma_cfg<4, 2, 2>(g, c, q, t, L, out, lse, sc, nsplit, st);
        case 2: return launch_dma_cfg<4, 2, 1>(g, c, q, t, L, out, lse, sc, nsplit, st);
        case 3: return launch_dma_cfg<2, 2, 1>(g, c, q, t, L, out, lse, sc, nsplit, st);
        case 4: return launch_dma_cfg<4, 1, 2>(g, c, q, t, L, out, lse, sc, nsplit, st);
        default: return launch_dma_cfg<2, 4, 1>(g, c, q, t, L, out, lse, sc, nsplit, st);
    }
}

}  // namespace infmllm
