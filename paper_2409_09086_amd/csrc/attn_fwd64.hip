// Chunk attention (Sec. 3.2) on bf16 matrix cores, 64 query rows per wavefront, for head_dim 128.
//
// Same arithmetic as the 32-row kernel (S^T = K.Q^T with a lane owning a query row, bf16 P as
// the B operand of O^T += V^T.P^T, V read through the LDS transpose read, lazily moved softmax
// reference), but every wavefront carries two 32-row query blocks.  A K or V fragment read from
// LDS then feeds two MFMAs, which halves LDS traffic per MFMA, and the two blocks give the
// scheduler independent MFMA and VALU streams to overlap inside one wavefront (one wavefront
// per SIMD, up to 512 registers).
//
// Workgroup = RG row groups (64 rows each) x KW key ways (wavefronts that share a row group and
// split every key tile; merged through LDS).  When the grid would leave CUs idle the key range
// of a row tile is also cut into `nsplit` pieces handled by different workgroups; each writes an
// un-normalised partial (fp32 O, reference maximum, sum) and a small second kernel combines them
// -- a kernel boundary is the one ordering across XCDs that needs no cache maintenance.
#include <type_traits>

#include "launch.h"
#include "mfma_common.h"

namespace infmllm {

namespace {

template <int RG, int KW>
struct Cfg64 {
    static constexpr int D = 128;
    static constexpr int NW = RG * KW, NT = 64 * NW;
    static constexpr int SUB = 32, TILE = KW * SUB;    // keys per wavefront / per workgroup per tile
    static constexpr int KP = D * 2 + 16;              // K row pitch in LDS (bytes)
    static constexpr int VP = D * 2 + 64;              // V row pitch in LDS (bytes)
    static constexpr int CPR = D / 8;                  // 16-byte chunks per row
    static constexpr int NLD = TILE * CPR / NT;        // chunks per thread per tensor
    static constexpr int LD_RSTEP = NT / CPR;
    static constexpr int KBYTES = TILE * KP, VBYTES = TILE * VP, BUF = KBYTES + VBYTES;
    static constexpr int OREG = 2 * (D / 2);           // fp32 accumulators of O^T per lane (two blocks)
    static constexpr int MERGE = (KW - 1) * RG * 64 * (OREG + 4) * 4;
    static constexpr int LDS = (2 * BUF) > MERGE ? (2 * BUF) : MERGE;
    static_assert(TILE * CPR % NT == 0 && NT % CPR == 0, "tile must split evenly over the threads");
    static_assert(TILE <= CACHE_PAD_ROWS, "workspace padding assumes smaller tiles");
};

// One softmax step of a 32x32 block of logits held as S^T (lane = query row): returns the two
// bf16 B operands of the P.V product and updates the lane's reference maximum and sum.
struct RowState {
    float m_ref, m_use, lsum;
};

template <int RG, int KW>
__global__ void __launch_bounds__(64 * RG * KW)
attn_fwd64_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
                  uint16_t* __restrict__ out, float* __restrict__ lse2, int t, int L, int Hq, int G, int cap,
                  int max_chunk, int hpw, int ntile, int ny, int nsplit, float* __restrict__ part_o,
                  float* __restrict__ part_ml, float c /* scale * log2(e) */)
{
    using C = Cfg64<RG, KW>;
    constexpr int D = 128;
    __shared__ __attribute__((aligned(16))) char smem[C::LDS];

    // Workgroup -> (row tile, head group, key split); all workgroups of one kv-head get ids of one
    // residue class mod 8 so that they share an XCD's L2 copy of the head's K and V.
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
    const int rg = wave % RG, kw = wave / RG;
    const int rgph = RG / hpw;                               // row groups per head inside the workgroup
    const int ngrp = G / hpw;
    const int h = by / ngrp, hgrp = by % ngrp;
    const int g = h * G + hgrp * hpw + rg % hpw;             // query head of this wavefront
    const int row0 = 64 * (bx * rgph + rg / hpw);            // first query row of this wavefront
    const int wg_rows_end = min(L, 64 * (bx + 1) * rgph);
    const int n_end = t + wg_rows_end;                       // keys any row of the workgroup can see
    const int wave_end = (row0 < L) ? t + min(L, row0 + 64) : 0;
    int my_row[2], my_lim[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        my_row[qb] = row0 + 32 * qb + l32;
        my_lim[qb] = t + min(my_row[qb], L - 1);             // last visible key of my row
    }

    const uint16_t* Kh = K + (size_t)h * cap * D;
    const uint16_t* Vh = V + (size_t)h * cap * D;

    // query fragments: B operand of S^T = K.Q^T, lane (row l32, half hh) holds Q[row][16s + 8hh .. +8)
    bf16x8 qf[2][D / 16];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const bool ok = my_row[qb] < L;
        const uint16_t* qp = q + ((size_t)(ok ? my_row[qb] : 0) * Hq + g) * D + 8 * hh;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            u32x4 v = *(const u32x4*)(qp + 16 * s);
            if (!ok) v = u32x4{0u, 0u, 0u, 0u};
            qf[qb][s] = as_bf16x8(v);
        }
    }

    f32x16 o[2][D / 32];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[qb][b][i] = 0.f;
    RowState rs[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) { rs[qb].m_ref = -__builtin_inff(); rs[qb].m_use = 0.f; rs[qb].lsum = 0.f; }

    // Register staging of the next tile.  A tile may run past the last cached row: the cache
    // buffers are padded and hold only finite values, the logits of such rows are masked, and a
    // finite V row times a zero weight adds nothing.
    u32x4 stK[C::NLD], stV[C::NLD];
    uint32_t ld_off[C::NLD];
#pragma unroll
    for (int u = 0; u < C::NLD; ++u) ld_off[u] = (uint32_t)((tid / C::CPR + u * C::LD_RSTEP) * D + (tid % C::CPR) * 8);
    auto fetch = [&](int kv0) {
        const uint16_t* kt = Kh + (size_t)kv0 * D;
        const uint16_t* vt = Vh + (size_t)kv0 * D;
#pragma unroll
        for (int u = 0; u < C::NLD; ++u) {
            stK[u] = *(const u32x4*)(kt + ld_off[u]);
            stV[u] = *(const u32x4*)(vt + ld_off[u]);
        }
    };
    const int st_k = (tid / C::CPR) * C::KP + (tid % C::CPR) * 16;
    const int st_v = C::KBYTES + (tid / C::CPR) * C::VP + (tid % C::CPR) * 16;
    auto stash = [&](int buf) {
        char* base = smem + buf * C::BUF;
#pragma unroll
        for (int u = 0; u < C::NLD; ++u) {
            *(u32x4*)(base + st_k + u * C::LD_RSTEP * C::KP) = stK[u];
            *(u32x4*)(base + st_v + u * C::LD_RSTEP * C::VP) = stV[u];
        }
    };
    const int koff = (kw * C::SUB + l32) * C::KP + 16 * hh;
    // transpose read: lane l of a 16-lane block supplies the address of key row l/4, 4 columns at 4*(l%4)
    const int voff = C::KBYTES + (kw * C::SUB + 4 * hh + ((lane & 15) >> 2)) * C::VP +
                     (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;

    // One tile for this wavefront.  Written as one straight block (the only branch is the rare
    // rescale) so that the scheduler can overlap the VALU work of one query block with the MFMAs
    // of the other.  MASK adds the causal mask; tiles every row sees whole run without it.
    auto process = [&](auto mask_tag, const char* kbase, const char* vbase, int sub0) {
        constexpr bool MASK = decltype(mask_tag)::value;
        // ---- S^T = K . Q^T for both query blocks; one K fragment feeds two MFMAs ----------------
        bf16x8 kf[D / 16];
#pragma unroll
        for (int s = 0; s < D / 16; ++s) kf[s] = as_bf16x8(*(const u32x4*)(kbase + 32 * s));
        f32x16 acc[2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[qb][i] = 0.f;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int s = 0; s < D / 16; ++s)
                acc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[qb][s], acc[qb], 0, 0, 0);
        // V fragments of this slice: A operand of O^T += V^T . P^T, shared by both blocks
        bf16x8 vf[2][D / 32];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int b = 0; b < D / 32; ++b) {
                const char* vp = vbase + 16 * tt * C::VP + 64 * b;
                const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)vp);
                const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(vp + 8 * C::VP));
                vf[tt][b] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        float mx[2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            if (MASK) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int kv = sub0 + 8 * (i / 4) + 4 * hh + (i % 4);
                    acc[qb][i] = (kv > my_lim[qb]) ? -__builtin_inff() : acc[qb][i];
                }
            }
            float m = acc[qb][0];
#pragma unroll
            for (int i = 1; i < 16; ++i) m = fmaxf(m, acc[qb][i]);
            mx[qb] = xhalf_max(m) * c;
        }
        // lazily moved reference: rescale only rows whose maximum grew by more than 2^TAU
        if (__any(mx[0] > rs[0].m_ref + RESCALE_TAU || mx[1] > rs[1].m_ref + RESCALE_TAU)) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                const float m_new = (mx[qb] > rs[qb].m_ref + RESCALE_TAU) ? mx[qb] : rs[qb].m_ref;
                const float mu = (m_new == -__builtin_inff()) ? 0.f : m_new;
                const float alpha = fast_exp2(rs[qb].m_ref - mu);    // 1 for rows that keep their reference
                rs[qb].m_ref = m_new;
                rs[qb].m_use = mu;
                rs[qb].lsum *= alpha;
#pragma unroll
                for (int b = 0; b < D / 32; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[qb][b][i] *= alpha;
            }
        }
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                bf16x8 pf;
#pragma unroll
                for (int p = 0; p < 8; ++p) {
                    const float e = fast_exp2(__builtin_fmaf(acc[qb][8 * tt + p], c, -rs[qb].m_use));
                    rs[qb].lsum += e;
                    pf[p] = (__bf16)e;
                }
#pragma unroll
                for (int b = 0; b < D / 32; ++b)
                    o[qb][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[tt][b], pf, o[qb][b], 0, 0, 0);
            }
    };

    const int ntiles_all = (n_end + C::TILE - 1) / C::TILE;
    const int tile_lo = (int)((long)ntiles_all * sp / nsplit), tile_hi = (int)((long)ntiles_all * (sp + 1) / nsplit);
    // tiles below this index are seen whole by all 64 rows of this wavefront
    const int full_x = t + row0 + 1 - (kw + 1) * C::SUB;     // last key of my slice <= first row's limit
    const int full_end = (row0 < L && full_x >= 0) ? full_x / C::TILE + 1 : 0;
    if (tile_lo < tile_hi) {
        fetch(tile_lo * C::TILE);
        stash(tile_lo & 1);
        if (tile_lo + 1 < tile_hi) fetch((tile_lo + 1) * C::TILE);
    }
    __syncthreads();
    for (int tile = tile_lo; tile < tile_hi; ++tile) {
        const int kv0 = tile * C::TILE, buf = tile & 1;
        const char* const kbase = smem + buf * C::BUF + koff;
        const char* const vbase = smem + buf * C::BUF + voff;
        const int sub0 = kv0 + kw * C::SUB;                  // first key of my slice of the tile
        if (tile < full_end) process(std::false_type{}, kbase, vbase, sub0);
        else if (sub0 < wave_end) process(std::true_type{}, kbase, vbase, sub0);
        // the other buffer was last read one iteration ago, before the barrier that ended it
        if (tile + 1 < tile_hi) stash(buf ^ 1);
        if (tile + 2 < tile_hi) fetch(kv0 + 2 * C::TILE);
        __syncthreads();
    }

    // ---- merge the key ways of a row group through LDS -------------------------------------------
    if (KW > 1) {
        float* mg = (float*)smem;
        constexpr int UNIT = 64 * (C::OREG + 4);
        if (kw > 0) {
            float* w = mg + (size_t)((kw - 1) * RG + rg) * UNIT;
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                w[(2 * qb) * 64 + lane] = rs[qb].m_ref;
                w[(2 * qb + 1) * 64 + lane] = rs[qb].lsum;
#pragma unroll
                for (int b = 0; b < D / 32; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) w[(4 + (qb * (D / 32) + b) * 16 + i) * 64 + lane] = o[qb][b][i];
            }
        }
        __syncthreads();
        if (kw == 0) {
            for (int k2 = 1; k2 < KW; ++k2) {
                const float* w = mg + (size_t)((k2 - 1) * RG + rg) * UNIT;
#pragma unroll
                for (int qb = 0; qb < 2; ++qb) {
                    const float m2 = w[(2 * qb) * 64 + lane], l2 = w[(2 * qb + 1) * 64 + lane];
                    const float mt = fmaxf(rs[qb].m_ref, m2);
                    const float mu = (mt == -__builtin_inff()) ? 0.f : mt;
                    const float a1 = fast_exp2(rs[qb].m_ref - mu), a2 = fast_exp2(m2 - mu);
                    rs[qb].lsum = rs[qb].lsum * a1 + l2 * a2;
#pragma unroll
                    for (int b = 0; b < D / 32; ++b)
#pragma unroll
                        for (int i = 0; i < 16; ++i)
                            o[qb][b][i] = o[qb][b][i] * a1 + w[(4 + (qb * (D / 32) + b) * 16 + i) * 64 + lane] * a2;
                    rs[qb].m_ref = mt;
                }
            }
        }
    }
    if (kw != 0) return;

    // ---- store: lane (row l32, half hh) holds O[row][32b + 8(i/4) + 4hh + i%4] ---------------------
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        if (my_row[qb] >= L) continue;
        const float ltot = xhalf_sum(rs[qb].lsum);
        if (nsplit == 1) {
            const float inv = 1.0f / ltot;
            uint16_t* op = out + ((size_t)my_row[qb] * Hq + g) * D;
#pragma unroll
            for (int b = 0; b < D / 32; ++b)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    bf16x4 w;
#pragma unroll
                    for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o[qb][b][4 * a + e] * inv);
                    *(bf16x4*)(op + 32 * b + 8 * a + 4 * hh) = w;
                }
            if (hh == 0) lse2[(size_t)g * max_chunk + my_row[qb]] = rs[qb].m_ref + __builtin_log2f(ltot);
        } else {
            // un-normalised partial of this key split: [split][row][head][D] fp32, (m, l) beside it
            const size_t rowi = ((size_t)sp * L + my_row[qb]) * Hq + g;
            float* op = part_o + rowi * D;
#pragma unroll
            for (int b = 0; b < D / 32; ++b)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    f32x4 w;
#pragma unroll
                    for (int e = 0; e < 4; ++e) w[e] = o[qb][b][4 * a + e];
                    *(f32x4*)(op + 32 * b + 8 * a + 4 * hh) = w;
                }
            if (hh == 0) {
                part_ml[rowi * 2] = rs[qb].m_ref;
                part_ml[rowi * 2 + 1] = ltot;
            }
        }
    }
}

// out[row][head][:] = sum_s w_s O_s / sum_s w_s l_s with w_s = exp2(m_s - max m); lse2 = max m + log2(sum).
// One thread per 8 output columns.
__global__ void __launch_bounds__(256)
attn_combine_kernel(const float* __restrict__ part_o, const float* __restrict__ part_ml, uint16_t* __restrict__ out,
                    float* __restrict__ lse2, int L, int Hq, int max_chunk, int nsplit)
{
    constexpr int D = 128;
    const long total = (long)L * Hq * (D / 8);
    for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (long)gridDim.x * blockDim.x) {
        const int x = (int)(idx % (D / 8));
        const long rowi = idx / (D / 8);                      // row * Hq + head
        float mt = -__builtin_inff();
        for (int s = 0; s < nsplit; ++s) mt = fmaxf(mt, part_ml[((size_t)s * L * Hq + rowi) * 2]);
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, lt = 0.f;
        for (int s = 0; s < nsplit; ++s) {
            const size_t r = (size_t)s * L * Hq + rowi;
            const float w = fast_exp2(part_ml[r * 2] - mt);   // an empty split has m = -inf, weight 0
            lt += w * part_ml[r * 2 + 1];
            const f32x4 a = *(const f32x4*)(part_o + r * D + 8 * x), b = *(const f32x4*)(part_o + r * D + 8 * x + 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) { acc[e] += w * a[e]; acc[4 + e] += w * b[e]; }
        }
        const float inv = 1.0f / lt;
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (__bf16)(acc[e] * inv);
        *(bf16x8*)(out + rowi * D + 8 * x) = o;
        if (x == 0) {
            const int row = (int)(rowi / Hq), g = (int)(rowi % Hq);
            lse2[(size_t)g * max_chunk + row] = mt + __builtin_log2f(lt);
        }
    }
}

template <int RG, int KW>
hipError_t launch64(const Geometry& g, const CacheView& c, const void* q, int t, int L, void* out, float* lse,
                    const FwdScratch& sc, int want_split, hipStream_t st)
{
    const int hpw = (RG % g.G == 0) ? g.G : ((g.G % RG == 0) ? RG : 1);
    const int rgph = RG / hpw;
    const int ntile = (L + 64 * rgph - 1) / (64 * rgph), ny = g.Hkv * (g.G / hpw);
    int nsplit = want_split;
    if (nsplit > 1 && (size_t)nsplit * L > sc.part_rows) nsplit = 1;     // scratch too small: no split
    hipLaunchKernelGGL((attn_fwd64_kernel<RG, KW>), dim3(ntile * ny * nsplit), dim3(64 * RG * KW), 0, st,
                       (const uint16_t*)q, (const uint16_t*)c.K, (const uint16_t*)c.V, (uint16_t*)out, lse, t, L,
                       g.Hq, g.G, g.cap, g.max_chunk, hpw, ntile, ny, nsplit, sc.part_o, sc.part_ml,
                       g.scale * LOG2E);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || nsplit == 1) return e;
    return launch_attn_combine(g, sc, L, nsplit, out, lse, st);
}

}  // namespace

hipError_t launch_attn_combine(const Geometry& g, const FwdScratch& sc, int L, int nsplit, void* out, float* lse,
                               hipStream_t st)
{
    const long total = (long)L * g.Hq * 16;
    int blocks = (int)((total + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(attn_combine_kernel, dim3(blocks), dim3(256), 0, st, sc.part_o, sc.part_ml, (uint16_t*)out,
                       lse, L, g.Hq, g.max_chunk, nsplit);
    return hipGetLastError();
}

hipError_t launch_attn_fwd64(const Geometry& g, const CacheView& c, const void* q, int t, int L, void* out,
                             float* lse, const FwdScratch& sc, int variant, int nsplit, hipStream_t st)
{
    if (g.d != 128) return hipErrorInvalidValue;
    switch (variant) {
        case 1: return launch64<4, 1>(g, c, q, t, L, out, lse, sc, nsplit, st);
        case 2: return launch64<1, 4>(g, c, q, t, L, out, lse, sc, nsplit, st);
        default: return launch64<2, 2>(g, c, q, t, L, out, lse, sc, nsplit, st);
    }
}

}  // namespace infmllm
