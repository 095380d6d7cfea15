// Chunk attention (Sec. 3.2) on bf16 MFMA for gfx950, head_dim 128: the variant for long key ranges.
//
// attn_fwd (attn_mfma.hip) gives a wavefront 32 query rows, so every K or V fragment it reads from LDS
// feeds one MFMA: 1 KB of LDS traffic per 32 cycles of matrix work per SIMD, which is all the LDS of a CU
// delivers.  Here a wavefront carries two 32-row query blocks A and B, a fragment feeds two MFMAs, and the
// matrix pipe is the busiest unit instead of the LDS.  The price is registers: two blocks' output
// accumulators, query fragments and logits need more than half of a SIMD's register file, so a SIMD holds
// ONE wavefront (four per workgroup, 256 query rows), and whatever that wavefront issues is all the SIMD
// does: one instruction per four cycles whatever its kind.  The loop is therefore a software pipeline over
// 32-key sub-blocks, written so that independent work of three sub-blocks sits side by side in one
// instruction stream:
//
//   period m :  MFMA   O += V(m-1)^T P(m-1)^T         (16 MFMAs, both blocks)
//               MFMA   S(m+1)^T = K(m+1) Q^T          (16 MFMAs, both blocks)
//               VALU   softmax of S(m) -> P(m)        (row maximum, exp2, row sum, bf16)
//               LDS    K fragments of sub-block m+2, V fragments of sub-block m
//               VMEM   staging of the tile three ahead
//
// K/V tiles of 64 keys rotate through four LDS buffers: the tile two ahead of the one being multiplied is
// written while the fourth buffer is still being read by wavefronts that lag, so one barrier per tile is
// enough.  A wavefront computes S^T = K.Q^T so that a lane owns a query row (row statistics in-lane, the
// bf16 weights already laid out as the B operand of O^T += V^T.P^T); V is read with the LDS transpose read.
// The softmax reference moves only when a row maximum outgrows it by 2^8; that rare step is taken on a side
// path between the period's two scheduling regions.
#include <type_traits>

#include "launch.h"
#include "mfma_common.h"

namespace infmllm {

namespace {

namespace w64 {
constexpr int D = 128;
constexpr int TILE = 64, NBUF = 4, NT = 256;
constexpr int KP = D * 2 + 16;                     // K row pitch in LDS (bytes): 16 rows -> 64 distinct banks
constexpr int VP = D * 2 + 64;                     // V row pitch: 4 rows x 64 B windows tile the banks
constexpr int KBYTES = TILE * KP, VBYTES = TILE * VP, BUF = KBYTES + VBYTES, LDS = NBUF * BUF;
constexpr int CPR = D / 8;                         // 16-byte pieces per row
constexpr int NLD = TILE * CPR / NT;               // pieces per thread per tensor per tile
constexpr int LD_RSTEP = NT / CPR;                 // rows between a thread's consecutive pieces
static_assert(LDS <= 160 * 1024, "four tiles must fit the LDS of a CU");
static_assert(TILE <= CACHE_PAD_ROWS, "workspace padding assumes smaller tiles");
}  // namespace w64

template <bool B> using Flag = std::integral_constant<bool, B>;

__global__ void __launch_bounds__(w64::NT) __attribute__((amdgpu_waves_per_eu(1, 1)))
attn_fwd64_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
                  const uint16_t* __restrict__ kc, const uint16_t* __restrict__ vc, int tc,
                  uint16_t* __restrict__ out, float* __restrict__ lse2, int t, int L, int Hq, int G, int cap,
                  int max_chunk, int hpw, int ntile, int ny, float c /* scale * log2(e) */)
{
    using namespace w64;
    __shared__ __attribute__((aligned(16))) char smem[LDS];

    // Workgroup -> (row tile, head group); all row tiles of a kv-head on one XCD (ids of one residue class mod 8).
    int bx, by;
    {
        const int bid = blockIdx.x;
        int rem;
        if ((ny & 7) == 0) {
            const int xcd = bid & 7, li = bid >> 3;
            by = xcd + 8 * (li / ntile);
            rem = li % ntile;
        } else {
            by = bid / ntile;
            rem = bid % ntile;
        }
        bx = ntile - 1 - rem;                                // longest (most keys visible) tiles first
    }
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wph = 4 / hpw;                                 // wavefronts (64-row blocks) per head in the workgroup
    const int ngrp = G / hpw;
    const int h = by / ngrp, hgrp = by % ngrp;
    const int g = h * G + hgrp * hpw + wave % hpw;           // query head of this wavefront
    const int row0 = 64 * (bx * wph + wave / hpw);           // first query row of this wavefront
    const int wg_rows_end = min(L, 64 * (bx + 1) * wph);
    const int n_end = t + wg_rows_end;                       // keys any row of the workgroup can see
    const int Hkv = Hq / G, n = t + L;
    int my_row[2], my_lim[2];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        my_row[x] = row0 + 32 * x + l32;
        my_lim[x] = t + min(my_row[x], L - 1);               // last visible key of my row
    }
    const uint16_t* Kh = K + (size_t)h * cap * D;
    const uint16_t* Vh = V + (size_t)h * cap * D;

    // query fragments: B operand of S^T = K.Q^T, lane (row l32, half hh) holds Q[row][16s + 8hh .. +8)
    bf16x8 qf[2][D / 16];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        const bool ok = my_row[x] < L;
        const uint16_t* qp = q + ((size_t)(ok ? my_row[x] : 0) * Hq + g) * D + 8 * hh;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            u32x4 v = *(const u32x4*)(qp + 16 * s);
            if (!ok) v = u32x4{0u, 0u, 0u, 0u};
            qf[x][s] = as_bf16x8(v);
        }
    }

    f32x16 o[2][D / 32];                                     // O^T accumulators of the two blocks
    f32x16 S[2];                                             // logits of the sub-block in its softmax stage, per block
    bf16x8 pf[2][2][2];                                      // weights: [sub-block parity][block][16-key step]
    bf16x8 kf[D / 16];                                       // K fragments of one sub-block: [head-dim step]
    bf16x8 vf[2][D / 32];                                    // V fragments of one sub-block: [16-key step][column block]
    float m_ref[2], m_use[2], lsum[2];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[x][b][i] = 0.f;
        m_ref[x] = -__builtin_inff(); m_use[x] = 0.f; lsum[x] = 0.f;
    }

    // ---- staging: global -> registers -> LDS, one 64-key tile at a time ----------------------------
    // A tile may run past the last key: rows past n are read from row n-1, their logits are masked.
    u32x4 stK[NLD], stV[NLD];
    const int srow = tid / CPR, scol8 = (tid % CPR) * 8;
    auto fetch = [&](int kv0) {
        if (kv0 + TILE <= tc) {
            const uint16_t* kt = Kh + (size_t)kv0 * D;       // uniform base + per-lane 32-bit offset
            const uint16_t* vt = Vh + (size_t)kv0 * D;
#pragma unroll
            for (int u = 0; u < NLD; ++u) {
                const uint32_t off = (uint32_t)((srow + u * LD_RSTEP) * D + scol8);
                stK[u] = *(const u32x4*)(kt + off);
                stV[u] = *(const u32x4*)(vt + off);
            }
        } else if (kv0 >= tc && kv0 + TILE <= n) {
            const uint16_t* kt = kc + ((size_t)(kv0 - tc) * Hkv + h) * D;
            const uint16_t* vt = vc + ((size_t)(kv0 - tc) * Hkv + h) * D;
#pragma unroll
            for (int u = 0; u < NLD; ++u) {
                const uint32_t off = (uint32_t)((srow + u * LD_RSTEP) * Hkv * D + scol8);
                stK[u] = *(const u32x4*)(kt + off);
                stV[u] = *(const u32x4*)(vt + off);
            }
        } else {
#pragma unroll
            for (int u = 0; u < NLD; ++u) {
                const int kv = min(kv0 + srow + u * LD_RSTEP, n - 1);
                const bool cached = kv < tc;
                const size_t off = cached ? ((size_t)h * cap + kv) * D + scol8 : ((size_t)(kv - tc) * Hkv + h) * D + scol8;
                stK[u] = *(const u32x4*)((cached ? K : kc) + off);
                stV[u] = *(const u32x4*)((cached ? V : vc) + off);
            }
        }
    };
    const int st_k = srow * KP + scol8 * 2, st_v = KBYTES + srow * VP + scol8 * 2;
    auto stash = [&](int tile) {
        char* base = smem + (tile & (NBUF - 1)) * BUF;
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            *(u32x4*)(base + st_k + u * LD_RSTEP * KP) = stK[u];
            *(u32x4*)(base + st_v + u * LD_RSTEP * VP) = stV[u];
        }
    };

    // ---- fragment reads -----------------------------------------------------------------------------
    const int koff = l32 * KP + 16 * hh;
    // transpose read: lane l of a 16-lane block supplies the address of key row l/4, 4 columns at 4*(l%4)
    const int voff = KBYTES + (4 * hh + ((lane & 15) >> 2)) * VP + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
    auto read_k = [&](int m) {                               // K fragments of sub-block m
        const char* kb = smem + ((m >> 1) & (NBUF - 1)) * BUF + (m & 1) * 32 * KP + koff;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) kf[s] = as_bf16x8(*(const u32x4*)(kb + 32 * s));
    };
    auto read_v = [&](int m) {                               // V fragments of sub-block m
        const char* vb = smem + ((m >> 1) & (NBUF - 1)) * BUF + (m & 1) * 32 * VP + voff;
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int b = 0; b < D / 32; ++b) {
                const char* vp = vb + 16 * tt * VP + 64 * b;
                const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)vp);
                const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(vp + 8 * VP));
                vf[tt][b] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
    };

    // ---- the pieces of a period ----------------------------------------------------------------------
    auto qk = [&]() {                                        // S = K . Q^T from kf, block A's chain then block B's
#pragma unroll
        for (int x = 0; x < 2; ++x) {
#pragma unroll
            for (int i = 0; i < 16; ++i) S[x][i] = 0.f;
#pragma unroll
            for (int s = 0; s < D / 16; ++s)
                S[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[x][s], S[x], 0, 0, 0);
        }
    };
    auto pv = [&](auto par, int tt0, int tt1) {              // O += V^T . P^T with P = pf[par], 16-key steps tt0 .. tt1-1
        constexpr int P = decltype(par)::value;
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            if (tt < tt0 || tt >= tt1) continue;
#pragma unroll
            for (int b = 0; b < D / 32; ++b)
#pragma unroll
                for (int x = 0; x < 2; ++x)
                    o[x][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[tt][b], pf[P][x][tt], o[x][b], 0, 0, 0);
        }
    };
    // mask (on tiles that reach past a row's limit) and scaled row maximum of S[x]
    auto row_max = [&](auto mask, int x, int sub0) -> float {
        if (decltype(mask)::value) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int kv = sub0 + 8 * (i / 4) + 4 * hh + (i % 4);
                if (kv > my_lim[x]) S[x][i] = -__builtin_inff();
            }
        }
        float mx = S[x][0];
#pragma unroll
        for (int i = 1; i < 16; ++i) mx = fmaxf(mx, S[x][i]);
        return xhalf_max(mx) * c;
    };
    auto rescale = [&](int x, float mx) {                    // rare: the reference of block x moves
        if (__any(mx > m_ref[x] + RESCALE_TAU)) {
            const float m_new = fmaxf(m_ref[x], mx);
            const float mu = (m_new == -__builtin_inff()) ? 0.f : m_new;
            const float alpha = fast_exp2(m_ref[x] - mu);    // m_ref = -inf gives 0
            m_ref[x] = m_new;
            m_use[x] = mu;
            lsum[x] *= alpha;
#pragma unroll
            for (int b = 0; b < D / 32; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[x][b][i] *= alpha;
        }
    };
    auto weights = [&](auto par, int x) {                    // P = exp2(S c - m), its row sum, bf16 copies
        constexpr int P = decltype(par)::value;
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const float e = fast_exp2(__builtin_fmaf(S[x][8 * tt + p], c, -m_use[x]));
                if (p & 1) s1 += e; else s0 += e;
                pf[P][x][tt][p] = (__bf16)e;
            }
        lsum[x] += s0 + s1;
    };

    const int ntiles = (n_end + TILE - 1) / TILE;
    const int nsub = 2 * ntiles;                             // sub-blocks 0 .. nsub-1
    const int first_masked = (t + min(row0, L - 1) + 1) / 32;  // sub-blocks from here on reach past some row's limit

    // One period: sub-block m is in its softmax stage (its logits are in S), sub-block m-1 in its O += V^T P^T
    // stage (PVF: it exists), sub-block m+1 in its S = K Q^T stage (QK: it exists).  PAR = parity of m.
    auto period = [&](int m, auto par, auto has_qk, auto has_pv, auto mask) {
        constexpr int P = decltype(par)::value;
        constexpr bool QK = decltype(has_qk)::value, PVF = decltype(has_pv)::value;
        if (QK) read_k(m + 1);                               // kf was consumed by the previous period's S = K Q^T
        // first products of sub-block m-1 on the matrix pipe while the row maxima of sub-block m are formed
        if (PVF) pv(Flag<P == 0>{}, 0, 1);
        const float mx0 = row_max(mask, 0, 32 * m), mx1 = row_max(mask, 1, 32 * m);
        if (__any(mx0 > m_ref[0] + RESCALE_TAU || mx1 > m_ref[1] + RESCALE_TAU)) {
            // rare: O has to hold all of sub-block m-1 before it is rescaled
            if (PVF) pv(Flag<P == 0>{}, 1, 2);
            rescale(0, mx0);
            rescale(1, mx1);
            weights(par, 0);
            weights(par, 1);
        } else {
            if (PVF) pv(Flag<P == 0>{}, 1, 2);
            weights(par, 0);
            weights(par, 1);
        }
        // logits of sub-block m+1 on the matrix pipe; the V fragments for the next period and the staging beside them
        if (QK) qk();
        read_v(m);
    };

    // ---- prologue: tiles 0 and 1 in LDS, tile 2 in the staging registers, S(0) formed -----------------
    fetch(0);
    stash(0);
    if (1 < ntiles) { fetch(TILE); stash(1); }
    if (2 < ntiles) fetch(2 * TILE);
    __syncthreads();
    read_k(0);
    qk();

    // ---- main loop: one tile (two periods) per iteration ----------------------------------------------
    for (int j = 0; j < ntiles; ++j) {
        const int m = 2 * j;
        const bool masked = m + 1 >= first_masked;
        if (j == 0) {
            if (masked) { period(m, Flag<false>{}, Flag<true>{}, Flag<false>{}, Flag<true>{}); }
            else { period(m, Flag<false>{}, Flag<true>{}, Flag<false>{}, Flag<false>{}); }
        } else {
            if (masked) { period(m, Flag<false>{}, Flag<true>{}, Flag<true>{}, Flag<true>{}); }
            else { period(m, Flag<false>{}, Flag<true>{}, Flag<true>{}, Flag<false>{}); }
        }
        if (j + 2 < ntiles) stash(j + 2);                    // loaded one iteration ago; its buffer was last read two barriers ago
        if (j + 3 < ntiles) fetch((j + 3) * TILE);
        if (j + 1 < ntiles) {
            if (masked) { period(m + 1, Flag<true>{}, Flag<true>{}, Flag<true>{}, Flag<true>{}); }
            else { period(m + 1, Flag<true>{}, Flag<true>{}, Flag<true>{}, Flag<false>{}); }
        } else {
            period(m + 1, Flag<true>{}, Flag<false>{}, Flag<true>{}, Flag<true>{});
        }
        __syncthreads();
    }
    pv(Flag<true>{}, 0, 2);                                  // the last sub-block (odd) still owes its O += V^T P^T

    // ---- normalise and store: lane (row l32, half hh) holds O[row][32b + 8(i/4) + 4hh + i%4] in o[x][b][i] ----
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        if (my_row[x] >= L) continue;
        const float ltot = lsum[x] + xhalf(lsum[x]);
        const float inv = 1.0f / ltot;
        uint16_t* op = out + ((size_t)my_row[x] * Hq + g) * D;
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                bf16x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o[x][b][4 * q4 + e] * inv);
                *(bf16x4*)(op + 32 * b + 8 * q4 + 4 * hh) = w;
            }
        if (hh == 0) lse2[(size_t)g * max_chunk + my_row[x]] = m_ref[x] + __builtin_log2f(ltot);
    }
}

}  // namespace

hipError_t launch_attn_mfma64(const Geometry& g, const CacheView& c, const KeySource& ks, const void* q, int t, int L,
                              void* out, float* lse, hipStream_t st)
{
    if (g.d != 128) return hipErrorInvalidValue;
    const int hpw = (g.G % 4 == 0) ? 4 : ((g.G % 2 == 0) ? 2 : 1);   // heads of a group that share a workgroup's K/V tiles
    const int wph = 4 / hpw;
    const int ntile = (L + 64 * wph - 1) / (64 * wph), ny = g.Hkv * (g.G / hpw);
    hipLaunchKernelGGL(attn_fwd64_kernel, dim3(ntile * ny), dim3(w64::NT), 0, st, (const uint16_t*)q, (const uint16_t*)c.K,
                       (const uint16_t*)c.V, (const uint16_t*)ks.k, (const uint16_t*)ks.v, ks.rows, (uint16_t*)out, lse, t, L,
                       g.Hq, g.G, g.cap, g.max_chunk, hpw, ntile, ny, (float)(g.scale * (double)LOG2E));
    return hipGetLastError();
}

}  // namespace infmllm
