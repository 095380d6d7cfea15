// bf16 matrix-core kernels for gfx950: chunk attention (Sec. 3.2) and the column score with
// the attention bias (Alg. 1 l.1-4).
//
// Why two kernels.  S[j] = mean_i p_ij needs the exact softmax weight p_ij = exp(s_ij - lse_i),
// and lse_i is known only once row i has met every key; a column partial taken under a running
// maximum cannot be repaired afterwards because the correction is per row.  The probability
// matrix may not go to HBM, so the scored block's logits are formed twice:
//
//   attn_fwd   : row-stationary flash attention.  Computes S^T = K.Q^T on 32x32x16 bf16 MFMA so
//                that a lane owns one query row: row maxima and sums are in-lane (one exchange
//                between the two half-waves per tile), and the bf16 weights are already laid
//                out as the B operand of O^T += V^T.P^T.  V stays row-major in LDS and is read
//                through the LDS transpose read, which hands each lane four consecutive keys of
//                one head-dim column.  Writes out and the row log-sum-exp (base 2).
//   score      : column-stationary.  A wavefront keeps its 64 key rows in registers as B
//                operands, streams the scored query rows through LDS, forms S = Q.K^T so that a
//                lane owns one key column, and adds exp2(s - lse) into per-register partial sums.
//                A column's sum is finished inside one wavefront, so W' does not depend on any
//                cross-workgroup reduction order.
//
// fp32 is kept from the MFMA accumulators to the score: the bf16 rounding of P is applied only
// to the copy that feeds the P.V product.
#include "launch.h"
#include "mfma_common.h"

namespace infmllm {

namespace {

constexpr int FWD_MAX_TILE = CACHE_PAD_ROWS;     // a key tile may run this far past the last cached row

// ---------------------------------------------------------------------------------------------
// attn_fwd
//   D    head_dim (64 | 128)
//   RB   32-row query blocks per workgroup (one wavefront each)
//   KW   key ways: wavefronts that share a query block and split every key tile between them
//   KVB  32-key blocks a wavefront handles per tile
// A workgroup of RB*KW wavefronts loads tiles of KW*KVB*32 cache rows into LDS.
// ---------------------------------------------------------------------------------------------
template <int D, int RB, int KW, int KVB>
struct FwdCfg {
    static constexpr int NW = RB * KW, NT = 64 * NW;
    static constexpr int SUB = KVB * 32, TILE = KW * SUB;
    static constexpr int KP = D * 2 + 16;              // K row pitch in LDS (bytes): 16 rows -> 64 distinct banks
    static constexpr int VP = D * 2 + 64;              // V row pitch: 4 rows x 64 B windows tile the banks
    static constexpr int CPR = D / 8;                  // 16-byte chunks per row
    static constexpr int NLD = TILE * CPR / NT;        // chunks per thread per tensor
    static constexpr int LD_RSTEP = NT / CPR;          // rows between a thread's consecutive chunks
    static constexpr int KBYTES = TILE * KP, VBYTES = TILE * VP, BUF = KBYTES + VBYTES;
    static constexpr int NBUF = (2 * BUF <= 160 * 1024) ? 2 : 1;
    static constexpr int OREG = D / 2;                 // fp32 accumulators of O^T per lane
    static constexpr int MERGE = (KW > 1 ? KW : 0) * RB * 64 * (OREG + 2) * 4;
    static constexpr int LDS = (NBUF * BUF) > MERGE ? (NBUF * BUF) : MERGE;
    static_assert(TILE * CPR % NT == 0 && NT % CPR == 0, "tile must split evenly over the threads");
    static_assert(TILE <= FWD_MAX_TILE, "workspace padding assumes smaller tiles");
};

// Tail of the attention kernel: merge the key ways of a query block through LDS, then normalise and
// store.  Every wavefront leaves its (m, l, O) in
// LDS; the KW wavefronts of a query block then each merge and store their own D / KW output columns,
// so the tail's LDS reads, arithmetic and stores are spread over the whole workgroup.
// Lane (row l32, half hh) holds O[row][32b + 8(i/4) + 4hh + i%4] in o[b][i].
template <int D, int RB, int KW>
__device__ __forceinline__ void fwd_finish(char* smem, bool sync_first, f32x16 (&o)[D / 32], float m_ref, float lsum,
                                           int rb, int kw, int lane, int hh, int my_row, int g, int L, int Hq,
                                           int max_chunk, uint16_t* __restrict__ out, float* __restrict__ lse2)
{
    constexpr int OREG = D / 2, NB = D / 32;
    static_assert(NB % KW == 0, "the output column blocks must split evenly over the key ways");
    constexpr int BPW = NB / KW;                              // column blocks stored by one wavefront
    float a[KW];
    const float* slot[KW];
    if (KW > 1) {
        if (sync_first) __syncthreads();
        float* mg = (float*)smem;
        float* w = mg + (size_t)(kw * RB + rb) * 64 * (OREG + 2);
        w[lane] = m_ref;
        w[64 + lane] = lsum;
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) w[(2 + b * 16 + i) * 64 + lane] = o[b][i];
        __syncthreads();
        if (my_row >= L) return;
        float mk[KW], mt = -__builtin_inff();
#pragma unroll
        for (int k = 0; k < KW; ++k) {
            slot[k] = mg + (size_t)(k * RB + rb) * 64 * (OREG + 2);
            mk[k] = slot[k][lane];
            mt = fmaxf(mt, mk[k]);
        }
        const float mu = (mt == -__builtin_inff()) ? 0.f : mt;
        lsum = 0.f;
#pragma unroll
        for (int k = 0; k < KW; ++k) {
            a[k] = fast_exp2(mk[k] - mu);                     // a way that saw no key has m = -inf, weight 0
            lsum += slot[k][64 + lane] * a[k];
        }
        m_ref = mt;
    } else {
        if (my_row >= L) return;
    }
    const float ltot = lsum + xhalf(lsum);
    const float inv = 1.0f / ltot;
    uint16_t* op = out + ((size_t)my_row * Hq + g) * D;
#pragma unroll
    for (int bb = 0; bb < BPW; ++bb) {
        const int b = kw * BPW + bb;
        float v[16];
        if (KW > 1) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float t = 0.f;
#pragma unroll
                for (int k = 0; k < KW; ++k) t += a[k] * slot[k][(2 + b * 16 + i) * 64 + lane];
                v[i] = t;
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) v[i] = o[bb][i];
        }
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            bf16x4 w;
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = (__bf16)(v[4 * q4 + e] * inv);
            *(bf16x4*)(op + 32 * b + 8 * q4 + 4 * hh) = w;
        }
    }
    if (kw == 0 && hh == 0) lse2[(size_t)g * max_chunk + my_row] = m_ref + __builtin_log2f(ltot);
}

template <int D, int RB, int KW, int KVB>
__global__ void __launch_bounds__(64 * RB * KW)
attn_fwd_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
                const uint16_t* __restrict__ kc, const uint16_t* __restrict__ vc, int tc,
                uint16_t* __restrict__ out, float* __restrict__ lse2, int t, int L, int Hq, int G, int cap,
                int max_chunk, int hpw, int ntile, int ny, float c /* scale * log2(e) */)
{
    using C = FwdCfg<D, RB, KW, KVB>;
    __shared__ __attribute__((aligned(16))) char smem[C::LDS];

    // Workgroup -> (row tile, head group).  Consecutive workgroup ids go round-robin over the 8
    // XCDs; all row tiles of one kv-head are given ids of one residue class so that they share
    // that XCD's L2 copy of the head's K and V.
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
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: branches on it are scalar
    const bool stage_first = C::NW == 8 && wave >= 4;        // wavefronts w and w + 4 share a SIMD
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

    // Register staging of the next tile.  A tile may run past the last cached row: the cache
    // buffers are padded by FWD_MAX_TILE rows and hold only finite values, the logits of such
    // rows are masked, and a finite V row times a zero weight adds nothing.
    u32x4 stK[C::NLD], stV[C::NLD];
    uint32_t ld_off[C::NLD];                                 // element offsets inside a tile, loop-invariant
#pragma unroll
    for (int u = 0; u < C::NLD; ++u) ld_off[u] = (uint32_t)((tid / C::CPR + u * C::LD_RSTEP) * D + (tid % C::CPR) * 8);
    // Rows below tc come from the cache; rows from tc on are the chunk's own keys, read in place
    // from the token-major chunk tensors (row stride Hkv*D), so that an evicting step needs no
    // separate append pass.
    const int Hkv = Hq / G;
    const int n = t + L;
    auto fetch = [&](int kv0) {
        if (kv0 + C::TILE <= tc) {
            const uint16_t* kt = Kh + (size_t)kv0 * D;       // uniform: scalar base + per-lane 32-bit offset
            const uint16_t* vt = Vh + (size_t)kv0 * D;
#pragma unroll
            for (int u = 0; u < C::NLD; ++u) {
                stK[u] = *(const u32x4*)(kt + ld_off[u]);
                stV[u] = *(const u32x4*)(vt + ld_off[u]);
            }
        } else if (kv0 >= tc && kv0 + C::TILE <= n) {
            // the whole tile lies inside the chunk: same scheme with the chunk's row stride
            const uint16_t* kt = kc + ((size_t)(kv0 - tc) * Hkv + h) * D;
            const uint16_t* vt = vc + ((size_t)(kv0 - tc) * Hkv + h) * D;
#pragma unroll
            for (int u = 0; u < C::NLD; ++u) {
                const uint32_t off = (uint32_t)((tid / C::CPR + u * C::LD_RSTEP) * Hkv * D + (tid % C::CPR) * 8);
                stK[u] = *(const u32x4*)(kt + off);
                stV[u] = *(const u32x4*)(vt + off);
            }
        } else {
            // a tile that straddles the cache/chunk boundary or runs past the last key
            const int col8 = (tid % C::CPR) * 8;
#pragma unroll
            for (int u = 0; u < C::NLD; ++u) {
                const int kv = min(kv0 + tid / C::CPR + u * C::LD_RSTEP, n - 1);   // rows past n are masked anyway
                const bool cached = kv < tc;
                const size_t off = cached ? ((size_t)h * cap + kv) * D + col8 : ((size_t)(kv - tc) * Hkv + h) * D + col8;
                stK[u] = *(const u32x4*)((cached ? K : kc) + off);
                stV[u] = *(const u32x4*)((cached ? V : vc) + off);
            }
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

    // byte offsets of this lane's fragments inside a buffer
    const int koff = (kw * C::SUB + l32) * C::KP + 16 * hh;
    // transpose read: lane l of a 16-lane block supplies the address of key row l/4, 4 columns at 4*(l%4)
    const int voff = C::KBYTES + (kw * C::SUB + 4 * hh + ((lane & 15) >> 2)) * C::VP +
                     (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;

    const int ntiles = (n_end + C::TILE - 1) / C::TILE;
    constexpr int tile_lo = 0;
    if (tile_lo < ntiles) fetch(tile_lo * C::TILE);
    if (C::NBUF == 2) {
        if (tile_lo < ntiles) stash(tile_lo & 1);
        if (tile_lo + 1 < ntiles) fetch((tile_lo + 1) * C::TILE);
        __syncthreads();
    }
    for (int tile = tile_lo; tile < ntiles; ++tile) {
        const int kv0 = tile * C::TILE;
        const int buf = (C::NBUF == 2) ? (tile & 1) : 0;
        if (C::NBUF == 1) {
            __syncthreads();                                 // everyone is done with the previous tile
            stash(0);
            __syncthreads();
            if (tile + 1 < ntiles) fetch(kv0 + C::TILE);
        }
        const char* const kbase = smem + buf * C::BUF + koff;
        const char* const vbase = smem + buf * C::BUF + voff;
        // The other buffer was last read one iteration ago, before the barrier that ended it, so the next
        // tile may be staged at any point of this iteration.  The second wavefront of every SIMD does it
        // first and the first one last: the two then reach their MFMA and VALU phases at different times
        // instead of queueing for the same pipe.
        if (C::NBUF == 2 && stage_first) {
            if (tile + 1 < ntiles) stash(buf ^ 1);
            if (tile + 2 < ntiles) fetch(kv0 + 2 * C::TILE);
        }

        const int sub0 = kv0 + kw * C::SUB;                  // first key of my slice of the tile
        if (sub0 < wave_end) {                               // else nothing visible for this wavefront
            // ---- S^T = K . Q^T -----------------------------------------------------------------
            f32x16 acc[KVB];
#pragma unroll
            for (int kb = 0; kb < KVB; ++kb) {
                bf16x8 kf[D / 16];
#pragma unroll
                for (int s = 0; s < D / 16; ++s) kf[s] = as_bf16x8(*(const u32x4*)(kbase + 32 * kb * C::KP + 32 * s));
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[kb][i] = 0.f;
#pragma unroll
                for (int s = 0; s < D / 16; ++s)
                    acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[s], acc[kb], 0, 0, 0);
                // all K fragments of the block are requested before the first MFMA waits for one
                __builtin_amdgcn_sched_group_barrier(0x100, D / 16, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, D / 16, 0);
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
                        const char* vp = vbase + (32 * kb + 16 * tt) * C::VP + 64 * b;
                        vlo[b] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)vp);
                        vhi[b] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(vp + 8 * C::VP));
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
        if (C::NBUF == 2) {
            if (!stage_first) {
                if (tile + 1 < ntiles) stash(buf ^ 1);
                if (tile + 2 < ntiles) fetch(kv0 + 2 * C::TILE);
            }
            __syncthreads();
        }
    }

    fwd_finish<D, RB, KW>(smem, C::NBUF == 1, o, m_ref, lsum, rb, kw, lane, hh, my_row, g, L, Hq, max_chunk, out, lse2);
}

// ---------------------------------------------------------------------------------------------
// score: W'[h][j] = (1/(G lq)) sum_{g in group h} sum_{i = L-lq}^{L-1} exp2(c q_i.k_j - lse2_i)
//                   - (cnd-1-j) b / cnd
// A column is a physical cache row (col < tc; its stream-order index j is rank[col]) or a chunk row
// (col >= tc, j = col).  Columns 0 .. ncol-1 are swept, ncol = max(tc, cnd): any cached row may be a
// candidate; W' is written at index j, for the columns with j < cnd.
// Workgroup = 8 wavefronts = 8 column groups of 32*CB key columns each, held in registers as MFMA
// operands; every wavefront takes all four 32-row query blocks of an iteration, which are staged once
// per workgroup (double-buffered in LDS) and so serve 256*CB columns.  Every scored row sees every
// candidate column, so there is no mask inside the block.
// ---------------------------------------------------------------------------------------------
template <int D, int CB>
__global__ void __launch_bounds__(512)
score_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ kc, int tc,
             const float* __restrict__ lse2, const float* __restrict__ carry, const int32_t* __restrict__ rank,
             float* __restrict__ Wb, int L, int lq, int Hq, int Hkv, int G, int cap, int max_chunk, int cnd, int ncol,
             int nxb, float c, float dstep /* b / c, Alg. 1 l.2 */, int rsplit, float* __restrict__ spart)
{
    constexpr int QP = D * 2 + 16;                            // pitch of a staged query row
    constexpr int CPR = D / 8;
    constexpr int TROWS = 128;                                // rows staged per iteration: four 32-row blocks
    constexpr int NLD = TROWS * CPR / 512;                    // 16-byte chunks per thread per iteration
    constexpr int QBYTES = TROWS * QP;
    constexpr int BUF = QBYTES + TROWS * 4;                   // rows + their log-sum-exp
    constexpr int LSE_ROWS = 4096;                            // scored rows whose log-sum-exp is kept in LDS
    __shared__ __attribute__((aligned(16))) char smem[2 * BUF];
    __shared__ float s_lse[LSE_ROWS];
    __shared__ int s_ticket;

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: what depends on it stays scalar
    const int cg = wave;                                      // column group
    // all column blocks of a kv-head get workgroup ids of one residue class mod 8, i.e. one XCD,
    // so that the head's scored queries are fetched into one L2 only
    // With rsplit > 1 the scored rows of a column block are shared out over rsplit workgroups (slice rs).
    int h, bx, rs;
    {
        const int bid = blockIdx.x, per_head = nxb * rsplit;
        int rem;
        if ((Hkv & 7) == 0) {
            const int xcd = bid & 7, li = bid >> 3;
            h = xcd + 8 * (li / per_head);
            rem = li % per_head;
        } else {
            h = bid / per_head;
            rem = bid % per_head;
        }
        bx = rem % nxb;
        rs = rem / nxb;
    }
    const int col0 = bx * (256 * CB) + cg * (32 * CB);

    f32x16 part[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) part[cb][i] = 0.f;

    const int nblk = (lq + 31) / 32;                          // 32-row blocks per query head
    const int total = G * nblk;                               // blocks to sweep, four per iteration
    const int niter_all = (total + 3) / 4;
    const int it_first = (int)((long)rs * niter_all / rsplit);               // this workgroup's iterations
    const int niter = (int)((long)(rs + 1) * niter_all / rsplit) - it_first;
    // Row log-sum-exp of every scored row of the group, once per workgroup: row (gg, i) -> s_lse[gg*lq + i].
    auto row_lse = [&](int g, int i) -> float { return lse2[(size_t)g * max_chunk + i]; };
    const bool lse_in_lds = G * lq <= LSE_ROWS;
    // every load is issued before the first value is stored, together with those of the first query blocks
    // and of the key tile below: the prologue then waits for memory once, not once per group of 512 rows
    float lse_in[LSE_ROWS / 512];
    if (lse_in_lds) {
#pragma unroll
        for (int u = 0; u < LSE_ROWS / 512; ++u) {
            const int x = tid + u * 512;
            lse_in[u] = x < G * lq ? row_lse(h * G + x / lq, L - lq + x % lq) : 0.f;
        }
    }

    // Staging of the next four blocks.  Chunk u of a thread is row rr of block slot u * RPU / 32 + sbase (the
    // slot is uniform over a wavefront), so the block's address is scalar and only toff is per lane.  The
    // loads are unconditional: a chunk past the last scored row, or of a block past the last one, is read
    // from the nearest valid row instead and zeroed on its way to LDS, which keeps branches out of the loop.
    u32x4 st[NLD];
    bool st_ok[NLD];
    float stl = 0.f;                                          // log-sum-exp of the staged row, or ...
    int stl_idx = -1;                                         // ... its index in s_lse (looked up when it is staged)
    constexpr int RPU = 512 / CPR;                            // rows between a thread's consecutive chunks: 32 or 64
    const int sbase = RPU > 32 ? (wave >> 2) : 0;
    const int rr = (tid / CPR) & 31;
    const uint32_t tcol = (uint32_t)((tid % CPR) * 8);
    const uint32_t rowlen = (uint32_t)(Hq * D);
    const uint32_t toff = (uint32_t)rr * rowlen + tcol;
    // (head in group, block in head) of the next block
    int fg = nblk > 0 ? (4 * it_first) / nblk : 0, fb = nblk > 0 ? (4 * it_first) % nblk : 0;
    // direct: take the rows' log-sum-exp from memory (before s_lse is complete)
    auto fetch = [&](bool direct = false) {
        int gk[4], bk[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {                         // past the last block: fg >= G
            gk[k] = fg; bk[k] = fb;
            const bool wrap = fb + 1 >= nblk;
            fb = wrap ? 0 : fb + 1;
            fg += wrap ? 1 : 0;
        }
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            constexpr int KS = RPU > 32 ? 2 : 1;              // slots between a thread's consecutive chunks
            const int g1 = sbase ? gk[(KS * u + 1) & 3] : gk[KS * u], b1 = sbase ? bk[(KS * u + 1) & 3] : bk[KS * u];
            const int i0 = L - lq + 32 * b1;                  // < L for every block in range
            const int gc = g1 < G ? g1 : G - 1;
            const uint16_t* base = q + ((size_t)i0 * Hq + h * G + gc) * D;
            const uint32_t lim = (uint32_t)(L - 1 - i0) * rowlen + tcol;   // this thread's columns in the last row
            st[u] = *(const u32x4*)(base + (toff < lim ? toff : lim));
            st_ok[u] = g1 < G && toff <= lim;                 // applied when the chunk is written to LDS
        }
        if (tid < TROWS) {
            const int k = tid >> 5;                           // block slot of the row whose lse this thread stages
            const int g1 = k == 0 ? gk[0] : k == 1 ? gk[1] : k == 2 ? gk[2] : gk[3];
            const int b1 = k == 0 ? bk[0] : k == 1 ? bk[1] : k == 2 ? bk[2] : bk[3];
            const int i = L - lq + 32 * b1 + (tid & 31);
            stl = __builtin_inff();                           // +inf: weight 0
            stl_idx = -1;
            if (g1 < G && i < L) {
                if (lse_in_lds && !direct) stl_idx = g1 * lq + (i - (L - lq));
                else stl = row_lse(h * G + g1, i);
            }
        }
    };
    auto stash = [&](int buf) {
        char* base = smem + buf * BUF;
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            const int ch = tid + u * 512;
            *(u32x4*)(base + (ch / CPR) * QP + (ch % CPR) * 16) = st_ok[u] ? st[u] : u32x4{0u, 0u, 0u, 0u};
        }
        if (tid < TROWS) *(float*)(base + QBYTES + tid * 4) = (stl_idx >= 0) ? s_lse[stl_idx] : stl;
    };
    if (niter > 0) fetch(true);
    // Key fragments: B operand of S = Q.K^T, lane (column l32, half hh) holds K[col][16s + 8hh .. +8), loaded in
    // that layout straight from memory (a wavefront's load touches 32 rows, 32 bytes of each; the four loads
    // that share a row's 128-byte line follow one another).  A column past the last one is all zeros.
    bf16x8 kf[CB][D / 16];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
        const int col = col0 + 32 * cb + l32;
        const bool ok = col < ncol;
        const int cc = ok ? col : 0;
        const uint16_t* kp = (cc < tc ? K + ((size_t)h * cap + cc) * D : kc + ((size_t)(cc - tc) * Hkv + h) * D) + 8 * hh;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            u32x4 v = *(const u32x4*)(kp + 16 * s);
            if (!ok) v = u32x4{0u, 0u, 0u, 0u};
            kf[cb][s] = as_bf16x8(v);
        }
    }
    if (lse_in_lds) {
#pragma unroll
        for (int u = 0; u < LSE_ROWS / 512; ++u) {
            const int x = tid + u * 512;
            if (x < G * lq) s_lse[x] = lse_in[u];
        }
    }
    if (niter > 0) {
        stash(0);
        if (niter > 1) fetch(true);
    }
    __syncthreads();                                          // first query blocks and s_lse are complete
    // Software pipeline over units of one 32-row block x one 32-column block (8 MFMAs at head_dim 128): while
    // the MFMAs of a unit are issued, the 16 logits of the unit before (in the other accumulator) are weighed,
    // two per MFMA slot: exp2(s c - lse) added to the column sums.  The slots are fenced so that the compiler
    // keeps them as written; the wavefront then always has vector work beside its MFMAs, and the two wavefronts
    // of a SIMD fill each other's gaps.  The query fragments of a block serve its CB units; each is replaced
    // by the next block's right after its last MFMA, eight slots before it is needed again.  The last unit of an
    // iteration is weighed beside the first of the next one (the log-sum-exps of its rows are in registers
    // before the barrier lets the buffer be rewritten), the very last one after the loop.
    constexpr int NS = D / 16;                                // MFMAs per unit
    static_assert(16 % NS == 0, "the logits of a unit are spread evenly over the slots of the next");
    constexpr int LPS = 16 / NS;                              // logits weighed per slot
    f32x16 accA, accB;
    f32x4 ls[4];                                              // log-sum-exps of the rows of the unit being weighed
    bf16x8 qf[NS];
    auto read_q = [&](const char* base, int k, int s) -> bf16x8 {
        return as_bf16x8(*(const u32x4*)(base + (32 * k + l32) * QP + 16 * hh + 32 * s));
    };
    // lane (column, half hh) holds rows 8a + 4hh + e of a block in register 4a + e
    auto load_ls = [&](const char* base, int k) {
        const float* lp = (const float*)(base + QBYTES) + 32 * k;
#pragma unroll
        for (int a = 0; a < 4; ++a) ls[a] = *(const f32x4*)(lp + 8 * a + 4 * hh);
    };
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // unit (block k, column block CBI): MFMAs into `cur`, the logits of the unit before out of `prev` into the
    // column sums of column block PCB
    auto unit = [&](const char* base, auto K_, auto CBI_, f32x16& cur, const f32x16& prev) {
        constexpr int k = decltype(K_)::value, cbi = decltype(CBI_)::value;
        constexpr int pcb = (cbi + CB - 1) % CB;              // column block of the unit before
        static_for<0, NS>([&](auto I) {
            constexpr int sidx = decltype(I)::value;
            cur = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[sidx], kf[cbi][sidx], sidx == 0 ? zero16 : cur, 0, 0, 0);
            if constexpr (cbi == CB - 1 && k < 3) qf[sidx] = read_q(base, k + 1, sidx);
#pragma unroll
            for (int x = 0; x < LPS; ++x) {
                const int i = LPS * sidx + x;
                part[pcb][i] += fast_exp2(__builtin_fmaf(prev[i], c, -ls[i / 4][i % 4]));
                // the sums are not read before the end of the kernel: without a use here the compiler moves the
                // weighing out of the slot, past the MFMAs that were to hide it
                asm volatile("" : "+v"(part[pcb][i]));
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        // the unit that follows weighs this one: from its last column block on, a block's rows are the next to be weighed
        if constexpr (cbi == 0) load_ls(base, k);
    };
    // before the first unit there is nothing to weigh: log-sum-exps of +inf give weights of zero
    accB = zero16;
#pragma unroll
    for (int a = 0; a < 4; ++a) ls[a] = f32x4{__builtin_inff(), __builtin_inff(), __builtin_inff(), __builtin_inff()};
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;
    for (int it = 0; it < niter; ++it) {
        const char* base = smem + (it & 1) * BUF;
#pragma unroll
        for (int sidx = 0; sidx < NS; ++sidx) qf[sidx] = read_q(base, 0, sidx);
        if constexpr (CB == 2) {
            unit(base, I0{}, I0{}, accA, accB);               // beside it: the last unit of the iteration before
            unit(base, I0{}, I1{}, accB, accA);
            unit(base, I1{}, I0{}, accA, accB);
            unit(base, I1{}, I1{}, accB, accA);
            unit(base, I2{}, I0{}, accA, accB);
            unit(base, I2{}, I1{}, accB, accA);
            unit(base, I3{}, I0{}, accA, accB);
            unit(base, I3{}, I1{}, accB, accA);
        } else {
            unit(base, I0{}, I0{}, accA, accB);
            unit(base, I1{}, I0{}, accB, accA);
            unit(base, I2{}, I0{}, accA, accB);
            unit(base, I3{}, I0{}, accB, accA);
        }
        // the other buffer was last read one iteration ago, before the barrier that ended it
        if (it + 1 < niter) stash((it + 1) & 1);
        if (it + 2 < niter) fetch();
        __syncthreads();
    }
    if (niter > 0) {                                          // the last unit: block 3, column block CB - 1
#pragma unroll
        for (int i = 0; i < 16; ++i) part[CB - 1][i] += fast_exp2(__builtin_fmaf(accB[i], c, -ls[i / 4][i % 4]));
    }
    // column sums: 16 registers, then the two half-waves (fixed order)
    float sum[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
        float s0 = 0.f;
#pragma unroll
        for (int a = 0; a < 4; ++a) s0 += (part[cb][4 * a] + part[cb][4 * a + 1]) + (part[cb][4 * a + 2] + part[cb][4 * a + 3]);
        sum[cb] = s0 + xhalf(s0);
    }
    // Row-split launch: every workgroup puts its raw column sums where the other slices' workgroups can read
    // them (agent-scope stores go through to memory), waits until they have left, and takes a ticket; the one
    // that arrives last adds the slices up and finishes the columns.  No workgroup waits for another one.
    float* my_part = nullptr;
    if (rsplit > 1) {
        my_part = spart + ((size_t)(h * rsplit + rs) * nxb + bx) * (256 * CB);
        if (hh == 0) {
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
                __hip_atomic_store(my_part + cg * 32 * CB + 32 * cb + l32, sum[cb], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        int* arrived = (int*)(spart + (size_t)SCORE_SPLIT_WGS * 256) + h * nxb + bx;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) s_ticket = __hip_atomic_fetch_add(arrived, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (s_ticket != rsplit - 1) return;
        if (tid == 0) __hip_atomic_store(arrived, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next launch
    }
    if (hh == 0) {
        const float norm = (lq > 0) ? 1.0f / (float)(G * lq) : 0.f;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            const int col = col0 + 32 * cb + l32;
            const int j = col < tc ? (col < ncol ? rank[(size_t)h * cap + col] : cnd) : col;   // stream-order index
            if (j < cnd) {
                float tot = sum[cb];
                if (rsplit > 1) {
                    // fixed order over the slices, whichever workgroup does the adding
                    tot = 0.f;
                    for (int sp = 0; sp < rsplit; ++sp)
                        tot += __hip_atomic_load(my_part + (sp - rs) * nxb * (256 * CB) + cg * 32 * CB + 32 * cb + l32,
                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                float w = tot * norm - (float)(cnd - 1 - j) * dstep;                       // Alg. 1 l.1, l.3-4
                if (carry) {
                    // cumulative policy: this step's S on top of what the row has gathered, no bias; the
                    // chunk's own rows (read in place, col >= tc) and rows never ranked (+inf) carry nothing
                    const float a = col < tc ? carry[(size_t)h * cap + col] : 0.f;
                    w = tot * norm + (a < __builtin_inff() ? a : 0.f);
                }
                Wb[(size_t)h * cap + j] = w;
            }
        }
    }
}

}  // namespace

template <int D, int RB, int KW, int KVB>
hipError_t launch_fwd_cfg(const Geometry& g, const CacheView& c, const KeySource& ks, const void* q, int t, int L,
                          void* out, float* lse, hipStream_t st)
{
    const int hpw = (RB % g.G == 0) ? g.G : ((g.G % RB == 0) ? RB : 1);
    const int rbph = RB / hpw;
    const int ntile = (L + 32 * rbph - 1) / (32 * rbph), ny = g.Hkv * (g.G / hpw);
    const dim3 grid(ntile * ny), block(64 * RB * KW);
    hipLaunchKernelGGL((attn_fwd_kernel<D, RB, KW, KVB>), grid, block, 0, st, (const uint16_t*)q, (const uint16_t*)c.K, (const uint16_t*)c.V,
                       (const uint16_t*)ks.k, (const uint16_t*)ks.v, ks.rows, (uint16_t*)out, lse, t, L, g.Hq, g.G,
                       g.cap, g.max_chunk, hpw, ntile, ny, (float)(g.scale * (double)LOG2E));
    return hipGetLastError();
}

hipError_t launch_attn_mfma(const Geometry& g, const CacheView& c, const KeySource& ks, const void* q, int t, int L,
                            void* out, float* lse, hipStream_t st)
{
    if (g.d == 64) return launch_fwd_cfg<64, 4, 1, 2>(g, c, ks, q, t, L, out, lse, st);
    if (g.d != 128) return hipErrorInvalidValue;
    // 128 query rows x 64 keys per wavefront-tile is the efficient shape; when that grid would cover
    // only about half of the chip (128 workgroups at 32 heads x 512 rows), 64-row workgroups with four
    // key ways inside the workgroup are faster.  g.attn_tile > 0 (a test hook) forces one shape.
    const int wgs128 = g.Hq * ((L + 31) / 32) / 4;
    // attn_fwd64 (attn_mfma64.hip: 64 query rows per wavefront, one wavefront per SIMD) is the faster kernel
    // where its grid of 256-row workgroups covers the chip and the key range is long enough to fill its pipeline.
    // Its workgroups occupy a CU each: the grid must fill at least 80 % of the rounds over the 256 CUs it takes.
    const int wgs64 = (g.Hq * ((L + 63) / 64) + 3) / 4;
    const int rounds64 = (wgs64 + 255) / 256;
    const bool fills = wgs64 * 5 >= rounds64 * 256 * 4;
    const int v = g.attn_tile > 0 ? g.attn_tile : (fills && t + L >= 1024 ? 5 : (wgs128 >= 140 ? 1 : 2));
    switch (v) {
        case 5: return launch_attn_mfma64(g, c, ks, q, t, L, out, lse, st);
        case 1: return launch_fwd_cfg<128, 4, 2, 2>(g, c, ks, q, t, L, out, lse, st);
        case 2: return launch_fwd_cfg<128, 2, 4, 1>(g, c, ks, q, t, L, out, lse, st);
        case 3: return launch_fwd_cfg<128, 4, 2, 1>(g, c, ks, q, t, L, out, lse, st);
        default: return launch_fwd_cfg<128, 4, 1, 2>(g, c, ks, q, t, L, out, lse, st);
    }
}

hipError_t launch_score_mfma(const Geometry& g, const CacheView& c, const KeySource& ks, const void* q,
                             const float* lse, const FwdScratch& sc, int t, int L, float* Wb, hipStream_t st)
{
    const int n = t + L, cnd = n - g.R, lq = g.R < L ? g.R : L;
    if (cnd <= 0) return hipSuccess;
    const int ncol = ks.rows > cnd ? ks.rows : cnd;          // every cached row, and the chunk rows below cnd
    const float cc = (float)(g.scale * (double)LOG2E);
    // 512 columns per workgroup (256 at head_dim 64, where the wider variant runs out of registers).  Where
    // that leaves CUs without one, the scored rows of a column block are shared out over up to four workgroups
    // (whose sums the last to finish adds up); where there are too few rows for that, a workgroup takes 256 columns.
    const int wcols = g.d == 128 ? 512 : 256;
    const int nxw = (ncol + wcols - 1) / wcols;
    const long wgsw = (long)nxw * g.Hkv;
    const int niter = (g.G * ((lq + 31) / 32) + 3) / 4;       // iterations of the kernel's row loop
    const long wgs256 = (long)((ncol + 255) / 256) * g.Hkv;
    int rsplit = 1;
    if (wgsw < 200 && wgs256 < 200) {
        rsplit = (int)(256 / wgsw);
        if (rsplit > 4) rsplit = 4;
        if (rsplit > niter / 2) rsplit = niter / 2;
        if (rsplit < 1 || !sc.score_part || wgsw * rsplit * (wcols / 256) > SCORE_SPLIT_WGS) rsplit = 1;
    }
    const bool wide = wgsw >= 200 || rsplit > 1;
    const int nxb = wide ? nxw : (ncol + 255) / 256;
    const dim3 grid(nxb * g.Hkv * rsplit), block(512);
#define INFMLLM_SCORE(DD, CB)                                                                              \
    hipLaunchKernelGGL((score_kernel<DD, CB>), grid, block, 0, st, (const uint16_t*)q, (const uint16_t*)c.K, \
                       (const uint16_t*)ks.k, ks.rows, lse,                                                  \
                       g.policy == POLICY_CUMULATIVE ? c.score : nullptr, c.rank, Wb, L, lq, g.Hq, g.Hkv, g.G, g.cap, \
                       g.max_chunk,                                                                          \
                       cnd, ncol, nxb, cc, (float)(g.bias / (double)cnd), rsplit, sc.score_part)
    if (g.d == 128 && wide) INFMLLM_SCORE(128, 2);
    else if (g.d == 128) INFMLLM_SCORE(128, 1);
    else if (g.d == 64) INFMLLM_SCORE(64, 1);
    else return hipErrorInvalidValue;
#undef INFMLLM_SCORE
    return hipGetLastError();
}

}  // namespace infmllm
