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
//
// Under the causal mask the chunk's later rows see more keys.  A wavefront's two blocks are therefore one from
// the front and one from the back of the head's rows, which gives every wavefront the same number of (row, key)
// pairs; when block A has seen its last key the loop continues with a 16-slot period for block B alone.
#include <type_traits>

#include "launch.h"
#include "mfma_common.h"

namespace infmllm {

namespace {

namespace w64 {
constexpr int D = 128;
constexpr int TILE = 64, NBUF = 4, NT = 256;
constexpr int ROWB = D * 2;                        // bytes of a K or V row; LDS rows are not padded (see the swizzles)
constexpr int TBYTES = TILE * ROWB;                // one tile of K or of V: 16 KB
constexpr int KREG = 0, VREG = NBUF * TBYTES;      // LDS regions: the K tiles, then the V tiles
constexpr int DUMP = 2 * NBUF * TBYTES;            // 1 KB per wavefront that loads nobody needs are sent to
constexpr int LDS = DUMP + 4 * 1024;
static_assert(LDS <= 160 * 1024, "the tiles must fit the LDS of a CU");
static_assert(NBUF * TBYTES <= 65536, "a region must be addressable with a 16-bit instruction offset");
static_assert(TILE <= CACHE_PAD_ROWS, "workspace padding assumes smaller tiles");
}  // namespace w64

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;

// LDS fragment reads as assembly: the tiles are written by loads that go from memory straight into LDS, and
// the compiler, which cannot tell one LDS buffer from another, would wait for every such load in flight
// before each LDS read it knows of.  These reads are therefore hidden from it and waited for by hand
// (lds_wait), which also pins them where they are written, ahead of the products they feed.
template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_b128(uint32_t addr)
{
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <int OFF>
__device__ __forceinline__ bf16x4 lds_read_tr16_b64(uint32_t addr)
{
    bf16x4 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
// waits for every LDS read issued so far; the registers are named so that their consumers stay behind the wait
__device__ __forceinline__ void lds_wait(bf16x8 (&f)[8])
{
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7]));
}

// Two weights into one register of bf16, as a statement the compiler leaves in the slot it is written in
// (it would gather the conversions of a period into one burst with no MFMA beside it).
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    uint32_t v;
    asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(v) : "v"(lo), "v"(hi));
    return v;
}

// S^T += K Q^T with the result in ordinary vector registers.  A kernel that needs more than 256 registers
// gets every MFMA the compiler selects with its result in accumulation registers, which the vector unit
// cannot read: each logit would cost a copy.  The logits' products are therefore written out; the compiler
// does not see them, so what it would check is checked here: consecutive products of a chain are at least
// two other instructions apart, and the logits are first read a quarter of a period after the last one.
__device__ __forceinline__ void mfma_qk_first(f32x16& S, bf16x8 k, bf16x8 q)
{
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(S) : "v"(k), "a"(q));
}
__device__ __forceinline__ void mfma_qk(f32x16& S, bf16x8 k, bf16x8 q)
{
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(S) : "v"(k), "a"(q));
}

__device__ __forceinline__ uint32_t pack_bf16_after_nop(float lo, float hi)   // with the idle cycle that rule asks for
{
    uint32_t v;
    asm volatile("s_nop 0\n\tv_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(v) : "v"(lo), "v"(hi));
    return v;
}

template <bool B> using Flag = std::integral_constant<bool, B>;

__global__ void __launch_bounds__(w64::NT) __attribute__((amdgpu_waves_per_eu(1, 1)))
attn_fwd64_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
                  const uint16_t* __restrict__ kc, const uint16_t* __restrict__ vc, int tc,
                  uint16_t* __restrict__ out, float* __restrict__ lse2, int t, int L, int Hq, int G, int cap,
                  int max_chunk, int hpw, int ntile, int ny, float c /* scale * log2(e) */)
{
    using namespace w64;
    __shared__ __attribute__((aligned(1024))) char smem[LDS];

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
    // The two 32-row blocks of a wavefront are block p from the front and block p from the back of the head's rows
    // (p = the wavefront's index among the head's wavefronts): under the causal mask a row sees t + row + 1 keys,
    // so every wavefront gets the same number of (row, key) pairs, where two neighbouring blocks would give the last
    // wavefront a quarter more keys than the first and make the launch as long as that one.  Block A is finished
    // first; the loop then goes on with block B alone (period1).
    const int npair = ntile * wph;                           // wavefronts per head, over all workgroups
    const int pair0 = bx * wph;                              // the workgroup's first pair
    const int blkA = pair0 + wave / hpw, blkB = 2 * npair - 1 - blkA;
    const int rowsB_end = min(L, 32 * (2 * npair - pair0));  // end of the workgroup's last block B (its first wavefront's)
    const int n_end = t + rowsB_end;                         // keys any row of the workgroup can see
    const int Hkv = Hq / G, n = t + L;
    int my_row[2], my_lim[2];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        my_row[x] = 32 * (x == 0 ? blkA : blkB) + l32;
        my_lim[x] = t + min(my_row[x], L - 1);               // last visible key of my row
    }
    const uint16_t* Kh = K + (size_t)h * cap * D;
    const uint16_t* Vh = V + (size_t)h * cap * D;
    const uint16_t* kch = kc + (size_t)h * D;                // chunk rows of this kv-head: row stride Hkv * D
    const uint16_t* vch = vc + (size_t)h * D;

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
            // the fragments live in accumulation registers, which the MFMA reads directly: as ordinary vector
            // registers they would be parked there anyway and copied back before every use
            asm volatile("" : "+a"(qf[x][s]));
        }
    }

    f32x16 o[2][D / 32];                                     // O^T accumulators of the two blocks
    f32x16 S[2];                                             // logits of the sub-block in its softmax stage, per block
    u32x4 pf[2][2];                                          // weights of one sub-block, bf16 pairs: [block][16-key step]
    bf16x8 kf[D / 16];                                       // K fragments of one sub-block: [head-dim step]
    bf16x8 vf[2 * (D / 32)];                                 // V fragments of one sub-block: [16-key step * 4 + column block]
    float m_ref[2], m_use[2], lsum[2];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[x][b][i] = 0.f;
        m_ref[x] = -__builtin_inff(); m_use[x] = 0.f; lsum[x] = 0.f;
    }

    // ---- tiles: memory -> LDS without passing through registers ---------------------------------------
    // One load instruction moves 16 bytes per lane into 1 KB of consecutive LDS: four rows of a tile.  LDS
    // rows are not padded, so the 16-byte pieces of a row are permuted instead, by choosing which piece of
    // its row a lane fetches: piece c of K row r lies in slot c ^ (r & 15) (the 16 rows that a quarter of a
    // fragment read touches hit 16 different slots), piece c of V row r in slot c ^ 2 (r & 7) (the four rows
    // of a transpose read lie 32 bytes apart, the pair of pieces it takes from a row stays together).
    // Wavefront w issues loads 4k + w (k = 0..3) of a tile: LDS rows 16k + 4w + lane/16.
    const int drow = 4 * wave + (lane >> 4);                 // LDS row of this lane in the wavefront's first load
    const int pieceK = (lane & 15) ^ (drow & 15), pieceV = (lane & 15) ^ (2 * (drow & 7));
    auto issue_tile = [&](int tile, int slot) {              // keys of `tile` into the buffer of tile number `slot`
        const int kv0 = tile * TILE;
        const int buf = slot & (NBUF - 1);
        const bool in_cache = kv0 + TILE <= tc, in_chunk = kv0 >= tc && kv0 + TILE <= n;
        if (in_cache || in_chunk) {
            // the whole tile lies in the cache or in the chunk tensors: uniform base and row stride
            const int rs = in_cache ? D : Hkv * D;
            const uint16_t* kt = in_cache ? Kh + (size_t)kv0 * D : kch + (size_t)(kv0 - tc) * rs;
            const uint16_t* vt = in_cache ? Vh + (size_t)kv0 * D : vch + (size_t)(kv0 - tc) * rs;
            const uint32_t offk = (uint32_t)(drow * rs + pieceK * 8), offv = (uint32_t)(drow * rs + pieceV * 8);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                lds_void* dk = (lds_void*)(smem + KREG + buf * TBYTES + (4 * k) * 1024 + wave * 1024);
                lds_void* dv = (lds_void*)(smem + VREG + buf * TBYTES + (4 * k) * 1024 + wave * 1024);
                __builtin_amdgcn_global_load_lds((global_void*)(kt + (offk + (uint32_t)(16 * k * rs))), dk, 16, 0, 0);
                __builtin_amdgcn_global_load_lds((global_void*)(vt + (offv + (uint32_t)(16 * k * rs))), dv, 16, 0, 0);
            }
        } else {
            // a tile that straddles the cache/chunk boundary or runs past the last key (rows past n: row n-1, masked)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int kv = min(kv0 + 16 * k + drow, n - 1);
                const bool cached = kv < tc;
                const size_t offa = (size_t)kv * D, offb = (size_t)(kv - tc) * Hkv * D;
                const uint16_t* const ka = Kh + offa;
                const uint16_t* const kb = kch + offb;
                const uint16_t* const va = Vh + offa;
                const uint16_t* const vb = vch + offb;
                const uint16_t* const ksrc = cached ? ka : kb;
                const uint16_t* const vsrc = cached ? va : vb;
                lds_void* dk = (lds_void*)(smem + KREG + buf * TBYTES + (4 * k) * 1024 + wave * 1024);
                lds_void* dv = (lds_void*)(smem + VREG + buf * TBYTES + (4 * k) * 1024 + wave * 1024);
                __builtin_amdgcn_global_load_lds((global_void*)(ksrc + pieceK * 8), dk, 16, 0, 0);
                __builtin_amdgcn_global_load_lds((global_void*)(vsrc + pieceV * 8), dv, 16, 0, 0);
            }
        }
    };

    // ---- fragment reads ---------------------------------------------------------------------------------
    // K fragment s of a sub-block: lane (key row l32, half hh) reads piece 2s + hh of its row.
    // V fragments: lane l of a 16-lane block supplies the address of key row l/4, 4 columns at 4*(l%4).
    // The addresses below are those of tile buffer 0; after every tile they move on by one buffer.
    uint32_t kaddr[D / 16], vaddr[D / 32];
    {
        const uint32_t base = (uint32_t)(uintptr_t)(lds_void*)smem;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) kaddr[s] = base + KREG + l32 * ROWB + (((2 * s + hh) ^ (l32 & 15)) * 16);
        const int vrow = 4 * hh + ((lane & 15) >> 2);       // key row inside a group of eight
        const int x2 = (lane >> 4) & 1, q4 = lane & 3;
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
            vaddr[b] = base + VREG + vrow * ROWB + (((4 * b + 2 * x2 + (q4 >> 1)) ^ (2 * (vrow & 7))) * 16) + 8 * (q4 & 1);
    }
    auto read_k = [&](auto sub) {                            // K fragments of sub-block `sub` of the current K tile
        constexpr int O = decltype(sub)::value * 32 * ROWB;
        kf[0] = lds_read_b128<O>(kaddr[0]); kf[1] = lds_read_b128<O>(kaddr[1]);
        kf[2] = lds_read_b128<O>(kaddr[2]); kf[3] = lds_read_b128<O>(kaddr[3]);
        kf[4] = lds_read_b128<O>(kaddr[4]); kf[5] = lds_read_b128<O>(kaddr[5]);
        kf[6] = lds_read_b128<O>(kaddr[6]); kf[7] = lds_read_b128<O>(kaddr[7]);
    };
    // A V fragment arrives as two halves, read straight into the two halves of the register quadruple the MFMA
    // takes (a copy made between a read and the wait would copy what the read has not delivered yet; the
    // compiler has no reason to make one, and tests/test_kernel_asm.py checks the generated code for it).  The
    // wait names the first fragment; the empty statements that follow it in program order name the others, so
    // that no product that reads a fragment can be placed ahead of the wait.
    auto wait_v = [&]() {
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(vf[0]));
        asm volatile("" : "+v"(vf[1]));
        asm volatile("" : "+v"(vf[2]));
        asm volatile("" : "+v"(vf[3]));
        asm volatile("" : "+v"(vf[4]));
        asm volatile("" : "+v"(vf[5]));
        asm volatile("" : "+v"(vf[6]));
        asm volatile("" : "+v"(vf[7]));
    };
    auto advance = [&](uint32_t (&a)[D / 16], int delta) {
#pragma unroll
        for (int s = 0; s < D / 16; ++s) a[s] += (uint32_t)delta;
    };
    auto advance_v = [&](int delta) {
#pragma unroll
        for (int b = 0; b < D / 32; ++b) vaddr[b] += (uint32_t)delta;
    };

    // ---- the loop's loads, one instruction at a time ---------------------------------------------------
    // The eight loads of the tile three ahead are issued one by one at fixed places of the two periods of an
    // iteration (a wavefront that issues them in a burst stands still while the memory pipeline takes them
    // in, and so does its SIMD).  A tile that straddles the cache/chunk boundary or runs past the last key
    // is requested whole by dma_begin; the eight steps then reload the head's first rows into a scratch
    // area of LDS, which keeps them free of branches and the count of loads in flight the same.
    // Per-lane source addresses of the next load of K and of V.  Consecutive loads, also across tiles, lie a
    // fixed number of rows apart as long as the tiles stay inside the cache or inside the chunk, so the
    // addresses are simply advanced after every load and set up anew only when the kind of tile changes.
    const int ntiles = (n_end + TILE - 1) / TILE;
    const uint16_t* dma_pk = Kh;
    const uint16_t* dma_pv = Vh;
    uint32_t dma_dst = 0, dma_rstep = 0, dma_dstep = 0, dma_reg = 0;
    int dma_kind = -1;                                       // 0 cache, 1 chunk, 2 scratch area (nothing to load)
    auto dma_begin = [&](int tile, int slot) {
        const int kv0 = tile * TILE;
        const bool in_cache = kv0 + TILE <= tc, in_chunk = kv0 >= tc && kv0 + TILE <= n;
        const int kind = tile >= ntiles ? 2 : (in_cache ? 0 : (in_chunk ? 1 : 3));
        if (kind != dma_kind) {                              // a handful of times per workgroup
            if (kind == 3) issue_tile(tile, slot);           // a tile that needs row-by-row addresses: all of it now
            if (kind == 0 || kind == 1) {
                const int rs = kind == 0 ? D : Hkv * D;
                dma_pk = (kind == 0 ? Kh + (size_t)kv0 * D : kch + (size_t)(kv0 - tc) * rs) + (drow * rs + pieceK * 8);
                dma_pv = (kind == 0 ? Vh + (size_t)kv0 * D : vch + (size_t)(kv0 - tc) * rs) + (drow * rs + pieceV * 8);
                dma_rstep = (uint32_t)(16 * rs);
                dma_dstep = 4096;
                dma_reg = 1;
            } else {
                dma_pk = Kh + pieceK * 8;                   // the head's row 0: there is always one
                dma_pv = Vh + pieceV * 8;
                dma_rstep = 0;
                dma_dstep = 0;
                dma_reg = 0;
            }
            dma_kind = kind == 3 ? -1 : kind;                // after a row-by-row tile the next one sets up again
        }
        dma_dst = dma_reg ? (uint32_t)((slot & (NBUF - 1)) * TBYTES + wave * 1024) : (uint32_t)(DUMP + wave * 1024);
    };
    auto dma_step = [&](int i) {                             // i = 0..7: rows 16 (i/2) .., K (i even) or V (i odd)
        const int k = i >> 1;
        if (!(i & 1)) {
            __builtin_amdgcn_global_load_lds((global_void*)dma_pk, (lds_void*)(smem + (dma_reg * KREG + dma_dst + k * dma_dstep)), 16, 0, 0);
            dma_pk += dma_rstep;
        } else {
            __builtin_amdgcn_global_load_lds((global_void*)dma_pv, (lds_void*)(smem + (dma_reg * VREG + dma_dst + k * dma_dstep)), 16, 0, 0);
            dma_pv += dma_rstep;
        }
    };

    // ---- the pieces of a period ----------------------------------------------------------------------
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
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // (m_ref + 2^3 in the exponent) / c of block A in the lower half-wave, of block B in the upper one: what a raw
    // logit has to exceed for the block's reference to move.  No reference yet: anything finite exceeds it.
    const float inv_c = 1.0f / c;
    float thr_mix = -__builtin_inff();
    // S c - m of the sub-block in its softmax stage; the second half of a period turns the entries into the
    // weights exp2(S c - m) in place, and the first half of the next period adds them to the row sums just
    // before it overwrites them (so that the additions, too, sit beside MFMAs that have time to spare)
    float tw[2][16];
    float lsa[2] = {0.f, 0.f}, lsb[2] = {0.f, 0.f};          // row sums in two halves, on top of lsum
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int e = 0; e < 16; ++e) tw[x][e] = 0.f;

    // sub-blocks from here on reach past the limit of some row of block A / of block B
    const int first_maskedA = (t + min(32 * blkA, L - 1) + 1) / 32, first_maskedB = (t + min(32 * blkB, L - 1) + 1) / 32;

    // One period: sub-block m is in its softmax stage (its logits are in S), sub-block m-1 in its O += V^T P^T
    // stage (its V fragments were requested a period ago), sub-block m+1 in its S = K Q^T stage.  SUB = m & 1.
    // Before the first sub-block the weights and V fragments are zero, past the last one the K fragments come
    // from a stale buffer and the logits formed from them are never used: no period needs a variant of its own.
    //
    // A period is 32 slots of one MFMA each, fenced so that the compiler keeps them as written; a slot also
    // carries its share of everything else, so that the wavefront never issues a burst of one kind:
    //   slots  0..15  O += V^T P^T of sub-block m-1; the K fragments of sub-block m+1 (one read per slot, first
    //                 eight); of sub-block m two logits per slot: (mask,) running row maximum, and S c - m with
    //                 the reference as it stands (redone on the rare side path if the reference moves)
    //   between       row maxima across the half-waves; the reference moves if one outgrew it by 2^8
    //   slots 16..31  S = K Q^T of sub-block m+1, block A's chain then block B's; the V fragments of sub-block m
    //                 (two reads per slot, first eight); two weights per slot: exp2, row sum, bf16
    // and four of the eight loads of the tile three ahead.
    auto masked_logit = [&](auto mask, int x, int e, int m) -> float {
        float sv = S[x][e];
        if constexpr (decltype(mask)::value) {
            const int kv = 32 * m + 8 * (e / 4) + 4 * hh + (e % 4);
            if (kv > my_lim[x]) sv = -__builtin_inff();
        }
        return sv;
    };
    auto period = [&](int m, auto sub, auto mask) {
        constexpr int SUB = decltype(sub)::value;
        constexpr int KO = (SUB == 0 ? 1 : 0) * 32 * ROWB;   // sub-block m+1: the other half of the K tile kaddr points at
        constexpr int VO = SUB * 32 * ROWB;
        wait_v();                                            // requested a period ago
        float mx[2] = {-__builtin_inff(), -__builtin_inff()};
        static_for<0, 16>([&](auto I) {
            constexpr int i = decltype(I)::value;
            constexpr int tt = i >> 3, b = (i >> 1) & 3, x = i & 1;
            o[x][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[4 * tt + b], as_bf16x8(pf[x][tt]), o[x][b], 0, 0, 0);
            if constexpr (i < 8) kf[i] = lds_read_b128<KO>(kaddr[i]);
            constexpr int xs = i >> 3, e0 = 2 * (i & 7);
            const float s0 = masked_logit(mask, xs, e0, m), s1 = masked_logit(mask, xs, e0 + 1, m);
            mx[xs] = fmaxf(fmaxf(mx[xs], s0), s1);
            lsa[xs] += tw[xs][e0];                           // weights of sub-block m-1
            lsb[xs] += tw[xs][e0 + 1];
            tw[xs][e0] = __builtin_fmaf(s0, c, -m_use[xs]);
            tw[xs][e0 + 1] = __builtin_fmaf(s1, c, -m_use[xs]);
            if constexpr (i == 3) dma_step(4 * SUB);
            if constexpr (i == 11) dma_step(4 * SUB + 1);
            __builtin_amdgcn_sched_barrier(0);
        });
        // One exchange between the half-waves serves both blocks: afterwards the lower half-wave holds block A's
        // row maxima and the upper one block B's, each compared with its own block's threshold (kept in the
        // logits' unscaled units).  Only if some row outgrew it are the maxima formed in every lane.
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx[0]), __float_as_uint(mx[1]), false, false);
        float mmix;
        asm("v_max_f32 %0, %1, %2" : "=v"(mmix) : "v"(__uint_as_float(sw[0])), "v"(__uint_as_float(sw[1])));
        if (__any(mmix > thr_mix)) {
            // rare: O and the row sums hold all of sub-block m-1 (in the old reference) when they are rescaled
            const float mx0 = xhalf_max(mx[0]) * c, mx1 = xhalf_max(mx[1]) * c;
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                lsum[x] += lsa[x] + lsb[x];
                lsa[x] = 0.f; lsb[x] = 0.f;
                const float old_use = m_use[x];
                rescale(x, x == 0 ? mx0 : mx1);
                const float shift = old_use - m_use[x];      // S c - m was formed with the old reference
#pragma unroll
                for (int e = 0; e < 16; ++e) tw[x][e] += shift;
            }
            thr_mix = ((hh ? m_ref[1] : m_ref[0]) + RESCALE_TAU) * inv_c;
        }
        lds_wait(kf);
        static_for<0, 16>([&](auto I) {
            constexpr int i = decltype(I)::value;
            constexpr int x = i >> 3, s = i & 7;
            if constexpr (s == 0) mfma_qk_first(S[x], kf[s], qf[x][s]);
            else mfma_qk(S[x], kf[s], qf[x][s]);
            if constexpr (i < 8) {
                // V fragment i = [16-key step i / 4][column block i % 4]: key rows 0..7 and 8..15 of the step
                const bf16x4 lo = lds_read_tr16_b64<VO + (i >> 2) * 16 * ROWB>(vaddr[i & 3]);
                const bf16x4 hi = lds_read_tr16_b64<VO + (i >> 2) * 16 * ROWB + 8 * ROWB>(vaddr[i & 3]);
                vf[i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
            constexpr int xw = i >> 3, e0 = 2 * (i & 7);     // weights e0, e0 + 1 of block xw: 16-key step e0 / 8
            tw[xw][e0] = fast_exp2(tw[xw][e0]);
            tw[xw][e0 + 1] = fast_exp2(tw[xw][e0 + 1]);
            // The pair of the slot before is packed here: the conversion is a statement of its own, which the
            // compiler does not check, and a result of the transcendental unit must not be read by the very
            // next instruction.  The MFMA at the head of this slot lies between the two.
            if constexpr (i > 0) {
                constexpr int xp = (i - 1) >> 3, ep = 2 * ((i - 1) & 7);
                pf[xp][ep >> 3][(ep & 7) >> 1] = pack_bf16(tw[xp][ep], tw[xp][ep + 1]);
            }
            if constexpr (i == 4) dma_step(4 * SUB + 2);
            if constexpr (i == 12) dma_step(4 * SUB + 3);
            __builtin_amdgcn_sched_barrier(0);
        });
        pf[1][1][3] = pack_bf16_after_nop(tw[1][14], tw[1][15]);
    };

    // The same period for block B alone, once every row of the workgroup's blocks A has seen its last key: 16
    // slots.  The logits are first read in the third slot, behind the two loads, so that the last product of the
    // chain that formed them (the slot before this period) has long been written; block A's registers keep what
    // they hold (weights of an all-masked sub-block, i.e. zeros, and finished sums).
    auto period1 = [&](int m, auto sub, auto mask) {
        constexpr int SUB = decltype(sub)::value;
        constexpr int KO = (SUB == 0 ? 1 : 0) * 32 * ROWB;
        constexpr int VO = SUB * 32 * ROWB;
        wait_v();
        float mx[2] = {-__builtin_inff(), -__builtin_inff()};
        static_for<0, 8>([&](auto I) {
            constexpr int i = decltype(I)::value;
            constexpr int tt = i >> 2, b = i & 3;
            o[1][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[4 * tt + b], as_bf16x8(pf[1][tt]), o[1][b], 0, 0, 0);
            kf[i] = lds_read_b128<KO>(kaddr[i]);
            if constexpr (i == 0) dma_step(4 * SUB);
            if constexpr (i == 1) dma_step(4 * SUB + 1);
            // logits 0..15 over slots 2..7: three, three, three, three, two, two
            constexpr int e_lo = i < 2 ? 0 : (i < 6 ? 3 * (i - 2) : 12 + 2 * (i - 6));
            constexpr int e_hi = i < 2 ? 0 : (i < 6 ? e_lo + 3 : e_lo + 2);
            static_for<e_lo, e_hi>([&](auto E) {
                constexpr int e = decltype(E)::value;
                const float sv = masked_logit(mask, 1, e, m);
                mx[1] = fmaxf(mx[1], sv);
                if constexpr (e & 1) lsb[1] += tw[1][e];
                else lsa[1] += tw[1][e];
                tw[1][e] = __builtin_fmaf(sv, c, -m_use[1]);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx[0]), __float_as_uint(mx[1]), false, false);
        float mmix;
        asm("v_max_f32 %0, %1, %2" : "=v"(mmix) : "v"(__uint_as_float(sw[0])), "v"(__uint_as_float(sw[1])));
        if (__any(mmix > thr_mix)) {                         // block A's half-wave compares -inf: never
            const float mx1 = xhalf_max(mx[1]) * c;
            lsum[1] += lsa[1] + lsb[1];
            lsa[1] = 0.f; lsb[1] = 0.f;
            const float old_use = m_use[1];
            rescale(1, mx1);
            const float shift = old_use - m_use[1];
#pragma unroll
            for (int e = 0; e < 16; ++e) tw[1][e] += shift;
            thr_mix = ((hh ? m_ref[1] : m_ref[0]) + RESCALE_TAU) * inv_c;
        }
        lds_wait(kf);
        static_for<0, 8>([&](auto I) {
            constexpr int i = decltype(I)::value;
            if constexpr (i == 0) mfma_qk_first(S[1], kf[i], qf[1][i]);
            else mfma_qk(S[1], kf[i], qf[1][i]);
            const bf16x4 lo = lds_read_tr16_b64<VO + (i >> 2) * 16 * ROWB>(vaddr[i & 3]);
            const bf16x4 hi = lds_read_tr16_b64<VO + (i >> 2) * 16 * ROWB + 8 * ROWB>(vaddr[i & 3]);
            vf[i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            constexpr int e0 = 2 * i;
            tw[1][e0] = fast_exp2(tw[1][e0]);
            tw[1][e0 + 1] = fast_exp2(tw[1][e0 + 1]);
            if constexpr (i > 0) {                           // the pair of the slot before (see period)
                constexpr int ep = 2 * (i - 1);
                pf[1][ep >> 3][(ep & 7) >> 1] = pack_bf16(tw[1][ep], tw[1][ep + 1]);
            }
            if constexpr (i == 2) dma_step(4 * SUB + 2);
            if constexpr (i == 6) dma_step(4 * SUB + 3);
            __builtin_amdgcn_sched_barrier(0);
        });
        pf[1][1][3] = pack_bf16_after_nop(tw[1][14], tw[1][15]);
    };

    // ---- prologue: tiles 0, 1 and 2 requested, 0 and 1 awaited, S(0) formed ------------------------------
    issue_tile(0, 0);
    issue_tile(min(1, ntiles - 1), 1);
    issue_tile(min(2, ntiles - 1), 2);
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) pf[x][tt] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int p = 0; p < 8; ++p) vf[i][p] = (__bf16)0.f;
    asm volatile("s_waitcnt vmcnt(8)" ::: "memory");         // all but the newest tile's eight loads have landed
    __builtin_amdgcn_s_barrier();
    read_k(Flag<false>{});
    lds_wait(kf);
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int s = 0; s < D / 16; ++s)
            S[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[x][s], s == 0 ? zero16 : S[x], 0, 0, 0);
    asm volatile("" : "+v"(S[0]), "+v"(S[1]));

    // ---- main loop: one tile (two periods) per iteration; the tiles that need no mask first -----------
    // In iteration j the K fragments come from tile j (second half) and tile j+1 (first half), the V fragments
    // from tile j; tile j+3 is requested into the buffer tile j-1 has left, and tile j+2 is awaited before the
    // barrier.  Past the last tile the last one is requested again, into a buffer nobody reads any more.
    // Block A's last visible key lies in sub-block mA (the workgroup's last block A decides for all its
    // wavefronts, which keeps them in step); its weights are multiplied in period mA + 1, and the sub-block after
    // it is all masked and leaves zeros in block A's weight registers.  From the tile after that period on the
    // wavefront runs period1.
    const int mA = (t + min(L, 32 * (pair0 + wph)) - 1) / 32;
    const int j_single = min(ntiles, (mA + 3) >> 1);
    const int j_maskedA = min(j_single, first_maskedA >> 1);  // tiles from here on hold a masked sub-block
    const int j_maskedB = min(ntiles, first_maskedB >> 1);
    auto tile_iter = [&](int j, auto mask, auto both) {
        const int wrap = ((j + 1) & (NBUF - 1)) == 0 ? TBYTES - NBUF * TBYTES : TBYTES;
        dma_begin(j + 3, j + 3);
        // K: tile j, sub-block 1;  V: tile j, sub-block 0
        if constexpr (decltype(both)::value) period(2 * j, Flag<false>{}, mask);
        else period1(2 * j, Flag<false>{}, mask);
        advance(kaddr, wrap);                                // K: on to tile j+1
        // K: tile j+1, sub-block 0;  V: tile j, sub-block 1
        if constexpr (decltype(both)::value) period(2 * j + 1, Flag<true>{}, mask);
        else period1(2 * j + 1, Flag<true>{}, mask);
        advance_v(wrap);
        // tile j+2 has landed (the eight loads of tile j+3 may still be on their way), and this wavefront's
        // LDS reads are done, before anyone overwrites what they read
        asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
    };
    int j = 0;
    for (; j < j_maskedA; ++j) tile_iter(j, Flag<false>{}, Flag<true>{});
    for (; j < j_single; ++j) tile_iter(j, Flag<true>{}, Flag<true>{});
    for (; j < j_maskedB; ++j) tile_iter(j, Flag<false>{}, Flag<false>{});
    for (; j < ntiles; ++j) tile_iter(j, Flag<true>{}, Flag<false>{});
#pragma unroll
    for (int x = 0; x < 2; ++x) {                            // ... and its weights are not in the row sums yet
        float tail = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) tail += tw[x][e];
        lsum[x] += lsa[x] + lsb[x] + tail;
    }
    wait_v();
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)                           // the last sub-block still owes its O += V^T P^T
#pragma unroll
        for (int b = 0; b < D / 32; ++b)
#pragma unroll
            for (int x = 0; x < 2; ++x)
                o[x][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[4 * tt + b], as_bf16x8(pf[x][tt]), o[x][b], 0, 0, 0);

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
    hipLaunchKernelGGL(attn_fwd64_kernel, dim3(ntile * ny), dim3(w64::NT), 0, st, (const uint16_t*)q,
                       (const uint16_t*)c.K, (const uint16_t*)c.V, (const uint16_t*)ks.k, (const uint16_t*)ks.v, ks.rows,
                       (uint16_t*)out, lse, t, L, g.Hq, g.G, g.cap, g.max_chunk, hpw, ntile, ny,
                       (float)(g.scale * (double)LOG2E));
    return hipGetLastError();
}

}  // namespace infmllm
