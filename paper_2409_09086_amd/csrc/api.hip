// Host side of the C ABI declared in include/infmllm.h: argument checks, workspace carving,
// the host bookkeeping of one stream (cached length, tokens streamed) and the sequence of
// kernel launches that makes up one streaming step.  No device memory is allocated here and nothing synchronises.
#include "../../include/infmllm.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "launch.h"

using namespace infmllm;

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

int fail_hip(hipError_t e, const char* what)
{
    return fail(INFMLLM_EHIP, "%s: %s", what, hipGetErrorString(e));
}

constexpr size_t ALIGN = 256;
size_t up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

// Workspace of infmllm_stream_attach_static: one array per GPU inside the library's code object, for callers
// that cannot allocate device memory.  `scratch` is a host-side stand-in for the symbol, never a device
// address: host code uses the address hipGetSymbolAddress returns for the current device, looked up once per
// device.  At most one stream per device holds the array at a time.
static __device__ __align__(256) unsigned char scratch[INFMLLM_STATIC_WORKSPACE_BYTES];
constexpr int MAX_DEVICES = 64;
std::mutex g_static_mu;
void* g_static_ptr[MAX_DEVICES];                 // device address of `scratch` on each GPU, null until looked up
const infmllm_stream* g_static_owner[MAX_DEVICES];

}  // namespace

struct infmllm_stream {
    Geometry g;
    int dtype;
    int impl;            // 0 = matrix cores where the dtype allows, 1 = plain arithmetic
    bool attached;
    int static_dev = -1; // device whose library-owned workspace this stream holds (-1: caller's workspace)
    hipStream_t st;
    CacheView cache;
    MoveList mv;         // retained rows the pending or running eviction moves
    int len;             // rows cached
    int64_t streamed;    // tokens streamed so far
    int last_cnd;        // candidates of the most recent evicting step (0 = none)
    // cache-relative rotary encoding (off while rope_base == 0): turned copies that attention and scoring read
    double rope_base = 0.0;
    void* K_rot = nullptr;      // [Hkv][cap (+pad)][d]
    void* kc_rot = nullptr;     // [max_chunk][Hkv][d]
    void* q_rot = nullptr;      // [max_chunk][Hq][d]
    double* rope_tab = nullptr; // [cap][d/2] (cos, sin)
    int rot_rows = 0;           // leading rows of the live cache whose K_rot entry is current
    // eviction left pending by infmllm_step_attend: scores are in Wb, the chunk is still read in place
    bool pending = false;
    KeySource pend_ks{0, nullptr, nullptr};
    int pend_n = 0, pend_L = 0;
    float* lse;          // [Hq][max_chunk]
    float* Wb;           // [Hkv][cap]
    int32_t* I;          // [Hkv][B]
    FwdScratch fwd;      // scratch of the row-split scoring launch
    float* dec_part;     // partials of the decoding step
    // optional per-kernel timing: one event pair per kernel per step, up to prof_cap steps
    std::vector<hipEvent_t> prof_ev;   // [prof_cap][INFMLLM_K_COUNT][2]
    std::vector<char> prof_used;       // [prof_cap][INFMLLM_K_COUNT]
    int prof_cap = 0, prof_steps = 0;

    unsigned prof_mask = ~0u;          // kernels whose events are recorded (bit INFMLLM_K_*)
    void mark(int kernel, int edge)
    {
        if (prof_steps >= prof_cap) return;
        const bool bracket = ((prof_mask >> INFMLLM_K_EVICT) & 1u) &&
                             ((kernel == INFMLLM_K_SELECT && edge == 0) || (kernel == INFMLLM_K_COMPACT && edge == 1));
        if (!((prof_mask >> kernel) & 1u) && !bracket) return;
        const size_t slot = (size_t)prof_steps * INFMLLM_K_COUNT + kernel;
        if (hipEventRecord(prof_ev[slot * 2 + edge], st) == hipSuccess) prof_used[slot] |= (char)(1 << edge);
    }
    void drop_events()
    {
        for (hipEvent_t e : prof_ev) (void)hipEventDestroy(e);
        prof_ev.clear(); prof_used.clear(); prof_cap = 0; prof_steps = 0;
    }

    struct Layout {
        size_t K, V, pos, score, rank, row, lse, Wb, I, mv_src, mv_dst, mv_x, mv_score, mv_count, score_part, dec_part, K_rot,
            kc_rot, q_rot, rope_tab, total;
    };
    Layout layout() const
    {
        Layout L;
        size_t off = 0;
        const size_t kv = up(((size_t)g.Hkv * g.cap + CACHE_PAD_ROWS) * g.d * g.elt);
        const size_t ps = up((size_t)g.Hkv * g.cap * 4);
        L.K = off; off += kv;
        L.V = off; off += kv;
        L.pos = off; off += ps;
        L.score = off; off += ps;
        L.rank = off; off += ps;
        L.row = off; off += ps;
        L.lse = off; off += up((size_t)g.Hq * g.max_chunk * 4);
        L.Wb = off; off += ps;
        L.I = off; off += up((size_t)g.Hkv * g.B * 4);
        const size_t ml = up((size_t)g.Hkv * (g.max_chunk + g.max_decode) * 4);
        L.mv_src = off; off += ml;
        L.mv_dst = off; off += ml;
        L.mv_x = off; off += ml;
        L.mv_score = off; off += ml;
        L.mv_count = off; off += up((size_t)g.Hkv * 4);
        // row-split scoring (bf16 streams): partial column sums and arrival counters
        L.score_part = off; off += up(g.elt == 2 ? (size_t)SCORE_SPLIT_WGS * (256 + 1) * 4 : 0);
        L.dec_part = off; off += up(g.max_decode > 0 ? (size_t)g.Hq * DECODE_MAX_SPLIT * (g.d + 2) * 4 + (size_t)g.Hkv * 4 : 0);
        const bool rope = rope_base > 0.0;
        L.K_rot = off; off += rope ? kv : 0;
        L.kc_rot = off; off += up(rope ? (size_t)g.max_chunk * g.Hkv * g.d * g.elt : 0);
        L.q_rot = off; off += up(rope ? (size_t)g.max_chunk * g.Hq * g.d * g.elt : 0);
        L.rope_tab = off; off += up(rope ? (size_t)g.cap * (g.d / 2) * 2 * sizeof(double) : 0);
        L.total = off;
        return L;
    }
};

extern "C" {

const char* infmllm_last_error(void) { return g_err.c_str(); }

int infmllm_stream_create(int budget, int recent, int heads, int kv_heads, int head_dim, int dtype,
                          infmllm_stream_t** out)
{
    if (!out) return fail(INFMLLM_EINVAL, "create: out is null");
    *out = nullptr;
    if (budget <= 0) return fail(INFMLLM_EINVAL, "create: budget must be positive (got %d)", budget);
    if (recent < 0 || recent > budget)
        return fail(INFMLLM_EINVAL, "create: recent must lie in 0..budget (got %d, budget %d)", recent, budget);
    if (heads <= 0 || kv_heads <= 0 || heads % kv_heads != 0)
        return fail(INFMLLM_EINVAL, "create: kv_heads must divide heads (got %d, %d)", heads, kv_heads);
    if (head_dim != 64 && head_dim != 128)
        return fail(INFMLLM_EINVAL, "create: head_dim must be 64 or 128 (got %d)", head_dim);
    if (dtype != INFMLLM_BF16 && dtype != INFMLLM_FP32)
        return fail(INFMLLM_EINVAL, "create: unknown dtype %d", dtype);
    if (budget > 131072)
        return fail(INFMLLM_EINVAL, "create: budget %d is beyond the supported 131072 rows", budget);
    infmllm_stream* s = new (std::nothrow) infmllm_stream();
    if (!s) return fail(INFMLLM_ENOMEM, "create: out of host memory");
    s->g.B = budget; s->g.R = recent; s->g.Hq = heads; s->g.Hkv = kv_heads; s->g.G = heads / kv_heads;
    s->g.d = head_dim; s->g.max_chunk = budget; s->g.max_decode = 0; s->g.cap = 2 * budget;
    s->g.elt = dtype == INFMLLM_BF16 ? 2 : 4;
    s->g.scale = 1.0 / std::sqrt((double)head_dim);
    s->g.bias = 1e-4;
    s->g.policy = POLICY_INFMLLM;
    s->g.attn_tile = 0;
    s->dtype = dtype; s->impl = 0; s->attached = false; s->st = nullptr; s->len = 0;
    s->streamed = 0; s->last_cnd = 0; s->lse = nullptr; s->Wb = nullptr; s->I = nullptr;
    *out = s;
    return INFMLLM_OK;
}

void infmllm_stream_destroy(infmllm_stream_t* s)
{
    if (!s) return;
    if (s->static_dev >= 0) {
        std::lock_guard<std::mutex> lk(g_static_mu);
        if (g_static_owner[s->static_dev] == s) g_static_owner[s->static_dev] = nullptr;
    }
    s->drop_events();
    delete s;
}

int infmllm_stream_set_param(infmllm_stream_t* s, int which, double value)
{
    if (!s) return fail(INFMLLM_EINVAL, "set_param: stream is null");
    if (s->attached) return fail(INFMLLM_ESTATE, "set_param: parameters are fixed once the stream is attached");
    if (!std::isfinite(value)) return fail(INFMLLM_EINVAL, "set_param: value is not finite");
    switch (which) {
        case INFMLLM_PARAM_BIAS:
            if (value < 0) return fail(INFMLLM_EINVAL, "set_param: bias must be >= 0");
            s->g.bias = value;
            return INFMLLM_OK;
        case INFMLLM_PARAM_SCALE:
            if (value <= 0) return fail(INFMLLM_EINVAL, "set_param: scale must be > 0");
            s->g.scale = value;
            return INFMLLM_OK;
        case INFMLLM_PARAM_MAX_CHUNK:
            if (value < 1 || value > (double)(1 << 24) || value != std::floor(value))
                return fail(INFMLLM_EINVAL, "set_param: max_chunk must be an integer in 1..2^24");
            s->g.max_chunk = (int)value;
            s->g.cap = s->g.B + s->g.max_decode + s->g.max_chunk;
            return INFMLLM_OK;
        case INFMLLM_PARAM_MAX_DECODE:
            if (value < 0 || value > (double)(1 << 24) || value != std::floor(value))
                return fail(INFMLLM_EINVAL, "set_param: max_decode must be an integer in 0..2^24");
            s->g.max_decode = (int)value;
            s->g.cap = s->g.B + s->g.max_decode + s->g.max_chunk;
            return INFMLLM_OK;
        case INFMLLM_PARAM_POLICY:
            if (value != 0 && value != 1 && value != 2 && value != 3)
                return fail(INFMLLM_EINVAL, "set_param: policy must be 0, 1, 2 or 3");
            s->g.policy = (int)value;
            return INFMLLM_OK;
        case INFMLLM_PARAM_ROPE_BASE:
            if (value != 0 && !(value > 1)) return fail(INFMLLM_EINVAL, "set_param: rope_base must be 0 (off) or > 1");
            s->rope_base = value;
            return INFMLLM_OK;
        case INFMLLM_PARAM_IMPL:
            if (value != 0 && value != 1) return fail(INFMLLM_EINVAL, "set_param: impl must be 0 or 1");
            s->impl = (int)value;
            return INFMLLM_OK;
        case INFMLLM_PARAM_ATTN_TILE:
            if (value < 0 || value > 5 || value != std::floor(value))
                return fail(INFMLLM_EINVAL, "set_param: attn_tile must be 0..5");
            s->g.attn_tile = (int)value;
            return INFMLLM_OK;
        default:
            return fail(INFMLLM_EINVAL, "set_param: unknown parameter %d", which);
    }
}

size_t infmllm_stream_workspace_bytes(const infmllm_stream_t* s) { return s ? s->layout().total : 0; }

int infmllm_stream_attach(infmllm_stream_t* s, void* ws, size_t bytes, void* hip_stream)
{
    if (!s) return fail(INFMLLM_EINVAL, "attach: stream is null");
    if (s->attached) return fail(INFMLLM_ESTATE, "attach: stream is already attached");
    if (!ws) return fail(INFMLLM_EINVAL, "attach: workspace is null");
    if ((uintptr_t)ws % ALIGN) return fail(INFMLLM_EINVAL, "attach: workspace must be 256-byte aligned");
    const infmllm_stream::Layout L = s->layout();
    if (bytes < L.total)
        return fail(INFMLLM_ENOMEM, "attach: workspace has %zu bytes, %zu needed", bytes, L.total);
    if ((size_t)s->g.cap * 4 > 150 * 1024 && (s->dtype == INFMLLM_FP32 || s->impl == 1))
        return fail(INFMLLM_EINVAL, "attach: budget + max_chunk = %d rows is beyond what the plain-arithmetic "
                                    "attention kernel keeps in LDS (38400)", s->g.cap);
    if (s->g.cap - s->g.R > 131072)
        return fail(INFMLLM_EINVAL, "attach: budget + max_decode + max_chunk - recent = %d exceeds the 131072 candidates "
                                    "a step can rank", s->g.cap - s->g.R);
    char* base = (char*)ws;
    {
        // kernels that read whole key tiles rely on every byte of the cache being finite
        hipError_t e = launch_zero(ws, L.total, (hipStream_t)hip_stream);
        if (e != hipSuccess) return fail_hip(e, "attach: clearing the workspace");
    }
    s->cache.K = base + L.K;
    s->cache.V = base + L.V;
    s->cache.pos = (int32_t*)(base + L.pos);
    s->cache.score = (float*)(base + L.score);
    s->cache.rank = (int32_t*)(base + L.rank);
    s->cache.row = (int32_t*)(base + L.row);
    s->mv.src = (int32_t*)(base + L.mv_src);
    s->mv.dst = (int32_t*)(base + L.mv_dst);
    s->mv.x = (int32_t*)(base + L.mv_x);
    s->mv.score = (float*)(base + L.mv_score);
    s->mv.count = (int32_t*)(base + L.mv_count);
    s->mv.max = s->g.max_chunk + s->g.max_decode;
    s->lse = (float*)(base + L.lse);
    s->Wb = (float*)(base + L.Wb);
    s->I = (int32_t*)(base + L.I);
    s->fwd.score_part = (float*)(base + L.score_part);
    s->dec_part = (float*)(base + L.dec_part);
    s->K_rot = base + L.K_rot;
    s->kc_rot = base + L.kc_rot;
    s->q_rot = base + L.q_rot;
    s->rope_tab = (double*)(base + L.rope_tab);
    s->rot_rows = 0;
    if (s->rope_base > 0.0) {
        // (cos, sin) of p * base^(-2i/d) in fp64 for every cache position p and pair i; the copy is finished
        // before this function returns (the host buffer is pageable and goes out of scope).  Within a position
        // pair i = 8a + e sits in slot e * (d/16) + a (see launch_rope).
        const int half = s->g.d / 2, groups = s->g.d / 16;
        std::vector<double> tab((size_t)s->g.cap * half * 2);
        for (int i = 0; i < half; ++i) {
            const double inv = std::pow(s->rope_base, -2.0 * (double)i / (double)s->g.d);
            const int slot = (i % 8) * groups + i / 8;
            for (int p = 0; p < s->g.cap; ++p) {
                const double ang = (double)p * inv;
                tab[((size_t)p * half + slot) * 2] = std::cos(ang);
                tab[((size_t)p * half + slot) * 2 + 1] = std::sin(ang);
            }
        }
        hipError_t e = hipMemcpyAsync(s->rope_tab, tab.data(), tab.size() * sizeof(double), hipMemcpyHostToDevice,
                                      (hipStream_t)hip_stream);
        if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)hip_stream);
        if (e != hipSuccess) return fail_hip(e, "attach: position table");
    }
    s->st = (hipStream_t)hip_stream;
    s->len = 0; s->streamed = 0; s->last_cnd = 0;
    s->attached = true;
    return INFMLLM_OK;
}

int infmllm_stream_attach_static(infmllm_stream_t* s, void* hip_stream)
{
    if (!s) return fail(INFMLLM_EINVAL, "attach_static: stream is null");
    if (s->attached) return fail(INFMLLM_ESTATE, "attach_static: stream is already attached");
    if (s->rope_base > 0.0)
        return fail(INFMLLM_EINVAL, "attach_static: streams with the rotary position table are not supported "
                                    "(the table is uploaded from a host buffer)");
    const size_t need = s->layout().total;
    if (need > (size_t)INFMLLM_STATIC_WORKSPACE_BYTES)
        return fail(INFMLLM_ENOMEM, "attach_static: the stream needs %zu bytes of workspace, the library's array holds %zu",
                    need, (size_t)INFMLLM_STATIC_WORKSPACE_BYTES);
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "attach_static: hipGetDevice");
    if (dev < 0 || dev >= MAX_DEVICES) return fail(INFMLLM_EINVAL, "attach_static: device index %d is not supported", dev);
    void* ptr = nullptr;
    {
        std::lock_guard<std::mutex> lk(g_static_mu);
        if (!g_static_ptr[dev]) {
            void* p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !p) return fail_hip(e, "attach_static: hipGetSymbolAddress");
            g_static_ptr[dev] = p;
        }
        if (g_static_owner[dev])
            return fail(INFMLLM_ESTATE, "attach_static: another stream holds this device's workspace array");
        g_static_owner[dev] = s;
        ptr = g_static_ptr[dev];
    }
    s->static_dev = dev;
    const int rc = infmllm_stream_attach(s, ptr, (size_t)INFMLLM_STATIC_WORKSPACE_BYTES, hip_stream);
    if (rc != INFMLLM_OK) {
        std::lock_guard<std::mutex> lk(g_static_mu);
        g_static_owner[dev] = nullptr;
        s->static_dev = -1;
    }
    return rc;
}

}  // extern "C"

namespace {

// a1-a4 of a step: append (unless the chunk is read in place), attention, and either the warm-up
// index list or the scores.  On return *evict says whether a5-a7 are still to run; the stream's
// counters are advanced only when they are not.
int step_front(infmllm_stream* s, const void* q, const void* k, const void* v, int L, void* out, int32_t* retained,
               int32_t* n_retained, bool* evict, KeySource* ks_out, const char* who)
{
    if (!s) return fail(INFMLLM_EINVAL, "%s: stream is null", who);
    if (!s->attached) return fail(INFMLLM_ESTATE, "%s: stream has no workspace attached", who);
    if (s->pending) return fail(INFMLLM_ESTATE, "%s: an eviction is pending on this stream", who);
    if (!q || !k || !v || !out) return fail(INFMLLM_EINVAL, "%s: q, k, v and out must not be null", who);
    if (L < 1) return fail(INFMLLM_EINVAL, "%s: chunk_len must be >= 1 (got %d)", who, L);
    if (L > s->g.max_chunk)
        return fail(INFMLLM_ECAPACITY, "%s: chunk_len %d exceeds max_chunk %d", who, L, s->g.max_chunk);
    if (s->streamed + L > (int64_t)INT32_MAX)
        return fail(INFMLLM_ECAPACITY, "%s: stream positions would exceed 2^31-1", who);

    const Geometry& g = s->g;
    const CacheView& cur = s->cache;
    const int t = s->len, n = t + L;
    const bool mfma = (s->dtype == INFMLLM_BF16 && s->impl == 0);
    hipError_t e;

    // An evicting step on the matrix-core path never appends: attention and scoring read the chunk's
    // rows in place and the placement writes the survivors into the rows the eviction frees.
    const bool in_place = mfma && n > g.B;
    const KeySource ks = in_place ? KeySource{t, k, v} : KeySource{n, nullptr, nullptr};
    if (!in_place) {
        s->mark(INFMLLM_K_APPEND, 0);
        if ((e = launch_append(g, cur, k, v, t, L, s->streamed, s->st)) != hipSuccess) return fail_hip(e, "append");
        s->mark(INFMLLM_K_APPEND, 1);
    }
    // With the position encoding on, attention and scoring read turned copies of the keys and queries;
    // selection and compaction go on working with the rows as given (ks).
    CacheView att = cur;
    KeySource ks_att = ks;
    const void* q_att = q;
    if (s->rope_base > 0.0) {
        s->mark(INFMLLM_K_ROPE, 0);
        const int have = s->rot_rows < t ? s->rot_rows : t;
        e = launch_rope(g, cur.K, s->K_rot, cur.rank, have, in_place ? t : n, in_place ? k : nullptr, s->kc_rot, q,
                        s->q_rot, t, L, s->rope_tab, s->st);
        if (e != hipSuccess) return fail_hip(e, "position encoding");
        s->mark(INFMLLM_K_ROPE, 1);
        att.K = s->K_rot;
        if (in_place) ks_att.k = s->kc_rot;
        q_att = s->q_rot;
        s->rot_rows = in_place ? t : n;
    }
    s->mark(INFMLLM_K_ATTN, 0);
    e = mfma ? launch_attn_mfma(g, att, ks_att, q_att, t, L, out, s->lse, s->st)
             : launch_attn_simple(g, att, q_att, t, L, out, s->lse, s->st);
    if (e != hipSuccess) return fail_hip(e, "attention");
    s->mark(INFMLLM_K_ATTN, 1);

    *evict = n > g.B;
    *ks_out = ks;
    if (n <= g.B) {
        // the chunk fits: nothing is evicted
        if ((e = launch_iota(g, n, retained, n_retained, s->st)) != hipSuccess) return fail_hip(e, "index list");
        s->len = n;
        s->last_cnd = 0;
        s->streamed += L;
        if (s->prof_steps < s->prof_cap) ++s->prof_steps;
        return INFMLLM_OK;
    }
    s->mark(INFMLLM_K_SCORE, 0);
    if (g.policy == POLICY_WINDOW || g.policy == POLICY_INITIAL_RECENT)
        e = launch_rank_scores(g, s->Wb, n - g.R, g.policy == POLICY_WINDOW ? 1.f : -1.f, s->st);
    else
        e = mfma ? launch_score_mfma(g, att, ks_att, q_att, s->lse, s->fwd, t, L, s->Wb, s->st)
                 : launch_score_simple(g, att, q_att, s->lse, t, L, s->Wb, s->st);
    if (e != hipSuccess) return fail_hip(e, "score");
    s->mark(INFMLLM_K_SCORE, 1);
    return INFMLLM_OK;
}

// host bookkeeping once a5-a7 of a step of L tokens (n keys before eviction) have been launched
void step_done(infmllm_stream* s, int n, int L)
{
    s->len = s->g.B;
    s->last_cnd = n - s->g.R;
    s->streamed += L;
    s->pending = false;
    s->rot_rows = 0;                                          // every row has a new stream-order index: the turned copies are stale
    if (s->prof_steps < s->prof_cap) ++s->prof_steps;
}

}  // namespace

extern "C" {

int infmllm_step(infmllm_stream_t* s, const void* q, const void* k, const void* v, int L, void* out,
                 int32_t* retained, int32_t* n_retained)
{
    bool evict = false;
    KeySource ks{0, nullptr, nullptr};
    const int rc = step_front(s, q, k, v, L, out, retained, n_retained, &evict, &ks, "step");
    if (rc != INFMLLM_OK || !evict) return rc;
    const Geometry& g = s->g;
    const int n = s->len + L;
    hipError_t e;
    s->mark(INFMLLM_K_SELECT, 0);
    if ((e = launch_select(g, s->Wb, n, ks.rows, s->I, retained, n_retained, s->cache, s->mv, s->st)) != hipSuccess)
        return fail_hip(e, "step: select");
    s->mark(INFMLLM_K_SELECT, 1);
    s->mark(INFMLLM_K_COMPACT, 0);
    // rows that can need a new home: the chunk rows read in place and the cached rows at or above the budget
    const int nmax = (n - ks.rows) + (ks.rows > g.B ? ks.rows - g.B : 0);
    if ((e = launch_place(g, s->cache, ks, s->streamed, s->mv, nmax, s->st)) != hipSuccess)
        return fail_hip(e, "step: placement");
    s->mark(INFMLLM_K_COMPACT, 1);
    step_done(s, n, L);
    return INFMLLM_OK;
}

int infmllm_step_attend(infmllm_stream_t* s, const void* q, const void* k, const void* v, int L, void* out,
                        int32_t* retained, int32_t* n_retained)
{
    bool evict = false;
    KeySource ks{0, nullptr, nullptr};
    const int rc = step_front(s, q, k, v, L, out, retained, n_retained, &evict, &ks, "step_attend");
    if (rc != INFMLLM_OK || !evict) return rc;
    s->pending = true;
    s->pend_ks = ks;
    s->pend_n = s->len + L;
    s->pend_L = L;
    return INFMLLM_OK;
}

int infmllm_stream_pending(const infmllm_stream_t* s) { return s ? (s->pending ? 1 : 0) : -1; }

int infmllm_evict_batched(infmllm_stream_t* const* streams, int count, int32_t* const* retained,
                          int32_t* const* n_retained)
{
    if (!streams || count < 1) return fail(INFMLLM_EINVAL, "evict_batched: no streams");
    const infmllm_stream* s0 = streams[0];
    for (int i = 0; i < count; ++i) {
        const infmllm_stream* s = streams[i];
        if (!s) return fail(INFMLLM_EINVAL, "evict_batched: stream %d is null", i);
        if (!s->attached || !s->pending) return fail(INFMLLM_ESTATE, "evict_batched: stream %d has no eviction pending", i);
        for (int j = 0; j < i; ++j)
            if (streams[j] == s) return fail(INFMLLM_EINVAL, "evict_batched: stream %d appears twice", i);
        const Geometry &a = s->g, &b = s0->g;
        if (a.B != b.B || a.R != b.R || a.Hq != b.Hq || a.Hkv != b.Hkv || a.d != b.d || a.cap != b.cap ||
            a.elt != b.elt || a.max_chunk != b.max_chunk || a.max_decode != b.max_decode || s->st != s0->st)
            return fail(INFMLLM_EINVAL, "evict_batched: stream %d differs from stream 0 in geometry or HIP stream", i);
    }
    infmllm_stream* lead = streams[0];
    for (int base = 0; base < count; base += EVICT_MAX_JOBS) {
        EvictBatch eb{};
        eb.count = count - base < EVICT_MAX_JOBS ? count - base : EVICT_MAX_JOBS;
        int nmax = 0;
        for (int j = 0; j < eb.count; ++j) {
            infmllm_stream* s = streams[base + j];
            EvictJob& job = eb.job[j];
            job.Wb = s->Wb; job.I = s->I;
            job.user_I = retained ? retained[base + j] : nullptr;
            job.user_count = n_retained ? n_retained[base + j] : nullptr;
            job.c = s->cache; job.mv = s->mv;
            job.kc = s->pend_ks.k; job.vc = s->pend_ks.v;
            job.tc = s->pend_ks.rows; job.pos0 = (int)s->streamed; job.n = s->pend_n;
            const int m = (job.n - job.tc) + (job.tc > s->g.B ? job.tc - s->g.B : 0);
            nmax = m > nmax ? m : nmax;
        }
        hipError_t e;
        lead->mark(INFMLLM_K_SELECT, 0);
        if ((e = launch_select_batch(lead->g, eb, lead->st)) != hipSuccess) return fail_hip(e, "evict_batched: select");
        lead->mark(INFMLLM_K_SELECT, 1);
        lead->mark(INFMLLM_K_COMPACT, 0);
        if ((e = launch_place_batch(lead->g, eb, nmax, lead->st)) != hipSuccess) return fail_hip(e, "evict_batched: placement");
        lead->mark(INFMLLM_K_COMPACT, 1);
        for (int j = 0; j < eb.count; ++j) step_done(streams[base + j], streams[base + j]->pend_n, streams[base + j]->pend_L);
    }
    return INFMLLM_OK;
}

int infmllm_stream_profile(infmllm_stream_t* s, int max_steps)
{
    if (!s) return fail(INFMLLM_EINVAL, "profile: stream is null");
    if (!s->attached) return fail(INFMLLM_ESTATE, "profile: stream has no workspace attached");
    if (max_steps < 0 || max_steps > 4096) return fail(INFMLLM_EINVAL, "profile: max_steps must lie in 0..4096");
    s->drop_events();
    const size_t nev = (size_t)max_steps * INFMLLM_K_COUNT * 2;
    s->prof_ev.reserve(nev);
    for (size_t i = 0; i < nev; ++i) {
        hipEvent_t ev;
        hipError_t e = hipEventCreate(&ev);
        if (e != hipSuccess) { s->drop_events(); return fail_hip(e, "profile: hipEventCreate"); }
        s->prof_ev.push_back(ev);
    }
    s->prof_used.assign((size_t)max_steps * INFMLLM_K_COUNT, 0);
    s->prof_cap = max_steps;
    s->prof_steps = 0;
    return INFMLLM_OK;
}

int infmllm_stream_profile_select(infmllm_stream_t* s, unsigned kernels)
{
    if (!s) return fail(INFMLLM_EINVAL, "profile_select: stream is null");
    if (kernels == 0 || (kernels >> INFMLLM_K_COUNT)) return fail(INFMLLM_EINVAL, "profile_select: bad kernel mask");
    s->prof_mask = kernels;
    return INFMLLM_OK;
}

int infmllm_stream_profile_read(infmllm_stream_t* s, float* ms, int* launches)
{
    if (!s || !ms || !launches) return fail(INFMLLM_EINVAL, "profile_read: null argument");
    for (int k = 0; k < INFMLLM_K_COUNT; ++k) { ms[k] = 0.f; launches[k] = 0; }
    for (int step = 0; step < s->prof_steps; ++step)
        for (int k = 0; k < INFMLLM_K_COUNT; ++k) {
            const size_t slot = (size_t)step * INFMLLM_K_COUNT + k;
            const bool whole_eviction = (k == INFMLLM_K_EVICT);
            const size_t first = whole_eviction ? (size_t)step * INFMLLM_K_COUNT + INFMLLM_K_SELECT : slot;
            const size_t last = whole_eviction ? (size_t)step * INFMLLM_K_COUNT + INFMLLM_K_COMPACT : slot;
            if (!(s->prof_used[first] & 1) || !(s->prof_used[last] & 2)) continue;
            if (!((s->prof_mask >> k) & 1u)) continue;
            hipError_t e = hipEventSynchronize(s->prof_ev[last * 2 + 1]);
            float dt = 0.f;
            if (e == hipSuccess) e = hipEventElapsedTime(&dt, s->prof_ev[first * 2], s->prof_ev[last * 2 + 1]);
            if (e != hipSuccess) return fail_hip(e, "profile_read: event");
            ms[k] += dt;
            ++launches[k];
        }
    std::fill(s->prof_used.begin(), s->prof_used.end(), 0);
    s->prof_steps = 0;
    return INFMLLM_OK;
}

// One decoding step on a stream whose state has been checked: launches, then the host-side counters.
static int decode_one(infmllm_stream* s, const void* q, const void* k, const void* v, void* out)
{
    s->mark(INFMLLM_K_DECODE, 0);
    hipError_t e;
    if (s->rope_base > 0.0) {
        // the token's row enters the cache as given; the decoding kernels see the turned copies (and put the
        // turned key at row t of K_rot themselves)
        const CacheView& cur = s->cache;
        const int t = s->len;
        if ((e = launch_append(s->g, cur, k, v, t, 1, s->streamed, s->st)) != hipSuccess) return fail_hip(e, "decode: append");
        e = launch_rope(s->g, cur.K, s->K_rot, cur.rank, s->rot_rows < t ? s->rot_rows : t, t, k, s->kc_rot, q, s->q_rot,
                        t, 1, s->rope_tab, s->st);
        if (e != hipSuccess) return fail_hip(e, "decode: position encoding");
        CacheView att = cur;
        att.K = s->K_rot;
        e = launch_decode(s->g, att, s->q_rot, s->kc_rot, v, t, s->streamed, out, s->dec_part, DECODE_MAX_SPLIT, s->st);
        s->rot_rows = t + 1;
    } else {
        e = launch_decode(s->g, s->cache, q, k, v, s->len, s->streamed, out, s->dec_part, DECODE_MAX_SPLIT, s->st);
    }
    if (e != hipSuccess) return fail_hip(e, "decode");
    s->mark(INFMLLM_K_DECODE, 1);
    s->len += 1;
    s->streamed += 1;
    s->last_cnd = 0;
    if (s->prof_steps < s->prof_cap) ++s->prof_steps;
    return INFMLLM_OK;
}

int infmllm_decode_n(infmllm_stream_t* s, const void* q, const void* k, const void* v, void* out, int n_tokens)
{
    if (!s) return fail(INFMLLM_EINVAL, "decode: stream is null");
    if (!s->attached) return fail(INFMLLM_ESTATE, "decode: stream has no workspace attached");
    if (s->pending) return fail(INFMLLM_ESTATE, "decode: an eviction is pending on this stream");
    if (!q || !k || !v || !out) return fail(INFMLLM_EINVAL, "decode: q, k, v and out must not be null");
    if (n_tokens < 1) return fail(INFMLLM_EINVAL, "decode: n_tokens must be positive (got %d)", n_tokens);
    if ((int64_t)s->len + n_tokens > (int64_t)s->g.B + s->g.max_decode)
        return fail(INFMLLM_ECAPACITY, "decode: %d cached rows + %d tokens exceed budget + max_decode = %d rows", s->len,
                    n_tokens, s->g.B + s->g.max_decode);
    if (s->streamed + n_tokens > (int64_t)INT32_MAX)
        return fail(INFMLLM_ECAPACITY, "decode: stream positions would exceed 2^31-1");
    const size_t qrow = (size_t)s->g.Hq * s->g.d * s->g.elt, krow = (size_t)s->g.Hkv * s->g.d * s->g.elt;
    for (int i = 0; i < n_tokens; ++i) {
        const int rc = decode_one(s, (const char*)q + i * qrow, (const char*)k + i * krow, (const char*)v + i * krow,
                                  (char*)out + i * qrow);
        if (rc != INFMLLM_OK) return rc;
    }
    return INFMLLM_OK;
}

int infmllm_decode(infmllm_stream_t* s, const void* q, const void* k, const void* v, void* out)
{
    return infmllm_decode_n(s, q, k, v, out, 1);
}

int infmllm_stream_len(const infmllm_stream_t* s) { return s ? s->len : -1; }

int infmllm_stream_max_len(const infmllm_stream_t* s) { return s ? s->g.B + s->g.max_decode : -1; }

int64_t infmllm_stream_streamed(const infmllm_stream_t* s) { return s ? s->streamed : -1; }

static int copy_rows(infmllm_stream* s, void* dst, size_t dpitch, const void* src, size_t spitch, size_t width,
                     const char* what)
{
    if (width == 0) return INFMLLM_OK;
    hipError_t e = hipMemcpy2DAsync(dst, dpitch, src, spitch, width, (size_t)s->g.Hkv, hipMemcpyDeviceToDevice, s->st);
    return e == hipSuccess ? INFMLLM_OK : fail_hip(e, what);
}

int infmllm_stream_positions(infmllm_stream_t* s, int32_t* pos)
{
    if (!s || !pos) return fail(INFMLLM_EINVAL, "positions: null argument");
    if (!s->attached) return fail(INFMLLM_ESTATE, "positions: stream has no workspace attached");
    if (s->pending) return fail(INFMLLM_ESTATE, "positions: an eviction is pending on this stream");
    hipError_t e = launch_export(s->g, s->cache, s->len, nullptr, nullptr, pos, nullptr, s->g.B + s->g.max_decode, s->st);
    return e == hipSuccess ? INFMLLM_OK : fail_hip(e, "positions");
}

int infmllm_stream_export(infmllm_stream_t* s, void* K, void* V, int32_t* pos, float* score)
{
    if (!s) return fail(INFMLLM_EINVAL, "export: stream is null");
    if (!s->attached) return fail(INFMLLM_ESTATE, "export: stream has no workspace attached");
    if (s->pending) return fail(INFMLLM_ESTATE, "export: an eviction is pending on this stream");
    hipError_t e = launch_export(s->g, s->cache, s->len, K, V, pos, score, s->len, s->st);
    return e == hipSuccess ? INFMLLM_OK : fail_hip(e, "export");
}

int infmllm_stream_import(infmllm_stream_t* s, const void* K, const void* V, const int32_t* pos, int len,
                          int64_t streamed)
{
    if (!s) return fail(INFMLLM_EINVAL, "import: stream is null");
    if (!s->attached) return fail(INFMLLM_ESTATE, "import: stream has no workspace attached");
    if (s->pending) return fail(INFMLLM_ESTATE, "import: an eviction is pending on this stream");
    if (len < 0 || len > s->g.B + s->g.max_decode)
        return fail(INFMLLM_EINVAL, "import: len must lie in 0..budget + max_decode (got %d)", len);
    if (len > 0 && (!K || !V || !pos)) return fail(INFMLLM_EINVAL, "import: K, V and pos must not be null");
    if (streamed < len || streamed > (int64_t)INT32_MAX) return fail(INFMLLM_EINVAL, "import: bad streamed count");
    const Geometry& g = s->g;
    const CacheView& c = s->cache;
    const size_t row = (size_t)g.d * g.elt;
    int rc = INFMLLM_OK;
    if (len > 0) {
        rc = copy_rows(s, c.K, g.cap * row, K, len * row, len * row, "import: K");
        if (rc == INFMLLM_OK) rc = copy_rows(s, c.V, g.cap * row, V, len * row, len * row, "import: V");
        if (rc == INFMLLM_OK) rc = copy_rows(s, c.pos, (size_t)g.cap * 4, pos, (size_t)len * 4, (size_t)len * 4, "import: pos");
        if (rc == INFMLLM_OK) {
            // the imported rows are in stream order: physical row = stream-order index
            hipError_t e = launch_reset_tables(g, c, len, s->st);
            if (e != hipSuccess) rc = fail_hip(e, "import: tables");
        }
        if (rc != INFMLLM_OK) return rc;
    }
    s->len = len;
    s->streamed = streamed;
    s->last_cnd = 0;
    s->rot_rows = 0;
    return INFMLLM_OK;
}

int infmllm_stream_last_scores(infmllm_stream_t* s, float* w, int* n_candidates)
{
    if (!s || !n_candidates) return fail(INFMLLM_EINVAL, "last_scores: null argument");
    if (!s->attached) return fail(INFMLLM_ESTATE, "last_scores: stream has no workspace attached");
    if (s->pending) return fail(INFMLLM_ESTATE, "last_scores: an eviction is pending on this stream");
    *n_candidates = s->last_cnd;
    if (s->last_cnd == 0 || !w) return INFMLLM_OK;
    return copy_rows(s, w, (size_t)s->last_cnd * 4, s->Wb, (size_t)s->g.cap * 4, (size_t)s->last_cnd * 4,
                     "last_scores: copy");
}

}  // extern "C"
