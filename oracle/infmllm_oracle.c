/*
 * Inf-MLLM streaming step: fp64 CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what one
 * streaming step over a size-constrained KV cache computes.  It exists so that the
 * HIP library can be checked against something written directly from the paper.
 * It shares no code with the HIP path, is never linked into it, and must only be
 * called from tests, the smoke check and the benchmark's cpu_baseline leg.
 *
 * What is followed, in the paper's notation (Inf-MLLM, arxiv 2409.09086):
 *   Sec. 3.2  : a prompt of L tokens arrives while t tokens are cached; its queries
 *               attend the t cached keys and the L new keys (n = t + L columns),
 *               giving the L x n attention-weight matrix W (post-softmax).
 *   Alg. 1 l.1: S = (1/l) * sum of rows W[m-l : m, 0 : n-l]      (column mean)
 *   Alg. 1 l.2: d = b / (n-l)
 *   Alg. 1 l.3: D = -[n-l-1, ..., 0] * d
 *   Alg. 1 l.4: W' = S + D                                       (biased score)
 *   Alg. 1 l.5: I_r = Top_k(W', r)
 *   Alg. 1 l.6: I_l = the last l columns
 *   Alg. 1 l.7: I = [I_r, I_l]
 *   Alg. 1 l.8: K_s, V_s = K[I,:], V[I,:]
 *
 * Readings taken where the paper is silent or ambiguous (each is listed in the
 * repository's design notes as well):
 *   - attention score = softmax probability (Sec. 3.3 speaks of scores summing to one).
 *   - two windows are told apart: R = number of most recent keys always kept
 *     (Alg. 1's l on the column side) and l_q = min(R, L) = number of last query rows
 *     that are averaged (Alg. 1's l on the row side).  R = l_q whenever R <= L.
 *   - scores are not carried from one step to the next (Alg. 1 has no such state).
 *   - one selection per kv-head; with grouped queries the G = Hq/Hkv query heads of a
 *     group are pooled by their mean.
 *   - I_r is put in ascending order, so the cache always stays in stream order.
 *   - I_l is the half-open range [n-R, n): R entries (Alg. 1 l.7 says r + l in all).
 *   - ties in W' go to the newer slot (larger index).
 *   - cached keys are all visible; inside the chunk attention is causal.
 *   - while n <= B nothing is evicted.
 *   - the chunk's attention output uses the cache before eviction.
 *
 * Comparison policies (Sec. 2 "KV cache eviction", Sec. 4.1 baselines), selectable with
 * oracle_set_policy; each only replaces the score W' that Alg. 1 l.5 ranks:
 *   1 window          : W'[j] = j            -> the cache is the newest B tokens
 *   2 initial + recent: W'[j] = -j           -> the r oldest cached tokens and the R newest
 *   3 cumulative      : W'[j] = A[j] + S[j]  -> A[j] = sum of S over the earlier steps in which
 *                       row j was a candidate (0 for a row never scored); no attention bias;
 *                       the retained rows carry W' on as their A.
 *   Reading: the paper names these methods without formulas; the three rules above are the
 *   plain statements of "keep recent", "keep initial and recent" and "keep the heaviest by
 *   accumulated attention" inside this step's (r, R) frame.
 *
 * Cache-relative position encoding (Sec. 3.4 "length extrapolation", Sec. 4.1: the models use
 * rotary position embeddings), selectable with oracle_set_rope; off by default:
 *   Reading: the paper states no formula.  Taken here: keys and values are cached as given
 *   (unrotated); whenever attention is computed, the key in cache row j is rotated by the angle
 *   of position j and the query of chunk row i by that of position t + i (the row its own key
 *   occupies), so that relative distances are distances inside the cache and never exceed its
 *   size.  Rotation: pairs (x[i], x[i + d/2]), angle p * base^(-2i/d), i < d/2 (the half-split
 *   form of rotary embeddings).  A model applies its rotary embedding to the projected q and k
 *   tensors and stores the result in the model's element type before the attention product
 *   (that is what "q and k arrive in the stream's dtype" means once the rotation is part of
 *   the step), so with oracle_set_rope(..., round_to = bf16 | fp32) the rotated values are
 *   rounded once, to nearest even, to that type; round_to = none keeps them exact, which is
 *   the mathematical statement of the same reading and the reference for how much that
 *   rounding can move a result.
 *
 * All arithmetic is IEEE double.  Inputs are taken as exact values (a bf16 or fp32
 * input converts to double without rounding).
 *
 * parity pins: see tests/test_oracle_pins.py (every function here is pinned).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* threads the head-parallel loop of oracle_attend will use */
int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

typedef struct oracle_stream {
    int B;        /* cache budget (r + R)                                 */
    int R;        /* recent window, key side                              */
    int Hq;       /* query heads                                          */
    int Hkv;      /* key/value heads                                      */
    int dh;       /* head dimension                                       */
    double b;     /* attention bias, Alg. 1 input                         */
    double scale; /* softmax scale applied to q.k                         */
    int t;        /* tokens now cached                                    */
    int64_t T;    /* tokens streamed so far (next stream position)        */
    int cap;      /* rows allocated per kv-head                           */
    double *K;    /* [Hkv][cap][dh]                                       */
    double *V;    /* [Hkv][cap][dh]                                       */
    int64_t *pos; /* [Hkv][cap] stream position of each cached row        */
    /* step in flight: set by oracle_attend, consumed by select/commit    */
    int pending;  /* 1 between attend and commit                          */
    int n;        /* t + L of the step in flight                          */
    int L;
    int evict;    /* n > B                                                */
    double *S;    /* [Hkv][cap] column mean, first c = n - R entries used */
    double *Wb;   /* [Hkv][cap] biased score                              */
    int policy;   /* 0 Alg. 1, 1 window, 2 initial + recent, 3 cumulative */
    double rope_base;   /* 0 = no position encoding                        */
    int rope_round;     /* rotated values rounded to: 0 nothing, 1 bf16, 2 fp32 */
    double *A;    /* [Hkv][cap] accumulated score of each cached row      */
} oracle_stream;

static int grow(oracle_stream *s, int need)
{
    if (need <= s->cap) return 0;
    int ncap = need;
    size_t row = (size_t)s->dh;
    double *K = (double *)calloc((size_t)s->Hkv * ncap * row, sizeof(double));
    double *V = (double *)calloc((size_t)s->Hkv * ncap * row, sizeof(double));
    int64_t *pos = (int64_t *)calloc((size_t)s->Hkv * ncap, sizeof(int64_t));
    double *S = (double *)calloc((size_t)s->Hkv * ncap, sizeof(double));
    double *Wb = (double *)calloc((size_t)s->Hkv * ncap, sizeof(double));
    double *A = (double *)calloc((size_t)s->Hkv * ncap, sizeof(double));
    if (!K || !V || !pos || !S || !Wb || !A) {
        free(K); free(V); free(pos); free(S); free(Wb); free(A);
        return -1;
    }
    for (int h = 0; h < s->Hkv; ++h) {
        if (s->t > 0) {
            memcpy(K + (size_t)h * ncap * row, s->K + (size_t)h * s->cap * row, (size_t)s->t * row * sizeof(double));
            memcpy(V + (size_t)h * ncap * row, s->V + (size_t)h * s->cap * row, (size_t)s->t * row * sizeof(double));
            memcpy(pos + (size_t)h * ncap, s->pos + (size_t)h * s->cap, (size_t)s->t * sizeof(int64_t));
            memcpy(A + (size_t)h * ncap, s->A + (size_t)h * s->cap, (size_t)s->t * sizeof(double));
        }
    }
    free(s->K); free(s->V); free(s->pos); free(s->S); free(s->Wb); free(s->A);
    s->K = K; s->V = V; s->pos = pos; s->S = S; s->Wb = Wb; s->A = A; s->cap = ncap;
    return 0;
}

oracle_stream *oracle_create(int budget, int recent, int heads, int kv_heads, int head_dim,
                             double bias, double scale)
{
    if (budget <= 0 || recent < 0 || recent > budget || heads <= 0 || kv_heads <= 0 ||
        heads % kv_heads != 0 || head_dim <= 0)
        return NULL;
    oracle_stream *s = (oracle_stream *)calloc(1, sizeof(oracle_stream));
    if (!s) return NULL;
    s->B = budget; s->R = recent; s->Hq = heads; s->Hkv = kv_heads; s->dh = head_dim;
    s->b = bias; s->scale = scale;
    return s;
}

void oracle_destroy(oracle_stream *s)
{
    if (!s) return;
    free(s->K); free(s->V); free(s->pos); free(s->S); free(s->Wb); free(s->A);
    free(s);
}

/* selects the score that Alg. 1 l.5 ranks (see the header); only between steps */
int oracle_set_policy(oracle_stream *s, int policy)
{
    if (!s || s->pending || policy < 0 || policy > 3) return -1;
    s->policy = policy;
    return 0;
}

/* cache-relative rotary encoding (see the header); round_to: 0 none, 1 bf16, 2 fp32; only between steps */
int oracle_set_rope(oracle_stream *s, double base, int round_to)
{
    if (!s || s->pending || !(base == 0.0 || base > 1.0) || round_to < 0 || round_to > 2) return -1;
    if (base > 0.0 && (s->dh & 1)) return -1;     /* the rotation pairs x[i] with x[i + d/2] */
    s->rope_base = base;
    s->rope_round = round_to;
    return 0;
}

static double round_to_type(double v, int round_to)
{
    if (round_to == 0) return v;
    float f = (float)v;                            /* IEEE round to nearest even */
    if (round_to == 2) return (double)f;
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7fffu + ((u >> 16) & 1u);               /* bf16: nearest even on the upper 16 bits */
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* y = x rotated to position p: (x[i], x[i + d/2]) turned by p * base^(-2i/d), then rounded */
static void rotate_row(const oracle_stream *s, const double *x, int p, double *y)
{
    const int half = s->dh / 2;
    for (int i = 0; i < half; ++i) {
        const double ang = (double)p * pow(s->rope_base, -2.0 * (double)i / (double)s->dh);
        const double c = cos(ang), sn = sin(ang);
        y[i] = round_to_type(x[i] * c - x[i + half] * sn, s->rope_round);
        y[i + half] = round_to_type(x[i + half] * c + x[i] * sn, s->rope_round);
    }
}

int oracle_len(const oracle_stream *s) { return s->t; }
int64_t oracle_streamed(const oracle_stream *s) { return s->T; }

/*
 * Sec. 3.2, first paragraph: store the prompt's K/V after the t cached rows, then
 * let the L new queries attend all n = t + L keys.  Row i of the chunk sees columns
 * 0 .. t+i.  W (L x n, row-major, zero where masked) receives the softmax weights of
 * one query head; out_g receives sum_j W[i][j] * V[j].
 */
static void attention_one_head(const oracle_stream *s, int g, const double *q, int L,
                               double *W, double *out)
{
    const int dh = s->dh, n = s->n, t = s->t;      /* t = cached before this step */
    const int h = g / (s->Hq / s->Hkv);
    const double *K = s->K + (size_t)h * s->cap * dh;
    const double *V = s->V + (size_t)h * s->cap * dh;
    double *Kr = NULL, *qr = NULL;                 /* rotated copies when the position encoding is on */
    if (s->rope_base > 0.0) {
        Kr = (double *)malloc((size_t)n * dh * sizeof(double));
        qr = (double *)malloc((size_t)dh * sizeof(double));
        for (int j = 0; j < n; ++j) rotate_row(s, K + (size_t)j * dh, j, Kr + (size_t)j * dh);
        K = Kr;
    }
    for (int i = 0; i < L; ++i) {
        const double *qi = q + ((size_t)i * s->Hq + g) * dh;
        if (qr) { rotate_row(s, qi, t + i, qr); qi = qr; }
        double *Wi = W + (size_t)i * n;
        const int vis = t + i + 1;                 /* visible columns 0 .. t+i */
        double mx = -INFINITY;
        for (int j = 0; j < vis; ++j) {
            const double *kj = K + (size_t)j * dh;
            double acc = 0.0;
            for (int x = 0; x < dh; ++x) acc += qi[x] * kj[x];
            Wi[j] = s->scale * acc;
            if (Wi[j] > mx) mx = Wi[j];
        }
        double Z = 0.0;
        for (int j = 0; j < vis; ++j) { Wi[j] = exp(Wi[j] - mx); Z += Wi[j]; }
        for (int j = 0; j < vis; ++j) Wi[j] /= Z;
        for (int j = vis; j < n; ++j) Wi[j] = 0.0;
        double *oi = out + ((size_t)i * s->Hq + g) * dh;
        for (int x = 0; x < dh; ++x) oi[x] = 0.0;
        for (int j = 0; j < vis; ++j) {
            const double *vj = V + (size_t)j * dh;
            const double w = Wi[j];
            for (int x = 0; x < dh; ++x) oi[x] += w * vj[x];
        }
    }
    free(Kr);
    free(qr);
}

/*
 * One prompt arrival up to and including the biased score (Sec. 3.2, Sec. 3.3,
 * Alg. 1 l.1-4).  q is [L][Hq][dh], k and v are [L][Hkv][dh], out is [L][Hq][dh].
 * Returns n = t + L, or a negative value on error.  The cache holds all n rows
 * afterwards; oracle_select / oracle_commit finish the step.
 */
int oracle_attend(oracle_stream *s, const double *q, const double *k, const double *v,
                  int L, double *out)
{
    if (!s || !q || !k || !v || !out || L <= 0 || s->pending) return -1;
    const int dh = s->dh, t = s->t, n = t + L;
    if (grow(s, n) != 0) return -2;

    /* append: rows t .. n-1 of every kv-head, stream positions T .. T+L-1 */
    for (int h = 0; h < s->Hkv; ++h) {
        for (int i = 0; i < L; ++i) {
            memcpy(s->K + ((size_t)h * s->cap + t + i) * dh, k + ((size_t)i * s->Hkv + h) * dh, dh * sizeof(double));
            memcpy(s->V + ((size_t)h * s->cap + t + i) * dh, v + ((size_t)i * s->Hkv + h) * dh, dh * sizeof(double));
            s->pos[(size_t)h * s->cap + t + i] = s->T + i;
            s->A[(size_t)h * s->cap + t + i] = 0.0;
        }
    }
    s->n = n; s->L = L; s->evict = (n > s->B);

    const int G = s->Hq / s->Hkv;
    const int c = n - s->R;                           /* candidate columns, Alg. 1: n - l   */
    const int lq = s->R < L ? s->R : L;               /* rows averaged,     Alg. 1: l       */
    double *Sg = NULL;                                /* per query head column mean [Hq][c] */
    if (s->evict) {
        Sg = (double *)calloc((size_t)s->Hq * (c > 0 ? c : 1), sizeof(double));
        if (!Sg) return -2;
    }
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int g = 0; g < s->Hq; ++g) {
        double *W = (double *)malloc((size_t)L * n * sizeof(double));
        if (!W) {
#pragma omp atomic write
            fail = 1;
            continue;
        }
        attention_one_head(s, g, q, L, W, out);
        if (s->evict && lq > 0) {
            /* Alg. 1 l.1: S = (1/l) sum_{i = m-l}^{m-1} W[i, 0 : n-l] */
            for (int j = 0; j < c; ++j) {
                double acc = 0.0;
                for (int i = L - lq; i < L; ++i) acc += W[(size_t)i * n + j];
                Sg[(size_t)g * c + j] = acc / (double)lq;
            }
        }
        free(W);
    }
    if (fail) { free(Sg); return -2; }

    if (s->evict) {
        const double d = s->b / (double)c;            /* Alg. 1 l.2 */
        for (int h = 0; h < s->Hkv; ++h) {
            double *S = s->S + (size_t)h * s->cap;
            double *Wb = s->Wb + (size_t)h * s->cap;
            for (int j = 0; j < c; ++j) {
                double acc = 0.0;                     /* mean over the group's query heads */
                for (int gg = 0; gg < G; ++gg) acc += Sg[(size_t)(h * G + gg) * c + j];
                S[j] = acc / (double)G;
                const double D = -(double)(c - 1 - j) * d;   /* Alg. 1 l.3 */
                Wb[j] = S[j] + D;                            /* Alg. 1 l.4 */
                if (s->policy == 1) Wb[j] = (double)j;                            /* newest first */
                if (s->policy == 2) Wb[j] = -(double)j;                           /* oldest first */
                if (s->policy == 3) Wb[j] = s->A[(size_t)h * s->cap + j] + S[j];  /* heaviest first */
            }
        }
        free(Sg);
    }
    s->T += L;
    s->t = n;          /* all n rows are cached until commit */
    s->pending = 1;
    return n;
}

/*
 * One decoding step (Sec. 3.2, last paragraph: the eviction runs when a prompt arrives, not while
 * tokens are decoded).  The new token's k, v ([1][Hkv][dh]) are appended, its query ([1][Hq][dh])
 * attends all t + 1 keys, and nothing is evicted: the cache may grow past B until the next prompt.
 * Returns the new cache length, or a negative value on error.
 */
int oracle_decode(oracle_stream *s, const double *q, const double *k, const double *v, double *out)
{
    if (!s || !q || !k || !v || !out || s->pending) return -1;
    const int dh = s->dh, t = s->t, n = t + 1;
    if (grow(s, n) != 0) return -2;
    for (int h = 0; h < s->Hkv; ++h) {
        memcpy(s->K + ((size_t)h * s->cap + t) * dh, k + (size_t)h * dh, dh * sizeof(double));
        memcpy(s->V + ((size_t)h * s->cap + t) * dh, v + (size_t)h * dh, dh * sizeof(double));
        s->pos[(size_t)h * s->cap + t] = s->T;
        s->A[(size_t)h * s->cap + t] = 0.0;
    }
    s->n = n;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int g = 0; g < s->Hq; ++g) {
        double *W = (double *)malloc((size_t)n * sizeof(double));      /* the 1 x n weight row */
        if (!W) {
#pragma omp atomic write
            fail = 1;
            continue;
        }
        attention_one_head(s, g, q, 1, W, out);
        free(W);
    }
    if (fail) return -2;
    s->T += 1;
    s->t = n;
    return n;
}

/* number of candidate columns c = n - R of the step in flight (0 if it does not evict) */
int oracle_candidates(const oracle_stream *s)
{
    return (s->pending && s->evict) ? s->n - s->R : 0;
}

/* copies S and W' ([Hkv][c] each, either may be NULL) of the step in flight */
int oracle_scores(const oracle_stream *s, double *S, double *Wb)
{
    if (!s->pending || !s->evict) return -1;
    const int c = s->n - s->R;
    for (int h = 0; h < s->Hkv; ++h) {
        if (S) memcpy(S + (size_t)h * c, s->S + (size_t)h * s->cap, (size_t)c * sizeof(double));
        if (Wb) memcpy(Wb + (size_t)h * c, s->Wb + (size_t)h * s->cap, (size_t)c * sizeof(double));
    }
    return c;
}

typedef struct { double w; int j; } scored;

static int by_score_desc_then_newer(const void *a, const void *b)
{
    const scored *x = (const scored *)a, *y = (const scored *)b;
    if (x->w > y->w) return -1;
    if (x->w < y->w) return 1;
    return (x->j > y->j) ? -1 : (x->j < y->j);
}

static int by_index_asc(const void *a, const void *b)
{
    return *(const int *)a - *(const int *)b;
}

/*
 * Alg. 1 l.5-7 for every kv-head of the step in flight.  I is [Hkv][B] (int32);
 * the first `count` entries of each row are written.  Returns count = min(n, B).
 */
int oracle_select(const oracle_stream *s, int32_t *I)
{
    if (!s || !I || !s->pending) return -1;
    const int n = s->n;
    if (!s->evict) {
        for (int h = 0; h < s->Hkv; ++h)
            for (int j = 0; j < n; ++j) I[(size_t)h * s->B + j] = j;
        return n;
    }
    const int c = n - s->R, r = s->B - s->R;
    scored *tmp = (scored *)malloc((size_t)(c > 0 ? c : 1) * sizeof(scored));
    if (!tmp) return -2;
    for (int h = 0; h < s->Hkv; ++h) {
        const double *Wb = s->Wb + (size_t)h * s->cap;
        int32_t *Ih = I + (size_t)h * s->B;
        for (int j = 0; j < c; ++j) { tmp[j].w = Wb[j]; tmp[j].j = j; }
        qsort(tmp, (size_t)c, sizeof(scored), by_score_desc_then_newer);   /* Top_k: r best first */
        for (int x = 0; x < r; ++x) Ih[x] = tmp[x].j;                       /* I_r */
        qsort(Ih, (size_t)r, sizeof(int32_t), by_index_asc);                /* keep stream order */
        for (int x = 0; x < s->R; ++x) Ih[r + x] = c + x;                   /* I_l = [n-R, n) */
    }
    free(tmp);
    return s->B;
}

/*
 * Alg. 1 l.8: K_s, V_s = K[I,:], V[I,:] (and the stream positions with them).
 * I is [Hkv][B]; the first `count` entries of each row must be strictly ascending
 * indices into the n rows now cached.  Ends the step in flight.
 */
int oracle_commit(oracle_stream *s, const int32_t *I, int count)
{
    if (!s || !I || !s->pending || count <= 0 || count > s->B || count > s->n) return -1;
    const int dh = s->dh;
    for (int h = 0; h < s->Hkv; ++h) {
        const int32_t *Ih = I + (size_t)h * s->B;
        for (int x = 0; x < count; ++x) {
            if (Ih[x] < 0 || Ih[x] >= s->n) return -3;
            if (x > 0 && Ih[x] <= Ih[x - 1]) return -3;
        }
    }
    for (int h = 0; h < s->Hkv; ++h) {
        const int32_t *Ih = I + (size_t)h * s->B;
        double *K = s->K + (size_t)h * s->cap * dh;
        double *V = s->V + (size_t)h * s->cap * dh;
        int64_t *pos = s->pos + (size_t)h * s->cap;
        double *A = s->A + (size_t)h * s->cap;
        const double *Wb = s->Wb + (size_t)h * s->cap;
        const int c = s->n - s->R;
        for (int x = 0; x < count; ++x) {          /* ascending and I[x] >= x: a forward move is safe */
            const int src = Ih[x];
            if (src != x) {
                memmove(K + (size_t)x * dh, K + (size_t)src * dh, dh * sizeof(double));
                memmove(V + (size_t)x * dh, V + (size_t)src * dh, dh * sizeof(double));
                pos[x] = pos[src];
            }
            /* cumulative policy: a row that was ranked carries its new total, the others keep theirs */
            if (s->policy == 3 && s->evict) A[x] = (src < c) ? Wb[src] : A[src];
            else A[x] = A[src];
        }
    }
    s->t = count;
    s->pending = 0;
    return 0;
}

/* accumulated scores of the cached rows, [Hkv][t] (cumulative policy; all zero otherwise) */
int oracle_accumulated(const oracle_stream *s, double *A)
{
    for (int h = 0; h < s->Hkv; ++h)
        memcpy(A + (size_t)h * s->t, s->A + (size_t)h * s->cap, (size_t)s->t * sizeof(double));
    return s->t;
}

/* copies the cache out: K, V are [Hkv][t][dh], pos is [Hkv][t]; any may be NULL */
int oracle_export(const oracle_stream *s, double *K, double *V, int64_t *pos)
{
    const int dh = s->dh, t = s->t;
    for (int h = 0; h < s->Hkv; ++h) {
        if (K) memcpy(K + (size_t)h * t * dh, s->K + (size_t)h * s->cap * dh, (size_t)t * dh * sizeof(double));
        if (V) memcpy(V + (size_t)h * t * dh, s->V + (size_t)h * s->cap * dh, (size_t)t * dh * sizeof(double));
        if (pos) memcpy(pos + (size_t)h * t, s->pos + (size_t)h * s->cap, (size_t)t * sizeof(int64_t));
    }
    return t;
}

/* replaces the cache: K, V are [Hkv][len][dh], pos is [Hkv][len]; streamed = next stream position */
int oracle_import(oracle_stream *s, const double *K, const double *V, const int64_t *pos,
                  int len, int64_t streamed)
{
    if (!s || s->pending || len < 0 || len > s->B || (len > 0 && (!K || !V || !pos))) return -1;
    s->t = 0;
    if (grow(s, len > 0 ? len : 1) != 0) return -2;
    const int dh = s->dh;
    for (int h = 0; h < s->Hkv; ++h) {
        memcpy(s->K + (size_t)h * s->cap * dh, K + (size_t)h * len * dh, (size_t)len * dh * sizeof(double));
        memcpy(s->V + (size_t)h * s->cap * dh, V + (size_t)h * len * dh, (size_t)len * dh * sizeof(double));
        memcpy(s->pos + (size_t)h * s->cap, pos + (size_t)h * len, (size_t)len * sizeof(int64_t));
        memset(s->A + (size_t)h * s->cap, 0, (size_t)len * sizeof(double));
    }
    s->t = len;
    s->T = streamed;
    return 0;
}
