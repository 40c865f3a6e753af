/*
 * CPU oracle for error-feedback-compressed distributed AMSGrad.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the HIP
 * library is checked against.  It shares no code with the HIP path and must never
 * be called from it; only tests, the smoke check and the benchmark's CPU-baseline
 * leg may load it.
 *
 * Every function is the definition in the paper written out, in fp32 with one
 * rounding per operation (build with -ffp-contract=off, no fast-math):
 *
 *   error feedback      Section 4, "Error feedback for SGD":
 *                         x_i = g_i + delta_i ; ghat_i = C(x_i) ; delta_i = x_i - ghat_i
 *   Top-k               Appendix A, "Top-k": keep the k coordinates of largest
 *                         magnitude, zero the rest (full sort, ties -> lower index)
 *   scaled sign         Appendix A, "Scaled sign": C(x) = ||x||_1 sign(x) / d,
 *                         applied per contiguous block with the block's own length
 *   server average      Section 3: gbar = (1/n) sum_i ghat_i
 *   AMSGrad             Section 3: m, v, vhat = max(vhat, v), x -= alpha Vhat^{-1/2} m
 *   naive compression   Section 4, "Naive compression": ghat_i = C(g_i), no memory
 *   no compression      Section 3: gbar = (1/n) sum_i g_i (vanilla distributed AMSGrad)
 *   Rand-k              Appendix A, "Rand-k": keep a random set S of k coordinates, drawn
 *                         anew for every (step, worker) by a counter-based generator
 *   CD-Adam             Section 5, Algorithm 1: Markov compression on the workers
 *                         (c_i = C(g_i - ghat_i), ghat_i += c_i), on the server
 *                         (ghat += mean c_i, c = C(ghat - gtilde), gtilde += c),
 *                         AMSGrad on gtilde
 *
 * Readings where the paper is silent are listed next to the code that takes them.
 * Pins: tests/test_oracle_pins.py (all functions here are pinned).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_TOPK = 0, ORACLE_BLOCKSIGN = 1, ORACLE_RANDK = 2 };
/* error feedback (Section 4) / CD-Adam (Algorithm 1) / naive compression (Section 4, first
 * paragraph, with AMSGrad in the place of SGD as in the paper's comparison) / no compression
 * (vanilla distributed AMSGrad, Section 3) */
enum { ORACLE_EF = 0, ORACLE_CD = 1, ORACLE_NAIVE = 2, ORACLE_NONE = 3 };

typedef struct oracle {
    int64_t d;
    int32_t n;
    int32_t compressor;
    int64_t k;          /* Top-k, Rand-k */
    uint64_t seed;      /* Rand-k: the generator's seed ... */
    uint32_t draw;      /* ... and how many steps have drawn from it */
    int32_t n_blocks;   /* block sign */
    int64_t *offsets;   /* n_blocks + 1 */
    float beta1, beta2, eps, lr;
    int32_t eps_mode;   /* 0: m/(sqrt(vhat)+eps)   1: m/sqrt(vhat+eps) */
    float *theta, *m, *v, *vhat; /* d */
    float *e;           /* n*d   error memory delta_i */
    float *c;           /* n*d   compressed vectors ghat_i of the last step */
    float *gbar;        /* d     their average */
    uint32_t *sel;      /* n*k   Top-k: selected indices, ascending, last step */
    float *scales;      /* n*n_blocks  block sign: scale per (worker, block), last step */
    /* CD-Adam (Algorithm 1) only */
    int32_t method;
    float *ghat_w;      /* n*d   ghat_i: Markov sequence of worker i */
    float *ghat_s;      /* d     ghat: the server's aggregate of them */
    float *gtil;        /* d     gtilde: Markov sequence of the aggregate, kept by server and workers */
    float *c_s;         /* d     the server's compressed message of the last step */
    uint32_t *sel_s;    /* k     Top-k: its selected indices */
    float *scales_s;    /* n_blocks  block sign: its scales */
} oracle_t;

/* ---- magnitude key ------------------------------------------------------------
 * Magnitude order is the order of the IEEE-754 bit pattern with the sign bit
 * cleared, read as an unsigned integer.  For finite values this is exactly the
 * order of |x| (Appendix A orders coordinates by |x_(1)| <= ... <= |x_(d)|);
 * +0 and -0 are equal, denormals are kept, Inf > finite, NaN > Inf. */
static uint32_t magnitude_key(float x)
{
    uint32_t u;
    memcpy(&u, &x, sizeof u);
    return u & 0x7fffffffu;
}

static int cmp_u64(const void *a, const void *b)
{
    uint64_t x = *(const uint64_t *)a, y = *(const uint64_t *)b;
    return (x > y) - (x < y);
}

static int cmp_u32(const void *a, const void *b)
{
    uint32_t x = *(const uint32_t *)a, y = *(const uint32_t *)b;
    return (x > y) - (x < y);
}

/* c[j] = x[j] on the k coordinates of largest key and +0.0 elsewhere; among equal keys the
 * coordinate of lower index wins.  sel_out (may be NULL) receives the k selected indices in
 * ascending order.  Method: sort all d (key descending, index ascending) and take the first k. */
static void keep_largest(const uint32_t *key, const float *x, int64_t d, int64_t k, float *c, uint32_t *sel_out)
{
    uint64_t *rec = (uint64_t *)malloc((size_t)d * sizeof *rec);
    for (int64_t j = 0; j < d; ++j) {
        /* ascending order of (inverted key, index) == key descending, index ascending */
        uint64_t inv = (uint64_t)(0xffffffffu - key[j]);
        rec[j] = (inv << 32) | (uint64_t)(uint32_t)j;
    }
    qsort(rec, (size_t)d, sizeof *rec, cmp_u64);
    for (int64_t j = 0; j < d; ++j) c[j] = 0.0f;
    for (int64_t r = 0; r < k; ++r) {
        uint32_t j = (uint32_t)(rec[r] & 0xffffffffu);
        c[j] = x[j];
        if (sel_out) sel_out[r] = j;
    }
    if (sel_out) qsort(sel_out, (size_t)k, sizeof *sel_out, cmp_u32);
    free(rec);
}

/* Top-k (Appendix A): the k coordinates of largest magnitude.  The paper is silent on ties:
 * the coordinate of lower index wins. */
void oracle_topk(const float *x, int64_t d, int64_t k, float *c, uint32_t *sel_out)
{
    uint32_t *key = (uint32_t *)malloc((size_t)d * sizeof *key);
    for (int64_t j = 0; j < d; ++j) key[j] = magnitude_key(x[j]);
    keep_largest(key, x, d, k, c, sel_out);
    free(key);
}

/* ---- Rand-k (Appendix A) ---------------------------------------------------------
 * C(x) = sum_{j in S} x_j e_j for a random S of k coordinates.  The paper does not say how S is
 * drawn.  Reading: every coordinate gets a pseudo-random 31-bit score that depends on
 * (seed, draw, who, j) only - draw counts the steps, who is the worker (n for the server of
 * Algorithm 1) - and S is the k coordinates of largest score, lower index first among equal
 * scores.  For fixed (seed, draw, who) the score is a bijection of the 32-bit index followed by a
 * shift, so at most two coordinates share a score; S does not depend on x.
 * The generator is counter-based (no state is carried from coordinate to coordinate) and built
 * from the 32-bit finaliser of MurmurHash3 (public domain): two xor-shift-multiply rounds. */
uint32_t oracle_mix32(uint32_t h)
{
    h ^= h >> 16;
    h *= 0x85ebca6bu;
    h ^= h >> 13;
    h *= 0xc2b2ae35u;
    h ^= h >> 16;
    return h;
}

uint32_t oracle_randk_score(uint64_t seed, uint32_t draw, uint32_t who, uint32_t j)
{
    const uint32_t per_step = oracle_mix32((uint32_t)seed + draw * 0x9e3779b9u);
    const uint32_t a = oracle_mix32(per_step ^ (uint32_t)(seed >> 32) ^ (who * 0x85ebca6bu));
    const uint32_t b = oracle_mix32(a + 0xc2b2ae35u);
    return oracle_mix32(oracle_mix32(j + a) ^ b) >> 1;
}

void oracle_randk(const float *x, int64_t d, int64_t k, uint64_t seed, uint32_t draw, uint32_t who, float *c,
                  uint32_t *sel_out)
{
    uint32_t *key = (uint32_t *)malloc((size_t)d * sizeof *key);
    for (int64_t j = 0; j < d; ++j) key[j] = oracle_randk_score(seed, draw, who, (uint32_t)j);
    keep_largest(key, x, d, k, c, sel_out);
    free(key);
}

/* Scaled sign (Appendix A) on each contiguous block [off[b], off[b+1]):
 *   s_b = (sum_{j in b} |x_j|) / |b| ,  c_j = s_b * sign(x_j).
 * The sum runs in index order in fp64 and is rounded to fp32 once, after the
 * division.  sign(x) is the IEEE sign bit (so +0 -> +s, -0 -> -s): every entry of
 * C(x) then has magnitude s_b, which is what makes ||C(x)||_1 = ||x||_1. */
void oracle_blocksign(const float *x, const int64_t *off, int32_t n_blocks, float *c, float *scales)
{
    for (int32_t b = 0; b < n_blocks; ++b) {
        double S = 0.0;
        for (int64_t j = off[b]; j < off[b + 1]; ++j) S += (double)fabsf(x[j]);
        float s = (float)(S / (double)(off[b + 1] - off[b]));
        if (scales) scales[b] = s;
        for (int64_t j = off[b]; j < off[b + 1]; ++j) c[j] = copysignf(s, x[j]);
    }
}

/* AMSGrad (Section 3; Algorithm 1, the four update lines) on one coordinate range.
 * No bias correction (the paper has none).  eps_mode 1 is the paper's
 * Vhat = diag(vhat + nu); eps_mode 0 puts the constant outside the root. */
void oracle_amsgrad(float *theta, float *m, float *v, float *vhat, const float *gbar, int64_t d,
                    float beta1, float beta2, float eps, float lr, int32_t eps_mode)
{
    const float omb1 = 1.0f - beta1;
    const float omb2 = 1.0f - beta2;
    for (int64_t j = 0; j < d; ++j) {
        float g = gbar[j];
        float mj = (beta1 * m[j]) + (omb1 * g);
        float vj = (beta2 * v[j]) + (omb2 * (g * g));
        float vh = fmaxf(vhat[j], vj);
        float den = eps_mode ? sqrtf(vh + eps) : (sqrtf(vh) + eps);
        m[j] = mj;
        v[j] = vj;
        vhat[j] = vh;
        theta[j] = theta[j] - (lr * mj) / den;
    }
}

/* ---- stateful optimiser -------------------------------------------------------- */

oracle_t *oracle_create(int64_t d, int32_t n, int32_t compressor, int64_t k_or_block, float beta1,
                        float beta2, float eps, float lr)
{
    oracle_t *o = (oracle_t *)calloc(1, sizeof *o);
    o->d = d;
    o->n = n;
    o->compressor = compressor;
    o->beta1 = beta1;
    o->beta2 = beta2;
    o->eps = eps;
    o->lr = lr;
    o->theta = (float *)calloc((size_t)d, sizeof(float));
    o->m = (float *)calloc((size_t)d, sizeof(float));
    o->v = (float *)calloc((size_t)d, sizeof(float));
    o->vhat = (float *)calloc((size_t)d, sizeof(float));
    o->gbar = (float *)calloc((size_t)d, sizeof(float));
    o->e = (float *)calloc((size_t)n * (size_t)d, sizeof(float));
    o->c = (float *)calloc((size_t)n * (size_t)d, sizeof(float));
    if (compressor == ORACLE_TOPK || compressor == ORACLE_RANDK) {
        o->k = k_or_block;
        o->sel = (uint32_t *)calloc((size_t)n * (size_t)o->k, sizeof(uint32_t));
    } else {
        /* uniform contiguous blocks of length B, the last one partial; a block
         * longer than d is the whole vector */
        int64_t B = k_or_block;
        int64_t nb = (d + B - 1) / B;
        o->n_blocks = (int32_t)nb;
        o->offsets = (int64_t *)malloc((size_t)(nb + 1) * sizeof(int64_t));
        for (int64_t b = 0; b <= nb; ++b) o->offsets[b] = (b * B < d) ? b * B : d;
        o->scales = (float *)calloc((size_t)n * (size_t)nb, sizeof(float));
    }
    return o;
}

void oracle_set_blocks(oracle_t *o, const int64_t *offsets, int32_t n_blocks)
{
    free(o->offsets);
    free(o->scales);
    o->n_blocks = n_blocks;
    o->offsets = (int64_t *)malloc((size_t)(n_blocks + 1) * sizeof(int64_t));
    memcpy(o->offsets, offsets, (size_t)(n_blocks + 1) * sizeof(int64_t));
    o->scales = (float *)calloc((size_t)o->n * (size_t)n_blocks, sizeof(float));
    if (o->method == ORACLE_CD) {
        free(o->scales_s);
        o->scales_s = (float *)calloc((size_t)n_blocks, sizeof(float));
    }
}

/* Selects the method; call before the first step.  CD-Adam starts from ghat_i = C(0) = 0 and
 * gtilde = C(mean ghat_i) = 0 (Algorithm 1, line 1: g_0 = 0, and both compressors map 0 to 0). */
void oracle_set_method(oracle_t *o, int32_t method)
{
    o->method = method;
    if (method != ORACLE_CD || o->ghat_w) return;
    o->ghat_w = (float *)calloc((size_t)o->n * (size_t)o->d, sizeof(float));
    o->ghat_s = (float *)calloc((size_t)o->d, sizeof(float));
    o->gtil = (float *)calloc((size_t)o->d, sizeof(float));
    o->c_s = (float *)calloc((size_t)o->d, sizeof(float));
    if (o->compressor != ORACLE_BLOCKSIGN)
        o->sel_s = (uint32_t *)calloc((size_t)o->k, sizeof(uint32_t));
    else
        o->scales_s = (float *)calloc((size_t)o->n_blocks, sizeof(float));
}

void oracle_set_theta(oracle_t *o, const float *theta) { memcpy(o->theta, theta, (size_t)o->d * sizeof(float)); }
void oracle_set_lr(oracle_t *o, float lr) { o->lr = lr; }
void oracle_set_eps_mode(oracle_t *o, int32_t mode) { o->eps_mode = mode; }
/* Rand-k: the seed, and the number of the next draw (= steps taken so far, for a resumed run) */
void oracle_set_rand(oracle_t *o, uint64_t seed, uint32_t draw)
{
    o->seed = seed;
    o->draw = draw;
}

/* One step on gradients g[n][d] (row-major).  Workers are independent until the
 * average, so the loop over workers may run on several threads; no sum is split
 * across threads, hence the result does not depend on the thread count. */
static void oracle_step_cd(oracle_t *o, const float *g);

void oracle_step(oracle_t *o, const float *g)
{
    const int64_t d = o->d;
    const int32_t n = o->n;
    if (o->method == ORACLE_CD) {
        oracle_step_cd(o, g);
        return;
    }
    const int memory = (o->method == ORACLE_EF);      /* naive compression: delta_i stays 0 */
    const int compress = (o->method != ORACLE_NONE);  /* no compression: ghat_i = g_i */

#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t i = 0; i < n; ++i) {
        float *e = o->e + (size_t)i * (size_t)d;
        float *c = o->c + (size_t)i * (size_t)d;
        const float *gi = g + (size_t)i * (size_t)d;
        if (!compress) {
            memcpy(c, gi, (size_t)d * sizeof(float));
            continue;
        }
        /* x_i = g_i + delta_i, kept in e until the error is written */
        if (memory)
            for (int64_t j = 0; j < d; ++j) e[j] = gi[j] + e[j];
        else
            memcpy(e, gi, (size_t)d * sizeof(float));
        if (o->compressor != ORACLE_BLOCKSIGN) {
            if (o->compressor == ORACLE_TOPK)
                oracle_topk(e, d, o->k, c, o->sel + (size_t)i * (size_t)o->k);
            else
                oracle_randk(e, d, o->k, o->seed, o->draw, (uint32_t)i, c, o->sel + (size_t)i * (size_t)o->k);
            /* delta_i = x_i - C(x_i): +0.0 where selected (x - x), x elsewhere (x - 0) */
            const uint32_t *sel = o->sel + (size_t)i * (size_t)o->k;
            for (int64_t r = 0; r < o->k; ++r) e[sel[r]] = 0.0f;
        } else {
            oracle_blocksign(e, o->offsets, o->n_blocks, c, o->scales + (size_t)i * (size_t)o->n_blocks);
            for (int64_t j = 0; j < d; ++j) e[j] = e[j] - c[j];
        }
        if (!memory) memset(e, 0, (size_t)d * sizeof(float));   /* what was not sent is forgotten */
    }

    /* gbar = (1/n) sum_i ghat_i : fp32 adds in ascending worker order, then one
     * division by n (always n, also where few or no workers contributed) */
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < d; ++j) {
        float acc = 0.0f;
        for (int32_t i = 0; i < n; ++i) acc += o->c[(size_t)i * (size_t)d + (size_t)j];
        o->gbar[j] = acc / (float)n;
    }

    /* worker-side AMSGrad update; all replicas are identical, one is kept */
    const int64_t chunk = 1 << 16;
    const int64_t n_chunks = (d + chunk - 1) / chunk;
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < n_chunks; ++q) {
        int64_t lo = q * chunk, len = (lo + chunk <= d) ? chunk : d - lo;
        oracle_amsgrad(o->theta + lo, o->m + lo, o->v + lo, o->vhat + lo, o->gbar + lo, len, o->beta1,
                       o->beta2, o->eps, o->lr, o->eps_mode);
    }
    o->draw += 1;
}

/* C on one vector with this optimiser's compressor; who: the worker, n for the server. */
static void oracle_compress(oracle_t *o, uint32_t who, const float *x, float *c, uint32_t *sel, float *scales)
{
    if (o->compressor == ORACLE_TOPK)
        oracle_topk(x, o->d, o->k, c, sel);
    else if (o->compressor == ORACLE_RANDK)
        oracle_randk(x, o->d, o->k, o->seed, o->draw, who, c, sel);
    else
        oracle_blocksign(x, o->offsets, o->n_blocks, c, scales);
}

/* One iteration of Algorithm 1 (CD-Adam), in its order.  The same compressor serves both
 * directions.  gbar receives mean_i c_i (what the server adds to ghat). */
static void oracle_step_cd(oracle_t *o, const float *g)
{
    const int64_t d = o->d;
    const int32_t n = o->n;

    /* workers: c_i = C(g_i - ghat_i) ; ghat_i = ghat_i + c_i */
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t i = 0; i < n; ++i) {
        float *gh = o->ghat_w + (size_t)i * (size_t)d;
        float *c = o->c + (size_t)i * (size_t)d;
        float *u = o->e + (size_t)i * (size_t)d;          /* scratch: the vector that is compressed */
        const float *gi = g + (size_t)i * (size_t)d;
        for (int64_t j = 0; j < d; ++j) u[j] = gi[j] - gh[j];
        oracle_compress(o, (uint32_t)i, u, c, o->sel ? o->sel + (size_t)i * (size_t)o->k : NULL,
                        o->scales ? o->scales + (size_t)i * (size_t)o->n_blocks : NULL);
        for (int64_t j = 0; j < d; ++j) gh[j] = gh[j] + c[j];
    }

    /* server: ghat = ghat + (1/n) sum_i c_i  (ascending worker order, one division by n) */
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < d; ++j) {
        float acc = 0.0f;
        for (int32_t i = 0; i < n; ++i) acc += o->c[(size_t)i * (size_t)d + (size_t)j];
        o->gbar[j] = acc / (float)n;
        o->ghat_s[j] = o->ghat_s[j] + o->gbar[j];
    }
    /* server: c = C(ghat - gtilde) ; gtilde = gtilde + c  (workers do the same addition) */
    {
        float *w = (float *)malloc((size_t)d * sizeof(float));
        for (int64_t j = 0; j < d; ++j) w[j] = o->ghat_s[j] - o->gtil[j];
        oracle_compress(o, (uint32_t)n, w, o->c_s, o->sel_s, o->scales_s);
        for (int64_t j = 0; j < d; ++j) o->gtil[j] = o->gtil[j] + o->c_s[j];
        free(w);
    }

    /* workers: AMSGrad with gtilde */
    const int64_t chunk = 1 << 16;
    const int64_t n_chunks = (d + chunk - 1) / chunk;
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < n_chunks; ++q) {
        int64_t lo = q * chunk, len = (lo + chunk <= d) ? chunk : d - lo;
        oracle_amsgrad(o->theta + lo, o->m + lo, o->v + lo, o->vhat + lo, o->gtil + lo, len, o->beta1,
                       o->beta2, o->eps, o->lr, o->eps_mode);
    }
    o->draw += 1;
}

float *oracle_theta(oracle_t *o) { return o->theta; }
float *oracle_m(oracle_t *o) { return o->m; }
float *oracle_v(oracle_t *o) { return o->v; }
float *oracle_vhat(oracle_t *o) { return o->vhat; }
float *oracle_gbar(oracle_t *o) { return o->gbar; }
float *oracle_error(oracle_t *o) { return o->e; }
float *oracle_compressed(oracle_t *o) { return o->c; }
uint32_t *oracle_selected(oracle_t *o) { return o->sel; }
float *oracle_scales(oracle_t *o) { return o->scales; }
int32_t oracle_n_blocks(oracle_t *o) { return o->n_blocks; }
float *oracle_ghat_workers(oracle_t *o) { return o->ghat_w; }
float *oracle_ghat_server(oracle_t *o) { return o->ghat_s; }
float *oracle_gtilde(oracle_t *o) { return o->gtil; }
float *oracle_server_compressed(oracle_t *o) { return o->c_s; }
uint32_t *oracle_server_selected(oracle_t *o) { return o->sel_s; }
float *oracle_server_scales(oracle_t *o) { return o->scales_s; }

void oracle_destroy(oracle_t *o)
{
    if (!o) return;
    free(o->theta); free(o->m); free(o->v); free(o->vhat); free(o->gbar);
    free(o->e); free(o->c); free(o->sel); free(o->scales); free(o->offsets);
    free(o->ghat_w); free(o->ghat_s); free(o->gtil); free(o->c_s); free(o->sel_s); free(o->scales_s);
    free(o);
}
