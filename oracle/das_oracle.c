/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct implementation of the target decoder that the
 * batched speculative verification step of DAS evaluates (the paper, Sec. 3 and
 * Sec. 4.1.2: the target model scores a multi-token draft in one pass and the
 * accepted tokens advance generation; the abstract, Sec. 5.1 and Sec. 6 fix
 * the result: outputs identical to decoding without speculation).  The paper
 * names the model family (Qwen-style decoders, Sec. 3 / Sec. 5) and does not
 * restate the architecture, so the definition written out here is the
 * standard one of that family:
 *
 *   h0 = E[tok]
 *   per layer:  u = RMSNorm(h; g1)
 *               q,k,v = u Wq^T, u Wk^T, u Wv^T           (no biases)
 *               RoPE(q, k) at the row's absolute position (rotate-half pairing)
 *               a = softmax(q k^T / sqrt(D)) v            causal, GQA: q head a
 *                                                         reads KV head a / G
 *               h += a Wo^T
 *               u = RMSNorm(h; g2)
 *               h += (silu(u Wg^T) * (u Wu^T)) Wd^T
 *   logits = RMSNorm(h; gf) Wlm^T
 *
 * Values are fp32; every reduction (dot products, sums of squares, softmax
 * sums) is accumulated in fp64.  KV is kept dense per sequence, in fp32.
 * One function evaluates a block of n consecutive rows of one sequence with a
 * causal mask inside the block; prefill, single-token decoding and draft
 * verification are all calls of it (n = prompt length, 1, 1+k).
 *
 * Only tests, the smoke check and the bench's cpu_baseline leg may use this
 * file.  It shares no code with the HIP library.
 */
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#include <omp.h>

typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float rope_theta, rms_eps;
} orc_config;

typedef struct {
    const float *g1, *wq, *wk, *wv, *wo, *g2, *wg, *wu, *wd;
} orc_layer;

typedef struct {
    orc_config c;
    const float *embed, *gf, *wlm;
    orc_layer *layers;
} orc_model;

typedef struct {
    int32_t cap;     /* positions allocated */
    float *k, *v;    /* [L][cap][Hkv][D] */
} orc_seq;

/* weights: canonical blob order, fp32, borrowed (must outlive the model) */
orc_model *orc_model_create(const orc_config *c, const float *w) {
    orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
    m->c = *c;
    m->layers = (orc_layer *)calloc((size_t)c->n_layers, sizeof(orc_layer));
    const size_t d = c->d_model, qd = (size_t)c->n_q_heads * c->head_dim,
                 kd = (size_t)c->n_kv_heads * c->head_dim, F = c->d_ffn, V = c->vocab;
    const float *p = w;
    m->embed = p; p += V * d;
    for (int l = 0; l < c->n_layers; ++l) {
        orc_layer *y = &m->layers[l];
        y->g1 = p; p += d;
        y->wq = p; p += qd * d;
        y->wk = p; p += kd * d;
        y->wv = p; p += kd * d;
        y->wo = p; p += d * qd;
        y->g2 = p; p += d;
        y->wg = p; p += F * d;
        y->wu = p; p += F * d;
        y->wd = p; p += d * F;
    }
    m->gf = p; p += d;
    m->wlm = p;
    return m;
}

void orc_model_destroy(orc_model *m) { if (m) { free(m->layers); free(m); } }

orc_seq *orc_seq_create(const orc_model *m, int32_t cap) {
    orc_seq *s = (orc_seq *)calloc(1, sizeof(orc_seq));
    size_t n = (size_t)m->c.n_layers * cap * m->c.n_kv_heads * m->c.head_dim;
    s->cap = cap;
    s->k = (float *)calloc(n, sizeof(float));
    s->v = (float *)calloc(n, sizeof(float));
    if (!s->k || !s->v) { free(s->k); free(s->v); free(s); return NULL; }
    return s;
}

void orc_seq_destroy(orc_seq *s) { if (s) { free(s->k); free(s->v); free(s); } }

/* direct access to one layer's dense K or V, [cap][Hkv][D] (tests import synthetic KV through it) */
float *orc_seq_kv(const orc_model *m, orc_seq *s, int32_t layer, int32_t which) {
    size_t per_layer = (size_t)s->cap * m->c.n_kv_heads * m->c.head_dim;
    return (which ? s->v : s->k) + per_layer * layer;
}

int32_t orc_num_threads(void) { return omp_get_max_threads(); }

/* y = x * rsqrt(mean(x^2) + eps) * g */
static void rmsnorm_row(const float *x, const float *g, float eps, int d, float *y) {
    double ss = 0.0;
    for (int i = 0; i < d; ++i) ss += (double)x[i] * (double)x[i];
    const double inv = 1.0 / sqrt(ss / d + (double)eps);
    for (int i = 0; i < d; ++i) y[i] = (float)((double)x[i] * inv * (double)g[i]);
}

static inline double dot_f64(const float *a, const float *b, int n) {
    double acc = 0.0;
#pragma omp simd reduction(+ : acc)
    for (int i = 0; i < n; ++i) acc += (double)a[i] * (double)b[i];
    return acc;
}

/* y[r][o] (+)= sum_i x[r][i] W[o][i];  rows are visited in blocks so x stays cached */
static void linear(const float *x, const float *W, int n, int in, int out, float *y, int accumulate) {
    const int RB = 32;
    for (int r0 = 0; r0 < n; r0 += RB) {
        const int r1 = r0 + RB < n ? r0 + RB : n;
#pragma omp parallel for schedule(static)
        for (int o = 0; o < out; ++o) {
            const float *w = W + (size_t)o * in;
            for (int r = r0; r < r1; ++r) {
                double acc = dot_f64(x + (size_t)r * in, w, in);
                float *dst = y + (size_t)r * out + o;
                *dst = accumulate ? (float)((double)*dst + acc) : (float)acc;
            }
        }
    }
}

/* rotate-half RoPE of one head vector at absolute position pos */
static void rope_head(float *x, int D, int64_t pos, double theta) {
    const int half = D / 2;
    for (int i = 0; i < half; ++i) {
        const double ang = (double)pos * pow(theta, -2.0 * i / D);
        const double c = cos(ang), s = sin(ang);
        const double a = x[i], b = x[i + half];
        x[i] = (float)(a * c - b * s);
        x[i + half] = (float)(b * c + a * s);
    }
}

/*
 * Evaluate rows start_pos .. start_pos+n-1 of one sequence (tokens[n]); row j
 * attends to KV positions 0 .. start_pos+j, of which 0 .. start_pos-1 must
 * already be in the sequence's KV and the rest are written by this call.
 * Logits are produced for rows first_logit_row .. n-1 into
 * logits[(n-first_logit_row)][V].  Returns 0, or -1 on a bad argument.
 */
int orc_forward(const orc_model *m, orc_seq *s, int32_t start_pos, int32_t n, const int32_t *tokens,
                int32_t first_logit_row, float *logits) {
    const orc_config *c = &m->c;
    const int d = c->d_model, Hq = c->n_q_heads, Hkv = c->n_kv_heads, D = c->head_dim, F = c->d_ffn,
              V = c->vocab, G = Hq / Hkv;
    if (D > 512 || n <= 0 || start_pos < 0 || start_pos + n > s->cap || first_logit_row < 0 || first_logit_row > n)
        return -1;
    for (int r = 0; r < n; ++r) if (tokens[r] < 0 || tokens[r] >= V) return -1;
    const size_t qd = (size_t)Hq * D, kd = (size_t)Hkv * D;
    float *h = (float *)malloc(sizeof(float) * (size_t)n * d);
    float *u = (float *)malloc(sizeof(float) * (size_t)n * d);
    float *q = (float *)malloc(sizeof(float) * (size_t)n * qd);
    float *att = (float *)malloc(sizeof(float) * (size_t)n * qd);
    float *gate = (float *)malloc(sizeof(float) * (size_t)n * F);
    float *up = (float *)malloc(sizeof(float) * (size_t)n * F);
    const double scale = 1.0 / sqrt((double)D);

    for (int r = 0; r < n; ++r)
        memcpy(h + (size_t)r * d, m->embed + (size_t)tokens[r] * d, sizeof(float) * d);

    for (int l = 0; l < c->n_layers; ++l) {
        const orc_layer *y = &m->layers[l];
        float *K = s->k + (size_t)l * s->cap * kd, *Vv = s->v + (size_t)l * s->cap * kd;
        for (int r = 0; r < n; ++r) rmsnorm_row(h + (size_t)r * d, y->g1, c->rms_eps, d, u + (size_t)r * d);
        linear(u, y->wq, n, d, (int)qd, q, 0);
        /* K and V rows go straight into the sequence's cache at their positions */
        linear(u, y->wk, n, d, (int)kd, K + (size_t)start_pos * kd, 0);
        linear(u, y->wv, n, d, (int)kd, Vv + (size_t)start_pos * kd, 0);
        for (int r = 0; r < n; ++r) {
            for (int a = 0; a < Hq; ++a) rope_head(q + (size_t)r * qd + (size_t)a * D, D, start_pos + r, c->rope_theta);
            for (int b = 0; b < Hkv; ++b) rope_head(K + (size_t)(start_pos + r) * kd + (size_t)b * D, D, start_pos + r, c->rope_theta);
        }
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
        for (int r = 0; r < n; ++r)
            for (int a = 0; a < Hq; ++a) {
                const int kvh = a / G, last = start_pos + r;   /* causal: positions 0..last */
                const float *qv = q + (size_t)r * qd + (size_t)a * D;
                double *sc = (double *)malloc(sizeof(double) * (size_t)(last + 1));
                double mx = -INFINITY;
                for (int t = 0; t <= last; ++t) {
                    sc[t] = dot_f64(qv, K + (size_t)t * kd + (size_t)kvh * D, D) * scale;
                    if (sc[t] > mx) mx = sc[t];
                }
                double Z = 0.0;
                for (int t = 0; t <= last; ++t) { sc[t] = exp(sc[t] - mx); Z += sc[t]; }
                float *o = att + (size_t)r * qd + (size_t)a * D;
                double acc[512];                               /* head_dim <= 512 */
                for (int e = 0; e < D; ++e) acc[e] = 0.0;
                for (int t = 0; t <= last; ++t) {              /* ascending t for every output */
                    const float *vr = Vv + (size_t)t * kd + (size_t)kvh * D;
                    for (int e = 0; e < D; ++e) acc[e] += sc[t] * (double)vr[e];
                }
                for (int e = 0; e < D; ++e) o[e] = (float)(acc[e] / Z);
                free(sc);
            }
        linear(att, y->wo, n, (int)qd, d, h, 1);
        for (int r = 0; r < n; ++r) rmsnorm_row(h + (size_t)r * d, y->g2, c->rms_eps, d, u + (size_t)r * d);
        linear(u, y->wg, n, d, F, gate, 0);
        linear(u, y->wu, n, d, F, up, 0);
        for (size_t i = 0; i < (size_t)n * F; ++i) {
            const double g = gate[i];
            gate[i] = (float)(g / (1.0 + exp(-g)) * (double)up[i]);   /* silu(g) * up */
        }
        linear(gate, y->wd, n, F, d, h, 1);
    }
    const int nl = n - first_logit_row;
    if (nl > 0) {
        for (int r = 0; r < nl; ++r)
            rmsnorm_row(h + (size_t)(first_logit_row + r) * d, m->gf, c->rms_eps, d, u + (size_t)r * d);
        linear(u, m->wlm, nl, d, V, logits, 0);
    }
    free(h); free(u); free(q); free(att); free(gate); free(up);
    return 0;
}

/* ---- single operations exposed so the pins can probe them one at a time ---- */
void orc_op_rmsnorm(const float *x, const float *g, float eps, int32_t d, float *y) { rmsnorm_row(x, g, eps, d, y); }
void orc_op_rope(float *x, int32_t D, int64_t pos, double theta) { rope_head(x, D, pos, theta); }
void orc_op_linear(const float *x, const float *W, int32_t n, int32_t in, int32_t out, float *y, int32_t acc) {
    linear(x, W, n, in, out, y, acc);
}
