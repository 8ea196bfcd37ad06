/*
 * CPU oracle for the verify pass of speculative sampling with KV caching.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the hot path
 * computes.  Only the test-suite, the smoke check and the bench's cpu_baseline leg may call it;
 * the GPU library never does, and the two share no code.
 *
 * What it follows (paper sections):
 *   - Section 3, Eq. (1): autoregressive sampling p(x_{n+1} | x_1..x_n), token by argmax or sampling.
 *   - Sections 2 and 4.2: KV caching - per-token keys/values are stored once and reused.
 *   - Sections 3 and 4.3: speculative sampling - a draft model proposes K tokens, the target model
 *     scores them in one K+1-row pass and accepts or rejects them so that the target distribution
 *     is recovered (the rule of Chen et al. that Section 3 credits: accept with probability
 *     min(1, p/q); on the first rejection resample from norm(max(0, p - q)); bonus token from
 *     the last row when nothing was rejected).
 *   - Section 4.4: two caches of different size; truncation of the stale tail is a length write.
 *   - Sections 2 and 3 assume a quantised model without fixing the precision.  The reading taken here:
 *     weight-only int8 with one scale per output row (orc_quantize_rows_int8), activations untouched;
 *     a quantised matrix stands for the real numbers scale_n * q[n][k].
 *
 * The paper names no architecture beyond a Llama-2 model id (Section 4.1), so the decoder is the
 * Llama-style one of the synthetic workloads: RMSNorm -> QKV -> rotary embedding (split-half
 * pairing) -> causal attention over the cache -> O projection + residual -> RMSNorm ->
 * SwiGLU FFN + residual; final RMSNorm -> LM head.  No biases, untied embedding, MHA.
 *
 * Precision: activations are fp32; every dot product, sum and transcendental is evaluated in fp64
 * in a fixed sequential order and rounded once to fp32; each output row is computed on its own,
 * so a result never depends on how many rows share a call.  With bf16 storage the only roundings
 * to bf16 (nearest-even) are the ones storage mandates: weights (given as bf16) and KV entries.
 *
 * Parity pins: every exported function is pinned by tests/test_oracle_*.py (library routines,
 * closed forms, invariants, brute force); none is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ storage types */

static inline float bf16_to_f32(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round-to-nearest-even fp32 -> bf16 (NaN kept quiet) */
uint16_t orc_f32_to_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

float orc_bf16_to_f32(uint16_t b) { return bf16_to_f32(b); }

/* element idx of a weight / cache array held in the storage type */
static inline double st_get(const void *a, int is_bf16, size_t idx) {
    return is_bf16 ? (double)bf16_to_f32(((const uint16_t *)a)[idx]) : (double)((const float *)a)[idx];
}

static inline void st_put(void *a, int is_bf16, size_t idx, float v) {
    if (is_bf16) ((uint16_t *)a)[idx] = orc_f32_to_bf16(v);
    else ((float *)a)[idx] = v;
}

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
/* How many threads the row loops may use from now on (timing on one core; no result depends on it: every output
 * row is computed by one thread, in the same order). */
void orc_set_num_threads(int n) {
#ifdef _OPENMP
    omp_set_num_threads(n < 1 ? 1 : n);
#else
    (void)n;
#endif
}

/* ------------------------------------------------------------------ decoder pieces */

/* RMSNorm: out_i = x_i * g_i / sqrt(mean(x^2) + eps) */
void orc_rmsnorm(const float *x, const float *g, int n, double eps, float *out) {
    double ss = 0.0;
    for (int i = 0; i < n; ++i) ss += (double)x[i] * (double)x[i];
    double r = 1.0 / sqrt(ss / (double)n + eps);
    for (int i = 0; i < n; ++i) out[i] = (float)((double)x[i] * r * (double)g[i]);
}

/* y_n = sum_k W[n][k] x_k, W row-major [N][K] in the storage type ("linear layers", Section 3) */
void orc_linear(const void *W, int is_bf16, const float *x, int N, int K, float *y) {
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        double acc = 0.0;
        size_t base = (size_t)n * (size_t)K;
        for (int k = 0; k < K; ++k) acc += st_get(W, is_bf16, base + k) * (double)x[k];
        y[n] = (float)acc;
    }
}

/* Weight-only int8 (the reading of the paper's "quantized model", Sections 2 and 3): row n of a matrix
 * becomes q[n][k] in [-127, 127] and one fp32 scale, s_n = fl32(max_k |w[n][k]| / 127) (1 for an all-zero
 * row) and q[n][k] = nearest integer (ties to even) of fl32(w[n][k] / s_n); every step is a single fp32
 * operation, so any IEEE implementation produces the same bytes.  W is in the storage type. */
void orc_quantize_rows_int8(const void *W, int is_bf16, int N, int K, int8_t *q, float *scale) {
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        size_t base = (size_t)n * (size_t)K;
        float amax = 0.0f;
        for (int k = 0; k < K; ++k) {
            float a = fabsf((float)st_get(W, is_bf16, base + k));
            if (a > amax) amax = a;
        }
        volatile float sv = amax > 0.0f ? amax / 127.0f : 1.0f; /* volatile: one rounding to fp32, no wider temporaries */
        float sc = sv;
        scale[n] = sc;
        for (int k = 0; k < K; ++k) {
            volatile float r = (float)st_get(W, is_bf16, base + k) / sc;
            float t = rintf(r); /* default rounding mode: nearest, ties to even */
            if (t > 127.0f) t = 127.0f;
            if (t < -127.0f) t = -127.0f;
            q[base + k] = (int8_t)t;
        }
    }
}

/* Weight-only int4 with group scales (the second, coarser reading of the same "quantized model"): along K, groups of
 * `group` consecutive entries of a row share one fp32 scale, s = fl32(max |w| / 7) over the group (1 for an all-zero
 * group), and q = nearest integer (ties to even) of fl32(w / s), clamped to [-7, 7].  Packing: byte b of a row holds
 * entry 2b in its low and entry 2b+1 in its high four bits (two's complement); scales are stored group-major,
 * scale[j][n] for group j of row n.  K must be a multiple of `group`, `group` even. */
void orc_quantize_rows_int4(const void *W, int is_bf16, int N, int K, int group, uint8_t *q, float *scale) {
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        size_t base = (size_t)n * (size_t)K;
        for (int j = 0; j < K / group; ++j) {
            float amax = 0.0f;
            for (int k = j * group; k < (j + 1) * group; ++k) {
                float a = fabsf((float)st_get(W, is_bf16, base + k));
                if (a > amax) amax = a;
            }
            volatile float sv = amax > 0.0f ? amax / 7.0f : 1.0f;
            float sc = sv;
            scale[(size_t)j * (size_t)N + n] = sc;
            for (int k = j * group; k < (j + 1) * group; ++k) {
                volatile float r = (float)st_get(W, is_bf16, base + k) / sc;
                float t = rintf(r);
                if (t > 7.0f) t = 7.0f;
                if (t < -7.0f) t = -7.0f;
                uint8_t nib = (uint8_t)((int)t & 0xf);
                uint8_t *byte = &q[(base + k) / 2];
                if (k & 1) *byte = (uint8_t)((*byte & 0x0f) | (nib << 4));
                else *byte = (uint8_t)((*byte & 0xf0) | nib);
            }
        }
    }
}

static inline int nibble_at(const uint8_t *q, size_t idx) {
    int v = (q[idx / 2] >> ((idx & 1) ? 4 : 0)) & 0xf;
    return v >= 8 ? v - 16 : v;
}

/* y_n = sum_j scale[j][n] * sum_{k in group j} q[n][k] x_k */
void orc_linear_w4(const uint8_t *q, const float *scale, const float *x, int N, int K, int group, float *y) {
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        double acc = 0.0;
        size_t base = (size_t)n * (size_t)K;
        for (int j = 0; j < K / group; ++j) {
            double part = 0.0;
            for (int k = j * group; k < (j + 1) * group; ++k) part += (double)nibble_at(q, base + k) * (double)x[k];
            acc += (double)scale[(size_t)j * (size_t)N + n] * part;
        }
        y[n] = (float)acc;
    }
}

/* y_n = scale_n * sum_k q[n][k] x_k: the linear layer of a weight-only int8 matrix */
void orc_linear_w8(const int8_t *q, const float *scale, const float *x, int N, int K, float *y) {
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        double acc = 0.0;
        size_t base = (size_t)n * (size_t)K;
        for (int k = 0; k < K; ++k) acc += (double)q[base + k] * (double)x[k];
        y[n] = (float)((double)scale[n] * acc);
    }
}

/* Rotary embedding of one head vector at absolute position pos, split-half pairing:
 * (v_j, v_{j+hd/2}) rotated by angle pos * base^(-2j/hd), j = 0..hd/2-1. */
void orc_rope(float *v, int hd, int64_t pos, double base) {
    int half = hd / 2;
    for (int j = 0; j < half; ++j) {
        double ang = (double)pos * pow(base, -2.0 * (double)j / (double)hd);
        double c = cos(ang), s = sin(ang);
        double a = v[j], b = v[j + half];
        v[j] = (float)(a * c - b * s);
        v[j + half] = (float)(a * s + b * c);
    }
}

static inline double silu(double x) { return x / (1.0 + exp(-x)); }

/* softmax(logits / T) in fp64, rounded once to fp32 */
void orc_softmax(const float *logits, int V, double T, float *out) {
    double m = -INFINITY;
    for (int v = 0; v < V; ++v) {
        double x = (double)logits[v] / T;
        if (x > m) m = x;
    }
    double Z = 0.0;
    for (int v = 0; v < V; ++v) Z += exp((double)logits[v] / T - m);
    for (int v = 0; v < V; ++v) out[v] = (float)(exp((double)logits[v] / T - m) / Z);
}

/* index of the largest element, lowest index on ties */
int orc_argmax(const float *x, int V) {
    int best = 0;
    for (int v = 1; v < V; ++v)
        if (x[v] > x[best]) best = v;
    return best;
}

/* ------------------------------------------------------------------ model + cache */

typedef struct {
    const void *wq, *wk, *wv, *wo, *wg, *wu, *wd;
    const float *g1, *g2;
    const float *sq, *sk, *sv, *so, *sg, *su, *sd; /* row scales: non-NULL = the matrix is int8 */
} orc_layer;

typedef struct {
    int n_layers, d_model, n_heads, head_dim, d_ff, vocab, is_bf16;
    double rope_base, rms_eps;
    orc_layer *layers;
    const void *embed, *lm_head;
    const float *gf;
    const float *s_head; /* row scales of an int8 LM head, or NULL */
    int wbits;           /* 8: scales are per row; 4: int4 matrices with group scales of ORC_W4_GROUP entries */
} orc_model;
#define ORC_W4_GROUP 128

/* KV cache of ONE sequence (Sections 2, 4.2): per layer, keys (already rotated) and values of
 * every past position, row-major [max_seq][n_heads*head_dim], in the storage type. */
typedef struct {
    int n_layers, max_seq, width, is_bf16;
    int len;
    void **k, **v;
} orc_kv;

orc_model *orc_model_new(int n_layers, int d_model, int n_heads, int head_dim, int d_ff, int vocab,
                         double rope_base, double rms_eps, int is_bf16) {
    orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
    m->n_layers = n_layers; m->d_model = d_model; m->n_heads = n_heads; m->head_dim = head_dim;
    m->d_ff = d_ff; m->vocab = vocab; m->rope_base = rope_base; m->rms_eps = rms_eps;
    m->is_bf16 = is_bf16;
    m->wbits = 8;
    m->layers = (orc_layer *)calloc((size_t)n_layers, sizeof(orc_layer));
    return m;
}

void orc_model_set_layer(orc_model *m, int l, const void *wq, const void *wk, const void *wv,
                         const void *wo, const void *wg, const void *wu, const void *wd,
                         const float *g1, const float *g2) {
    orc_layer *L = &m->layers[l];
    L->wq = wq; L->wk = wk; L->wv = wv; L->wo = wo; L->wg = wg; L->wu = wu; L->wd = wd;
    L->g1 = g1; L->g2 = g2;
}

void orc_model_set_io(orc_model *m, const void *embed, const float *gf, const void *lm_head) {
    m->embed = embed; m->gf = gf; m->lm_head = lm_head;
}

/* Declares the seven matrices of layer l (and, with l == -1, the LM head through s[0]) to be int8 with
 * these row scales; the matrix pointers given to orc_model_set_layer / orc_model_set_io then point to int8. */
void orc_model_set_scales(orc_model *m, int l, const float *const *s) {
    if (l < 0) { m->s_head = s[0]; return; }
    orc_layer *L = &m->layers[l];
    L->sq = s[0]; L->sk = s[1]; L->sv = s[2]; L->so = s[3]; L->sg = s[4]; L->su = s[5]; L->sd = s[6];
}

void orc_model_set_wbits(orc_model *m, int bits) { m->wbits = bits; }

/* one linear layer of the model: quantised when the scales are there (int8 per row, or int4 in groups), else the storage type */
static void lin_q(const orc_model *m, const void *W, const float *scale, const float *x, int N, int K, float *y) {
    if (scale && m->wbits == 4) orc_linear_w4((const uint8_t *)W, scale, x, N, K, ORC_W4_GROUP, y);
    else if (scale) orc_linear_w8((const int8_t *)W, scale, x, N, K, y);
    else orc_linear(W, m->is_bf16, x, N, K, y);
}

void orc_model_free(orc_model *m) {
    if (!m) return;
    free(m->layers);
    free(m);
}

orc_kv *orc_kv_new(const orc_model *m, int max_seq) {
    orc_kv *c = (orc_kv *)calloc(1, sizeof(orc_kv));
    c->n_layers = m->n_layers; c->max_seq = max_seq; c->width = m->n_heads * m->head_dim;
    c->is_bf16 = m->is_bf16; c->len = 0;
    c->k = (void **)calloc((size_t)m->n_layers, sizeof(void *));
    c->v = (void **)calloc((size_t)m->n_layers, sizeof(void *));
    size_t esz = m->is_bf16 ? 2 : 4;
    for (int l = 0; l < m->n_layers; ++l) {
        c->k[l] = calloc((size_t)max_seq * (size_t)c->width, esz);
        c->v[l] = calloc((size_t)max_seq * (size_t)c->width, esz);
    }
    return c;
}

void orc_kv_free(orc_kv *c) {
    if (!c) return;
    for (int l = 0; l < c->n_layers; ++l) { free(c->k[l]); free(c->v[l]); }
    free(c->k); free(c->v); free(c);
}

int orc_kv_len(const orc_kv *c) { return c->len; }

/* Truncation (Section 4.4): the stale tail is dropped by moving the length; no data moves. */
int orc_kv_set_len(orc_kv *c, int len) {
    if (len < 0 || len > c->len) return -1;
    c->len = len;
    return 0;
}

/* Raw append of n_rows already-rotated K rows and V rows (storage type) to one layer at
 * positions pos0..pos0+n_rows-1.  The length moves only through orc_kv_advance. */
int orc_kv_write(orc_kv *c, int layer, int pos0, const void *k_rows, const void *v_rows, int n_rows) {
    if (layer < 0 || layer >= c->n_layers || pos0 < 0 || pos0 + n_rows > c->max_seq) return -1;
    size_t esz = c->is_bf16 ? 2 : 4;
    size_t off = (size_t)pos0 * (size_t)c->width * esz, n = (size_t)n_rows * (size_t)c->width * esz;
    memcpy((char *)c->k[layer] + off, k_rows, n);
    memcpy((char *)c->v[layer] + off, v_rows, n);
    return 0;
}

int orc_kv_advance(orc_kv *c, int n_rows) {
    if (c->len + n_rows > c->max_seq) return -1;
    c->len += n_rows;
    return 0;
}

/* Causal attention of one query row (all heads) at absolute position pos over cache positions
 * 0..pos of one layer: s_j = q.k_j / sqrt(hd), P = softmax_j(s), o = sum_j P_j v_j. */
static void attention_row(const orc_model *m, const orc_kv *c, int layer, const float *q, int pos,
                          float *o) {
    int H = m->n_heads, hd = m->head_dim, W = c->width;
    double scale = 1.0 / sqrt((double)hd);
#pragma omp parallel for schedule(static)
    for (int h = 0; h < H; ++h) {
        int n = pos + 1;
        double *s = (double *)malloc((size_t)n * sizeof(double));
        double mx = -INFINITY;
        for (int j = 0; j < n; ++j) {
            double acc = 0.0;
            for (int e = 0; e < hd; ++e)
                acc += (double)q[h * hd + e] * st_get(c->k[layer], c->is_bf16, (size_t)j * W + h * hd + e);
            s[j] = acc * scale;
            if (s[j] > mx) mx = s[j];
        }
        double Z = 0.0;
        for (int j = 0; j < n; ++j) { s[j] = exp(s[j] - mx); Z += s[j]; }
        for (int e = 0; e < hd; ++e) {
            double acc = 0.0;
            for (int j = 0; j < n; ++j)
                acc += s[j] * st_get(c->v[layer], c->is_bf16, (size_t)j * W + h * hd + e);
            o[h * hd + e] = (float)(acc / Z);
        }
        free(s);
    }
}

/* All decoder layers over M new rows of hidden state h [M][d] (in place) at positions
 * len..len+M-1: appends the rows' K/V to the cache and advances its length by M.
 * This is the K+1-row pass of Section 3 when h holds [last committed token, d_1..d_K]. */
int orc_layers_forward(const orc_model *m, orc_kv *c, float *h, int M) {
    int d = m->d_model, H = m->n_heads, hd = m->head_dim, F = m->d_ff, W = H * hd;
    int bf = m->is_bf16;
    if (c->len + M > c->max_seq) return -1;
    float *a = (float *)malloc(sizeof(float) * (size_t)d);
    float *q = (float *)malloc(sizeof(float) * (size_t)W * (size_t)M);
    float *kk = (float *)malloc(sizeof(float) * (size_t)W);
    float *vv = (float *)malloc(sizeof(float) * (size_t)W);
    float *o = (float *)malloc(sizeof(float) * (size_t)W);
    float *t = (float *)malloc(sizeof(float) * (size_t)d);
    float *gg = (float *)malloc(sizeof(float) * (size_t)F);
    float *uu = (float *)malloc(sizeof(float) * (size_t)F);
    for (int l = 0; l < m->n_layers; ++l) {
        const orc_layer *L = &m->layers[l];
        /* projections + rotary + cache append, row by row */
        for (int i = 0; i < M; ++i) {
            int pos = c->len + i;
            orc_rmsnorm(h + (size_t)i * d, L->g1, d, m->rms_eps, a);
            lin_q(m, L->wq, L->sq, a, W, d, q + (size_t)i * W);
            lin_q(m, L->wk, L->sk, a, W, d, kk);
            lin_q(m, L->wv, L->sv, a, W, d, vv);
            for (int hh = 0; hh < H; ++hh) {
                orc_rope(q + (size_t)i * W + hh * hd, hd, pos, m->rope_base);
                orc_rope(kk + hh * hd, hd, pos, m->rope_base);
            }
            for (int e = 0; e < W; ++e) {
                st_put(c->k[l], bf, (size_t)pos * W + e, kk[e]);
                st_put(c->v[l], bf, (size_t)pos * W + e, vv[e]);
            }
        }
        /* attention reads every key/value, the row's own included, back from the cache */
        for (int i = 0; i < M; ++i) {
            float *hi = h + (size_t)i * d;
            attention_row(m, c, l, q + (size_t)i * W, c->len + i, o);
            lin_q(m, L->wo, L->so, o, d, W, t);
            for (int e = 0; e < d; ++e) hi[e] = hi[e] + t[e];
            orc_rmsnorm(hi, L->g2, d, m->rms_eps, a);
            lin_q(m, L->wg, L->sg, a, F, d, gg);
            lin_q(m, L->wu, L->su, a, F, d, uu);
            for (int e = 0; e < F; ++e) gg[e] = (float)(silu((double)gg[e]) * (double)uu[e]);
            lin_q(m, L->wd, L->sd, gg, d, F, t);
            for (int e = 0; e < d; ++e) hi[e] = hi[e] + t[e];
        }
    }
    c->len += M;
    free(a); free(q); free(kk); free(vv); free(o); free(t); free(gg); free(uu);
    return 0;
}

/* h_i = E[token_i] */
int orc_embed(const orc_model *m, const int32_t *tokens, int M, float *h) {
    for (int i = 0; i < M; ++i) {
        if (tokens[i] < 0 || tokens[i] >= m->vocab) return -1;
        for (int e = 0; e < m->d_model; ++e)
            h[(size_t)i * m->d_model + e] = (float)st_get(m->embed, m->is_bf16, (size_t)tokens[i] * m->d_model + e);
    }
    return 0;
}

/* logits_i = RMSNorm(h_i, gf) . W_lm^T */
void orc_head(const orc_model *m, const float *h, int M, float *logits) {
    float *a = (float *)malloc(sizeof(float) * (size_t)m->d_model);
    for (int i = 0; i < M; ++i) {
        orc_rmsnorm(h + (size_t)i * m->d_model, m->gf, m->d_model, m->rms_eps, a);
        lin_q(m, m->lm_head, m->s_head, a, m->vocab, m->d_model, logits + (size_t)i * m->vocab);
    }
    free(a);
}

/* Forward over M token rows against the cache -> logits [M][vocab] (may be NULL to skip the head). */
int orc_forward(const orc_model *m, orc_kv *c, const int32_t *tokens, int M, float *logits) {
    float *h = (float *)malloc(sizeof(float) * (size_t)M * (size_t)m->d_model);
    int rc = orc_embed(m, tokens, M, h);
    if (rc == 0) rc = orc_layers_forward(m, c, h, M);
    if (rc == 0 && logits) orc_head(m, h, M, logits);
    free(h);
    return rc;
}

/* ------------------------------------------------------------------ accept / resample */

/* Bernoulli(min(1, p/q)) realised without a division, in fp32:
 * accept <=> p >= q  or  fl32(u * q) < p.   q = 0 accepts (p >= q). */
int orc_accept(float u, float p, float q) {
    if (p >= q) return 1;
    volatile float t = u * q; /* one IEEE fp32 multiply, round-to-nearest-even, never fused */
    return t < p;
}

/* fixed-point weight of a probability-like fp32 value r in [0, 1]: trunc(r * 2^32) */
static inline uint64_t fx_weight(float r) {
    if (!(r > 0.0f)) return 0;
    return (uint64_t)((double)r * 4294967296.0);
}

static inline float residual(float p, float q) {
    volatile float r = p - q; /* one fp32 subtract */
    return r > 0.0f ? r : 0.0f;
}

/* Integer inverse CDF.  Weights w_v are given by the callback-free form below: kind 0 uses
 * w_v = fx(p_v), kind 1 uses w_v = fx(max(0, p_v - q_v)).  u is a multiple of 2^-24 in [0,1).
 * S = sum w_v; threshold T = floor(m * S / 2^24) with m = u * 2^24; the result is the smallest v
 * whose inclusive prefix sum exceeds T.  Returns -1 when S = 0. */
static int inv_cdf(const float *p, const float *q, int V, float u) {
    uint64_t S = 0;
    for (int v = 0; v < V; ++v) S += q ? fx_weight(residual(p[v], q[v])) : fx_weight(p[v]);
    if (S == 0) return -1;
    uint64_t mant = (uint64_t)((double)u * 16777216.0);
    unsigned __int128 prod = (unsigned __int128)mant * (unsigned __int128)S;
    uint64_t T = (uint64_t)(prod >> 24);
    uint64_t C = 0;
    for (int v = 0; v < V; ++v) {
        C += q ? fx_weight(residual(p[v], q[v])) : fx_weight(p[v]);
        if (C > T) return v;
    }
    return V - 1; /* unreachable: T < S */
}

/* token ~ p by the integer inverse CDF; argmax (lowest index) when every weight quantises to 0 */
int orc_sample(const float *p, int V, float u) {
    int t = inv_cdf(p, NULL, V, u);
    return t >= 0 ? t : orc_argmax(p, V);
}

/* token ~ norm(max(0, p - q)); falls back to orc_sample(p) when the residual quantises to 0 */
int orc_sample_residual(const float *p, const float *q, int V, float u) {
    int t = inv_cdf(p, q, V, u);
    return t >= 0 ? t : orc_sample(p, V, u);
}

/* Top-p ("nucleus") selection, the other token selection rule Section 3 names besides argmax: keep the most
 * probable tokens whose probabilities add up to at least top_p, renormalise, sample from what is left.
 * The paper gives no arithmetic; the reading taken here makes the kept set exact and order-independent:
 *   w_v = min(trunc(p_v * 2^32), 2^32 - 1), S = sum w_v (integers; S = 0: the row is returned unchanged);
 *   P24 = nearest integer to top_p * 2^24, clamped to [1, 2^24]; target T = ceil(P24 * S / 2^24), at least 1;
 *   tokens ordered by (w descending, index ascending); kept = the shortest prefix whose weights add up to >= T;
 *   S' = sum of the kept weights, Z' = fl32(S') * 2^-32, out_v = fl32(p_v / Z') for kept v, else 0.
 * Applied to the target's and the draft's rows alike before the rejection step, the step then emits the
 * filtered target distribution (the guarantee of Section 3 holds for any pair of distributions). */
typedef struct { uint32_t w; int32_t v; } orc_wv;
static int cmp_wv(const void *a, const void *b) {
    const orc_wv *x = (const orc_wv *)a, *y = (const orc_wv *)b;
    if (x->w != y->w) return x->w > y->w ? -1 : 1;
    return x->v < y->v ? -1 : (x->v > y->v ? 1 : 0);
}
static inline uint32_t fx_weight32(float r) {
    uint64_t w = fx_weight(r);
    return w > 0xffffffffu ? 0xffffffffu : (uint32_t)w;
}
int orc_top_p_filter(const float *p, int V, float top_p, float *out) {
    orc_wv *o = (orc_wv *)malloc(sizeof(orc_wv) * (size_t)V);
    uint64_t S = 0;
    for (int v = 0; v < V; ++v) { o[v].w = fx_weight32(p[v]); o[v].v = v; S += o[v].w; }
    int kept = 0;
    if (S == 0) {
        for (int v = 0; v < V; ++v) out[v] = p[v];
        free(o);
        return V;
    }
    double pr = rint((double)top_p * 16777216.0);
    uint64_t P24 = pr < 1.0 ? 1 : (pr > 16777216.0 ? 16777216u : (uint64_t)pr);
    unsigned __int128 prod = (unsigned __int128)P24 * (unsigned __int128)S + 16777215u;
    uint64_t T = (uint64_t)(prod >> 24);
    if (T < 1) T = 1;
    qsort(o, (size_t)V, sizeof(orc_wv), cmp_wv);
    uint64_t C = 0;
    while (kept < V && C < T) C += o[kept++].w;
    volatile float zs = (float)C;          /* uint64 -> fp32, round to nearest even */
    float Z = zs * 2.3283064365386963e-10f; /* * 2^-32, exact */
    for (int v = 0; v < V; ++v) out[v] = 0.0f;
    for (int i = 0; i < kept; ++i) {
        volatile float r = p[o[i].v] / Z;
        out[o[i].v] = r;
    }
    free(o);
    return kept;
}

/* Top-k selection (Section 3 lists it with top-p among the usual token selection rules): keep the k most probable
 * tokens, renormalise.  Same arithmetic as top-p: weights w_v as above, tokens ordered by (w descending, index
 * ascending), kept = the first k of that order (k >= V: the row is returned unchanged, like top_p >= 1);
 * S' = sum of the kept weights (S' = 0: the row is returned unchanged), Z' = fl32(S') * 2^-32,
 * out_v = fl32(p_v / Z') for kept v, else 0.  With both rules in force top-k is applied first and top-p works on its
 * output.  Returns the number of tokens kept. */
int orc_top_k_filter(const float *p, int V, int k, float *out) {
    if (k >= V || k < 1) {
        for (int v = 0; v < V; ++v) out[v] = p[v];
        return V;
    }
    orc_wv *o = (orc_wv *)malloc(sizeof(orc_wv) * (size_t)V);
    for (int v = 0; v < V; ++v) { o[v].w = fx_weight32(p[v]); o[v].v = v; }
    qsort(o, (size_t)V, sizeof(orc_wv), cmp_wv);
    uint64_t C = 0;
    for (int i = 0; i < k; ++i) C += o[i].w;
    if (C == 0) {
        for (int v = 0; v < V; ++v) out[v] = p[v];
        free(o);
        return V;
    }
    volatile float zs = (float)C;           /* uint64 -> fp32, round to nearest even */
    float Z = zs * 2.3283064365386963e-10f; /* * 2^-32, exact */
    for (int v = 0; v < V; ++v) out[v] = 0.0f;
    for (int i = 0; i < k; ++i) {
        volatile float r = p[o[i].v] / Z;
        out[o[i].v] = r;
    }
    free(o);
    return k;
}

/* The modified rejection step (Sections 3, 4.3) for a batch of sequences.
 * p [B][K+1][V], q [B][K][V] probabilities; draft [B][K]; u [B][K+1]: u[b][i<K] decides draft
 * token i, u[b][K] drives the one sampling that happens (residual resample or bonus).
 * n_accepted[b] = number of leading accepted draft tokens, next[b] = the token that follows. */
int orc_speculative_accept(const float *p, const float *q, const int32_t *draft, const float *u,
                           int B, int K, int V, int32_t *n_accepted, int32_t *next) {
    for (int b = 0; b < B; ++b) {
        const float *pb = p + (size_t)b * (K + 1) * V;
        const float *qb = q + (size_t)b * K * V;
        int a = 0;
        for (int i = 0; i < K; ++i) {
            int d = draft[b * K + i];
            if (d < 0 || d >= V) return -1;
            if (!orc_accept(u[b * (K + 1) + i], pb[(size_t)i * V + d], qb[(size_t)i * V + d])) break;
            ++a;
        }
        float us = u[b * (K + 1) + K];
        n_accepted[b] = a;
        if (a < K) next[b] = orc_sample_residual(pb + (size_t)a * V, qb + (size_t)a * V, V, us);
        else next[b] = orc_sample(pb + (size_t)K * V, V, us);
    }
    return 0;
}

/* Greedy (argmax) mode: p and q are one-hot at their argmax, so a draft token is accepted iff it
 * is the target's argmax, and the next token is the target's argmax at the first mismatch (or of
 * the bonus row).  p_logits [B][K+1][V]. */
int orc_greedy_accept(const float *p_logits, const int32_t *draft, int B, int K, int V,
                      int32_t *n_accepted, int32_t *next) {
    for (int b = 0; b < B; ++b) {
        const float *pb = p_logits + (size_t)b * (K + 1) * V;
        int a = 0;
        for (int i = 0; i < K; ++i) {
            if (draft[b * K + i] != orc_argmax(pb + (size_t)i * V, V)) break;
            ++a;
        }
        n_accepted[b] = a;
        next[b] = orc_argmax(pb + (size_t)a * V, V);
    }
    return 0;
}
