/* CPU oracle for D^3 decoding.  TEST INFRASTRUCTURE ONLY -- see d3_oracle.h.
 *
 * Written for checking by eye against the definitions, not for speed: one token
 * at a time, one dot product at a time, summed left to right.
 */
#include "d3_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifndef D3O_REAL
#define D3O_REAL double
#endif
typedef D3O_REAL real;

struct d3o_model {
    d3o_config cfg;
    const void *tok_emb;
    d3o_layer *layers;
    const float *final_norm;
    const void *lm_head;
};

struct d3o_seq {
    const d3o_model *m;
    int32_t max_seq;
    real *K, *V; /* [L][max_seq][H_kv*hd] */
};

static int g_threads = 1;

int d3o_real_size(void) { return (int)sizeof(real); }
void d3o_set_threads(int n) { g_threads = n < 1 ? 1 : n; }

/* ---- schedule (Section 3.4: keep floor(L*alpha^i) blocks; Table 6: drop window) ---- */

int d3o_plan_depth(int32_t L, double alpha, int32_t start, int32_t min_keep, int32_t n_steps,
                   int32_t *keep, int32_t *drop_begin, int32_t *layer_ids)
{
    if (L < 1 || !(alpha > 0.0) || !(alpha <= 1.0) || start < 0 || start >= L || min_keep < 0 ||
        min_keep > L || n_steps < 0)
        return -1;
    volatile double p = 1.0; /* volatile: each product is rounded to binary64, no contraction */
    for (int32_t i = 0; i < n_steps; ++i) {
        int32_t k = (int32_t)floor((double)L * p);
        if (k < min_keep) k = min_keep;
        int32_t n = L - k;
        int32_t s = start < L - n ? start : L - n;
        if (keep) keep[i] = k;
        if (drop_begin) drop_begin[i] = s;
        if (layer_ids) {
            int32_t j = 0;
            for (int32_t l = 0; l < L; ++l)
                if (l < s || l >= s + n) layer_ids[(size_t)i * L + j++] = l;
            for (; j < L; ++j) layer_ids[(size_t)i * L + j] = -1;
        }
        p = p * alpha;
    }
    return 0;
}

/* Linear decay between bounds (the comparison schedule named in Section 3.4 / Section 4.1; the bounds are
 * arguments because the paper prints none): keep[i] = floor(y_i) on the straight line y_i = keep_first -
 * (keep_first - keep_last) * i / (n_steps - 1), evaluated exactly as one integer quotient (the numerator is
 * never negative).  Window placement is Table 6's rule, as above. */
int d3o_plan_depth_linear(int32_t L, int32_t keep_first, int32_t keep_last, int32_t start, int32_t n_steps,
                          int32_t *keep, int32_t *drop_begin, int32_t *layer_ids)
{
    if (L < 1 || keep_last < 0 || keep_last > keep_first || keep_first > L || start < 0 || start >= L || n_steps < 0)
        return -1;
    for (int32_t i = 0; i < n_steps; ++i) {
        int64_t den = n_steps > 1 ? n_steps - 1 : 1;
        int64_t num = (int64_t)keep_first * den - (int64_t)(keep_first - keep_last) * i;
        int32_t k = (int32_t)(num / den);
        int32_t n = L - k;
        int32_t s = start < L - n ? start : L - n;
        if (keep) keep[i] = k;
        if (drop_begin) drop_begin[i] = s;
        if (layer_ids) {
            int32_t j = 0;
            for (int32_t l = 0; l < L; ++l)
                if (l < s || l >= s + n) layer_ids[(size_t)i * L + j++] = l;
            for (; j < L; ++j) layer_ids[(size_t)i * L + j] = -1;
        }
    }
    return 0;
}

/* ---- weights ---- */

static inline real weight_at(const void *w, int32_t dtype, size_t idx)
{
    if (dtype == 0) return (real)((const float *)w)[idx];
    uint32_t bits = (uint32_t)((const uint16_t *)w)[idx] << 16; /* bf16 -> float32, exact */
    float f;
    memcpy(&f, &bits, sizeof f);
    return (real)f;
}

/* y[r] = sum_c W[r][c] * x[c], W row-major [rows][cols]. */
static void matvec(const void *W, int32_t dtype, int32_t rows, int32_t cols, const real *x, real *y)
{
#ifdef _OPENMP
#pragma omp parallel for num_threads(g_threads) schedule(static)
#endif
    for (int32_t r = 0; r < rows; ++r) {
        real acc = 0;
        for (int32_t c = 0; c < cols; ++c) acc += weight_at(W, dtype, (size_t)r * cols + c) * x[c];
        y[r] = acc;
    }
}

/* ---- block pieces ---- */

/* RMSNorm: out = x / sqrt(mean(x^2) + eps) * gain. */
static void rmsnorm(const real *x, const float *gain, int32_t n, real eps, real *out)
{
    real ss = 0;
    for (int32_t j = 0; j < n; ++j) ss += x[j] * x[j];
    real inv = (real)1 / (real)sqrt((double)(ss / (real)n + eps));
    for (int32_t j = 0; j < n; ++j) out[j] = x[j] * inv * (real)gain[j];
}

/* Rotary embedding of one head, half-split pairing: dims (j, j + hd/2) rotate by
 * the angle pos * base^(-2j/hd). */
static void rope(real *v, int32_t hd, int32_t pos, double base)
{
    int32_t half = hd / 2;
    for (int32_t j = 0; j < half; ++j) {
        double angle = (double)pos * pow(base, -2.0 * (double)j / (double)hd);
        real c = (real)cos(angle), s = (real)sin(angle);
        real a = v[j], b = v[j + half];
        v[j] = a * c - b * s;
        v[j + half] = a * s + b * c;
    }
}

static void softmax(real *v, int32_t n)
{
    real mx = v[0];
    for (int32_t j = 1; j < n; ++j)
        if (v[j] > mx) mx = v[j];
    real sum = 0;
    for (int32_t j = 0; j < n; ++j) {
        v[j] = (real)exp((double)(v[j] - mx));
        sum += v[j];
    }
    for (int32_t j = 0; j < n; ++j) v[j] /= sum;
}

static real silu(real x) { return x / ((real)1 + (real)exp((double)-x)); }

/* One query head over rows 0..n_rows-1: out = softmax(q.K^T / sqrt(hd)) V.
 * K and V point at this head's slice of row 0; rows are row_stride apart. */
static void attention_head(const real *q, const real *K, const real *V, int32_t n_rows, int32_t hd,
                           int32_t row_stride, real *scores, real *out)
{
    real scale = (real)1 / (real)sqrt((double)hd);
    for (int32_t t = 0; t < n_rows; ++t) {
        real acc = 0;
        for (int32_t j = 0; j < hd; ++j) acc += q[j] * K[(size_t)t * row_stride + j];
        scores[t] = acc * scale;
    }
    softmax(scores, n_rows);
    for (int32_t j = 0; j < hd; ++j) {
        real acc = 0;
        for (int32_t t = 0; t < n_rows; ++t) acc += scores[t] * V[(size_t)t * row_stride + j];
        out[j] = acc;
    }
}

/* ---- model / sequence ---- */

d3o_model *d3o_model_new(const d3o_config *cfg, const void *tok_emb, const d3o_layer *layers,
                         const float *final_norm, const void *lm_head)
{
    if (!cfg || !tok_emb || !layers || !final_norm || !lm_head) return NULL;
    if (cfg->L < 1 || cfg->d < 1 || cfg->H < 1 || cfg->H_kv < 1 || cfg->H % cfg->H_kv != 0 ||
        cfg->hd < 2 || cfg->hd % 2 != 0 || cfg->F < 1 || cfg->V < 1 ||
        (cfg->weight_dtype != 0 && cfg->weight_dtype != 1))
        return NULL;
    d3o_model *m = (d3o_model *)calloc(1, sizeof *m);
    m->cfg = *cfg;
    m->tok_emb = tok_emb;
    m->layers = (d3o_layer *)malloc(sizeof(d3o_layer) * (size_t)cfg->L);
    memcpy(m->layers, layers, sizeof(d3o_layer) * (size_t)cfg->L);
    m->final_norm = final_norm;
    m->lm_head = lm_head;
    return m;
}

void d3o_model_free(d3o_model *m)
{
    if (!m) return;
    free(m->layers);
    free(m);
}

d3o_seq *d3o_seq_new(const d3o_model *m, int32_t max_seq)
{
    if (!m || max_seq < 1) return NULL;
    d3o_seq *s = (d3o_seq *)calloc(1, sizeof *s);
    size_t n = (size_t)m->cfg.L * max_seq * m->cfg.H_kv * m->cfg.hd;
    s->m = m;
    s->max_seq = max_seq;
    s->K = (real *)calloc(n, sizeof(real));
    s->V = (real *)calloc(n, sizeof(real));
    if (!s->K || !s->V) {
        d3o_seq_free(s);
        return NULL;
    }
    return s;
}

void d3o_seq_free(d3o_seq *s)
{
    if (!s) return;
    free(s->K);
    free(s->V);
    free(s);
}

static size_t kv_index(const d3o_seq *s, int32_t layer, int32_t pos)
{
    const d3o_config *c = &s->m->cfg;
    return ((size_t)layer * s->max_seq + pos) * ((size_t)c->H_kv * c->hd);
}

int d3o_forward_token(d3o_seq *s, int32_t token, int32_t pos, const int32_t *layer_ids, int32_t n_ids,
                      double *hidden_out, double *logits_out)
{
    if (!s || pos < 0 || pos >= s->max_seq || n_ids < 0 || (n_ids > 0 && !layer_ids)) return -1;
    const d3o_model *m = s->m;
    const d3o_config *c = &m->cfg;
    if (token < 0 || token >= c->V || n_ids > c->L) return -1;
    for (int32_t j = 0; j < n_ids; ++j)
        if (layer_ids[j] < 0 || layer_ids[j] >= c->L || (j > 0 && layer_ids[j] <= layer_ids[j - 1])) return -1;

    const int32_t d = c->d, hd = c->hd, q_dim = c->H * hd, kv_dim = c->H_kv * hd, F = c->F;
    const int32_t group = c->H / c->H_kv; /* query heads per KV head */
    const int32_t dt = c->weight_dtype;

    real *x = (real *)malloc(sizeof(real) * d);       /* residual stream */
    real *a = (real *)malloc(sizeof(real) * d);       /* normed input */
    real *q = (real *)malloc(sizeof(real) * q_dim);
    real *o = (real *)malloc(sizeof(real) * q_dim);   /* attention output, heads concatenated */
    real *t = (real *)malloc(sizeof(real) * d);       /* projection back to width d */
    real *g = (real *)malloc(sizeof(real) * F);
    real *u = (real *)malloc(sizeof(real) * F);
    real *scores = (real *)malloc(sizeof(real) * (size_t)(pos + 1));

    /* embedding */
    for (int32_t j = 0; j < d; ++j) x[j] = weight_at(m->tok_emb, dt, (size_t)token * d + j);
    if (hidden_out)
        for (int32_t j = 0; j < d; ++j) hidden_out[j] = (double)x[j];

    for (int32_t e = 0; e < n_ids; ++e) {
        const int32_t l = layer_ids[e];
        const d3o_layer *w = &m->layers[l];
        real *k_row = s->K + kv_index(s, l, pos);
        real *v_row = s->V + kv_index(s, l, pos);

        /* attention half */
        rmsnorm(x, w->attn_norm, d, (real)c->eps, a);
        matvec(w->wq, dt, q_dim, d, a, q);
        matvec(w->wk, dt, kv_dim, d, a, k_row);
        matvec(w->wv, dt, kv_dim, d, a, v_row);
        for (int32_t h = 0; h < c->H; ++h) rope(q + (size_t)h * hd, hd, pos, c->rope_base);
        for (int32_t h = 0; h < c->H_kv; ++h) rope(k_row + (size_t)h * hd, hd, pos, c->rope_base);
        for (int32_t h = 0; h < c->H; ++h) {
            const int32_t kvh = h / group;
            attention_head(q + (size_t)h * hd, s->K + kv_index(s, l, 0) + (size_t)kvh * hd,
                           s->V + kv_index(s, l, 0) + (size_t)kvh * hd, pos + 1, hd, kv_dim, scores,
                           o + (size_t)h * hd);
        }
        matvec(w->wo, dt, d, q_dim, o, t);
        for (int32_t j = 0; j < d; ++j) x[j] += t[j];

        /* SwiGLU MLP half */
        rmsnorm(x, w->mlp_norm, d, (real)c->eps, a);
        matvec(w->w_gate, dt, F, d, a, g);
        matvec(w->w_up, dt, F, d, a, u);
        for (int32_t j = 0; j < F; ++j) g[j] = silu(g[j]) * u[j];
        matvec(w->w_down, dt, d, F, g, t);
        for (int32_t j = 0; j < d; ++j) x[j] += t[j];

        if (hidden_out)
            for (int32_t j = 0; j < d; ++j) hidden_out[(size_t)(e + 1) * d + j] = (double)x[j];
    }

    if (logits_out) {
        real *lg = (real *)malloc(sizeof(real) * c->V);
        rmsnorm(x, m->final_norm, d, (real)c->eps, a);
        matvec(m->lm_head, dt, c->V, d, a, lg);
        for (int32_t j = 0; j < c->V; ++j) logits_out[j] = (double)lg[j];
        free(lg);
    }

    free(x); free(a); free(q); free(o); free(t); free(g); free(u); free(scores);
    return 0;
}

/* The steps of d3o_forward_token up to the cache write of the first listed block, and nothing after them:
 * embedding -> RMSNorm -> Wk, Wv -> RoPE(k) -> K[layer][pos], V[layer][pos].  A test that needs a long prompt's
 * cache rows of the first block, but not the prompt's outputs, fills the cache this way. */
int d3o_first_block_kv(d3o_seq *s, int32_t token, int32_t pos, int32_t layer)
{
    if (!s || pos < 0 || pos >= s->max_seq) return -1;
    const d3o_model *m = s->m;
    const d3o_config *c = &m->cfg;
    if (token < 0 || token >= c->V || layer < 0 || layer >= c->L) return -1;
    const int32_t d = c->d, hd = c->hd, kv_dim = c->H_kv * hd;
    const int32_t dt = c->weight_dtype;
    const d3o_layer *w = &m->layers[layer];
    real *x = (real *)malloc(sizeof(real) * d);
    real *a = (real *)malloc(sizeof(real) * d);
    real *k_row = s->K + kv_index(s, layer, pos);
    real *v_row = s->V + kv_index(s, layer, pos);
    for (int32_t j = 0; j < d; ++j) x[j] = weight_at(m->tok_emb, dt, (size_t)token * d + j);
    rmsnorm(x, w->attn_norm, d, (real)c->eps, a);
    matvec(w->wk, dt, kv_dim, d, a, k_row);
    matvec(w->wv, dt, kv_dim, d, a, v_row);
    for (int32_t h = 0; h < c->H_kv; ++h) rope(k_row + (size_t)h * hd, hd, pos, c->rope_base);
    free(x); free(a);
    return 0;
}

int32_t d3o_argmax(const double *logits, int32_t n)
{
    int32_t best = 0;
    for (int32_t j = 1; j < n; ++j)
        if (logits[j] > logits[best]) best = j;
    return best;
}

int d3o_fill_missing_kv(d3o_seq *s, int32_t pos, int32_t drop_begin, int32_t n_drop)
{
    if (!s || pos < 0 || pos >= s->max_seq) return -1;
    const d3o_config *c = &s->m->cfg;
    if (n_drop < 0 || drop_begin < 0 || drop_begin + n_drop > c->L) return -1;
    const size_t row = (size_t)c->H_kv * c->hd;
    int32_t src = drop_begin > 0 ? drop_begin - 1 : drop_begin + n_drop;
    for (int32_t l = drop_begin; l < drop_begin + n_drop; ++l) {
        real *k = s->K + kv_index(s, l, pos), *v = s->V + kv_index(s, l, pos);
        if (src >= c->L) { /* nothing ran for this token */
            memset(k, 0, row * sizeof(real));
            memset(v, 0, row * sizeof(real));
        } else {
            memcpy(k, s->K + kv_index(s, src, pos), row * sizeof(real));
            memcpy(v, s->V + kv_index(s, src, pos), row * sizeof(real));
        }
    }
    return 0;
}

/* RECOMPUTE fill (Section 3.2: the hidden state is copied through the skipped blocks and their KV is
 * recomputed from it): for every block l in [drop_begin, drop_begin + n_drop),
 * a = RMSNorm(h; attn_norm_l), K[l][pos] = RoPE(W_k^l a, pos), V[l][pos] = W_v^l a. */
int d3o_fill_recompute(d3o_seq *s, int32_t pos, int32_t drop_begin, int32_t n_drop, const double *h)
{
    if (!s || !h || pos < 0 || pos >= s->max_seq) return -1;
    const d3o_model *m = s->m;
    const d3o_config *c = &m->cfg;
    if (n_drop < 0 || drop_begin < 0 || drop_begin + n_drop > c->L) return -1;
    const int32_t d = c->d, hd = c->hd, kv_dim = c->H_kv * hd;
    real *x = (real *)malloc(sizeof(real) * d);
    real *a = (real *)malloc(sizeof(real) * d);
    for (int32_t j = 0; j < d; ++j) x[j] = (real)h[j];
    for (int32_t l = drop_begin; l < drop_begin + n_drop; ++l) {
        const d3o_layer *w = &m->layers[l];
        real *k_row = s->K + kv_index(s, l, pos);
        real *v_row = s->V + kv_index(s, l, pos);
        rmsnorm(x, w->attn_norm, d, (real)c->eps, a);
        matvec(w->wk, c->weight_dtype, kv_dim, d, a, k_row);
        matvec(w->wv, c->weight_dtype, kv_dim, d, a, v_row);
        for (int32_t hh = 0; hh < c->H_kv; ++hh) rope(k_row + (size_t)hh * hd, hd, pos, c->rope_base);
    }
    free(x); free(a);
    return 0;
}

int d3o_get_kv(const d3o_seq *s, int32_t layer, int32_t pos, double *k_out, double *v_out)
{
    if (!s || layer < 0 || layer >= s->m->cfg.L || pos < 0 || pos >= s->max_seq) return -1;
    const size_t row = (size_t)s->m->cfg.H_kv * s->m->cfg.hd;
    for (size_t j = 0; j < row; ++j) {
        if (k_out) k_out[j] = (double)s->K[kv_index(s, layer, pos) + j];
        if (v_out) v_out[j] = (double)s->V[kv_index(s, layer, pos) + j];
    }
    return 0;
}

/* ---- exported sub-functions (double in/out, computed in `real`) ---- */

void d3o_rmsnorm(const double *x, const float *gain, int32_t n, double eps, double *out)
{
    real *xi = (real *)malloc(sizeof(real) * n), *xo = (real *)malloc(sizeof(real) * n);
    for (int32_t j = 0; j < n; ++j) xi[j] = (real)x[j];
    rmsnorm(xi, gain, n, (real)eps, xo);
    for (int32_t j = 0; j < n; ++j) out[j] = (double)xo[j];
    free(xi); free(xo);
}

void d3o_rope(double *vec, int32_t hd, int32_t pos, double base)
{
    real *v = (real *)malloc(sizeof(real) * hd);
    for (int32_t j = 0; j < hd; ++j) v[j] = (real)vec[j];
    rope(v, hd, pos, base);
    for (int32_t j = 0; j < hd; ++j) vec[j] = (double)v[j];
    free(v);
}

void d3o_softmax(double *v, int32_t n)
{
    real *t = (real *)malloc(sizeof(real) * n);
    for (int32_t j = 0; j < n; ++j) t[j] = (real)v[j];
    softmax(t, n);
    for (int32_t j = 0; j < n; ++j) v[j] = (double)t[j];
    free(t);
}

double d3o_silu(double x) { return (double)silu((real)x); }

void d3o_attention_head(const double *q, const double *K, const double *V, int32_t n_rows, int32_t hd,
                        int32_t row_stride, double *out)
{
    size_t nkv = (size_t)(n_rows - 1) * row_stride + hd;
    real *qi = (real *)malloc(sizeof(real) * hd), *Ki = (real *)malloc(sizeof(real) * nkv);
    real *Vi = (real *)malloc(sizeof(real) * nkv), *sc = (real *)malloc(sizeof(real) * n_rows);
    real *oi = (real *)malloc(sizeof(real) * hd);
    for (int32_t j = 0; j < hd; ++j) qi[j] = (real)q[j];
    for (size_t j = 0; j < nkv; ++j) { Ki[j] = (real)K[j]; Vi[j] = (real)V[j]; }
    attention_head(qi, Ki, Vi, n_rows, hd, row_stride, sc, oi);
    for (int32_t j = 0; j < hd; ++j) out[j] = (double)oi[j];
    free(qi); free(Ki); free(Vi); free(sc); free(oi);
}
