/*
 * CPU oracle (test infrastructure): the decoder-only transformer forward.
 *
 * The paper (Sec. 3.1, Sec. 4.1 Step 2) only requires a single causal forward
 * of the model over the window once the prompt is in the cache; it gives no
 * architecture.
 * The architecture is the one the workload configurations name: pre-norm
 * blocks, RMSNorm, rotary position embedding on q and k (rotate-half pairing
 * (i, i + hd/2), angle pos * theta^(-2i/hd)), grouped-query attention with
 * scale 1/sqrt(hd), SwiGLU MLP, untied output head, no biases.
 *
 * All arithmetic is double precision; weights are fp32 values widened on use;
 * logits are rounded to fp32 at the very end.  Tokens of a window are taken
 * one position at a time, each attending to every earlier cached position and
 * itself -- the definition of a causal forward, with no blocking or fusion.
 */
#include "oracle_internal.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* Y[m][n] = sum_k W[n][k] X[m][k] */
static void linear(const float *W, int N, int K, const double *X, int M, double *Y) {
    long work = (long)N * K * M;
#pragma omp parallel for schedule(static) if (work > 200000)
    for (int n = 0; n < N; ++n) {
        const float *w = W + (size_t)n * K;
        for (int m = 0; m < M; ++m) {
            const double *x = X + (size_t)m * K;
            double acc = 0.0;
            for (int k = 0; k < K; ++k) acc += (double)w[k] * x[k];
            Y[(size_t)m * N + n] = acc;
        }
    }
}

static void rmsnorm(const double *x, const float *gain, int d, double eps, double *out) {
    double ss = 0.0;
    for (int i = 0; i < d; ++i) ss += x[i] * x[i];
    double inv = 1.0 / sqrt(ss / d + eps);
    for (int i = 0; i < d; ++i) out[i] = x[i] * inv * (double)gain[i];
}

static void rope(double *vec, int hd, int pos, double theta) {
    int half = hd / 2;
    for (int i = 0; i < half; ++i) {
        double angle = (double)pos * pow(theta, -2.0 * i / hd);
        double c = cos(angle), s = sin(angle);
        double a = vec[i], b = vec[i + half];
        vec[i] = a * c - b * s;
        vec[i + half] = b * c + a * s;
    }
}

oracle_cache *oracle_cache_new(const oracle_model_desc *md) {
    oracle_cache *c = (oracle_cache *)calloc(1, sizeof *c);
    int hd = md->d_model / md->n_heads;
    c->row = (size_t)md->n_kv_heads * hd;
    c->per_layer = c->row * (size_t)md->max_ctx;
    size_t n = c->per_layer * (size_t)md->n_layers;
    c->k = (double *)calloc(n, sizeof(double));
    c->v = (double *)calloc(n, sizeof(double));
    c->len = 0;
    if (!c->k || !c->v) { oracle_cache_free(c); return NULL; }
    return c;
}

void oracle_cache_free(oracle_cache *c) {
    if (!c) return;
    free(c->k);
    free(c->v);
    free(c);
}

/* Runs n tokens at positions cache->len .. cache->len + n - 1, writing their
 * keys and values there (cache->len itself is NOT advanced: the caller commits
 * however many positions it accepts).  If logits != NULL it receives
 * [n][V_s] fp32 rows for the sampled sub-range of the vocabulary. */
int oracle_forward(const oracle_model_desc *md, const oracle_weights *w, oracle_cache *cache,
                   const int32_t *tokens, int n, float *logits) {
    const int d = md->d_model, H = md->n_heads, Hkv = md->n_kv_heads, F = md->d_ff;
    const int hd = d / H, group = H / Hkv;
    const int Vs = md->sample_hi - md->sample_lo;
    const int pos0 = cache->len;
    if (pos0 + n > md->max_ctx) return -5;

    double *x = (double *)malloc(sizeof(double) * (size_t)n * d);
    double *xn = (double *)malloc(sizeof(double) * (size_t)n * d);
    double *q = (double *)malloc(sizeof(double) * (size_t)n * H * hd);
    double *kk = (double *)malloc(sizeof(double) * (size_t)n * Hkv * hd);
    double *vv = (double *)malloc(sizeof(double) * (size_t)n * Hkv * hd);
    double *att = (double *)malloc(sizeof(double) * (size_t)n * H * hd);
    double *proj = (double *)malloc(sizeof(double) * (size_t)n * d);
    double *gate = (double *)malloc(sizeof(double) * (size_t)n * F);
    double *up = (double *)malloc(sizeof(double) * (size_t)n * F);
    double *score = (double *)malloc(sizeof(double) * (size_t)(pos0 + n));

    for (int m = 0; m < n; ++m)
        for (int i = 0; i < d; ++i) x[(size_t)m * d + i] = (double)w->tok_emb[(size_t)tokens[m] * d + i];

    for (int l = 0; l < md->n_layers; ++l) {
        double *Kc = cache->k + cache->per_layer * (size_t)l;
        double *Vc = cache->v + cache->per_layer * (size_t)l;
        for (int m = 0; m < n; ++m) rmsnorm(x + (size_t)m * d, w->attn_norm[l], d, md->rms_eps, xn + (size_t)m * d);
        linear(w->wq[l], H * hd, d, xn, n, q);
        linear(w->wk[l], Hkv * hd, d, xn, n, kk);
        linear(w->wv[l], Hkv * hd, d, xn, n, vv);
        for (int m = 0; m < n; ++m) {
            int pos = pos0 + m;
            for (int h = 0; h < H; ++h) rope(q + ((size_t)m * H + h) * hd, hd, pos, md->rope_theta);
            for (int h = 0; h < Hkv; ++h) rope(kk + ((size_t)m * Hkv + h) * hd, hd, pos, md->rope_theta);
            memcpy(Kc + cache->row * (size_t)pos, kk + (size_t)m * Hkv * hd, sizeof(double) * cache->row);
            memcpy(Vc + cache->row * (size_t)pos, vv + (size_t)m * Hkv * hd, sizeof(double) * cache->row);
        }
        const double scale = 1.0 / sqrt((double)hd);
        for (int m = 0; m < n; ++m) {
            int visible = pos0 + m + 1; /* causal: every cached position and itself */
            for (int h = 0; h < H; ++h) {
                const double *qv = q + ((size_t)m * H + h) * hd;
                int kvh = h / group;
                double mx = -INFINITY;
                for (int t = 0; t < visible; ++t) {
                    const double *kv = Kc + cache->row * (size_t)t + (size_t)kvh * hd;
                    double s = 0.0;
                    for (int i = 0; i < hd; ++i) s += qv[i] * kv[i];
                    score[t] = s * scale;
                    if (score[t] > mx) mx = score[t];
                }
                double denom = 0.0;
                for (int t = 0; t < visible; ++t) {
                    score[t] = exp(score[t] - mx);
                    denom += score[t];
                }
                double *o = att + ((size_t)m * H + h) * hd;
                for (int i = 0; i < hd; ++i) o[i] = 0.0;
                for (int t = 0; t < visible; ++t) {
                    const double *vrow = Vc + cache->row * (size_t)t + (size_t)kvh * hd;
                    double pr = score[t] / denom;
                    for (int i = 0; i < hd; ++i) o[i] += pr * vrow[i];
                }
            }
        }
        linear(w->wo[l], d, H * hd, att, n, proj);
        for (size_t i = 0; i < (size_t)n * d; ++i) x[i] += proj[i];

        for (int m = 0; m < n; ++m) rmsnorm(x + (size_t)m * d, w->mlp_norm[l], d, md->rms_eps, xn + (size_t)m * d);
        linear(w->w_gate[l], F, d, xn, n, gate);
        linear(w->w_up[l], F, d, xn, n, up);
        for (size_t i = 0; i < (size_t)n * F; ++i) {
            double g = gate[i];
            gate[i] = g / (1.0 + exp(-g)) * up[i]; /* silu(g) * u */
        }
        linear(w->w_down[l], d, F, gate, n, proj);
        for (size_t i = 0; i < (size_t)n * d; ++i) x[i] += proj[i];
    }

    if (logits) {
        for (int m = 0; m < n; ++m) rmsnorm(x + (size_t)m * d, w->final_norm, d, md->rms_eps, xn + (size_t)m * d);
        double *lg = (double *)malloc(sizeof(double) * (size_t)n * Vs);
        linear(w->lm_head + (size_t)md->sample_lo * d, Vs, d, xn, n, lg);
        for (size_t i = 0; i < (size_t)n * Vs; ++i) logits[i] = (float)lg[i];
        free(lg);
    }
    free(score); free(up); free(gate); free(proj); free(att); free(vv); free(kk); free(q); free(xn); free(x);
    return 0;
}

int oracle_forward_logits(const oracle_model_desc *md, const oracle_weights *w, const int32_t *tokens, int32_t n,
                          float *logits) {
    oracle_model_desc local = *md;
    if (local.max_ctx < n) local.max_ctx = n;
    oracle_cache *c = oracle_cache_new(&local);
    if (!c) return -2;
    int rc = oracle_forward(&local, w, c, tokens, n, logits);
    oracle_cache_free(c);
    return rc;
}

int oracle_forward_window_logits(const oracle_model_desc *md, const oracle_weights *w, const int32_t *prefix,
                                 int32_t n_cached, const int32_t *window, int32_t n, float *logits) {
    oracle_model_desc local = *md;
    if (local.max_ctx < n_cached + n) local.max_ctx = n_cached + n;
    oracle_cache *c = oracle_cache_new(&local);
    if (!c) return -2;
    int rc = 0;
    if (n_cached > 0) rc = oracle_forward(&local, w, c, prefix, n_cached, NULL);
    c->len = n_cached;
    if (rc == 0) rc = oracle_forward(&local, w, c, window, n, logits);
    oracle_cache_free(c);
    return rc;
}
