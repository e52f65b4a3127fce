/*
 * CPU oracle (test infrastructure): randomness, the sampling distribution of a
 * position and the accept / residual / reuse decisions.
 *
 * Paper passages followed:
 *   Sec. 3.1  top-K sampling from the softmax over the vocabulary
 *   Sec. 5.1  guidance weight, K, reuse threshold tau
 *   Sec. 4.1  Eq. 2 (accept iff r < min(1, p/q)), Eq. 3 (residual
 *             normalise(max(0, p - q))), Eq. 4 (confidence p/q), Eq. 5 (reuse)
 *
 * The paper states the rules on real-valued probabilities.  To make every
 * decision a reproducible function of the fp32 logits this file fixes one
 * arithmetic: fp32 for the guided logit, an explicitly specified exponential,
 * integer weights w = trunc(e * 2^40) with an integer normaliser Z, decisions
 * in double on P = w / Z, and draws by integer inverse CDF.
 * Compile with -ffp-contract=off.
 */
#include "sjd_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ Philox */
/* Philox4x32 with 10 rounds as published by Salmon, Moraes, Dror and Shaw
 * (SC'11): two 32x32->64 multiplies per round, key bumped by Weyl constants. */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* ------------------------------------------------- the specified exponential */
/* EXP(x) for x <= 0: k = rint(x * log2 e); r = x - k ln2 by a two-constant
 * split; degree-6 Taylor polynomial of e^r by Horner with fused multiply-adds;
 * scaled by 2^k through the exponent field.  Returns 0 below -60. */
float oracle_exp_neg(float x) {
    if (x < -60.0f) return 0.0f;
    float kf = rintf(x * 0x1.715476p+0f);
    float r = fmaf(kf, -0x1.62ep-1f, x);
    r = fmaf(kf, -0x1.0bfbe8p-15f, r);
    float p = 0x1.6c16c2p-10f;          /* 1/720 */
    p = fmaf(p, r, 0x1.111112p-7f);     /* 1/120 */
    p = fmaf(p, r, 0x1.555556p-5f);     /* 1/24  */
    p = fmaf(p, r, 0x1.555556p-3f);     /* 1/6   */
    p = fmaf(p, r, 0.5f);
    p = fmaf(p, r, 1.0f);
    p = fmaf(p, r, 1.0f);
    int32_t k = (int32_t)kf;            /* in [-87, 0] */
    uint32_t bits = (uint32_t)(k + 127) << 23;
    float scale;
    memcpy(&scale, &bits, sizeof scale);
    return p * scale;
}

uint64_t oracle_weight_of(float e) { return (uint64_t)(e * 0x1p40f); }

static int cmp_float_desc(const void *a, const void *b) {
    float x = *(const float *)a, y = *(const float *)b;
    return (x < y) - (x > y);
}

/* Guidance on raw logits z = l_u + s (l_c - l_u), times 1/T, then top-K with
 * ties at the K-th value kept, then softmax weights relative to the maximum.
 * Only ids in [allow_lo, allow_hi) are candidates (a forced-token mask: every
 * other id has probability 0, as if its logit were minus infinity). */
void oracle_sampling_row_range(const float *logit_c, const float *logit_u, int32_t V, float cfg_scale,
                               float temperature, int32_t top_k, int32_t allow_lo, int32_t allow_hi, float *e,
                               uint64_t *Z) {
    float inv_t = 1.0f / temperature;
    int32_t n = allow_hi - allow_lo;
    float *z = (float *)malloc(sizeof(float) * (size_t)V);
    float *sorted = (float *)malloc(sizeof(float) * (size_t)n);
    for (int32_t v = 0; v < V; ++v) {
        float d = logit_c[v] - logit_u[v];
        z[v] = fmaf(cfg_scale, d, logit_u[v]) * inv_t;
    }
    memcpy(sorted, z + allow_lo, sizeof(float) * (size_t)n);
    qsort(sorted, (size_t)n, sizeof(float), cmp_float_desc);
    float m = sorted[0];
    float t = (top_k >= n) ? sorted[n - 1] : sorted[top_k - 1];
    uint64_t total = 0;
    for (int32_t v = 0; v < V; ++v) {
        int allowed = v >= allow_lo && v < allow_hi;
        e[v] = (allowed && z[v] >= t) ? oracle_exp_neg(z[v] - m) : 0.0f;
        total += oracle_weight_of(e[v]);
    }
    *Z = total;
    free(sorted);
    free(z);
}

void oracle_sampling_row(const float *logit_c, const float *logit_u, int32_t V, float cfg_scale,
                         float temperature, int32_t top_k, float *e, uint64_t *Z) {
    oracle_sampling_row_range(logit_c, logit_u, V, cfg_scale, temperature, top_k, 0, V, e, Z);
}

/* ----------------------------------------------------------------- decisions */
static double prob(uint64_t w, uint64_t Z) { return (double)w / (double)Z; }

/* Eq. 2 with r = (u32 + 1/2) 2^-32 in (0,1): accept iff r q < p. */
int32_t oracle_accept(uint32_t u32, uint64_t w_p, uint64_t Z_p, uint64_t w_q, uint64_t Z_q) {
    double r = ((double)u32 + 0.5) * 0x1p-32;
    double P = prob(w_p, Z_p), Q = prob(w_q, Z_q);
    return r * Q < P;
}

/* Eq. 4-5: keep the draft iff C = p/q > tau, written p > tau q. */
int32_t oracle_keep(float tau, uint64_t w_p, uint64_t Z_p, uint64_t w_q, uint64_t Z_q) {
    double P = prob(w_p, Z_p), Q = prob(w_q, Z_q);
    return P > (double)tau * Q;
}

static uint64_t mulhi64(uint64_t a, uint64_t b) { return (uint64_t)(((unsigned __int128)a * b) >> 64); }

/* Inverse CDF over integer weights in ascending token order: the first v whose
 * inclusive prefix sum exceeds floor(u64 * Z / 2^64). */
int32_t oracle_draw(const float *e_p, uint64_t Z_p, int32_t V, uint64_t u64) {
    uint64_t target = mulhi64(u64, Z_p);
    uint64_t prefix = 0;
    for (int32_t v = 0; v < V; ++v) {
        prefix += oracle_weight_of(e_p[v]);
        if (prefix > target) return v;
    }
    return V - 1; /* unreachable when Z_p is the sum of the weights */
}

static uint64_t residual_weight(double P, double Q) {
    double d = P - Q;
    return d > 0.0 ? (uint64_t)(d * 0x1p44) : 0;
}

/* Eq. 3: draw from max(0, p - q) normalised; if the quantised residual is
 * empty fall back to p. */
int32_t oracle_draw_residual(const float *e_p, uint64_t Z_p, const float *e_q, uint64_t Z_q, int32_t V,
                             uint64_t u64) {
    uint64_t R = 0;
    for (int32_t v = 0; v < V; ++v) {
        double P = prob(oracle_weight_of(e_p[v]), Z_p);
        double Q = e_q ? prob(oracle_weight_of(e_q[v]), Z_q) : prob(1, (uint64_t)V);
        R += residual_weight(P, Q);
    }
    if (R == 0) return oracle_draw(e_p, Z_p, V, u64);
    uint64_t target = mulhi64(u64, R);
    uint64_t prefix = 0;
    for (int32_t v = 0; v < V; ++v) {
        double P = prob(oracle_weight_of(e_p[v]), Z_p);
        double Q = e_q ? prob(oracle_weight_of(e_q[v]), Z_q) : prob(1, (uint64_t)V);
        prefix += residual_weight(P, Q);
        if (prefix > target) return v;
    }
    return V - 1;
}

/* Eq. 3 against a one-hot reference q = delta_x (a draft that was copied, not drawn): max(0, p - q) is p with the
 * entry of x removed; if nothing else has weight fall back to p. */
int32_t oracle_draw_residual_onehot(const float *e_p, uint64_t Z_p, int32_t x, int32_t V, uint64_t u64) {
    uint64_t R = 0;
    for (int32_t v = 0; v < V; ++v) R += residual_weight(prob(oracle_weight_of(e_p[v]), Z_p), v == x ? 1.0 : 0.0);
    if (R == 0) return oracle_draw(e_p, Z_p, V, u64);
    uint64_t target = mulhi64(u64, R);
    uint64_t prefix = 0;
    for (int32_t v = 0; v < V; ++v) {
        prefix += residual_weight(prob(oracle_weight_of(e_p[v]), Z_p), v == x ? 1.0 : 0.0);
        if (prefix > target) return v;
    }
    return V - 1;
}

void oracle_law_trials(const float *e_p, uint64_t Z_p, const float *e_q, uint64_t Z_q, int32_t V,
                       uint64_t seed, int64_t n_trials, int64_t *counts, int64_t *n_rejected) {
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    int64_t rejected = 0;
    for (int64_t t = 0; t < n_trials; ++t) {
        uint32_t ctr[4] = {(uint32_t)t, (uint32_t)((uint64_t)t >> 32), 0, 7}, a[4], b[4];
        oracle_philox4x32_10(ctr, key, a);
        ctr[2] = 1;
        oracle_philox4x32_10(ctr, key, b);
        uint64_t u_draft = ((uint64_t)a[1] << 32) | a[2];
        uint64_t u_resid = ((uint64_t)b[1] << 32) | b[2];
        int32_t x = e_q ? oracle_draw(e_q, Z_q, V, u_draft) : (int32_t)(((uint64_t)a[3] * (uint64_t)V) >> 32);
        uint64_t w_q = e_q ? oracle_weight_of(e_q[x]) : 1;
        uint64_t z_q = e_q ? Z_q : (uint64_t)V;
        if (oracle_accept(a[0], oracle_weight_of(e_p[x]), Z_p, w_q, z_q)) {
            counts[x] += 1;
        } else {
            rejected += 1;
            counts[oracle_draw_residual(e_p, Z_p, e_q, Z_q, V, u_resid)] += 1;
        }
    }
    *n_rejected = rejected;
}
