/*
 * CPU oracle for one SJD++ decoding path -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, double-precision implementation of what the GPU library
 * computes: a pre-norm decoder-only transformer forward over a Jacobi window
 * against a flat KV cache, classifier-free guidance as a cond/uncond pair, and
 * the speculative-Jacobi verify / residual-resample / reuse rule of the paper
 * (Sec. 4.1, the speculative Jacobi iteration, Steps 1-4: acceptance rule,
 * residual distribution, confidence ratio, reuse rule; the no-reuse refinement
 * rule of Sec. 5 is the tau = +inf setting).
 *
 * Nothing in the product path may include, link or call this file's code; it
 * is used by tests, the smoke check and the benchmark's CPU-baseline leg.
 * It shares no code with the GPU library.  All pointers are HOST pointers.
 *
 * Parity status of each part (what pins it, see tests/test_oracle_*.py):
 *   philox4x32-10 ............ published known-answer vectors
 *   EXP / sampling weights ... double-precision softmax, K = V, K = 1;
 *                              forced-token ranges: the unmasked routine on
 *                              the sliced row, a range of one id is one-hot
 *   integer inverse CDF ...... exhaustive enumeration on small normalisers
 *   accept + residual ........ Theorem 1 (appendix) by chi-square, closed-form
 *                              rejection rate, p = q never rejects
 *   transformer forward ...... library-routine reference (torch CPU, double),
 *                              causality, cache consistency, RoPE shift
 *   whole decode ............. L = 1 is ancestral sampling, K = 1 is greedy AR,
 *                              tau = +inf joint law on a toy model
 *   reuse rule (tau finite) .. PARITY UNPINNED as a law: the paper claims only
 *                              empirical quality preservation for it; pinned as
 *                              a deterministic function and by its two limits.
 */
#ifndef SJD_ORACLE_H
#define SJD_ORACLE_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, d_ff;
    int32_t vocab, sample_lo, sample_hi; /* logits exist for ids in [lo, hi) */
    double rms_eps, rope_theta;
    int32_t window;  /* L: anchor + L-1 drafts */
    int32_t max_ctx; /* positions per branch */
} oracle_model_desc;

/* fp32 values (bf16 configurations pass bf16-rounded values widened to fp32).
 * Linear weights are [out_features][in_features] row-major, y = W x. */
typedef struct {
    const float *tok_emb;    /* [vocab][d] */
    const float *final_norm; /* [d] */
    const float *lm_head;    /* [vocab][d] */
    const float *const *attn_norm, *const *wq, *const *wk, *const *wv, *const *wo;
    const float *const *mlp_norm, *const *w_gate, *const *w_up, *const *w_down;
} oracle_weights;

typedef struct {
    float cfg_scale, temperature;
    int32_t top_k;
    float reuse_tau; /* 0.5 = SJD++ (Sec. 5.1); +INF = SJD without reuse */
    uint64_t seed;
    /* Sec. 4.2, how a window slot that has never had a draft is filled:
     *   0 uniformly over the sampled ids; 1 copy of the token to its left (a); 2 copy of the token one image row
     *   above, row_width tokens back (b); 3 drawn from the distribution its left neighbour was drawn from (c);
     *   4 drawn from the distribution of the token one image row above (d). */
    int32_t init_mode;
    int32_t row_width; /* tokens per image row, modes 2 and 4 */
} oracle_sampling;

typedef struct {
    int32_t n_accepted, n_finalized, reject_index, done;
} oracle_step_result;

typedef struct oracle_ctx oracle_ctx;

/* ---- counter-based randomness (Salmon et al., SC'11: Philox4x32, 10 rounds) */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* ---- sampling distribution of one position (guidance, temperature, top-k,
 *      softmax weights).  e[v] is the fp32 weight EXP(z_v - max) of kept
 *      entries, 0 for dropped ones; *Z is the integer normaliser. */
float oracle_exp_neg(float x);
uint64_t oracle_weight_of(float e);
void oracle_sampling_row(const float *logit_c, const float *logit_u, int32_t V, float cfg_scale,
                         float temperature, int32_t top_k, float *e, uint64_t *Z);

/* The same with a forced-token mask: only ids in [allow_lo, allow_hi) (indices
 * into the row, 0 <= allow_lo < allow_hi <= V) can have weight. */
void oracle_sampling_row_range(const float *logit_c, const float *logit_u, int32_t V, float cfg_scale,
                               float temperature, int32_t top_k, int32_t allow_lo, int32_t allow_hi, float *e,
                               uint64_t *Z);

/* ---- decisions on integer weights (probability = w / Z) */
int32_t oracle_accept(uint32_t u32, uint64_t w_p, uint64_t Z_p, uint64_t w_q, uint64_t Z_q);
int32_t oracle_keep(float tau, uint64_t w_p, uint64_t Z_p, uint64_t w_q, uint64_t Z_q);
int32_t oracle_draw(const float *e_p, uint64_t Z_p, int32_t V, uint64_t u64);
/* q_e == NULL means the uniform reference (w = 1, Z = V). */
int32_t oracle_draw_residual(const float *e_p, uint64_t Z_p, const float *e_q, uint64_t Z_q, int32_t V,
                             uint64_t u64);
/* the same against a one-hot reference at x (a copied draft) */
int32_t oracle_draw_residual_onehot(const float *e_p, uint64_t Z_p, int32_t x, int32_t V, uint64_t u64);

/* Statistical helper for the Theorem-1 pins: n_trials times, draw x ~ q with
 * the integer inverse CDF, test acceptance against p, on rejection draw from
 * the residual; counts[v] += 1 for the resulting token, *n_rejected counts
 * rejections.  Randomness: Philox with key = seed, counter = (trial, 0, 0, 7). */
void oracle_law_trials(const float *e_p, uint64_t Z_p, const float *e_q, uint64_t Z_q, int32_t V,
                       uint64_t seed, int64_t n_trials, int64_t *counts, int64_t *n_rejected);

/* ---- decoder */
int oracle_create(const oracle_model_desc *, const oracle_weights *, const oracle_sampling *,
                  int32_t max_seqs, oracle_ctx **out);
void oracle_destroy(oracle_ctx *);
int oracle_prefill(oracle_ctx *, int32_t n_seqs, const int32_t *const *cond_ids, const int32_t *cond_len,
                   const int32_t *const *uncond_ids, const int32_t *uncond_len,
                   const int32_t *n_image_tokens);
/* Forced tokens: image position i of sequence `seq` may only take ids in
 * [first_id[i], end_id[i]) (absolute ids inside the sampled range), i <
 * n_positions; every other id has probability 0 there.  After oracle_prefill,
 * which resets all positions to the whole sampled range. */
int oracle_set_token_ranges(oracle_ctx *, int32_t seq, const int32_t *first_id, const int32_t *end_id,
                            int32_t n_positions);
int oracle_step(oracle_ctx *, oracle_step_result *out /* [n_seqs] */);
/* Same decisions, but the logits come from the caller instead of the forward:
 * logits is [n_seqs][2 (cond, uncond)][L][V_s] fp32; the KV cache is not
 * touched (its length still advances). */
int oracle_step_from_logits(oracle_ctx *, const float *logits, oracle_step_result *out);
/* Forward of the coming step only: logits of the current window, no decision
 * and no state change; a following oracle_step_from_logits may then advance
 * the decode on other logits for the same window. */
int oracle_peek_logits(oracle_ctx *, float *dst);
/* Logits of the most recent oracle_step, [n_seqs][2][L][V_s]. */
int oracle_copy_logits(oracle_ctx *, float *dst);
int oracle_get_tokens(oracle_ctx *, int32_t seq, int32_t *dst, int32_t cap, int32_t *n_out);
/* Window after the last step: tokens[L] (slot 0 = anchor) and, per slot, the
 * row index (of the last step) serving as its reference, -1 = uniform. */
int oracle_get_window(oracle_ctx *, int32_t seq, int32_t *tokens, int32_t *ref_rows, int32_t *n_slots);
int oracle_set_num_threads(int32_t n); /* returns the thread count in effect */

/* Decodes one prompt n_trials times (seeds seed0 + t) and histograms the
 * decoded sequences: counts[sum_i (tok_i - sample_lo) V_s^i] += 1. */
int oracle_decode_trials(const oracle_model_desc *, const oracle_weights *, const oracle_sampling *,
                         const int32_t *cond, int32_t cond_len, const int32_t *uncond, int32_t uncond_len,
                         int32_t n_image, uint64_t seed0, int64_t n_trials, int64_t *counts, int64_t *n_steps);

/* Full causal forward of one branch from an empty cache: logits[n][V_s]. */
int oracle_forward_logits(const oracle_model_desc *, const oracle_weights *, const int32_t *tokens, int32_t n,
                          float *logits);
/* Forward of a window of n tokens on top of `n_cached` tokens already in a
 * fresh cache built from `prefix` (cache consistency pin). */
int oracle_forward_window_logits(const oracle_model_desc *, const oracle_weights *, const int32_t *prefix,
                                 int32_t n_cached, const int32_t *window, int32_t n, float *logits);

#ifdef __cplusplus
}
#endif
#endif
