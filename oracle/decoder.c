/*
 * CPU oracle (test infrastructure): the speculative Jacobi decoding loop.
 *
 * Sec. 4.1 of the paper, in its order:
 *   Step 1  the window holds the drafts that were not accepted plus newly
 *           initialised ones; each draft carries the distribution it was
 *           predicted with at the previous iteration (its reference q);
 *   Step 2  one causal forward over the window gives the new distributions p;
 *   Step 3  drafts are accepted left to right with probability min(1, p/q)
 *           (Eq. 2); accepted tokens are final;
 *   Step 4  the first unaccepted position is redrawn from the residual
 *           normalise(max(0, p - q)) (Eq. 3); every later draft is kept if its
 *           confidence p/q exceeds tau (Eq. 4-5) and otherwise redrawn from p;
 *           tau = +inf is the rule without reuse (Eq. 6).
 *
 * Readings where the paper is silent (listed in the design notes):
 *   - the first window input is the last final token (anchor), so output row k
 *     is the distribution of the position after input k, and the draft in slot
 *     k + 1 is verified against row k;
 *   - the token drawn at the first unaccepted position is final at once; if
 *     every draft is accepted a token is drawn from the last row instead;
 *   - a draft that never had a row (freshly initialised, drawn uniformly over
 *     the sampled range) has the uniform distribution as its reference;
 *   - the last row of a rejecting step has no draft: its slot enters the next
 *     window drawn from that row;
 *   - near the end of the image the window shrinks to the tokens remaining.
 *
 * Sec. 4.2 (initialisation with a spatial prior) changes only how a slot that
 * has never had a draft is filled (init_mode of the sampling parameters):
 *   (a) copy of the token to its left, (b) copy of the token one image row
 *   above, (c) a draw from the distribution the left neighbour was drawn from.
 * A copied draft was "drawn" from the one-hot distribution at that token, so
 * that is its reference; a draft of (c) has the row it was drawn from.  Slots
 * of the very first window (no image token exists yet) and slots of (b) in
 * the first image row are filled uniformly.  (d) draws from the distribution
 * of the token one image row above: for a token that is final, the row under
 * which it became final (the last row_width of them are kept per sequence);
 * for one that is still a draft in the window, that draft's own reference.
 *
 * Randomness: Philox4x32-10, key = seed, counter = (step, row, sequence, 0).
 * Word 0 is the acceptance uniform of the draft verified at that row, words
 * 1-2 the 64-bit uniform of the one draw made at that row, word 3 a fresh
 * uniform draft.  step = 0 is the initial window, steps count from 1.
 */
#include "oracle_internal.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { OK = 0, EINVAL_ = -1, ENOMEM_ = -2, ESTATE_ = -3, ECAPACITY_ = -5 };
enum { REF_UNIFORM = -1, REF_ONEHOT = -2, REF_HIST0 = -3 };

typedef struct {
    int32_t cond_len, uncond_len, n_image;
    int32_t n_img; /* image tokens final so far */
    int32_t *out;  /* [n_image] */
    int32_t *allow_lo, *allow_hi; /* [n_image] ids (relative to sample_lo) image position i may take: [lo, hi) */
    int32_t anchor[2];
    int32_t *tok;     /* [L] window tokens, slot 0 unused (anchor above) */
    int32_t *ref_row; /* [L] slot -> row of `ref_e` that is its reference, -1 = uniform, -2 = one-hot at the draft,
                       * <= -3: row -3 - ref of `hist_e` */
    float *hist_e;    /* [row_width][V_s] mode 4: row under which image token i became final, at i % row_width */
    uint64_t *hist_Z; /* [row_width] */
    float *ref_e;     /* [L][V_s] rows of the previous step */
    uint64_t *ref_Z;  /* [L] */
    oracle_cache *cache[2];
    int32_t done;
} seq_state;

struct oracle_ctx {
    oracle_model_desc md;
    oracle_weights w;
    oracle_sampling sp;
    int32_t max_seqs, n_seqs, Vs, L;
    uint32_t step;
    int prefilled;
    seq_state *seq;
    float *logits;  /* [max_seqs][2][L][V_s] of the last step */
    float *new_e;   /* [L][V_s] scratch */
    uint64_t *new_Z;
};

int oracle_set_num_threads(int32_t n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
    return omp_get_max_threads();
#else
    (void)n;
    return 1;
#endif
}

static void seq_release(seq_state *s) {
    free(s->out); free(s->allow_lo); free(s->allow_hi); free(s->tok); free(s->ref_row); free(s->ref_e); free(s->ref_Z); free(s->hist_e); free(s->hist_Z);
    oracle_cache_free(s->cache[0]);
    oracle_cache_free(s->cache[1]);
    memset(s, 0, sizeof *s);
}

int oracle_create(const oracle_model_desc *md, const oracle_weights *w, const oracle_sampling *sp,
                  int32_t max_seqs, oracle_ctx **out) {
    if (!md || !w || !sp || !out || max_seqs < 1) return EINVAL_;
    if (md->window < 1 || md->n_layers < 1 || md->n_heads < 1 || md->n_kv_heads < 1) return EINVAL_;
    if (md->d_model % md->n_heads || md->n_heads % md->n_kv_heads || (md->d_model / md->n_heads) % 2) return EINVAL_;
    if (md->sample_lo < 0 || md->sample_hi > md->vocab || md->sample_hi <= md->sample_lo) return EINVAL_;
    if (sp->top_k < 1 || !(sp->temperature > 0.0f)) return EINVAL_;
    if (sp->init_mode < 0 || sp->init_mode > 4 || ((sp->init_mode == 2 || sp->init_mode == 4) && sp->row_width < 1)) return EINVAL_;
    oracle_ctx *c = (oracle_ctx *)calloc(1, sizeof *c);
    if (!c) return ENOMEM_;
    c->md = *md; c->w = *w; c->sp = *sp;
    c->max_seqs = max_seqs;
    c->Vs = md->sample_hi - md->sample_lo;
    c->L = md->window;
    c->seq = (seq_state *)calloc((size_t)max_seqs, sizeof(seq_state));
    c->logits = (float *)calloc((size_t)max_seqs * 2 * c->L * c->Vs, sizeof(float));
    c->new_e = (float *)calloc((size_t)c->L * c->Vs, sizeof(float));
    c->new_Z = (uint64_t *)calloc((size_t)c->L, sizeof(uint64_t));
    if (!c->seq || !c->logits || !c->new_e || !c->new_Z) { oracle_destroy(c); return ENOMEM_; }
    *out = c;
    return OK;
}

void oracle_destroy(oracle_ctx *c) {
    if (!c) return;
    if (c->seq) for (int s = 0; s < c->max_seqs; ++s) seq_release(&c->seq[s]);
    free(c->seq); free(c->logits); free(c->new_e); free(c->new_Z);
    free(c);
}

static void philox(const oracle_ctx *c, uint32_t step, uint32_t row, uint32_t seq, uint32_t out[4]) {
    uint32_t ctr[4] = {step, row, seq, 0};
    uint32_t key[2] = {(uint32_t)c->sp.seed, (uint32_t)(c->sp.seed >> 32)};
    oracle_philox4x32_10(ctr, key, out);
}

static int32_t fresh_token(const oracle_ctx *c, uint32_t word3) {
    return c->md.sample_lo + (int32_t)(((uint64_t)word3 * (uint64_t)c->Vs) >> 32);
}

int oracle_prefill(oracle_ctx *c, int32_t n_seqs, const int32_t *const *cond_ids, const int32_t *cond_len,
                   const int32_t *const *uncond_ids, const int32_t *uncond_len,
                   const int32_t *n_image_tokens) {
    if (!c || !cond_ids || !cond_len || !uncond_ids || !uncond_len || !n_image_tokens) return EINVAL_;
    if (n_seqs < 1) return EINVAL_;
    if (n_seqs > c->max_seqs) return ECAPACITY_;
    for (int s = 0; s < n_seqs; ++s) {
        if (cond_len[s] < 1 || uncond_len[s] < 1 || n_image_tokens[s] < 1) return EINVAL_;
        if (cond_len[s] + n_image_tokens[s] > c->md.max_ctx) return ECAPACITY_;
        if (uncond_len[s] + n_image_tokens[s] > c->md.max_ctx) return ECAPACITY_;
        for (int i = 0; i < cond_len[s]; ++i)
            if (cond_ids[s][i] < 0 || cond_ids[s][i] >= c->md.vocab) return EINVAL_;
        for (int i = 0; i < uncond_len[s]; ++i)
            if (uncond_ids[s][i] < 0 || uncond_ids[s][i] >= c->md.vocab) return EINVAL_;
    }
    for (int s = 0; s < c->max_seqs; ++s) seq_release(&c->seq[s]);
    c->n_seqs = n_seqs;
    c->step = 0;
    for (int s = 0; s < n_seqs; ++s) {
        seq_state *q = &c->seq[s];
        q->cond_len = cond_len[s]; q->uncond_len = uncond_len[s]; q->n_image = n_image_tokens[s];
        q->out = (int32_t *)calloc((size_t)q->n_image, sizeof(int32_t));
        q->allow_lo = (int32_t *)calloc((size_t)q->n_image, sizeof(int32_t));
        q->allow_hi = (int32_t *)calloc((size_t)q->n_image, sizeof(int32_t));
        if (!q->allow_lo || !q->allow_hi) return ENOMEM_;
        for (int i = 0; i < q->n_image; ++i) q->allow_hi[i] = c->Vs;   /* no forced tokens until the caller sets some */
        q->tok = (int32_t *)calloc((size_t)c->L, sizeof(int32_t));
        q->ref_row = (int32_t *)calloc((size_t)c->L, sizeof(int32_t));
        q->ref_e = (float *)calloc((size_t)c->L * c->Vs, sizeof(float));
        q->ref_Z = (uint64_t *)calloc((size_t)c->L, sizeof(uint64_t));
        if (c->sp.init_mode == 4) {
            q->hist_e = (float *)calloc((size_t)c->sp.row_width * c->Vs, sizeof(float));
            q->hist_Z = (uint64_t *)calloc((size_t)c->sp.row_width, sizeof(uint64_t));
            if (!q->hist_e || !q->hist_Z) return ENOMEM_;
        }
        q->cache[0] = oracle_cache_new(&c->md);
        q->cache[1] = oracle_cache_new(&c->md);
        if (!q->out || !q->tok || !q->ref_row || !q->ref_e || !q->ref_Z || !q->cache[0] || !q->cache[1]) return ENOMEM_;
        /* all prompt tokens but the last go into the cache; the last one is
         * the first window input */
        const int32_t *ids[2] = {cond_ids[s], uncond_ids[s]};
        const int32_t len[2] = {cond_len[s], uncond_len[s]};
        for (int b = 0; b < 2; ++b) {
            if (len[b] > 1) {
                int rc = oracle_forward(&c->md, &c->w, q->cache[b], ids[b], len[b] - 1, NULL);
                if (rc) return rc;
            }
            q->cache[b]->len = len[b] - 1;
            q->anchor[b] = ids[b][len[b] - 1];
        }
        int32_t Le = q->n_image < c->L ? q->n_image : c->L;
        for (int k = 1; k < Le; ++k) {
            uint32_t r[4];
            philox(c, 0, (uint32_t)k, (uint32_t)s, r);
            q->tok[k] = fresh_token(c, r[3]);
            q->ref_row[k] = -1;
        }
    }
    c->prefilled = 1;
    return OK;
}

int oracle_set_token_ranges(oracle_ctx *c, int32_t seq, const int32_t *first_id, const int32_t *end_id,
                            int32_t n_positions) {
    if (!c || !first_id || !end_id) return EINVAL_;
    if (!c->prefilled) return ESTATE_;
    if (seq < 0 || seq >= c->n_seqs || n_positions < 0 || n_positions > c->seq[seq].n_image) return EINVAL_;
    for (int i = 0; i < n_positions; ++i)
        if (first_id[i] < c->md.sample_lo || end_id[i] > c->md.sample_hi || first_id[i] >= end_id[i]) return EINVAL_;
    for (int i = 0; i < n_positions; ++i) {
        c->seq[seq].allow_lo[i] = first_id[i] - c->md.sample_lo;
        c->seq[seq].allow_hi[i] = end_id[i] - c->md.sample_lo;
    }
    return OK;
}

/* probability weight of token id `tok` under reference of slot k */
static void ref_of(const oracle_ctx *c, const seq_state *q, int k, int32_t tok, uint64_t *w, uint64_t *Z) {
    if (q->ref_row[k] == REF_ONEHOT) { *w = 1; *Z = 1; return; } /* tok is the copied token itself */
    if (q->ref_row[k] <= REF_HIST0) {
        const int h = REF_HIST0 - q->ref_row[k];
        *w = oracle_weight_of(q->hist_e[(size_t)h * c->Vs + (tok - c->md.sample_lo)]);
        *Z = q->hist_Z[h];
        return;
    }
    if (q->ref_row[k] < 0) { *w = 1; *Z = (uint64_t)c->Vs; return; }
    const float *row = q->ref_e + (size_t)q->ref_row[k] * c->Vs;
    *w = oracle_weight_of(row[tok - c->md.sample_lo]);
    *Z = q->ref_Z[q->ref_row[k]];
}

/* Steps 3 and 4 for one sequence, given this step's rows (new_e, new_Z). */
static void decide(oracle_ctx *c, int s, int Le, oracle_step_result *res) {
    seq_state *q = &c->seq[s];
    const int Vs = c->Vs, lo = c->md.sample_lo;
    const uint32_t step = c->step;
    uint32_t r[4];

    /* Step 3: leading run of accepted drafts; draft in slot k against row k-1 */
    int a = 0;
    for (int k = 1; k < Le; ++k) {
        philox(c, step, (uint32_t)(k - 1), (uint32_t)s, r);
        int32_t x = q->tok[k];
        uint64_t wq, Zq;
        ref_of(c, q, k, x, &wq, &Zq);
        uint64_t wp = oracle_weight_of(c->new_e[(size_t)(k - 1) * Vs + (x - lo)]);
        if (!oracle_accept(r[0], wp, c->new_Z[k - 1], wq, Zq)) break;
        a += 1;
    }
    const int rejected = a < Le - 1;

    /* Step 4, first unaccepted position: residual draw (or a plain draw from
     * the last row when nothing was rejected) */
    philox(c, step, (uint32_t)a, (uint32_t)s, r);
    uint64_t u64 = ((uint64_t)r[1] << 32) | r[2];
    const float *pa = c->new_e + (size_t)a * Vs;
    int32_t y;
    if (rejected) {
        int rr = q->ref_row[a + 1];
        const float *qe = rr < 0 ? NULL : q->ref_e + (size_t)rr * Vs;
        uint64_t qZ = rr < 0 ? 0 : q->ref_Z[rr];
        if (rr <= REF_HIST0) { qe = q->hist_e + (size_t)(REF_HIST0 - rr) * Vs; qZ = q->hist_Z[REF_HIST0 - rr]; }
        if (rr == REF_ONEHOT) y = lo + oracle_draw_residual_onehot(pa, c->new_Z[a], q->tok[a + 1] - lo, Vs, u64);
        else y = lo + oracle_draw_residual(pa, c->new_Z[a], qe, qZ, Vs, u64);
    } else {
        y = lo + oracle_draw(pa, c->new_Z[a], Vs, u64);
    }

    for (int k = 1; k <= a; ++k) q->out[q->n_img + k - 1] = q->tok[k];
    q->out[q->n_img + a] = y;
    if (c->sp.init_mode == 4) /* image token n_img + i became final under row i of this step */
        for (int i = 0; i <= a; ++i) {
            const int h = (q->n_img + i) % c->sp.row_width;
            memcpy(q->hist_e + (size_t)h * Vs, c->new_e + (size_t)i * Vs, sizeof(float) * (size_t)Vs);
            q->hist_Z[h] = c->new_Z[i];
        }
    q->n_img += a + 1;
    q->cache[0]->len += a + 1;
    q->cache[1]->len += a + 1;

    res->n_accepted = a;
    res->n_finalized = a + 1;
    res->reject_index = rejected ? a + 1 : -1;

    const int remaining = q->n_image - q->n_img;
    if (remaining == 0) {
        q->done = 1;
        res->done = 1;
        return;
    }
    res->done = 0;

    /* next window: slot k' holds what was slot k = k' + a + 1 */
    const int Le2 = remaining < c->L ? remaining : c->L;
    int32_t *tok2 = (int32_t *)malloc(sizeof(int32_t) * (size_t)c->L);
    int32_t *ref2 = (int32_t *)malloc(sizeof(int32_t) * (size_t)c->L);
    for (int k2 = 1; k2 < Le2; ++k2) {
        int k = k2 + a + 1;
        if (k <= Le - 1) {
            /* Eq. 4-5 at a later position: draft of slot k, row k-1 */
            int32_t x = q->tok[k];
            uint64_t wq, Zq;
            ref_of(c, q, k, x, &wq, &Zq);
            const float *prow = c->new_e + (size_t)(k - 1) * Vs;
            if (oracle_keep(c->sp.reuse_tau, oracle_weight_of(prow[x - lo]), c->new_Z[k - 1], wq, Zq)) {
                tok2[k2] = x;
            } else {
                philox(c, step, (uint32_t)(k - 1), (uint32_t)s, r);
                tok2[k2] = lo + oracle_draw(prow, c->new_Z[k - 1], Vs, ((uint64_t)r[1] << 32) | r[2]);
            }
            ref2[k2] = k - 1;
        } else if (k == Le) {
            /* the last row had no draft: its slot is drawn from that row */
            philox(c, step, (uint32_t)(Le - 1), (uint32_t)s, r);
            tok2[k2] = lo + oracle_draw(c->new_e + (size_t)(Le - 1) * Vs, c->new_Z[Le - 1], Vs,
                                        ((uint64_t)r[1] << 32) | r[2]);
            ref2[k2] = Le - 1;
        } else {
            /* a slot that never had a draft (Sec. 4.2); image index of its token: n_img + k2 - 1 */
            const int mode = c->sp.init_mode, up = q->n_img + k2 - 1 - c->sp.row_width;
            philox(c, step, (uint32_t)k, (uint32_t)s, r);
            if (mode == 1) {
                tok2[k2] = k2 == 1 ? y : tok2[k2 - 1];
                ref2[k2] = REF_ONEHOT;
            } else if (mode == 2 && c->sp.row_width >= 1 && up >= 0) {
                tok2[k2] = up < q->n_img ? q->out[up] : tok2[up - q->n_img + 1];
                ref2[k2] = REF_ONEHOT;
            } else if (mode == 4 && up >= 0) {
                /* the distribution of the token one image row above: final -> the kept row; still a draft of this
                 * window -> whatever that slot's reference is (a row of this step, a kept row, or uniform) */
                const int ref = up < q->n_img ? REF_HIST0 - up % c->sp.row_width : ref2[up - q->n_img + 1];
                const uint64_t u = ((uint64_t)r[1] << 32) | r[2];
                if (ref == REF_UNIFORM) tok2[k2] = fresh_token(c, r[3]);
                else if (ref >= 0) tok2[k2] = lo + oracle_draw(c->new_e + (size_t)ref * Vs, c->new_Z[ref], Vs, u);
                else tok2[k2] = lo + oracle_draw(q->hist_e + (size_t)(REF_HIST0 - ref) * Vs, q->hist_Z[REF_HIST0 - ref], Vs, u);
                ref2[k2] = ref;
            } else if (mode == 3) {
                /* its left neighbour (or that one's, ...) was drawn from the last row of this step */
                tok2[k2] = lo + oracle_draw(c->new_e + (size_t)(Le - 1) * Vs, c->new_Z[Le - 1], Vs,
                                            ((uint64_t)r[1] << 32) | r[2]);
                ref2[k2] = Le - 1;
            } else {
                tok2[k2] = fresh_token(c, r[3]);
                ref2[k2] = REF_UNIFORM;
            }
        }
    }
    q->anchor[0] = q->anchor[1] = y;
    for (int k2 = 1; k2 < Le2; ++k2) { q->tok[k2] = tok2[k2]; q->ref_row[k2] = ref2[k2]; }
    for (int k2 = Le2; k2 < c->L; ++k2) { q->tok[k2] = 0; q->ref_row[k2] = -1; }
    memcpy(q->ref_e, c->new_e, sizeof(float) * (size_t)Le * Vs);
    memcpy(q->ref_Z, c->new_Z, sizeof(uint64_t) * (size_t)Le);
    free(ref2);
    free(tok2);
}

/* Step 2 for sequence s: both branches over the current window; fills
 * c->logits[s] (rows >= Le are zero).  Writes keys/values at the tentative
 * positions cache->len .. cache->len + Le - 1 without committing them. */
static int forward_current(oracle_ctx *c, int s, int Le) {
    seq_state *q = &c->seq[s];
    const int L = c->L, Vs = c->Vs;
    float *lg = c->logits + (size_t)s * 2 * L * Vs;
    int32_t *win = (int32_t *)malloc(sizeof(int32_t) * (size_t)L);
    memset(lg, 0, sizeof(float) * (size_t)2 * L * Vs);
    int rc = 0;
    for (int b = 0; b < 2 && rc == 0; ++b) {
        win[0] = q->anchor[b];
        for (int k = 1; k < Le; ++k) win[k] = q->tok[k];
        rc = oracle_forward(&c->md, &c->w, q->cache[b], win, Le, lg + (size_t)b * L * Vs);
    }
    free(win);
    return rc;
}

static int step_impl(oracle_ctx *c, const float *given_logits, oracle_step_result *out) {
    if (!c || !out) return EINVAL_;
    if (!c->prefilled) return ESTATE_;
    const int L = c->L, Vs = c->Vs;
    c->step += 1;
    for (int s = 0; s < c->n_seqs; ++s) {
        seq_state *q = &c->seq[s];
        oracle_step_result *res = &out[s];
        if (q->done) {
            res->n_accepted = 0; res->n_finalized = 0; res->reject_index = -1; res->done = 1;
            continue;
        }
        const int remaining = q->n_image - q->n_img;
        const int Le = remaining < L ? remaining : L;
        float *lg = c->logits + (size_t)s * 2 * L * Vs;
        if (given_logits) {
            memcpy(lg, given_logits + (size_t)s * 2 * L * Vs, sizeof(float) * (size_t)2 * L * Vs);
        } else {
            int rc = forward_current(c, s, Le);
            if (rc) return rc;
        }
        for (int k = 0; k < Le; ++k) /* row k is the distribution of image position n_img + k */
            oracle_sampling_row_range(lg + (size_t)k * Vs, lg + (size_t)(L + k) * Vs, Vs, c->sp.cfg_scale,
                                      c->sp.temperature, c->sp.top_k, q->allow_lo[q->n_img + k], q->allow_hi[q->n_img + k],
                                      c->new_e + (size_t)k * Vs, &c->new_Z[k]);
        decide(c, s, Le, res);
    }
    return OK;
}

/* The forward of the coming step only (no decision, no state change other
 * than the tentative cache rows): logits [n_seqs][2][L][V_s]. */
int oracle_peek_logits(oracle_ctx *c, float *dst) {
    if (!c || !dst) return EINVAL_;
    if (!c->prefilled) return ESTATE_;
    const int L = c->L, Vs = c->Vs;
    for (int s = 0; s < c->n_seqs; ++s) {
        seq_state *q = &c->seq[s];
        float *lg = c->logits + (size_t)s * 2 * L * Vs;
        if (q->done) { memset(lg, 0, sizeof(float) * (size_t)2 * L * Vs); continue; }
        const int remaining = q->n_image - q->n_img;
        int rc = forward_current(c, s, remaining < L ? remaining : L);
        if (rc) return rc;
    }
    memcpy(dst, c->logits, sizeof(float) * (size_t)c->n_seqs * 2 * L * Vs);
    return OK;
}

int oracle_step(oracle_ctx *c, oracle_step_result *out) { return step_impl(c, NULL, out); }

int oracle_step_from_logits(oracle_ctx *c, const float *logits, oracle_step_result *out) {
    if (!logits) return EINVAL_;
    return step_impl(c, logits, out);
}

int oracle_copy_logits(oracle_ctx *c, float *dst) {
    if (!c || !dst) return EINVAL_;
    memcpy(dst, c->logits, sizeof(float) * (size_t)c->n_seqs * 2 * c->L * c->Vs);
    return OK;
}

int oracle_get_tokens(oracle_ctx *c, int32_t seq, int32_t *dst, int32_t cap, int32_t *n_out) {
    if (!c || seq < 0 || seq >= c->n_seqs || !n_out) return EINVAL_;
    const seq_state *q = &c->seq[seq];
    int n = q->n_img < cap ? q->n_img : cap;
    if (dst) memcpy(dst, q->out, sizeof(int32_t) * (size_t)n);
    *n_out = q->n_img;
    return OK;
}

int oracle_get_window(oracle_ctx *c, int32_t seq, int32_t *tokens, int32_t *ref_rows, int32_t *n_slots) {
    if (!c || seq < 0 || seq >= c->n_seqs || !tokens || !ref_rows || !n_slots) return EINVAL_;
    const seq_state *q = &c->seq[seq];
    int remaining = q->n_image - q->n_img;
    int Le = remaining < c->L ? remaining : c->L;
    tokens[0] = q->anchor[0];
    ref_rows[0] = -1;
    for (int k = 1; k < c->L; ++k) { tokens[k] = k < Le ? q->tok[k] : 0; ref_rows[k] = k < Le ? q->ref_row[k] : -1; }
    *n_slots = Le;
    return OK;
}

/* Statistical helper for the end-to-end Theorem-1 pin: decodes one prompt
 * n_trials times with seeds seed0, seed0 + 1, ... and histograms the decoded
 * sequences, indexed sum_i (token_i - sample_lo) * V_s^i.  *n_steps receives
 * the total number of oracle_step calls. */
int oracle_decode_trials(const oracle_model_desc *md, const oracle_weights *w, const oracle_sampling *sp,
                         const int32_t *cond, int32_t cond_len, const int32_t *uncond, int32_t uncond_len,
                         int32_t n_image, uint64_t seed0, int64_t n_trials, int64_t *counts, int64_t *n_steps) {
    int64_t steps = 0;
    const int Vs = md->sample_hi - md->sample_lo;
    for (int64_t t = 0; t < n_trials; ++t) {
        oracle_sampling local = *sp;
        local.seed = seed0 + (uint64_t)t;
        oracle_ctx *c = NULL;
        int rc = oracle_create(md, w, &local, 1, &c);
        if (rc) return rc;
        rc = oracle_prefill(c, 1, &cond, &cond_len, &uncond, &uncond_len, &n_image);
        oracle_step_result res = {0, 0, 0, 0};
        while (rc == 0 && !res.done) {
            rc = oracle_step(c, &res);
            steps += 1;
        }
        if (rc) { oracle_destroy(c); return rc; }
        int64_t index = 0, mul = 1;
        for (int i = 0; i < n_image; ++i) {
            index += (int64_t)(c->seq[0].out[i] - md->sample_lo) * mul;
            mul *= Vs;
        }
        counts[index] += 1;
        oracle_destroy(c);
    }
    *n_steps = steps;
    return OK;
}
