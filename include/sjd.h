/*
 * sjd -- speculative Jacobi decoding (SJD++) of a discrete autoregressive
 * image-token transformer on one AMD MI355X (gfx950).  C ABI.
 *
 * The library decodes image tokens after a text prompt with the iteration of
 * Sec. 4.1 of the paper (the speculative Jacobi iteration): a window of L tokens
 * (the last final token followed by L-1 drafts) is run through ONE causal
 * forward of the transformer against a paged KV cache, as a conditional /
 * unconditional pair for classifier-free guidance (Sec. 5.1: guidance weight,
 * top-K); drafts are accepted left to right with probability min(1, p/q)
 * (Eq. 2), the first unaccepted position is redrawn from the residual
 * normalise(max(0, p - q)) (Eq. 3), and each later draft is kept when its
 * confidence p/q exceeds tau and redrawn from p otherwise (Eq. 4-5; tau = +inf
 * is the rule without reuse, Eq. 6).
 *
 * Conventions
 *  - every function returns SJD_OK (0) or a negative sjd_status and never
 *    throws or aborts; sjd_last_error() gives a text for the last failure of a
 *    context (or of sjd_create when passed NULL);
 *  - "device" pointers are HIP device pointers on the current device, "host"
 *    pointers are ordinary process memory;
 *  - hip_stream is a hipStream_t passed as void* (NULL = the default stream);
 *    it is borrowed and must outlive the context; all work of a context is
 *    enqueued on it.  On an ordinary stream sjd_step records its launches once
 *    (stream capture, thread-local mode) and replays them as a HIP graph; on
 *    the default stream, which cannot be captured, it launches them one by one;
 *  - a context is not thread-safe; different contexts are independent.
 */
#ifndef SJD_H
#define SJD_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sjd_ctx sjd_ctx;

enum sjd_status {
    SJD_OK = 0,
    SJD_EINVAL = -1,    /* bad argument or unsupported shape          */
    SJD_ENOMEM = -2,    /* device or host allocation failed           */
    SJD_ESTATE = -3,    /* call order violated                        */
    SJD_EDEVICE = -4,   /* a HIP call failed                          */
    SJD_ECAPACITY = -5  /* more sequences / context than created for  */
};

enum sjd_dtype { SJD_F32 = 0, SJD_BF16 = 1 };

/* kernel_flags bits */
enum {
    SJD_KERNELS_REFERENCE = 1, /* use the plain (non-MFMA) GEMM and attention kernels */
    SJD_NO_GRAPH = 2,          /* never capture the step into a HIP graph: launch its
                                * kernels one by one                                   */
    SJD_KERNELS_ROWGROUPS = 4, /* bf16, >= 256 rows: keep the 64-row-group streaming projection
                                * kernels instead of the LDS-staged tile kernels       */
    SJD_ATTENTION_CHUNKED = 8, /* bf16: always split the context over workgroups and merge
                                * in a second kernel, also where one workgroup per head
                                * would do (short contexts)                            */
    SJD_KERNELS_TILES = 16,    /* bf16, >= 256 rows: the tile kernels also for models too
                                * narrow to fill the chip with 256 x 128 tiles         */
    SJD_NO_L2_WARM = 32,       /* bf16, <= 64 rows: projection launches carry no extra
                                * workgroups that touch the next launch's weights and
                                * key/value pages into L2 (same results either way)    */
    SJD_TILES_256_ROWS = 64,   /* bf16, >= 256 rows: every tile kernel launch uses 256-row
                                * workgroup tiles (default: 128-row tiles where they
                                * balance the CUs better)                              */
    SJD_NO_ROW_SPLIT = 128,    /* bf16, 17..32 rows: projections of at most 64 column groups
                                * with one workgroup per group (default: two, 16 rows each);
                                * more rows: 64-row groups also for projections of so few
                                * column groups that 32-row groups would each get a CU     */
    SJD_NO_MIXED_WIDTH = 256,  /* bf16: no launch mixes workgroup shapes.  <= 64 rows: gate/up and
                                * head projections of more than 256 column groups with one
                                * workgroup per group (default: one workgroup per CU, some of
                                * them two groups wide); >= 256 rows: one tile height per launch
                                * (default: 256-row tiles on every CU with the remaining column
                                * tiles as 128-row tiles beside them, where the 256-row tiles
                                * number between one and two per CU)                    */
    SJD_KEEP_LOGITS = 1024,    /* keep the fp32 logits of every step for sjd_debug_copy_logits.  Without it the
                                * vocabulary head of the fused bf16 path writes only the guided logits
                                * z = (l_u + s (l_c - l_u)) / T of each position (windows of 32, or one sequence
                                * with a window of 16), which is all the sampling stage reads            */
    SJD_NO_HEAD_FUSION = 2048, /* the vocabulary head always writes the logits and the sampling kernel combines the
                                * two branches (same results either way)                                 */
    SJD_NO_K_ROTATION = 512    /* bf16, row-group projection kernels: every workgroup walks K
                                * from 0 (default: each starts at its own offset and wraps,
                                * so that they do not all ask for the same activation lines
                                * at the same time; sums differ in the last bits only)  */
};

/* Architecture and capacities; plain data, copied by sjd_create.
 * Pre-norm decoder blocks: RMSNorm, rotary embedding on q and k (rotate-half
 * pairing (i, i + hd/2), angle pos * rope_theta^(-2i/hd)), grouped-query
 * attention with scale 1/sqrt(hd), SwiGLU MLP, final RMSNorm, untied head.
 * The paper fixes none of this (Sec. 3.1 only asks for a transformer that
 * predicts a categorical distribution); it is the shape of the workloads. */
typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, d_ff;
    int32_t vocab, sample_lo, sample_hi; /* token ids in [sample_lo, sample_hi) are sampled */
    float rms_eps, rope_theta;
    int32_t dtype;           /* sjd_dtype: storage of weights, activations fed to GEMMs, KV cache */
    int32_t max_seqs;        /* prompts decoded together (each is a cond + uncond pair) */
    int32_t max_ctx;         /* positions per branch: prompt + image tokens             */
    int32_t window;          /* L >= 1: the last final token + L-1 drafts              */
    int32_t kv_page_tokens;  /* tokens per KV page; multiple of 32; 0 = 64              */
    int32_t kernel_flags;
} sjd_model_desc;

/* DEVICE pointers to weights of type `dtype`.  Linear weights are
 * [out_features][in_features] row-major (y = W x); per-layer members are HOST
 * arrays of n_layers device pointers.  sjd_create copies (and re-lays-out)
 * everything it needs: nothing is referenced after it returns. */
typedef struct {
    const void *tok_emb;    /* [vocab][d_model] */
    const void *final_norm; /* [d_model]        */
    const void *lm_head;    /* [vocab][d_model] */
    const void *const *attn_norm; /* [d_model]                     */
    const void *const *wq;        /* [n_heads*hd][d_model]         */
    const void *const *wk;        /* [n_kv_heads*hd][d_model]      */
    const void *const *wv;        /* [n_kv_heads*hd][d_model]      */
    const void *const *wo;        /* [d_model][n_heads*hd]         */
    const void *const *mlp_norm;  /* [d_model]                     */
    const void *const *w_gate;    /* [d_ff][d_model]               */
    const void *const *w_up;      /* [d_ff][d_model]               */
    const void *const *w_down;    /* [d_model][d_ff]               */
} sjd_weights;

/* Sampling distribution and decoding rule (Sec. 5.1).
 * p = softmax over the top_k largest of z = (l_u + cfg_scale (l_c - l_u)) /
 * temperature (ties at the k-th value kept).  Randomness is Philox4x32-10 keyed
 * by `seed` with counter (step, row, sequence, 0). */
typedef struct {
    float cfg_scale, temperature;
    int32_t top_k;
    float reuse_tau;  /* 0.5 in the paper; +INF disables reuse (Eq. 6) */
    uint64_t seed;
    /* Sec. 4.2, how a window slot that has never had a draft is filled (slots of the first window, before any image
     * token exists, are always uniform):
     *   0  drawn uniformly over the sampled ids (reference: uniform);
     *   1  copy of the token to its left (reference: one-hot at that token);
     *   2  copy of the token one image row above, row_width tokens back (one-hot; uniform in the first row);
     *   3  drawn from the distribution its left neighbour was drawn from, i.e. the last row of the step
     *      (reference: that row);
     *   4  drawn from the distribution of the token one image row above: the row under which that token became
     *      final (the context keeps the last row_width of them per sequence), or the reference of the draft at
     *      that place if it is still in the window (reference: the same; uniform in the first image row). */
    int32_t init_mode;
    int32_t row_width; /* tokens per image row; used by init_mode 2 and 4 (>= 1 there) */
} sjd_sampling;

typedef struct {
    int32_t n_accepted;   /* drafts accepted this step (Eq. 2)                          */
    int32_t n_finalized;  /* tokens made final this step = n_accepted + 1, 0 if done    */
    int32_t reject_index; /* window slot of the first rejected draft, -1 if none        */
    int32_t done;         /* 1 once all image tokens of the sequence are final          */
} sjd_step_result;

/* Creates a context on the current device: allocates KV pages for
 * max_seqs * 2 * max_ctx positions, workspaces and decoding state; copies the
 * weights.  Errors: SJD_EINVAL (null pointer, unsupported shape: bf16 needs
 * hd % 32 == 0, d_model % 16 == 0, d_ff % 16 == 0), SJD_ENOMEM, SJD_EDEVICE. */
int sjd_create(const sjd_model_desc *desc, const sjd_weights *weights, const sjd_sampling *sampling,
               void *hip_stream, sjd_ctx **out);

/* Starts n_seqs decodes (Sec. 4.1: the text prompt is run through the model first).  All
 * arrays are HOST arrays of length n_seqs, read during the call only.  Every
 * prompt token but the last is run through the model into the KV cache; the
 * last one becomes the first window input; the L-1 drafts are drawn uniformly.
 * May be called again to start new decodes.  Errors: SJD_EINVAL (null, length
 * < 1, id outside the vocabulary), SJD_ECAPACITY (n_seqs > max_seqs or
 * prompt + image tokens > max_ctx; nothing is enqueued), SJD_EDEVICE. */
int sjd_prefill(sjd_ctx *ctx, int32_t n_seqs, const int32_t *const *cond_ids, const int32_t *cond_len,
                const int32_t *const *uncond_ids, const int32_t *uncond_len, const int32_t *n_image_tokens);

/* One speculative Jacobi iteration for every unfinished sequence (Sec. 4.1
 * Steps 1-4).  out is a HOST array of n_seqs results.  The call returns after
 * the step has completed on the device.  Sequences that are done are left
 * untouched (n_finalized = 0, done = 1).  Errors: SJD_ESTATE (no prefill),
 * SJD_EINVAL, SJD_EDEVICE. */
int sjd_step(sjd_ctx *ctx, sjd_step_result *out);

/* Frees everything the context owns.  NULL is allowed. */
void sjd_destroy(sjd_ctx *ctx);

/* Copies the image tokens of sequence `seq` that are final so far into dst
 * (HOST, capacity cap, may be NULL when cap == 0); *n_out receives their count. */
int sjd_get_tokens(sjd_ctx *ctx, int32_t seq, int32_t *dst, int32_t cap, int32_t *n_out);

/* Current window of sequence `seq` (HOST arrays of length `window`): tokens
 * (slot 0 = last final token) and per slot the output row of the previous step
 * that is its reference distribution (-1 = uniform); *n_slots = slots in use. */
int sjd_get_window(sjd_ctx *ctx, int32_t seq, int32_t *tokens, int32_t *ref_rows, int32_t *n_slots);

/* Forced tokens (structure tokens of an image grammar, such as the end-of-row
 * token that closes every row of a 48 x 49 token image): image position i of
 * sequence `seq` may only take ids in [first_id[i], end_id[i]), i < n_positions
 * (HOST arrays; absolute ids inside [sample_lo, sample_hi)).  Ids outside the
 * range get probability 0 at that position before top-K (Sec. 3.1) is applied,
 * so a range of one id forces that token.  Drafts are still initialised over all
 * sampled ids; one that falls outside its position's range has p = 0 and is
 * rejected by Eq. 2 with certainty.  Call after sjd_prefill (which resets every
 * position to the whole sampled range); positions >= n_positions keep theirs.
 * Errors: SJD_ESTATE (no prefill), SJD_EINVAL (bad index, empty range, range
 * outside the sampled ids, n_positions > image tokens of the sequence). */
int sjd_set_token_ranges(sjd_ctx *ctx, int32_t seq, const int32_t *first_id, const int32_t *end_id, int32_t n_positions);

const char *sjd_last_error(const sjd_ctx *ctx);

/* fp32 logits of the last step, [n_seqs][2 (cond, uncond)][window][V_s],
 * V_s = sample_hi - sample_lo, to HOST memory.  SJD_ESTATE when the context does
 * not keep them (created without SJD_KEEP_LOGITS and its head writes guided
 * logits only). */
int sjd_debug_copy_logits(sjd_ctx *ctx, float *dst_host);

/* Runs Steps 3-4 on caller-provided logits (HOST, layout as above) instead of
 * the forward: the KV cache is not written, its length advances as usual. */
int sjd_debug_step_from_logits(sjd_ctx *ctx, const float *logits_host, sjd_step_result *out);

/* Snapshot of the decoding state of the current batch, to HOST memory and back.
 * What Sec. 4.1 carries from one iteration to the next is small and explicit:
 * the accepted tokens, the window's drafts with the distributions they were
 * drawn from (the previous iteration's rows), the step counter that indexes the
 * random stream, and the cache of the accepted prefix.  A snapshot holds exactly
 * that (cache pages of accepted positions only), so a half-decoded batch can be
 * parked and resumed, or rolled back: after sjd_snapshot_restore the following
 * sjd_step calls return what they returned after sjd_snapshot_save, bit for bit.
 *   sjd_snapshot_size     *bytes = size a save would write now (it grows with
 *                         the accepted prefix).
 *   sjd_snapshot_save     writes the snapshot to dst_host (cap bytes available);
 *                         *written = its size.  SJD_ECAPACITY if cap is too small.
 *   sjd_snapshot_restore  src_host / bytes as written by a save on a context
 *                         created with the same model description and sampling
 *                         parameters (anything else, a truncated or altered
 *                         buffer: SJD_EINVAL, context unchanged).  Replaces
 *                         whatever batch the context held; no prefill needed.
 * All three return after the copies completed; SJD_ESTATE before the first
 * prefill (size, save).  The buffer is plain bytes owned by the caller; its
 * format is private to the library version that wrote it. */
int sjd_snapshot_size(sjd_ctx *ctx, uint64_t *bytes);
int sjd_snapshot_save(sjd_ctx *ctx, void *dst_host, uint64_t cap, uint64_t *written);
int sjd_snapshot_restore(sjd_ctx *ctx, const void *src_host, uint64_t bytes);

/* Per-kernel timing.  With tracing on, sjd_step brackets every kernel launch
 * with HIP events on the context's stream and accumulates their durations.
 * sjd_trace_read copies up to cap entries: name (static string), number of
 * launches, total milliseconds; *n_out = number of kernel classes. */
typedef struct {
    const char *name;
    int64_t launches;
    double total_ms;
} sjd_trace_entry;
int sjd_trace_enable(sjd_ctx *ctx, int32_t on);
int sjd_trace_reset(sjd_ctx *ctx);
int sjd_trace_read(sjd_ctx *ctx, sjd_trace_entry *dst, int32_t cap, int32_t *n_out);

/* ---- single operations, for kernel-level tests and microbenchmarks.
 * All pointers are DEVICE pointers in plain row-major layouts; the calls
 * allocate temporaries, run on `hip_stream` and return after completion. */

/* C[M][N] (fp32) = A[M][K] * W[N][K]^T with the GEMM kernel the decoder uses
 * for `dtype` (reference kernel if flags has SJD_KERNELS_REFERENCE).
 * splits <= 0 lets the library choose the split-K factor.  `repeat` >= 1
 * launches the kernel that many times; *avg_ms (HOST, may be NULL) receives the
 * mean kernel time measured with HIP events. */
int sjd_op_gemm(void *hip_stream, int32_t dtype, int32_t flags, const void *A, const void *W, float *C, int32_t M,
                int32_t N, int32_t K, int32_t splits, int32_t repeat, float *avg_ms);

/* sjd_op_gemm for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels,
 * with the temporaries (both operands re-laid-out for the kernels and the split-K
 * partial sums) in a 32 MiB workspace that is part of the library image on every
 * device.  The call allocates nothing, creates no events and returns after completion.
 * SJD_ECAPACITY when the temporaries of M x N x K exceed the workspace
 * (bf16: 2 (ceil32(M) + ceil32(N)) K + 4 splits M N bytes, each part rounded up to 256).
 * All calls on one device share the workspace: calls that overlap on one device
 * (different streams or threads) race; serialise them. */
int sjd_op_gemm_static(void *hip_stream, int32_t dtype, int32_t flags, const void *A, const void *W, float *C, int32_t M,
                       int32_t N, int32_t K, int32_t splits);

/* Window attention of one (sequence, branch): q [n][H][hd], k and v
 * [ctx + n][Hkv][hd] of `dtype` (the first ctx positions are the cache, the
 * last n the window), out [n][H][hd] fp32.  Query i sees positions
 * 0 .. ctx + i. */
int sjd_op_window_attention(void *hip_stream, int32_t dtype, int32_t flags, const void *q, const void *k,
                            const void *v, float *out, int32_t n, int32_t ctx, int32_t n_heads,
                            int32_t n_kv_heads, int32_t head_dim, int32_t page_tokens, int32_t repeat,
                            float *avg_ms);

/* Sampling distribution of `rows` positions (Sec. 3.1 top-K sampling with the
 * guidance weight of Sec. 5.1): logits_c / logits_u [rows][V] fp32 -> e [rows][V]
 * fp32 softmax weights (0 outside the top-k set) and Z [rows] uint64 integer
 * normalisers.  allow_lo / allow_hi (DEVICE [rows], both or neither NULL): row r
 * may only keep ids in [allow_lo[r], allow_hi[r]).  kept_ids [rows][V] and
 * kept_cnt [rows] (DEVICE, may be NULL) receive the form in which the decoder
 * stores a row: the ids with a weight, ascending, and their number. */
int sjd_op_sampling_rows(void *hip_stream, const float *logits_c, const float *logits_u, float *e, uint64_t *Z,
                         int32_t rows, int32_t V, float cfg_scale, float temperature, int32_t top_k,
                         const int32_t *allow_lo, const int32_t *allow_hi, int32_t *kept_ids, int32_t *kept_cnt,
                         int32_t repeat, float *avg_ms);

/* out[4*i .. 4*i+3] = Philox4x32-10(counter = (i, row, seq, 0), key = seed), i < n. */
int sjd_op_philox(void *hip_stream, uint64_t seed, uint32_t row, uint32_t seq, uint32_t *out, int32_t n);

#ifdef __cplusplus
}
#endif
#endif
