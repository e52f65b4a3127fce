// Host-side launch interface of the decision stage (sampling distribution, verification,
// residual / refresh draws, window update).  Implemented in decide.hip, which is compiled with
// floating-point contraction off: its results are specified bit for bit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sjd.h"

// Device-resident decoding state of a context (all pointers are device pointers).
struct DecideState {
    int32_t L;         // window
    int32_t V;         // sampled vocabulary size V_s
    int32_t lo;        // sample_lo
    int32_t max_img;   // capacity of out_tok per sequence
    int32_t *win_tok;  // [S][L]   window tokens (slot 0 unused)
    int32_t *anchor;   // [S][2]   first window input of the cond / uncond branch
    int32_t *ref_row;  // [S][L]   slot -> reference row of the previous step, -1 = uniform, -2 = one-hot at the draft,
                       //          <= -3: kept row -3 - ref (hist_*)
    int32_t *n_img;    // [S]      image tokens final so far
    int32_t *n_image;  // [S]      image tokens wanted
    int32_t *kv_len;   // [S][2]   committed cache positions per branch
    int32_t *Le;       // [S]      effective window of the coming / current step, 0 = done or unused
    int32_t *out_tok;  // [S][max_img]
    int32_t *acc_len;  // [S]      accepted drafts of the current step
    int32_t *cand;     // [S][L]   per output row: the token drawn (or kept) there this step
    int32_t *cand_new; // [S][L]   per slot of the NEXT window: the draw for a slot that never had a draft (init_mode 3)
    uint32_t *step;    // [1]      step counter (0 after prefill)
    // Rows of the sampling distribution, stored as the kept (id, weight) pairs in ascending id order: top-K leaves a
    // few thousand of V entries.  A row has room for `cap` = V pairs (ties at the K-th value, or K >= V, can keep a
    // whole row); only the first cnt are ever written or read.  Ping-pong by step parity: this step's rows and the
    // previous step's, which are the references of the window's drafts.
    int32_t cap;
    int32_t *ids_buf[2]; // [S][L][cap] ids relative to sample_lo
    float *e_buf[2];     // [S][L][cap] softmax weights EXP(z - max z)
    int32_t *cnt_buf[2]; // [S][L]
    uint64_t *Z_buf[2];  // [S][L] integer normalisers
    // init_mode 4: the row under which image token i became final, at i % row_width
    int32_t *hist_ids;   // [S][row_width][cap]
    float *hist_e;       // [S][row_width][cap]
    int32_t *hist_cnt;   // [S][row_width]
    uint64_t *hist_Z;    // [S][row_width]
    // Forced-token masks: image position i of sequence s may only take ids in [allow_lo, allow_hi) (relative to
    // sample_lo); every other id has probability 0 there.  [S][max_img]; the whole range by default.
    int32_t *allow_lo, *allow_hi;
    sjd_step_result *res; // [S]
};

struct SamplingParams {
    float cfg_scale, inv_temperature, tau;
    int32_t top_k;
    uint64_t seed;
    int32_t init_mode, row_width;  // Sec. 4.2 initialisation of new slots (see sjd_sampling)
};

// Rows of the forward: token and position per GEMM row, cache length and active rows per segment
// (segment = sequence * 2 + branch).
struct RowMap {
    int32_t *row_tok;  // [S*2*L]  token id, -1 = inactive row
    int32_t *row_pos;  // [S*2*L]
    int32_t *seg_kv;   // [S*2]
    int32_t *seg_n;    // [S*2]
};

hipError_t launch_init_window(hipStream_t st, const DecideState &d, const SamplingParams &sp, int n_seqs, int max_seqs,
                              const int32_t *prompt_last /*[S][2]*/, const int32_t *prompt_len /*[S][2]*/,
                              const int32_t *n_image /*[S]*/);
hipError_t launch_stage_window(hipStream_t st, const DecideState &d, const RowMap &rm, int n_seqs);
hipError_t launch_stage_prompt(hipStream_t st, const RowMap &rm, const int32_t *prompt /*[S][2][max_prompt]*/,
                               const int32_t *prompt_len, int max_prompt, int chunk, int L, int n_seqs);
// logits: [n_seqs][2][L][V]; z (may be NULL): the guided logits [n_seqs][L][V] already combined by the vocabulary head,
// read instead of the logits
hipError_t launch_sample_rows(hipStream_t st, const DecideState &d, const SamplingParams &sp, const float *logits,
                              int n_seqs, const float *z);
hipError_t launch_verify(hipStream_t st, const DecideState &d, const SamplingParams &sp, int n_seqs);
hipError_t launch_draw(hipStream_t st, const DecideState &d, const SamplingParams &sp, int n_seqs);
hipError_t launch_commit(hipStream_t st, const DecideState &d, const SamplingParams &sp, int n_seqs);
// init_mode 4 only, between launch_draw and launch_commit: keeps the rows under which this step's tokens became final
hipError_t launch_keep_rows(hipStream_t st, const DecideState &d, const SamplingParams &sp, int n_seqs);

// stand-alone forms for kernel tests
// rows of [V] logits -> kept pairs ids / e [rows][V] (ascending ids), cnt [rows], Z [rows]; allow_lo / allow_hi [rows]
// (may be NULL) restrict row r to ids in [allow_lo[r], allow_hi[r])
hipError_t launch_sampling_rows_plain(hipStream_t st, const float *lc, const float *lu, int32_t *ids, float *e, int32_t *cnt,
                                      uint64_t *Z, int rows, int V, const SamplingParams &sp, const int32_t *allow_lo,
                                      const int32_t *allow_hi);
// e_dense [rows][V] (zero-filled by the caller) <- the kept pairs
hipError_t launch_scatter_rows(hipStream_t st, const int32_t *ids, const float *e, const int32_t *cnt, float *e_dense, int rows,
                               int V);
hipError_t launch_philox_fill(hipStream_t st, uint64_t seed, uint32_t row, uint32_t seq, uint32_t *out, int n);
