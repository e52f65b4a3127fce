// Host side of the sjd library: the C ABI of include/sjd.h, the context, the paged KV cache and the
// fixed kernel sequence of one speculative Jacobi iteration (Sec. 4.1 of the paper, Steps 1-4).
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <type_traits>
#include <vector>

#include "common.hip.h"
#include "decide.h"
#include "kernels_attention.hip.h"
#include "kernels_forward.hip.h"
#include "kernels_gemm.hip.h"
#include "kernels_skinny.hip.h"
#include "kernels_tile.hip.h"

void sjd_set_error(char *buf, const char *fmt, ...) {
    if (!buf) return;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, 512, fmt, ap);
    va_end(ap);
}

namespace {

char g_create_error[512] = "";

enum KernelClass {
    KC_STAGE = 0, KC_EMBED, KC_ADDNORM, KC_GEMM_QKV, KC_ROPE_KV, KC_ATTENTION, KC_GEMM_O, KC_GEMM_GATEUP, KC_SWIGLU,
    KC_GEMM_DOWN, KC_GEMM_HEAD, KC_SAMPLE_ROWS, KC_VERIFY, KC_DRAW, KC_COMMIT, KC_COUNT
};
const char *const kKernelClassName[KC_COUNT] = {
    "stage_rows", "embed", "addnorm", "gemm_qkv", "rope_kv_write", "window_attention", "gemm_out", "gemm_gate_up", "swiglu",
    "gemm_down", "gemm_head", "sample_rows", "verify", "draw", "commit"};

struct Tracer {
    bool on = false;
    std::vector<hipEvent_t> pool;   // pairs: start, stop
    std::vector<int> cls;           // class of each recorded pair
    size_t used = 0;
    int64_t launches[KC_COUNT] = {0};
    double total_ms[KC_COUNT] = {0};
};

struct LayerWeights {
    float *attn_norm = nullptr, *mlp_norm = nullptr;
    void *wqkv = nullptr, *wo = nullptr, *wgu = nullptr, *wdown = nullptr;
};

}  // namespace

struct sjd_ctx {
    sjd_model_desc md;
    sjd_sampling sampling;
    SamplingParams sp;
    hipStream_t stream = nullptr;
    char err[512] = "";
    int hd = 0, Vs = 0, L = 0, S = 0, n_seqs = 0, pt = 0, pps = 0, n_pages = 0, max_visible = 0;
    int n_cus = 256, n_xcds = 8;   // compute units and XCDs (L2 domains) of the device, read at create
    bool prefilled = false, all_done = false;
    // one sjd_step = the same launch sequence with the same arguments every time (what changes lives in device
    // memory): captured once per batch size into a HIP graph and replayed
    bool use_graph = false;
    // ... one graph per attention regime (below)
    hipGraph_t graph[2] = {nullptr, nullptr};
    hipGraphExec_t graph_exec[2] = {nullptr, nullptr};
    int graph_n_seqs[2] = {0, 0};
    bool attn_mfma = false;
    int attn_chunk = 0, attn_nchunks = 0;
    // Window attention runs as one workgroup per (segment, head) while that is the faster of the two kernels (enough
    // such workgroups to fill the chip, or a context of up to a few thousand tokens), and as chunks over workgroups
    // plus a merge kernel beyond: chosen per step from the cache lengths, which the host follows from the verdicts
    // it reads back anyway.
    bool attn_onepass_ok = false;          // the context may use the one-pass kernel at all
    bool attn_onepass = false;             // regime of the launches being enqueued
    std::vector<int32_t> kv_host;          // committed cache positions per segment (sequence * 2 + branch)
    float *part_o = nullptr, *part_ml = nullptr;
    float *row_ssq = nullptr;              // [M][ceil(d / 256)] partial sums of squares of the residual stream's rows
    QkvRow *row_meta = nullptr;            // per-row tables of the fused path, rewritten by every forward
    float2 *row_rot = nullptr;
    bool l2_warm = true;                   // projection launches touch the next projection's weights
    uint32_t *pf_sink = nullptr;
    float *skinny_part = nullptr;          // partial tiles of K-split fused projections
    size_t skinny_part_elems = 0;
    bool fused = false;  // small-M path: fused projection kernels, RMSNorm gains folded into the weights
    // weights (owned)
    void *tok_emb = nullptr, *lm_head = nullptr;
    float *final_norm = nullptr;
    std::vector<LayerWeights> layers;
    float *rope_cos = nullptr, *rope_sin = nullptr;
    // KV pages
    void *kpool = nullptr, *vpool = nullptr;
    size_t pool_layer_bytes = 0;
    int32_t *page_table = nullptr;
    std::vector<int32_t> page_table_host;  // what sjd_prefill uploaded (snapshots carry it)
    std::vector<int32_t> n_image_host;     // image tokens wanted per sequence of the current batch
    // workspaces
    float *x = nullptr, *partial = nullptr, *logits = nullptr;
    float *z = nullptr;                    // [S][L][V_s] guided logits written by the fused vocabulary head
    bool z_used = false;                   // the last forward's head wrote z (and the logits only if they are kept)
    bool keep_logits = false;
    void *xn = nullptr, *q = nullptr, *attn = nullptr, *h = nullptr;
    size_t partial_elems = 0;
    RowMap rm{};
    DecideState ds{};
    int32_t *prompt_dev = nullptr, *prompt_len_dev = nullptr, *prompt_last_dev = nullptr, *n_image_dev = nullptr;
    sjd_step_result *res_host = nullptr;
    std::vector<void *> allocations;
    Tracer tracer;
};

namespace {

template <typename P> int dev_alloc(sjd_ctx *c, P **out, size_t bytes, bool zero = true) {
    void *p = nullptr;
    if (bytes == 0) bytes = 16;
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess) {
        sjd_set_error(c->err, "hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
        return SJD_ENOMEM;
    }
    c->allocations.push_back(p);
    if (zero) {
        e = hipMemsetAsync(p, 0, bytes, c->stream);
        if (e != hipSuccess) {
            sjd_set_error(c->err, "hipMemsetAsync failed: %s", hipGetErrorString(e));
            return SJD_EDEVICE;
        }
    }
    *out = reinterpret_cast<P *>(p);
    return SJD_OK;
}

void trace_begin(sjd_ctx *c, int cls) {
    Tracer &t = c->tracer;
    if (!t.on) return;
    if (t.used + 2 > t.pool.size()) {
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { t.on = false; return; }
        t.pool.push_back(a);
        t.pool.push_back(b);
    }
    t.cls.push_back(cls);
    (void)hipEventRecord(t.pool[t.used], c->stream);
}
void trace_end(sjd_ctx *c) {
    Tracer &t = c->tracer;
    if (!t.on) return;
    (void)hipEventRecord(t.pool[t.used + 1], c->stream);
    t.used += 2;
}
// after the stream has been synchronised
void trace_collect(sjd_ctx *c) {
    Tracer &t = c->tracer;
    for (size_t i = 0; i + 1 < t.used; i += 2) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, t.pool[i], t.pool[i + 1]) == hipSuccess) {
            t.total_ms[t.cls[i / 2]] += ms;
            t.launches[t.cls[i / 2]] += 1;
        }
    }
    t.used = 0;
    t.cls.clear();
}

#define SJD_LAUNCH(c, cls, expr)                                                                   \
    do {                                                                                           \
        trace_begin(c, cls);                                                                       \
        hipError_t e__ = (expr);                                                                   \
        trace_end(c);                                                                              \
        if (e__ != hipSuccess) {                                                                   \
            sjd_set_error((c)->err, "launch of %s failed: %s", kKernelClassName[cls], hipGetErrorString(e__)); \
            return SJD_EDEVICE;                                                                    \
        }                                                                                          \
    } while (0)

template <typename F> hipError_t after(F &&f) {
    f();
    return hipGetLastError();
}

bool use_reference(const sjd_ctx *c) { return c->md.dtype == SJD_F32 || (c->md.kernel_flags & SJD_KERNELS_REFERENCE); }

// ------------------------------------------------------------------------------------- GEMM dispatch
// C_partial[splits][M][N]; returns the number of splits written.
template <typename T>
int run_gemm(sjd_ctx *c, int cls, const T *A, const T *W, float *C, int M, int N, int K, int force_splits, int *splits_out);

template <>
int run_gemm<float>(sjd_ctx *c, int cls, const float *A, const float *W, float *C, int M, int N, int K, int, int *splits_out) {
    *splits_out = 1;
    SJD_LAUNCH(c, cls, launch_gemm_reference<float>(c->stream, A, W, C, M, N, K));
    return SJD_OK;
}

template <>
int run_gemm<bf16_t>(sjd_ctx *c, int cls, const bf16_t *A, const bf16_t *W, float *C, int M, int N, int K, int force_splits,
                     int *splits_out) {
    if (c->md.kernel_flags & SJD_KERNELS_REFERENCE) {
        *splits_out = 1;
        SJD_LAUNCH(c, cls, launch_gemm_reference<bf16_t>(c->stream, A, W, C, M, N, K));
        return SJD_OK;
    }
    GemmPlan p = plan_gemm_bf16(M, N, K, force_splits);
    if ((size_t)p.splits * M * N > c->partial_elems && C == c->partial) {
        // never happens: the workspace is sized with the same plan at create
        sjd_set_error(c->err, "split-K workspace too small");
        return SJD_EINVAL;
    }
    *splits_out = p.splits;
    SJD_LAUNCH(c, cls, launch_gemm_bf16(c->stream, p, A, W, C, M, N, K));
    return SJD_OK;
}

// ---------------------------------------------------------------------------------------- attention
template <typename T> int run_attention(sjd_ctx *c, const KvPool &pool, int M);

template <> int run_attention<float>(sjd_ctx *c, const KvPool &pool, int M) {
    SJD_LAUNCH(c, KC_ATTENTION, launch_attention_reference<float>(c->stream, (const float *)c->q, pool, c->rm.row_tok, c->rm.seg_kv,
                                                                  (float *)c->attn, nullptr, M, c->L, c->md.n_heads,
                                                                  c->md.n_kv_heads, c->hd, c->max_visible));
    return SJD_OK;
}

template <> int run_attention<bf16_t>(sjd_ctx *c, const KvPool &pool, int M) {
    if (!c->attn_mfma) {
        SJD_LAUNCH(c, KC_ATTENTION, launch_attention_reference<bf16_t>(c->stream, (const bf16_t *)c->q, pool, c->rm.row_tok,
                                                                       c->rm.seg_kv, (bf16_t *)c->attn, nullptr, M, c->L,
                                                                       c->md.n_heads, c->md.n_kv_heads, c->hd, c->max_visible));
        return SJD_OK;
    }
    AttnArgs a;
    a.q = (const bf16_t *)c->q;
    a.pool = pool;
    a.row_tok = c->rm.row_tok;
    a.seg_kv = c->rm.seg_kv;
    a.seg_n = c->rm.seg_n;
    a.part_o = c->part_o;
    a.part_ml = c->part_ml;
    a.out_act = (bf16_t *)c->attn;
    a.out_plain = nullptr;
    a.L = c->L; a.H = c->md.n_heads; a.Hkv = c->md.n_kv_heads; a.hd = c->hd;
    a.chunk = c->attn_chunk;
    a.n_chunks = c->attn_nchunks;
    a.n_qt = ceil_div(c->L, 32);
    a.scale_log2e = (float)(1.4426950408889634 / sqrt((double)c->hd));
    SJD_LAUNCH(c, KC_ATTENTION, launch_attention_mfma(c->stream, a, M / c->L, c->attn_onepass));
    return SJD_OK;
}

// ------------------------------------------------------------------------------------------ forward
// Runs the rows described by c->rm through the model.  Keys and values of active rows are written to
// their pages; with_head also produces fp32 logits [M][V_s].
template <typename T> int forward(sjd_ctx *c, bool with_head) {
    const sjd_model_desc &md = c->md;
    const int M = c->n_seqs * 2 * c->L, d = md.d_model, H = md.n_heads, Hkv = md.n_kv_heads, hd = c->hd, F = md.d_ff;
    const int Nqkv = (H + 2 * Hkv) * hd;
    hipStream_t st = c->stream;
    SJD_LAUNCH(c, KC_EMBED, after([&] { embed_kernel<T><<<M, 256, 0, st>>>((const T *)c->tok_emb, c->rm.row_tok, c->x, d); }));
    int down_splits = 0;
    for (int l = 0; l < md.n_layers; ++l) {
        const LayerWeights &lw = c->layers[l];
        KvPool pool;
        pool.k = (char *)c->kpool + c->pool_layer_bytes * l;
        pool.v = (char *)c->vpool + c->pool_layer_bytes * l;
        pool.page_table = c->page_table;
        pool.pages_per_seg = c->pps;
        pool.page_tokens = c->pt;

        SJD_LAUNCH(c, KC_ADDNORM, after([&] {
                       addnorm_kernel<T><<<M, 256, 0, st>>>(c->x, l == 0 ? nullptr : c->partial, down_splits, M, lw.attn_norm,
                                                            (T *)c->xn, d, md.rms_eps);
                   }));
        int splits = 1;
        int rc = run_gemm<T>(c, KC_GEMM_QKV, (const T *)c->xn, (const T *)lw.wqkv, c->partial, M, Nqkv, d, 0, &splits);
        if (rc) return rc;
        SJD_LAUNCH(c, KC_ROPE_KV, after([&] {
                       rope_kv_kernel<T><<<M, 256, 0, st>>>(c->partial, splits, M, c->rm.row_tok, c->rm.row_pos, c->rope_cos,
                                                            c->rope_sin, (T *)c->q, pool, c->L, H, Hkv, hd);
                   }));
        if ((rc = run_attention<T>(c, pool, M))) return rc;
        rc = run_gemm<T>(c, KC_GEMM_O, (const T *)c->attn, (const T *)lw.wo, c->partial, M, d, H * hd, 0, &splits);
        if (rc) return rc;
        SJD_LAUNCH(c, KC_ADDNORM, after([&] {
                       addnorm_kernel<T><<<M, 256, 0, st>>>(c->x, c->partial, splits, M, lw.mlp_norm, (T *)c->xn, d, md.rms_eps);
                   }));
        rc = run_gemm<T>(c, KC_GEMM_GATEUP, (const T *)c->xn, (const T *)lw.wgu, c->partial, M, 2 * F, d, 0, &splits);
        if (rc) return rc;
        SJD_LAUNCH(c, KC_SWIGLU, after([&] { swiglu_kernel<T><<<M, 256, 0, st>>>(c->partial, splits, M, (T *)c->h, F); }));
        rc = run_gemm<T>(c, KC_GEMM_DOWN, (const T *)c->h, (const T *)lw.wdown, c->partial, M, d, F, 0, &down_splits);
        if (rc) return rc;
    }
    if (with_head) {
        SJD_LAUNCH(c, KC_ADDNORM, after([&] {
                       addnorm_kernel<T><<<M, 256, 0, st>>>(c->x, c->partial, down_splits, M, c->final_norm, (T *)c->xn, d,
                                                            md.rms_eps);
                   }));
        int splits = 1;
        int rc = run_gemm<T>(c, KC_GEMM_HEAD, (const T *)c->xn, (const T *)c->lm_head, c->logits, M, c->Vs, d, 1, &splits);
        if (rc) return rc;
    }
    return SJD_OK;
}

// Small-M bf16 path: five kernels per layer (QKV+RoPE+KV write, attention, out+residual, gate/up+SwiGLU,
// down+residual); c->xn holds the bf16 copy of the residual stream.
int forward_fused(sjd_ctx *c, bool with_head) {
    const sjd_model_desc &md = c->md;
    const int M = c->n_seqs * 2 * c->L, d = md.d_model, H = md.n_heads, Hkv = md.n_kv_heads, hd = c->hd, F = md.d_ff;
    // up to 64 rows: one row group; more (a multiple of 64 by construction): row groups of 64 over the same weights
    const int m_groups = M <= 64 ? 1 : M / 64;
    const int MT = M <= 64 ? ceil_div(M, 32) : 2;
    const int n_cus = c->n_cus;
    hipStream_t st = c->stream;
    SJD_LAUNCH(c, KC_EMBED, after([&] {
                   RowTables rt;
                   rt.row_pos = c->rm.row_pos; rt.rope_cos = c->rope_cos; rt.rope_sin = c->rope_sin;
                   rt.page_table = c->page_table; rt.pages_per_seg = c->pps; rt.page_tokens = c->pt;
                   rt.L = c->L; rt.H = H; rt.hd = hd; rt.meta = c->row_meta; rt.rot = c->row_rot;
                   rt.ssq_part = c->row_ssq; rt.ssq_n = ceil_div(d, 256);
                   embed_dual_kernel<<<M, 256, 0, st>>>((const bf16_t *)c->tok_emb, c->rm.row_tok, c->x, (bf16_t *)c->xn, d, rt);
               }));
    SkinnyArgs a;
    memset(&a, 0, sizeof a);
    a.M = M;
    a.n_cus = n_cus;
    a.m_groups = m_groups;
    a.eps = md.rms_eps;
    a.row_meta = c->row_meta;
    a.k_rot = (md.kernel_flags & SJD_NO_K_ROTATION) ? 0 : 1;
    a.row_rot = c->row_rot;
    a.q_out = (bf16_t *)c->q;
    a.L = c->L; a.H = H; a.Hkv = Hkv; a.hd = hd; a.F = F;
    a.x = c->x;
    a.xb = (bf16_t *)c->xn;
    a.h = (bf16_t *)c->h;
    a.logits = c->logits;
    const int nbw_d = ceil_div(d, 32) >= 128 ? 2 : 1;
    a.part = c->skinny_part;
    auto whole_k = [&]() { a.ksplit = 1; a.kb_per_split = a.KB; };
    auto no_room = [&]() { sjd_set_error(c->err, "split-K workspace too small"); return SJD_EINVAL; };
    // Wavefronts per workgroup, measured: 8 pull a workgroup's share through the CU's L1 faster than 4 and halve
    // the epilogue's elements per thread; once a launch fills most CUs with weights that come from HBM (the 7B
    // shapes' gate/up and head) a CU's outstanding misses are the limit either way, the second wavefront of a SIMD
    // only queues behind the first, and 4 win by the cheaper LDS reduction.
    auto nw_for = [](int groups) { return groups >= 200 ? 4 : 8; };
    // many rows: LDS-staged 256 x 128 tiles (the projections are a dense contraction there, not a weight stream)
    // ... provided the model is wide enough for 256 x 128 tiles to fill the chip (QKV: >= 96 tiles); a narrow model
    // with a long window keeps the row-group kernels, which give it more workgroups
    const bool tile = M >= TILE_M && !(md.kernel_flags & SJD_KERNELS_ROWGROUPS) &&
                      ((md.kernel_flags & SJD_KERNELS_TILES) || ceil_div((H + 2 * Hkv) * (hd / 64) * 2, 4) * ceil_div(M, TILE_M) >= 96);
    // output / down projection: x += A W^T.  One kernel when a workgroup's share is small, else K split over
    // grid.y with the partial sums added by resid_reduce_kernel after the kernel boundary.
    // Every few-row projection launch carries extra workgroups that touch the weights of the projection after it,
    // so that those are in the L2 of the XCD that will read them when that launch starts (the launches are short
    // and latency-bound: first touch from HBM costs 2-3x the time of an L2 hit, and the chip is mostly idle).
    struct Proj { const void *W; int groups, nbw, KB; bool whole; };
    const int groups_d = ceil_div(ceil_div(d, 32), nbw_d), groups_qkv = (H + 2 * Hkv) * (hd / 64);
    // More than 32 rows and so few column groups that a workgroup per group and 32-row tile still finds a CU of its
    // own: row groups of 32 rows instead of 64 (all row groups of a column group on one XCD, whose L2 serves the
    // later readers of the weights).  Each workgroup pulls half the activations, twice as many CUs work.
    auto rows2_for = [&](int groups) {
        return MT == 2 && 2 * m_groups * 8 * ceil_div(groups, 8) <= n_cus && !(md.kernel_flags & SJD_NO_ROW_SPLIT);
    };
    // computing workgroups of a launch over `groups` column groups
    auto compute_wgs = [&](int groups, bool r2, int row_split) {
        if (r2) return 2 * m_groups * 8 * ceil_div(groups, 8);
        if (row_split == 2) return 16 * ceil_div(groups, 8);
        return m_groups > 1 ? m_groups * 8 * ceil_div(groups, 8) : groups;
    };
    const int mt_resid = rows2_for(groups_d) ? 1 : MT;   // 32-row tiles per workgroup of an output / down projection
    auto resid_whole = [&](int K) { return (double)(nbw_d * 32 + mt_resid * 32) * K * 2.0 <= 512e3; };
    auto warm = [&](int cur_groups, const Proj &nx) {
        a.pf_wgs = 0;
        if (!c->l2_warm || tile || !nx.whole || !nx.W) return;
        const uint32_t slab = (uint32_t)nx.nbw * nx.KB * 1024;
        int fit = (int)std::min<size_t>(nx.groups, ((size_t)24 << 20) / slab);   // what the L2s hold beside the current weights
        int wgs = (int)(((size_t)fit * slab / (96 << 10) + 7) / 8 * 8);
        wgs = std::min(wgs, (n_cus - cur_groups) / 8 * 8);
        if (wgs < 8 || (m_groups > 1 && wgs < 32)) return;   // long-window launches: a handful of CUs only delays them
        // few CUs left: touch no more than they get through while the launch computes (a CU streams ~45 GB/s from
        // HBM, the launches take 7-10 us: 320 KB each), the first slabs
        fit = (int)std::min<size_t>(fit, (size_t)wgs * (320 << 10) / slab);
        if (fit < 1) return;
        a.pf_base = (const char *)nx.W; a.pf_slab_bytes = slab; a.pf_groups = fit; a.pf_wgs = wgs; a.pf_sink = c->pf_sink;
    };
    // The same for the keys and values of the next one-pass attention launch (one workgroup per (head, segment), in
    // that order); call after warm(): takes what is left of the CUs.
    auto warm_kv = [&](int cur_groups, const KvPool &pool) {
        a.kv_wgs = 0;
        if (!c->l2_warm || tile || m_groups > 1 || !c->attn_mfma || !c->attn_onepass || c->L > 32) return;
        const size_t kv_bytes = (size_t)(M / c->L) * Hkv * md.max_ctx * hd * 2 * sizeof(bf16_t);
        const int room = (n_cus - cur_groups - a.pf_wgs) / 8 * 8;
        a.kv_wgs = std::max(0, std::min(room, (int)((kv_bytes / (48 << 10) + 7) / 8 * 8)));
        a.kv_pairs = (M / c->L) * H;
        a.kv_seg_kv = c->rm.seg_kv;
        a.kv_pool = pool;
        a.pf_sink = c->pf_sink;
    };
    // few column groups and one 32-row tile: two workgroups per group, 16 rows each (half the activation lines per
    // workgroup; the loop is bound by what a CU's L1 delivers).  Measured on the 36 x 1280 shape: output, down and QKV
    // projections (40-60 groups) gain, gate/up (108 groups: too few CUs left for the warm-up workgroups) loses.
    auto row_split_for = [&](int groups) { return MT == 1 && M > 16 && groups <= 64 && !(md.kernel_flags & SJD_NO_ROW_SPLIT) ? 2 : 1; };
    const Proj none = {nullptr, 0, 0, 0, false};
    const bool mixed_ok = !(md.kernel_flags & SJD_NO_MIXED_WIDTH);
    // Many-row kernels take the RMSNorm row sums of squares from the kernel that wrote the residual stream (embedding
    // gather or split-K reduction) instead of accumulating them in their k-loops
    const int tile_rows = (md.kernel_flags & SJD_TILES_256_ROWS) ? 256 : 0;  // 0: chosen per launch
    bool ssq_ready = true;   // the embedding kernel wrote them
    float *const ssq_out = tile ? c->row_ssq : nullptr;
    auto use_ssq = [&]() { a.row_ssq_part = tile && ssq_ready ? c->row_ssq : nullptr; a.row_ssq_n = ceil_div(d, 256); };
    auto resid = [&](int cls, const void *A, const void *W, int K, const Proj &nx, const KvPool *kv_next) -> int {
        a.A = (const bf16_t *)A; a.W = (const bf16_t *)W; a.KB = K / 16; a.N = d;
        a.pf_wgs = 0;
        a.row_ssq_part = nullptr;
        if (tile) {
            const int n_blocks = ceil_div(d, 64) * 2, wgs = ceil_div(n_blocks, 4) * ceil_div(M, TILE_M);
            int ks = std::min(8, std::max(1, n_cus / wgs));
            while (ks > 1 && a.KB / ks < 32) --ks;
            a.kb_per_split = ceil_div(a.KB, ks);
            a.ksplit = ceil_div(a.KB, a.kb_per_split);
            if (a.ksplit == 1) {
                SJD_LAUNCH(c, cls, launch_tile<EPI_RESID>(st, a, n_blocks, tile_rows, mixed_ok));
                ssq_ready = false;
                return SJD_OK;
            }
            if ((size_t)a.ksplit * M * d > c->skinny_part_elems) return no_room();
            SJD_LAUNCH(c, cls, launch_tile<EPI_PARTIAL>(st, a, n_blocks, tile_rows, mixed_ok));
            const int ksplit = a.ksplit;
            SJD_LAUNCH(c, KC_ADDNORM, after([&] {
                           resid_reduce_kernel<<<dim3(ceil_div(d, 1024), M), 256, 0, st>>>(c->skinny_part, ksplit, M, d, c->x, (bf16_t *)c->xn, ssq_out);
                       }));
            ssq_ready = true;
            return SJD_OK;
        }
        const int groups = ceil_div(ceil_div(d, 32), nbw_d);
        const double wg_bytes = (double)(nbw_d * 32 + mt_resid * 32) * K * 2.0;
        int ks = 1;
        if (wg_bytes > 512e3) {
            ks = std::min(8, std::max(1, n_cus / (groups * m_groups)));
            while (ks > 1 && a.KB / ks < 32) --ks;
        }
        if (ks == 1) {
            whole_k();
            a.row_split = row_split_for(groups);
            const bool r2 = rows2_for(groups);
            a.m_groups = r2 ? 2 * m_groups : m_groups;
            const int n_compute = compute_wgs(groups, r2, a.row_split);
            warm(n_compute, nx);
            if (kv_next) warm_kv(n_compute, *kv_next);
            SJD_LAUNCH(c, cls, launch_skinny<EPI_RESID>(st, a, r2 ? 1 : MT, groups, nbw_d, nw_for(groups)));
            a.pf_wgs = a.kv_wgs = 0;
            a.row_split = 1;
            a.m_groups = m_groups;
            return SJD_OK;
        }
        a.kb_per_split = ceil_div(a.KB, ks);
        a.ksplit = ceil_div(a.KB, a.kb_per_split);
        if ((size_t)a.ksplit * M * d > c->skinny_part_elems) return no_room();
        SJD_LAUNCH(c, cls, launch_skinny<EPI_PARTIAL>(st, a, MT, groups, nbw_d, nw_for(groups * a.ksplit)));
        const int ksplit = a.ksplit;
        SJD_LAUNCH(c, KC_ADDNORM, after([&] {
                       resid_reduce_kernel<<<dim3(ceil_div(d, 1024), M), 256, 0, st>>>(c->skinny_part, ksplit, M, d, c->x, (bf16_t *)c->xn, ssq_out);
                   }));
        return SJD_OK;
    };
    for (int l = 0; l < md.n_layers; ++l) {
        const LayerWeights &lw = c->layers[l];
        KvPool pool;
        pool.k = (char *)c->kpool + c->pool_layer_bytes * l;
        pool.v = (char *)c->vpool + c->pool_layer_bytes * l;
        pool.page_table = c->page_table;
        pool.pages_per_seg = c->pps;
        pool.page_tokens = c->pt;
        a.pool = pool;
        a.A = (const bf16_t *)c->xn; a.W = (const bf16_t *)lw.wqkv; a.KB = d / 16;
        if (tile) {
            whole_k();
            use_ssq();
            SJD_LAUNCH(c, KC_GEMM_QKV, launch_tile<EPI_QKV>(st, a, (H + 2 * Hkv) * (hd / 64) * 2, tile_rows, mixed_ok));
        } else {
            whole_k();
            a.row_split = row_split_for(groups_qkv);
            const bool r2 = rows2_for(groups_qkv);
            a.m_groups = r2 ? 2 * m_groups : m_groups;
            const int n_compute = compute_wgs(groups_qkv, r2, a.row_split);
            warm(n_compute, Proj{lw.wo, groups_d, nbw_d, H * hd / 16, resid_whole(H * hd)});
            if (l == 0) warm_kv(n_compute, pool);  // later layers: requested by the down projection before them
            SJD_LAUNCH(c, KC_GEMM_QKV, launch_skinny<EPI_QKV>(st, a, r2 ? 1 : MT, groups_qkv, 2, nw_for(groups_qkv)));
            a.pf_wgs = a.kv_wgs = 0;
            a.row_split = 1;
            a.m_groups = m_groups;
        }
        { int rc = run_attention<bf16_t>(c, pool, M); if (rc) return rc; }
        { int rc = resid(KC_GEMM_O, c->attn, lw.wo, H * hd, Proj{lw.wgu, F / 32, 2, d / 16, true}, nullptr); if (rc) return rc; }
        a.A = (const bf16_t *)c->xn; a.W = (const bf16_t *)lw.wgu; a.KB = d / 16;
        if (tile) {
            whole_k();
            use_ssq();
            SJD_LAUNCH(c, KC_GEMM_GATEUP, launch_tile<EPI_SWIGLU>(st, a, F / 32 * 2, tile_rows, mixed_ok));
        } else {
            whole_k();
            a.row_split = row_split_for(F / 32);
            const bool r2 = rows2_for(F / 32);
            a.m_groups = r2 ? 2 * m_groups : m_groups;
            const int n_compute = compute_wgs(F / 32, r2, a.row_split);
            warm(n_compute, Proj{lw.wdown, groups_d, nbw_d, F / 16, resid_whole(F)});
            if (mixed_ok && skinny_mixed_applies(a, F / 32, 2, nw_for(F / 32))) SJD_LAUNCH(c, KC_GEMM_GATEUP, launch_skinny_mixed<EPI_SWIGLU>(st, a, MT, F / 32));
            else SJD_LAUNCH(c, KC_GEMM_GATEUP, launch_skinny<EPI_SWIGLU>(st, a, r2 ? 1 : MT, F / 32, 2, nw_for(F / 32)));
            a.pf_wgs = 0;
            a.row_split = 1;
            a.m_groups = m_groups;
        }
        const Proj after_down = l + 1 < md.n_layers ? Proj{c->layers[l + 1].wqkv, groups_qkv, 2, d / 16, true}
                                : with_head         ? Proj{c->lm_head, ceil_div(ceil_div(c->Vs, 32), 2), 2, d / 16, true}
                                                    : none;
        KvPool pool_next = pool;
        pool_next.k = (char *)c->kpool + c->pool_layer_bytes * (l + 1);
        pool_next.v = (char *)c->vpool + c->pool_layer_bytes * (l + 1);
        { int rc = resid(KC_GEMM_DOWN, c->h, lw.wdown, F, after_down, l + 1 < md.n_layers ? &pool_next : nullptr); if (rc) return rc; }
    }
    if (with_head) {
        a.A = (const bf16_t *)c->xn; a.W = (const bf16_t *)c->lm_head; a.KB = d / 16; a.N = c->Vs;
        // Guidance fused into the head where a position's conditional and unconditional rows meet in one thread of the
        // epilogue: windows of 32 (row tiles alternate conditional / unconditional) and one sequence with a window of 16
        const int groups_v = ceil_div(ceil_div(c->Vs, 32), 2);
        const bool head_mixed = !tile && mixed_ok && skinny_mixed_applies(a, groups_v, 2, nw_for(groups_v));
        const bool head_r2 = !tile && !head_mixed && rows2_for(groups_v);
        int z_mode = 0;
        if (c->z && !(md.kernel_flags & SJD_NO_HEAD_FUSION)) {
            if (c->L == 32 && (tile || (MT == 2 && !head_r2))) z_mode = 1;
            else if (c->L == 16 && M == 32 && !tile) z_mode = 2;
        }
        a.z_out = c->z; a.z_mode = z_mode; a.cfg_scale = c->sp.cfg_scale; a.inv_t = c->sp.inv_temperature;
        a.logits = z_mode == 0 || c->keep_logits ? c->logits : nullptr;
        c->z_used = z_mode != 0;
        if (tile) {
            whole_k();
            use_ssq();
            SJD_LAUNCH(c, KC_GEMM_HEAD, launch_tile<EPI_HEAD>(st, a, ceil_div(c->Vs, 64) * 2, z_mode ? 256 : tile_rows));
        } else {
            whole_k();
            if (head_mixed) SJD_LAUNCH(c, KC_GEMM_HEAD, launch_skinny_mixed<EPI_HEAD>(st, a, MT, groups_v));
            else {
                const bool r2 = head_r2;
                a.m_groups = r2 ? 2 * m_groups : m_groups;
                SJD_LAUNCH(c, KC_GEMM_HEAD, launch_skinny<EPI_HEAD>(st, a, r2 ? 1 : MT, groups_v, 2, nw_for(groups_v)));
                a.m_groups = m_groups;
            }
        }
    }
    return SJD_OK;
}

int forward_any(sjd_ctx *c, bool with_head) {
    if (c->fused) return forward_fused(c, with_head);
    return c->md.dtype == SJD_F32 ? forward<float>(c, with_head) : forward<bf16_t>(c, with_head);
}

// ------------------------------------------------------------------------------------------ create
template <typename T> int copy_weights(sjd_ctx *c, const sjd_weights *w) {
    const sjd_model_desc &md = c->md;
    const int d = md.d_model, H = md.n_heads, Hkv = md.n_kv_heads, hd = c->hd, F = md.d_ff;
    hipStream_t st = c->stream;
    int rc;
    T *emb;
    if ((rc = dev_alloc(c, &emb, (size_t)md.vocab * d * sizeof(T), false))) return rc;
    SJD_HIP_TRY(c->err, hipMemcpyAsync(emb, w->tok_emb, (size_t)md.vocab * d * sizeof(T), hipMemcpyDeviceToDevice, st));
    c->tok_emb = emb;
    auto gain = [&](const void *src, float **dst) -> int {
        int r = dev_alloc(c, dst, (size_t)d * sizeof(float));
        if (r) return r;
        to_float_kernel<T><<<ceil_div(d, 256), 256, 0, st>>>((const T *)src, *dst, d);
        return hipGetLastError() == hipSuccess ? SJD_OK : SJD_EDEVICE;
    };
    auto pack = [&](T *dst, const void *src, int N, int K, int row0) -> int {
        if (!src) { sjd_set_error(c->err, "null weight pointer"); return SJD_EINVAL; }
        pack_weight_kernel<T><<<1024, 256, 0, st>>>((const T *)src, dst, N, K, row0);
        return hipGetLastError() == hipSuccess ? SJD_OK : SJD_EDEVICE;
    };
    if ((rc = gain(w->final_norm, &c->final_norm))) return rc;
    T *head;
    if ((rc = dev_alloc(c, &head, Layout<T>::w_elems(c->Vs, d) * sizeof(T)))) return rc;
    if ((rc = pack(head, (const T *)w->lm_head + (size_t)md.sample_lo * d, c->Vs, d, 0))) return rc;
    c->lm_head = head;
    c->layers.resize(md.n_layers);
    for (int l = 0; l < md.n_layers; ++l) {
        LayerWeights &lw = c->layers[l];
        if (!w->attn_norm[l] || !w->mlp_norm[l]) { sjd_set_error(c->err, "null weight pointer"); return SJD_EINVAL; }
        if ((rc = gain(w->attn_norm[l], &lw.attn_norm))) return rc;
        if ((rc = gain(w->mlp_norm[l], &lw.mlp_norm))) return rc;
        T *qkv, *o, *gu, *down;
        const int Nqkv = (H + 2 * Hkv) * hd;
        if ((rc = dev_alloc(c, &qkv, Layout<T>::w_elems(Nqkv, d) * sizeof(T)))) return rc;
        if ((rc = pack(qkv, w->wq[l], H * hd, d, 0))) return rc;
        if ((rc = pack(qkv, w->wk[l], Hkv * hd, d, H * hd))) return rc;
        if ((rc = pack(qkv, w->wv[l], Hkv * hd, d, (H + Hkv) * hd))) return rc;
        if ((rc = dev_alloc(c, &o, Layout<T>::w_elems(d, H * hd) * sizeof(T)))) return rc;
        if ((rc = pack(o, w->wo[l], d, H * hd, 0))) return rc;
        if ((rc = dev_alloc(c, &gu, Layout<T>::w_elems(2 * F, d) * sizeof(T)))) return rc;
        if ((rc = pack(gu, w->w_gate[l], F, d, 0))) return rc;
        if ((rc = pack(gu, w->w_up[l], F, d, F))) return rc;
        if ((rc = dev_alloc(c, &down, Layout<T>::w_elems(d, F) * sizeof(T)))) return rc;
        if ((rc = pack(down, w->w_down[l], d, F, 0))) return rc;
        lw.wqkv = qkv; lw.wo = o; lw.wgu = gu; lw.wdown = down;
    }
    return SJD_OK;
}

// Weights of the fused small-M path: gains folded in, QKV rows in (head, rotary pair) order, gate and up
// interleaved by blocks of 32.
int copy_weights_fused(sjd_ctx *c, const sjd_weights *w) {
    typedef bf16_t T;
    const sjd_model_desc &md = c->md;
    const int d = md.d_model, H = md.n_heads, Hkv = md.n_kv_heads, hd = c->hd, F = md.d_ff;
    hipStream_t st = c->stream;
    int rc;
    T *emb;
    if ((rc = dev_alloc(c, &emb, (size_t)md.vocab * d * sizeof(T), false))) return rc;
    SJD_HIP_TRY(c->err, hipMemcpyAsync(emb, w->tok_emb, (size_t)md.vocab * d * sizeof(T), hipMemcpyDeviceToDevice, st));
    c->tok_emb = emb;
    float *gain;  // scratch, reused per matrix (stream order keeps it safe)
    if ((rc = dev_alloc(c, &gain, (size_t)d * sizeof(float)))) return rc;
    auto pack = [&](T *dst, const void *s0, const void *s1, const void *s2, int n0, int n1, int N, int K, const void *g,
                    PackMap pm) -> int {
        if (!s0 || (n0 < N && !s1) || (n1 < N && !s2)) { sjd_set_error(c->err, "null weight pointer"); return SJD_EINVAL; }
        if (g) to_float_kernel<T><<<ceil_div(K, 256), 256, 0, st>>>((const T *)g, gain, K);
        pack_weight_fused_kernel<<<2048, 256, 0, st>>>((const T *)s0, (const T *)s1, (const T *)s2, n0, n1, g ? gain : nullptr, dst,
                                                       N, K, pm);
        return hipGetLastError() == hipSuccess ? SJD_OK : SJD_EDEVICE;
    };
    const PackMap ident{0, hd, F}, qkvmap{1, hd, F}, gumap{2, hd, F};
    T *head;
    if ((rc = dev_alloc(c, &head, Layout<T>::w_elems(ceil_div(c->Vs, 64) * 64, d) * sizeof(T)))) return rc;
    if ((rc = pack(head, (const T *)w->lm_head + (size_t)md.sample_lo * d, nullptr, nullptr, c->Vs, c->Vs, c->Vs, d, w->final_norm, ident)))
        return rc;
    c->lm_head = head;
    c->layers.resize(md.n_layers);
    const int Nqkv = (H + 2 * Hkv) * hd, dpad = ceil_div(d, 64) * 64;
    for (int l = 0; l < md.n_layers; ++l) {
        LayerWeights &lw = c->layers[l];
        if (!w->attn_norm[l] || !w->mlp_norm[l]) { sjd_set_error(c->err, "null weight pointer"); return SJD_EINVAL; }
        T *qkv, *o, *gu, *down;
        if ((rc = dev_alloc(c, &qkv, Layout<T>::w_elems(Nqkv, d) * sizeof(T)))) return rc;
        if ((rc = pack(qkv, w->wq[l], w->wk[l], w->wv[l], H * hd, (H + Hkv) * hd, Nqkv, d, w->attn_norm[l], qkvmap))) return rc;
        if ((rc = dev_alloc(c, &o, Layout<T>::w_elems(dpad, H * hd) * sizeof(T)))) return rc;
        if ((rc = pack(o, w->wo[l], nullptr, nullptr, d, d, d, H * hd, nullptr, ident))) return rc;
        if ((rc = dev_alloc(c, &gu, Layout<T>::w_elems(2 * F, d) * sizeof(T)))) return rc;
        if ((rc = pack(gu, w->w_gate[l], w->w_up[l], nullptr, F, 2 * F, 2 * F, d, w->mlp_norm[l], gumap))) return rc;
        if ((rc = dev_alloc(c, &down, Layout<T>::w_elems(dpad, F) * sizeof(T)))) return rc;
        if ((rc = pack(down, w->w_down[l], nullptr, nullptr, d, d, d, F, nullptr, ident))) return rc;
        lw.wqkv = qkv; lw.wo = o; lw.wgu = gu; lw.wdown = down;
    }
    return SJD_OK;
}

template <typename T> int alloc_buffers(sjd_ctx *c) {
    const sjd_model_desc &md = c->md;
    const int S = c->S, L = c->L, M = S * 2 * L, d = md.d_model, H = md.n_heads, Hkv = md.n_kv_heads, hd = c->hd, F = md.d_ff;
    const int Nqkv = (H + 2 * Hkv) * hd;
    int rc;
    // KV pages
    c->pps = ceil_div(md.max_ctx, c->pt);
    c->n_pages = S * 2 * c->pps;
    c->pool_layer_bytes = (size_t)c->n_pages * Hkv * c->pt * hd * sizeof(T);
    if ((rc = dev_alloc(c, &c->kpool, c->pool_layer_bytes * md.n_layers))) return rc;
    if ((rc = dev_alloc(c, &c->vpool, c->pool_layer_bytes * md.n_layers))) return rc;
    if ((rc = dev_alloc(c, &c->page_table, (size_t)S * 2 * c->pps * sizeof(int32_t)))) return rc;
    // workspaces
    if ((rc = dev_alloc(c, &c->x, (size_t)M * d * sizeof(float)))) return rc;
    size_t pe = 0;
    const int shapes[4][2] = {{Nqkv, d}, {d, H * hd}, {2 * F, d}, {d, F}};
    for (auto &s : shapes) {
        size_t need = (size_t)M * s[0];
        if (md.dtype == SJD_BF16 && !(md.kernel_flags & SJD_KERNELS_REFERENCE)) {
            // worst case over the number of sequences actually decoded (M = n * 2 * L)
            for (int n = 1; n <= S; ++n) {
                GemmPlan p = plan_gemm_bf16(n * 2 * L, s[0], s[1], 0);
                size_t e = (size_t)p.splits * (n * 2 * L) * s[0];
                if (e > need) need = e;
            }
        }
        if (need > pe) pe = need;
    }
    c->partial_elems = pe;
    if ((rc = dev_alloc(c, &c->partial, pe * sizeof(float)))) return rc;
    if ((rc = dev_alloc(c, &c->logits, (size_t)M * c->Vs * sizeof(float)))) return rc;
    if ((rc = dev_alloc(c, &c->xn, Layout<T>::a_elems(M, d) * sizeof(T)))) return rc;
    if ((rc = dev_alloc(c, &c->attn, Layout<T>::a_elems(M, H * hd) * sizeof(T)))) return rc;
    if ((rc = dev_alloc(c, &c->h, Layout<T>::a_elems(M, F) * sizeof(T)))) return rc;
    if ((rc = dev_alloc(c, &c->q, (size_t)S * 2 * H * Layout<T>::q_elems(L, hd) * sizeof(T)))) return rc;
    if (c->fused) {
        if ((rc = dev_alloc(c, &c->z, (size_t)S * L * c->Vs * sizeof(float)))) return rc;
        // partial tiles of K-split projections: at most 8 splits of the widest projection (2 column blocks, 2 row tiles)
        const int widest = std::max(std::max((H + 2 * Hkv) * (hd / 64), F / 32), ceil_div(c->Vs, 64));
        c->skinny_part_elems = std::max((size_t)widest * 8 * (2 * 2 * 1024 + 64), (size_t)8 * M * d);
        if ((rc = dev_alloc(c, &c->skinny_part, c->skinny_part_elems * sizeof(float)))) return rc;
        if ((rc = dev_alloc(c, &c->pf_sink, 256))) return rc;
        if ((rc = dev_alloc(c, &c->row_ssq, (size_t)M * ceil_div(d, 256) * sizeof(float)))) return rc;
        if ((rc = dev_alloc(c, &c->row_meta, (size_t)M * sizeof(QkvRow)))) return rc;
        if ((rc = dev_alloc(c, &c->row_rot, (size_t)M * (hd / 2) * sizeof(float2)))) return rc;
        c->l2_warm = !(md.kernel_flags & SJD_NO_L2_WARM);
    }
    if (c->attn_mfma) {
        // chunk length: about 640 wavefronts at full context (measured: every chunk costs a partial result of
        // 32 x hd floats per head, written and read back, which at 128-token chunks is as many bytes as the keys and
        // values themselves; fewer, longer chunks win until the workgroups no longer fill the chip), at least 128
        // tokens, a multiple of 64
        long want = (long)md.max_ctx * S * 2 * H * ceil_div(L, 32) / 640;
        int chunk = (int)((want + 63) / 64) * 64;
        if (chunk < 128) chunk = 128;
        c->attn_chunk = chunk;
        c->attn_onepass_ok = !(md.kernel_flags & SJD_ATTENTION_CHUNKED);
        c->attn_nchunks = ceil_div(md.max_ctx, chunk);
        const size_t slots = (size_t)S * 2 * H * ceil_div(L, 32) * c->attn_nchunks;
        if ((rc = dev_alloc(c, &c->part_o, slots * 32 * hd * sizeof(float)))) return rc;
        if ((rc = dev_alloc(c, &c->part_ml, slots * 64 * sizeof(float)))) return rc;
    }
    return SJD_OK;
}

int alloc_state(sjd_ctx *c) {
    const int S = c->S, L = c->L, M = S * 2 * L;
    int rc;
    if ((rc = dev_alloc(c, &c->rm.row_tok, (size_t)M * 4))) return rc;
    if ((rc = dev_alloc(c, &c->rm.row_pos, (size_t)M * 4))) return rc;
    if ((rc = dev_alloc(c, &c->rm.seg_kv, (size_t)S * 2 * 4))) return rc;
    if ((rc = dev_alloc(c, &c->rm.seg_n, (size_t)S * 2 * 4))) return rc;
    DecideState &d = c->ds;
    d.L = L; d.V = c->Vs; d.lo = c->md.sample_lo; d.max_img = c->md.max_ctx;
    if ((rc = dev_alloc(c, &d.win_tok, (size_t)S * L * 4))) return rc;
    if ((rc = dev_alloc(c, &d.anchor, (size_t)S * 2 * 4))) return rc;
    if ((rc = dev_alloc(c, &d.ref_row, (size_t)S * L * 4))) return rc;
    if ((rc = dev_alloc(c, &d.n_img, (size_t)S * 4))) return rc;
    if ((rc = dev_alloc(c, &d.n_image, (size_t)S * 4))) return rc;
    if ((rc = dev_alloc(c, &d.kv_len, (size_t)S * 2 * 4))) return rc;
    if ((rc = dev_alloc(c, &d.Le, (size_t)S * 4))) return rc;
    if ((rc = dev_alloc(c, &d.out_tok, (size_t)S * d.max_img * 4))) return rc;
    if ((rc = dev_alloc(c, &d.acc_len, (size_t)S * 4))) return rc;
    if ((rc = dev_alloc(c, &d.cand, (size_t)S * L * 4))) return rc;
    if ((rc = dev_alloc(c, &d.cand_new, (size_t)S * L * 4))) return rc;
    d.cap = c->Vs;   // room for a whole row of kept pairs (ties at the K-th value can keep everything); pages that are never
                     // written are never touched
    if (c->sp.init_mode == 4) {
        const size_t rows = (size_t)S * c->sp.row_width;
        if ((rc = dev_alloc(c, &d.hist_ids, rows * d.cap * sizeof(int32_t), false))) return rc;
        if ((rc = dev_alloc(c, &d.hist_e, rows * d.cap * sizeof(float), false))) return rc;
        if ((rc = dev_alloc(c, &d.hist_cnt, rows * sizeof(int32_t)))) return rc;
        if ((rc = dev_alloc(c, &d.hist_Z, rows * sizeof(uint64_t)))) return rc;
    }
    if ((rc = dev_alloc(c, &d.step, 4))) return rc;
    for (int b = 0; b < 2; ++b) {
        if ((rc = dev_alloc(c, &d.ids_buf[b], (size_t)S * L * d.cap * sizeof(int32_t), false))) return rc;
        if ((rc = dev_alloc(c, &d.e_buf[b], (size_t)S * L * d.cap * sizeof(float), false))) return rc;
        if ((rc = dev_alloc(c, &d.cnt_buf[b], (size_t)S * L * sizeof(int32_t)))) return rc;
        if ((rc = dev_alloc(c, &d.Z_buf[b], (size_t)S * L * sizeof(uint64_t)))) return rc;
    }
    if ((rc = dev_alloc(c, &d.allow_lo, (size_t)S * d.max_img * 4))) return rc;
    if ((rc = dev_alloc(c, &d.allow_hi, (size_t)S * d.max_img * 4))) return rc;
    if ((rc = dev_alloc(c, &d.res, (size_t)S * sizeof(sjd_step_result)))) return rc;
    if ((rc = dev_alloc(c, &c->prompt_dev, (size_t)S * 2 * c->md.max_ctx * 4))) return rc;
    if ((rc = dev_alloc(c, &c->prompt_len_dev, (size_t)S * 2 * 4))) return rc;
    if ((rc = dev_alloc(c, &c->prompt_last_dev, (size_t)S * 2 * 4))) return rc;
    if ((rc = dev_alloc(c, &c->n_image_dev, (size_t)S * 4))) return rc;
    hipError_t e = hipHostMalloc((void **)&c->res_host, (size_t)S * sizeof(sjd_step_result), hipHostMallocDefault);
    if (e != hipSuccess) { sjd_set_error(c->err, "hipHostMalloc failed: %s", hipGetErrorString(e)); return SJD_ENOMEM; }
    return SJD_OK;
}

int make_rope_tables(sjd_ctx *c) {
    const int half = c->hd / 2, n = c->md.max_ctx;
    std::vector<float> cs((size_t)n * half), sn((size_t)n * half);
    for (int pos = 0; pos < n; ++pos)
        for (int i = 0; i < half; ++i) {
            const double angle = (double)pos * pow((double)c->md.rope_theta, -2.0 * i / c->hd);
            cs[(size_t)pos * half + i] = (float)cos(angle);
            sn[(size_t)pos * half + i] = (float)sin(angle);
        }
    int rc;
    if ((rc = dev_alloc(c, &c->rope_cos, cs.size() * 4, false))) return rc;
    if ((rc = dev_alloc(c, &c->rope_sin, sn.size() * 4, false))) return rc;
    SJD_HIP_TRY(c->err, hipMemcpy(c->rope_cos, cs.data(), cs.size() * 4, hipMemcpyHostToDevice));
    SJD_HIP_TRY(c->err, hipMemcpy(c->rope_sin, sn.data(), sn.size() * 4, hipMemcpyHostToDevice));
    return SJD_OK;
}

int validate_desc(const sjd_model_desc *md, const sjd_weights *w, const sjd_sampling *sp, char *err) {
    if (!md || !w || !sp) { sjd_set_error(err, "null argument"); return SJD_EINVAL; }
    if (md->n_layers < 1 || md->d_model < 1 || md->n_heads < 1 || md->n_kv_heads < 1 || md->d_ff < 1 || md->vocab < 1) {
        sjd_set_error(err, "non-positive model dimension"); return SJD_EINVAL;
    }
    if (md->d_model % md->n_heads || md->n_heads % md->n_kv_heads) { sjd_set_error(err, "heads do not divide"); return SJD_EINVAL; }
    const int hd = md->d_model / md->n_heads;
    if (hd % 2) { sjd_set_error(err, "odd head dimension"); return SJD_EINVAL; }
    if (md->sample_lo < 0 || md->sample_hi > md->vocab || md->sample_hi <= md->sample_lo) {
        sjd_set_error(err, "bad sampled id range"); return SJD_EINVAL;
    }
    if (md->dtype != SJD_F32 && md->dtype != SJD_BF16) { sjd_set_error(err, "unknown dtype"); return SJD_EINVAL; }
    if (md->max_seqs < 1 || md->max_ctx < 2 || md->window < 1 || md->window > 1024) {
        sjd_set_error(err, "bad capacity (max_seqs >= 1, max_ctx >= 2, 1 <= window <= 1024)"); return SJD_EINVAL;
    }
    if (md->kv_page_tokens < 0 || md->kv_page_tokens % 32) { sjd_set_error(err, "kv_page_tokens must be a multiple of 32"); return SJD_EINVAL; }
    if (md->dtype == SJD_BF16 && (hd % 32 || md->d_model % 16 || md->d_ff % 16)) {
        sjd_set_error(err, "bf16 needs head_dim %% 32 == 0, d_model %% 16 == 0, d_ff %% 16 == 0"); return SJD_EINVAL;
    }
    if (!(md->rms_eps > 0.0f) || !(md->rope_theta > 0.0f)) { sjd_set_error(err, "bad rms_eps / rope_theta"); return SJD_EINVAL; }
    if (sp->top_k < 1 || !(sp->temperature > 0.0f) || sp->init_mode < 0 || sp->init_mode > 4 ||
        ((sp->init_mode == 2 || sp->init_mode == 4) && sp->row_width < 1) || sp->reuse_tau != sp->reuse_tau || sp->reuse_tau < 0.0f) {
        sjd_set_error(err, "bad sampling parameters (top_k >= 1, temperature > 0, tau >= 0, init_mode 0..4, row_width >= 1 for init_mode 2 and 4)"); return SJD_EINVAL;
    }
    if (!w->tok_emb || !w->final_norm || !w->lm_head || !w->attn_norm || !w->wq || !w->wk || !w->wv || !w->wo || !w->mlp_norm ||
        !w->w_gate || !w->w_up || !w->w_down) {
        sjd_set_error(err, "null weight pointer"); return SJD_EINVAL;
    }
    return SJD_OK;
}

// from_logits: the logits buffer was filled by the caller (no forward ran): the guided logits are computed from it
int run_decide(sjd_ctx *c, bool from_logits) {
    SJD_LAUNCH(c, KC_SAMPLE_ROWS, launch_sample_rows(c->stream, c->ds, c->sp, c->logits, c->n_seqs, c->z_used && !from_logits ? c->z : nullptr));
    SJD_LAUNCH(c, KC_VERIFY, launch_verify(c->stream, c->ds, c->sp, c->n_seqs));
    SJD_LAUNCH(c, KC_DRAW, launch_draw(c->stream, c->ds, c->sp, c->n_seqs));
    if (c->sp.init_mode == 4) SJD_LAUNCH(c, KC_COMMIT, launch_keep_rows(c->stream, c->ds, c->sp, c->n_seqs));
    SJD_LAUNCH(c, KC_COMMIT, launch_commit(c->stream, c->ds, c->sp, c->n_seqs));
    return SJD_OK;
}

int finish_step(sjd_ctx *c, sjd_step_result *out) {
    SJD_HIP_TRY(c->err, hipMemcpyAsync(c->res_host, c->ds.res, (size_t)c->n_seqs * sizeof(sjd_step_result), hipMemcpyDeviceToHost,
                                       c->stream));
    SJD_HIP_TRY(c->err, hipStreamSynchronize(c->stream));
    trace_collect(c);
    bool all = true;
    for (int s = 0; s < c->n_seqs; ++s) {
        out[s] = c->res_host[s];
        all = all && out[s].done;
        c->kv_host[s * 2] += out[s].n_finalized;
        c->kv_host[s * 2 + 1] += out[s].n_finalized;
    }
    c->all_done = all;
    return SJD_OK;
}

// everything one decoding step launches, in stream order (the host reads the verdicts back afterwards)
int enqueue_step(sjd_ctx *c) {
    SJD_LAUNCH(c, KC_STAGE, launch_stage_window(c->stream, c->ds, c->rm, c->n_seqs));
    int rc = forward_any(c, true);
    if (rc) return rc;
    return run_decide(c, false);
}

void drop_graph(sjd_ctx *c, int g) {
    if (c->graph_exec[g]) (void)hipGraphExecDestroy(c->graph_exec[g]);
    if (c->graph[g]) (void)hipGraphDestroy(c->graph[g]);
    c->graph_exec[g] = nullptr;
    c->graph[g] = nullptr;
    c->graph_n_seqs[g] = 0;
}

// one-pass attention for the coming launches iff the longest visible context (cache + rows) is short
void choose_attention(sjd_ctx *c, int max_kv) {
    c->attn_onepass = c->attn_mfma && c->attn_onepass_ok && attention_onepass_pays(max_kv + c->L, c->hd, c->n_seqs * 2 * c->md.n_heads, c->n_cus);
}

}  // namespace

// =================================================================================================
extern "C" {

const char *sjd_last_error(const sjd_ctx *ctx) { return ctx ? ctx->err : g_create_error; }

void sjd_destroy(sjd_ctx *c) {
    if (!c) return;
    (void)hipStreamSynchronize(c->stream);
    drop_graph(c, 0);
    drop_graph(c, 1);
    for (void *p : c->allocations) (void)hipFree(p);
    if (c->res_host) (void)hipHostFree(c->res_host);
    for (hipEvent_t e : c->tracer.pool) (void)hipEventDestroy(e);
    delete c;
}

int sjd_create(const sjd_model_desc *desc, const sjd_weights *weights, const sjd_sampling *sampling, void *hip_stream,
               sjd_ctx **out) {
    if (!out) { sjd_set_error(g_create_error, "null output pointer"); return SJD_EINVAL; }
    *out = nullptr;
    int rc = validate_desc(desc, weights, sampling, g_create_error);
    if (rc) return rc;
    sjd_ctx *c = new (std::nothrow) sjd_ctx();
    if (!c) { sjd_set_error(g_create_error, "out of host memory"); return SJD_ENOMEM; }
    c->md = *desc;
    c->sampling = *sampling;
    c->stream = (hipStream_t)hip_stream;
    c->hd = desc->d_model / desc->n_heads;
    c->Vs = desc->sample_hi - desc->sample_lo;
    c->L = desc->window;
    c->S = desc->max_seqs;
    c->pt = desc->kv_page_tokens ? desc->kv_page_tokens : 64;
    c->md.kv_page_tokens = c->pt;
    c->max_visible = desc->max_ctx + 1;
    c->sp.cfg_scale = sampling->cfg_scale;
    c->sp.inv_temperature = 1.0f / sampling->temperature;
    c->sp.tau = sampling->reuse_tau;
    c->sp.top_k = sampling->top_k;
    c->sp.seed = sampling->seed;
    c->sp.init_mode = sampling->init_mode;
    c->sp.row_width = sampling->row_width;
    {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess) {
            if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) c->n_cus = v;
            if (hipDeviceGetAttribute(&v, hipDeviceAttributeNumberOfXccs, dev) == hipSuccess && v > 0) c->n_xcds = v;
        }
        (void)hipGetLastError();
    }
    c->keep_logits = (desc->kernel_flags & SJD_KEEP_LOGITS) != 0;
    const bool f32 = desc->dtype == SJD_F32;
    c->use_graph = !(desc->kernel_flags & SJD_NO_GRAPH) && hip_stream != nullptr;  // the default stream cannot be captured
    c->attn_mfma = !f32 && !(desc->kernel_flags & SJD_KERNELS_REFERENCE) &&
                   attention_mfma_supported(c->L, desc->n_heads, desc->n_kv_heads, c->hd, c->pt);
    c->fused = !f32 && !(desc->kernel_flags & SJD_KERNELS_REFERENCE) && c->hd % 64 == 0 && (c->S * 2 * c->L <= 64 || (2 * c->L) % 64 == 0) &&
               desc->d_model % 32 == 0 && desc->d_ff % 32 == 0;
    rc = f32 ? copy_weights<float>(c, weights) : (c->fused ? copy_weights_fused(c, weights) : copy_weights<bf16_t>(c, weights));
    if (!rc) rc = f32 ? alloc_buffers<float>(c) : alloc_buffers<bf16_t>(c);
    if (!rc) rc = alloc_state(c);
    if (!rc) rc = make_rope_tables(c);
    if (!rc && hipStreamSynchronize(c->stream) != hipSuccess) {
        sjd_set_error(c->err, "device error while copying the weights: %s", hipGetErrorString(hipGetLastError()));
        rc = SJD_EDEVICE;
    }
    if (rc) {
        memcpy(g_create_error, c->err, sizeof g_create_error);
        sjd_destroy(c);
        return rc;
    }
    *out = c;
    return SJD_OK;
}

int sjd_prefill(sjd_ctx *c, int32_t n_seqs, const int32_t *const *cond_ids, const int32_t *cond_len,
                const int32_t *const *uncond_ids, const int32_t *uncond_len, const int32_t *n_image_tokens) {
    if (!c) return SJD_EINVAL;
    if (!cond_ids || !cond_len || !uncond_ids || !uncond_len || !n_image_tokens || n_seqs < 1) {
        sjd_set_error(c->err, "null argument or n_seqs < 1");
        return SJD_EINVAL;
    }
    if (n_seqs > c->S) { sjd_set_error(c->err, "n_seqs %d > max_seqs %d", n_seqs, c->S); return SJD_ECAPACITY; }
    int max_prompt = 1;
    for (int s = 0; s < n_seqs; ++s) {
        if (!cond_ids[s] || !uncond_ids[s] || cond_len[s] < 1 || uncond_len[s] < 1 || n_image_tokens[s] < 1) {
            sjd_set_error(c->err, "sequence %d: null prompt, empty prompt or no image tokens", s);
            return SJD_EINVAL;
        }
        if (cond_len[s] + n_image_tokens[s] > c->md.max_ctx || uncond_len[s] + n_image_tokens[s] > c->md.max_ctx) {
            sjd_set_error(c->err, "sequence %d: prompt + image tokens exceed max_ctx %d", s, c->md.max_ctx);
            return SJD_ECAPACITY;
        }
        for (int i = 0; i < cond_len[s]; ++i)
            if (cond_ids[s][i] < 0 || cond_ids[s][i] >= c->md.vocab) { sjd_set_error(c->err, "token id outside the vocabulary"); return SJD_EINVAL; }
        for (int i = 0; i < uncond_len[s]; ++i)
            if (uncond_ids[s][i] < 0 || uncond_ids[s][i] >= c->md.vocab) { sjd_set_error(c->err, "token id outside the vocabulary"); return SJD_EINVAL; }
        if (cond_len[s] > max_prompt) max_prompt = cond_len[s];
        if (uncond_len[s] > max_prompt) max_prompt = uncond_len[s];
    }
    c->prefilled = false;
    c->n_seqs = n_seqs;
    const int L = c->L;
    // host staging
    std::vector<int32_t> prompt((size_t)n_seqs * 2 * max_prompt, 0), plen((size_t)n_seqs * 2), plast((size_t)n_seqs * 2);
    std::vector<int32_t> table((size_t)c->S * 2 * c->pps, 0);
    // Pages are handed out round-robin over the segments, so that the pages of one segment are not
    // contiguous in the pool; a segment takes only the pages its prompt + image need.
    {
        std::vector<int> need((size_t)n_seqs * 2), got((size_t)n_seqs * 2, 0);
        int next = 0, pending = 0;
        for (int s = 0; s < n_seqs; ++s) {
            need[s * 2] = ceil_div(cond_len[s] + n_image_tokens[s], c->pt);
            need[s * 2 + 1] = ceil_div(uncond_len[s] + n_image_tokens[s], c->pt);
            pending += need[s * 2] + need[s * 2 + 1];
        }
        if (pending > c->n_pages) { sjd_set_error(c->err, "KV page pool exhausted"); return SJD_ECAPACITY; }
        while (pending > 0)
            for (int seg = 0; seg < n_seqs * 2; ++seg)
                if (got[seg] < need[seg]) { table[(size_t)seg * c->pps + got[seg]++] = next++; --pending; }
    }
    for (int s = 0; s < n_seqs; ++s) {
        const int32_t *ids[2] = {cond_ids[s], uncond_ids[s]};
        const int len[2] = {cond_len[s], uncond_len[s]};
        for (int b = 0; b < 2; ++b) {
            memcpy(&prompt[((size_t)s * 2 + b) * max_prompt], ids[b], sizeof(int32_t) * len[b]);
            plen[s * 2 + b] = len[b];
            plast[s * 2 + b] = ids[b][len[b] - 1];
        }
    }
    hipStream_t st = c->stream;
    SJD_HIP_TRY(c->err, hipMemcpyAsync(c->prompt_dev, prompt.data(), prompt.size() * 4, hipMemcpyHostToDevice, st));
    SJD_HIP_TRY(c->err, hipMemcpyAsync(c->prompt_len_dev, plen.data(), plen.size() * 4, hipMemcpyHostToDevice, st));
    SJD_HIP_TRY(c->err, hipMemcpyAsync(c->prompt_last_dev, plast.data(), plast.size() * 4, hipMemcpyHostToDevice, st));
    SJD_HIP_TRY(c->err, hipMemcpyAsync(c->n_image_dev, n_image_tokens, (size_t)n_seqs * 4, hipMemcpyHostToDevice, st));
    SJD_HIP_TRY(c->err, hipMemcpyAsync(c->page_table, table.data(), table.size() * 4, hipMemcpyHostToDevice, st));
    SJD_HIP_TRY(c->err, hipStreamSynchronize(st));  // the host staging vectors may go away on an early return
    c->page_table_host = table;
    c->n_image_host.assign(n_image_tokens, n_image_tokens + n_seqs);
    c->kv_host.assign((size_t)n_seqs * 2, 0);
    for (int s = 0; s < n_seqs; ++s) { c->kv_host[s * 2] = cond_len[s] - 1; c->kv_host[s * 2 + 1] = uncond_len[s] - 1; }
    const int chunks = ceil_div(max_prompt - 1, L);
    for (int ch = 0; ch < chunks; ++ch) {
        choose_attention(c, ch * L);
        SJD_LAUNCH(c, KC_STAGE, launch_stage_prompt(st, c->rm, c->prompt_dev, c->prompt_len_dev, max_prompt, ch, L, n_seqs));
        int rc = forward_any(c, false);
        if (rc) return rc;
    }
    SJD_LAUNCH(c, KC_STAGE, launch_init_window(st, c->ds, c->sp, n_seqs, c->S, c->prompt_last_dev, c->prompt_len_dev, c->n_image_dev));
    SJD_HIP_TRY(c->err, hipStreamSynchronize(st));
    trace_collect(c);
    c->prefilled = true;
    c->all_done = false;
    return SJD_OK;
}

int sjd_step(sjd_ctx *c, sjd_step_result *out) {
    if (!c) return SJD_EINVAL;
    if (!out) { sjd_set_error(c->err, "null result pointer"); return SJD_EINVAL; }
    if (!c->prefilled) { sjd_set_error(c->err, "sjd_step before sjd_prefill"); return SJD_ESTATE; }
    int rc;
    int max_kv = 0;
    for (int32_t kv : c->kv_host) max_kv = std::max(max_kv, (int)kv);
    choose_attention(c, max_kv);
    const int g = c->attn_onepass ? 1 : 0;
    if (c->use_graph && !c->tracer.on) {   // per-kernel event timing needs the kernels one by one
        if (c->graph_exec[g] && c->graph_n_seqs[g] != c->n_seqs) drop_graph(c, g);
        if (!c->graph_exec[g]) {
            SJD_HIP_TRY(c->err, hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal));
            rc = enqueue_step(c);
            hipGraph_t gr = nullptr;
            const hipError_t e = hipStreamEndCapture(c->stream, &gr);  // always end the capture, also after a failed launch
            if (rc) { if (gr) (void)hipGraphDestroy(gr); return rc; }
            if (e != hipSuccess || !gr) { sjd_set_error(c->err, "stream capture of the step failed: %s", hipGetErrorString(e)); return SJD_EDEVICE; }
            c->graph[g] = gr;
            SJD_HIP_TRY(c->err, hipGraphInstantiate(&c->graph_exec[g], c->graph[g], nullptr, nullptr, 0));
            c->graph_n_seqs[g] = c->n_seqs;
        }
        SJD_HIP_TRY(c->err, hipGraphLaunch(c->graph_exec[g], c->stream));
    } else if ((rc = enqueue_step(c))) {
        return rc;
    }
    return finish_step(c, out);
}

int sjd_debug_step_from_logits(sjd_ctx *c, const float *logits_host, sjd_step_result *out) {
    if (!c) return SJD_EINVAL;
    if (!out || !logits_host) { sjd_set_error(c->err, "null pointer"); return SJD_EINVAL; }
    if (!c->prefilled) { sjd_set_error(c->err, "step before sjd_prefill"); return SJD_ESTATE; }
    SJD_HIP_TRY(c->err, hipMemcpyAsync(c->logits, logits_host, (size_t)c->n_seqs * 2 * c->L * c->Vs * sizeof(float),
                                       hipMemcpyHostToDevice, c->stream));
    SJD_LAUNCH(c, KC_STAGE, launch_stage_window(c->stream, c->ds, c->rm, c->n_seqs));
    int rc = run_decide(c, true);
    if (rc) return rc;
    return finish_step(c, out);
}

int sjd_debug_copy_logits(sjd_ctx *c, float *dst_host) {
    if (!c || !dst_host) return SJD_EINVAL;
    if (!c->prefilled) { sjd_set_error(c->err, "no step yet"); return SJD_ESTATE; }
    if (c->z_used && !c->keep_logits) {
        sjd_set_error(c->err, "the logits are not kept: this context's vocabulary head writes guided logits only (create it with SJD_KEEP_LOGITS)");
        return SJD_ESTATE;
    }
    SJD_HIP_TRY(c->err, hipStreamSynchronize(c->stream));
    SJD_HIP_TRY(c->err, hipMemcpy(dst_host, c->logits, (size_t)c->n_seqs * 2 * c->L * c->Vs * sizeof(float), hipMemcpyDeviceToHost));
    return SJD_OK;
}

int sjd_get_tokens(sjd_ctx *c, int32_t seq, int32_t *dst, int32_t cap, int32_t *n_out) {
    if (!c || !n_out) return SJD_EINVAL;
    if (!c->prefilled) { sjd_set_error(c->err, "no prefill yet"); return SJD_ESTATE; }
    if (seq < 0 || seq >= c->n_seqs || cap < 0 || (cap > 0 && !dst)) { sjd_set_error(c->err, "bad sequence index or buffer"); return SJD_EINVAL; }
    int32_t n = 0;
    SJD_HIP_TRY(c->err, hipStreamSynchronize(c->stream));
    SJD_HIP_TRY(c->err, hipMemcpy(&n, c->ds.n_img + seq, 4, hipMemcpyDeviceToHost));
    const int32_t k = n < cap ? n : cap;
    if (k > 0) SJD_HIP_TRY(c->err, hipMemcpy(dst, c->ds.out_tok + (size_t)seq * c->ds.max_img, (size_t)k * 4, hipMemcpyDeviceToHost));
    *n_out = n;
    return SJD_OK;
}

int sjd_get_window(sjd_ctx *c, int32_t seq, int32_t *tokens, int32_t *ref_rows, int32_t *n_slots) {
    if (!c || !tokens || !ref_rows || !n_slots) return SJD_EINVAL;
    if (!c->prefilled) { sjd_set_error(c->err, "no prefill yet"); return SJD_ESTATE; }
    if (seq < 0 || seq >= c->n_seqs) { sjd_set_error(c->err, "bad sequence index"); return SJD_EINVAL; }
    const int L = c->L;
    int32_t le = 0;
    SJD_HIP_TRY(c->err, hipStreamSynchronize(c->stream));
    SJD_HIP_TRY(c->err, hipMemcpy(tokens, c->ds.win_tok + (size_t)seq * L, (size_t)L * 4, hipMemcpyDeviceToHost));
    SJD_HIP_TRY(c->err, hipMemcpy(ref_rows, c->ds.ref_row + (size_t)seq * L, (size_t)L * 4, hipMemcpyDeviceToHost));
    SJD_HIP_TRY(c->err, hipMemcpy(tokens, c->ds.anchor + (size_t)seq * 2, 4, hipMemcpyDeviceToHost));
    SJD_HIP_TRY(c->err, hipMemcpy(&le, c->ds.Le + seq, 4, hipMemcpyDeviceToHost));
    ref_rows[0] = -1;
    *n_slots = le;
    return SJD_OK;
}

int sjd_set_token_ranges(sjd_ctx *c, int32_t seq, const int32_t *first_id, const int32_t *end_id, int32_t n_positions) {
    if (!c) return SJD_EINVAL;
    if (!c->prefilled) { sjd_set_error(c->err, "sjd_set_token_ranges before sjd_prefill"); return SJD_ESTATE; }
    if (seq < 0 || seq >= c->n_seqs || !first_id || !end_id || n_positions < 0 || (size_t)seq >= c->n_image_host.size() ||
        n_positions > c->n_image_host[seq]) {
        sjd_set_error(c->err, "bad sequence index, null array or more positions than image tokens");
        return SJD_EINVAL;
    }
    std::vector<int32_t> lo(n_positions), hi(n_positions);
    for (int i = 0; i < n_positions; ++i) {
        if (first_id[i] < c->md.sample_lo || end_id[i] > c->md.sample_hi || first_id[i] >= end_id[i]) {
            sjd_set_error(c->err, "position %d: id range [%d, %d) is empty or leaves the sampled ids", i, first_id[i], end_id[i]);
            return SJD_EINVAL;
        }
        lo[i] = first_id[i] - c->md.sample_lo;
        hi[i] = end_id[i] - c->md.sample_lo;
    }
    SJD_HIP_TRY(c->err, hipStreamSynchronize(c->stream));
    if (n_positions > 0) {
        SJD_HIP_TRY(c->err, hipMemcpy(c->ds.allow_lo + (size_t)seq * c->ds.max_img, lo.data(), (size_t)n_positions * 4, hipMemcpyHostToDevice));
        SJD_HIP_TRY(c->err, hipMemcpy(c->ds.allow_hi + (size_t)seq * c->ds.max_img, hi.data(), (size_t)n_positions * 4, hipMemcpyHostToDevice));
    }
    return SJD_OK;
}

int sjd_trace_enable(sjd_ctx *c, int32_t on) {
    if (!c) return SJD_EINVAL;
    c->tracer.on = on != 0;
    return SJD_OK;
}
int sjd_trace_reset(sjd_ctx *c) {
    if (!c) return SJD_EINVAL;
    for (int i = 0; i < KC_COUNT; ++i) { c->tracer.launches[i] = 0; c->tracer.total_ms[i] = 0.0; }
    return SJD_OK;
}
int sjd_trace_read(sjd_ctx *c, sjd_trace_entry *dst, int32_t cap, int32_t *n_out) {
    if (!c || !n_out || (cap > 0 && !dst)) return SJD_EINVAL;
    for (int i = 0; i < KC_COUNT && i < cap; ++i) {
        dst[i].name = kKernelClassName[i];
        dst[i].launches = c->tracer.launches[i];
        dst[i].total_ms = c->tracer.total_ms[i];
    }
    *n_out = KC_COUNT;
    return SJD_OK;
}

}  // extern "C"

// ------------------------------------------------------------------------------------------ snapshots
// The state that Sec. 4.1 carries from one iteration to the next: the accepted tokens, the window's drafts with the
// rows they were drawn from (the previous iteration's distributions), and the cache of the accepted prefix.
namespace {

struct SnapshotHeader {
    uint64_t magic, total_bytes;
    int32_t version, n_seqs, all_done;
    // the context a snapshot fits: same model, capacities and sampling set-up
    int32_t n_layers, d_model, n_heads, n_kv_heads, hd, Vs, L, S, max_ctx, pt, pps, dtype, init_mode, row_width;
    uint64_t seed;
    float cfg_scale, temperature, reuse_tau;
    int32_t top_k;
    int32_t pages_used[1];  // [n_seqs * 2] follows (flexible; the struct is written with its real length)
};
constexpr uint64_t kSnapshotMagic = 0x31544e53444a53ull;  // "SJDSNT1"

// the per-sequence device arrays of the decoding state: pointer, bytes per sequence
struct StateArray { void *p; size_t per_seq; };
std::vector<StateArray> state_arrays(sjd_ctx *c) {
    const DecideState &d = c->ds;
    const size_t L = c->L, V = c->Vs;
    const size_t cap = d.cap;
    std::vector<StateArray> a = {
        {d.win_tok, L * 4}, {d.anchor, 8}, {d.ref_row, L * 4}, {d.n_img, 4}, {d.n_image, 4}, {d.kv_len, 8}, {d.Le, 4},
        {d.out_tok, (size_t)d.max_img * 4}, {d.acc_len, 4}, {d.cand, L * 4}, {d.cand_new, L * 4},
        {d.ids_buf[0], L * cap * 4}, {d.ids_buf[1], L * cap * 4}, {d.e_buf[0], L * cap * 4}, {d.e_buf[1], L * cap * 4},
        {d.cnt_buf[0], L * 4}, {d.cnt_buf[1], L * 4}, {d.Z_buf[0], L * 8}, {d.Z_buf[1], L * 8},
        {d.allow_lo, (size_t)d.max_img * 4}, {d.allow_hi, (size_t)d.max_img * 4}, {d.res, sizeof(sjd_step_result)}};
    if (c->sp.init_mode == 4) {
        a.push_back({d.hist_ids, (size_t)c->sp.row_width * cap * 4});
        a.push_back({d.hist_e, (size_t)c->sp.row_width * cap * 4});
        a.push_back({d.hist_cnt, (size_t)c->sp.row_width * 4});
        a.push_back({d.hist_Z, (size_t)c->sp.row_width * 8});
    }
    (void)V;
    return a;
}
size_t snapshot_header_bytes(int n_seqs) { return (sizeof(SnapshotHeader) + (size_t)(2 * n_seqs) * 4 + 15) / 16 * 16; }

// pages in use per segment (committed positions only: the window's entries are rewritten by every step)
int snapshot_pages(sjd_ctx *c, std::vector<int32_t> &pages) {
    std::vector<int32_t> kv((size_t)c->n_seqs * 2);
    SJD_HIP_TRY(c->err, hipStreamSynchronize(c->stream));
    SJD_HIP_TRY(c->err, hipMemcpy(kv.data(), c->ds.kv_len, kv.size() * 4, hipMemcpyDeviceToHost));
    pages.resize(kv.size());
    for (size_t i = 0; i < kv.size(); ++i) pages[i] = ceil_div(kv[i], c->pt);
    return SJD_OK;
}
size_t snapshot_bytes(sjd_ctx *c, int n_seqs, const std::vector<int32_t> &pages) {
    size_t n = snapshot_header_bytes(n_seqs) + (size_t)c->S * 2 * c->pps * 4 + 16 /* step counter */;
    for (const StateArray &a : state_arrays(c)) n += a.per_seq * n_seqs;
    size_t total_pages = 0;
    for (int32_t p : pages) total_pages += p;
    const size_t page_bytes = c->pool_layer_bytes / c->n_pages;  // one page of one layer's key (or value) pool, all kv heads
    return n + total_pages * page_bytes * 2 * c->md.n_layers;
}
bool snapshot_fits(const sjd_ctx *c, const SnapshotHeader &h) {
    return h.n_layers == c->md.n_layers && h.d_model == c->md.d_model && h.n_heads == c->md.n_heads &&
           h.n_kv_heads == c->md.n_kv_heads && h.hd == c->hd && h.Vs == c->Vs && h.L == c->L && h.S == c->S &&
           h.max_ctx == c->md.max_ctx && h.pt == c->pt && h.pps == c->pps && h.dtype == c->md.dtype &&
           h.init_mode == c->sp.init_mode && h.row_width == c->sp.row_width && h.seed == c->sp.seed &&
           h.cfg_scale == c->sampling.cfg_scale && h.temperature == c->sampling.temperature &&
           (h.reuse_tau == c->sampling.reuse_tau || (h.reuse_tau != h.reuse_tau && c->sampling.reuse_tau != c->sampling.reuse_tau)) &&
           h.top_k == c->sampling.top_k;
}

}  // namespace

extern "C" {

int sjd_snapshot_size(sjd_ctx *c, uint64_t *bytes) {
    if (!c || !bytes) return SJD_EINVAL;
    if (!c->prefilled) { sjd_set_error(c->err, "no prefill yet"); return SJD_ESTATE; }
    std::vector<int32_t> pages;
    int rc = snapshot_pages(c, pages);
    if (rc) return rc;
    *bytes = snapshot_bytes(c, c->n_seqs, pages);
    return SJD_OK;
}

int sjd_snapshot_save(sjd_ctx *c, void *dst_host, uint64_t cap, uint64_t *written) {
    if (!c || !dst_host || !written) return SJD_EINVAL;
    if (!c->prefilled) { sjd_set_error(c->err, "no prefill yet"); return SJD_ESTATE; }
    std::vector<int32_t> pages;
    int rc = snapshot_pages(c, pages);
    if (rc) return rc;
    const size_t total = snapshot_bytes(c, c->n_seqs, pages);
    if (cap < total) { sjd_set_error(c->err, "snapshot needs %zu bytes, buffer has %llu", total, (unsigned long long)cap); return SJD_ECAPACITY; }
    char *w = (char *)dst_host;
    const size_t hb = snapshot_header_bytes(c->n_seqs);
    memset(w, 0, hb);
    SnapshotHeader *h = (SnapshotHeader *)w;
    h->magic = kSnapshotMagic; h->total_bytes = total; h->version = 1; h->n_seqs = c->n_seqs; h->all_done = c->all_done;
    h->n_layers = c->md.n_layers; h->d_model = c->md.d_model; h->n_heads = c->md.n_heads; h->n_kv_heads = c->md.n_kv_heads;
    h->hd = c->hd; h->Vs = c->Vs; h->L = c->L; h->S = c->S; h->max_ctx = c->md.max_ctx; h->pt = c->pt; h->pps = c->pps;
    h->dtype = c->md.dtype; h->init_mode = c->sp.init_mode; h->row_width = c->sp.row_width; h->seed = c->sp.seed;
    h->cfg_scale = c->sampling.cfg_scale; h->temperature = c->sampling.temperature; h->reuse_tau = c->sampling.reuse_tau;
    h->top_k = c->sampling.top_k;
    memcpy(h->pages_used, pages.data(), pages.size() * 4);
    w += hb;
    memcpy(w, c->page_table_host.data(), c->page_table_host.size() * 4);
    w += c->page_table_host.size() * 4;
    SJD_HIP_TRY(c->err, hipMemcpy(w, c->ds.step, 4, hipMemcpyDeviceToHost));
    w += 16;
    for (const StateArray &a : state_arrays(c)) {
        SJD_HIP_TRY(c->err, hipMemcpy(w, a.p, a.per_seq * c->n_seqs, hipMemcpyDeviceToHost));
        w += a.per_seq * c->n_seqs;
    }
    const size_t page_bytes = c->pool_layer_bytes / c->n_pages;  // one page of one layer's key (or value) pool, all kv heads
    for (int l = 0; l < c->md.n_layers; ++l)
        for (int kv = 0; kv < 2; ++kv) {
            const char *pool = (const char *)(kv ? c->vpool : c->kpool) + c->pool_layer_bytes * l;
            for (int seg = 0; seg < c->n_seqs * 2; ++seg)
                for (int i = 0; i < pages[seg]; ++i) {
                    const int page = c->page_table_host[(size_t)seg * c->pps + i];
                    SJD_HIP_TRY(c->err, hipMemcpyAsync(w, pool + (size_t)page * page_bytes, page_bytes, hipMemcpyDeviceToHost, c->stream));
                    w += page_bytes;
                }
        }
    SJD_HIP_TRY(c->err, hipStreamSynchronize(c->stream));
    *written = (uint64_t)(w - (char *)dst_host);
    return SJD_OK;
}

int sjd_snapshot_restore(sjd_ctx *c, const void *src_host, uint64_t bytes) {
    if (!c || !src_host) return SJD_EINVAL;
    if (bytes < sizeof(SnapshotHeader)) { sjd_set_error(c->err, "snapshot truncated"); return SJD_EINVAL; }
    const SnapshotHeader *h = (const SnapshotHeader *)src_host;
    if (h->magic != kSnapshotMagic || h->version != 1) { sjd_set_error(c->err, "not a snapshot of this library version"); return SJD_EINVAL; }
    if (!snapshot_fits(c, *h)) { sjd_set_error(c->err, "snapshot was taken from a context with another model, capacity or sampling set-up"); return SJD_EINVAL; }
    if (h->n_seqs < 1 || h->n_seqs > c->S || h->total_bytes != bytes) { sjd_set_error(c->err, "snapshot truncated or corrupt"); return SJD_EINVAL; }
    const int n_seqs = h->n_seqs;
    std::vector<int32_t> pages(h->pages_used, h->pages_used + 2 * n_seqs);
    for (int32_t p : pages)
        if (p < 0 || p > c->pps) { sjd_set_error(c->err, "snapshot corrupt (page count)"); return SJD_EINVAL; }
    if (bytes < snapshot_header_bytes(n_seqs) || snapshot_bytes(c, n_seqs, pages) != bytes) {
        sjd_set_error(c->err, "snapshot truncated or corrupt");
        return SJD_EINVAL;
    }
    const char *r = (const char *)src_host + snapshot_header_bytes(n_seqs);
    const size_t table_n = (size_t)c->S * 2 * c->pps;
    std::vector<int32_t> table((const int32_t *)r, (const int32_t *)r + table_n);
    for (int seg = 0; seg < n_seqs * 2; ++seg)
        for (int i = 0; i < pages[seg]; ++i)
            if (table[(size_t)seg * c->pps + i] < 0 || table[(size_t)seg * c->pps + i] >= c->n_pages) {
                sjd_set_error(c->err, "snapshot corrupt (page table)");
                return SJD_EINVAL;
            }
    // The decoding state: the kernels index memory with these values, so every one of them is checked against the
    // context's capacities before anything is uploaded (a buffer of the right size with wrong contents must be an
    // error here, not an out-of-bounds access in the next step).
    {
        const std::vector<StateArray> arrays = state_arrays(c);
        std::vector<const char *> at(arrays.size());
        const char *q = r + table_n * 4 + 16;
        for (size_t i = 0; i < arrays.size(); ++i) { at[i] = q; q += arrays[i].per_seq * n_seqs; }
        enum { A_WIN, A_ANCHOR, A_REF, A_NIMG, A_NIMAGE, A_KV, A_LE, A_OUT, A_ACC, A_CAND, A_CANDNEW, A_IDS0, A_IDS1, A_E0, A_E1,
               A_CNT0, A_CNT1, A_Z0, A_Z1, A_ALO, A_AHI, A_RES, A_HIDS, A_HE, A_HCNT, A_HZ };
        auto i32 = [&](int which, size_t idx) { return ((const int32_t *)at[which])[idx]; };
        const int L = c->L, V = c->Vs, cap = c->ds.cap, max_img = c->ds.max_img, lo = c->md.sample_lo, hi = c->md.sample_hi;
        const int rw = c->sp.init_mode == 4 ? c->sp.row_width : 0;
        auto bad = [&](const char *what, int s) { sjd_set_error(c->err, "snapshot corrupt (%s of sequence %d)", what, s); return SJD_EINVAL; };
        for (int s = 0; s < n_seqs; ++s) {
            const int n_image = i32(A_NIMAGE, s), n_img = i32(A_NIMG, s), Le = i32(A_LE, s);
            if (n_image < 0 || n_image > max_img || n_img < 0 || n_img > n_image) return bad("token counts", s);
            if (Le < 0 || Le > L || Le > n_image - n_img) return bad("window length", s);
            for (int b = 0; b < 2; ++b) {
                const int kv = i32(A_KV, (size_t)s * 2 + b);
                if (kv < 0 || (long)kv + (n_image - n_img) > c->md.max_ctx) return bad("cache length", s);
                // every page the rest of the decode will read or write
                const int need = ceil_div(kv + (n_image - n_img), c->pt);
                for (int i = 0; i < need; ++i) {
                    const int32_t pg = table[((size_t)s * 2 + b) * c->pps + i];
                    if (pg < 0 || pg >= c->n_pages) return bad("page table", s);
                }
                const int anchor = i32(A_ANCHOR, (size_t)s * 2 + b);
                if (anchor < 0 || anchor >= c->md.vocab) return bad("window tokens", s);
            }
            if (i32(A_ACC, s) < -1 || i32(A_ACC, s) >= L) return bad("accept count", s);
            for (int k = 1; k < Le; ++k) {
                const int tok = i32(A_WIN, (size_t)s * L + k), ref = i32(A_REF, (size_t)s * L + k);
                if (tok < lo || tok >= hi) return bad("window tokens", s);
                if (ref >= L || ref < -2 - rw) return bad("reference rows", s);
            }
            for (int k = 0; k < L; ++k) {
                const int t0 = i32(A_CAND, (size_t)s * L + k), t1 = i32(A_CANDNEW, (size_t)s * L + k);
                if (t0 < 0 || t0 >= c->md.vocab || t1 < 0 || t1 >= c->md.vocab) return bad("drawn tokens", s);
            }
            for (int i = 0; i < n_image; ++i) {
                const int a0 = i32(A_ALO, (size_t)s * max_img + i), a1 = i32(A_AHI, (size_t)s * max_img + i);
                if (a0 < 0 || a1 > V || a0 >= a1) return bad("token ranges", s);
            }
            auto rows_ok = [&](int ids_arr, int cnt_arr, size_t row0, int n_rows) {
                for (int k = 0; k < n_rows; ++k) {
                    const int n = i32(cnt_arr, row0 + k);
                    if (n < 0 || n > cap) return false;
                    const int32_t *ids = (const int32_t *)at[ids_arr] + (row0 + k) * cap;
                    for (int i = 0; i < n; ++i)
                        if (ids[i] < 0 || ids[i] >= V || (i > 0 && ids[i] <= ids[i - 1])) return false;
                }
                return true;
            };
            if (!rows_ok(A_IDS0, A_CNT0, (size_t)s * L, L) || !rows_ok(A_IDS1, A_CNT1, (size_t)s * L, L)) return bad("stored rows", s);
            if (rw > 0 && !rows_ok(A_HIDS, A_HCNT, (size_t)s * rw, rw)) return bad("kept rows", s);
        }
    }
    // everything checked: from here on the context's batch is replaced
    SJD_HIP_TRY(c->err, hipStreamSynchronize(c->stream));
    c->prefilled = false;
    c->n_seqs = n_seqs;
    c->page_table_host = table;
    SJD_HIP_TRY(c->err, hipMemcpy(c->page_table, table.data(), table_n * 4, hipMemcpyHostToDevice));
    r += table_n * 4;
    SJD_HIP_TRY(c->err, hipMemcpy(c->ds.step, r, 4, hipMemcpyHostToDevice));
    r += 16;
    for (const StateArray &a : state_arrays(c)) {
        SJD_HIP_TRY(c->err, hipMemcpy(a.p, r, a.per_seq * n_seqs, hipMemcpyHostToDevice));
        r += a.per_seq * n_seqs;
    }
    const size_t page_bytes = c->pool_layer_bytes / c->n_pages;  // one page of one layer's key (or value) pool, all kv heads
    for (int l = 0; l < c->md.n_layers; ++l)
        for (int kv = 0; kv < 2; ++kv) {
            char *pool = (char *)(kv ? c->vpool : c->kpool) + c->pool_layer_bytes * l;
            for (int seg = 0; seg < n_seqs * 2; ++seg)
                for (int i = 0; i < pages[seg]; ++i) {
                    const int page = table[(size_t)seg * c->pps + i];
                    SJD_HIP_TRY(c->err, hipMemcpyAsync(pool + (size_t)page * page_bytes, r, page_bytes, hipMemcpyHostToDevice, c->stream));
                    r += page_bytes;
                }
        }
    SJD_HIP_TRY(c->err, hipStreamSynchronize(c->stream));
    c->all_done = h->all_done != 0;
    c->prefilled = true;
    {   // host copy of the image lengths (sjd_set_token_ranges checks against it)
        const std::vector<StateArray> arrays = state_arrays(c);
        const char *q = (const char *)src_host + snapshot_header_bytes(n_seqs) + table_n * 4 + 16;
        for (int i = 0; i < 4; ++i) q += arrays[i].per_seq * n_seqs;
        c->n_image_host.assign((const int32_t *)q, (const int32_t *)q + n_seqs);
        q += arrays[4].per_seq * n_seqs;   // the cache lengths follow the image lengths
        c->kv_host.assign((const int32_t *)q, (const int32_t *)q + 2 * n_seqs);
    }
    return SJD_OK;
}

}  // extern "C"

#include "sjd_ops.hip.h"
