// Single-operation entry points of include/sjd.h (kernel-level tests and microbenchmarks).
// Included at the end of sjd_api.hip.
#pragma once

namespace {

struct Scratch {
    std::vector<void *> ptrs;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    ~Scratch() {
        for (void *p : ptrs) (void)hipFree(p);
        if (ev0) (void)hipEventDestroy(ev0);
        if (ev1) (void)hipEventDestroy(ev1);
    }
    template <typename P> bool alloc(P **out, size_t bytes, hipStream_t st) {
        void *p = nullptr;
        if (hipMalloc(&p, bytes ? bytes : 16) != hipSuccess) return false;
        ptrs.push_back(p);
        if (hipMemsetAsync(p, 0, bytes ? bytes : 16, st) != hipSuccess) return false;
        *out = reinterpret_cast<P *>(p);
        return true;
    }
    bool events() { return hipEventCreate(&ev0) == hipSuccess && hipEventCreate(&ev1) == hipSuccess; }
};

#define OP_TRY(expr)                                                                                  \
    do {                                                                                              \
        hipError_t e__ = (expr);                                                                      \
        if (e__ != hipSuccess) {                                                                      \
            sjd_set_error(g_create_error, "%s failed: %s", #expr, hipGetErrorString(e__));            \
            return SJD_EDEVICE;                                                                       \
        }                                                                                             \
    } while (0)

// Bytes of the three temporaries of a GEMM call, each rounded up to 256: the two operands in the kernels' layout and the
// split-K partial sums [splits][M][N] that the GEMM kernel writes and reduce_partials_kernel adds up.
struct GemmTemps { size_t a_bytes, w_bytes, part_bytes; int n_splits; GemmPlan plan; bool ref; };
template <typename T> GemmTemps gemm_temps(int flags, int M, int N, int K, int splits) {
    GemmTemps t;
    t.ref = std::is_same<T, float>::value || (flags & SJD_KERNELS_REFERENCE);
    t.plan = GemmPlan{};
    if (!t.ref) t.plan = plan_gemm_bf16(M, N, K, splits);   // bf16: K is a positive multiple of 16 (checked by the entry points)
    t.n_splits = t.ref ? 1 : t.plan.splits;
    auto up = [](size_t b) { return (b + 255) / 256 * 256; };
    t.a_bytes = up(Layout<T>::a_elems(M, K) * sizeof(T));
    t.w_bytes = up(Layout<T>::w_elems(N, K) * sizeof(T));
    t.part_bytes = up((size_t)t.n_splits * M * N * sizeof(float));
    return t;
}

// The launches of a GEMM call on temporaries the caller provides; ev0 / ev1 (may be null) bracket the GEMM launches.
template <typename T>
int gemm_on_temps(hipStream_t st, const GemmTemps &t, const void *A, const void *W, float *C, T *Ap, T *Wp, float *partial, int M,
                  int N, int K, int repeat, hipEvent_t ev0, hipEvent_t ev1) {
    pack_act_kernel<T><<<512, 256, 0, st>>>((const T *)A, Ap, M, K);
    OP_TRY(hipGetLastError());
    pack_weight_kernel<T><<<1024, 256, 0, st>>>((const T *)W, Wp, N, K, 0);
    OP_TRY(hipGetLastError());
    if (ev0) OP_TRY(hipEventRecord(ev0, st));
    for (int r = 0; r < repeat; ++r) {
        if (t.ref) OP_TRY(launch_gemm_reference<T>(st, Ap, Wp, partial, M, N, K));
        else OP_TRY(launch_gemm_bf16(st, t.plan, (const bf16_t *)Ap, (const bf16_t *)Wp, partial, M, N, K));
    }
    if (ev1) OP_TRY(hipEventRecord(ev1, st));
    reduce_partials_kernel<<<(unsigned)ceil_div_sz((size_t)M * N, 256), 256, 0, st>>>(partial, t.n_splits, (size_t)M * N, C);
    OP_TRY(hipGetLastError());
    OP_TRY(hipStreamSynchronize(st));
    return SJD_OK;
}

template <typename T>
int op_gemm(hipStream_t st, int flags, const void *A, const void *W, float *C, int M, int N, int K, int splits, int repeat,
            float *avg_ms) {
    Scratch s;
    T *Ap, *Wp;
    float *partial;
    const GemmTemps t = gemm_temps<T>(flags, M, N, K, splits);
    if (!s.alloc(&Ap, t.a_bytes, st) || !s.alloc(&Wp, t.w_bytes, st) || !s.alloc(&partial, t.part_bytes, st) || !s.events()) {
        sjd_set_error(g_create_error, "allocation failed");
        return SJD_ENOMEM;
    }
    const int rc = gemm_on_temps<T>(st, t, A, W, C, Ap, Wp, partial, M, N, K, repeat, s.ev0, s.ev1);
    if (rc) return rc;
    if (avg_ms) {
        float ms = 0.0f;
        OP_TRY(hipEventElapsedTime(&ms, s.ev0, s.ev1));
        *avg_ms = ms / repeat;
    }
    return SJD_OK;
}

// ---- the same call without any allocation: its temporaries live in a file-scope device array.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
// In host code the name `scratch` is only a handle of the symbol; the array's address on a device comes from
// hipGetSymbolAddress, once per device (every device holds its own copy at its own address).
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {nullptr};
std::mutex g_scratch_mutex;

int static_scratch(unsigned char **out) {
    int dev = -1;
    OP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) { sjd_set_error(g_create_error, "device index %d out of range", dev); return SJD_EDEVICE; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        OP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) { sjd_set_error(g_create_error, "hipGetSymbolAddress returned a null address"); return SJD_EDEVICE; }
        g_scratch_ptr[dev] = p;
    }
    *out = (unsigned char *)g_scratch_ptr[dev];
    return SJD_OK;
}

__global__ void zero_fill_kernel(u32x4 *p, size_t n16) {
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) p[i] = z;
}

template <typename T>
int op_gemm_static(hipStream_t st, int flags, const void *A, const void *W, float *C, int M, int N, int K, int splits) {
    const GemmTemps t = gemm_temps<T>(flags, M, N, K, splits);
    const size_t need = t.a_bytes + t.w_bytes + t.part_bytes;
    if (need > kStaticScratchBytes) {
        sjd_set_error(g_create_error, "sjd_op_gemm_static: %d x %d x %d needs %zu bytes of temporaries, the static workspace holds %zu",
                      M, N, K, need, kStaticScratchBytes);
        return SJD_ECAPACITY;
    }
    unsigned char *base = nullptr;
    const int rc = static_scratch(&base);
    if (rc) return rc;
    // The workspace keeps the last call's contents.  The operand copies are padded to whole 32-row fragments and the pack
    // kernels write the real rows only: clear both (a fill kernel, not a memset node, so that the call can be captured).
    zero_fill_kernel<<<256, 256, 0, st>>>((u32x4 *)base, (t.a_bytes + t.w_bytes) / 16);
    OP_TRY(hipGetLastError());
    return gemm_on_temps<T>(st, t, A, W, C, (T *)base, (T *)(base + t.a_bytes), (float *)(base + t.a_bytes + t.w_bytes), M, N, K, 1,
                            nullptr, nullptr);
}

template <typename T>
int op_attention(hipStream_t st, int flags, const void *q, const void *k, const void *v, float *out, int n, int ctx, int H,
                 int Hkv, int hd, int pt, int repeat, float *avg_ms) {
    Scratch s;
    const int n_tok = ctx + n, pages = ceil_div(n_tok, pt);
    KvPool pool;
    T *qp;
    int32_t *table, *row_tok, *seg_kv;
    const size_t pool_bytes = (size_t)pages * Hkv * pt * hd * sizeof(T);
    if (!s.alloc(&pool.k, pool_bytes, st) || !s.alloc(&pool.v, pool_bytes, st) || !s.alloc(&table, (size_t)pages * 4, st) ||
        !s.alloc(&row_tok, (size_t)n * 4, st) || !s.alloc(&seg_kv, 4, st) ||
        !s.alloc(&qp, (size_t)H * Layout<T>::q_elems(n, hd) * sizeof(T), st) || !s.events()) {
        sjd_set_error(g_create_error, "allocation failed");
        return SJD_ENOMEM;
    }
    std::vector<int32_t> tab(pages);
    for (int i = 0; i < pages; ++i) tab[i] = pages - 1 - i;  // pages deliberately out of order
    OP_TRY(hipMemcpyAsync(table, tab.data(), (size_t)pages * 4, hipMemcpyHostToDevice, st));
    OP_TRY(hipMemcpyAsync(seg_kv, &ctx, 4, hipMemcpyHostToDevice, st));
    OP_TRY(hipStreamSynchronize(st));
    pool.page_table = table;
    pool.pages_per_seg = pages;
    pool.page_tokens = pt;
    pack_kv_kernel<T><<<512, 256, 0, st>>>((const T *)k, (const T *)v, pool, n_tok, Hkv, hd);
    OP_TRY(hipGetLastError());
    pack_q_kernel<T><<<64, 256, 0, st>>>((const T *)q, qp, n, H, hd, n);
    OP_TRY(hipGetLastError());
    const bool mfma = std::is_same<T, bf16_t>::value && !(flags & SJD_KERNELS_REFERENCE) && attention_mfma_supported(n, H, Hkv, hd, pt);
    AttnArgs a;
    memset(&a, 0, sizeof a);
    if (mfma) {
        int32_t *seg_n;
        a.chunk = 128;
        a.n_chunks = ceil_div(n_tok, a.chunk);
        a.n_qt = ceil_div(n, 32);
        if (!s.alloc(&a.part_o, (size_t)H * a.n_qt * a.n_chunks * 32 * hd * sizeof(float), st) ||
            !s.alloc(&a.part_ml, (size_t)H * a.n_qt * a.n_chunks * 64 * sizeof(float), st) || !s.alloc(&seg_n, 4, st)) {
            sjd_set_error(g_create_error, "allocation failed");
            return SJD_ENOMEM;
        }
        OP_TRY(hipMemcpyAsync(seg_n, &n, 4, hipMemcpyHostToDevice, st));
        OP_TRY(hipStreamSynchronize(st));
        a.q = (const bf16_t *)qp; a.pool = pool; a.row_tok = row_tok; a.seg_kv = seg_kv; a.seg_n = seg_n;
        a.out_act = nullptr; a.out_plain = out;
        a.L = n; a.H = H; a.Hkv = Hkv; a.hd = hd;
        a.scale_log2e = (float)(1.4426950408889634 / sqrt((double)hd));
    }
    OP_TRY(hipEventRecord(s.ev0, st));
    for (int r = 0; r < repeat; ++r) {
        if (mfma) OP_TRY(launch_attention_mfma(st, a, 1, !(flags & SJD_ATTENTION_CHUNKED) && attention_onepass_pays(n_tok, hd)));
        else OP_TRY(launch_attention_reference<T>(st, qp, pool, row_tok, seg_kv, (T *)nullptr, out, n, n, H, Hkv, hd, n_tok + 1));
    }
    OP_TRY(hipEventRecord(s.ev1, st));
    OP_TRY(hipStreamSynchronize(st));
    if (avg_ms) {
        float ms = 0.0f;
        OP_TRY(hipEventElapsedTime(&ms, s.ev0, s.ev1));
        *avg_ms = ms / repeat;
    }
    return SJD_OK;
}

}  // namespace

extern "C" {

int sjd_op_gemm(void *hip_stream, int32_t dtype, int32_t flags, const void *A, const void *W, float *C, int32_t M, int32_t N,
                int32_t K, int32_t splits, int32_t repeat, float *avg_ms) {
    if (!A || !W || !C || M < 1 || N < 1 || K < 1 || repeat < 1) { sjd_set_error(g_create_error, "bad argument"); return SJD_EINVAL; }
    if (dtype == SJD_F32) return op_gemm<float>((hipStream_t)hip_stream, flags, A, W, C, M, N, K, splits, repeat, avg_ms);
    if (dtype == SJD_BF16) {
        if (K % 16) { sjd_set_error(g_create_error, "bf16 GEMM needs K %% 16 == 0"); return SJD_EINVAL; }
        return op_gemm<bf16_t>((hipStream_t)hip_stream, flags, A, W, C, M, N, K, splits, repeat, avg_ms);
    }
    sjd_set_error(g_create_error, "unknown dtype");
    return SJD_EINVAL;
}

int sjd_op_gemm_static(void *hip_stream, int32_t dtype, int32_t flags, const void *A, const void *W, float *C, int32_t M,
                       int32_t N, int32_t K, int32_t splits) {
    if (!A || !W || !C || M < 1 || N < 1 || K < 1) { sjd_set_error(g_create_error, "bad argument"); return SJD_EINVAL; }
    if (dtype == SJD_F32) return op_gemm_static<float>((hipStream_t)hip_stream, flags, A, W, C, M, N, K, splits);
    if (dtype == SJD_BF16) {
        if (K % 16) { sjd_set_error(g_create_error, "bf16 GEMM needs K %% 16 == 0"); return SJD_EINVAL; }
        return op_gemm_static<bf16_t>((hipStream_t)hip_stream, flags, A, W, C, M, N, K, splits);
    }
    sjd_set_error(g_create_error, "unknown dtype");
    return SJD_EINVAL;
}

int sjd_op_window_attention(void *hip_stream, int32_t dtype, int32_t flags, const void *q, const void *k, const void *v,
                            float *out, int32_t n, int32_t ctx, int32_t n_heads, int32_t n_kv_heads, int32_t head_dim,
                            int32_t page_tokens, int32_t repeat, float *avg_ms) {
    if (!q || !k || !v || !out || n < 1 || ctx < 0 || n_heads < 1 || n_kv_heads < 1 || n_heads % n_kv_heads || head_dim < 2 ||
        head_dim % 2 || page_tokens < 32 || page_tokens % 32 || repeat < 1) {
        sjd_set_error(g_create_error, "bad argument");
        return SJD_EINVAL;
    }
    if (dtype == SJD_F32)
        return op_attention<float>((hipStream_t)hip_stream, flags, q, k, v, out, n, ctx, n_heads, n_kv_heads, head_dim, page_tokens,
                                   repeat, avg_ms);
    if (dtype == SJD_BF16) {
        if (head_dim % 32) { sjd_set_error(g_create_error, "bf16 attention needs head_dim %% 32 == 0"); return SJD_EINVAL; }
        return op_attention<bf16_t>((hipStream_t)hip_stream, flags, q, k, v, out, n, ctx, n_heads, n_kv_heads, head_dim,
                                    page_tokens, repeat, avg_ms);
    }
    sjd_set_error(g_create_error, "unknown dtype");
    return SJD_EINVAL;
}

int sjd_op_sampling_rows(void *hip_stream, const float *logits_c, const float *logits_u, float *e, uint64_t *Z, int32_t rows,
                         int32_t V, float cfg_scale, float temperature, int32_t top_k, const int32_t *allow_lo,
                         const int32_t *allow_hi, int32_t *kept_ids, int32_t *kept_cnt, int32_t repeat, float *avg_ms) {
    if (!logits_c || !logits_u || !e || !Z || rows < 1 || V < 1 || top_k < 1 || !(temperature > 0.0f) || repeat < 1 ||
        (allow_lo == nullptr) != (allow_hi == nullptr)) {
        sjd_set_error(g_create_error, "bad argument");
        return SJD_EINVAL;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    Scratch s;
    int32_t *ids, *cnt;
    float *ev;
    if (!s.events() || !s.alloc(&ids, (size_t)rows * V * 4, st) || !s.alloc(&ev, (size_t)rows * V * 4, st) ||
        !s.alloc(&cnt, (size_t)rows * 4, st)) {
        sjd_set_error(g_create_error, "allocation failed");
        return SJD_ENOMEM;
    }
    if (allow_lo) {   // the ranges are the caller's: check them before a kernel indexes with them
        std::vector<int32_t> lo(rows), hi(rows);
        OP_TRY(hipMemcpy(lo.data(), allow_lo, (size_t)rows * 4, hipMemcpyDeviceToHost));
        OP_TRY(hipMemcpy(hi.data(), allow_hi, (size_t)rows * 4, hipMemcpyDeviceToHost));
        for (int r = 0; r < rows; ++r)
            if (lo[r] < 0 || hi[r] > V || lo[r] >= hi[r]) { sjd_set_error(g_create_error, "row %d: bad id range", r); return SJD_EINVAL; }
    }
    SamplingParams sp;
    sp.cfg_scale = cfg_scale;
    sp.inv_temperature = 1.0f / temperature;
    sp.tau = 0.0f;
    sp.top_k = top_k;
    sp.seed = 0;
    OP_TRY(hipEventRecord(s.ev0, st));
    for (int r = 0; r < repeat; ++r) OP_TRY(launch_sampling_rows_plain(st, logits_c, logits_u, ids, ev, cnt, Z, rows, V, sp, allow_lo, allow_hi));
    OP_TRY(hipEventRecord(s.ev1, st));
    // the dense form of the rows: zeros, then the kept pairs
    OP_TRY(hipMemsetAsync(e, 0, (size_t)rows * V * sizeof(float), st));
    OP_TRY(launch_scatter_rows(st, ids, ev, cnt, e, rows, V));
    if (kept_ids) OP_TRY(hipMemcpyAsync(kept_ids, ids, (size_t)rows * V * 4, hipMemcpyDeviceToDevice, st));
    if (kept_cnt) OP_TRY(hipMemcpyAsync(kept_cnt, cnt, (size_t)rows * 4, hipMemcpyDeviceToDevice, st));
    OP_TRY(hipStreamSynchronize(st));
    if (avg_ms) {
        float ms = 0.0f;
        OP_TRY(hipEventElapsedTime(&ms, s.ev0, s.ev1));
        *avg_ms = ms / repeat;
    }
    return SJD_OK;
}

int sjd_op_philox(void *hip_stream, uint64_t seed, uint32_t row, uint32_t seq, uint32_t *out, int32_t n) {
    if (!out || n < 1) { sjd_set_error(g_create_error, "bad argument"); return SJD_EINVAL; }
    OP_TRY(launch_philox_fill((hipStream_t)hip_stream, seed, row, seq, out, n));
    OP_TRY(hipStreamSynchronize((hipStream_t)hip_stream));
    return SJD_OK;
}

}  // extern "C"
