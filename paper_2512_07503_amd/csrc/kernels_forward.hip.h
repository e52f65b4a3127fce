// Element-wise kernels of the transformer forward: embedding gather, residual add + RMSNorm,
// rotary embedding + KV page write, SwiGLU.  Each also folds in the reduction of the split-K partial
// sums of the GEMM before it, in a fixed order (results are run-to-run deterministic).
//
// The paper only requires a single causal forward of the model over the window (Sec. 4.1, Step 2);
// the block structure is the one the workload shapes name.
#pragma once
#include "common.hip.h"
#include "decide.h"

template <typename T>
__global__ void embed_kernel(const T *__restrict__ emb, const int32_t *__restrict__ row_tok, float *__restrict__ x, int d) {
    const int m = blockIdx.x;
    const int tok = row_tok[m];
    for (int i = threadIdx.x; i < d; i += blockDim.x) x[(size_t)m * d + i] = tok >= 0 ? to_float<T>(emb[(size_t)tok * d + i]) : 0.0f;
}

// deterministic block sum of one float per thread (blockDim.x <= 1024, multiple of 64)
SJD_D float block_sum_f32(float v, float *scratch /* 17 floats shared */) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if (lane == 0) scratch[wave] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.0f;
        for (int i = 0; i < nw; ++i) t += scratch[i];
        scratch[16] = t;
    }
    __syncthreads();
    return scratch[16];
}

// x[m] += sum_s partial[s][m] (if partial != NULL);  xn[m] = x[m] * rsqrt(mean(x[m]^2) + eps) * gain
// xn is written in the GEMM-operand layout of T.
template <typename T>
__global__ void addnorm_kernel(float *__restrict__ x, const float *__restrict__ partial, int splits, int M,
                               const float *__restrict__ gain, T *__restrict__ xn, int d, float eps) {
    const int m = blockIdx.x;
    __shared__ float scratch[17];
    float ss = 0.0f;
    for (int i = threadIdx.x; i < d; i += blockDim.x) {
        float v = x[(size_t)m * d + i];
        if (partial) {
            for (int s = 0; s < splits; ++s) v += partial[((size_t)s * M + m) * d + i];
            x[(size_t)m * d + i] = v;
        }
        ss = fmaf(v, v, ss);
    }
    ss = block_sum_f32(ss, scratch);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += blockDim.x) {
        float v = x[(size_t)m * d + i];
        xn[Layout<T>::a_index(m, i, d)] = from_float<T>(v * inv * gain[i]);
    }
}

struct KvPool {
    void *k, *v;                 // this layer's pools: [n_pages][Hkv][page_tokens * hd]
    const int32_t *page_table;   // [segments][pages_per_seg]
    int pages_per_seg, page_tokens;
};

// qkv partial sums [splits][M][(H + 2 Hkv) * hd] -> rotated q (attention operand layout, per segment
// and head), rotated k and v into the KV pages at the row's position.
template <typename T>
__global__ void rope_kv_kernel(const float *__restrict__ partial, int splits, int M, const int32_t *__restrict__ row_tok,
                               const int32_t *__restrict__ row_pos, const float *__restrict__ rope_cos,
                               const float *__restrict__ rope_sin, T *__restrict__ q_out, KvPool pool, int L, int H,
                               int Hkv, int hd) {
    const int m = blockIdx.x;
    if (row_tok[m] < 0) return;
    const int seg = m / L, i_win = m % L, pos = row_pos[m];
    const int half = hd >> 1, N = (H + 2 * Hkv) * hd;
    const size_t qseg = Layout<T>::q_elems(L, hd);
    const int page = pool.page_table[seg * pool.pages_per_seg + pos / pool.page_tokens];
    const int t = pos % pool.page_tokens;
    const size_t blk = (size_t)pool.page_tokens * hd;
    auto val = [&](int col) {
        float v = 0.0f;
        for (int s = 0; s < splits; ++s) v += partial[((size_t)s * M + m) * N + col];
        return v;
    };
    // q and k: one thread per rotated pair
    for (int idx = threadIdx.x; idx < (H + Hkv) * half; idx += blockDim.x) {
        const int h = idx / half, i = idx % half;
        const float a = val(h * hd + i), b = val(h * hd + i + half);
        const float c = rope_cos[(size_t)pos * half + i], s = rope_sin[(size_t)pos * half + i];
        const float r0 = a * c - b * s, r1 = b * c + a * s;
        if (h < H) {
            T *dst = q_out + ((size_t)seg * H + h) * qseg;
            dst[Layout<T>::q_index(i_win, i, hd)] = from_float<T>(r0);
            dst[Layout<T>::q_index(i_win, i + half, hd)] = from_float<T>(r1);
        } else {
            T *dst = (T *)pool.k + ((size_t)page * Hkv + (h - H)) * blk;
            dst[Layout<T>::k_index(t, i, hd)] = from_float<T>(r0);
            dst[Layout<T>::k_index(t, i + half, hd)] = from_float<T>(r1);
        }
    }
    for (int idx = threadIdx.x; idx < Hkv * hd; idx += blockDim.x) {
        const int h = idx / hd, j = idx % hd;
        T *dst = (T *)pool.v + ((size_t)page * Hkv + h) * blk;
        dst[Layout<T>::v_index(t, j, hd)] = from_float<T>(val((H + Hkv) * hd + idx));
    }
}

// gate/up partial sums [splits][M][2F] -> silu(gate) * up in the GEMM-operand layout
template <typename T>
__global__ void swiglu_kernel(const float *__restrict__ partial, int splits, int M, T *__restrict__ h, int F) {
    const int m = blockIdx.x;
    for (int j = threadIdx.x; j < F; j += blockDim.x) {
        float g = 0.0f, u = 0.0f;
        for (int s = 0; s < splits; ++s) {
            g += partial[((size_t)s * M + m) * 2 * F + j];
            u += partial[((size_t)s * M + m) * 2 * F + F + j];
        }
        h[Layout<T>::a_index(m, j, F)] = from_float<T>(g / (1.0f + expf(-g)) * u);
    }
}

// ------------------------------------------------------------------------------- weight re-layout
// dst (GEMM-operand layout of T, rows [row0, row0 + N) of a matrix with K columns) <- src [N][K] row-major
template <typename T>
__global__ void pack_weight_kernel(const T *__restrict__ src, T *__restrict__ dst, int N, int K, int row0) {
    const size_t total = (size_t)N * K;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int n = (int)(idx / K), k = (int)(idx % K);
        dst[Layout<T>::w_index(row0 + n, k, K)] = src[idx];
    }
}

template <typename T>
__global__ void to_float_kernel(const T *__restrict__ src, float *__restrict__ dst, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = to_float<T>(src[i]);
}

// plain row-major [M][K] -> GEMM-operand layout (used by the single-operation entry points)
template <typename T>
__global__ void pack_act_kernel(const T *__restrict__ src, T *__restrict__ dst, int M, int K) {
    const size_t total = (size_t)M * K;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int m = (int)(idx / K), k = (int)(idx % K);
        dst[Layout<T>::a_index(m, k, K)] = src[idx];
    }
}

// C[m][n] = sum_s partial[s][m][n]
__global__ void reduce_partials_kernel(const float *__restrict__ partial, int splits, size_t MN, float *__restrict__ C) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= MN) return;
    float v = 0.0f;
    for (int s = 0; s < splits; ++s) v += partial[(size_t)s * MN + i];
    C[i] = v;
}
