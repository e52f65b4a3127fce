// Window attention: the L queries of a (sequence, branch) attend to the committed cache positions
// [0, kv) and, causally, to the window positions kv .. kv + i (Sec. 4.1 Step 2: "a causal mask in the
// attention mechanism").  Keys and values live in pages addressed through a page table.
#pragma once
#include "common.hip.h"
#include "kernels_forward.hip.h"

// ------------------------------------------------------------------------------------ reference
// One wavefront per (row, head): scores into LDS, softmax, then lanes split the head dimension.
// out_act (GEMM-operand layout [M][H*hd] of T) and / or out_plain ([M][H][hd] fp32) receive the result.
template <typename T>
__global__ void attention_reference_kernel(const T *__restrict__ q, KvPool pool, const int32_t *__restrict__ row_tok,
                                           const int32_t *__restrict__ seg_kv, T *__restrict__ out_act,
                                           float *__restrict__ out_plain, int L, int H, int Hkv, int hd, float scale) {
    extern __shared__ float smem[];
    float *qs = smem, *sc = smem + hd;
    const int m = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    const int seg = m / L, i_win = m % L;
    if (row_tok[m] < 0) {
        for (int j = lane; j < hd; j += 64) {
            if (out_act) out_act[Layout<T>::a_index(m, h * hd + j, H * hd)] = from_float<T>(0.0f);
            if (out_plain) out_plain[((size_t)m * H + h) * hd + j] = 0.0f;
        }
        return;
    }
    const int kvh = h / (H / Hkv);
    const int n_vis = seg_kv[seg] + i_win + 1;
    const T *qsrc = q + ((size_t)seg * H + h) * Layout<T>::q_elems(L, hd);
    for (int j = lane; j < hd; j += 64) qs[j] = to_float<T>(qsrc[Layout<T>::q_index(i_win, j, hd)]);
    __syncthreads();
    const size_t blk = (size_t)pool.page_tokens * hd;
    const int32_t *pt = pool.page_table + (size_t)seg * pool.pages_per_seg;
    float mx = -INFINITY;
    for (int t = lane; t < n_vis; t += 64) {
        const T *kb = (const T *)pool.k + ((size_t)pt[t / pool.page_tokens] * Hkv + kvh) * blk;
        const int tt = t % pool.page_tokens;
        float s = 0.0f;
        for (int j = 0; j < hd; ++j) s = fmaf(qs[j], to_float<T>(kb[Layout<T>::k_index(tt, j, hd)]), s);
        s *= scale;
        sc[t] = s;
        mx = fmaxf(mx, s);
    }
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    float sum = 0.0f;
    for (int t = lane; t < n_vis; t += 64) {
        const float p = expf(sc[t] - mx);
        sc[t] = p;
        sum += p;
    }
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    __syncthreads();
    const float inv = 1.0f / sum;
    for (int j = lane; j < hd; j += 64) {
        float acc = 0.0f;
        for (int t = 0; t < n_vis; ++t) {
            const T *vb = (const T *)pool.v + ((size_t)pt[t / pool.page_tokens] * Hkv + kvh) * blk;
            acc = fmaf(sc[t], to_float<T>(vb[Layout<T>::v_index(t % pool.page_tokens, j, hd)]), acc);
        }
        acc *= inv;
        if (out_act) out_act[Layout<T>::a_index(m, h * hd + j, H * hd)] = from_float<T>(acc);
        if (out_plain) out_plain[((size_t)m * H + h) * hd + j] = acc;
    }
}

template <typename T>
inline hipError_t launch_attention_reference(hipStream_t st, const T *q, const KvPool &pool, const int32_t *row_tok,
                                             const int32_t *seg_kv, T *out_act, float *out_plain, int M, int L, int H, int Hkv,
                                             int hd, int max_visible) {
    const size_t smem = sizeof(float) * (size_t)(hd + max_visible);
    attention_reference_kernel<T><<<dim3(M, H), 64, smem, st>>>(q, pool, row_tok, seg_kv, out_act, out_plain, L, H, Hkv, hd,
                                                                1.0f / sqrtf((float)hd));
    return hipGetLastError();
}

// plain [n_tok][Hkv][hd] keys / values of ONE segment -> pages (identity page table), single-operation tests
template <typename T>
__global__ void pack_kv_kernel(const T *__restrict__ ksrc, const T *__restrict__ vsrc, KvPool pool, int n_tok, int Hkv, int hd) {
    const size_t total = (size_t)n_tok * Hkv * hd;
    const size_t blk = (size_t)pool.page_tokens * hd;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int j = (int)(idx % hd), h = (int)((idx / hd) % Hkv), t = (int)(idx / ((size_t)hd * Hkv));
        const int page = pool.page_table[t / pool.page_tokens], tt = t % pool.page_tokens;
        ((T *)pool.k)[((size_t)page * Hkv + h) * blk + Layout<T>::k_index(tt, j, hd)] = ksrc[idx];
        ((T *)pool.v)[((size_t)page * Hkv + h) * blk + Layout<T>::v_index(tt, j, hd)] = vsrc[idx];
    }
}

// plain [n][H][hd] queries of one segment -> attention operand layout
template <typename T>
__global__ void pack_q_kernel(const T *__restrict__ src, T *__restrict__ dst, int n, int H, int hd, int L) {
    const size_t total = (size_t)n * H * hd;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int j = (int)(idx % hd), h = (int)((idx / hd) % H), i = (int)(idx / ((size_t)hd * H));
        dst[(size_t)h * Layout<T>::q_elems(L, hd) + Layout<T>::q_index(i, j, hd)] = src[idx];
    }
}
