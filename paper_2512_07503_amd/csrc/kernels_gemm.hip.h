// Projection GEMMs  C[m][n] = sum_k A[m][k] W[n][k]  (QKV, output, gate/up, down and the vocabulary
// head: the dense contractions of the forward, Sec. 4.1 Step 2).
//
// M = 2 * sequences * window is small (32 ... 512) while the weights are large, so below M ~ 300 the
// kernels are bound by streaming W from HBM exactly once.  bf16 operands are stored fragment-major
// (see Layout<bf16_t>): a wavefront reads a 32 x 16 operand fragment with one coalesced 1 KiB load and
// feeds it straight into v_mfma_f32_32x32x16_bf16; W never passes through LDS.  K is split across
// workgroups to fill the 256 CUs; the partial sums [splits][M][N] are reduced, in a fixed order, by the
// element-wise kernel that consumes them.
#pragma once
#include "common.hip.h"

// ------------------------------------------------------------------------------------ reference
// One wavefront per (output column n, block of 8 rows): lanes stride over k, then a shuffle tree.
// Works for both dtypes through the layout functions; fp32 accumulation with fused multiply-adds.
template <typename T>
__global__ void gemm_reference_kernel(const T *__restrict__ A, const T *__restrict__ W, float *__restrict__ C, int M, int N,
                                      int K) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = blockIdx.x * (blockDim.x >> 6) + wave;
    const int m0 = blockIdx.y * 8;
    if (n >= N) return;
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
    for (int k = lane; k < K; k += 64) {
        const float w = to_float<T>(W[Layout<T>::w_index(n, k, K)]);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int m = m0 + j;
            if (m < M) acc[j] = fmaf(to_float<T>(A[Layout<T>::a_index(m, k, K)]), w, acc[j]);
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        float v = acc[j];
        for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
        if (lane == 0 && m0 + j < M) C[(size_t)(m0 + j) * N + n] = v;
    }
}

// ------------------------------------------------------------------------------------ MFMA, bf16
// Workgroup = 4 wavefronts; wavefront w owns NBW column blocks of 32 and MT row tiles of 32 over the
// k-blocks [split * kb_per_split, ...).  grid = (ceil(NB / (4 NBW)), splits, ceil(MTILES / MT)).
template <int MT, int NBW>
__global__ __launch_bounds__(256) void gemm_bf16_mfma_kernel(const bf16_t *__restrict__ A, const bf16_t *__restrict__ W,
                                                             float *__restrict__ C, int M, int N, int KB, int kb_per_split) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int NB = (N + 31) >> 5, MTILES = (M + 31) >> 5;
    const int nb0 = (blockIdx.x * 4 + wave) * NBW;
    if (nb0 >= NB) return;
    const int mt0 = blockIdx.z * MT;
    const int kb_begin = blockIdx.y * kb_per_split;
    const int kb_end = kb_begin + kb_per_split < KB ? kb_begin + kb_per_split : KB;

    const u32x4 *Ap = reinterpret_cast<const u32x4 *>(A);
    const u32x4 *Wp = reinterpret_cast<const u32x4 *>(W);
    // fragment (tile, kb) starts at 16-byte index (tile * KB + kb) * 64; out-of-range tiles are clamped
    // (their results are never stored)
    size_t a_off[MT], w_off[NBW];
#pragma unroll
    for (int j = 0; j < MT; ++j) a_off[j] = (size_t)(mt0 + j < MTILES ? mt0 + j : MTILES - 1) * KB * 64 + lane;
#pragma unroll
    for (int i = 0; i < NBW; ++i) w_off[i] = (size_t)(nb0 + i < NB ? nb0 + i : NB - 1) * KB * 64 + lane;

    f32x16 acc[MT][NBW];
#pragma unroll
    for (int j = 0; j < MT; ++j)
#pragma unroll
        for (int i = 0; i < NBW; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][i][v] = 0.0f;

    for (int kb = kb_begin; kb < kb_end; ++kb) {
        u32x4 b[NBW], a[MT];
#pragma unroll
        for (int i = 0; i < NBW; ++i) b[i] = __builtin_nontemporal_load(Wp + w_off[i] + (size_t)kb * 64);
#pragma unroll
        for (int j = 0; j < MT; ++j) a[j] = Ap[a_off[j] + (size_t)kb * 64];
#pragma unroll
        for (int j = 0; j < MT; ++j)
#pragma unroll
            for (int i = 0; i < NBW; ++i)
                acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[j]),
                                                                    __builtin_bit_cast(bf16x8, b[i]), acc[j][i], 0, 0, 0);
    }

    // accumulator element v of lane l is C[row = 8 (v / 4) + 4 (l / 32) + v % 4][col = l % 32] of the tile
    float *Cs = C + (size_t)blockIdx.y * M * N;
#pragma unroll
    for (int j = 0; j < MT; ++j) {
        if (mt0 + j >= MTILES) continue;
#pragma unroll
        for (int i = 0; i < NBW; ++i) {
            const int col = (nb0 + i) * 32 + (lane & 31);
            if (nb0 + i >= NB || col >= N) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = (mt0 + j) * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (row < M) Cs[(size_t)row * N + col] = acc[j][i][v];
            }
        }
    }
}

struct GemmPlan {
    int mt, nbw, splits, kb_per_split;
    dim3 grid;
};

// Split-K factor and tile shape for an M x N x K bf16 GEMM: aim at >= ~4 wavefronts per SIMD worth of
// independent weight streams while keeping at least 8 k-blocks (128 k) per split.
inline GemmPlan plan_gemm_bf16(int M, int N, int K, int force_splits) {
    GemmPlan p;
    const int NB = (N + 31) / 32, KB = K / 16, MTILES = (M + 31) / 32;
    p.mt = MTILES >= 2 ? 2 : 1;
    p.nbw = NB >= 512 ? 2 : 1;
    const int mz = (MTILES + p.mt - 1) / p.mt;
    const int waves = ((NB + p.nbw - 1) / p.nbw) * mz;
    int splits = force_splits > 0 ? force_splits : (2048 + waves - 1) / waves;
    int max_splits = KB / 8 > 0 ? KB / 8 : 1;
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    p.kb_per_split = (KB + splits - 1) / splits;
    p.splits = (KB + p.kb_per_split - 1) / p.kb_per_split;
    p.grid = dim3((NB + 4 * p.nbw - 1) / (4 * p.nbw), p.splits, mz);
    return p;
}

inline hipError_t launch_gemm_bf16(hipStream_t st, const GemmPlan &p, const bf16_t *A, const bf16_t *W, float *C, int M, int N,
                                   int K) {
    const int KB = K / 16;
    if (p.mt == 1 && p.nbw == 1) gemm_bf16_mfma_kernel<1, 1><<<p.grid, 256, 0, st>>>(A, W, C, M, N, KB, p.kb_per_split);
    else if (p.mt == 1 && p.nbw == 2) gemm_bf16_mfma_kernel<1, 2><<<p.grid, 256, 0, st>>>(A, W, C, M, N, KB, p.kb_per_split);
    else if (p.mt == 2 && p.nbw == 1) gemm_bf16_mfma_kernel<2, 1><<<p.grid, 256, 0, st>>>(A, W, C, M, N, KB, p.kb_per_split);
    else gemm_bf16_mfma_kernel<2, 2><<<p.grid, 256, 0, st>>>(A, W, C, M, N, KB, p.kb_per_split);
    return hipGetLastError();
}

template <typename T>
inline hipError_t launch_gemm_reference(hipStream_t st, const T *A, const T *W, float *C, int M, int N, int K) {
    dim3 grid((N + 3) / 4, (M + 7) / 8);
    gemm_reference_kernel<T><<<grid, 256, 0, st>>>(A, W, C, M, N, K);
    return hipGetLastError();
}
