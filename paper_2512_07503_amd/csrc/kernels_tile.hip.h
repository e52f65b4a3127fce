// Projection GEMMs for many rows (M >= 256, several sequences per call): here the forward of Sec. 4.1 Step 2
// stops being bound by streaming weights and becomes a dense contraction, so operands are staged through LDS
// and shared by the wavefronts of a workgroup instead of every wavefront pulling its own copy through L1.
//
// Workgroup = 4 wavefronts computing a 256-row x 128-column tile over a K range; wavefront w owns rows
// [64 w, 64 w + 64) of it across all 128 columns (2 x 4 MFMA tiles of 32 x 32, 128 accumulator registers).
//   activations  each wavefront's rows are its own, so their fragments go from global memory straight into MFMA
//                operand registers (fragment-major: one coalesced 16-byte load per lane), never through LDS
//   weights      the 4 column blocks are shared by all wavefronts: each fetches one block's fragment and drops it
//                into LDS, every wavefront reads all four back
// A pipeline stage is TILE_KS k-steps of 16 (per k-step 8 MFMAs per wavefront against 4 LDS fragment reads) and
// ends in one workgroup barrier; two LDS buffers, TILE_RING stages of global loads in flight in registers.  LDS
// moves 20 KiB per k-step (the all-through-LDS 2 x 2 arrangement moved 36 KiB and measured LDS-bound), and L1 sees
// each operand byte once per workgroup: 12 KiB per k-step, a quarter of the small-row kernel's.  Weights are
// loaded cacheable: the row tiles of a column tile run side by side and the second one finds them in L2.
//
// Epilogues and operand layouts are those of the small-row kernel (skinny_epilogue): column blocks (0, 1) and
// (2, 3) of a tile are rotary / gate-up pairs.  RMSNorm row sums of squares come from the activation fragments as
// they are consumed.
#pragma once
#include "kernels_skinny.hip.h"

constexpr int TILE_M = 256, TILE_N = 128;
constexpr int TILE_KS = 1;    // k-steps (of 16) per pipeline stage, i.e. per workgroup barrier
constexpr int TILE_RING = 4;  // stages of global loads in flight per wavefront (KS x RING = 4 k-steps measured best)

template <int EPI, int KS = TILE_KS, int D = TILE_RING, int MINW = 2>
__global__ __launch_bounds__(256, MINW) void gemm_tile_kernel(SkinnyArgs a, int n_blocks, int row_tiles32, int col_tiles, int row_tiles) {
    constexpr bool kNorm = EPI != EPI_RESID && EPI != EPI_PARTIAL;
    constexpr int U = D % 2 == 0 ? D : 2 * D;  // unroll: ring slot and LDS buffer of an iteration are compile-time
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // blockIdx.x -> (column tile ct, row tile rt).  Workgroups go to the 8 XCDs round-robin by linear id: keep the
    // row tiles of one column tile on one XCD (they share the weights in its L2) when the count allows it.
    int ct, rt;
    {
        const int id = blockIdx.x, span = 8 * row_tiles;
        if (col_tiles % 8 == 0) {
            ct = (id / span) * 8 + (id & 7);
            rt = (id % span) >> 3;
        } else {
            ct = id / row_tiles;
            rt = id % row_tiles;
        }
    }
    const int KB = a.KB, ks = blockIdx.y;
    const int kb_lo = ks * a.kb_per_split;
    const int kb_hi = kb_lo + a.kb_per_split < KB ? kb_lo + a.kb_per_split : KB;
    const int n_k = kb_hi - kb_lo;             // k-steps of this workgroup
    const int n_it = (n_k + KS - 1) / KS;      // pipeline stages

    // this wavefront's operands: activation row tiles (of 32) 8 rt + 2 wave + {0, 1}, straight into registers;
    // weight block 4 ct + wave, its share of the stage in LDS.  Indices past the end are clamped (their
    // products land in rows / columns the epilogue never stores).
    const int ra0 = min(rt * 8 + 2 * wave, row_tiles32 - 1), ra1 = min(rt * 8 + 2 * wave + 1, row_tiles32 - 1);
    const int rb = min(ct * 4 + wave, n_blocks - 1);
    const u32x4 *A0 = reinterpret_cast<const u32x4 *>(a.A) + (size_t)ra0 * KB * 64 + lane;
    const u32x4 *A1 = reinterpret_cast<const u32x4 *>(a.A) + (size_t)ra1 * KB * 64 + lane;
    const u32x4 *B0 = reinterpret_cast<const u32x4 *>(a.W) + (size_t)rb * KB * 64 + lane;

    // k-loop: stage[buffer][k-step of the stage][weight block][lane]; epilogue: 8 KiB per wavefront to index its
    // accumulators by a run-time register number
    __shared__ u32x4 smem[2048];
    static_assert(2 * KS * 4 * 64 <= 2048, "stage buffers exceed the LDS array");
    u32x4 (*stage)[KS][4][64] = reinterpret_cast<u32x4 (*)[KS][4][64]>(smem);
    __shared__ float ssq_lds[4][2][32];

    f32x16 acc[2][4];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][i][v] = 0.0f;
    float ssq[2] = {0.0f, 0.0f};

    if (n_it > 0) {
        u32x4 ra[D][KS][2], rbw[D][KS];
        const u32x4 zero4 = {0u, 0u, 0u, 0u};
        // k-steps past the end re-read the last fragments (cache hits); their activations are zeroed when consumed
#define TILE_KB(step, q) ((size_t)(kb_lo + min((step) * KS + (q), n_k - 1)) * 64)
#define TILE_LOAD_A(slot, step)                                                             \
    do {                                                                                    \
        _Pragma("unroll") for (int q_ = 0; q_ < KS; ++q_) {                                 \
            ra[slot][q_][0] = A0[TILE_KB(step, q_)];                                        \
            ra[slot][q_][1] = A1[TILE_KB(step, q_)];                                        \
        }                                                                                   \
    } while (0)
#define TILE_LOAD_B(slot, step)                                                             \
    do {                                                                                    \
        _Pragma("unroll") for (int q_ = 0; q_ < KS; ++q_) rbw[slot][q_] = B0[TILE_KB(step, q_)]; \
    } while (0)
#define TILE_STORE_B(buf, slot, step)                                                       \
    do {                                                                                    \
        _Pragma("unroll") for (int q_ = 0; q_ < KS; ++q_) stage[buf][q_][wave][lane] = rbw[slot][q_]; \
    } while (0)

#pragma unroll
        for (int s = 0; s < D; ++s) {
            TILE_LOAD_A(s, s);
            TILE_LOAD_B(s, s);
        }
        __builtin_amdgcn_sched_barrier(0);
        TILE_STORE_B(0, 0, 0);
        TILE_LOAD_B(0, D);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        for (int it0 = 0; it0 < n_it; it0 += U) {
#pragma unroll
            for (int su = 0; su < U; ++su) {
                const int it = it0 + su;
                const int slot = su % D, nslot = (su + 1) % D, cur = su & 1;
                bf16x8 bfr[KS][4];
#pragma unroll
                for (int q = 0; q < KS; ++q)
#pragma unroll
                    for (int i = 0; i < 4; ++i) bfr[q][i] = __builtin_bit_cast(bf16x8, stage[cur][q][i][lane]);
#pragma unroll
                for (int q = 0; q < KS; ++q) {
                    const bool valid = it * KS + q < n_k;
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const u32x4 araw = valid ? ra[slot][q][j] : zero4;
                        const bf16x8 av = __builtin_bit_cast(bf16x8, araw);
                        if (kNorm) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const uint32_t pr = araw[e];
                                const float lo = __builtin_bit_cast(float, pr << 16), hi = __builtin_bit_cast(float, pr & 0xFFFF0000u);
                                ssq[j] = fmaf(lo, lo, ssq[j]);
                                ssq[j] = fmaf(hi, hi, ssq[j]);
                            }
                        }
#pragma unroll
                        for (int i = 0; i < 4; ++i) acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bfr[q][i], acc[j][i], 0, 0, 0);
                    }
                }
                TILE_LOAD_A(slot, it + D);
                // the next stage's weights into the other buffer (nobody reads it before the barrier below)
                TILE_STORE_B(cur ^ 1, nslot, it + 1);
                TILE_LOAD_B(nslot, it + 1 + D);
                __builtin_amdgcn_sched_barrier(0);
                __syncthreads();
            }
        }
#undef TILE_KB
#undef TILE_LOAD_A
#undef TILE_LOAD_B
#undef TILE_STORE_B
    }

    if (kNorm) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const float t = ssq[j] + __shfl_xor(ssq[j], 32, 64);
            if (lane < 32) ssq_lds[wave][j][lane] = t;
        }
        __syncthreads();
    }
    // The epilogue body is long; unrolled 64 times it would exceed what the compiler unrolls, and a rolled loop
    // cannot index accumulator registers.  Each lane parks one row tile x column pair (32 values) in LDS (its own
    // slots, so no barrier) and walks them in a rolled loop.
    const int col = lane & 31;
    float *park = reinterpret_cast<float *>(smem) + wave * 2048 + lane;
    // QKV: the row-dependent part of the destination (integer divisions, page lookup) once per row, not per element
    __shared__ QkvRow qrow[EPI == EPI_QKV ? TILE_M : 1];
    if (EPI == EPI_QKV) {
        const int m = rt * TILE_M + tid;
        if (m < a.M) qrow[EPI == EPI_QKV ? tid : 0] = qkv_row(a, m);
        __syncthreads();
    }
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int g = ct * 2 + p;
            if (g * 2 >= n_blocks) continue;  // past the last column pair
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) park[(i * 16 + v) * 64] = acc[j][p * 2 + i][v];
#pragma unroll 1
            for (int v = 0; v < 16; ++v) {
                const int row = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                const int m = rt * TILE_M + (wave * 2 + j) * 32 + row;
                if (m >= a.M) continue;
                float inv = 1.0f;
                if (kNorm) inv = 1.0f / sqrtf(ssq_lds[wave][j][row] / (float)(KB * 16) + a.eps);
                const float vals[2] = {park[v * 64], park[(16 + v) * 64]};
                if constexpr (EPI == EPI_QKV) {
                    const QkvRow &r = qrow[(wave * 2 + j) * 32 + row];
                    float c, sn;
                    qkv_rotation(a, m, g, col, c, sn);
                    qkv_store(a, r, g, col, vals[0] * inv, vals[1] * inv, c, sn);
                } else {
                    float xin[2] = {0.0f, 0.0f};
                    if constexpr (EPI == EPI_RESID) {
#pragma unroll
                        for (int i = 0; i < 2; ++i) {
                            const int n = (g * 2 + i) * 32 + col;
                            if (n < a.N) xin[i] = a.x[(size_t)m * a.N + n];
                        }
                    }
                    skinny_epilogue<EPI, 2>(a, ks, m, g, col, vals, inv, xin);
                }
            }
        }
}

// n_blocks = packed 32-column blocks of W.  The K range of a workgroup is a.kb_per_split k-blocks (grid.y = a.ksplit).
template <int EPI>
inline hipError_t launch_tile(hipStream_t st, const SkinnyArgs &a, int n_blocks) {
    if (a.M <= 0 || n_blocks <= 0 || a.KB <= 0 || a.ksplit < 1 || (size_t)a.kb_per_split * a.ksplit < (size_t)a.KB) return hipErrorInvalidValue;
    if (EPI != EPI_PARTIAL && a.ksplit != 1) return hipErrorInvalidValue;
    const int row_tiles32 = (a.M + 31) / 32, row_tiles = (a.M + TILE_M - 1) / TILE_M, col_tiles = (n_blocks + 3) / 4;
    const dim3 grid(col_tiles * row_tiles, a.ksplit);
    gemm_tile_kernel<EPI><<<grid, 256, 0, st>>>(a, n_blocks, row_tiles32, col_tiles, row_tiles);
    return hipGetLastError();
}
