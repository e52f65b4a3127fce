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
// (2, 3) of a tile are rotary / gate-up pairs.  RMSNorm row sums of squares come from the kernel that wrote the
// rows (partial sums per row, added in a fixed order by the epilogue) when it provides them, else from the
// activation fragments as they are consumed - which costs a third of the loop's issue slots.
//
// What bounds it (measured): replaying only the loop's global loads takes 80 % of the kernel's time whatever the
// depth of the ring - all workgroups of an XCD ask its L2 for the same few lines at the same time (a k-step's
// activation fragments; every weight line once per row tile), which it serves at under half the rate it reaches on
// scattered reads - and under sustained MFMA load the shader clock settles near 1.7-1.9 GHz.  More k-steps per
// barrier, deeper rings, LDS reads a stage ahead, a fifth wavefront requesting lines ahead and eight wavefronts per
// tile all measured within 1 % or worse; fewer operand bytes per MFMA would need larger tiles than 512 rows on 256
// CUs leave room for.
#pragma once
#include "kernels_skinny.hip.h"

constexpr int TILE_M = 256, TILE_N = 128;
constexpr int TILE_KS = 1;    // k-steps (of 16) per pipeline stage, i.e. per workgroup barrier
#ifndef SJD_TILE_RING
#define SJD_TILE_RING 4
#endif
constexpr int TILE_RING = SJD_TILE_RING;  // stages of global loads in flight per wavefront

// The work of one workgroup: tile (column tile ct0 + ..., row tile ...) number `wg` of a list of col_tiles x row_tiles
// tiles that starts at column tile ct0, K range `ks`.
template <int EPI, bool SSQ_LOOP, int RT, int KS, int D>
SJD_D void tile_body(const SkinnyArgs &a, const int wg, const int ks, int n_blocks, int row_tiles32, int col_tiles, int row_tiles, int ct0) {
    constexpr bool kNorm = EPI != EPI_RESID && EPI != EPI_PARTIAL;
    constexpr bool kSsqLoop = kNorm && SSQ_LOOP;  // else the rows' sums of squares come from the kernel that wrote the rows
    constexpr int U = D % 2 == 0 ? D : 2 * D;  // unroll: ring slot and LDS buffer of an iteration are compile-time
    constexpr int TM = 128 * RT;              // rows of the workgroup's tile: wavefront w owns rows [32 RT w, 32 RT (w + 1))
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // blockIdx.x -> (column tile ct, row tile rt).  Workgroups go to the 8 XCDs round-robin by linear id, and every
    // XCD has its own L2: all row tiles of a column tile run on XCD ct % 8, so that its weights are fetched from HBM
    // by one L2 only.  id = 8 j + x enumerates XCD x's list of (column tile x + 8 (j / row_tiles), row tile
    // j % row_tiles); the grid is padded to 8 ceil(col_tiles / 8) column tiles and the padding exits here.
    const int ct_rel = (wg & 7) + 8 * ((wg >> 3) / row_tiles), rt = (wg >> 3) % row_tiles;
    if (ct_rel >= col_tiles) return;
    const int ct = ct0 + ct_rel;
    const int KB = a.KB;
    const int kb_lo = ks * a.kb_per_split;
    const int kb_hi = kb_lo + a.kb_per_split < KB ? kb_lo + a.kb_per_split : KB;
    const int n_k = kb_hi - kb_lo;             // k-steps of this workgroup
    const int n_it = (n_k + KS - 1) / KS;      // pipeline stages

    // this wavefront's operands: activation row tiles (of 32) RT (4 rt + wave) + {0 .. RT - 1}, straight into registers;
    // weight block 4 ct + wave, its share of the stage in LDS.  Indices past the end are clamped (their
    // products land in rows / columns the epilogue never stores).
    const u32x4 *Aj[RT];
#pragma unroll
    for (int j = 0; j < RT; ++j)
        Aj[j] = reinterpret_cast<const u32x4 *>(a.A) + (size_t)min((rt * 4 + wave) * RT + j, row_tiles32 - 1) * KB * 64 + lane;
    const int rb = min(ct * 4 + wave, n_blocks - 1);
    const u32x4 *B0 = reinterpret_cast<const u32x4 *>(a.W) + (size_t)rb * KB * 64 + lane;

    // k-loop: stage[buffer][k-step of the stage][weight block][lane]; epilogue: 8 KiB per wavefront to index its
    // accumulators by a run-time register number
    __shared__ u32x4 smem[2048];
    static_assert(2 * KS * 4 * 64 <= 2048, "stage buffers exceed the LDS array");
    u32x4 (*stage)[KS][4][64] = reinterpret_cast<u32x4 (*)[KS][4][64]>(smem);
    __shared__ float ssq_lds[4][RT][32];

    f32x16 acc[RT][4];
#pragma unroll
    for (int j = 0; j < RT; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][i][v] = 0.0f;
    float ssq[RT];
#pragma unroll
    for (int j = 0; j < RT; ++j) ssq[j] = 0.0f;

    if (n_it > 0) {
        u32x4 ra[D][KS][RT], rbw[D][KS];
        const u32x4 zero4 = {0u, 0u, 0u, 0u};
        // k-steps past the end re-read the last fragments (cache hits); their activations are zeroed when consumed
#define TILE_KB(step, q) ((size_t)(kb_lo + min((step) * KS + (q), n_k - 1)) * 64)
#define TILE_LOAD_A(slot, step)                                                             \
    do {                                                                                    \
        _Pragma("unroll") for (int q_ = 0; q_ < KS; ++q_)                                   \
            _Pragma("unroll") for (int j_ = 0; j_ < RT; ++j_) ra[slot][q_][j_] = Aj[j_][TILE_KB(step, q_)]; \
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
        // one pipeline stage: su = position in the unrolled group (ring slot and LDS buffer are compile-time)
        auto stage_step = [&](int su, int it) {
            const int slot = su % D, nslot = (su + 1) % D, cur = su & 1;
            bf16x8 bfr[KS][4];
#pragma unroll
            for (int q = 0; q < KS; ++q)
#pragma unroll
                for (int i = 0; i < 4; ++i) bfr[q][i] = __builtin_bit_cast(bf16x8, stage[cur][q][i][lane]);
#pragma unroll
            for (int q = 0; q < KS; ++q) {
                const bool valid = KS == 1 || it * KS + q < n_k;   // KS = 1: every stage that runs is a real k-step
#pragma unroll
                for (int j = 0; j < RT; ++j) {
                    const u32x4 araw = valid ? ra[slot][q][j] : zero4;
                    const bf16x8 av = __builtin_bit_cast(bf16x8, araw);
                    if (kSsqLoop) {
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
        };
        // Whole groups of U stages run without a test (the matrix cores are the bound here: every vector
        // instruction in this loop takes issue slots from the MFMAs); the last n_it % U stages behind uniform branches.
        int it0 = 0;
        for (; it0 + U <= n_it; it0 += U) {
#pragma unroll
            for (int su = 0; su < U; ++su) stage_step(su, it0 + su);
        }
#pragma unroll
        for (int su = 0; su < U; ++su)
            if (it0 + su < n_it) stage_step(su, it0 + su);
#undef TILE_KB
#undef TILE_LOAD_A
#undef TILE_LOAD_B
#undef TILE_STORE_B
    }

    // 1 / rms of the tile's rows, once per row (ssq_lds holds the factor, not the sum)
    const float inv_k = 1.0f / (float)(KB * 16);
    if (kSsqLoop) {
#pragma unroll
        for (int j = 0; j < RT; ++j) {
            const float t = ssq[j] + __shfl_xor(ssq[j], 32, 64);
            if (lane < 32) ssq_lds[wave][j][lane] = 1.0f / sqrtf(t * inv_k + a.eps);
        }
        __syncthreads();
    } else if (kNorm) {
        // row tid of the tile: its partial sums of squares in their fixed order
        const int m = rt * TM + tid;
        float t = 0.0f;
        if (tid < TM && m < a.M)
            for (int c = 0; c < a.row_ssq_n; ++c) t += a.row_ssq_part[(size_t)m * a.row_ssq_n + c];
        if (tid < TM) ssq_lds[tid / (32 * RT)][(tid >> 5) % RT][tid & 31] = 1.0f / sqrtf(t * inv_k + a.eps);
        __syncthreads();
    }
    // Vocabulary head with the guidance fused in: a wavefront's two row tiles are the conditional and the unconditional
    // rows of one sequence's window of 32 (256-row tiles only), so z = (l_u + s (l_c - l_u)) / T comes straight from the
    // two accumulators of a position.
    if constexpr (EPI == EPI_HEAD && RT == 2) {
        if (a.z_mode == 1) {
            const int colz = lane & 31;
            float inv_c[16], inv_u[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                inv_c[v] = ssq_lds[wave][0][row];
                inv_u[v] = ssq_lds[wave][1][row];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int n = (ct * 4 + i) * 32 + colz;
                if (ct * 4 + i >= n_blocks || n >= a.N) continue;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                    const int mc = rt * TM + wave * 64 + row, mu = mc + 32;
                    if (mu >= a.M) continue;
                    a.z_out[((size_t)(mc >> 6) * 32 + row) * a.N + n] = guided_z(acc[0][i][v], inv_c[v], acc[1][i][v], inv_u[v], a.cfg_scale, a.inv_t);
                    if (a.logits) {
                        a.logits[(size_t)mc * a.N + n] = acc[0][i][v] * inv_c[v];
                        a.logits[(size_t)mu * a.N + n] = acc[1][i][v] * inv_u[v];
                    }
                }
            }
            return;
        }
    }
    const int col = lane & 31;
    if constexpr (EPI != EPI_QKV) {
        // short bodies: straight from the accumulators, four rows at a time (the residual values of all four are
        // requested before the first is used)
#pragma unroll
        for (int j = 0; j < RT; ++j)
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const int g = ct * 2 + p;
                if (g * 2 >= n_blocks) continue;  // past the last column pair
#pragma unroll
                for (int v0 = 0; v0 < 16; v0 += 4) {
                    const int row0 = 2 * v0 + 4 * (lane >> 5), m0 = rt * TM + (wave * RT + j) * 32 + row0;
                    float xin[4][2];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        xin[u][0] = xin[u][1] = 0.0f;
                        if constexpr (EPI == EPI_RESID) {
                            if (m0 + u >= a.M) continue;
#pragma unroll
                            for (int i = 0; i < 2; ++i) {
                                const int n = (g * 2 + i) * 32 + col;
                                if (n < a.N) xin[u][i] = a.x[(size_t)(m0 + u) * a.N + n];
                            }
                        }
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        if (m0 + u >= a.M) continue;
                        const float inv = kNorm ? ssq_lds[wave][j][row0 + u] : 1.0f;
                        const float vals[2] = {acc[j][p * 2][v0 + u], acc[j][p * 2 + 1][v0 + u]};
                        skinny_epilogue<EPI, 2>(a, ks, m0 + u, g * 2, col, vals, inv, xin[u]);
                    }
                }
            }
        return;
    }
    // QKV: the body is long; unrolled 64 times it would exceed what the compiler unrolls, and a rolled loop cannot
    // index accumulator registers.  Each lane parks one row tile x column pair (32 values) in LDS (its own slots, so
    // no barrier) and walks them in a rolled loop.
    float *park = reinterpret_cast<float *>(smem) + wave * 2048 + lane;
    // the row-dependent part of the destination (integer divisions, page lookup) once per row, not per element
    __shared__ QkvRow qrow[EPI == EPI_QKV ? TM : 1];
    if (EPI == EPI_QKV) {
        const int m = rt * TM + tid;
        if (tid < TM && m < a.M) qrow[EPI == EPI_QKV ? tid : 0] = qkv_row(a, m);
        __syncthreads();
    }
#pragma unroll
    for (int j = 0; j < RT; ++j)
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int g = ct * 2 + p;
            if (g * 2 >= n_blocks) continue;  // past the last column pair
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) park[(i * 16 + v) * 64] = acc[j][p * 2 + i][v];
            // four rows at a time: their rotations are requested before the first is used
#pragma unroll 1
            for (int v0 = 0; v0 < 16; v0 += 4) {
                const int row0 = 2 * v0 + 4 * (lane >> 5), m0 = rt * TM + (wave * RT + j) * 32 + row0;
                float rc[4], rs[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    rc[u] = 1.0f;
                    rs[u] = 0.0f;
                    if (m0 + u < a.M) qkv_rotation(a, m0 + u, g, col, rc[u], rs[u]);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int v = v0 + u;
                    if (m0 + u >= a.M) continue;
                    const float inv = ssq_lds[wave][j][row0 + u];
                    qkv_store(a, qrow[(wave * RT + j) * 32 + row0 + u], g, col, park[v * 64] * inv, park[(16 + v) * 64] * inv, rc[u], rs[u]);
                }
            }
        }
}

template <int EPI, bool SSQ_LOOP = true, int RT = 2, int KS = TILE_KS, int D = TILE_RING>
__global__ __launch_bounds__(256, RT == 2 ? 2 : 3) void gemm_tile_kernel(SkinnyArgs a, int n_blocks, int row_tiles32, int col_tiles, int row_tiles) {
    tile_body<EPI, SSQ_LOOP, RT, KS, D>(a, blockIdx.x, blockIdx.y, n_blocks, row_tiles32, col_tiles, row_tiles, 0);
}

// Two tile heights in one launch.  256-row tiles move a quarter fewer operand bytes per MFMA than 128-row tiles, but a
// launch whose 256-row tiles number between one and two per CU leaves the CUs with one or two of them side by side.
// Here workgroups [0, wg_split) take 256-row tiles of the column tiles [0, ct_split) - one per CU - and the others take
// the remaining column tiles as 128-row tiles, which fill the second slot of the CUs (the register count of the
// 256-row body admits two workgroups per CU, whatever their height).  wg_split is a multiple of 8, so both lists keep
// the workgroup id -> XCD correspondence of tile_body.
template <int EPI, bool SSQ_LOOP>
__global__ __launch_bounds__(256, 2) void gemm_tile_mixed_kernel(SkinnyArgs a, int n_blocks, int row_tiles32, int col_tiles, int ct_split, int wg_split,
                                                                int row_tiles2, int row_tiles1) {
    if ((int)blockIdx.x < wg_split) tile_body<EPI, SSQ_LOOP, 2, TILE_KS, TILE_RING>(a, blockIdx.x, blockIdx.y, n_blocks, row_tiles32, ct_split, row_tiles2, 0);
    else tile_body<EPI, SSQ_LOOP, 1, TILE_KS, TILE_RING>(a, blockIdx.x - wg_split, blockIdx.y, n_blocks, row_tiles32, col_tiles - ct_split, row_tiles1, ct_split);
}

// Rows per workgroup tile for n_blocks column blocks over M rows.  256 rows (two 32-row tiles per wavefront) need
// the fewest operand bytes per MFMA: 0.75 KiB against 1.25 KiB for 128 rows, whose weight fragments alone would
// take the whole LDS bandwidth at full MFMA rate.  128 rows are chosen where they spread the work better: when
// 256-row tiles would not even fill the CUs, or when the most loaded CU (a launch takes as long as that one)
// gets less work - ceil(workgroups / CUs) tiles of 256 rows against as many half-size ones.
inline int tile_rows_for(int M, int n_blocks, int ksplit, int n_cus) {
    const int col_tiles = (n_blocks + 3) / 4;
    const long wg2 = (long)col_tiles * ((M + 255) / 256) * ksplit, wg1 = (long)col_tiles * ((M + 127) / 128) * ksplit;
    if (wg2 < n_cus) return 128;
    const long cost2 = 2 * ((wg2 + n_cus - 1) / n_cus), cost1 = (wg1 + n_cus - 1) / n_cus;
    return cost1 < cost2 ? 128 : 256;
}

// n_blocks = packed 32-column blocks of W.  The K range of a workgroup is a.kb_per_split k-blocks (grid.y = a.ksplit).
template <int EPI>
inline hipError_t launch_tile(hipStream_t st, const SkinnyArgs &a, int n_blocks, int tile_rows = 0, bool two_heights = true) {
    const int tile_rows_in = tile_rows;   // 0: the launcher chooses
    if (a.M <= 0 || n_blocks <= 0 || a.KB <= 0 || a.ksplit < 1 || (size_t)a.kb_per_split * a.ksplit < (size_t)a.KB) return hipErrorInvalidValue;
    if (EPI != EPI_PARTIAL && a.ksplit != 1) return hipErrorInvalidValue;
    if (tile_rows == 0) tile_rows = tile_rows_for(a.M, n_blocks, a.ksplit, a.n_cus > 0 ? a.n_cus : 256);
    const int row_tiles32 = (a.M + 31) / 32, row_tiles = (a.M + tile_rows - 1) / tile_rows, col_tiles = (n_blocks + 3) / 4;
    const dim3 grid(8 * ((col_tiles + 7) / 8) * row_tiles, a.ksplit);
    constexpr bool kNorm = EPI != EPI_RESID && EPI != EPI_PARTIAL;
    const bool ssq_loop = !(kNorm && a.row_ssq_part);
    // Between one and two 256-row tiles per CU: one 256-row tile on every CU, the other column tiles as 128-row tiles
    // beside them (measured at 512 x 22016 x 4096: 95.5 us against 108.0 with 128-row tiles and 126 with 256-row tiles)
    const int n_cus = a.n_cus > 0 ? a.n_cus : 256;
    const int rt2 = (a.M + 255) / 256, rt1 = (a.M + 127) / 128;
    // (not where 128-row tiles alone give every CU the same number of workgroups: 1024 x 12288 x 4096, three per CU,
    // 120.6 us against 132.7 mixed)
    if (two_heights && tile_rows_in == 0 && EPI != EPI_HEAD && a.ksplit == 1 && rt1 > rt2 && col_tiles * rt2 > n_cus && col_tiles * rt2 < 2 * n_cus &&
        n_cus / rt2 >= 8 && (col_tiles * rt1) % n_cus != 0) {
        const int ct_split = n_cus / rt2 / 8 * 8;
        const int wg_split = ct_split * rt2, wg_rest = 8 * ((col_tiles - ct_split + 7) / 8) * rt1;
        if (ssq_loop) gemm_tile_mixed_kernel<EPI, true><<<dim3(wg_split + wg_rest, 1), 256, 0, st>>>(a, n_blocks, row_tiles32, col_tiles, ct_split, wg_split, rt2, rt1);
        else gemm_tile_mixed_kernel<EPI, false><<<dim3(wg_split + wg_rest, 1), 256, 0, st>>>(a, n_blocks, row_tiles32, col_tiles, ct_split, wg_split, rt2, rt1);
        return hipGetLastError();
    }
    if (tile_rows == 128) {
        if (ssq_loop) gemm_tile_kernel<EPI, true, 1><<<grid, 256, 0, st>>>(a, n_blocks, row_tiles32, col_tiles, row_tiles);
        else gemm_tile_kernel<EPI, false, 1><<<grid, 256, 0, st>>>(a, n_blocks, row_tiles32, col_tiles, row_tiles);
    } else {
        if (ssq_loop) gemm_tile_kernel<EPI, true, 2><<<grid, 256, 0, st>>>(a, n_blocks, row_tiles32, col_tiles, row_tiles);
        else gemm_tile_kernel<EPI, false, 2><<<grid, 256, 0, st>>>(a, n_blocks, row_tiles32, col_tiles, row_tiles);
    }
    return hipGetLastError();
}
