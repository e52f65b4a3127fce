// Fused projection kernels for small row counts (M = 2 * sequences * window <= 64): the regime of
// Sec. 4.1 Step 2 where every GEMM of the forward is bound by streaming its weights from HBM once.
//
// One workgroup of NW wavefronts owns NBW column blocks of 32 and ALL of K: wavefront w takes the
// k-blocks w, w + NW, w + 2 NW, ... and keeps a ring of DEPTH fragment loads in flight (each a fully
// coalesced 1 KiB read of fragment-major W straight into MFMA operand registers); the NW partial
// accumulators are summed through LDS, so no partial sums ever go to HBM and the epilogue sees final
// values.  The epilogues absorb what would otherwise be separate memory-bound kernels:
//   QKV     per-row RMSNorm scale, rotary embedding, queries to the attention layout, keys/values into
//           their KV pages
//   RESID   residual add into the fp32 stream + the bf16 copy of the stream that feeds the next GEMM
//   SWIGLU  per-row RMSNorm scale, silu(gate) * up
//   HEAD    per-row RMSNorm scale, fp32 logits
//   PARTIAL plain fp32 partial sums [ksplit][M][N] of a K range (grid.y = ksplit); resid_reduce_kernel adds them
//           up after the kernel boundary.  Used when one workgroup per column group would have to pull more
//           than ~0.5 MB through its CU (wide K, M = 64): splitting K also splits the activation re-reads.
// RMSNorm is folded in: the gain is multiplied into the weights when they are packed, the input is
// the raw residual stream in bf16, its per-row sum of squares is accumulated from the very A fragments
// the MFMA consumes, and the row scale 1/rms is applied to the accumulators (it commutes with the
// contraction).
#pragma once
#include <algorithm>

#include "common.hip.h"
#include "kernels_forward.hip.h"

#ifndef SJD_SKINNY_DEPTH
#define SJD_SKINNY_DEPTH 8   // slots of the operand ring of a wavefront
#endif

enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_HEAD = 3, EPI_PARTIAL = 4 };

// Where row m of the QKV projection goes.  The operand layouts of queries, keys and values are all of the form
// f(row) + g(head dimension), so everything that depends on the row alone is worked out once per row:
struct QkvRow {
    int pos;    // absolute position (rotary angle), -1 for a row that is not computed
    int q_off;  // element offset of this row in the query buffer of head 0: sequence segment and window index
    int page;   // KV page of the position
    int k_off;  // row part of the element offset inside a (page, head) block of keys
    int v_off;  // same for values
};
struct SkinnyArgs {
    const bf16_t *A;   // [MT][KB][64][8] raw activations, fragment-major
    const bf16_t *W;   // [groups * NBW][KB][64][8]
    int M, KB;
    int n_cus;         // compute units of the device (launch heuristics on the host)
    int groups;        // column groups (set by the launcher)
    int m_groups;      // row groups of MT * 32 rows, each run by its own workgroups over the same weights (M > 64)
    int row_split;     // 2: (one 32-row tile, whole K) two workgroups per column group, 16 rows each; else 1
    int k_rot;         // 1: workgroup id starts its k-loop (id / 8) iterations in (see skinny_body), 0: all start at k = 0
    int n_heavy;       // mixed-width launch (set by its launcher): workgroups [0, n_heavy) take two column groups each
    float eps;
    // RESID
    float *x;          // [M][N] fp32 residual stream, updated in place
    bf16_t *xb;        // the same in bf16, fragment-major [M][N]
    int N;             // also the logits row length for HEAD
    // Many-row kernels: per-row sums of squares of the (bf16) input rows, as row_ssq_n partial sums per row written
    // by the kernel that produced the rows; NULL: taken from the activation fragments inside the k-loop
    const float *row_ssq_part;
    int row_ssq_n;
    // QKV: per-row tables written once per forward by embed_dual_kernel (no dependent loads in the projections)
    const QkvRow *row_meta;   // [M]
    const float2 *row_rot;    // [M][hd / 2] (cos, sin) of the row's position; (1, 0) for rows that are not computed
    bf16_t *q_out;
    KvPool pool;
    int L, H, Hkv, hd;
    // SWIGLU
    bf16_t *h;
    int F;
    // HEAD
    float *logits;           // [M][N] fp32 logits (NULL: not kept)
    // HEAD with the guidance fused in (Sec. 5.1 guidance weight): rows come as a conditional tile and the
    // unconditional tile of the same positions, and the epilogue writes z = (l_u + s (l_c - l_u)) / T per position,
    // [positions][N], so that the sampling kernel reads one row per position and the logits need not be stored.
    // z_mode 0: off; 1: window of 32, row tile 2 q is conditional and 2 q + 1 unconditional for sequence q;
    // 2: one sequence, window of 16: rows 0..15 conditional, 16..31 unconditional.
    float *z_out;
    int z_mode;
    float cfg_scale, inv_t;
    // PARTIAL: K split across workgroups (grid.y = ksplit), plain partial sums; the other epilogues run with ksplit 1
    int ksplit, kb_per_split;
    float *part;             // [ksplit][M][N]
    // L2 warm-up of the NEXT projection's weights: workgroups [groups, groups + pf_wgs) of a launch with one row
    // group and whole K only touch memory.  The next launch's workgroup g' will read slab g' (pf_slab_bytes at
    // pf_base + g' * pf_slab_bytes, g' < pf_groups) and runs on XCD g' % 8, whose L2 the touching workgroup shares.
    const char *pf_base;
    uint32_t pf_slab_bytes;
    int pf_groups, pf_wgs;   // pf_wgs: a multiple of 8, 0 = none
    uint32_t *pf_sink;       // a device word nobody reads; a (practically never taken) store to it keeps the loads alive
    // ... and of the keys and values that the next attention launch will read (workgroups [groups + pf_wgs,
    // groups + pf_wgs + kv_wgs)): the complete pages of the context before this forward's rows, which no launch of
    // this forward writes.  Attention workgroup p = (segment p / H, head p % H) runs on XCD p % 8.
    int kv_wgs;                 // a multiple of 8, 0 = none
    KvPool kv_pool;             // the pools of the layer whose attention comes next
    int kv_pairs;               // segments * H
    const int32_t *kv_seg_kv;   // [segments] tokens in the cache before this forward's rows
};

SJD_D QkvRow qkv_row(const SkinnyArgs &a, int m) { return a.row_meta[m]; }
// Column group g = (head, sub-block of 32 dimensions); v0 / v1 are dimensions j0 = 32 sub + col and j0 + hd / 2 of
// that head (a rotary pair): rotate q and k, then queries to the attention operand layout, keys / values into
// their page.
// (cos, sin) of the rotation that qkv_store applies to this element pair of row m: (1, 0) for value heads
SJD_D void qkv_rotation(const SkinnyArgs &a, int m, int g, int col, float &c, float &s) {
    const int pairs = a.hd >> 6;
    const int head = g / pairs, sub = g % pairs, half = a.hd >> 1;
    c = 1.0f;
    s = 0.0f;
    if (head < a.H + a.Hkv) {
        const float2 cs = a.row_rot[(size_t)m * half + sub * 32 + col];
        c = cs.x;
        s = cs.y;
    }
}
SJD_D void qkv_store(const SkinnyArgs &a, const QkvRow &r, int g, int col, float v0, float v1, float c, float s) {
    if (r.pos < 0) return;
    const int pairs = a.hd >> 6;
    const int head = g / pairs, sub = g % pairs, half = a.hd >> 1;
    const int j0 = sub * 32 + col, j1 = j0 + half;
    {
        const float r0 = v0 * c - v1 * s, r1 = v1 * c + v0 * s;
        v0 = r0;
        v1 = r1;
    }
    if (head < a.H) {
        bf16_t *dst = a.q_out + (size_t)head * Layout<bf16_t>::q_elems(a.L, a.hd) + r.q_off;
        dst[Layout<bf16_t>::q_index(0, j0, a.hd)] = float_to_bf16(v0);
        dst[Layout<bf16_t>::q_index(0, j1, a.hd)] = float_to_bf16(v1);
    } else {
        const size_t blk = (size_t)a.pool.page_tokens * a.hd;
        if (head < a.H + a.Hkv) {
            bf16_t *dst = (bf16_t *)a.pool.k + ((size_t)r.page * a.Hkv + (head - a.H)) * blk + r.k_off;
            dst[Layout<bf16_t>::k_index(0, j0, a.hd)] = float_to_bf16(v0);
            dst[Layout<bf16_t>::k_index(0, j1, a.hd)] = float_to_bf16(v1);
        } else {
            bf16_t *dst = (bf16_t *)a.pool.v + ((size_t)r.page * a.Hkv + (head - a.H - a.Hkv)) * blk + r.v_off;
            dst[Layout<bf16_t>::v_index(0, j0, a.hd)] = float_to_bf16(v0);
            dst[Layout<bf16_t>::v_index(0, j1, a.hd)] = float_to_bf16(v1);
        }
    }
}

// z = fma(s, l_c - l_u, l_u) / T on logits l = value * (1 / rms), every operation rounded on its own (the decision stage
// is specified bit for bit on these values, and the compiler may otherwise contract the products into the sums)
SJD_D float guided_z(float val_c, float inv_c, float val_u, float inv_u, float s, float inv_t) {
    const float lc = __fmul_rn(val_c, inv_c), lu = __fmul_rn(val_u, inv_u);
    return __fmul_rn(__fmaf_rn(s, __fsub_rn(lc, lu), lu), inv_t);
}

// One output element pair of the projection epilogues: row m, column `col` of NBW consecutive column blocks
// (val[i] = block blk0 + i), inv = 1 / rms of row m (1 where the epilogue does not normalise).
// xin: the residual-stream values x[m][n_i] (RESID only; the caller loads them, early if it can).
template <int EPI, int NBW>
SJD_D void skinny_epilogue(const SkinnyArgs &a, int ks, int m, int blk0, int col, const float (&val)[NBW], float inv,
                           const float (&xin)[NBW]) {
    if constexpr (EPI == EPI_PARTIAL) {
#pragma unroll
        for (int i = 0; i < NBW; ++i) {
            const int n = (blk0 + i) * 32 + col;
            if (n < a.N) a.part[((size_t)ks * a.M + m) * a.N + n] = val[i];
        }
    } else if constexpr (EPI == EPI_RESID) {
#pragma unroll
        for (int i = 0; i < NBW; ++i) {
            const int n = (blk0 + i) * 32 + col;
            if (n < a.N) {
                const float nv = xin[i] + val[i];
                a.x[(size_t)m * a.N + n] = nv;
                a.xb[Layout<bf16_t>::a_index(m, n, a.N)] = float_to_bf16(nv);
            }
        }
    } else if constexpr (EPI == EPI_HEAD) {
#pragma unroll
        for (int i = 0; i < NBW; ++i) {
            const int n = (blk0 + i) * 32 + col;
            if (n < a.N) a.logits[(size_t)m * a.N + n] = val[i] * inv;
        }
    } else if constexpr (EPI == EPI_SWIGLU) {
        // blocks come in pairs: gate columns [32 p, 32 p + 32) in block 2 p, the matching up columns in block 2 p + 1
        static_assert(NBW % 2 == 0, "gate and up blocks come in pairs");
#pragma unroll
        for (int i = 0; i < NBW; i += 2) {
            const float gt = val[i] * inv, up = val[i + 1] * inv;
            const int n = ((blk0 + i) >> 1) * 32 + col;
            // hardware exp2 and reciprocal (1 ulp each): the result is rounded to bf16 next
            if (n < a.F) a.h[Layout<bf16_t>::a_index(m, n, a.F)] = float_to_bf16(__fdividef(gt, 1.0f + __expf(-gt)) * up);
        }
    } else {
        static_assert(EPI != EPI_QKV, "the QKV epilogue is qkv_row + qkv_rotation + qkv_store, called by the kernels");
    }
}

// Workgroup `id` (linear, >= first_id) of a launch reads one word of every 128-byte line of its share of the next
// launch's weight slabs, which brings the lines into the L2 of the XCD it runs on.  Workgroups go to XCDs round-robin
// by linear id, so it takes slabs g' with g' % 8 == id % 8; the pf_wgs / 8 workgroups of one XCD split those evenly.
SJD_D void l2_warm_next(const SkinnyArgs &a, int id, int first_id, int tid, int threads) {
    const int xcd = id & 7, rank = (id - first_id) >> 3, ranks = a.pf_wgs >> 3;
    const int n_slabs = a.pf_groups > xcd ? (a.pf_groups - xcd + 7) >> 3 : 0;
    const uint32_t lines_per_slab = a.pf_slab_bytes >> 7;
    const uint32_t total = (uint32_t)n_slabs * lines_per_slab, per = (total + ranks - 1) / ranks;
    const uint32_t lo = rank * per, hi = lo + per < total ? lo + per : total;
    uint32_t sink = 0;
#pragma unroll 8
    for (uint32_t i = lo + tid; i < hi; i += threads) {
        const uint32_t s = i / lines_per_slab, l = i - s * lines_per_slab;
        sink ^= *reinterpret_cast<const uint32_t *>(a.pf_base + (size_t)(xcd + 8 * s) * a.pf_slab_bytes + (size_t)l * 128);
    }
    if (sink == 0x9e3779b9u) *a.pf_sink = sink;  // a word nobody reads; the store only keeps the loads alive
}

SJD_D void l2_warm_kv(const SkinnyArgs &a, int id, int first_id, int tid, int threads) {
    const int xcd = id & 7, rank = (id - first_id) >> 3, ranks = a.kv_wgs >> 3;
    const int G = a.H / a.Hkv;
    const size_t blk_bytes = (size_t)a.kv_pool.page_tokens * a.hd * sizeof(bf16_t);  // one (page, kv head) block of keys or values
    const uint32_t blk_lines = (uint32_t)(blk_bytes >> 7), pair_lines = (uint32_t)a.kv_pool.pages_per_seg * 2 * blk_lines;
    const uint32_t n_pairs = a.kv_pairs > xcd ? (uint32_t)(a.kv_pairs - xcd + 7) >> 3 : 0;  // this XCD's (segment, head) pairs
    uint32_t sink = 0;
    // One flat index space over (pair, page, keys | values, line), so that a thread's few lines are independent of
    // each other: the page count of the segment and the page table entry load side by side, then the line.
#pragma unroll 2
    for (uint32_t i = rank * threads + tid; i < n_pairs * pair_lines; i += ranks * threads) {
        const uint32_t j = i / pair_lines, r0 = i - j * pair_lines;
        const uint32_t pg = r0 / (2 * blk_lines), r = r0 - pg * 2 * blk_lines;
        const int p = xcd + 8 * (int)j, seg = p / a.H, kvh = (p % a.H) / G;
        const int pages = a.kv_seg_kv[seg] / a.kv_pool.page_tokens;
        const int page = a.kv_pool.page_table[seg * a.kv_pool.pages_per_seg + pg];
        if ((int)pg < pages) {
            const char *base = r < blk_lines ? (const char *)a.kv_pool.k : (const char *)a.kv_pool.v;
            sink ^= *reinterpret_cast<const uint32_t *>(base + ((size_t)page * a.Hkv + kvh) * blk_bytes + (size_t)(r % blk_lines) * 128);
        }
    }
    if (sink == 0x9e3779b9u) *a.pf_sink = sink;
}

template <int MT, int NBW, int NW, int DEPTH, int EPI, bool SPLIT>
SJD_D void skinny_body(const SkinnyArgs &a, int g, int mg, int half, int blk0);

template <int MT, int NBW, int NW, int DEPTH, int EPI, bool SPLIT = false>
__global__ __launch_bounds__(NW * 64) void gemm_skinny_kernel(SkinnyArgs a) {
    const int tid = threadIdx.x;
    // computing workgroups come first: one per column group, or (row_split 2) two, listed per XCD like row groups
    const int n_compute = SPLIT ? 16 * ((a.groups + 7) / 8) : a.m_groups > 1 ? 8 * ((a.groups + 7) / 8) * a.m_groups : a.groups;
    if ((int)blockIdx.x >= n_compute && (a.pf_wgs | a.kv_wgs)) {  // whole workgroup: only touches what the next launches read
        if ((int)blockIdx.x < n_compute + a.pf_wgs) l2_warm_next(a, blockIdx.x, n_compute, tid, NW * 64);
        else l2_warm_kv(a, blockIdx.x, n_compute + a.pf_wgs, tid, NW * 64);
        return;
    }
    // blockIdx.x enumerates (column group g, row group mg).  With several row groups all row groups of a column
    // group run on XCD g % 8 (workgroups go to XCDs round-robin by linear id, and every XCD has its own L2), so that
    // one L2 fetches the group's weights from HBM: id = 8 j + x is entry j of XCD x's list of
    // (g = x + 8 (j / m_groups), mg = j % m_groups); the grid is padded to 8 ceil(groups / 8) groups.
    int g = blockIdx.x, mg = 0;
    if (a.m_groups > 1) {
        g = (blockIdx.x & 7) + 8 * ((blockIdx.x >> 3) / a.m_groups);
        mg = (blockIdx.x >> 3) % a.m_groups;
        if (g >= a.groups) return;
    }
    // row_split 2: this workgroup computes rows [16 half, 16 half + 16) of the 32-row tile only.  The loop is bound
    // by what the CU's L1 delivers, and half the rows are half the activation lines (lane l of a fragment holds row
    // l % 32, so the other half's lanes simply do not load); the MFMAs run on zeros for them, which costs nothing here.
    int half = 0;
    if (SPLIT) {
        g = (blockIdx.x & 7) + 8 * ((blockIdx.x >> 4));
        half = (blockIdx.x >> 3) & 1;
        if (g >= a.groups) return;
    }
    skinny_body<MT, NBW, NW, DEPTH, EPI, SPLIT>(a, g, mg, half, g * NBW);
}

// Workgroups of two widths in one launch, for more than 256 column groups of two blocks (gate/up and vocabulary
// head of the wide models).  A CU keeps a bounded number of bytes in flight, and every workgroup pulls all 64 x K
// activations beside its weights: with one group per workgroup some CUs get two workgroups (2 x (weights +
// activations)) while the others idle half the time.  Here the first n_heavy workgroups take two consecutive groups
// (4 blocks: one pass over the activations for both) and the others one, n_heavy + (groups - 2 n_heavy) workgroups in
// all: 256 for up to 512 groups.  The register count admits one workgroup per CU, so each CU gets one.
template <int MT, int NW, int DEPTH, int EPI>
__global__ __launch_bounds__(NW * 64) void gemm_skinny_mixed_kernel(SkinnyArgs a) {
    static_assert(EPI == EPI_SWIGLU || EPI == EPI_HEAD, "epilogues that take any even number of blocks");
    const int w = blockIdx.x;
    // (the wide body's ring has 3/4 of the slots: 6 fragments per slot instead of 4, more bytes in flight all the same)
    if (w < a.n_heavy) skinny_body<MT, 4, NW, DEPTH * 3 / 4, EPI, false>(a, 2 * w, 0, 0, 4 * w);
    else skinny_body<MT, 2, NW, DEPTH, EPI, false>(a, a.n_heavy + w, 0, 0, 2 * (a.n_heavy + w));
}

// The workgroup's work: column blocks [blk0, blk0 + NBW) (column group g of the QKV epilogue), row group mg.
template <int MT, int NBW, int NW, int DEPTH, int EPI, bool SPLIT>
SJD_D void skinny_body(const SkinnyArgs &a, int g, int mg, int half, int blk0) {
    constexpr bool kNorm = EPI != EPI_RESID && EPI != EPI_PARTIAL;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps the k-loop control flow scalar
    const bool a_lane = !SPLIT || ((lane >> 4) & 1) == half;  // SPLIT false: a constant, the loads below stay unconditional
    const int KB = a.KB, m_base = mg * MT * 32;
    const u32x4 *Wp = reinterpret_cast<const u32x4 *>(a.W) + (size_t)blk0 * KB * 64 + lane;
    const u32x4 *Ap = reinterpret_cast<const u32x4 *>(a.A) + (size_t)mg * MT * KB * 64 + lane;
    // this workgroup's k-blocks: [kb_lo, kb_hi); wavefront w takes kb_lo + w, kb_lo + w + NW, ...
    const int ks = blockIdx.y;
    const int kb_lo = ks * a.kb_per_split;
    const int kb_hi = kb_lo + a.kb_per_split < KB ? kb_lo + a.kb_per_split : KB;
    const int n_it = kb_lo + wave < kb_hi ? (kb_hi - kb_lo - wave + NW - 1) / NW : 0;
    // All workgroups of a launch read the same activation fragments; started together at k = 0 they would ask the same
    // L2 channel for the same lines at the same time all the way.  Workgroup id therefore walks its k-blocks in the
    // rotated order rot, rot + 1, ..., n_it - 1, 0, ..., rot - 1 (ids 8 apart share an XCD's L2: rot = id / 8).
    const int rot = n_it > 0 ? (int)(((blockIdx.x >> 3) * (unsigned)a.k_rot) % (unsigned)n_it) : 0;
    auto kb_of = [&](int it) {
        const int r = it + rot;
        return (size_t)(kb_lo + wave + (r >= n_it ? r - n_it : r) * NW);
    };

    // What the epilogue will need from memory is requested now, ahead of the weight stream, so that its latency
    // is not paid after the last MFMA: residual values (RESID), row destination and rotation (QKV).  Thread t ends
    // up with elements e = t, t + 64 NW, ... of every tile (see the reduction below).
    constexpr int EPT = 1024 / (NW * 64);  // elements per thread per tile
    [[maybe_unused]] float xpre[MT][NBW][EPT];
    [[maybe_unused]] QkvRow qrow[MT][EPT];
    [[maybe_unused]] float rot_c[MT][EPT], rot_s[MT][EPT];
    if (EPI == EPI_RESID || EPI == EPI_QKV) {
#pragma unroll
        for (int j = 0; j < MT; ++j)
#pragma unroll
            for (int hh = 0; hh < EPT; ++hh) {
                const int v = wave + NW * hh;
                const int m = m_base + j * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (EPI == EPI_RESID) {
#pragma unroll
                    for (int i = 0; i < NBW; ++i) {
                        const int n = (blk0 + i) * 32 + (lane & 31);
                        xpre[j][i][hh] = m < a.M && n < a.N && (!SPLIT || ((m >> 4) & 1) == half) ? a.x[(size_t)m * a.N + n] : 0.0f;
                    }
                } else {
                    qrow[j][hh].pos = -1;
                    rot_c[j][hh] = 1.0f;
                    rot_s[j][hh] = 0.0f;
                    if (m < a.M && (!SPLIT || ((m >> 4) & 1) == half)) {
                        qrow[j][hh] = qkv_row(a, m);
                        qkv_rotation(a, m, g, lane & 31, rot_c[j][hh], rot_s[j][hh]);
                    }
                }
            }
    }

    f32x16 acc[MT][NBW];
#pragma unroll
    for (int j = 0; j < MT; ++j)
#pragma unroll
        for (int i = 0; i < NBW; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][i][v] = 0.0f;
    float ssq[MT];
#pragma unroll
    for (int j = 0; j < MT; ++j) ssq[j] = 0.0f;

    // Ring of DEPTH slots; a wavefront with fewer than DEPTH iterations fills the spare slots with its last
    // fragment (never consumed).
    if (n_it > 0) {
        u32x4 bq[DEPTH][NBW], aq[DEPTH][MT];
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) {
            const size_t kb = kb_of(s < n_it ? s : n_it - 1);
#pragma unroll
            for (int i = 0; i < NBW; ++i) bq[s][i] = __builtin_nontemporal_load(Wp + ((size_t)i * KB + kb) * 64);
#pragma unroll
            for (int j = 0; j < MT; ++j) aq[s][j] = a_lane ? Ap[((size_t)j * KB + kb) * 64] : u32x4{0u, 0u, 0u, 0u};
        }
        __builtin_amdgcn_sched_barrier(0);
        auto consume = [&](int s) {
#pragma unroll
            for (int j = 0; j < MT; ++j) {
                const u32x4 araw = aq[s][j];
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
                for (int i = 0; i < NBW; ++i)
                    acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(bf16x8, bq[s][i]), acc[j][i], 0, 0, 0);
            }
        };
        auto refill = [&](int s, int it) {
            const size_t kb = kb_of(it);
#pragma unroll
            for (int i = 0; i < NBW; ++i) bq[s][i] = __builtin_nontemporal_load(Wp + ((size_t)i * KB + kb) * 64);
#pragma unroll
            for (int j = 0; j < MT; ++j) aq[s][j] = a_lane ? Ap[((size_t)j * KB + kb) * 64] : u32x4{0u, 0u, 0u, 0u};
        };
        // Steady state: groups of DEPTH iterations whose refills are all fragments that will be used.  The body is
        // branch-free so that the compiler counts outstanding loads exactly (a slot is consumed while the
        // DEPTH - 1 younger ones are still in flight).
        int it0 = 0;
        for (; it0 + 2 * DEPTH <= n_it; it0 += DEPTH) {
#pragma unroll
            for (int s = 0; s < DEPTH; ++s) {
                consume(s);
                refill(s, it0 + s + DEPTH);
                __builtin_amdgcn_sched_barrier(0);  // keep the refill here: the scheduler must not sink it towards its use
            }
        }
        // The last n_it - it0 < 2 DEPTH iterations: refill only what is still needed (the conditions are
        // wavefront-uniform), then drain.  Every fragment is loaded exactly once: with the weights already in L2 the
        // loop is bound by what the CU's L1 delivers, so a redundant load costs as much as a useful one.
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) {
            if (it0 + s < n_it) {
                consume(s);
                if (it0 + s + DEPTH < n_it) refill(s, it0 + s + DEPTH);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int s = 0; s < DEPTH; ++s)
            if (it0 + DEPTH + s < n_it) consume(s);
    }

    // ---- sum the NW partial tiles through LDS; thread t ends up with elements e = t and t + 512 of every
    //      tile: accumulator register v = e / 64 of lane l = e % 64, i.e. row 8 (v / 4) + 4 (l / 32) + v % 4,
    //      column l % 32.
    __shared__ float red[NW][16][64];
    __shared__ float ssq_lds[NW][MT][32];
    if (kNorm) {
#pragma unroll
        for (int j = 0; j < MT; ++j) {
            const float t = ssq[j] + __shfl_xor(ssq[j], 32, 64);
            if (lane < 32) ssq_lds[wave][j][lane] = t;
        }
    }
    float out[MT][NBW][EPT];
#pragma unroll
    for (int j = 0; j < MT; ++j)
#pragma unroll
        for (int i = 0; i < NBW; ++i) {
            __syncthreads();
#pragma unroll
            for (int v = 0; v < 16; ++v) red[wave][v][lane] = acc[j][i][v];
            __syncthreads();
#pragma unroll
            for (int hh = 0; hh < EPT; ++hh) {
                const int v = wave + NW * hh;
                float s = 0.0f;
#pragma unroll
                for (int w = 0; w < NW; ++w) s += red[w][v][lane];
                out[j][i][hh] = s;
            }
        }

    const int col = lane & 31;
    if constexpr (EPI == EPI_HEAD) {
        if (a.z_mode != 0) {
            // conditional / unconditional value pairs of a position sit in the same thread: tiles j = 0 / 1 of a 64-row
            // group (z_mode 1), or rows r / r + 16 of the one tile, i.e. hh / hh + EPT / 2 (z_mode 2)
            auto inv_of = [&](int j, int row) {
                float t = 0.0f;
#pragma unroll
                for (int w = 0; w < NW; ++w) t += ssq_lds[w][j][row];
                return 1.0f / sqrtf(t / (float)(KB * 16) + a.eps);
            };
            constexpr int HP = MT == 2 ? EPT : EPT / 2;   // positions per thread and column block
#pragma unroll
            for (int hp = 0; hp < HP; ++hp) {
                const int v = wave + NW * hp;
                const int row = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                const int jc = 0, ju = MT == 2 ? 1 : 0, hc = hp, hu = MT == 2 ? hp : hp + EPT / 2;
                const int row_u = MT == 2 ? row : row + 16;
                const int mc = m_base + row, mu = MT == 2 ? m_base + 32 + row : m_base + row_u;
                if (mu >= a.M) continue;
                const float inv_c = inv_of(jc, row), inv_u = inv_of(ju, row_u);
                const int pos = MT == 2 ? mg * 32 + row : row;
#pragma unroll
                for (int i = 0; i < NBW; ++i) {
                    const int n = (blk0 + i) * 32 + col;
                    if (n >= a.N) continue;
                    a.z_out[(size_t)pos * a.N + n] = guided_z(out[jc][i][hc], inv_c, out[ju][i][hu], inv_u, a.cfg_scale, a.inv_t);
                    if (a.logits) {
                        a.logits[(size_t)mc * a.N + n] = out[jc][i][hc] * inv_c;
                        a.logits[(size_t)mu * a.N + n] = out[ju][i][hu] * inv_u;
                    }
                }
            }
            return;
        }
    }
#pragma unroll
    for (int j = 0; j < MT; ++j)
#pragma unroll
        for (int hh = 0; hh < EPT; ++hh) {
            const int v = wave + NW * hh;
            const int row = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            const int m = m_base + j * 32 + row;
            if (m >= a.M || (SPLIT && (row >> 4) != half)) continue;
            float inv = 1.0f;
            if (kNorm) {
                float t = 0.0f;
#pragma unroll
                for (int w = 0; w < NW; ++w) t += ssq_lds[w][j][row];
                inv = 1.0f / sqrtf(t / (float)(KB * 16) + a.eps);
            }
            float vals[NBW], xin[NBW];
#pragma unroll
            for (int i = 0; i < NBW; ++i) {
                vals[i] = out[j][i][hh];
                xin[i] = EPI == EPI_RESID ? xpre[j][i][hh] : 0.0f;
            }
            if constexpr (EPI == EPI_QKV) qkv_store(a, qrow[j][hh], g, col, vals[0] * inv, vals[NBW - 1] * inv, rot_c[j][hh], rot_s[j][hh]);
            else skinny_epilogue<EPI, NBW>(a, ks, m, blk0, col, vals, inv, xin);
        }
}

// Embedding gather for the fused path: fp32 residual stream + its bf16 fragment-major copy.  The block of row m
// also writes the row's entry of the tables that every QKV projection of this forward reads: destination offsets
// (sequence segment, window index, KV page of the position) and the rotary (cos, sin) of the position.
struct RowTables {
    const int32_t *row_pos;
    const float *rope_cos, *rope_sin;   // [max_ctx][hd / 2]
    const int32_t *page_table;
    int pages_per_seg, page_tokens, L, H, hd;
    QkvRow *meta;
    float2 *rot;
    float *ssq_part;   // [M][ssq_n] sum of squares of the row in slot 0, zeros in the others (may be NULL)
    int ssq_n;
};
__global__ void embed_dual_kernel(const bf16_t *__restrict__ emb, const int32_t *__restrict__ row_tok, float *__restrict__ x,
                                  bf16_t *__restrict__ xb, int d, RowTables t) {
    const int m = blockIdx.x;
    const int tok = row_tok[m];
    const int half = t.hd >> 1;
    const int pos = tok >= 0 ? t.row_pos[m] : -1;
    if (threadIdx.x == 0) {
        QkvRow r;
        r.pos = pos; r.q_off = 0; r.page = 0; r.k_off = 0; r.v_off = 0;
        if (pos >= 0) {
            const int seg = m / t.L, i_win = m % t.L;
            r.q_off = seg * t.H * (int)Layout<bf16_t>::q_elems(t.L, t.hd) + (int)Layout<bf16_t>::q_index(i_win, 0, t.hd);
            r.page = t.page_table[seg * t.pages_per_seg + pos / t.page_tokens];
            const int tk = pos % t.page_tokens;
            r.k_off = (int)Layout<bf16_t>::k_index(tk, 0, t.hd);
            r.v_off = (int)Layout<bf16_t>::v_index(tk, 0, t.hd);
        }
        t.meta[m] = r;
    }
    for (int j = threadIdx.x; j < half; j += blockDim.x)
        t.rot[(size_t)m * half + j] = pos >= 0 ? make_float2(t.rope_cos[(size_t)pos * half + j], t.rope_sin[(size_t)pos * half + j])
                                               : make_float2(1.0f, 0.0f);
    float sq = 0.0f;
    for (int i = threadIdx.x; i < d; i += blockDim.x) {
        const bf16_t v = tok >= 0 ? emb[(size_t)tok * d + i] : (bf16_t)0;
        const float f = bf16_to_float(v);
        x[(size_t)m * d + i] = f;
        xb[Layout<bf16_t>::a_index(m, i, d)] = v;
        sq = fmaf(f, f, sq);
    }
    if (t.ssq_part) {
        __shared__ float scratch[17];
        const float total = block_sum_f32(sq, scratch);
        for (int c = threadIdx.x; c < t.ssq_n; c += blockDim.x) t.ssq_part[(size_t)m * t.ssq_n + c] = c == 0 ? total : 0.0f;
    }
}

// Weight re-layout for the fused path.  dst block (group * nbw + i) of 32 rows <- source rows given by
// `map`: src_row = map(dst_row); gain (may be NULL) is multiplied into column k.
struct PackMap {
    int mode;     // 0 identity, 1 = QKV head/pair order, 2 = gate/up interleave
    int hd, F;    // mode 1: head dimension; mode 2: rows of the gate matrix
};
SJD_HD int packmap_src_row(const PackMap &pm, int dst_row) {
    if (pm.mode == 1) {  // groups of 64 rows: head = grp / pairs, sub = grp % pairs; tile i -> block sub + i * pairs
        const int pairs = pm.hd >> 6, grp = dst_row >> 6, i = (dst_row >> 5) & 1, c = dst_row & 31;
        const int head = grp / pairs, sub = grp % pairs;
        return head * pm.hd + (sub + i * pairs) * 32 + c;
    }
    if (pm.mode == 2) {  // groups of 64 rows: 32 gate rows then the 32 up rows of the same columns
        const int grp = dst_row >> 6, i = (dst_row >> 5) & 1, c = dst_row & 31;
        return i * pm.F + grp * 32 + c;
    }
    return dst_row;
}

// src: logical [N][K] matrix given as up to 3 row-major pieces stacked by rows (n0, n1 = end rows of piece 0, 1)
__global__ void pack_weight_fused_kernel(const bf16_t *__restrict__ s0, const bf16_t *__restrict__ s1, const bf16_t *__restrict__ s2,
                                         int n0, int n1, const float *__restrict__ gain, bf16_t *__restrict__ dst, int N, int K,
                                         PackMap pm) {
    const size_t total = (size_t)N * K;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int nd = (int)(idx / K), k = (int)(idx % K);
        const int ns = packmap_src_row(pm, nd);
        if (ns >= N) continue;  // rows beyond the matrix stay zero
        const bf16_t *src = ns < n0 ? s0 + (size_t)ns * K : (ns < n1 ? s1 + (size_t)(ns - n0) * K : s2 + (size_t)(ns - n1) * K);
        float v = bf16_to_float(src[k]);
        if (gain) v *= gain[k];
        dst[Layout<bf16_t>::w_index(nd, k, K)] = float_to_bf16(v);
    }
}

// x[m][n] += sum_ks part[ks][m][n];  xb = bf16(x) in GEMM-operand layout.
// One wavefront per (row, 256 columns): a lane takes four consecutive columns (16-byte loads of the stream and of every
// partial sum, one 8-byte store of the four bf16, which are neighbours in the operand layout), and the chunk's sum of
// squares is a wavefront reduction: no barrier.  grid (ceil(N / 1024), M), 256 threads.
// ssq_part (may be NULL): [M][ceil(N / 256)] sums of squares of the bf16 values written per chunk.
__global__ __launch_bounds__(256) void resid_reduce_kernel(const float *__restrict__ part, int ksplit, int M, int N, float *__restrict__ x,
                                                           bf16_t *__restrict__ xb, float *__restrict__ ssq_part) {
    const int m = blockIdx.y, chunk = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int n_chunks = (N + 255) >> 8, n = chunk * 256 + lane * 4;
    float sq = 0.0f;
    if ((N & 3) == 0 && n + 3 < N) {
        const size_t idx = (size_t)m * N + n;
        float4 v = *reinterpret_cast<const float4 *>(x + idx);
        for (int k = 0; k < ksplit; ++k) {
            const float4 p = *reinterpret_cast<const float4 *>(part + (size_t)k * M * N + idx);
            v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
        }
        *reinterpret_cast<float4 *>(x + idx) = v;
        const bf16_t b0 = float_to_bf16(v.x), b1 = float_to_bf16(v.y), b2 = float_to_bf16(v.z), b3 = float_to_bf16(v.w);
        uint2 packed;
        packed.x = (uint32_t)b0 | ((uint32_t)b1 << 16);
        packed.y = (uint32_t)b2 | ((uint32_t)b3 << 16);
        *reinterpret_cast<uint2 *>(xb + Layout<bf16_t>::a_index(m, n, N)) = packed;   // n % 4 == 0: one 8-element group
        const float f0 = bf16_to_float(b0), f1 = bf16_to_float(b1), f2 = bf16_to_float(b2), f3 = bf16_to_float(b3);
        sq = (f0 * f0 + f1 * f1) + (f2 * f2 + f3 * f3);
    } else {
        for (int nn = n; nn < n + 4 && nn < N; ++nn) {
            const size_t idx = (size_t)m * N + nn;
            float v = x[idx];
            for (int k = 0; k < ksplit; ++k) v += part[(size_t)k * M * N + idx];
            x[idx] = v;
            const bf16_t b = float_to_bf16(v);
            xb[Layout<bf16_t>::a_index(m, nn, N)] = b;
            sq += bf16_to_float(b) * bf16_to_float(b);
        }
    }
    if (ssq_part) {
        for (int off = 32; off > 0; off >>= 1) sq += __shfl_xor(sq, off, 64);
        if (lane == 0 && chunk < n_chunks) ssq_part[(size_t)m * n_chunks + chunk] = sq;
    }
}

template <int EPI, int NW>
inline hipError_t launch_skinny_nw(hipStream_t st, const SkinnyArgs &a_in, int MT, int groups, int nbw) {
    constexpr int DEPTH = SJD_SKINNY_DEPTH;
    SkinnyArgs a = a_in;
    a.groups = groups;
    if (a.ksplit != 1) a.pf_wgs = a.kv_wgs = 0;
    if (a.row_split == 2 && (MT != 1 || a.m_groups > 1 || a.ksplit != 1 || EPI == EPI_PARTIAL)) return hipErrorInvalidValue;
    const int n_compute = a.row_split == 2 ? 16 * ((groups + 7) / 8) : a.m_groups > 1 ? 8 * ((groups + 7) / 8) * a.m_groups : groups;
    const dim3 grid(n_compute + a.pf_wgs + a.kv_wgs, a.ksplit);
    constexpr bool kPair = EPI == EPI_QKV || EPI == EPI_SWIGLU;  // epilogues that need two column blocks
    if (nbw == 2) {
        if (MT == 1 && a.row_split == 2) gemm_skinny_kernel<1, 2, NW, DEPTH, EPI, true><<<grid, NW * 64, 0, st>>>(a);
        else if (MT == 1) gemm_skinny_kernel<1, 2, NW, DEPTH, EPI><<<grid, NW * 64, 0, st>>>(a);
        else gemm_skinny_kernel<2, 2, NW, DEPTH, EPI><<<grid, NW * 64, 0, st>>>(a);
    } else {
        if (kPair) return hipErrorInvalidValue;
        constexpr int E1 = kPair ? EPI_RESID : EPI;
        if (MT == 1 && a.row_split == 2) gemm_skinny_kernel<1, 1, NW, DEPTH, E1, true><<<grid, NW * 64, 0, st>>>(a);
        else if (MT == 1) gemm_skinny_kernel<1, 1, NW, DEPTH, E1><<<grid, NW * 64, 0, st>>>(a);
        else gemm_skinny_kernel<2, 1, NW, DEPTH, E1><<<grid, NW * 64, 0, st>>>(a);
    }
    return hipGetLastError();
}

// More column groups (of two blocks) than CUs, one row group, whole K, 4 wavefronts: one workgroup per CU (up to twice as
// many groups as CUs), the first groups - CUs of them two groups wide; beyond that every workgroup is two groups wide.
inline bool skinny_mixed_applies(const SkinnyArgs &a, int groups, int nbw, int nw) {
    return groups > a.n_cus && nbw == 2 && nw == 4 && a.m_groups <= 1 && a.ksplit == 1 && a.row_split != 2;
}
template <int EPI>
inline hipError_t launch_skinny_mixed(hipStream_t st, const SkinnyArgs &a_in, int MT, int groups) {
    constexpr int DEPTH = SJD_SKINNY_DEPTH;
    SkinnyArgs a = a_in;
    if (!skinny_mixed_applies(a, groups, 2, 4) || MT < 1 || MT > 2) return hipErrorInvalidValue;
    a.groups = groups;
    a.pf_wgs = a.kv_wgs = 0;
    a.n_heavy = std::min(groups / 2, groups - a.n_cus);
    const int light = groups - 2 * a.n_heavy;
    if (MT == 1) gemm_skinny_mixed_kernel<1, 4, DEPTH, EPI><<<a.n_heavy + light, 256, 0, st>>>(a);
    else gemm_skinny_mixed_kernel<2, 4, DEPTH, EPI><<<a.n_heavy + light, 256, 0, st>>>(a);
    return hipGetLastError();
}

// nw = wavefronts per workgroup (4 or 8), the caller's choice.
template <int EPI>
inline hipError_t launch_skinny(hipStream_t st, const SkinnyArgs &a, int MT, int groups, int nbw, int nw = 8) {
    return nw == 4 ? launch_skinny_nw<EPI, 4>(st, a, MT, groups, nbw) : launch_skinny_nw<EPI, 8>(st, a, MT, groups, nbw);
}
