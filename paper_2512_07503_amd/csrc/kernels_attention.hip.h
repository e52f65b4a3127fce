// Window attention: the L queries of a (sequence, branch) attend to the committed cache positions
// [0, kv) and, causally, to the window positions kv .. kv + i (Sec. 4.1 Step 2: the parallel forward over
// the window is causal).  Keys and values live in pages addressed through a page table.
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

// ------------------------------------------------------------------------------------ MFMA, bf16
// Flash-decoding over the paged cache.  A wavefront owns one (segment, query head, chunk of `chunk`
// tokens, tile of 32 window rows); windows longer than 32 are covered by several query tiles.  Per block of 32
// tokens:
//   S^T (tokens x queries) = K (A operand, fragment-major page) x Q^T (B operand)       hd / 16 MFMAs
//   online softmax per query = per accumulator column: in-lane over 16 values + one cross-half shuffle
//   O^T (dims x queries)  += V^T (A operand) x P^T (B operand)                            2 hd / 32 MFMAs
// P^T needs no data movement: accumulator registers 8 i .. 8 i + 7 of S^T, rounded to bf16, ARE the B
// operand of the i-th PV MFMA, because the value pages are stored in the matching token order
// (Layout<bf16_t>::v_index).  Keys and values stream from HBM exactly once per (segment, kv head):
// the G query heads of a kv head run as G wavefronts of one workgroup and share the fetches in L1/L2.
// Chunks are merged by attention_combine_kernel.
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 hw_bf16x2_t __attribute__((ext_vector_type(2)));

struct AttnArgs {
    const bf16_t *q;       // [segments][H][q_elems(L, hd)]
    KvPool pool;
    const int32_t *row_tok;  // [segments * L]
    const int32_t *seg_kv;   // cached positions per segment
    const int32_t *seg_n;    // active window rows per segment
    float *part_o;           // [segments * H * n_qt * n_chunks][32][hd]
    float *part_ml;          // [segments * H * n_qt * n_chunks][2][32]  (running max, running sum)
    bf16_t *out_act;         // [M][H * hd] GEMM-operand layout
    float *out_plain;        // optional [M][H][hd]
    int L, H, Hkv, hd, chunk, n_chunks;
    int n_qt;                // query tiles of 32 window rows = ceil(L / 32)
    float scale_log2e;       // 1 / sqrt(hd) * log2(e)
};

// One wavefront's pass over the 32-token blocks t_begin, t_begin + t_stride, ... < t_end of (segment seg, query
// head h, query tile qt): leaves the unnormalised O^T in o, the running maximum (base-2 logits) in m_run and this
// lane's half of the running sum in l_run; window row = 32 qt + lane % 32.
template <int HD, int D>
SJD_D void attention_wave(const AttnArgs &a, int seg, int h, int kvh, int qt, int t_begin, int t_end, int t_stride, int kv, int n_tot, int lane,
                          f32x16 (&o)[HD / 32], float &m_run, float &l_run) {
    constexpr int KF = HD / 16, DB = HD / 32;
    const u32x4 *qp = reinterpret_cast<const u32x4 *>(a.q + ((size_t)seg * a.H + h) * Layout<bf16_t>::q_elems(a.L, HD)) +
                      (size_t)qt * KF * 64 + lane;
    u32x4 qf[KF];
#pragma unroll
    for (int kb = 0; kb < KF; ++kb) qf[kb] = qp[kb * 64];

    const int32_t *pt = a.pool.page_table + (size_t)seg * a.pool.pages_per_seg;
    const int ptok = a.pool.page_tokens;
    const size_t blk = (size_t)ptok * HD;  // elements of one (page, kv head) block
    auto kfrag = [&](int t0) {            // first fragment of the 32-token block starting at t0
        return reinterpret_cast<const u32x4 *>((const bf16_t *)a.pool.k + ((size_t)pt[t0 / ptok] * a.Hkv + kvh) * blk) +
               (size_t)((t0 % ptok) >> 5) * KF * 64 + lane;
    };
    auto vfrag = [&](int t0) {
        return reinterpret_cast<const u32x4 *>((const bf16_t *)a.pool.v + ((size_t)pt[t0 / ptok] * a.Hkv + kvh) * blk) +
               (size_t)((t0 % ptok) >> 5) * 2 * DB * 64 + lane;
    };

#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = 0.0f;
    m_run = -INFINITY;
    l_run = 0.0f;
    if (t_begin >= t_end) return;
    const int query = 32 * qt + (lane & 31);
    const int last_vis = kv + query < n_tot - 1 ? kv + query : n_tot - 1;  // last token this lane's query sees

    // Ring of D blocks of keys and values in flight (32 registers per slot at HD = 64, 64 at HD = 128): a wavefront
    // with at most D blocks (short contexts split over the wavefronts of a workgroup) requests all of them at once
    // and pays the memory latency once.
    u32x4 kf[D][KF], vf[D][2 * DB];
    const int n_blk = (t_end - t_begin + t_stride - 1) / t_stride;
    auto load_k = [&](int s, int b) {
        const u32x4 *kp = kfrag(t_begin + b * t_stride);
#pragma unroll
        for (int kb = 0; kb < KF; ++kb) kf[s][kb] = kp[kb * 64];
    };
    auto load_v = [&](int s, int b) {
        const u32x4 *vp = vfrag(t_begin + b * t_stride);
#pragma unroll
        for (int f = 0; f < 2 * DB; ++f) vf[s][f] = vp[f * 64];
    };
    // one block: scores, online softmax, O += V P; `next` >= 0: block to request into the slot as soon as its
    // keys (after the scores) and values (after the PV product) have been consumed
    auto block = [&](int s, int b, int next) {
        const int t0 = t_begin + b * t_stride;
        f32x16 sc;
#pragma unroll
        for (int v = 0; v < 16; ++v) sc[v] = 0.0f;
#pragma unroll
        for (int kb = 0; kb < KF; ++kb)
            sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[s][kb]), __builtin_bit_cast(bf16x8, qf[kb]), sc, 0, 0, 0);
        if (next >= 0) load_k(s, next);
        __builtin_amdgcn_sched_barrier(0);
        // The softmax arithmetic below is what bounds a short-context workgroup (all of a head's blocks run on one
        // CU), so it is kept lean and branch-free: one compare per score for the causal / length mask, raw
        // v_exp_f32 (arguments <= 0; results below 2^-126 may flush to 0), hardware pair conversion to bf16 (round
        // to nearest even).
        {
            const int tb = t0 + 4 * (lane >> 5) - last_vis;  // token of accumulator register v is visible iff tb + 8 (v / 4) + v % 4 <= 0
#pragma unroll
            for (int v = 0; v < 16; ++v) sc[v] = tb <= -(8 * (v >> 2) + (v & 3)) ? sc[v] : -INFINITY;
        }
        float mx = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sc[v]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * a.scale_log2e;  // base-2 logits from here on
        const float m_new = fmaxf(m_run, mx);
        // a query with nothing visible so far keeps m = -inf; avoid (-inf) - (-inf)
        const float m_use = m_new == -INFINITY ? 0.0f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
        float psum = 0.0f;
        uint32_t pk[8];
#pragma unroll
        for (int v = 0; v < 16; v += 2) {
            const f32x2_t pp = {__builtin_amdgcn_exp2f(fmaf(sc[v], a.scale_log2e, -m_use)),
                                __builtin_amdgcn_exp2f(fmaf(sc[v + 1], a.scale_log2e, -m_use))};
            const uint32_t u = __builtin_bit_cast(uint32_t, __builtin_convertvector(pp, hw_bf16x2_t));
            // the sum of what is actually multiplied
            psum += __builtin_bit_cast(float, u << 16) + __builtin_bit_cast(float, u & 0xFFFF0000u);
            pk[v >> 1] = u;
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
        const u32x4 p0 = {pk[0], pk[1], pk[2], pk[3]}, p1 = {pk[4], pk[5], pk[6], pk[7]};
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[s][db]), __builtin_bit_cast(bf16x8, p0), o[db], 0, 0, 0);
            o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[s][DB + db]), __builtin_bit_cast(bf16x8, p1), o[db], 0, 0, 0);
        }
        if (next >= 0) load_v(s, next);
        __builtin_amdgcn_sched_barrier(0);
    };
#pragma unroll
    for (int s = 0; s < D; ++s)
        if (s < n_blk) {
            load_k(s, s);
            load_v(s, s);
        }
    __builtin_amdgcn_sched_barrier(0);
    int b0 = 0;
    for (; b0 + 2 * D <= n_blk; b0 += D) {  // every refill of these groups is a block that exists: branch-free body
#pragma unroll
        for (int s = 0; s < D; ++s) block(s, b0 + s, b0 + s + D);
    }
#pragma unroll
    for (int s = 0; s < D; ++s)
        if (b0 + s < n_blk) block(s, b0 + s, b0 + s + D < n_blk ? b0 + s + D : -1);
#pragma unroll
    for (int s = 0; s < D; ++s)
        if (b0 + D + s < n_blk) block(s, b0 + D + s, -1);
}

template <int HD>
__global__ __launch_bounds__(256) void attention_mfma_kernel(AttnArgs a) {
    constexpr int DB = HD / 32;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int G = a.H / a.Hkv;
    const int c = blockIdx.x, kvh = blockIdx.y, seg = blockIdx.z / a.n_qt, qt = blockIdx.z % a.n_qt;
    const int h = kvh * G + wave;
    const int n_act = a.seg_n[seg];
    const int kv = a.seg_kv[seg];
    const int n_tot = n_act > 0 ? kv + n_act : 0;
    const int n_vis = min(n_tot, kv + 32 * (qt + 1));  // nothing later is visible to this query tile
    const int t_begin = c * a.chunk;
    if (t_begin >= n_vis || 32 * qt >= n_act) return;
    const int t_end = t_begin + a.chunk < n_vis ? t_begin + a.chunk : n_vis;
    f32x16 o[DB];
    float m_run, l_run;
    attention_wave<HD, (HD <= 64 ? 3 : 2)>(a, seg, h, kvh, qt, t_begin, t_end, 32, kv, n_tot, lane, o, m_run, l_run);
    const int query = lane & 31;
    l_run += __shfl_xor(l_run, 32, 64);
    const size_t slot = (((size_t)seg * a.H + h) * a.n_qt + qt) * a.n_chunks + c;
    float *po = a.part_o + slot * 32 * HD + (size_t)query * HD;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) po[db * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)] = o[db][v];
    if (lane < 32) {
        a.part_ml[slot * 64 + query] = m_run;
        a.part_ml[slot * 64 + 32 + query] = l_run;
    }
}

// Short contexts (keys + values of one head within a few hundred KB): one workgroup per (segment, query head) does
// the whole softmax.  Its NS wavefronts take the 32-token blocks round-robin, then merge through LDS:
// out = sum_w 2^(m_w - m) O_w / sum_w 2^(m_w - m) l_w, written straight into the next GEMM's operand layout.
// No partial results go to HBM and no second kernel is launched.
template <int HD, int NS>
__global__ __launch_bounds__(NS * 64) void attention_onepass_kernel(AttnArgs a) {
    constexpr int DB = HD / 32, EPT = 16 / NS;
    static_assert(16 % NS == 0, "NS must divide 16");
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int h = blockIdx.x, seg = blockIdx.y, qt = blockIdx.z;
    const int kvh = h / (a.H / a.Hkv);
    const int n_act = a.seg_n[seg];
    const int kv = a.seg_kv[seg];
    const int n_tot = n_act > 0 ? kv + n_act : 0;
    const int n_vis = 32 * qt < n_act ? min(n_tot, kv + 32 * (qt + 1)) : 0;  // nothing later is visible to this query tile
    f32x16 o[DB];
    float m_run, l_run;
    attention_wave<HD, (HD <= 64 ? 3 : 1)>(a, seg, h, kvh, qt, 32 * wave, n_vis, 32 * NS, kv, n_tot, lane, o, m_run, l_run);
    const int query = lane & 31;
    l_run += __shfl_xor(l_run, 32, 64);

    __shared__ float ml[NS][2][32];
    __shared__ float red[NS][16][64];
    if (lane < 32) {
        ml[wave][0][query] = m_run;
        ml[wave][1][query] = l_run;
    }
    __syncthreads();
    float m_all = -INFINITY;
#pragma unroll
    for (int w = 0; w < NS; ++w) m_all = fmaxf(m_all, ml[w][0][query]);
    const float m_use = m_all == -INFINITY ? 0.0f : m_all;
    float denom = 0.0f;
#pragma unroll
    for (int w = 0; w < NS; ++w) denom += exp2f(ml[w][0][query] - m_use) * ml[w][1][query];
    const float scale = exp2f(m_run - m_use);  // 0 for a wavefront that saw nothing
    const int m = seg * a.L + 32 * qt + query;
    const bool row = 32 * qt + query < a.L;
    const bool active = row && a.row_tok[m] >= 0 && denom > 0.0f;
    const float inv = active ? 1.0f / denom : 0.0f;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
        __syncthreads();
#pragma unroll
        for (int v = 0; v < 16; ++v) red[wave][v][lane] = o[db][v] * scale;
        __syncthreads();
#pragma unroll
        for (int hh = 0; hh < EPT; ++hh) {
            const int v = wave + NS * hh;
            float t = 0.0f;
#pragma unroll
            for (int w = 0; w < NS; ++w) t += red[w][v][lane];
            t = active ? t * inv : 0.0f;  // 0 * inf (an idle row's garbage) must not become NaN
            const int j = db * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            if (row) {
                if (a.out_act) a.out_act[Layout<bf16_t>::a_index(m, h * HD + j, a.H * HD)] = float_to_bf16(t);
                if (a.out_plain) a.out_plain[((size_t)m * a.H + h) * HD + j] = t;
            }
        }
    }
}

// Merges the chunks of every (row, head): out = sum_c 2^(m_c - m) O_c / sum_c 2^(m_c - m) l_c.
// Workgroup = one wavefront on 8 window rows of one (segment, head, query tile): lane = (row, eighth of the head
// dimensions).  The chunk loops carry no dependence from one load to the next (the maximum first, then the
// weights), so the partial results of all chunks are in flight together.
template <int HD>
__global__ __launch_bounds__(64) void attention_combine_kernel(AttnArgs a) {
    constexpr int DPT = HD / 8;  // head dimensions per lane
    const int rq = blockIdx.x & 3, pair = blockIdx.x >> 2;
    const int qt = pair % a.n_qt, sh = pair / a.n_qt, h = sh % a.H, seg = sh / a.H;
    const int iq = rq * 8 + (threadIdx.x >> 3), dg = threadIdx.x & 7;
    const int i_win = 32 * qt + iq;
    if (i_win >= a.L) return;
    const int m = seg * a.L + i_win;
    const bool active = a.row_tok[m] >= 0;
    const int kv = a.seg_kv[seg];
    const int n_vis = min(kv + a.seg_n[seg], kv + 32 * (qt + 1));  // the chunks this row's query tile went through
    const int nc = active ? (n_vis + a.chunk - 1) / a.chunk : 0;
    const size_t slot0 = (size_t)pair * a.n_chunks;
    const float *ml = a.part_ml + slot0 * 64 + iq;
    float mx = -INFINITY;
#pragma unroll 4
    for (int c = 0; c < nc; ++c) mx = fmaxf(mx, ml[(size_t)c * 64]);
    float denom = 0.0f;
    float acc[DPT];
#pragma unroll
    for (int d = 0; d < DPT; ++d) acc[d] = 0.0f;
    const float *po = a.part_o + slot0 * 32 * HD + (size_t)iq * HD + dg * DPT;
#pragma unroll 4
    for (int c = 0; c < nc; ++c) {
        const float w = exp2f(ml[(size_t)c * 64] - mx);
        denom = fmaf(w, ml[(size_t)c * 64 + 32], denom);
        const float4 *p4 = reinterpret_cast<const float4 *>(po + (size_t)c * 32 * HD);
#pragma unroll
        for (int v = 0; v < DPT / 4; ++v) {
            const float4 x = p4[v];
            acc[4 * v] = fmaf(w, x.x, acc[4 * v]);
            acc[4 * v + 1] = fmaf(w, x.y, acc[4 * v + 1]);
            acc[4 * v + 2] = fmaf(w, x.z, acc[4 * v + 2]);
            acc[4 * v + 3] = fmaf(w, x.w, acc[4 * v + 3]);
        }
    }
    const float inv = nc > 0 && denom > 0.0f ? 1.0f / denom : 0.0f;
#pragma unroll
    for (int d = 0; d < DPT; ++d) {
        const int j = dg * DPT + d;
        const float v = acc[d] * inv;
        if (a.out_act) a.out_act[Layout<bf16_t>::a_index(m, h * HD + j, a.H * HD)] = float_to_bf16(v);
        if (a.out_plain) a.out_plain[((size_t)m * a.H + h) * HD + j] = v;
    }
}

inline bool attention_mfma_supported(int L, int H, int Hkv, int hd, int page_tokens) {
    return L >= 1 && (hd == 64 || hd == 128) && H / Hkv <= 4 && page_tokens % 32 == 0;
}

// One workgroup per (segment, head), no partial results and no merge launch, against chunks of the context spread
// over more workgroups: the single launch wins whenever its workgroups alone fill the chip (`pairs` = segments x
// heads from half the CU count on), and otherwise while a head's keys and values are a stream of up to 1.25 MiB for
// its CU (2 560 tokens of 128-wide heads).  Measured along whole images of the 7B shapes, per layer: 64 pairs,
// 32 kv heads: 11.0 against 19.5 us at 300 tokens, 30.7 against 32.8 at 2 400; 64 pairs, 8 kv heads: 10.0 against
// 22.6 at 300, 24.7 against 29.2 at 2 100, 32.4 against 30.7 at 3 100, 39.9 against 32.6 at 4 100; 512 pairs: 25.6
// against 34.4 at 300, 119 against 141 at 2 400.
inline bool attention_onepass_pays(int max_tokens, int hd, int pairs = 0, int n_cus = 256) {
    return 2 * pairs >= n_cus || (size_t)max_tokens * hd * 4 <= 1280 * 1024;
}

// n_segments segments of L rows each.  onepass: contexts short enough for one workgroup per (segment, head).
inline hipError_t launch_attention_mfma(hipStream_t st, const AttnArgs &a, int n_segments, bool onepass = false) {
    if (onepass) {
        const dim3 grid(a.H, n_segments, a.n_qt);
        if (a.hd == 64) attention_onepass_kernel<64, 8><<<grid, 512, 0, st>>>(a);
        else attention_onepass_kernel<128, 8><<<grid, 512, 0, st>>>(a);
        return hipGetLastError();
    }
    dim3 grid(a.n_chunks, a.Hkv, n_segments * a.n_qt);
    const int G = a.H / a.Hkv;
    if (a.hd == 64) attention_mfma_kernel<64><<<grid, G * 64, 0, st>>>(a);
    else attention_mfma_kernel<128><<<grid, G * 64, 0, st>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int combine_wgs = n_segments * a.H * a.n_qt * 4;
    if (a.hd == 64) attention_combine_kernel<64><<<combine_wgs, 64, 0, st>>>(a);
    else attention_combine_kernel<128><<<combine_wgs, 64, 0, st>>>(a);
    return hipGetLastError();
}
