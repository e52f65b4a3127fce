// Decision stage of one speculative Jacobi iteration (Sec. 4.1 of the paper, Steps 3 and 4) and the
// sampling distribution it works on (Sec. 3.1 top-K sampling, Sec. 5.1 guidance weight and threshold).
//
// Every result of this file is specified bit for bit as a function of the fp32 logits:
//   z      = fma(cfg_scale, l_c - l_u, l_u) * (1 / temperature)              in fp32
//   kept   = { v : z_v >= K-th largest z }   (ties kept)
//   e_v    = EXP(z_v - max z) for kept v, else 0; EXP is the fixed fp32 operation sequence below
//   w_v    = trunc(e_v * 2^40) as uint64,  Z = sum_v w_v                      probability = w / Z
//   accept (Eq. 2)   r * Q < P          with r = (u32 + 1/2) 2^-32, P = (double)w_p / (double)Z_p
//   keep   (Eq. 4-5) P > (double)tau * Q
//   draw   from p    first v with prefix_w(v) > floor(u64 * Z / 2^64)
//   draw   (Eq. 3)   same over rho_v = trunc(max(0, P_v - Q_v) * 2^44); if all rho are 0, from p
// Uniform numbers are Philox4x32-10 (Salmon et al., SC'11) with key = seed and counter
// (step, row, sequence, 0): word 0 = acceptance test of the draft verified at `row`, words 1-2 = the
// 64-bit uniform of the one draw made at `row`, word 3 = a fresh uniform draft.
//
// This translation unit must be compiled with -ffp-contract=off.
#include <type_traits>
#include "decide.h"

#include "common.hip.h"

#pragma clang fp contract(off)

namespace {

// ------------------------------------------------------------------------------------ primitives
SJD_D void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1, uint32_t out[4]) {
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

SJD_D void draw_words(uint64_t seed, uint32_t step, uint32_t row, uint32_t seq, uint32_t out[4]) {
    philox4x32_10(step, row, seq, 0u, (uint32_t)seed, (uint32_t)(seed >> 32), out);
}

// EXP(x), x <= 0: k = rint(x log2 e), r = x - k ln2 (two-constant split), degree-6 Taylor polynomial
// by Horner with fused multiply-adds, times 2^k built in the exponent field; 0 below -60.
SJD_D float exp_neg(float x) {
    if (x < -60.0f) return 0.0f;
    float kf = __builtin_rintf(x * 0x1.715476p+0f);
    float r = __builtin_fmaf(kf, -0x1.62ep-1f, x);
    r = __builtin_fmaf(kf, -0x1.0bfbe8p-15f, r);
    float p = 0x1.6c16c2p-10f;
    p = __builtin_fmaf(p, r, 0x1.111112p-7f);
    p = __builtin_fmaf(p, r, 0x1.555556p-5f);
    p = __builtin_fmaf(p, r, 0x1.555556p-3f);
    p = __builtin_fmaf(p, r, 0.5f);
    p = __builtin_fmaf(p, r, 1.0f);
    p = __builtin_fmaf(p, r, 1.0f);
    int k = (int)kf;
    float scale = __builtin_bit_cast(float, (uint32_t)(k + 127) << 23);
    return p * scale;
}

SJD_D uint64_t weight_of(float e) { return (uint64_t)(e * 0x1p40f); }

SJD_D double prob(uint64_t w, uint64_t Z) { return (double)w / (double)Z; }

SJD_D bool accept_rule(uint32_t u32, uint64_t wp, uint64_t Zp, uint64_t wq, uint64_t Zq) {
    double r = ((double)u32 + 0.5) * 0x1p-32;
    double P = prob(wp, Zp), Q = prob(wq, Zq);
    return r * Q < P;
}

SJD_D bool keep_rule(float tau, uint64_t wp, uint64_t Zp, uint64_t wq, uint64_t Zq) {
    double P = prob(wp, Zp), Q = prob(wq, Zq);
    return P > (double)tau * Q;
}

SJD_D uint64_t mulhi64(uint64_t a, uint64_t b) { return __umul64hi(a, b); }

SJD_D uint64_t residual_weight(double P, double Q) {
    double d = P - Q;
    return d > 0.0 ? (uint64_t)(d * 0x1p44) : 0ull;
}

// float -> unsigned key with the same order (-0 is folded into +0)
SJD_D uint32_t order_key(float z) {
    uint32_t b = __builtin_bit_cast(uint32_t, z);
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
SJD_D float key_to_float(uint32_t k) {
    uint32_t b = (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k;
    return __builtin_bit_cast(float, b);
}

SJD_D float guided(float lc, float lu, float s, float inv_t) {
    float d = lc - lu;
    return __builtin_fmaf(s, d, lu) * inv_t;
}

// --------------------------------------------------------------------------- block-wide helpers
SJD_D uint64_t shfl_down_u64(uint64_t v, int delta) {
    uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    lo = __shfl_down(lo, delta, 64);
    hi = __shfl_down(hi, delta, 64);
    return ((uint64_t)hi << 32) | lo;
}

// sum of one uint64 per thread over the block (integer: order does not matter); result in all threads
SJD_D uint64_t block_sum_u64(uint64_t v, uint64_t *scratch /* >= 17 entries */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    for (int d = 32; d > 0; d >>= 1) v += shfl_down_u64(v, d);
    __syncthreads();
    if (lane == 0) scratch[wave] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint64_t t = 0;
        for (int i = 0; i < nw; ++i) t += scratch[i];
        scratch[16] = t;
    }
    __syncthreads();
    return scratch[16];
}

SJD_D uint32_t block_max_u32(uint32_t v, uint32_t *scratch /* >= 17 */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    for (int d = 32; d > 0; d >>= 1) {
        uint32_t o = __shfl_down(v, d, 64);
        v = o > v ? o : v;
    }
    __syncthreads();
    if (lane == 0) scratch[wave] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = 0;
        for (int i = 0; i < nw; ++i) t = scratch[i] > t ? scratch[i] : t;
        scratch[16] = t;
    }
    __syncthreads();
    return scratch[16];
}

// ------------------------------------------------------------------ a10: the sampling distribution
// One block per row.  Radix select (4 passes of 8 bits over order keys) finds the K-th largest guided
// logit exactly; the logits are re-read from L2 in every pass.
struct SampleRowsArgs {
    const float *lc_base, *lu_base;  // row r = (s, k): base + s * seq_stride + k * V
    long seq_stride;
    int L;                           // rows per sequence
    float *e_base[2];                // + (s * L + k) * V; index = *step & 1 (0 when step == NULL)
    uint64_t *Z_base[2];             // + s * L + k
    const uint32_t *step;
    const int32_t *Le;               // [S] active rows per sequence, NULL = all
    int V, top_k;
    float cfg_scale, inv_t;
};

__global__ void sample_rows_kernel(SampleRowsArgs a) {
    const int r = blockIdx.x, s = r / a.L, k = r % a.L;
    if (a.Le && k >= a.Le[s]) return;
    const float *lc = a.lc_base + (long)s * a.seq_stride + (long)k * a.V;
    const float *lu = a.lu_base + (long)s * a.seq_stride + (long)k * a.V;
    const uint32_t par = a.step ? (*a.step & 1u) : 0u;
    float *e = a.e_base[par] + ((long)s * a.L + k) * a.V;
    const int V = a.V, tid = threadIdx.x, nt = blockDim.x;

    __shared__ uint32_t hist[256];
    __shared__ uint32_t sel[2];
    __shared__ uint32_t scratch32[17];
    __shared__ uint64_t scratch64[17];

    uint32_t kmax = 0;
    for (int v = tid; v < V; v += nt) {
        uint32_t key = order_key(guided(lc[v], lu[v], a.cfg_scale, a.inv_t));
        kmax = key > kmax ? key : kmax;
    }
    kmax = block_max_u32(kmax, scratch32);
    const float m = key_to_float(kmax);

    uint32_t thresh = 0;  // keep everything
    if (a.top_k < V) {
        uint32_t prefix = 0, mask = 0, want = (uint32_t)a.top_k;
        for (int shift = 24; shift >= 0; shift -= 8) {
            for (int i = tid; i < 256; i += nt) hist[i] = 0;
            __syncthreads();
            for (int v = tid; v < V; v += nt) {
                uint32_t key = order_key(guided(lc[v], lu[v], a.cfg_scale, a.inv_t));
                if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
            }
            __syncthreads();
            if (tid == 0) {
                uint32_t cum = 0;
                int b = 255;
                for (; b > 0; --b) {
                    if (cum + hist[b] >= want) break;
                    cum += hist[b];
                }
                sel[0] = (uint32_t)b;
                sel[1] = want - cum;  // rank wanted inside the selected bin
            }
            __syncthreads();
            prefix |= sel[0] << shift;
            mask |= 255u << shift;
            want = sel[1];
            __syncthreads();
        }
        thresh = prefix;
    }

    uint64_t zsum = 0;
    for (int v = tid; v < V; v += nt) {
        float z = guided(lc[v], lu[v], a.cfg_scale, a.inv_t);
        float ev = order_key(z) >= thresh ? exp_neg(z - m) : 0.0f;
        e[v] = ev;
        zsum += weight_of(ev);
    }
    zsum = block_sum_u64(zsum, scratch64);
    if (tid == 0) a.Z_base[par][(long)s * a.L + k] = zsum;
}

// Register-resident form for V <= 1024 * VPT: the guided logits of a row are read from HBM once and stay in
// registers (thread t holds elements t, t + 1024, ...).  The K-th largest key is found one bit at a time, most
// significant first: count the candidates whose next bit is 1; if at least `want` of them exist the K-th
// largest has that bit set, otherwise it does not and `want` drops by that count.  32 counting rounds of
// wavefront ballots and one LDS exchange each, exact; after the first 10 bits the rounds run over the compacted
// list of keys that still compete (see below).
// adds one wave-uniform count per wavefront over a block of 16 wavefronts; scratch (16-byte aligned) alternates
// between rounds.  The 16 counts come back as four 16-byte LDS reads: a round of the select is this exchange and
// little else, and a loop of 16 dependent single reads made it twice as long.
SJD_D uint32_t block_sum_wave_counts(uint32_t wave_count, uint32_t *scratch /* [16] */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) scratch[wave] = wave_count;
    __syncthreads();
    const uint4 *q = reinterpret_cast<const uint4 *>(scratch);
    const uint4 a = q[0], b = q[1], c = q[2], d = q[3];
    return ((a.x + a.y) + (a.z + a.w)) + ((b.x + b.y) + (b.z + b.w)) + ((c.x + c.y) + (c.z + c.w)) + ((d.x + d.y) + (d.z + d.w));
}

// Wall-clock stamps of block 0 for probes (compiled out of the library)
#ifdef SJD_PHASE_TIMING
__device__ unsigned long long g_sample_phase[8];
#define SJD_SAMPLE_STAMP(i) do { if (blockIdx.x == 0 && threadIdx.x == 0) g_sample_phase[i] = wall_clock64(); } while (0)
#else
#define SJD_SAMPLE_STAMP(i) do { } while (0)
#endif

template <int VPT>
__global__ __launch_bounds__(1024) void sample_rows_reg_kernel(SampleRowsArgs a) {
    const int r = blockIdx.x, s = r / a.L, k = r % a.L;
    if (a.Le && k >= a.Le[s]) return;
    const float *lc = a.lc_base + (long)s * a.seq_stride + (long)k * a.V;
    const float *lu = a.lu_base + (long)s * a.seq_stride + (long)k * a.V;
    const uint32_t par = a.step ? (*a.step & 1u) : 0u;
    float *e = a.e_base[par] + ((long)s * a.L + k) * a.V;
    const int V = a.V, tid = threadIdx.x;
    __shared__ __align__(16) uint32_t cnt[2][16];
    __shared__ __align__(16) uint32_t cnt2[16];
    __shared__ uint32_t scratch32[17];
    __shared__ uint64_t scratch64[17];

    SJD_SAMPLE_STAMP(0);
    uint32_t key[VPT];  // order key of the guided logit; 0 (below every real key) past the end of the row
    uint32_t kmax = 0;
    // The loads are unconditional (index clamped to the row) and issued in batches: a load under `if (v < V)` is
    // waited for inside its branch, and a thread would pay one memory round trip per element.
    constexpr int kBatch = VPT < 16 ? VPT : 16;
#pragma unroll
    for (int i0 = 0; i0 < VPT; i0 += kBatch) {
        float c[kBatch], u[kBatch];
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const int v = tid + (i0 + j) * 1024, vv = v < V ? v : V - 1;
            c[j] = lc[vv];
            u[j] = lu[vv];
        }
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const int i = i0 + j, v = tid + i * 1024;
            const uint32_t kk = order_key(guided(c[j], u[j], a.cfg_scale, a.inv_t));
            key[i] = v < V ? kk : 0u;
            kmax = key[i] > kmax ? key[i] : kmax;
        }
    }
    kmax = block_max_u32(kmax, scratch32);
    const float m = key_to_float(kmax);
    SJD_SAMPLE_STAMP(1);

    uint32_t thresh = 0;
    if (a.top_k < V) {
        uint32_t prefix = 0, want = (uint32_t)a.top_k;
        // one counting round over the keys in registers
        auto round_all = [&](int bit) {
            const uint32_t hi_mask = bit == 31 ? 0u : ~((2u << bit) - 1u);  // bits above `bit`
            const uint32_t probe = prefix | (1u << bit);
            uint32_t c = 0;  // wave-uniform: ballots, not shuffles
#pragma unroll
            for (int i = 0; i < VPT; ++i) c += (uint32_t)__popcll(__ballot((key[i] & (hi_mask | (1u << bit))) == probe));
            c = block_sum_wave_counts(c, cnt[bit & 1]);
            if (c >= want) prefix = probe; else want -= c;
        };
        // The top kSplitBits bits (sign, exponent, first mantissa bit) over all keys.  What still competes for the
        // K-th place afterwards are the keys that share those bits with it: usually a few percent of the row.  If
        // they fit the LDS list they are compacted (any order: the rounds only count) and the remaining rounds run
        // over at most kCandPerThread keys per thread instead of VPT; otherwise the rounds go on over all keys.
        constexpr int kSplitBits = 10, kCandPerThread = 4, kCandMax = 1024 * kCandPerThread;
        for (int bit = 31; bit > 31 - kSplitBits; --bit) round_all(bit);
        SJD_SAMPLE_STAMP(2);
        constexpr uint32_t top_mask = ~((1u << (32 - kSplitBits)) - 1u);
        __shared__ uint32_t cand[kCandMax];
        __shared__ uint32_t n_cand_lds;
        uint32_t n_cand = 0;
#pragma unroll
        for (int i = 0; i < VPT; ++i) n_cand += (uint32_t)__popcll(__ballot((key[i] & top_mask) == prefix));
        n_cand = block_sum_wave_counts(n_cand, cnt2);
        if (n_cand <= (uint32_t)kCandMax) {
            if (tid == 0) n_cand_lds = 0u;
            __syncthreads();
#pragma unroll
            for (int i = 0; i < VPT; ++i)
                if ((key[i] & top_mask) == prefix) cand[atomicAdd(&n_cand_lds, 1u)] = key[i];
            __syncthreads();
            SJD_SAMPLE_STAMP(3);
            uint32_t ck[kCandPerThread];
            bool cv[kCandPerThread];
#pragma unroll
            for (int j = 0; j < kCandPerThread; ++j) {
                cv[j] = (uint32_t)(tid + 1024 * j) < n_cand;
                ck[j] = cv[j] ? cand[tid + 1024 * j] : 0u;
            }
            for (int bit = 31 - kSplitBits; bit >= 0; --bit) {
                const uint32_t hi_mask = ~((2u << bit) - 1u);
                const uint32_t probe = prefix | (1u << bit);
                uint32_t c = 0;
#pragma unroll
                for (int j = 0; j < kCandPerThread; ++j)
                    c += (uint32_t)__popcll(__ballot(cv[j] && (ck[j] & (hi_mask | (1u << bit))) == probe));
                c = block_sum_wave_counts(c, cnt[bit & 1]);
                if (c >= want) prefix = probe; else want -= c;
            }
        } else {
            for (int bit = 31 - kSplitBits; bit >= 0; --bit) round_all(bit);
        }
        thresh = prefix;
    }
    SJD_SAMPLE_STAMP(4);

    uint64_t zsum = 0;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int v = tid + i * 1024;
        if (v < V) {
            const float z = key_to_float(key[i]);
            const float ev = key[i] >= thresh ? exp_neg(z - m) : 0.0f;
            e[v] = ev;
            zsum += weight_of(ev);
        }
    }
    SJD_SAMPLE_STAMP(5);
    zsum = block_sum_u64(zsum, scratch64);
    if (tid == 0) a.Z_base[par][(long)s * a.L + k] = zsum;
    SJD_SAMPLE_STAMP(6);
}

hipError_t launch_sample_rows_any(hipStream_t st, const SampleRowsArgs &a, int rows) {
    const int V = a.V;
    if (V <= 1024 * 4) sample_rows_reg_kernel<4><<<rows, 1024, 0, st>>>(a);
    else if (V <= 1024 * 16) sample_rows_reg_kernel<16><<<rows, 1024, 0, st>>>(a);
    else if (V <= 1024 * 32) sample_rows_reg_kernel<32><<<rows, 1024, 0, st>>>(a);
    else if (V <= 1024 * 64) sample_rows_reg_kernel<64><<<rows, 1024, 0, st>>>(a);
    else sample_rows_kernel<<<rows, 1024, 0, st>>>(a);
    return hipGetLastError();
}

// --------------------------------------------------------------------------------- window set-up
__global__ void init_window_kernel(DecideState d, uint64_t seed, int n_seqs, const int32_t *prompt_last,
                                   const int32_t *prompt_len, const int32_t *n_image) {
    const int s = blockIdx.x;
    if (s == 0 && threadIdx.x == 0) *d.step = 0u;
    if (s >= n_seqs) {
        if (threadIdx.x == 0) { d.Le[s] = 0; d.n_img[s] = 0; d.n_image[s] = 0; }
        return;
    }
    const int N = n_image[s];
    const int Le = N < d.L ? N : d.L;
    if (threadIdx.x == 0) {
        d.n_img[s] = 0;
        d.n_image[s] = N;
        d.Le[s] = Le;
        for (int b = 0; b < 2; ++b) {
            d.kv_len[s * 2 + b] = prompt_len[s * 2 + b] - 1;
            d.anchor[s * 2 + b] = prompt_last[s * 2 + b];
        }
    }
    for (int k = threadIdx.x; k < d.L; k += blockDim.x) {
        int tok = 0;
        if (k >= 1 && k < Le) {
            uint32_t w[4];
            draw_words(seed, 0u, (uint32_t)k, (uint32_t)s, w);
            tok = d.lo + (int)__umulhi(w[3], (uint32_t)d.V);
        }
        d.win_tok[s * d.L + k] = tok;
        d.ref_row[s * d.L + k] = -1;
    }
}

// Rows of the coming forward over the window; also advances the step counter.
__global__ void stage_window_kernel(DecideState d, RowMap rm, int n_seqs) {
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    if (m == 0) *d.step += 1u;
    if (m >= n_seqs * 2 * d.L) return;
    const int k = m % d.L, seg = m / d.L, s = seg >> 1;
    const int Le = d.Le[s];
    const int kv = d.kv_len[seg];
    rm.row_tok[m] = k < Le ? (k == 0 ? d.anchor[seg] : d.win_tok[s * d.L + k]) : -1;
    rm.row_pos[m] = kv + k;
    if (k == 0) { rm.seg_kv[seg] = kv; rm.seg_n[seg] = Le; }
}

// Rows of prefill chunk `chunk`: prompt positions chunk*L .. chunk*L + L - 1 of every segment, as far
// as they lie before the last prompt token.
__global__ void stage_prompt_kernel(RowMap rm, const int32_t *prompt, const int32_t *prompt_len, int max_prompt, int chunk,
                                    int L, int n_seqs) {
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    if (m >= n_seqs * 2 * L) return;
    const int k = m % L, seg = m / L;
    const int start = chunk * L;
    int n = prompt_len[seg] - 1 - start;
    n = n < 0 ? 0 : (n > L ? L : n);
    rm.row_tok[m] = k < n ? prompt[(long)seg * max_prompt + start + k] : -1;
    rm.row_pos[m] = start + k;
    if (k == 0) { rm.seg_kv[seg] = start; rm.seg_n[seg] = n; }
}

constexpr int kRefUniform = -1, kRefOneHot = -2, kRefHist0 = -3;  // values of ref_row below 0 (<= -3: kept row -3 - ref)

// Row and normaliser a reference code points at (nullptr: uniform or one-hot, which have no row)
SJD_D const float *ref_row_ptr(const DecideState &d, int s, int rr, const float *e_ref, const uint64_t *Z_ref, int row_width,
                               uint64_t &Z) {
    if (rr >= 0) { Z = Z_ref[rr]; return e_ref + (long)rr * d.V; }
    if (rr <= kRefHist0) {
        const int h = kRefHist0 - rr;
        Z = d.hist_Z[s * row_width + h];
        return d.hist_e + ((long)s * row_width + h) * d.V;
    }
    Z = rr == kRefOneHot ? 1ull : (uint64_t)d.V;
    return nullptr;
}

// ------------------------------------------------------------------- a11: verification (Eq. 2)
// One block per sequence; every draft is tested in parallel, the first rejection is found with a
// wavefront ballot per 64 drafts and a minimum across wavefronts.
__global__ void verify_kernel(DecideState d, uint64_t seed, int row_width) {
    const int s = blockIdx.x, L = d.L, V = d.V;
    const int Le = d.Le[s];
    if (Le == 0) return;
    const uint32_t step = *d.step;
    const float *e_new = d.e_buf[step & 1u] + (long)s * L * V;
    const float *e_ref = d.e_buf[(step & 1u) ^ 1u] + (long)s * L * V;
    const uint64_t *Z_new = d.Z_buf[step & 1u] + s * L;
    const uint64_t *Z_ref = d.Z_buf[(step & 1u) ^ 1u] + s * L;
    __shared__ int first_reject;
    if (threadIdx.x == 0) first_reject = Le;
    __syncthreads();
    for (int base = 1; base < Le; base += blockDim.x) {
        const int k = base + threadIdx.x;
        bool rejected = false;
        if (k < Le) {
            uint32_t w[4];
            draw_words(seed, step, (uint32_t)(k - 1), (uint32_t)s, w);
            const int x = d.win_tok[s * L + k] - d.lo;
            const uint64_t wp = weight_of(e_new[(long)(k - 1) * V + x]);
            const int rr = d.ref_row[s * L + k];  // -1 uniform: 1 / V;  -2 one-hot at this very token: 1 / 1
            uint64_t Zq;
            const float *qrow = ref_row_ptr(d, s, rr, e_ref, Z_ref, row_width, Zq);
            const uint64_t wq = qrow ? weight_of(qrow[x]) : 1ull;
            rejected = !accept_rule(w[0], wp, Z_new[k - 1], wq, Zq);
        }
        const uint64_t mask = __ballot(rejected);
        if ((threadIdx.x & 63) == 0 && mask != 0ull) atomicMin(&first_reject, base + (threadIdx.x & ~63) + __builtin_ctzll(mask));
    }
    __syncthreads();
    if (threadIdx.x == 0) d.acc_len[s] = first_reject - 1;
}

// ---------------------------------------------------- a12 / a13: the draws of a step (Eq. 3, Eq. 5)
// Block-wide inverse CDF over integer weights weight(v), v in [0, V): returns the first v whose inclusive
// prefix sum exceeds floor(u64 * total / 2^64), or -1 when total == 0.  Two levels: (1) each wavefront sums a
// contiguous segment with coalesced reads, every thread scans the <= 16 segment totals and knows which segment
// holds the target; (2) the whole block re-reads that segment, a few consecutive ids per thread, one
// block-wide scan of the per-thread sums names the thread, which walks its ids.  Integer sums: exact.
SJD_D uint64_t shfl_up_u64(uint64_t v, int delta) {
    uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    lo = __shfl_up(lo, delta, 64);
    hi = __shfl_up(hi, delta, 64);
    return ((uint64_t)hi << 32) | lo;
}

// support(v): a cheap test that is true wherever weight(v) != 0 (may be true elsewhere).  With top-K most weights of
// a row are 0 and the costly ones (the residual takes two double-precision divisions per id) are only evaluated
// where the test holds: a thread marks its ids in a bit mask first, with unconditional batched loads, then walks
// the marked ones - a few per thread instead of all.  The sums are integer sums, so nothing changes in the result.
struct AnySupport { SJD_D bool operator()(int) const { return true; } };
template <typename F, typename S = AnySupport>
SJD_D int block_inverse_cdf(F weight, int V, uint64_t u64, uint64_t *sums /* [20] shared */, S support = S()) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6, nt = blockDim.x;
    // level 1: wavefront w owns the contiguous segment [w * seg, (w + 1) * seg), read 64 consecutive ids at a time
    const int per = (V + nt - 1) / nt;          // ids per thread at level 2
    const int seg = per * 64;
    const int v0 = wave * seg, v1 = v0 + seg < V ? v0 + seg : V;
    uint64_t local = 0;
    if (!std::is_same<S, AnySupport>::value && per <= 64) {
        uint64_t marked = 0;
#pragma unroll 8
        for (int i = 0; i < per; ++i) {
            const int v = v0 + lane + 64 * i;
            const bool sup = support(v < V ? v : V - 1);   // the load inside is unconditional
            if (v < v1 && sup) marked |= 1ull << i;
        }
        while (marked) {
            const int i = __builtin_ctzll(marked);
            marked &= marked - 1ull;
            local += weight(v0 + lane + 64 * i);
        }
    } else {
        // batches of 8 ids with clamped, unconditional loads (a loop of load - add pays a memory round trip per id)
        for (int i0 = 0; i0 < per; i0 += 8) {
            uint64_t wv[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int v = v0 + lane + 64 * (i0 + j);
                wv[j] = weight(v < V ? v : V - 1);
                if (v >= v1) wv[j] = 0;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) local += wv[j];
        }
    }
    for (int d = 32; d > 0; d >>= 1) local += shfl_down_u64(local, d);
    __syncthreads();
    if (lane == 0) sums[wave] = local;
    __syncthreads();
    uint64_t total = 0;
    for (int i = 0; i < nw; ++i) total += sums[i];
    if (total == 0) return -1;
    const uint64_t target = mulhi64(u64, total);
    int hit_seg = 0;
    uint64_t before = 0;
    for (int i = 0; i < nw; ++i) {           // the segment whose range of prefix sums holds the target
        if (before + sums[i] > target) { hit_seg = i; break; }
        before += sums[i];
    }
    // level 2: the whole block re-reads that segment, thread t owning the `chunk` consecutive ids from s0 + t * chunk
    const int s0 = hit_seg * seg, s1 = s0 + seg < V ? s0 + seg : V;
    const int chunk = (seg + nt - 1) / nt;
    const int c0 = s0 + tid * chunk, c1 = c0 + chunk < s1 ? c0 + chunk : s1;
    uint64_t mine = 0;
    for (int v = c0; v < c1; ++v) mine += weight(v);
    uint64_t incl = mine;
    for (int d = 1; d < 64; d <<= 1) {
        const uint64_t o = shfl_up_u64(incl, d);
        if (lane >= d) incl += o;
    }
    __syncthreads();
    if (lane == 63) sums[wave] = incl;
    __syncthreads();
    uint64_t excl = before + incl - mine;
    for (int i = 0; i < wave; ++i) excl += sums[i];
    if (excl <= target && target < excl + mine) {   // exactly one thread
        uint64_t run = excl;
        for (int v = c0; v < c1; ++v) {
            run += weight(v);
            if (run > target) { sums[18] = (uint64_t)v; break; }
        }
    }
    __syncthreads();
    return (int)(int64_t)sums[18];
}

// One block per output row k of every sequence.  With a accepted drafts:
//   k == a            the token that becomes final: residual draw (Eq. 3) against the reference of the
//                     rejected draft, or a plain draw from row a when every draft was accepted;
//   a < k <= Le - 2   slot k + 1: kept if p > tau q (Eq. 4-5) else redrawn from row k;
//   k == Le - 1 > a   no draft was predicted by this row: its slot is drawn from it.
// With init_mode 3 the grid has 2 L blocks per sequence: block kk >= Le is the new slot with old index kk + 1 (it has
// no row of its own) and draws from the last row Le - 1 with its own counter, if the next window has that slot.
// Where a new slot of init_mode 4 takes its distribution from: the token row_width places back.  Returns a reference
// code as stored in ref_row for the NEXT window (>= 0 row of this step, -1 uniform, <= -3 kept row) and, in *src_new,
// the row of THIS step to draw from when that token becomes final in this very step (its kept row is written later).
SJD_D int above_source(int k2, int n_img, int a, int Le, int row_width, int *src_new) {
    const int n_new = n_img + a + 1;
    *src_new = -1;
    for (int j = k2;;) {
        const int up = n_new + j - 1 - row_width;
        if (up < 0) return kRefUniform;
        if (up < n_new) {
            if (up >= n_img) *src_new = up - n_img;
            return kRefHist0 - up % row_width;
        }
        j = up - n_new + 1;                      // the place above is slot j of the next window
        if (j + a + 1 <= Le) return j + a;       // it has a row of this step: its reference
    }
}

__global__ void draw_kernel(DecideState d, uint64_t seed, float tau, int rows_per_seq, int init_mode, int row_width) {
    const int r = blockIdx.x, L = d.L, V = d.V, s = r / rows_per_seq;
    int k = r % rows_per_seq;
    const int Le = d.Le[s];
    if (Le == 0) return;
    const int a = d.acc_len[s];
    int new_slot = -1;  // index in the next window of the never-drafted slot this block draws for
    if (k >= Le) {
        if (rows_per_seq == L) return;  // no draws for new slots in the other modes
        const int remaining = d.n_image[s] - (d.n_img[s] + a + 1);
        const int Le2 = remaining < L ? remaining : L;
        new_slot = k + 1 - a - 1;
        if (new_slot >= Le2) return;
    } else if (k < a) {
        return;
    }
    const uint32_t step = *d.step;
    const float *e_new = d.e_buf[step & 1u] + (long)s * L * V;
    const float *e_ref = d.e_buf[(step & 1u) ^ 1u] + (long)s * L * V;
    const uint64_t *Z_new = d.Z_buf[step & 1u] + s * L;
    const uint64_t *Z_ref = d.Z_buf[(step & 1u) ^ 1u] + s * L;
    extern __shared__ uint64_t sums[];

    uint32_t w[4];
    draw_words(seed, step, (uint32_t)(new_slot >= 0 ? k + 1 : k), (uint32_t)s, w);
    const uint64_t u64 = ((uint64_t)w[1] << 32) | w[2];
    if (new_slot >= 0) {
        // init_mode 3: the last row of this step; init_mode 4: the distribution of the token one image row above
        const float *src = e_new + (long)(Le - 1) * V;
        uint64_t Zs = Z_new[Le - 1];
        if (init_mode == 4) {
            int src_new;
            const int code = above_source(new_slot, d.n_img[s], a, Le, row_width, &src_new);
            if (code == kRefUniform) return;   // a uniform draft: the window update makes it
            if (src_new >= 0) { src = e_new + (long)src_new * V; Zs = Z_new[src_new]; }
            else if (code >= 0) { src = e_new + (long)code * V; Zs = Z_new[code]; }
            else src = ref_row_ptr(d, s, code, e_ref, Z_ref, row_width, Zs);
        }
        auto from_src = [&](int v) { return weight_of(src[v]); };
        const int t = block_inverse_cdf(from_src, V, u64, sums);
        if (threadIdx.x == 0) d.cand_new[s * L + new_slot] = d.lo + t;
        return;
    }
    const float *pk = e_new + (long)k * V;
    const uint64_t Zp = Z_new[k];
    auto from_p = [&](int v) { return weight_of(pk[v]); };

    int tok;
    if (k == a && a < Le - 1) {
        const int rr = d.ref_row[s * L + a + 1];
        uint64_t Zq;
        const float *qrow = ref_row_ptr(d, s, rr, e_ref, Z_ref, row_width, Zq);
        const int x = d.win_tok[s * L + a + 1] - d.lo;
        auto resid = [&](int v) {
            double P = prob(weight_of(pk[v]), Zp);
            double Q = rr == kRefOneHot ? (v == x ? 1.0 : 0.0) : prob(qrow ? weight_of(qrow[v]) : 1ull, Zq);
            return residual_weight(P, Q);
        };
        // p(v) has weight 0 below 2^-40 (weight_of), and where p is 0 so is max(0, p - q)
        auto p_support = [&](int v) { return pk[v] >= 0x1p-40f; };
        tok = block_inverse_cdf(resid, V, u64, sums, p_support);
        if (tok < 0) tok = block_inverse_cdf(from_p, V, u64, sums);
    } else if (k > a && k <= Le - 2) {
        const int x = d.win_tok[s * L + k + 1] - d.lo;
        const int rr = d.ref_row[s * L + k + 1];
        uint64_t Zq;
        const float *qrow = ref_row_ptr(d, s, rr, e_ref, Z_ref, row_width, Zq);
        const uint64_t wq = qrow ? weight_of(qrow[x]) : 1ull;
        if (keep_rule(tau, weight_of(pk[x]), Zp, wq, Zq)) {
            tok = x;
        } else {
            tok = block_inverse_cdf(from_p, V, u64, sums);
        }
    } else {
        tok = block_inverse_cdf(from_p, V, u64, sums);
    }
    if (threadIdx.x == 0) d.cand[s * L + k] = d.lo + tok;
}

// ----------------------------------------------- a14: finalise, shift the window, refill, commit
__global__ void commit_kernel(DecideState d, uint64_t seed, int init_mode, int row_width) {
    const int s = blockIdx.x, L = d.L;
    const int Le = d.Le[s];
    sjd_step_result *res = d.res + s;
    if (Le == 0) {
        if (threadIdx.x == 0) { res->n_accepted = 0; res->n_finalized = 0; res->reject_index = -1; res->done = 1; }
        return;
    }
    const uint32_t step = *d.step;
    const int a = d.acc_len[s];
    const int n_img = d.n_img[s], N = d.n_image[s];
    const int y = d.cand[s * L + a];
    int32_t *out = d.out_tok + (long)s * d.max_img;
    for (int k = 1 + threadIdx.x; k <= a; k += blockDim.x) out[n_img + k - 1] = d.win_tok[s * L + k];
    const int remaining = N - (n_img + a + 1);
    const int Le2 = remaining < L ? remaining : L;
    __syncthreads();  // every read of the old window is done
    for (int k2 = 1 + threadIdx.x; k2 < L; k2 += blockDim.x) {
        int tok = 0, ref = -1;
        if (k2 < Le2) {
            const int k = k2 + a + 1;
            if (k <= Le) {           // slot k of this step (k == Le: the slot predicted by the last row)
                tok = d.cand[s * L + k - 1];
                ref = k - 1;
            } else {                 // a slot that never had a draft (Sec. 4.2)
                const int n_new = n_img + a + 1;  // image tokens final after this step; this slot's token is n_new + k2 - 1
                auto uniform_of = [&](int kk) {   // the uniform draft of old slot index kk
                    uint32_t w[4];
                    draw_words(seed, step, (uint32_t)kk, (uint32_t)s, w);
                    return d.lo + (int)__umulhi(w[3], (uint32_t)d.V);
                };
                if (init_mode == 1) {
                    // every new slot repeats its left neighbour, so all of them equal the last slot that has a row
                    // (k == Le, present only after a rejection) or else the token that just became final
                    tok = a < Le - 1 ? d.cand[s * L + Le - 1] : y;
                    ref = kRefOneHot;
                } else if (init_mode == 2) {
                    // the token row_width places back; that place may itself be a new slot of this window, filled
                    // by the same rule: follow the chain
                    int j = k2;
                    for (;;) {
                        const int up = n_new + j - 1 - row_width;
                        if (up < 0) {                       // first image row: slot j is uniform (and k2 copies it)
                            tok = uniform_of(j + a + 1);
                            ref = j == k2 ? kRefUniform : kRefOneHot;
                            break;
                        }
                        ref = kRefOneHot;
                        if (up < n_img + a) { tok = out[up]; break; }   // final before this step, or accepted in it (copied above)
                        if (up == n_new - 1) { tok = y; break; }
                        j = up - n_new + 1;                 // slot j of the next window
                        if (j + a + 1 <= Le) { tok = d.cand[s * L + j + a]; break; }       // a slot that has a row
                    }
                } else if (init_mode == 3) {
                    tok = d.cand_new[s * L + k2];
                    ref = Le - 1;
                } else if (init_mode == 4) {
                    int src_new;
                    ref = above_source(k2, n_img, a, Le, row_width, &src_new);
                    tok = ref == kRefUniform ? uniform_of(k) : d.cand_new[s * L + k2];
                } else {
                    tok = uniform_of(k);
                }
            }
        }
        d.win_tok[s * L + k2] = tok;
        d.ref_row[s * L + k2] = ref;
    }
    if (threadIdx.x == 0) {
        out[n_img + a] = y;
        d.n_img[s] = n_img + a + 1;
        d.kv_len[s * 2] += a + 1;
        d.kv_len[s * 2 + 1] += a + 1;
        d.anchor[s * 2] = y;
        d.anchor[s * 2 + 1] = y;
        d.Le[s] = Le2;  // 0 when the image is complete
        res->n_accepted = a;
        res->n_finalized = a + 1;
        res->reject_index = a < Le - 1 ? a + 1 : -1;
        res->done = remaining == 0 ? 1 : 0;
    }
}

// init_mode 4: image token n_img + i became final under row i of this step (i <= a).  One block per (sequence, i);
// where several of them share a slot of the ring (row_width <= a) the last one is the one kept.
__global__ void keep_rows_kernel(DecideState d, int row_width) {
    const int L = d.L, V = d.V, s = blockIdx.x / L, i = blockIdx.x % L;
    if (d.Le[s] == 0) return;
    const int a = d.acc_len[s];
    if (i > a || i + row_width <= a) return;
    const uint32_t step = *d.step;
    const float *src = d.e_buf[step & 1u] + ((long)s * L + i) * V;
    const int h = (d.n_img[s] + i) % row_width;
    float *dst = d.hist_e + ((long)s * row_width + h) * V;
    for (int v = threadIdx.x; v < V; v += blockDim.x) dst[v] = src[v];
    if (threadIdx.x == 0) d.hist_Z[s * row_width + h] = d.Z_buf[step & 1u][s * L + i];
}

__global__ void philox_fill_kernel(uint64_t seed, uint32_t row, uint32_t seq, uint32_t *out, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint32_t w[4];
    draw_words(seed, (uint32_t)i, row, seq, w);
    for (int j = 0; j < 4; ++j) out[4 * i + j] = w[j];
}


}  // namespace

hipError_t launch_init_window(hipStream_t st, const DecideState &d, const SamplingParams &sp, int n_seqs, int max_seqs,
                              const int32_t *prompt_last, const int32_t *prompt_len, const int32_t *n_image) {
    init_window_kernel<<<max_seqs, 64, 0, st>>>(d, sp.seed, n_seqs, prompt_last, prompt_len, n_image);
    return hipGetLastError();
}

hipError_t launch_stage_window(hipStream_t st, const DecideState &d, const RowMap &rm, int n_seqs) {
    const int M = n_seqs * 2 * d.L;
    stage_window_kernel<<<ceil_div(M, 256), 256, 0, st>>>(d, rm, n_seqs);
    return hipGetLastError();
}

hipError_t launch_stage_prompt(hipStream_t st, const RowMap &rm, const int32_t *prompt, const int32_t *prompt_len,
                               int max_prompt, int chunk, int L, int n_seqs) {
    const int M = n_seqs * 2 * L;
    stage_prompt_kernel<<<ceil_div(M, 256), 256, 0, st>>>(rm, prompt, prompt_len, max_prompt, chunk, L, n_seqs);
    return hipGetLastError();
}

hipError_t launch_sample_rows(hipStream_t st, const DecideState &d, const SamplingParams &sp, const float *logits,
                              int n_seqs) {
    SampleRowsArgs a;
    a.lc_base = logits;
    a.lu_base = logits + (long)d.L * d.V;
    a.seq_stride = 2l * d.L * d.V;
    a.L = d.L;
    a.e_base[0] = d.e_buf[0]; a.e_base[1] = d.e_buf[1];
    a.Z_base[0] = d.Z_buf[0]; a.Z_base[1] = d.Z_buf[1];
    a.step = d.step;
    a.Le = d.Le;
    a.V = d.V;
    a.top_k = sp.top_k;
    a.cfg_scale = sp.cfg_scale;
    a.inv_t = sp.inv_temperature;
    return launch_sample_rows_any(st, a, n_seqs * d.L);
}

hipError_t launch_sampling_rows_plain(hipStream_t st, const float *lc, const float *lu, float *e, uint64_t *Z, int rows,
                                      int V, const SamplingParams &sp) {
    SampleRowsArgs a;
    a.lc_base = lc;
    a.lu_base = lu;
    a.seq_stride = 0;
    a.L = rows;
    a.e_base[0] = a.e_base[1] = e;
    a.Z_base[0] = a.Z_base[1] = Z;
    a.step = nullptr;
    a.Le = nullptr;
    a.V = V;
    a.top_k = sp.top_k;
    a.cfg_scale = sp.cfg_scale;
    a.inv_t = sp.inv_temperature;
    return launch_sample_rows_any(st, a, rows);
}

hipError_t launch_verify(hipStream_t st, const DecideState &d, const SamplingParams &sp, int n_seqs) {
    verify_kernel<<<n_seqs, 256, 0, st>>>(d, sp.seed, sp.row_width);
    return hipGetLastError();
}

hipError_t launch_draw(hipStream_t st, const DecideState &d, const SamplingParams &sp, int n_seqs) {
    const int rows_per_seq = sp.init_mode >= 3 ? 2 * d.L : d.L;
    draw_kernel<<<n_seqs * rows_per_seq, d.V >= 8192 ? 1024 : 256, 20 * sizeof(uint64_t), st>>>(d, sp.seed, sp.tau, rows_per_seq,
                                                                                                 sp.init_mode, sp.row_width);
    return hipGetLastError();
}

hipError_t launch_commit(hipStream_t st, const DecideState &d, const SamplingParams &sp, int n_seqs) {
    commit_kernel<<<n_seqs, 64, 0, st>>>(d, sp.seed, sp.init_mode, sp.row_width);
    return hipGetLastError();
}

hipError_t launch_keep_rows(hipStream_t st, const DecideState &d, const SamplingParams &sp, int n_seqs) {
    keep_rows_kernel<<<n_seqs * d.L, 256, 0, st>>>(d, sp.row_width);
    return hipGetLastError();
}

hipError_t launch_philox_fill(hipStream_t st, uint64_t seed, uint32_t row, uint32_t seq, uint32_t *out, int n) {
    philox_fill_kernel<<<ceil_div(n, 256), 256, 0, st>>>(seed, row, seq, out, n);
    return hipGetLastError();
}
