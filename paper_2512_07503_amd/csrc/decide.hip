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
// One workgroup of 1024 threads per position.  The guided logits of the row are read from memory once and stay in
// registers as order keys (thread t holds ids t, t + 1024, ...); the row leaves the kernel as its kept (id, weight)
// pairs in ascending id order plus the integer normaliser.
//
// The K-th largest key is found exactly by narrowing a range of candidates with LDS histograms:
//   round 0   bins of 2^17 consecutive keys counted down from the maximum key (order keys are the float's bits, so
//             that is 64 bins per binade: fine where the top of a row lies, and the bulk of a row spreads over
//             hundreds of bins, so the histogram's atomics rarely collide).  Keys more than 2047 bins away, among them
//             every negative logit, share the last bin and are counted per wavefront.  The bin that holds the K-th
//             largest key and the number of keys above it follow from a prefix sum over the bins;
//   rounds 1+ 2048 equal bins over the remaining key range [lo, hi] until lo == hi (each round takes 11 bits off
//             the range: at most three rounds).
// Ties at the K-th value are all kept (they share a key), so nothing ever needs a tie-break.
struct SampleRowsArgs {
    const float *z_base;             // guided logits z, row (s, k) at (s * L + k) * V; NULL: computed here from the two below
    const float *lc_base, *lu_base;  // row r = (s, k): base + s * seq_stride + k * V
    long seq_stride;
    int L;                           // rows per sequence
    int32_t *ids_base[2];            // + (s * L + k) * cap; index = *step & 1 (0 when step == NULL)
    float *e_base[2];
    int32_t *cnt_base[2];            // + s * L + k
    uint64_t *Z_base[2];
    long cap;
    const uint32_t *step;
    const int32_t *Le;               // [S] active rows per sequence, NULL = all
    // allowed id range of a row (NULL = all ids): allow_lo / allow_hi index s * allow_stride + allow_first[s] + k
    // (allow_first NULL: 0)
    const int32_t *allow_lo, *allow_hi, *allow_first;
    long allow_stride;
    int V, top_k;
    float cfg_scale, inv_t;
};

constexpr int kSelBins = 2048;
constexpr int kBin0Shift = 17;   // round 0 of the select: 2^17 order keys per bin = 64 bins per binade of the logit

// First bin (ascending index) at which the running sum of hist reaches `want` (1 <= want <= total); `before` = the
// sum of the bins below it.  2048 bins, 1024 threads (two bins each); result in all threads.
SJD_D void find_bin(const uint32_t *hist, uint32_t want, uint32_t *wsum /* [16] */, uint32_t *out /* [2] */, uint32_t &bin,
                    uint32_t &before) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t c0 = hist[2 * tid], c1 = hist[2 * tid + 1], mine = c0 + c1;
    uint32_t incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(incl, d, 64);
        if (lane >= d) incl += o;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    uint32_t excl = incl - mine;
    for (int w = 0; w < wave; ++w) excl += wsum[w];
    if (excl < want && want <= excl + mine) {   // exactly one thread
        const bool first = want <= excl + c0;
        out[0] = 2 * tid + (first ? 0 : 1);
        out[1] = first ? excl : excl + c0;
    }
    __syncthreads();
    bin = out[0];
    before = out[1];
    __syncthreads();   // out and wsum may be reused
}

template <int VPT>
__global__ __launch_bounds__(1024) void sample_rows_sparse_kernel(SampleRowsArgs a) {
    const int r = blockIdx.x, s = r / a.L, k = r % a.L;
    if (a.Le && k >= a.Le[s]) return;
    const float *lc = a.lc_base + (long)s * a.seq_stride + (long)k * a.V;
    const float *lu = a.lu_base + (long)s * a.seq_stride + (long)k * a.V;
    const uint32_t par = a.step ? (*a.step & 1u) : 0u;
    const long row = (long)s * a.L + k;
    int32_t *ids = a.ids_base[par] + row * a.cap;
    float *e = a.e_base[par] + row * a.cap;
    const int V = a.V, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int alo = 0, ahi = V;
    if (a.allow_lo) {
        const long j = (long)s * a.allow_stride + (a.allow_first ? a.allow_first[s] : 0) + k;
        alo = a.allow_lo[j];
        ahi = a.allow_hi[j];
    }
    __shared__ uint32_t hist[kSelBins];
    __shared__ uint32_t wsum[16], sel[2];
    __shared__ uint32_t scratch32[17];
    __shared__ uint64_t scratch64[17];

    uint32_t key[VPT];  // order key of the guided logit; 0 (below every real key) for ids that are not candidates
    uint32_t kmax = 0;
    // The loads are unconditional (index clamped to the row) and issued in batches: a load under `if (v < V)` is
    // waited for inside its branch, and a thread would pay one memory round trip per element.
    constexpr int kBatch = VPT < 16 ? VPT : 16;
    const float *zrow = a.z_base ? a.z_base + row * V : nullptr;   // block-uniform
#pragma unroll
    for (int i0 = 0; i0 < VPT; i0 += kBatch) {
        float c[kBatch], u[kBatch];
        if (zrow) {   // one uniform branch around a whole batch: a branch per load would make each wait for its data
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int v = tid + (i0 + j) * 1024;
                c[j] = zrow[v < V ? v : V - 1];
                u[j] = 0.0f;
            }
        } else {
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int v = tid + (i0 + j) * 1024, vv = v < V ? v : V - 1;
                c[j] = lc[vv];
                u[j] = lu[vv];
            }
        }
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const int i = i0 + j, v = tid + i * 1024;
            const uint32_t kk = order_key(zrow ? c[j] : guided(c[j], u[j], a.cfg_scale, a.inv_t));
            key[i] = (uint32_t)(v - alo) < (uint32_t)(ahi - alo) ? kk : 0u;
            kmax = key[i] > kmax ? key[i] : kmax;
        }
        __builtin_amdgcn_sched_barrier(0);   // one batch of loads in flight at a time: the keys need the registers
    }
    kmax = block_max_u32(kmax, scratch32);
    const float m = key_to_float(kmax);

    uint32_t thresh = 1u;   // every candidate
    if (a.top_k < ahi - alo) {
        // round 0: bins of the key distance to the maximum, 2^17 keys each
        hist[2 * tid] = 0u;
        hist[2 * tid + 1] = 0u;
        __syncthreads();
        uint32_t n_far = 0;   // wave-uniform
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const uint32_t b = (kmax - key[i]) >> kBin0Shift;
            if (key[i] && b < (uint32_t)(kSelBins - 1)) atomicAdd(&hist[b], 1u);
            // everything further away (half of a row: the negative logits) shares the last bin: counted per wavefront
            n_far += (uint32_t)__popcll(__ballot(key[i] && b >= (uint32_t)(kSelBins - 1)));
        }
        if (lane == 0 && n_far) atomicAdd(&hist[kSelBins - 1], n_far);
        __syncthreads();
        uint32_t bin, before;
        find_bin(hist, (uint32_t)a.top_k, wsum, sel, bin, before);
        uint32_t want = (uint32_t)a.top_k - before;   // rank of the K-th largest among the keys of that bin, from the top
        uint32_t hi = kmax - (bin << kBin0Shift);     // a bin is a range of keys: (hi - 2^17, hi], the last one [1, hi]
        uint32_t lo = bin < (uint32_t)(kSelBins - 1) && hi > (1u << kBin0Shift) ? hi - ((1u << kBin0Shift) - 1u) : 1u;
        // rounds 1+: equal bins over [lo, hi], counted from the top
        for (int round = 0; round < 4 && lo != hi; ++round) {   // block-uniform; three rounds exhaust 32 bits
            const uint32_t span = hi - lo;
            const int width = 32 - __builtin_clz(span);          // bits of span
            const int shift = width > 11 ? width - 11 : 0;       // (span >> shift) < 2048
            hist[2 * tid] = 0u;
            hist[2 * tid + 1] = 0u;
            __syncthreads();
#pragma unroll
            for (int i = 0; i < VPT; ++i)
                if (key[i] >= lo && key[i] <= hi) atomicAdd(&hist[kSelBins - 1 - ((key[i] - lo) >> shift)], 1u);
            __syncthreads();
            find_bin(hist, want, wsum, sel, bin, before);
            want -= before;
            const uint32_t nlo = lo + ((uint32_t)(kSelBins - 1 - bin) << shift);
            uint32_t nhi = nlo + ((1u << shift) - 1u);
            if (nhi < nlo || nhi > hi) nhi = hi;
            lo = nlo;
            hi = nhi;
        }
        thresh = lo;
    }

    // kept pairs in ascending id order: id = tid + 1024 i, so (i, wave, lane) ascending.  Every wavefront counts its
    // kept ids per i; a prefix sum over the (i, wave) counts gives each wavefront's first output slot.
    __shared__ uint32_t base[VPT * 16];
    {
        uint32_t count_i = 0;   // lane i of a wavefront ends up with the wavefront's count for index i (VPT <= 64)
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const uint32_t c = (uint32_t)__popcll(__ballot(key[i] >= thresh && key[i] != 0u));
            count_i = lane == i ? c : count_i;
        }
        if (lane < VPT) base[lane * 16 + wave] = count_i;
    }
    __syncthreads();
    {
        const uint32_t mine = tid < VPT * 16 ? base[tid] : 0u;
        uint32_t incl = mine;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t o = __shfl_up(incl, d, 64);
            if (lane >= d) incl += o;
        }
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        uint32_t excl = incl - mine;
        for (int w = 0; w < wave; ++w) excl += wsum[w];
        if (tid < VPT * 16) base[tid] = excl;
        if (tid == VPT * 16 - 1) a.cnt_base[par][row] = (int32_t)(excl + mine);
        __syncthreads();
    }
    // (the ballots are taken again rather than kept: VPT 64-bit masks would not fit the scalar registers; the empty
    // asm keeps the compiler from carrying them over from the counting pass)
    asm volatile("" : "+s"(thresh));
    int tid_again = tid;   // likewise: the ids tid + 1024 i are rebuilt here, not carried in 64 registers from the loads
    asm volatile("" : "+v"(tid_again));
    uint64_t zsum = 0;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const bool keep = key[i] >= thresh && key[i] != 0u;
        const uint64_t mask = __ballot(keep);
        if (keep) {
            const uint32_t pos = base[i * 16 + wave] + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
            const float ev = exp_neg(key_to_float(key[i]) - m);
            ids[pos] = tid_again + i * 1024;
            e[pos] = ev;
            zsum += weight_of(ev);
        }
        __builtin_amdgcn_sched_barrier(0);   // one index at a time: nothing of the next ones is fetched ahead into registers
    }
    zsum = block_sum_u64(zsum, scratch64);
    if (tid == 0) a.Z_base[par][row] = zsum;
}

// Rows wider than 64 * 1024 ids: the same result from a multi-pass radix select over keys that are recomputed from the
// logits in every pass (one workgroup per row; kept pairs appended by one wavefront at a time in id order).
__global__ __launch_bounds__(1024) void sample_rows_wide_kernel(SampleRowsArgs a) {
    const int r = blockIdx.x, s = r / a.L, k = r % a.L;
    if (a.Le && k >= a.Le[s]) return;
    const float *lc = a.lc_base + (long)s * a.seq_stride + (long)k * a.V;
    const float *lu = a.lu_base + (long)s * a.seq_stride + (long)k * a.V;
    const uint32_t par = a.step ? (*a.step & 1u) : 0u;
    const long row = (long)s * a.L + k;
    int32_t *ids = a.ids_base[par] + row * a.cap;
    float *e = a.e_base[par] + row * a.cap;
    const int V = a.V, tid = threadIdx.x, nt = blockDim.x, lane = tid & 63, wave = tid >> 6;
    int alo = 0, ahi = V;
    if (a.allow_lo) {
        const long j = (long)s * a.allow_stride + (a.allow_first ? a.allow_first[s] : 0) + k;
        alo = a.allow_lo[j];
        ahi = a.allow_hi[j];
    }
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sel[2];
    __shared__ uint32_t scratch32[17];
    __shared__ uint64_t scratch64[17];
    __shared__ uint32_t wcnt[16];
    const float *zrow = a.z_base ? a.z_base + row * a.V : nullptr;
    auto key_of = [&](int v) { return order_key(zrow ? zrow[v] : guided(lc[v], lu[v], a.cfg_scale, a.inv_t)); };

    uint32_t kmax = 0;
    for (int v = alo + tid; v < ahi; v += nt) {
        const uint32_t kk = key_of(v);
        kmax = kk > kmax ? kk : kmax;
    }
    kmax = block_max_u32(kmax, scratch32);
    const float m = key_to_float(kmax);

    uint32_t thresh = 1u;
    if (a.top_k < ahi - alo) {
        uint32_t prefix = 0, mask = 0, want = (uint32_t)a.top_k;
        for (int shift = 24; shift >= 0; shift -= 8) {
            for (int i = tid; i < 256; i += nt) hist[i] = 0;
            __syncthreads();
            for (int v = alo + tid; v < ahi; v += nt) {
                const uint32_t kk = key_of(v);
                if ((kk & mask) == prefix) atomicAdd(&hist[(kk >> shift) & 255u], 1u);
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
    uint32_t n_out = 0;   // block-uniform
    for (int v0 = alo; v0 < ahi; v0 += nt) {
        const int v = v0 + tid;
        const uint32_t kk = v < ahi ? key_of(v) : 0u;
        const bool keep = v < ahi && kk >= thresh;
        const uint64_t mk = __ballot(keep);
        if (lane == 0) wcnt[wave] = (uint32_t)__popcll(mk);
        __syncthreads();
        uint32_t pos = n_out, total = 0;
        for (int w = 0; w < 16; ++w) {
            if (w < wave) pos += wcnt[w];
            total += wcnt[w];
        }
        if (keep) {
            pos += (uint32_t)__popcll(mk & ((1ull << lane) - 1ull));
            const float ev = exp_neg(key_to_float(kk) - m);
            ids[pos] = v;
            e[pos] = ev;
            zsum += weight_of(ev);
        }
        n_out += total;
        __syncthreads();
    }
    zsum = block_sum_u64(zsum, scratch64);
    if (tid == 0) {
        a.Z_base[par][row] = zsum;
        a.cnt_base[par][row] = (int32_t)n_out;
    }
}

hipError_t launch_sample_rows_any(hipStream_t st, const SampleRowsArgs &a, int rows) {
    const int V = a.V;
    if (V <= 1024 * 4) sample_rows_sparse_kernel<4><<<rows, 1024, 0, st>>>(a);
    else if (V <= 1024 * 16) sample_rows_sparse_kernel<16><<<rows, 1024, 0, st>>>(a);
    else if (V <= 1024 * 32) sample_rows_sparse_kernel<32><<<rows, 1024, 0, st>>>(a);
    else if (V <= 1024 * 64) sample_rows_sparse_kernel<64><<<rows, 1024, 0, st>>>(a);
    else sample_rows_wide_kernel<<<rows, 1024, 0, st>>>(a);
    return hipGetLastError();
}

__global__ void scatter_rows_kernel(const int32_t *ids, const float *e, const int32_t *cnt, float *e_dense, int V) {
    const int r = blockIdx.x, n = cnt[r];
    for (int i = threadIdx.x; i < n; i += blockDim.x) e_dense[(long)r * V + ids[(long)r * V + i]] = e[(long)r * V + i];
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
    for (int i = threadIdx.x; i < d.max_img; i += blockDim.x) {   // no forced tokens until the caller sets some
        d.allow_lo[(long)s * d.max_img + i] = 0;
        d.allow_hi[(long)s * d.max_img + i] = d.V;
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
    if (k == 0 && (seg & 1) == 0) d.acc_len[s] = Le - 1;   // "every draft accepted" until the verification finds a rejection
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

// A stored row: kept ids (ascending) with their weights, or one of the two distributions that have no row.
struct RowRef {
    const int32_t *ids;
    const float *e;
    int n;          // kept pairs
    uint64_t Z;
    int kind;       // 0 = stored row, kRefUniform, kRefOneHot
};

// weight of id x in a stored row (0 if it was not kept)
SJD_D uint64_t row_weight(const RowRef &r, int x) {
    int lo = 0, hi = r.n;   // first index whose id is >= x
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (r.ids[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo < r.n && r.ids[lo] == x ? weight_of(r.e[lo]) : 0ull;
}

SJD_D RowRef step_row(const DecideState &d, uint32_t par, int s, int k) {
    const long row = (long)s * d.L + k;
    RowRef r;
    r.ids = d.ids_buf[par] + row * d.cap;
    r.e = d.e_buf[par] + row * d.cap;
    r.n = d.cnt_buf[par][row];
    r.Z = d.Z_buf[par][row];
    r.kind = 0;
    return r;
}

// The distribution a reference code points at: a row of the previous step, a kept row, uniform or one-hot
SJD_D RowRef ref_row_of(const DecideState &d, uint32_t par_ref, int s, int rr, int row_width) {
    if (rr >= 0) return step_row(d, par_ref, s, rr);
    RowRef r;
    if (rr <= kRefHist0) {
        const long h = (long)s * row_width + (kRefHist0 - rr);
        r.ids = d.hist_ids + h * d.cap;
        r.e = d.hist_e + h * d.cap;
        r.n = d.hist_cnt[h];
        r.Z = d.hist_Z[h];
        r.kind = 0;
        return r;
    }
    r.ids = nullptr; r.e = nullptr; r.n = 0;
    r.Z = rr == kRefOneHot ? 1ull : (uint64_t)d.V;
    r.kind = rr;
    return r;
}
// weight of the draft x itself under its reference (a one-hot reference sits at that very token)
SJD_D uint64_t ref_weight_of_draft(const RowRef &q, int x) { return q.kind == 0 ? row_weight(q, x) : 1ull; }

// weight of id x in a stored row, looked up by a whole wavefront: every lane compares a share of the ids (independent,
// coalesced loads in batches; a binary search would be a dozen dependent round trips to memory)
SJD_D uint64_t wave_row_weight(const RowRef &r, int x, int lane) {
    int hit = -1;
    for (int i0 = 0; i0 < r.n; i0 += 64 * 8) {
        int id[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int i = i0 + j * 64 + lane;
            id[j] = r.ids[i < r.n ? i : r.n - 1];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int i = i0 + j * 64 + lane;
            if (i < r.n && id[j] == x) hit = i;
        }
    }
    const uint64_t found = __ballot(hit >= 0);
    if (!found) return 0ull;
    const int src = __builtin_ctzll(found);
    const float e = hit >= 0 ? r.e[hit] : 0.0f;
    return weight_of(__shfl(e, src, 64));
}

// ------------------------------------------------------------------- a11: verification (Eq. 2)
// One wavefront per draft (4 per block, grid.y = sequence): all drafts are tested in parallel and the first rejection
// is the minimum over the rejected ones.  stage_window_kernel has set acc_len[s] = Le - 1 (no rejection).
__global__ __launch_bounds__(256) void verify_kernel(DecideState d, uint64_t seed, int row_width) {
    const int s = blockIdx.y, L = d.L, lane = threadIdx.x & 63;
    const int k = 1 + blockIdx.x * 4 + (threadIdx.x >> 6);   // draft in slot k against row k - 1
    const int Le = d.Le[s];
    if (k >= Le) return;
    const uint32_t step = *d.step, par = step & 1u;
    uint32_t w[4];
    draw_words(seed, step, (uint32_t)(k - 1), (uint32_t)s, w);
    const int x = d.win_tok[s * L + k] - d.lo;
    const RowRef p = step_row(d, par, s, k - 1);
    const RowRef q = ref_row_of(d, par ^ 1u, s, d.ref_row[s * L + k], row_width);
    const uint64_t wp = wave_row_weight(p, x, lane);
    const uint64_t wq = q.kind == 0 ? wave_row_weight(q, x, lane) : 1ull;
    if (lane == 0 && !accept_rule(w[0], wp, p.Z, wq, q.Z)) atomicMin(&d.acc_len[s], k - 1);
}

// ---------------------------------------------------- a12 / a13: the draws of a step (Eq. 3, Eq. 5)
SJD_D uint64_t shfl_up_u64(uint64_t v, int delta) {
    uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    lo = __shfl_up(lo, delta, 64);
    hi = __shfl_up(hi, delta, 64);
    return ((uint64_t)hi << 32) | lo;
}

// Block-wide inverse CDF over the integer weights weight(i) of the n kept pairs of a row (ascending id, so the
// prefix sums run in ascending token order; ids that were not kept have weight 0 and cannot be hit): returns the
// first i whose inclusive prefix sum exceeds floor(u64 * total / 2^64), or -1 when total == 0.  Thread t owns the
// consecutive pairs [t * per, t * per + per); a block-wide scan of the per-thread sums names the thread that holds
// the target, which walks its pairs.  Integer sums: exact in any order.
template <typename F>
SJD_D int block_inverse_cdf(F weight, int n, uint64_t u64, uint64_t *sums /* [20] shared */) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6, nt = blockDim.x;
    const int per = (n + nt - 1) / nt;
    const int c0 = tid * per < n ? tid * per : n, c1 = c0 + per < n ? c0 + per : n;
    uint64_t mine = 0;
    for (int i0 = c0; i0 < c1; i0 += 8) {   // batches of 8 with clamped, unconditional evaluation: their loads go out together
        uint64_t wv[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) wv[j] = weight(i0 + j < n ? i0 + j : n - 1);
#pragma unroll
        for (int j = 0; j < 8; ++j) mine += i0 + j < c1 ? wv[j] : 0ull;
    }
    uint64_t incl = mine;
    for (int d = 1; d < 64; d <<= 1) {
        const uint64_t o = shfl_up_u64(incl, d);
        if (lane >= d) incl += o;
    }
    __syncthreads();
    if (lane == 63) sums[wave] = incl;
    __syncthreads();
    uint64_t total = 0, excl = incl - mine;
    for (int i = 0; i < nw; ++i) {
        if (i < wave) excl += sums[i];
        total += sums[i];
    }
    if (total == 0) return -1;
    const uint64_t target = mulhi64(u64, total);
    if (excl <= target && target < excl + mine) {   // exactly one thread
        uint64_t run = excl;
        for (int i = c0; i < c1; ++i) {
            run += weight(i);
            if (run > target) { sums[18] = (uint64_t)i; break; }
        }
    }
    __syncthreads();
    return (int)(int64_t)sums[18];
}

// A stored row that fits is copied into LDS by the whole block (one coalesced pass) and read from there afterwards:
// the draws walk a row several times and the residual looks every kept id of p up in q, which from global memory
// would be chains of dependent round trips.
constexpr int kRowLdsCap = 3584;
SJD_D void stage_row(RowRef &r, int32_t *ids_s, float *e_s) {
    if (r.kind != 0 || r.n > kRowLdsCap) return;   // block-uniform
    for (int i0 = threadIdx.x; i0 < r.n; i0 += 8 * blockDim.x) {   // 16 loads per thread in flight
        int id[8];
        float ev[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int i = i0 + j * blockDim.x, ii = i < r.n ? i : r.n - 1;
            id[j] = r.ids[ii];
            ev[j] = r.e[ii];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int i = i0 + j * blockDim.x;
            if (i < r.n) { ids_s[i] = id[j]; e_s[i] = ev[j]; }
        }
    }
    r.ids = ids_s;
    r.e = e_s;
}

// token drawn from a stored row (id relative to sample_lo)
SJD_D int draw_from_row(const RowRef &p, uint64_t u64, uint64_t *sums) {
    auto w = [&](int i) { return weight_of(p.e[i]); };
    const int i = block_inverse_cdf(w, p.n, u64, sums);
    return p.ids[i < 0 ? 0 : i];
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
    const int r = blockIdx.x, L = d.L, s = r / rows_per_seq;
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
    const uint32_t step = *d.step, par = step & 1u;
    __shared__ uint64_t sums[20];
    __shared__ int32_t p_ids[kRowLdsCap], q_ids[kRowLdsCap];
    __shared__ float p_e[kRowLdsCap], q_e[kRowLdsCap];

    uint32_t w[4];
    draw_words(seed, step, (uint32_t)(new_slot >= 0 ? k + 1 : k), (uint32_t)s, w);
    const uint64_t u64 = ((uint64_t)w[1] << 32) | w[2];
    if (new_slot >= 0) {
        // init_mode 3: the last row of this step; init_mode 4: the distribution of the token one image row above
        RowRef src = step_row(d, par, s, Le - 1);
        if (init_mode == 4) {
            int src_new;
            const int code = above_source(new_slot, d.n_img[s], a, Le, row_width, &src_new);
            if (code == kRefUniform) return;   // a uniform draft: the window update makes it
            if (src_new >= 0) src = step_row(d, par, s, src_new);
            else if (code >= 0) src = step_row(d, par, s, code);
            else src = ref_row_of(d, par ^ 1u, s, code, row_width);
        }
        stage_row(src, p_ids, p_e);
        __syncthreads();
        const int t = draw_from_row(src, u64, sums);
        if (threadIdx.x == 0) d.cand_new[s * L + new_slot] = d.lo + t;
        return;
    }
    RowRef p = step_row(d, par, s, k);
    stage_row(p, p_ids, p_e);

    int tok;
    if (k == a && a < Le - 1) {
        RowRef q = ref_row_of(d, par ^ 1u, s, d.ref_row[s * L + a + 1], row_width);
        stage_row(q, q_ids, q_e);
        __syncthreads();
        const int x = d.win_tok[s * L + a + 1] - d.lo;
        // max(0, p - q) is 0 wherever p is: the pairs of p are all there is to sum over
        auto resid = [&](int i) {
            const int v = p.ids[i];
            const double P = prob(weight_of(p.e[i]), p.Z);
            const double Q = q.kind == kRefOneHot ? (v == x ? 1.0 : 0.0) : prob(q.kind == 0 ? row_weight(q, v) : 1ull, q.Z);
            return residual_weight(P, Q);
        };
        const int i = block_inverse_cdf(resid, p.n, u64, sums);
        tok = i >= 0 ? p.ids[i] : draw_from_row(p, u64, sums);
    } else if (k > a && k <= Le - 2) {
        const int x = d.win_tok[s * L + k + 1] - d.lo;
        RowRef q = ref_row_of(d, par ^ 1u, s, d.ref_row[s * L + k + 1], row_width);
        stage_row(q, q_ids, q_e);
        __syncthreads();
        if (keep_rule(tau, row_weight(p, x), p.Z, ref_weight_of_draft(q, x), q.Z)) tok = x;
        else tok = draw_from_row(p, u64, sums);
    } else {
        __syncthreads();
        tok = draw_from_row(p, u64, sums);
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
    const int L = d.L, s = blockIdx.x / L, i = blockIdx.x % L;
    if (d.Le[s] == 0) return;
    const int a = d.acc_len[s];
    if (i > a || i + row_width <= a) return;
    const RowRef src = step_row(d, *d.step & 1u, s, i);
    const long h = (long)s * row_width + (d.n_img[s] + i) % row_width;
    for (int j = threadIdx.x; j < src.n; j += blockDim.x) {
        d.hist_ids[h * d.cap + j] = src.ids[j];
        d.hist_e[h * d.cap + j] = src.e[j];
    }
    if (threadIdx.x == 0) {
        d.hist_cnt[h] = src.n;
        d.hist_Z[h] = src.Z;
    }
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
                              int n_seqs, const float *z) {
    SampleRowsArgs a;
    a.z_base = z;
    a.lc_base = logits;
    a.lu_base = logits + (long)d.L * d.V;
    a.seq_stride = 2l * d.L * d.V;
    a.L = d.L;
    for (int b = 0; b < 2; ++b) {
        a.ids_base[b] = d.ids_buf[b]; a.e_base[b] = d.e_buf[b]; a.cnt_base[b] = d.cnt_buf[b]; a.Z_base[b] = d.Z_buf[b];
    }
    a.cap = d.cap;
    a.step = d.step;
    a.Le = d.Le;
    a.allow_lo = d.allow_lo;
    a.allow_hi = d.allow_hi;
    a.allow_first = d.n_img;      // row k of sequence s predicts image position n_img[s] + k
    a.allow_stride = d.max_img;
    a.V = d.V;
    a.top_k = sp.top_k;
    a.cfg_scale = sp.cfg_scale;
    a.inv_t = sp.inv_temperature;
    return launch_sample_rows_any(st, a, n_seqs * d.L);
}

hipError_t launch_sampling_rows_plain(hipStream_t st, const float *lc, const float *lu, int32_t *ids, float *e, int32_t *cnt,
                                      uint64_t *Z, int rows, int V, const SamplingParams &sp, const int32_t *allow_lo,
                                      const int32_t *allow_hi) {
    SampleRowsArgs a;
    a.z_base = nullptr;
    a.lc_base = lc;
    a.lu_base = lu;
    a.seq_stride = 0;
    a.L = rows;
    a.ids_base[0] = a.ids_base[1] = ids;
    a.e_base[0] = a.e_base[1] = e;
    a.cnt_base[0] = a.cnt_base[1] = cnt;
    a.Z_base[0] = a.Z_base[1] = Z;
    a.cap = V;
    a.step = nullptr;
    a.Le = nullptr;
    a.allow_lo = allow_lo;
    a.allow_hi = allow_hi;
    a.allow_first = nullptr;
    a.allow_stride = 0;
    a.V = V;
    a.top_k = sp.top_k;
    a.cfg_scale = sp.cfg_scale;
    a.inv_t = sp.inv_temperature;
    return launch_sample_rows_any(st, a, rows);
}

hipError_t launch_scatter_rows(hipStream_t st, const int32_t *ids, const float *e, const int32_t *cnt, float *e_dense, int rows,
                               int V) {
    scatter_rows_kernel<<<rows, 256, 0, st>>>(ids, e, cnt, e_dense, V);
    return hipGetLastError();
}

hipError_t launch_verify(hipStream_t st, const DecideState &d, const SamplingParams &sp, int n_seqs) {
    if (d.L > 1) verify_kernel<<<dim3(ceil_div(d.L - 1, 4), n_seqs), 256, 0, st>>>(d, sp.seed, sp.row_width);
    return hipGetLastError();
}

hipError_t launch_draw(hipStream_t st, const DecideState &d, const SamplingParams &sp, int n_seqs) {
    const int rows_per_seq = sp.init_mode >= 3 ? 2 * d.L : d.L;
    draw_kernel<<<n_seqs * rows_per_seq, 256, 0, st>>>(d, sp.seed, sp.tau, rows_per_seq, sp.init_mode, sp.row_width);
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
