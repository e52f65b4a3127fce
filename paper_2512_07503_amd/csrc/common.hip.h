// Shared device/host helpers of the sjd library: data layouts in HBM, bf16 conversion,
// error handling.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/sjd.h"

typedef uint16_t bf16_t;  // raw bfloat16 bits in memory

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // 16 bytes = one lane's share of a fragment

#define SJD_HD __host__ __device__ __forceinline__
#define SJD_D __device__ __forceinline__

SJD_HD float bf16_to_float(bf16_t h) {
    uint32_t u = (uint32_t)h << 16;
    return __builtin_bit_cast(float, u);
}
// round to nearest, ties to even (inputs are finite)
SJD_HD bf16_t float_to_bf16(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename T> SJD_HD float to_float(T v);
template <> SJD_HD float to_float<float>(float v) { return v; }
template <> SJD_HD float to_float<bf16_t>(bf16_t v) { return bf16_to_float(v); }
template <typename T> SJD_HD T from_float(float v);
template <> SJD_HD float from_float<float>(float v) { return v; }
template <> SJD_HD bf16_t from_float<bf16_t>(float v) { return float_to_bf16(v); }

SJD_HD int ceil_div(int a, int b) { return (a + b - 1) / b; }
SJD_HD size_t ceil_div_sz(size_t a, size_t b) { return (a + b - 1) / b; }

// ---------------------------------------------------------------------------------------------
// Data layouts.
//
// fp32 mode keeps everything row-major.  bf16 mode stores every GEMM operand, the KV pages and the
// queries "fragment-major": in the order in which the 64 lanes of a wavefront feed a
// v_mfma_f32_32x32x16_bf16, so that one operand fragment (32 rows x 16 k, 1 KiB) is 1 KiB of
// contiguous memory and a wavefront fetches it with one fully coalesced 16-byte-per-lane load.
// Lane l of a fragment holds 8 consecutive k of row (l % 32), starting at k = 8 * (l / 32).
// ---------------------------------------------------------------------------------------------
template <typename T> struct Layout;

template <> struct Layout<float> {
    // activation matrix feeding a GEMM, logical [M][K]
    static SJD_HD size_t a_index(int m, int k, int K) { return (size_t)m * K + k; }
    static SJD_HD size_t a_elems(int M, int K) { return (size_t)M * K; }
    // weight matrix, logical [N][K]
    static SJD_HD size_t w_index(int n, int k, int K) { return (size_t)n * K + k; }
    static SJD_HD size_t w_elems(int N, int K) { return (size_t)N * K; }
    // one (page, kv head) block of keys / values, logical [page_tokens][hd]
    static SJD_HD size_t k_index(int t, int j, int hd) { return (size_t)t * hd + j; }
    static SJD_HD size_t v_index(int t, int j, int hd) { return (size_t)t * hd + j; }
    // queries of one (sequence, branch, head): logical [L][hd]
    static SJD_HD size_t q_index(int i, int j, int hd) { return (size_t)i * hd + j; }
    static SJD_HD size_t q_elems(int L, int hd) { return (size_t)L * hd; }
};

template <> struct Layout<bf16_t> {
    // [M/32][K/16][64 lanes][8]: lane = 32 * ((k % 16) / 8) + m % 32
    static SJD_HD size_t a_index(int m, int k, int K) {
        return ((((size_t)(m >> 5) * (K >> 4) + (k >> 4)) * 64) + (((k >> 3) & 1) << 5) + (m & 31)) * 8 + (k & 7);
    }
    static SJD_HD size_t a_elems(int M, int K) { return (size_t)ceil_div(M, 32) * 32 * K; }
    static SJD_HD size_t w_index(int n, int k, int K) { return a_index(n, k, K); }
    static SJD_HD size_t w_elems(int N, int K) { return (size_t)ceil_div(N, 32) * 32 * K; }
    // keys of a page: operand with rows = tokens, k = head dimension:
    // [t/32][j/16][lane = 32*((j%16)/8) + t%32][j%8]
    static SJD_HD size_t k_index(int t, int j, int hd) {
        return ((((size_t)(t >> 5) * (hd >> 4) + (j >> 4)) * 64) + (((j >> 3) & 1) << 5) + (t & 31)) * 8 + (j & 7);
    }
    // values of a page: operand with rows = head dimension, k = tokens, in the token order in which a
    // 32x32 accumulator tile of scores (rows = tokens) leaves the matrix core: within a block of 32
    // tokens, token u of the i-th half (u = t % 16) sits in k-slot (g = (u % 8) / 4, e = 4 * (u / 8) + u % 4).
    // [t/32][(t%32)/16][j/32][lane = 32*g + j%32][e]
    static SJD_HD size_t v_index(int t, int j, int hd) {
        int u = t & 15;
        int g = (u & 7) >> 2, e = ((u >> 3) << 2) + (u & 3);
        size_t frag = ((size_t)(t >> 5) * 2 + ((t >> 4) & 1)) * (hd >> 5) + (j >> 5);
        return (frag * 64 + (g << 5) + (j & 31)) * 8 + e;
    }
    // queries: operand with rows (columns of the transposed product) = window index, k = head dimension
    // [i/32][j/16][lane = 32*((j%16)/8) + i%32][j%8]
    static SJD_HD size_t q_index(int i, int j, int hd) {
        return ((((size_t)(i >> 5) * (hd >> 4) + (j >> 4)) * 64) + (((j >> 3) & 1) << 5) + (i & 31)) * 8 + (j & 7);
    }
    static SJD_HD size_t q_elems(int L, int hd) { return (size_t)ceil_div(L, 32) * 32 * hd; }
};

// ---------------------------------------------------------------------------------------------
// Host-side error plumbing
// ---------------------------------------------------------------------------------------------
#define SJD_HIP_TRY(ctx_err, expr)                                                              \
    do {                                                                                        \
        hipError_t e__ = (expr);                                                                \
        if (e__ != hipSuccess) {                                                                \
            sjd_set_error(ctx_err, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__), __FILE__, __LINE__); \
            return SJD_EDEVICE;                                                                 \
        }                                                                                       \
    } while (0)

void sjd_set_error(char *buf, const char *fmt, ...);
