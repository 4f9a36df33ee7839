// Register blocks of the radix-2 negacyclic transforms shared by the N = 2^16 kernels and the small-ring kernels:
// four butterfly stages on 16 points, or two on 4 points, held by one thread (Harvey butterflies, Shoup twiddle
// products with the three-multiply approximate quotient, lazy ranges).
#pragma once
#include "modarith.h"

// q4 = 4q throughout this file.
template <bool WIDE>
__device__ __forceinline__ void ct_bfly(u64& X, u64& Y, u64 w, u64 w_sh, u64 q, u64 q4) {
    if (WIDE) X = csub(X, q4);
    u64 T = shoup_lazy4(Y, w, w_sh, q);
    Y = (X + q4) - T;
    X = X + T;
}

__device__ __forceinline__ void gs_bfly(u64& X, u64& Y, u64 w, u64 w_sh, u64 q, u64 q4) {
    u64 s = csub(X + Y, q4);
    u64 d = (X + q4) - Y;
    Y = shoup_lazy4(d, w, w_sh, q);
    X = s;
}

// Four forward stages on 16 register points; stage u pairs (k, k + (8>>u)); the twiddle of the
// pair's group g = k >> (4-u) is tw[(1 << (s0+u)) + (G << u) + g], G = group of the 16 points at
// stage s0.
template <bool WIDE>
__device__ __forceinline__ void fwd_block4(u64 (&x)[16], const u64* __restrict__ tw, const u64* __restrict__ tw_sh,
                                           uint32_t s0, uint32_t G, u64 q, u64 q4) {
#pragma unroll
    for (int u = 0; u < 4; u++) {
        const int dist = 8 >> u;
        const uint32_t base = (1u << (s0 + u)) + (G << u);
#pragma unroll
        for (int g = 0; g < (1 << u); g++) {
            const u64 w = tw[base + g], w_sh = tw_sh[base + g];
#pragma unroll
            for (int k = 0; k < dist; k++) {
                const int a = g * 2 * dist + k;
                ct_bfly<WIDE>(x[a], x[a + dist], w, w_sh, q, q4);
            }
        }
    }
}

// Four inverse stages (point distance 1,2,4,8 in register index), same twiddle indexing.
__device__ __forceinline__ void inv_block4(u64 (&x)[16], const u64* __restrict__ tw, const u64* __restrict__ tw_sh,
                                           uint32_t s0, uint32_t G, u64 q, u64 q4) {
#pragma unroll
    for (int u = 3; u >= 0; u--) {
        const int dist = 8 >> u;
        const uint32_t base = (1u << (s0 + u)) + (G << u);
#pragma unroll
        for (int g = 0; g < (1 << u); g++) {
            const u64 w = tw[base + g], w_sh = tw_sh[base + g];
#pragma unroll
            for (int k = 0; k < dist; k++) {
                const int a = g * 2 * dist + k;
                gs_bfly(x[a], x[a + dist], w, w_sh, q, q4);
            }
        }
    }
}

// Two forward / inverse stages on 4 register points (same pairing and twiddle indexing as the 16-point blocks).
template <bool WIDE>
__device__ __forceinline__ void fwd_block2(u64 (&x)[4], const u64* tw, const u64* tw_sh, uint32_t s0, uint32_t G, u64 q, u64 q4) {
    const uint32_t b0 = (1u << s0) + G, b1 = (2u << s0) + 2 * G;
    const u64 w0 = tw[b0], w0s = tw_sh[b0], w1 = tw[b1], w1s = tw_sh[b1], w2 = tw[b1 + 1], w2s = tw_sh[b1 + 1];
    ct_bfly<WIDE>(x[0], x[2], w0, w0s, q, q4);
    ct_bfly<WIDE>(x[1], x[3], w0, w0s, q, q4);
    ct_bfly<WIDE>(x[0], x[1], w1, w1s, q, q4);
    ct_bfly<WIDE>(x[2], x[3], w2, w2s, q, q4);
}

__device__ __forceinline__ void inv_block2(u64 (&x)[4], const u64* tw, const u64* tw_sh, uint32_t s0, uint32_t G, u64 q, u64 q4) {
    const uint32_t b0 = (1u << s0) + G, b1 = (2u << s0) + 2 * G;
    const u64 w0 = tw[b0], w0s = tw_sh[b0], w1 = tw[b1], w1s = tw_sh[b1], w2 = tw[b1 + 1], w2s = tw_sh[b1 + 1];
    gs_bfly(x[0], x[1], w1, w1s, q, q4);
    gs_bfly(x[2], x[3], w2, w2s, q, q4);
    gs_bfly(x[0], x[2], w0, w0s, q, q4);
    gs_bfly(x[1], x[3], w0, w0s, q, q4);
}

// The same two-stage blocks with their three twiddles (and Shoup companions) fetched ahead of time: r = {w0, w0', w1,
// w1', w2, w2'} as tw_block2 loads them.
__device__ __forceinline__ void tw_block2(u64 (&r)[6], const u64* __restrict__ tw, const u64* __restrict__ tw_sh, uint32_t s0, uint32_t G) {
    const uint32_t b0 = (1u << s0) + G, b1 = (2u << s0) + 2 * G;
    r[0] = tw[b0]; r[1] = tw_sh[b0]; r[2] = tw[b1]; r[3] = tw_sh[b1]; r[4] = tw[b1 + 1]; r[5] = tw_sh[b1 + 1];
}
template <bool WIDE>
__device__ __forceinline__ void fwd_block2_r(u64 (&x)[4], const u64 (&r)[6], u64 q, u64 q4) {
    ct_bfly<WIDE>(x[0], x[2], r[0], r[1], q, q4);
    ct_bfly<WIDE>(x[1], x[3], r[0], r[1], q, q4);
    ct_bfly<WIDE>(x[0], x[1], r[2], r[3], q, q4);
    ct_bfly<WIDE>(x[2], x[3], r[4], r[5], q, q4);
}
__device__ __forceinline__ void inv_block2_r(u64 (&x)[4], const u64 (&r)[6], u64 q, u64 q4) {
    gs_bfly(x[0], x[1], r[2], r[3], q, q4);
    gs_bfly(x[2], x[3], r[4], r[5], q, q4);
    gs_bfly(x[0], x[2], r[0], r[1], q, q4);
    gs_bfly(x[1], x[3], r[0], r[1], q, q4);
}

// v mod q for v < 100q: a 7-bit quotient estimated from the top bits (never too large, at most 2
// too small), then two conditional subtractions.  The lazy form stops before them: a value below 3q congruent to v.
__device__ __forceinline__ u64 reduce_small_lazy(u64 v, u64 q, uint32_t bits, uint32_t mrec) {
    const uint32_t sh = bits - 8;                       // q >> sh in [128, 256)
    uint32_t v1 = (uint32_t)(v >> sh);                  // < 100 * 256
    uint32_t qh = (v1 * mrec) >> 24;                    // mrec = floor(2^24 / ((q >> sh) + 1))
    return v - (u64)qh * q;
}
__device__ __forceinline__ u64 reduce_small(u64 v, u64 q, uint32_t bits, uint32_t mrec) {
    u64 r = reduce_small_lazy(v, q, bits, mrec);
    r = csub(r, 2 * q);
    return csub(r, q);
}

