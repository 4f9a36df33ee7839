// Device-side 64-bit modular arithmetic for gfx950.
//
// gfx950 has no 64x64->128 multiply; wide products are built from 32x32->64 multiply-adds
// (v_mad_u64_u32), which issue at the same rate as fp64 FMA on this chip, so the cost model is
// "count the 32-bit multiplies".  Twiddle-like multiplications by a constant known in advance
// use Shoup's precomputed quotient; sums of products are accumulated in 128 bits and reduced
// once with a Barrett step.
#pragma once
#include "he_internal.h"

__device__ __forceinline__ u64 mulhi64(u64 a, u64 b) { return __umul64hi(a, b); }

// w*y mod q in [0, 2q) for any y < 2^64, given w < q and w_sh = floor(w*2^64/q)  (Shoup).
__device__ __forceinline__ u64 shoup_lazy(u64 y, u64 w, u64 w_sh, u64 q) {
    u64 h = mulhi64(w_sh, y);
    return w * y - h * q;
}

__device__ __forceinline__ u64 csub(u64 x, u64 q) { return x >= q ? x - q : x; }

// High word of a*b from three 32x32 products (the low*low product and the carries out of the
// middle column are dropped): never above the true value, at most 2 below it.
__device__ __forceinline__ u64 mulhi64_approx(u64 a, u64 b) {
    const uint32_t al = (uint32_t)a, ah = (uint32_t)(a >> 32), bl = (uint32_t)b, bh = (uint32_t)(b >> 32);
    const u64 mid = (u64)__umulhi(ah, bl) + (u64)__umulhi(al, bh);
    return (u64)ah * bh + mid;
}

// w*y mod q in [0, 4q): Shoup's product with the approximate quotient above (one multiply fewer
// and no carry chain; the quotient is at most 2 short, each unit adds q to the remainder).
__device__ __forceinline__ u64 shoup_lazy4(u64 y, u64 w, u64 w_sh, u64 q) {
    u64 h = mulhi64_approx(w_sh, y);
    return w * y - h * q;
}

// canonical w*y mod q
__device__ __forceinline__ u64 shoup_mul(u64 y, u64 w, u64 w_sh, u64 q) { return csub(shoup_lazy(y, w, w_sh, q), q); }

// x mod q for x < 2^(bits+63), mu = floor(2^(bits+63)/q): quotient estimate is at most 2 low.
__device__ __forceinline__ u64 barrett128(u128 x, u64 q, u64 mu, uint32_t bits) {
    u64 x1 = (u64)(x >> (bits - 1));
    u64 qh = mulhi64(x1, mu);
    u64 r = (u64)x - qh * q;
    r = csub(r, 2 * q);
    return csub(r, q);
}

// Same with the three-product quotient and no final correction: result in [0, 5q), congruent to x.
__device__ __forceinline__ u64 barrett128_lazy(u128 x, u64 q, u64 mu, uint32_t bits) {
    u64 x1 = (u64)(x >> (bits - 1));
    u64 qh = mulhi64_approx(x1, mu);
    return (u64)x - qh * q;
}

// x mod q for a single word x (any value), through the same Barrett constant.
__device__ __forceinline__ u64 barrett64(u64 x, u64 q, u64 mu, uint32_t bits) { return barrett128((u128)x, q, mu, bits); }

__device__ __forceinline__ u64 addmod(u64 a, u64 b, u64 q) { return csub(a + b, q); }
__device__ __forceinline__ u64 submod(u64 a, u64 b, u64 q) { return a >= b ? a - b : a + q - b; }

__device__ __forceinline__ u64 mulmod(u64 a, u64 b, const ModConst& m) { return barrett128((u128)a * b, m.q, m.mu, m.bits); }
