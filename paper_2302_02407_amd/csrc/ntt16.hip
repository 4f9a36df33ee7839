// N = 2^16 fast path of the negacyclic NTT / iNTT (ring of paper Section 2.1).
//
// The limb is viewed as 256 x 256 (row-major).  A transform is two launches of 8 stages:
//   forward : pass A on columns (stages 0..7, row distance 128..1), pass B on rows (stages 8..15);
//   inverse : pass B on rows (stages 15..8), pass A on columns (stages 7..0) + final scaling.
// Inside a pass every thread keeps 16 points of one 256-point sub-transform in registers and
// runs 4 butterfly stages on them, then the 16 threads of the sub-transform exchange points
// through LDS and run the other 4 stages: one LDS round trip replaces eight.  Points are held
// either "strided" (thread t holds e = t + 16k, k-distance 8,4,2,1 = point distance 128..16) or
// "contiguous" (e = 16t + j, point distance 8..1).
//
// Arithmetic: Harvey butterflies with Shoup twiddles whose quotient is taken from three 32-bit
// products, so a twiddle product lands in [0,4q).  For moduli below 2^57 the forward butterflies
// never reduce: each stage adds at most 4q to the bound, 16 stages stay below 65q < 2^64, and
// one small-quotient reduction canonicalises at the very end.  Wider moduli (below 2^60) keep
// [0,8q) with one conditional subtraction of 4q per butterfly.  The inverse keeps [0,4q)
// throughout (sums are reduced, differences re-enter through the twiddle product).
#include "modarith.h"
#include "ntt_blocks.h"

#define T16_THREADS 256

// Forward outputs may stay unreduced (below 69q) when the modulus is below 2^63/552: then a sum of
// 8 products of such a value with a canonical one still fits the 128-bit Barrett input range.
#define LAZY_Q_MAX ((1ull << 63) / 552)

struct Ntt16Args {
    uint32_t lazy;      // forward, last pass: leave outputs unreduced where LAZY_Q_MAX allows
    uint32_t rs_mod;    // forward, first pass reading the Rescale rounding term: modulus index of the dropped limb
    u64* dst;           // limb i is written / transformed in place at dst + i*N
    const ModConst* mc;
    const u64* tw;      // [M][N] forward or inverse twiddles
    const u64* tw_sh;
};
// Where the first pass reads limb i: segment (limb[i] >> 12) at limb offset (limb[i] & 0xFFF).
struct SrcList {
    const u64* seg[HE_MAX_SEGS];
    uint16_t limb[HE_MAX_LAUNCH_LIMBS];
};
__device__ __forceinline__ const u64* src_of(const SrcList& sl, uint32_t limb) {
    const uint32_t e = sl.limb[limb];
    return sl.seg[e >> 12] + ((size_t)(e & 0xFFFu) << 16);
}
// Work order of the row passes.  Their twiddles depend on (modulus, tile), so limbs that share a
// modulus should run the same tile back to back on the same XCD (one L2 per XCD; workgroups are
// handed to the 8 XCDs round-robin).  order[] lists the live limbs sorted by modulus, padded with
// 0xFFFF to a multiple of the chunk size C = 1 << log_chunk; the linear work index
// L = (chunk_of_limbs*16 + tile)*C + j walks the C limbs of a chunk for one tile, and
// workgroup id -> L keeps each run of C consecutive L on one XCD.
struct RowSched {
    uint16_t order[HE_MAX_LAUNCH_LIMBS];
    uint32_t log_chunk;
};

__device__ __forceinline__ bool row_sched_decode(const RowSched& rs, uint32_t& limb, uint32_t& tile) {
    const uint32_t lc = rs.log_chunk, idx = blockIdx.x;
    const uint32_t xcd = idx & 7u, slot = idx >> 3;
    const uint32_t L = ((((slot >> lc) << 3) + xcd) << lc) | (slot & ((1u << lc) - 1u));
    const uint32_t pchunk = L >> (4 + lc), rem = L & ((16u << lc) - 1u);
    tile = rem >> lc;
    limb = rs.order[(pchunk << lc) + (rem & ((1u << lc) - 1u))];
    return limb != 0xFFFFu;
}

// Inverse stages for moduli below 2^54 with no reduction at all: sums are left to grow and differences are taken
// against a multiple of q that covers the inputs.  With inputs below 2^log_b * q a stage leaves sums below
// 2^(log_b+1) * q and twiddle products below 4q, so the bound of the next stage is 2^max(log_b+1, 2) * q.  Eight
// stages from canonical inputs stay below 512 q < 2^63.
template <int STAGES>
__device__ __forceinline__ void inv_block_lazy(u64 (&x)[16], const u64* __restrict__ tw, const u64* __restrict__ tw_sh,
                                               uint32_t s0, uint32_t G, u64 q, uint32_t log_b) {
#pragma unroll
    for (int u = 3; u > 3 - STAGES; u--) {
        const int dist = 8 >> u;
        const uint32_t base = (1u << (s0 + u)) + (G << u);
        const u64 bq = q << log_b;                       // covers every input of this stage
#pragma unroll
        for (int g = 0; g < (1 << u); g++) {
            const u64 w = tw[base + g], w_sh = tw_sh[base + g];
#pragma unroll
            for (int k = 0; k < dist; k++) {
                const int a = g * 2 * dist + k;
                const u64 X = x[a], Y = x[a + dist];
                x[a] = X + Y;
                x[a + dist] = shoup_lazy4((X + bq) - Y, w, w_sh, q);
            }
        }
        // sums double the bound; twiddle products are below 4q
        log_b = log_b + 1 < 2 ? 2 : log_b + 1;
    }
}

// Inverse stages 3, 2, 1 of the limb (the first three of the last register block); stage 0 is done by
// the caller together with the output scaling.
__device__ __forceinline__ void inv_block3(u64 (&x)[16], const u64* __restrict__ tw, const u64* __restrict__ tw_sh, u64 q, u64 q4) {
#pragma unroll
    for (int u = 3; u >= 1; u--) {
        const int dist = 8 >> u;
        const uint32_t base = 1u << u;
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

// Inner product of four points over the digits: sum[k] += digit_j[src[k]] * key_j[16 k] for j < beta, JW digits
// at a time so that their loads are in flight together.  JW = 3 is the exact form for three digits (the paper's
// dnum at the top levels): no padding digit, no predicates; the caller guarantees beta == 3.  Digit own_j is read
// from `own` (the switched polynomial's limb itself), the others from raised + j * dig_stride.
template <int JW>
__device__ __forceinline__ void ip_accumulate(u128 (&sum)[4], const u64* __restrict__ raised, const u64* __restrict__ own, uint32_t own_j,
                                              const u64* __restrict__ key, size_t dig_stride, size_t key_stride, uint32_t beta,
                                              const uint32_t (&src)[4]) {
    for (uint32_t j0 = 0; j0 < (JW == 3 ? 3u : beta); j0 += JW) {
        u64 dv[JW][4], kv[JW][4];
#pragma unroll
        for (uint32_t jj = 0; jj < (uint32_t)JW; jj++) {
            const uint32_t j = j0 + jj;
            const bool live = JW == 3 || j < beta;
            const u64* dj = j == own_j ? own : raised + (live ? j : 0) * dig_stride;
            const u64* kj = key + (live ? j : 0) * key_stride;
#pragma unroll
            for (int k = 0; k < 4; k++) {
                dv[jj][k] = live ? dj[src[k]] : 0;
                kv[jj][k] = live ? kj[16 * k] : 0;
            }
        }
#pragma unroll
        for (uint32_t jj = 0; jj < (uint32_t)JW; jj++)
#pragma unroll
            for (int k = 0; k < 4; k++) sum[k] += (u128)dv[jj][k] * kv[jj][k];
    }
}

// ---------------------------------------------------------------- forward
// Pass A: workgroup = 16 adjacent columns x all 256 rows of one limb; tid = t*16 + col.
// RS: the source is the coefficient form of the limb that Rescale drops (modulus ml); what is transformed is the negated
// rounding term ((v + h) mod q_l) mod q - (h mod q), h = floor(q_l / 2), of this limb's modulus m.
template <bool WIDE, bool RS>
__device__ __forceinline__ void fwd_pass_a(const u64* __restrict__ src, u64* __restrict__ dst, u64* sm, const u64* tw,
                                           const u64* tw_sh, uint32_t tile, u64 q, u64 q4, const ModConst& m, const ModConst& ml) {
    const uint32_t t = threadIdx.x >> 4, cl = threadIdx.x & 15, c = tile * 16 + cl;
    u64 x[16];
#pragma unroll
    for (int k = 0; k < 16; k++) x[k] = src[(size_t)(t + 16 * k) * 256 + c];
    if (RS) {
        const u64 h = ml.q >> 1, hr = barrett64(h, m.q, m.mu, m.bits);
#pragma unroll
        for (int k = 0; k < 16; k++) x[k] = submod(barrett64(addmod(x[k], h, ml.q), m.q, m.mu, m.bits), hr, q);
    }
    fwd_block4<WIDE>(x, tw, tw_sh, 0, 0, q, q4);
    // row r of the tile sits at (r + (r >> 4)) * 16: one spare row per 16 keeps the four row groups
    // that a wavefront reads back at once on different banks
#pragma unroll
    for (int k = 0; k < 16; k++) sm[(t + 17 * k) * 16 + cl] = x[k];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 16; j++) x[j] = sm[(17 * t + j) * 16 + cl];
    fwd_block4<WIDE>(x, tw, tw_sh, 4, t, q, q4);
#pragma unroll
    for (int j = 0; j < 16; j++) dst[(size_t)(16 * t + j) * 256 + c] = x[j];
}

__device__ __forceinline__ uint32_t galois_src16(uint32_t j, uint32_t g) {
    uint32_t k = __brev(j) >> 16;
    uint32_t kp = (g * k + ((g - 1) >> 1)) & 0xFFFFu;
    return __brev(kp) >> 16;
}

// Pass B: workgroup = 16 consecutive rows (256-point blocks); tid = blk*16 + t.  With EPI the
// canonical result is not stored: it feeds the ModDown epilogue, which writes the outputs.  The
// epilogue's operands (accumulator, rotated c0, the ciphertext itself) are fetched before the
// butterflies start so that their latency is hidden behind the arithmetic.
// EPI: 0 = plain transform; 1 = ModDown epilogue with the accumulator read from memory; 2 = ModDown epilogue
// that also computes the accumulator (the key-switch inner product of this limb) from the raised digits and
// the key, so that the q-limbs of the accumulator never exist in memory.
template <bool WIDE, int EPI>
__device__ __forceinline__ void fwd_pass_b(u64* __restrict__ data, u64* sm, const u64* tw, const u64* tw_sh, uint32_t tile,
                                           const ModConst& m, uint32_t mrec, const ModDownEpilogue& ep, uint32_t limb, bool lazy) {
    const u64 q = m.q, q2 = m.q2, q4 = 2 * m.q2;
    const bool keep_lazy = !WIDE && lazy && q < LAZY_Q_MAX;
    const uint32_t blk = threadIdx.x >> 4, t = threadIdx.x & 15, b = tile * 16 + blk;
    u64* row = data + (size_t)b * 256;
    u64* s = sm + blk * 272;                            // 16 groups of 17: conflict-free both ways
    u64 x[16];
#pragma unroll
    for (int k = 0; k < 16; k++) x[k] = row[t + 16 * k];
    // epilogue operands for the points e = t + 16k this thread will finally own
    u64 ea[EPI == 1 ? 16 : 1], ec[EPI == 1 ? 16 : 1];
    u64* out = nullptr;
    u64 pinv = 0, pinv_sh = 0;
    bool has_c0 = false, has_self = false;
    const u64* self = nullptr;
    const u64* c0 = nullptr;
    uint32_t g = 1, r = 0, job = 0, comp = 0;
    if (EPI) {
        const uint32_t pc = limb / ep.L1;
        r = limb - pc * ep.L1; job = pc >> 1; comp = pc & 1u;
        pinv = ep.pinv[r]; pinv_sh = ep.pinv_sh[r];
        out = (comp ? ep.out1[job] : ep.out0[job]) + ((size_t)r << 16) + (size_t)b * 256;
        c0 = (comp == 0 && ep.c0[job]) ? ep.c0[job] + ((size_t)r << 16) : nullptr;
        has_c0 = c0 != nullptr;
        const u64* sp = comp ? ep.self1[job] : ep.self0[job];
        has_self = sp != nullptr;
        self = has_self ? sp + ((size_t)r << 16) + (size_t)b * 256 : nullptr;
        g = ep.g[ep.n_terms ? 0 : job];
        if (EPI == 1) {
            const u64* acc = ep.acc + ((size_t)(pc * ep.R + r) << 16) + (size_t)b * 256;
#pragma unroll
            for (int k = 0; k < 16; k++) {
                const uint32_t e = t + 16 * k;
                ea[k] = acc[e];
                ec[k] = has_c0 ? c0[g == 1 ? b * 256 + e : galois_src16(b * 256 + e, g)] : 0;
            }
        }
    }
    fwd_block4<WIDE>(x, tw, tw_sh, 8, b, q, q4);
#pragma unroll
    for (int k = 0; k < 16; k++) s[t + 17 * k] = x[k];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 16; j++) x[j] = s[17 * t + j];
    fwd_block4<WIDE>(x, tw, tw_sh, 12, 16 * b + t, q, q4);
    if (!keep_lazy) {
#pragma unroll
        for (int j = 0; j < 16; j++) x[j] = WIDE ? csub(csub(csub(x[j], q4), q2), q) : reduce_small(x[j], q, m.bits, mrec);
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 16; j++) s[17 * t + j] = x[j];
    __syncthreads();
    // (acc - ntt) * P^-1 lazily in [0,4q), plus up to two canonical addends: below 6q; the transform value is
    // below 128q when left unreduced, canonical otherwise
    const u64 bias = keep_lazy ? (q << 7) : q;
    if (EPI == 0) {
#pragma unroll
        for (int k = 0; k < 16; k++) row[t + 16 * k] = s[t + 17 * k];
    } else if (EPI == 1) {
#pragma unroll
        for (int k = 0; k < 16; k++) {
            const uint32_t e = t + 16 * k;
            u64 v = shoup_lazy4(ea[k] + bias - s[t + 17 * k], pinv, pinv_sh, q) + ec[k];
            if (has_self) v += self[e];
            out[e] = csub(csub(csub(v, q4), q2), q);
        }
    } else {
        // digit j of limb r is the switched polynomial itself where limb r belongs to digit j, else the raised
        // digit; four points at a time so that their loads are in flight together.  With ep.n_terms > 0 the
        // launch serves one output whose accumulator is the sum over n_terms (polynomial, Galois element, key)
        // terms - a sum of rotations with one ModDown - and the per-job arrays are indexed by term.
        const uint32_t beta = ep.beta, own_j = r / ep.alpha, n_terms = ep.n_terms ? ep.n_terms : 1u;
        const size_t dig_stride = (size_t)ep.R << 16, key_stride = (size_t)(2 * ep.M) << 16;
        if (EPI == 3) {
            // one digit (the low levels the paper's networks run at): every q-limb is the digit's own, and all 16
            // points' operands are fetched at once - at these sizes a launch is a few work groups per CU and its time
            // is the length of its dependent load chains
            const u64* own = ep.own[job] + ((size_t)r << 16);
            const u64* key = ep.evk[job] + ((size_t)(comp * ep.M + r) << 16) + (size_t)b * 256;
            u64 dv[16], kv[16], cv[16], sv[16];
#pragma unroll
            for (int k = 0; k < 16; k++) {
                const uint32_t e = t + 16 * k;
                const uint32_t src = g == 1 ? b * 256 + e : galois_src16(b * 256 + e, g);
                dv[k] = own[src];
                kv[k] = key[e];
                cv[k] = has_c0 ? c0[src] : 0;
                sv[k] = has_self ? self[e] : 0;
            }
#pragma unroll
            for (int k = 0; k < 16; k++) {
                const uint32_t e = t + 16 * k;
                const u64 a = barrett128_lazy((u128)dv[k] * kv[k], q, m.mu, m.bits);
                const u64 v = shoup_lazy4(a + bias - s[t + 17 * k], pinv, pinv_sh, q) + cv[k] + sv[k];
                out[e] = csub(csub(csub(v, q4), q2), q);
            }
            return;
        }
#pragma unroll
        for (int k0 = 0; k0 < 16; k0 += 4) {
            u64 tot[4] = {0, 0, 0, 0};
            uint32_t src[4];
            u64 cv[4], sv[4];
#pragma unroll
            for (int k = 0; k < 4; k++) {
                const uint32_t e = t + 16 * (k0 + k);
                src[k] = g == 1 ? b * 256 + e : galois_src16(b * 256 + e, g);     // g = Galois element of the job / of term 0
                cv[k] = has_c0 ? c0[src[k]] : 0;
                sv[k] = has_self ? self[e] : 0;
            }
            // The products of all terms and digits go into one 128-bit sum per point, reduced whenever eight
            // products are pending (the raised digits may be unreduced, below 69q: eight products stay below
            // 2^(bits+63)).  Partial sums are reduced to [0, 5q) only (three-product quotient, no correction) and added
            // up: at most 7 of them (16 terms of 3 digits), below 35q, and the P^-1 product below takes any 64-bit
            // value; for the widest moduli they are kept canonical instead.
            u128 sum[4] = {0, 0, 0, 0};
            uint32_t pending = 0;
            for (uint32_t term = 0; term < n_terms; term++) {
                const uint32_t idx = ep.n_terms ? term : job;
                const u64* own = ep.own[idx] + ((size_t)r << 16);
                const u64* raised = ep.raised[idx] + ((size_t)r << 16);
                const u64* key = ep.evk[idx] + ((size_t)(comp * ep.M + r) << 16) + (size_t)b * 256;
                if (term) {
                    const uint32_t gt = ep.g[idx];
#pragma unroll
                    for (int k = 0; k < 4; k++) {
                        const uint32_t e = t + 16 * (k0 + k);
                        src[k] = gt == 1 ? b * 256 + e : galois_src16(b * 256 + e, gt);
                    }
                    if (pending + beta > 8) {
#pragma unroll
                        for (int k = 0; k < 4; k++) {
                            tot[k] = WIDE ? addmod(tot[k], barrett128(sum[k], q, m.mu, m.bits), q) : tot[k] + barrett128_lazy(sum[k], q, m.mu, m.bits);
                            sum[k] = 0;
                        }
                        pending = 0;
                    }
                }
                if (beta == 3) ip_accumulate<3>(sum, raised, own, own_j, key + t + 16 * k0, dig_stride, key_stride, beta, src);
                else ip_accumulate<4>(sum, raised, own, own_j, key + t + 16 * k0, dig_stride, key_stride, beta, src);
                pending += beta;
            }
#pragma unroll
            for (int k = 0; k < 4; k++)
                tot[k] = WIDE ? addmod(tot[k], barrett128(sum[k], q, m.mu, m.bits), q) : tot[k] + barrett128_lazy(sum[k], q, m.mu, m.bits);
#pragma unroll
            for (int k = 0; k < 4; k++) {
                const uint32_t e = t + 16 * (k0 + k);
                const u64 v = shoup_lazy4(tot[k] + bias - s[e + k0 + k], pinv, pinv_sh, q) + cv[k] + sv[k];
                out[e] = csub(csub(csub(v, q4), q2), q);
            }
        }
    }
}

template <bool RS>
__global__ __launch_bounds__(T16_THREADS) void ntt16_fwd_a_kernel(Ntt16Args a, LimbList ll, SrcList sl) {
    __shared__ u64 sm[272 * 16];
    const uint32_t limb = blockIdx.x >> 4, tile = blockIdx.x & 15;
    const uint32_t mi = ll.mod[limb];
    if (mi == 0xFFu) return;
    const ModConst m = a.mc[mi];
    const ModConst ml = a.mc[RS ? a.rs_mod : mi];
    const u64* src = src_of(sl, limb);
    u64* dst = a.dst + ((size_t)limb << 16);
    const u64* tw = a.tw + ((size_t)mi << 16);
    const u64* tw_sh = a.tw_sh + ((size_t)mi << 16);
    if (m.bits > 57) fwd_pass_a<true, RS>(src, dst, sm, tw, tw_sh, tile, m.q, 2 * m.q2, m, ml);
    else fwd_pass_a<false, RS>(src, dst, sm, tw, tw_sh, tile, m.q, 2 * m.q2, m, ml);
}

template <int EPI>
__global__ __launch_bounds__(T16_THREADS) void ntt16_fwd_b_kernel(Ntt16Args a, LimbList ll, RowSched rs, ModDownEpilogue ep) {
    __shared__ u64 sm[16 * 272];
    uint32_t limb, tile;
    if (!row_sched_decode(rs, limb, tile)) return;
    const uint32_t mi = ll.mod[limb];
    const ModConst m = a.mc[mi];
    u64* data = a.dst + ((size_t)limb << 16);
    const u64* tw = a.tw + ((size_t)mi << 16);
    const u64* tw_sh = a.tw_sh + ((size_t)mi << 16);
    if (m.bits > 57) {
        fwd_pass_b<true, EPI>(data, sm, tw, tw_sh, tile, m, 0, ep, limb, false);
    } else {
        const uint32_t mrec = (1u << 24) / ((uint32_t)(m.q >> (m.bits - 8)) + 1);
        fwd_pass_b<false, EPI>(data, sm, tw, tw_sh, tile, m, mrec, ep, limb, a.lazy != 0);
    }
}

// ---------------------------------------------------------------- inverse
// Pass B (rows) first: stages 15..12 on contiguous points, exchange, stages 11..8 on strided points.
// With IP the inputs are not read: they are the key-switch inner product of the special-prime limbs, computed
// here from the raised digits and the key (four points at a time so that their loads are in flight together).
template <bool IP>
__global__ __launch_bounds__(T16_THREADS) void ntt16_inv_b_kernel(Ntt16Args a, LimbList ll, SrcList sl, RowSched rs, IpPrologue ip) {
    __shared__ u64 sm[16 * 272];
    uint32_t limb, tile;
    if (!row_sched_decode(rs, limb, tile)) return;
    const uint32_t mi = ll.mod[limb];
    const ModConst m = a.mc[mi];
    const u64 q = m.q, q4 = 2 * m.q2;
    const u64* tw = a.tw + ((size_t)mi << 16);
    const u64* tw_sh = a.tw_sh + ((size_t)mi << 16);
    const uint32_t blk = threadIdx.x >> 4, t = threadIdx.x & 15, b = tile * 16 + blk;
    const u64* in = src_of(sl, limb) + (size_t)b * 256;
    u64* out = a.dst + ((size_t)limb << 16) + (size_t)b * 256;
    u64* s = sm + blk * 272;
    u64 x[16];
    if (!IP) {
#pragma unroll
        for (int k = 0; k < 16; k++) s[t + 17 * k] = in[t + 16 * k];
    } else {
        // with ip.n_terms > 0 the launch serves one output whose accumulator is the sum over n_terms
        // (polynomial, Galois element, key) terms and the per-job arrays are indexed by term
        const uint32_t pc = limb / ip.k, tp = limb - pc * ip.k, job = pc >> 1, comp = pc & 1u;
        const uint32_t beta = ip.beta, n_terms = ip.n_terms ? ip.n_terms : 1u;
        const size_t dig_stride = (size_t)ip.R << 16, key_stride = (size_t)(2 * ip.M) << 16;
        if (beta == 1 && ip.n_terms == 0) {
            // one digit: all 16 points' operands fetched at once (see the epilogue of the forward row pass)
            const uint32_t g = ip.g[job];
            const u64* raised = ip.raised[job] + ((size_t)(ip.L1 + tp) << 16);
            const u64* key = ip.evk[job] + ((size_t)(comp * ip.M + ip.nq + tp) << 16) + (size_t)b * 256;
            u64 dv[16], kv[16];
#pragma unroll
            for (int k = 0; k < 16; k++) {
                const uint32_t e = t + 16 * k;
                dv[k] = raised[g == 1 ? b * 256 + e : galois_src16(b * 256 + e, g)];
                kv[k] = key[e];
            }
#pragma unroll
            for (int k = 0; k < 16; k++) s[t + 17 * k] = barrett128((u128)dv[k] * kv[k], q, m.mu, m.bits);
        } else
#pragma unroll
        for (int k0 = 0; k0 < 16; k0 += 4) {
            // all terms and digits into one 128-bit sum per point, reduced (to the canonical residue the transform
            // expects) whenever eight products are pending
            u64 tot[4] = {0, 0, 0, 0};
            u128 sum[4] = {0, 0, 0, 0};
            uint32_t pending = 0;
            for (uint32_t term = 0; term < n_terms; term++) {
                const uint32_t idx = ip.n_terms ? term : job;
                const uint32_t g = ip.g[idx];
                const u64* raised = ip.raised[idx] + ((size_t)(ip.L1 + tp) << 16);
                const u64* key = ip.evk[idx] + ((size_t)(comp * ip.M + ip.nq + tp) << 16) + (size_t)b * 256;
                uint32_t src[4];
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    const uint32_t e = t + 16 * (k0 + k);
                    src[k] = g == 1 ? b * 256 + e : galois_src16(b * 256 + e, g);
                }
                if (pending + beta > 8) {
#pragma unroll
                    for (int k = 0; k < 4; k++) {
                        tot[k] = addmod(tot[k], barrett128(sum[k], q, m.mu, m.bits), q);
                        sum[k] = 0;
                    }
                    pending = 0;
                }
                if (beta == 3) ip_accumulate<3>(sum, raised, nullptr, 0xFFFFFFFFu, key + t + 16 * k0, dig_stride, key_stride, beta, src);
                else ip_accumulate<4>(sum, raised, nullptr, 0xFFFFFFFFu, key + t + 16 * k0, dig_stride, key_stride, beta, src);
                pending += beta;
            }
#pragma unroll
            for (int k = 0; k < 4; k++) s[t + 17 * (k0 + k)] = addmod(tot[k], barrett128(sum[k], q, m.mu, m.bits), q);
        }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 16; j++) x[j] = s[17 * t + j];
    // moduli below 2^54: no reduction inside the pass.  Canonical inputs: bounds (in units of q) 1 -> 4 -> 8 -> 16
    // -> 32 after the first block, -> 512 after the second; one quotient step brings the outputs back below 4q.
    const bool lazy = m.bits <= 54;
    if (lazy) inv_block_lazy<4>(x, tw, tw_sh, 12, 16 * b + t, q, 0);
    else inv_block4(x, tw, tw_sh, 12, 16 * b + t, q, q4);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 16; j++) s[17 * t + j] = x[j];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) x[k] = s[t + 17 * k];
    if (lazy) {
        inv_block_lazy<4>(x, tw, tw_sh, 8, b, q, 5);
        const u64 one_sh = m.one_sh;                     // floor(2^64 / q): the Shoup companion of the constant 1
#pragma unroll
        for (int k = 0; k < 16; k++) x[k] = shoup_lazy4(x[k], 1, one_sh, q);
    } else {
        inv_block4(x, tw, tw_sh, 8, b, q, q4);
    }
#pragma unroll
    for (int k = 0; k < 16; k++) out[t + 16 * k] = x[k];
}

// Pass A (columns): stages 7..4 on rows 16t+j, exchange, stages 3..0 on rows t+16k, final scale.
template <bool CUSTOM_SCALE>
__global__ __launch_bounds__(T16_THREADS) void ntt16_inv_a_kernel(Ntt16Args a, LimbList ll, ScaleList sc, uint32_t scale_period) {
    __shared__ u64 sm[4096];
    const uint32_t limb = blockIdx.x >> 4, tile = blockIdx.x & 15;
    const uint32_t mi = ll.mod[limb];
    if (mi == 0xFFu) return;
    const ModConst m = a.mc[mi];
    const u64 q = m.q, q2 = m.q2, q4 = 2 * m.q2;
    const u64* tw = a.tw + ((size_t)mi << 16);
    const u64* tw_sh = a.tw_sh + ((size_t)mi << 16);
    u64* data = a.dst + ((size_t)limb << 16);
    const uint32_t t = threadIdx.x >> 4, cl = threadIdx.x & 15, c = tile * 16 + cl;
    u64 x[16];
#pragma unroll
    for (int j = 0; j < 16; j++) x[j] = data[(size_t)(16 * t + j) * 256 + c];
    inv_block4(x, tw, tw_sh, 4, t, q, q4);
#pragma unroll
    for (int j = 0; j < 16; j++) sm[(16 * t + j) * 16 + cl] = x[j];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) x[k] = sm[(t + 16 * k) * 16 + cl];
    inv_block3(x, tw, tw_sh, q, q4);
    // stage 0 (one twiddle for the whole limb) with the output scaling folded in: the sum is
    // multiplied by the scale, the difference by scale * twiddle
    const uint32_t si = CUSTOM_SCALE ? limb % scale_period : 0;
    const u64 cs = CUSTOM_SCALE ? sc.s[si] : m.ninv, cs_sh = CUSTOM_SCALE ? sc.s_sh[si] : m.ninv_sh;
    const u64 cw = CUSTOM_SCALE ? sc.w[si] : m.ninv_w, cw_sh = CUSTOM_SCALE ? sc.w_sh[si] : m.ninv_w_sh;
#pragma unroll
    for (int k = 0; k < 8; k++) {
        const u64 X = x[k], Y = x[k + 8];
        x[k] = shoup_lazy4(X + Y, cs, cs_sh, q);
        x[k + 8] = shoup_lazy4((X + q4) - Y, cw, cw_sh, q);
    }
#pragma unroll
    for (int k = 0; k < 16; k++) data[(size_t)(t + 16 * k) * 256 + c] = csub(csub(x[k], q2), q);
}

// ---------------------------------------------------------------- column passes fused around the basis conversion
// Latency path for small launches (a few limbs: the low levels the paper's networks run at), where the chip is mostly
// idle and a call is bound by its chain of dependent launches.  The last inverse pass, the basis conversion and the
// first forward pass all work on columns of the 256 x 256 view, so one work group takes ONE column through all
// three: every source limb of a group (a digit of ModUp, the special-prime limbs of one ModDown component; at most 8)
// goes through the inverse column stages and its output scaling into LDS, then every target limb is converted from
// those (128-bit sums, lazy Barrett), run through the forward column stages and written.  One launch instead of
// three; the coefficient-form limbs and the converted limbs never exist in memory.  One wavefront per limb, four
// points per lane (two stages in registers, then an exchange through LDS), so that a conversion of a single digit
// already spreads over every compute unit; the 8-byte accesses this makes (a column is strided by 2 KiB) cost
// bandwidth that a launch this small does not need.
#define CF_THREADS 512
#define CF_WAVES 8
#define CF_EX 272            // 256 points + one spare per 16

__device__ __forceinline__ uint32_t cf_pos(uint32_t i) { return i + (i >> 4); }

__global__ __launch_bounds__(CF_THREADS) void ntt16_colfuse_kernel(ColFuse cf, ScaleList sc, const ModConst* mc, const u64* tw,
                                                                   const u64* tw_sh, const u64* itw, const u64* itw_sh) {
    __shared__ u64 ys[CF_WAVES * 256];
    __shared__ u64 ex[CF_WAVES * CF_EX];
    // work groups go to the XCDs round-robin: give each XCD 32 adjacent columns, so that the sixteen columns that
    // share a 128-byte line are read and written through one L2
    const uint32_t g = blockIdx.x >> 8, c = (blockIdx.x & 7) * 32 + ((blockIdx.x >> 3) & 31);
    const uint32_t w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const CfGroup gp = cf.grp[g];
    const uint32_t ns = gp.ns, set = gp.set, nt = cf.nt[set];
    u64* exw = ex + w * CF_EX;
    u64 x[4];
    // Everything a wavefront will need is requested before anything is computed, so that the dependent memory round
    // trips (arguments -> constants of the modulus -> data and twiddles) are paid once, not once per phase: the source
    // limb's points and all its twiddles, and for the first target limb its modulus and conversion constants.
    const bool src_on = w < ns;
    const uint32_t mi = gp.mod0 + (src_on ? w : 0);
    const u64* data = gp.src + ((size_t)(src_on ? w : 0) << 16) + c;
    if (src_on) {
#pragma unroll
        for (int k = 0; k < 4; k++) x[k] = data[(size_t)(4 * lane + k) * 256];
    }
    u64 t1[4][6];
#pragma unroll
    for (int blk = 0; blk < 4; blk++) tw_block2(t1[blk], itw + ((size_t)mi << 16), itw_sh + ((size_t)mi << 16), 2 * blk, lane >> (6 - 2 * blk));
    const ModConst m1 = mc[mi];
    const uint32_t si = gp.sc0 + (src_on ? w : 0);
    const u64 cs = sc.s[si], cs_sh = sc.s_sh[si];
    uint32_t mr = cf.tgt_mod[set][w < nt ? w : 0];
    ModConst m2 = mc[mr];
    u64 hat[CF_WAVES];                                       // a row of the table is padded to 8 entries, zeros past ns
#pragma unroll
    for (int i = 0; i < CF_WAVES; i++) hat[i] = gp.hat[(size_t)mr * cf.hat_w + i];
    {   // inverse column stages 7..0 of source w (wavefronts beyond the group's sources idle through the barriers)
        const u64 q = m1.q, q4 = 2 * m1.q2;
#pragma unroll
        for (int blk = 3; blk >= 0; blk--) {
            const uint32_t s0 = 2 * blk, log_span = 6 - s0, span = 1u << log_span;
            const uint32_t G = lane >> log_span, base = (G << (8 - s0)) + (lane & (span - 1));
            if (blk < 3) {
                __syncthreads();
                if (src_on) {
#pragma unroll
                    for (int k = 0; k < 4; k++) x[k] = exw[cf_pos(base + (k << log_span))];
                }
            }
            if (src_on) {
                inv_block2_r(x, t1[blk], q, q4);
                if (blk > 0) {
#pragma unroll
                    for (int k = 0; k < 4; k++) exw[cf_pos(base + (k << log_span))] = x[k];
                } else {
#pragma unroll
                    for (int k = 0; k < 4; k++) ys[w * 256 + lane + 64 * k] = csub(shoup_lazy(x[k], cs, cs_sh, q), q);
                }
            }
        }
    }
    for (uint32_t t0 = 0; t0 < nt; t0 += CF_WAVES) {
        const uint32_t ti = t0 + w;
        const bool active = ti < nt;
        if (t0) {                                            // later rounds fetch their constants as they start
            mr = cf.tgt_mod[set][active ? ti : 0];
            m2 = mc[mr];
#pragma unroll
            for (int i = 0; i < CF_WAVES; i++) hat[i] = gp.hat[(size_t)mr * cf.hat_w + i];
        }
        u64 t2[4][6];
#pragma unroll
        for (int blk = 0; blk < 4; blk++) tw_block2(t2[blk], tw + ((size_t)mr << 16), tw_sh + ((size_t)mr << 16), 2 * blk, lane >> (6 - 2 * blk));
        __syncthreads();                                     // the sources are in ys (first round)
        const u64 q = m2.q, q4 = 2 * m2.q2;
        const bool wide = m2.bits > 57;
        if (active) {
            u128 acc[4] = {};
#pragma unroll
            for (int i = 0; i < CF_WAVES; i++) {
                if ((uint32_t)i < ns) {
#pragma unroll
                    for (int k = 0; k < 4; k++) acc[k] += (u128)ys[i * 256 + lane + 64 * k] * hat[i];
                }
            }
#pragma unroll
            for (int k = 0; k < 4; k++) x[k] = barrett128_lazy(acc[k], q, m2.mu, m2.bits);      // below 5q
        }
#pragma unroll
        for (int blk = 0; blk < 4; blk++) {
            const uint32_t s0 = 2 * blk, log_span = 6 - s0, span = 1u << log_span;
            const uint32_t G = lane >> log_span, base = (G << (8 - s0)) + (lane & (span - 1));
            if (blk > 0) {
                __syncthreads();
                if (active) {
#pragma unroll
                    for (int k = 0; k < 4; k++) x[k] = exw[cf_pos(base + (k << log_span))];
                }
            }
            if (active) {
                if (wide) fwd_block2_r<true>(x, t2[blk], q, q4);
                else fwd_block2_r<false>(x, t2[blk], q, q4);
                if (blk < 3) {
#pragma unroll
                    for (int k = 0; k < 4; k++) exw[cf_pos(base + (k << log_span))] = x[k];
                }
            }
        }
        if (active) {
            u64* dst = gp.dst + ((size_t)cf.tgt_limb[set][ti] << 16) + c;
#pragma unroll
            for (int k = 0; k < 4; k++) dst[(size_t)(4 * lane + k) * 256] = x[k];
        }
    }
}

int32_t launch_colfuse(he_ctx* ctx, const ColFuse& cf, const ScaleList& sc, uint32_t limb_passes) {
    if (cf.n_groups == 0) return HE_OK;
    if (cf.n_groups > CF_MAX_GROUPS) return he_fail(ctx, HE_ERR_BADARG, "column fusion: too many groups");
    for (uint32_t g = 0; g < cf.n_groups; g++)
        if (cf.grp[g].ns == 0 || cf.grp[g].ns > CF_WAVES || cf.grp[g].set >= CF_MAX_SETS || cf.grp[g].mod0 + cf.grp[g].ns > ctx->M ||
            cf.grp[g].sc0 + cf.grp[g].ns > HE_MAX_MODULI || !cf.grp[g].src || !cf.grp[g].dst || !cf.grp[g].hat)
            return he_fail(ctx, HE_ERR_BADARG, "column fusion: bad group %u", g);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (ctx->prof_on) {
        HE_HIP(ctx, hipEventCreate(&e0));
        HE_HIP(ctx, hipEventCreate(&e1));
        HE_HIP(ctx, hipEventRecord(e0, ctx->stream));
    }
    hipLaunchKernelGGL(ntt16_colfuse_kernel, dim3(cf.n_groups * 256), dim3(CF_THREADS), 0, ctx->stream, cf, sc, ctx->d_mc, ctx->d_tw,
                       ctx->d_tw_sh, ctx->d_itw, ctx->d_itw_sh);
    HE_HIP(ctx, hipGetLastError());
    if (ctx->prof_on) {
        HE_HIP(ctx, hipEventRecord(e1, ctx->stream));
        ctx->prof_events.push_back({e0, e1, limb_passes, 0u, 0u});
    }
    return HE_OK;
}

// ---------------------------------------------------------------- butterfly-rate probe
// The vector-ALU roof of the transforms, measured rather than derived: the register blocks of the passes
// above (four stages on 16 points, twiddles from a 256-entry table that stays in the first-level cache)
// run back to back with no other memory traffic.  Values wrap around after a few rounds; the timing does
// not depend on them.
template <bool FWD, bool WIDE>
__global__ __launch_bounds__(T16_THREADS) void bfly_probe_kernel(const u64* __restrict__ tw, const u64* __restrict__ tw_sh, u64 q,
                                                                 u64* __restrict__ out, uint32_t rounds) {
    const u64 q4 = 4 * q;
    const uint32_t t = threadIdx.x & 15;
    u64 x[16];
#pragma unroll
    for (int k = 0; k < 16; k++) x[k] = (u64)(blockIdx.x * T16_THREADS + threadIdx.x) * 16 + k;
    for (uint32_t r = 0; r < rounds; r++) {
        if (FWD) fwd_block4<WIDE>(x, tw, tw_sh, 4, t, q, q4);
        else if (WIDE) inv_block4(x, tw, tw_sh, 4, t, q, q4);
        else inv_block_lazy<4>(x, tw, tw_sh, 4, t, q, 2);
    }
    u64 v = 0;
#pragma unroll
    for (int k = 0; k < 16; k++) v ^= x[k];
    out[blockIdx.x * T16_THREADS + threadIdx.x] = v;
}

int32_t probe_butterfly_rates(he_ctx* ctx, u64* d_out, uint32_t groups, double rate_out[3]) {
    const uint32_t rounds = 64;                          // 32 butterflies per thread per round
    uint32_t narrow = 0, wide = ctx->M;
    for (uint32_t i = 0; i < ctx->M; i++) if (ctx->h_mc[i].bits > 57) { wide = i; break; }
    hipEvent_t e0, e1;
    HE_HIP(ctx, hipEventCreate(&e0));
    HE_HIP(ctx, hipEventCreate(&e1));
    for (int which = 0; which < 3; which++) {
        const uint32_t mi = which == 2 ? wide : narrow;
        rate_out[which] = 0.0;
        if (mi >= ctx->M || (which != 2 && ctx->h_mc[mi].bits > 57)) continue;
        const u64* tw = (which == 1 ? ctx->d_itw : ctx->d_tw) + (size_t)mi * ctx->N;
        const u64* tw_sh = (which == 1 ? ctx->d_itw_sh : ctx->d_tw_sh) + (size_t)mi * ctx->N;
        for (int rep = 0; rep < 2; rep++) {              // the first launch warms up
            HE_HIP(ctx, hipEventRecord(e0, ctx->stream));
            if (which == 0) hipLaunchKernelGGL((bfly_probe_kernel<true, false>), dim3(groups), dim3(T16_THREADS), 0, ctx->stream, tw, tw_sh, ctx->mod[mi], d_out, rounds);
            else if (which == 1 && ctx->h_mc[mi].bits > 54) hipLaunchKernelGGL((bfly_probe_kernel<false, true>), dim3(groups), dim3(T16_THREADS), 0, ctx->stream, tw, tw_sh, ctx->mod[mi], d_out, rounds);
            else if (which == 1) hipLaunchKernelGGL((bfly_probe_kernel<false, false>), dim3(groups), dim3(T16_THREADS), 0, ctx->stream, tw, tw_sh, ctx->mod[mi], d_out, rounds);
            else hipLaunchKernelGGL((bfly_probe_kernel<true, true>), dim3(groups), dim3(T16_THREADS), 0, ctx->stream, tw, tw_sh, ctx->mod[mi], d_out, rounds);
            HE_HIP(ctx, hipGetLastError());
            HE_HIP(ctx, hipEventRecord(e1, ctx->stream));
            HE_HIP(ctx, hipEventSynchronize(e1));
        }
        float ms = 0.f;
        HE_HIP(ctx, hipEventElapsedTime(&ms, e0, e1));
        rate_out[which] = (double)groups * T16_THREADS * 32.0 * rounds / (ms * 1e-3);
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return HE_OK;
}

// ---------------------------------------------------------------- host
int32_t launch_transform16(he_ctx* ctx, const TransformDesc& d) {
    const uint32_t n = d.n;
    LimbList ll;
    SrcList sl;
    uint32_t live = 0;
    for (uint32_t s = 0; s < HE_MAX_SEGS; s++) sl.seg[s] = s < d.n_seg ? d.seg[s] : d.seg[0];
    for (uint32_t i = 0; i < n; i++) {
        uint32_t seg = d.src_seg ? d.src_seg[i] : 0, lim = d.src_limb ? d.src_limb[i] : i;
        if (seg >= HE_MAX_SEGS || seg >= d.n_seg || lim >= 4096) return he_fail(ctx, HE_ERR_BADARG, "transform: source limb out of range");
        sl.limb[i] = (uint16_t)((seg << 12) | lim);
        if (d.mod_idx[i] == 0xFFu) { ll.mod[i] = 0xFF; continue; }
        if (d.mod_idx[i] >= ctx->M) return he_fail(ctx, HE_ERR_BADARG, "transform: modulus index %u out of range", d.mod_idx[i]);
        ll.mod[i] = (uint8_t)d.mod_idx[i];
        live++;
    }
    if (live == 0) return HE_OK;
    const bool fwd = d.fwd;
    Ntt16Args a;
    a.dst = d.dst; a.mc = ctx->d_mc;
    a.lazy = (d.fwd && d.lazy_out) ? 1u : 0u;
    a.rs_mod = d.rescale_from ? d.rescale_from - 1 : 0;
    if (d.rescale_from && (!d.fwd || d.rescale_from > ctx->M || d.only_pass == 2))
        return he_fail(ctx, HE_ERR_BADARG, "transform: the Rescale rounding term is read by the first pass of a forward transform");
    a.tw = fwd ? ctx->d_tw : ctx->d_itw;
    a.tw_sh = fwd ? ctx->d_tw_sh : ctx->d_itw_sh;
    dim3 grid(n * 16), block(T16_THREADS);
    // row-pass schedule: live limbs sorted by modulus (stable counting sort), chunked
    RowSched rs;
    uint32_t distinct = 0;
    {
        uint32_t count[HE_MAX_MODULI] = {0}, start[HE_MAX_MODULI];
        for (uint32_t i = 0; i < n; i++) if (ll.mod[i] != 0xFF) count[ll.mod[i]]++;
        uint32_t acc = 0;
        for (uint32_t m = 0; m < ctx->M; m++) { start[m] = acc; acc += count[m]; if (count[m]) distinct++; }
        for (uint32_t i = 0; i < n; i++) if (ll.mod[i] != 0xFF) rs.order[start[ll.mod[i]]++] = (uint16_t)i;
    }
    uint32_t lc = 0;
    while (lc < 4 && (2u << lc) * distinct <= live) lc++;      // chunk <= average group size, at most 16
    rs.log_chunk = lc;
    uint32_t padded = (live + (1u << lc) - 1) & ~((1u << lc) - 1u);
    for (uint32_t i = live; i < padded && i < HE_MAX_LAUNCH_LIMBS; i++) rs.order[i] = 0xFFFF;
    dim3 grid_rows(padded * 16);
    for (int pass = 0; pass < 2; pass++) {
        if (d.only_pass && d.only_pass != (uint32_t)pass + 1) continue;
        hipEvent_t e0 = nullptr, e1 = nullptr;
        if (ctx->prof_on) {
            HE_HIP(ctx, hipEventCreate(&e0));
            HE_HIP(ctx, hipEventCreate(&e1));
            HE_HIP(ctx, hipEventRecord(e0, ctx->stream));
        }
        if (fwd && pass == 0 && d.rescale_from) hipLaunchKernelGGL(ntt16_fwd_a_kernel<true>, grid, block, 0, ctx->stream, a, ll, sl);
        else if (fwd && pass == 0) hipLaunchKernelGGL(ntt16_fwd_a_kernel<false>, grid, block, 0, ctx->stream, a, ll, sl);
        else if (fwd && d.ep && d.ep->fused && d.ep->beta == 1 && d.ep->n_terms == 0)      // single digit: its own instantiation
            hipLaunchKernelGGL(ntt16_fwd_b_kernel<3>, grid_rows, block, 0, ctx->stream, a, ll, rs, *d.ep);
        else if (fwd && d.ep && d.ep->fused) hipLaunchKernelGGL(ntt16_fwd_b_kernel<2>, grid_rows, block, 0, ctx->stream, a, ll, rs, *d.ep);
        else if (fwd && d.ep) hipLaunchKernelGGL(ntt16_fwd_b_kernel<1>, grid_rows, block, 0, ctx->stream, a, ll, rs, *d.ep);
        else if (fwd) { ModDownEpilogue none = {}; hipLaunchKernelGGL(ntt16_fwd_b_kernel<0>, grid_rows, block, 0, ctx->stream, a, ll, rs, none); }
        else if (pass == 0 && d.ip) hipLaunchKernelGGL(ntt16_inv_b_kernel<true>, grid_rows, block, 0, ctx->stream, a, ll, sl, rs, *d.ip);
        else if (pass == 0) { IpPrologue none = {}; hipLaunchKernelGGL(ntt16_inv_b_kernel<false>, grid_rows, block, 0, ctx->stream, a, ll, sl, rs, none); }
        else if (d.scale) hipLaunchKernelGGL(ntt16_inv_a_kernel<true>, grid, block, 0, ctx->stream, a, ll, *d.scale, d.scale_period);
        else { ScaleList none; hipLaunchKernelGGL(ntt16_inv_a_kernel<false>, grid, block, 0, ctx->stream, a, ll, none, 1u); }
        HE_HIP(ctx, hipGetLastError());
        if (ctx->prof_on) {
            HE_HIP(ctx, hipEventRecord(e1, ctx->stream));
            // the two components of a job share the gathered digit limbs: beta per pair of limbs
            uint32_t dig = 0;
            if (!fwd && pass == 0 && d.ip) dig = d.ip->beta * (live / 2);
            if (fwd && pass == 1 && d.ep && d.ep->fused) dig = d.ep->beta * (live / 2);
            const uint32_t kind = fwd ? (pass == 0 ? 0u : (d.ep ? 2u : 1u)) : (pass == 0 ? (d.ip ? 4u : 3u) : 5u);
            ctx->prof_events.push_back({e0, e1, live, dig, kind});
        }
    }
    if (fwd) ctx->cnt.ntt_limbs += live; else ctx->cnt.intt_limbs += live;
    return HE_OK;
}
