// Latency path for rings whose limb fits one work group's LDS (N <= 2^12, 32 KiB): a key switch in two launches
// and a rescale in one.  At these sizes a call is bound by the chain of dependent launches and, inside a launch,
// by the chain of dependent memory round trips, not by arithmetic.  So each work group produces one OUTPUT limb
// from start to finish, recomputing what it shares with its neighbours instead of exchanging it through memory,
// and issues every global load it will need before it starts computing: operands at the top of the kernel,
// each transform's twiddle table one transform ahead (into registers, then into LDS, where the stages read it).
//   ModUp    (hybrid key switching, paper Appendix: evaluation keys, dnum): work group (source, digit j, target
//            limb r) inverse-transforms the digit's <= 4 limbs in LDS, accumulates the basis conversion to r in
//            registers, transforms forward and writes raised_j[r];
//   ModDown  work group (job, component, q-limb r) forms the inner products of limb r and of every special-prime
//            limb from the operands it loaded (digits gathered by the Galois map), inverse-transforms the
//            special-prime ones in LDS, accumulates the conversion to r, transforms forward and writes
//            (acc - conv) * P^-1 (+ rotated c0) (+ addend);
//   Rescale  (Section 2.1) work group (ciphertext, component, limb r) inverse-transforms the dropped limb,
//            forms the correction term modulo q_r, transforms it forward and writes (c_r + delta) * q_l^-1.
// The arithmetic is the engine's (same digits, same conversion without overflow correction, same ModDown without
// rounding term), so the results are the same bits as the multi-launch path that larger rings and wider digits take.
#include "modarith.h"
#include "ntt_blocks.h"

#define SR_THREADS 1024
#define SR_PTS 4          // points per thread: 1024 threads x 4 = the largest limb (2^12)
#define SR_MAX_SRC 4      // limbs per digit and special primes this path handles
#define SR_LDS (4096 + 256)

// LDS position of element i: one spare slot per 16 spreads the strided accesses of the late stages over the banks.
__device__ __forceinline__ uint32_t sp(uint32_t i) { return i + (i >> 4); }

// A twiddle table (N factors and their Shoup companions) on its way from memory to LDS: fetched into registers
// while the previous transform still uses the LDS copy, committed once that transform is done.
struct TwRegs { u64 w[SR_PTS], s[SR_PTS]; };

__device__ __forceinline__ void tw_fetch(TwRegs& r, const u64* __restrict__ tw, const u64* __restrict__ tw_sh, uint32_t N) {
#pragma unroll
    for (uint32_t p = 0; p < SR_PTS; p++) {
        const uint32_t e = threadIdx.x + SR_THREADS * p;
        if (e < N) { r.w[p] = tw[e]; r.s[p] = tw_sh[e]; }
    }
}
__device__ __forceinline__ void tw_commit(const TwRegs& r, u64* twl, u64* twl_sh, uint32_t N) {
#pragma unroll
    for (uint32_t p = 0; p < SR_PTS; p++) {
        const uint32_t e = threadIdx.x + SR_THREADS * p;
        if (e < N) { twl[e] = r.w[p]; twl_sh[e] = r.s[p]; }
    }
}

// Forward transform of the whole limb in LDS (decimation in time, psi folded into the twiddles; natural order in,
// bit-reversed out): register blocks of two stages on 4 points per thread with one LDS exchange between blocks,
// then one radix-2 stage when logN is odd.  Twiddles from the LDS table.  Inputs below 4q, results canonical.
// Ends with a barrier.
template <bool WIDE>
__device__ __forceinline__ void lds_ntt_fwd_t(u64* sm, const u64* twl, const u64* twl_sh, const ModConst& m, uint32_t logN) {
    const u64 q = m.q, q2 = 2 * q, q4 = 4 * q;
    const uint32_t N = 1u << logN, nb = logN >> 1;
    // the blocks leave values below 52q (never reduced) or, for the widest moduli, below 8q
    const uint32_t mrec = WIDE ? 0u : (1u << 24) / ((uint32_t)(q >> (m.bits - 8)) + 1);
    for (uint32_t blk = 0; blk < nb; blk++) {
        const uint32_t s0 = 2 * blk, log_span = logN - s0 - 2, span = 1u << log_span;
        for (uint32_t tid = threadIdx.x; tid < (N >> 2); tid += SR_THREADS) {
            const uint32_t G = tid >> log_span, off = tid & (span - 1), base = (G << (logN - s0)) + off;
            u64 x[4];
#pragma unroll
            for (int k = 0; k < 4; k++) x[k] = sm[sp(base + (k << log_span))];
            fwd_block2<WIDE>(x, twl, twl_sh, s0, G, q, q4);
            if (blk + 1 == nb) {
#pragma unroll
                for (int k = 0; k < 4; k++) x[k] = WIDE ? csub(csub(csub(x[k], q4), q2), q) : reduce_small(x[k], q, m.bits, mrec);
            }
#pragma unroll
            for (int k = 0; k < 4; k++) sm[sp(base + (k << log_span))] = x[k];
        }
        __syncthreads();
    }
    if (logN & 1u) {
        const uint32_t s = logN - 1;
        for (uint32_t b = threadIdx.x; b < (N >> 1); b += SR_THREADS) {
            const uint32_t e0 = sp(2 * b), e1 = sp(2 * b + 1), k = (1u << s) + b;
            const u64 x = sm[e0];
            const u64 v = shoup_lazy(sm[e1], twl[k], twl_sh[k], q);
            sm[e0] = csub(csub(x + v, q2), q);
            sm[e1] = csub(csub(x - v + q2, q2), q);
        }
        __syncthreads();
    }
}
__device__ __forceinline__ void lds_ntt_fwd(u64* sm, const u64* twl, const u64* twl_sh, const ModConst& m, uint32_t logN) {
    if (m.bits > 57) lds_ntt_fwd_t<true>(sm, twl, twl_sh, m, logN);
    else lds_ntt_fwd_t<false>(sm, twl, twl_sh, m, logN);
}

// Inverse transform in LDS (bit-reversed in, natural out): the last stage as a radix-2 stage first when logN is
// odd, then the register blocks from the highest stages down; every value times `scale` (which carries N^-1) as
// the last block stores it.  Inputs canonical, results canonical.  Ends with a barrier.
__device__ __forceinline__ void lds_ntt_inv(u64* sm, const u64* twl, const u64* twl_sh, const ModConst& m, uint32_t logN, u64 scale,
                                            u64 scale_sh) {
    const u64 q = m.q, q2 = 2 * q, q4 = 4 * q;
    const uint32_t N = 1u << logN, nb = logN >> 1;
    if (logN & 1u) {
        const uint32_t s = logN - 1;
        for (uint32_t b = threadIdx.x; b < (N >> 1); b += SR_THREADS) {
            const uint32_t e0 = sp(2 * b), e1 = sp(2 * b + 1), k = (1u << s) + b;
            const u64 x = sm[e0], y = sm[e1];
            sm[e0] = csub(x + y, q2);
            sm[e1] = shoup_lazy(x - y + q2, twl[k], twl_sh[k], q);
        }
        __syncthreads();
    }
    for (uint32_t blk = nb; blk-- > 0;) {
        const uint32_t s0 = 2 * blk, log_span = logN - s0 - 2, span = 1u << log_span;
        for (uint32_t tid = threadIdx.x; tid < (N >> 2); tid += SR_THREADS) {
            const uint32_t G = tid >> log_span, off = tid & (span - 1), base = (G << (logN - s0)) + off;
            u64 x[4];
#pragma unroll
            for (int k = 0; k < 4; k++) x[k] = sm[sp(base + (k << log_span))];
            inv_block2(x, twl, twl_sh, s0, G, q, q4);
            if (blk == 0) {
#pragma unroll
                for (int k = 0; k < 4; k++) x[k] = csub(shoup_lazy(x[k], scale, scale_sh, q), q);
            }
#pragma unroll
            for (int k = 0; k < 4; k++) sm[sp(base + (k << log_span))] = x[k];
        }
        __syncthreads();
    }
}

__device__ __forceinline__ uint32_t galois_src_sr(uint32_t j, uint32_t g, uint32_t logN) {
    uint32_t k = __brev(j) >> (32 - logN);
    uint32_t kp = (g * k + ((g - 1) >> 1)) & ((1u << logN) - 1);
    return __brev(kp) >> (32 - logN);
}

struct SrTables {
    const ModConst* mc;
    const u64 *tw, *tw_sh, *itw, *itw_sh;   // [M][N]
    uint32_t logN;
};

// ---------------------------------------------------------------- ModUp
struct SrUpArgs {
    const u64* c1[8];          // sources [L1][N], NTT form
    u64* raised;               // [n_src][beta][R][N]; a digit's own limbs are left unwritten
    const u64* hat;            // conversion constants [digit][size-1][modulus][i padded to aw]
    u64 scale[HE_MAX_MODULI];  // per source limb: N^-1 * (Q_j/q_i)^-1 mod q_i, and its Shoup companion
    u64 scale_sh[HE_MAX_MODULI];
    uint32_t L1, R, beta, alpha, M, nq, level, aw, n_out;   // n_out = output limbs per source
    uint8_t oj[512], orr[512]; // output o of a source: digit, raised-basis limb
};

__global__ __launch_bounds__(SR_THREADS) void sr_modup_kernel(SrUpArgs a, SrTables tb) {
    __shared__ u64 sm[SR_LDS];
    __shared__ u64 twl[4096], twl_sh[4096];
    const uint32_t N = 1u << tb.logN;
    const uint32_t s = blockIdx.x / a.n_out, o = blockIdx.x % a.n_out;
    const uint32_t j = a.oj[o], r = a.orr[o];
    const uint32_t lo = j * a.alpha, sz = min(a.alpha, a.L1 - lo);
    const uint32_t mr = r <= a.level ? r : a.nq + (r - a.level - 1);
    const ModConst m = tb.mc[mr];
    const u64* hat = a.hat + ((size_t)(j * a.alpha + (sz - 1)) * a.M + mr) * a.aw;
    // every operand first: the digit's limbs (points e = threadIdx.x + 1024 p), the first table
    u64 in[SR_MAX_SRC][SR_PTS];
    u64 h[SR_MAX_SRC];
#pragma unroll
    for (uint32_t i = 0; i < SR_MAX_SRC; i++) {
        const u64* src = a.c1[s] + ((size_t)(lo + (i < sz ? i : 0)) << tb.logN);
        h[i] = i < sz ? hat[i] : 0;
#pragma unroll
        for (uint32_t p = 0; p < SR_PTS; p++) {
            const uint32_t e = threadIdx.x + SR_THREADS * p;
            in[i][p] = (i < sz && e < N) ? src[e] : 0;
        }
    }
    TwRegs tr;
    tw_fetch(tr, tb.itw + ((size_t)lo << tb.logN), tb.itw_sh + ((size_t)lo << tb.logN), N);
    u128 acc[SR_PTS] = {};
#pragma unroll
    for (uint32_t i = 0; i < SR_MAX_SRC; i++) {
        if (i < sz) {
            const uint32_t mi = lo + i;
            const ModConst mq = tb.mc[mi];
#pragma unroll
            for (uint32_t p = 0; p < SR_PTS; p++) {
                const uint32_t e = threadIdx.x + SR_THREADS * p;
                if (e < N) sm[sp(e)] = in[i][p];
            }
            tw_commit(tr, twl, twl_sh, N);
            __syncthreads();
            // the table of the next transform travels while this one runs
            if (i + 1 < sz) tw_fetch(tr, tb.itw + ((size_t)(mi + 1) << tb.logN), tb.itw_sh + ((size_t)(mi + 1) << tb.logN), N);
            else tw_fetch(tr, tb.tw + ((size_t)mr << tb.logN), tb.tw_sh + ((size_t)mr << tb.logN), N);
            lds_ntt_inv(sm, twl, twl_sh, mq, tb.logN, a.scale[mi], a.scale_sh[mi]);
#pragma unroll
            for (uint32_t p = 0; p < SR_PTS; p++) {
                const uint32_t e = threadIdx.x + SR_THREADS * p;
                if (e < N) acc[p] += (u128)sm[sp(e)] * h[i];
            }
            __syncthreads();
        }
    }
#pragma unroll
    for (uint32_t p = 0; p < SR_PTS; p++) {
        const uint32_t e = threadIdx.x + SR_THREADS * p;
        if (e < N) sm[sp(e)] = barrett128(acc[p], m.q, m.mu, m.bits);
    }
    tw_commit(tr, twl, twl_sh, N);
    __syncthreads();
    lds_ntt_fwd(sm, twl, twl_sh, m, tb.logN);
    u64* dst = a.raised + ((size_t)((s * a.beta + j) * a.R + r) << tb.logN);
    for (uint32_t e = threadIdx.x; e < N; e += SR_THREADS) dst[e] = sm[sp(e)];
}

// ---------------------------------------------------------------- inner product + ModDown
struct SrDownArgs {
    const u64* dn_hat;         // [M][pw]: (P/p_t) mod modulus
    u64 scale[SR_MAX_SRC];     // N^-1 * (P/p_t)^-1 mod p_t and Shoup companions
    u64 scale_sh[SR_MAX_SRC];
    uint32_t k, nq, level, pw;
};

__global__ __launch_bounds__(SR_THREADS) void sr_moddown_kernel(ModDownEpilogue ep, SrDownArgs a, SrTables tb) {
    __shared__ u64 sm[SR_LDS];
    __shared__ u64 twl[4096], twl_sh[4096];
    const uint32_t N = 1u << tb.logN, L1 = ep.L1, R = ep.R, beta = ep.beta;
    const uint32_t pc = blockIdx.x / L1, r = blockIdx.x - pc * L1, job = pc >> 1, comp = pc & 1u;
    const ModConst m = tb.mc[r];
    const uint32_t g = ep.g[job];
    const u64* raised = ep.raised[job];
    const u64* evk = ep.evk[job];
    TwRegs tr;
    tw_fetch(tr, tb.itw + ((size_t)a.nq << tb.logN), tb.itw_sh + ((size_t)a.nq << tb.logN), N);
    uint32_t src[SR_PTS];
#pragma unroll
    for (uint32_t p = 0; p < SR_PTS; p++) {
        const uint32_t e = threadIdx.x + SR_THREADS * p;
        src[p] = (e < N && g != 1) ? galois_src_sr(e, g, tb.logN) : e;
    }
    // every inner product first, so that all operand loads are in flight together: limb r of the accumulator (digit
    // j's own limbs come from the switched polynomial itself), the epilogue's addends, the special-prime limbs
    const uint32_t own_j = r / ep.alpha;
    const u64* own = ep.own[job] + ((size_t)r << tb.logN);
    const u64* c0 = (comp == 0 && ep.c0[job]) ? ep.c0[job] + ((size_t)r << tb.logN) : nullptr;
    const u64* self = comp ? ep.self1[job] : ep.self0[job];
    u64 aq[SR_PTS], add0[SR_PTS], add1[SR_PTS], pl[SR_MAX_SRC][SR_PTS];
#pragma unroll
    for (uint32_t p = 0; p < SR_PTS; p++) {
        const uint32_t e = threadIdx.x + SR_THREADS * p;
        aq[p] = add0[p] = add1[p] = 0;
        if (e < N) {
            u128 sum = 0;
            for (uint32_t j = 0; j < beta; j++) {
                const u64 d = j == own_j ? own[src[p]] : raised[((size_t)(j * R + r) << tb.logN) + src[p]];
                sum += (u128)d * evk[((size_t)((j * 2 + comp) * ep.M + r) << tb.logN) + e];
            }
            aq[p] = barrett128(sum, m.q, m.mu, m.bits);
            if (c0) add0[p] = c0[src[p]];
            if (self) add1[p] = self[((size_t)r << tb.logN) + e];
        }
    }
#pragma unroll
    for (uint32_t t = 0; t < SR_MAX_SRC; t++) {
        const uint32_t mt = a.nq + (t < a.k ? t : 0);
        const ModConst mp = tb.mc[mt];
#pragma unroll
        for (uint32_t p = 0; p < SR_PTS; p++) {
            const uint32_t e = threadIdx.x + SR_THREADS * p;
            pl[t][p] = 0;
            if (t < a.k && e < N) {
                u128 sum = 0;
                for (uint32_t j = 0; j < beta; j++)
                    sum += (u128)raised[((size_t)(j * R + L1 + t) << tb.logN) + src[p]] *
                           evk[((size_t)((j * 2 + comp) * ep.M + mt) << tb.logN) + e];
                pl[t][p] = barrett128(sum, mp.q, mp.mu, mp.bits);
            }
        }
    }
    u128 acc[SR_PTS] = {};
#pragma unroll
    for (uint32_t t = 0; t < SR_MAX_SRC; t++) {
        if (t < a.k) {
            const uint32_t mt = a.nq + t;
            const ModConst mp = tb.mc[mt];
#pragma unroll
            for (uint32_t p = 0; p < SR_PTS; p++) {
                const uint32_t e = threadIdx.x + SR_THREADS * p;
                if (e < N) sm[sp(e)] = pl[t][p];
            }
            tw_commit(tr, twl, twl_sh, N);
            __syncthreads();
            if (t + 1 < a.k) tw_fetch(tr, tb.itw + ((size_t)(mt + 1) << tb.logN), tb.itw_sh + ((size_t)(mt + 1) << tb.logN), N);
            else tw_fetch(tr, tb.tw + ((size_t)r << tb.logN), tb.tw_sh + ((size_t)r << tb.logN), N);
            lds_ntt_inv(sm, twl, twl_sh, mp, tb.logN, a.scale[t], a.scale_sh[t]);
            const u64 h = a.dn_hat[(size_t)r * a.pw + t];
#pragma unroll
            for (uint32_t p = 0; p < SR_PTS; p++) {
                const uint32_t e = threadIdx.x + SR_THREADS * p;
                if (e < N) acc[p] += (u128)sm[sp(e)] * h;
            }
            __syncthreads();
        }
    }
#pragma unroll
    for (uint32_t p = 0; p < SR_PTS; p++) {
        const uint32_t e = threadIdx.x + SR_THREADS * p;
        if (e < N) sm[sp(e)] = barrett128(acc[p], m.q, m.mu, m.bits);
    }
    tw_commit(tr, twl, twl_sh, N);
    __syncthreads();
    lds_ntt_fwd(sm, twl, twl_sh, m, tb.logN);
    u64* out = (comp ? ep.out1[job] : ep.out0[job]) + ((size_t)r << tb.logN);
    const u64 pinv = ep.pinv[r], pinv_sh = ep.pinv_sh[r];
#pragma unroll
    for (uint32_t p = 0; p < SR_PTS; p++) {
        const uint32_t e = threadIdx.x + SR_THREADS * p;
        if (e < N) {
            u64 v = shoup_mul(submod(aq[p], sm[sp(e)], m.q), pinv, pinv_sh, m.q);
            if (c0) v = addmod(v, add0[p], m.q);
            if (self) v = addmod(v, add1[p], m.q);
            out[e] = v;
        }
    }
}

// ---------------------------------------------------------------- rescale
struct SrRescaleArgs {
    const u64* ct[HE_MAX_KS_JOBS];   // [2][level+1][N]
    u64* out[HE_MAX_KS_JOBS];        // [2][level][N]
    const u64 *qlinv, *qlinv_sh;     // q_level^-1 mod q_r
    uint32_t level;
};

__global__ __launch_bounds__(SR_THREADS) void sr_rescale_kernel(SrRescaleArgs a, SrTables tb) {
    __shared__ u64 sm[SR_LDS];
    __shared__ u64 twl[4096], twl_sh[4096];
    const uint32_t N = 1u << tb.logN, level = a.level;
    const uint32_t jc = blockIdx.x / level, r = blockIdx.x - jc * level, job = jc >> 1, comp = jc & 1u;
    const ModConst ml = tb.mc[level], mr = tb.mc[r];
    const u64* top = a.ct[job] + ((size_t)(comp * (level + 1) + level) << tb.logN);
    const u64* in = a.ct[job] + ((size_t)(comp * (level + 1) + r) << tb.logN);
    const u64 qlinv = a.qlinv[r], qlinv_sh = a.qlinv_sh[r];
    TwRegs tr;
    tw_fetch(tr, tb.itw + ((size_t)level << tb.logN), tb.itw_sh + ((size_t)level << tb.logN), N);
    u64 cr[SR_PTS];
#pragma unroll
    for (uint32_t p = 0; p < SR_PTS; p++) {
        const uint32_t e = threadIdx.x + SR_THREADS * p;
        cr[p] = 0;
        if (e < N) { sm[sp(e)] = top[e]; cr[p] = in[e]; }
    }
    tw_commit(tr, twl, twl_sh, N);
    __syncthreads();
    tw_fetch(tr, tb.tw + ((size_t)r << tb.logN), tb.tw_sh + ((size_t)r << tb.logN), N);
    lds_ntt_inv(sm, twl, twl_sh, ml, tb.logN, ml.ninv, ml.ninv_sh);
    const u64 h = ml.q >> 1, hr = barrett64(h, mr.q, mr.mu, mr.bits);
    for (uint32_t e = threadIdx.x; e < N; e += SR_THREADS) {
        const u64 t = addmod(sm[sp(e)], h, ml.q);
        sm[sp(e)] = submod(hr, barrett64(t, mr.q, mr.mu, mr.bits), mr.q);
    }
    tw_commit(tr, twl, twl_sh, N);
    __syncthreads();
    lds_ntt_fwd(sm, twl, twl_sh, mr, tb.logN);
    u64* out = a.out[job] + ((size_t)(comp * level + r) << tb.logN);
#pragma unroll
    for (uint32_t p = 0; p < SR_PTS; p++) {
        const uint32_t e = threadIdx.x + SR_THREADS * p;
        if (e < N) out[e] = shoup_mul(addmod(cr[p], sm[sp(e)], mr.q), qlinv, qlinv_sh, mr.q);
    }
}

// ---------------------------------------------------------------- host
static SrTables sr_tables(const he_ctx* c) { return {c->d_mc, c->d_tw, c->d_tw_sh, c->d_itw, c->d_itw_sh, c->logN}; }

bool small_ring_path(const he_ctx* c, uint32_t level) {
    const uint32_t beta = (level + c->alpha) / c->alpha;
    return c->logN <= 12 && c->alpha <= SR_MAX_SRC && c->np >= 1 && c->np <= SR_MAX_SRC && beta <= 8 && beta * (level + 1 + c->np) <= 512;
}

int32_t sr_modup(he_ctx* c, const KsSrc* srcs, uint32_t cb, uint32_t level, u64* raised) {
    const uint32_t L1 = level + 1, R = L1 + c->np, al = c->alpha, beta = (level + al) / al;
    SrUpArgs a;
    if (cb > 8) return he_fail(c, HE_ERR_BADARG, "small-ring ModUp: more than 8 sources");
    for (uint32_t s = 0; s < 8; s++) a.c1[s] = srcs[s < cb ? s : 0].c1;
    a.raised = raised; a.hat = c->d_up_hat;
    a.L1 = L1; a.R = R; a.beta = beta; a.alpha = al; a.M = c->M; a.nq = c->nq; a.level = level; a.aw = (al + 7u) & ~7u;
    for (uint32_t i = 0; i < L1; i++) {
        const uint32_t j = i / al, lo = j * al, hi = (j + 1) * al < L1 ? (j + 1) * al : L1, sz = hi - lo;
        a.scale[i] = h_mulmod(c->h_mc[i].ninv, c->h_up_invhat[(size_t)(j * al + (sz - 1)) * al + (i - lo)], c->mod[i]);
        a.scale_sh[i] = h_shoup(a.scale[i], c->mod[i]);
    }
    a.n_out = 0;
    for (uint32_t j = 0; j < beta; j++) {
        const uint32_t lo = j * al, hi = (j + 1) * al < L1 ? (j + 1) * al : L1;
        for (uint32_t r = 0; r < R; r++) {
            if (r >= lo && r < hi) continue;
            a.oj[a.n_out] = (uint8_t)j; a.orr[a.n_out] = (uint8_t)r; a.n_out++;
        }
    }
    hipLaunchKernelGGL(sr_modup_kernel, dim3(cb * a.n_out), dim3(SR_THREADS), 0, c->stream, a, sr_tables(c));
    HE_HIP(c, hipGetLastError());
    // logical transform counts (each work group repeats the inverse transforms of its digit)
    c->cnt.intt_limbs += (uint64_t)cb * L1;
    c->cnt.ntt_limbs += (uint64_t)cb * a.n_out;
    c->cnt.modup += cb;
    return HE_OK;
}

int32_t sr_moddown(he_ctx* c, uint32_t level, uint32_t J, const ModDownEpilogue& ep) {
    const uint32_t L1 = level + 1, k = c->np;
    SrDownArgs a;
    a.dn_hat = c->d_dn_hat; a.k = k; a.nq = c->nq; a.level = level; a.pw = (k + 7u) & ~7u;
    for (uint32_t t = 0; t < k; t++) {
        const u64 p = c->mod[c->nq + t];
        a.scale[t] = h_mulmod(c->h_mc[c->nq + t].ninv, c->h_dn_invhat[t], p);
        a.scale_sh[t] = h_shoup(a.scale[t], p);
    }
    hipLaunchKernelGGL(sr_moddown_kernel, dim3(J * 2 * L1), dim3(SR_THREADS), 0, c->stream, ep, a, sr_tables(c));
    HE_HIP(c, hipGetLastError());
    c->cnt.intt_limbs += (uint64_t)J * 2 * k;
    c->cnt.ntt_limbs += (uint64_t)J * 2 * L1;
    c->cnt.moddown += J;
    return HE_OK;
}

int32_t sr_rescale(he_ctx* c, const u64* const* cts, u64* const* outs, uint32_t n, uint32_t level) {
    for (uint32_t b0 = 0; b0 < n; b0 += HE_MAX_KS_JOBS) {
        const uint32_t nb = n - b0 < HE_MAX_KS_JOBS ? n - b0 : HE_MAX_KS_JOBS;
        SrRescaleArgs a;
        for (uint32_t i = 0; i < nb; i++) { a.ct[i] = cts[b0 + i]; a.out[i] = outs[b0 + i]; }
        a.qlinv = c->d_qlinv + (size_t)level * c->nq; a.qlinv_sh = c->d_qlinv_sh + (size_t)level * c->nq; a.level = level;
        hipLaunchKernelGGL(sr_rescale_kernel, dim3(nb * 2 * level), dim3(SR_THREADS), 0, c->stream, a, sr_tables(c));
        HE_HIP(c, hipGetLastError());
        c->cnt.intt_limbs += (uint64_t)2 * nb;
        c->cnt.ntt_limbs += (uint64_t)2 * nb * level;
        c->cnt.rescale += nb;
    }
    return HE_OK;
}
