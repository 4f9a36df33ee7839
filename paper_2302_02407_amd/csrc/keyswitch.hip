// Hybrid key switching with dnum digits (the inner step of CRot; paper Section 2.1 for CRot,
// Appendix for evaluation keys and dnum), batched rotations, and rescale.
//
//   ModUp   : digit limbs -> coefficient form (iNTT with the factor (Q_j/q_i)^-1 folded into
//             the N^-1 scaling) -> fast basis conversion to every other limb of
//             {q_0..q_l, p_*} (128-bit accumulation, one Barrett step) -> NTT.
//   inner   : acc_c[r] = sum_j sigma_g(raised_j)[r] * evk_j,c[r]   (sigma_g as a gather).  At N = 2^16 this
//             sum is evaluated inside the transforms of ModDown that consume it (special-prime limbs as
//             the first inverse pass loads its rows, q-limbs in the epilogue of the last forward pass)
//             and acc is never stored; other ring sizes run the stand-alone kernels below.
//   ModDown : p-limbs -> coefficient form (iNTT with (P/p_t)^-1 folded in) -> conversion to
//             q_0..q_l -> NTT -> (acc - conv) * P^-1 (+ sigma_g(c0) for a rotation).
// Neither conversion corrects the overflow multiple; each term is a canonical residue and
// the sum is reduced exactly, so results are defined bit for bit.
//
// The engine takes a list of sources (ciphertexts to raise) and a list of jobs (source, Galois
// element, key, output).  Sources are raised several at a time and the jobs' ModDown chains
// run HE_MAX_KS_JOBS at a time, so that every launch covers hundreds of limbs even when one
// ciphertext has only 24; jobs that use the same key share one pass over the key.
#include <algorithm>

#include "modarith.h"
#include "ntt_blocks.h"

#define KS_THREADS 256
#define CONV_MAX_JOBS 8
#define CONV_TGT_PER_BLOCK 8

__device__ __forceinline__ uint32_t galois_src_ks(uint32_t j, uint32_t g, uint32_t logN) {
    uint32_t k = __brev(j) >> (32 - logN);
    uint32_t kp = (g * k + ((g - 1) >> 1)) & ((1u << logN) - 1);
    return __brev(kp) >> (32 - logN);
}

struct ConvJob {
    const u64* src;       // [ns][N] coefficient form, already multiplied by the inverse "hat" factors
    u64* dst;             // target limb t is written at dst + tgt_limb[t]*N
    const u64* hat;       // hat[m*hat_w + i] = (S/s_i) mod modulus m, zero for i >= ns
    uint32_t ns, nt, hat_w, pad;   // hat_w = ns rounded up to a multiple of 8 (<= 64)
    uint8_t tgt_limb[HE_MAX_MODULI];
    uint8_t tgt_mod[HE_MAX_MODULI];
};
// njobs descriptors, each applied `reps` times with src/dst advanced by a fixed stride per repeat.
struct ConvBatch {
    ConvJob job[CONV_MAX_JOBS];
    uint32_t njobs, reps;
    size_t src_stride, dst_stride;   // elements per repeat
};

// Fast basis conversion.  grid: (N/512, ceil(nt_max/CONV_TGT_PER_BLOCK), njobs*reps); each thread
// owns two adjacent coefficients (16-byte loads and stores).  The block's conversion constants
// and target moduli are staged in LDS once and then read as broadcasts.
//
// ONE_CHUNK (at most 8 source limbs): sources stay in registers across all targets, split into
// 30-bit halves, and so are the constants; the four partial sums of 8 products of 30-bit halves
// stay below 2^63, so they are plain 32x32+64 multiply-add chains with no carry handling, and
// the 128-bit sum is assembled once per output (all moduli are below 2^60).
//
// LAZY: outputs are left in [0, 5q) (congruent, not canonical); only for buffers whose sole consumer
// is the N = 2^16 forward transform, whose lazy bounds absorb it.
template <bool ONE_CHUNK, bool LAZY>
__global__ __launch_bounds__(KS_THREADS) void baseconv_kernel(ConvBatch b, const ModConst* mc, uint32_t logN) {
    __shared__ u64 s_hat[CONV_TGT_PER_BLOCK * 64];
    __shared__ uint32_t s_h0[CONV_TGT_PER_BLOCK * 8], s_h1[CONV_TGT_PER_BLOCK * 8];
    __shared__ u64 s_q[CONV_TGT_PER_BLOCK], s_mu[CONV_TGT_PER_BLOCK];
    __shared__ uint32_t s_bits[CONV_TGT_PER_BLOCK];
    const uint32_t ji = blockIdx.z % b.njobs, rep = blockIdx.z / b.njobs;
    const ConvJob& job = b.job[ji];
    const u64* src = job.src + rep * b.src_stride;
    u64* dst = job.dst + rep * b.dst_stride;
    const uint32_t t0 = blockIdx.y * CONV_TGT_PER_BLOCK;
    if (t0 >= job.nt) return;
    const uint32_t nt = min((uint32_t)CONV_TGT_PER_BLOCK, job.nt - t0);
    const uint32_t ns = job.ns, w = job.hat_w;
    for (uint32_t idx = threadIdx.x; idx < nt * w; idx += KS_THREADS) {
        uint32_t tt = idx / w, i = idx - tt * w;
        u64 h = job.hat[(size_t)job.tgt_mod[t0 + tt] * w + i];
        if (ONE_CHUNK) {
            if (i < 8) {                       // entries beyond the (at most 8) sources are zero padding
                s_h0[tt * 8 + i] = (uint32_t)h & 0x3FFFFFFFu;
                s_h1[tt * 8 + i] = (uint32_t)(h >> 30);
            }
        } else {
            s_hat[tt * 64 + i] = h;
        }
    }
    if (threadIdx.x < nt) {
        const ModConst m = mc[job.tgt_mod[t0 + threadIdx.x]];
        s_q[threadIdx.x] = m.q; s_mu[threadIdx.x] = m.mu; s_bits[threadIdx.x] = m.bits;
    }
    __syncthreads();
    const size_t n = (size_t)(blockIdx.x * KS_THREADS + threadIdx.x) * 2;
    if (n >= ((size_t)1 << logN)) return;      // rings smaller than one block of coefficient pairs
    if (ONE_CHUNK) {
        uint32_t ya0[8], ya1[8], yb0[8], yb1[8];   // 30-bit halves of the two coefficients' sources
#pragma unroll
        for (uint32_t i = 0; i < 8; i++) {
            ulonglong2 v = i < ns ? *reinterpret_cast<const ulonglong2*>(src + ((size_t)i << logN) + n) : make_ulonglong2(0, 0);
            ya0[i] = (uint32_t)v.x & 0x3FFFFFFFu; ya1[i] = (uint32_t)(v.x >> 30);
            yb0[i] = (uint32_t)v.y & 0x3FFFFFFFu; yb1[i] = (uint32_t)(v.y >> 30);
        }
        for (uint32_t tt = 0; tt < nt; tt++) {
            const u64 q = s_q[tt], mu = s_mu[tt];
            const uint32_t bits = s_bits[tt];
            u64 a00 = 0, a01 = 0, a10 = 0, a11 = 0, b00 = 0, b01 = 0, b10 = 0, b11 = 0;
#pragma unroll
            for (uint32_t i = 0; i < 8; i++) {
                const uint32_t h0 = s_h0[tt * 8 + i], h1 = s_h1[tt * 8 + i];
                a00 += (u64)ya0[i] * h0; a01 += (u64)ya0[i] * h1; a10 += (u64)ya1[i] * h0; a11 += (u64)ya1[i] * h1;
                b00 += (u64)yb0[i] * h0; b01 += (u64)yb0[i] * h1; b10 += (u64)yb1[i] * h0; b11 += (u64)yb1[i] * h1;
            }
            u128 sa = (u128)a00 + ((u128)(a01 + a10) << 30) + ((u128)a11 << 60);
            u128 sb = (u128)b00 + ((u128)(b01 + b10) << 30) + ((u128)b11 << 60);
            ulonglong2 o = LAZY ? make_ulonglong2(barrett128_lazy(sa, q, mu, bits), barrett128_lazy(sb, q, mu, bits))
                                : make_ulonglong2(barrett128(sa, q, mu, bits), barrett128(sb, q, mu, bits));
            *reinterpret_cast<ulonglong2*>(dst + ((size_t)job.tgt_limb[t0 + tt] << logN) + n) = o;
        }
    } else {
        for (uint32_t tt = 0; tt < nt; tt++) {
            const u64 q = s_q[tt], mu = s_mu[tt];
            const uint32_t bits = s_bits[tt];
            const u64* h = s_hat + tt * 64;
            u128 a0 = 0, a1 = 0;
            for (uint32_t i0 = 0; i0 < ns; i0 += 8) {
                if (i0) { a0 = barrett128(a0, q, mu, bits); a1 = barrett128(a1, q, mu, bits); }
                for (uint32_t i = i0; i < min(i0 + 8, ns); i++) {
                    ulonglong2 v = *reinterpret_cast<const ulonglong2*>(src + ((size_t)i << logN) + n);
                    a0 += (u128)v.x * h[i];
                    a1 += (u128)v.y * h[i];
                }
            }
            ulonglong2 o = make_ulonglong2(barrett128(a0, q, mu, bits), barrett128(a1, q, mu, bits));
            *reinterpret_cast<ulonglong2*>(dst + ((size_t)job.tgt_limb[t0 + tt] << logN) + n) = o;
        }
    }
}

// Jobs of one launch grouped by key: group z holds jobs [start[z], start[z]+count[z]) which all use
// evk[z] and Galois element g[z].
struct IpBatch {
    const u64* evk[HE_MAX_KS_JOBS];
    uint32_t g[HE_MAX_KS_JOBS];
    uint32_t start[HE_MAX_KS_JOBS];
    uint32_t count[HE_MAX_KS_JOBS];
    const u64* raised[HE_MAX_KS_JOBS];   // per job: [beta][R][N] (own limbs not materialised)
    const u64* own[HE_MAX_KS_JOBS];      // per job: the switched polynomial [level+1][N]
};

// grid: (N/256, R, groups).  acc [job][2][R][N].  A block loads the key values of its limb once
// and reuses them for every job of the group.  A digit's own limbs (limb r of digit r/alpha) are
// never materialised in `raised`: they are read from the job's input polynomial.
template <int BETA_MAX>
__global__ __launch_bounds__(KS_THREADS) void inner_product_kernel(IpBatch ib, u64* __restrict__ acc, const ModConst* mc,
                                                                   uint32_t logN, uint32_t R, uint32_t beta, uint32_t M,
                                                                   uint32_t level, uint32_t nq, uint32_t alpha) {
    const uint32_t n = blockIdx.x * KS_THREADS + threadIdx.x;
    const uint32_t r = blockIdx.y, z = blockIdx.z;
    const uint32_t mi = r <= level ? r : nq + (r - level - 1);
    const ModConst m = mc[mi];
    const uint32_t g = ib.g[z];
    const uint32_t src = g == 1 ? n : galois_src_ks(n, g, logN);
    const u64* evk = ib.evk[z];
    u64 kb[BETA_MAX], ka[BETA_MAX];
#pragma unroll
    for (uint32_t j = 0; j < BETA_MAX; j++) {
        kb[j] = j < beta ? evk[((size_t)((j * 2 + 0) * M + mi) << logN) + n] : 0;
        ka[j] = j < beta ? evk[((size_t)((j * 2 + 1) * M + mi) << logN) + n] : 0;
    }
    for (uint32_t jb = ib.start[z]; jb < ib.start[z] + ib.count[z]; jb++) {
        const u64* raised = ib.raised[jb];
        const u64* own = ib.own[jb];
        u128 a0 = 0, a1 = 0;
#pragma unroll
        for (uint32_t j = 0; j < BETA_MAX; j++) {
            if (j < beta) {
                const u64* dj = (r <= level && r / alpha == j) ? own + ((size_t)r << logN) : raised + ((size_t)(j * R + r) << logN);
                u64 d = dj[src];
                a0 += (u128)d * kb[j];
                a1 += (u128)d * ka[j];
            }
        }
        u64* out = acc + ((size_t)jb * 2 * R << logN);
        out[((size_t)r << logN) + n] = barrett128(a0, m.q, m.mu, m.bits);
        out[((size_t)(R + r) << logN) + n] = barrett128(a1, m.q, m.mu, m.bits);
    }
}

// Any number of digits (reduces every 8 terms); no key reuse in registers.
__global__ __launch_bounds__(KS_THREADS) void inner_product_wide_kernel(IpBatch ib, u64* __restrict__ acc, const ModConst* mc,
                                                                        uint32_t logN, uint32_t R, uint32_t beta, uint32_t M,
                                                                        uint32_t level, uint32_t nq, uint32_t alpha) {
    const uint32_t n = blockIdx.x * KS_THREADS + threadIdx.x;
    const uint32_t r = blockIdx.y, z = blockIdx.z;
    const uint32_t mi = r <= level ? r : nq + (r - level - 1);
    const ModConst m = mc[mi];
    const uint32_t g = ib.g[z];
    const uint32_t src = g == 1 ? n : galois_src_ks(n, g, logN);
    const u64* evk = ib.evk[z];
    for (uint32_t jb = ib.start[z]; jb < ib.start[z] + ib.count[z]; jb++) {
        const u64* raised = ib.raised[jb];
        const u64* own = ib.own[jb];
        u128 a0 = 0, a1 = 0;
        for (uint32_t j = 0; j < beta; j++) {
            if (j && (j & 7) == 0) {
                a0 = barrett128(a0, m.q, m.mu, m.bits);
                a1 = barrett128(a1, m.q, m.mu, m.bits);
            }
            const u64* dj = (r <= level && r / alpha == j) ? own + ((size_t)r << logN) : raised + ((size_t)(j * R + r) << logN);
            u64 d = dj[src];
            a0 += (u128)d * evk[((size_t)((j * 2 + 0) * M + mi) << logN) + n];
            a1 += (u128)d * evk[((size_t)((j * 2 + 1) * M + mi) << logN) + n];
        }
        u64* out = acc + ((size_t)jb * 2 * R << logN);
        out[((size_t)r << logN) + n] = barrett128(a0, m.q, m.mu, m.bits);
        out[((size_t)(R + r) << logN) + n] = barrett128(a1, m.q, m.mu, m.bits);
    }
}

// Generic-ring ModDown epilogue.  grid: (N/256, L1, 2*jobs).  conv [job][2][L1][N].
__global__ __launch_bounds__(KS_THREADS) void moddown_final_kernel(const u64* __restrict__ conv, ModDownEpilogue ep,
                                                                   const ModConst* mc, uint32_t logN) {
    const uint32_t n = blockIdx.x * KS_THREADS + threadIdx.x;
    const uint32_t r = blockIdx.y, pc = blockIdx.z, job = pc >> 1, comp = pc & 1u;
    const u64 q = mc[r].q;
    u64 a = ep.acc[((size_t)(pc * ep.R + r) << logN) + n];
    u64 c = conv[((size_t)(pc * ep.L1 + r) << logN) + n];
    u64 v = shoup_mul(submod(a, c, q), ep.pinv[r], ep.pinv_sh[r], q);
    const uint32_t g = ep.g[job];
    if (comp == 0 && ep.c0[job]) v = addmod(v, ep.c0[job][((size_t)r << logN) + (g == 1 ? n : galois_src_ks(n, g, logN))], q);
    const u64* self = comp ? ep.self1[job] : ep.self0[job];
    if (self) v = addmod(v, self[((size_t)r << logN) + n], q);
    (comp ? ep.out1[job] : ep.out0[job])[((size_t)r << logN) + n] = v;
}

int32_t launch_moddown_final(he_ctx* c, const u64* conv, uint32_t n_jobs, const ModDownEpilogue& ep) {
    dim3 grid(c->N / KS_THREADS, ep.L1, 2 * n_jobs), block(KS_THREADS);
    hipLaunchKernelGGL(moddown_final_kernel, grid, block, 0, c->stream, conv, ep, c->d_mc, c->logN);
    HE_HIP(c, hipGetLastError());
    return HE_OK;
}

// ---------------------------------------------------------------- rescale kernels
// grid: (N/256, level, 2*n).  t = coefficient-form limb `level` of (job, comp) (tmp[job*2+comp][N]);
// delta[job][comp][r] = (h mod q_r) - ((t + h mod q_l) mod q_r), h = floor(q_l/2); negate != 0 stores -delta (for the
// forward transform whose epilogue subtracts what it transformed).
__global__ __launch_bounds__(KS_THREADS) void rescale_delta_kernel(const u64* __restrict__ tmp, u64* __restrict__ delta,
                                                                   const ModConst* mc, uint32_t logN, uint32_t level, uint32_t negate) {
    const uint32_t n = blockIdx.x * KS_THREADS + threadIdx.x;
    const uint32_t r = blockIdx.y, jc = blockIdx.z;
    const ModConst ml = mc[level], mr = mc[r];
    u64 h = ml.q >> 1;
    u64 t = addmod(tmp[((size_t)jc << logN) + n], h, ml.q);
    u64 tr = barrett64(t, mr.q, mr.mu, mr.bits);
    u64 hr = barrett64(h, mr.q, mr.mu, mr.bits);
    delta[((size_t)(jc * level + r) << logN) + n] = negate ? submod(tr, hr, mr.q) : submod(hr, tr, mr.q);
}

// ---------------------------------------------------------------- host: tables

static uint32_t num_digits(const he_ctx* c, uint32_t level) { return (level + c->alpha) / c->alpha; }
static uint32_t pad8(uint32_t x) { return (x + 7u) & ~7u; }

int32_t ks_init_tables(he_ctx* c) {
    const uint32_t nq = c->nq, np = c->np, M = c->M, al = c->alpha, dn = c->dnum;
    // rescale: q_l^-1 mod q_r
    {
        std::vector<u64> inv((size_t)nq * nq, 0), inv_sh((size_t)nq * nq, 0);
        for (uint32_t l = 0; l < nq; l++)
            for (uint32_t r = 0; r < nq; r++) {
                if (r == l) continue;
                u64 v = h_invmod(c->mod[l] % c->mod[r], c->mod[r]);
                inv[(size_t)l * nq + r] = v;
                inv_sh[(size_t)l * nq + r] = h_shoup(v, c->mod[r]);
            }
        size_t b = inv.size() * sizeof(u64);
        HE_HIP(c, hipMalloc(&c->d_qlinv, b));
        HE_HIP(c, hipMalloc(&c->d_qlinv_sh, b));
        HE_HIP(c, hipMemcpy(c->d_qlinv, inv.data(), b, hipMemcpyHostToDevice));
        HE_HIP(c, hipMemcpy(c->d_qlinv_sh, inv_sh.data(), b, hipMemcpyHostToDevice));
    }
    if (np == 0) return HE_OK;
    // ModUp: digit j holding its first sz limbs (sz = 1..alpha), Q = product of those limbs.
    // Device layout [j][sz-1][modulus m][i padded to aw]: the constants of one target are contiguous.
    const uint32_t aw = pad8(al), pw = pad8(np);
    std::vector<u64> hat((size_t)dn * al * M * aw, 0);
    c->h_up_invhat.assign((size_t)dn * al * al, 0);
    for (uint32_t j = 0; j < dn; j++) {
        uint32_t lo = j * al;
        for (uint32_t sz = 1; sz <= al && lo + sz <= nq; sz++)
            for (uint32_t i = 0; i < sz; i++) {
                size_t slab = (size_t)(j * al + (sz - 1));
                u64 own = 0;
                for (uint32_t m = 0; m < M; m++) {
                    u64 v = 1;
                    for (uint32_t k = 0; k < sz; k++)
                        if (k != i) v = h_mulmod(v, c->mod[lo + k] % c->mod[m], c->mod[m]);
                    hat[(slab * M + m) * aw + i] = v;
                    if (m == lo + i) own = v;
                }
                c->h_up_invhat[slab * al + i] = h_invmod(own, c->mod[lo + i]);
            }
    }
    // ModDown: P/p_t mod every modulus ([m][t padded to pw]), (P/p_t)^-1 mod p_t, P^-1 mod q_r
    std::vector<u64> dhat((size_t)M * pw, 0), pinv(nq), pinv_sh(nq);
    c->h_dn_invhat.assign(np, 0);
    for (uint32_t t = 0; t < np; t++) {
        for (uint32_t m = 0; m < M; m++) {
            u64 v = 1;
            for (uint32_t k = 0; k < np; k++)
                if (k != t) v = h_mulmod(v, c->mod[nq + k] % c->mod[m], c->mod[m]);
            dhat[(size_t)m * pw + t] = v;
        }
        c->h_dn_invhat[t] = h_invmod(dhat[(size_t)(nq + t) * pw + t], c->mod[nq + t]);
    }
    for (uint32_t r = 0; r < nq; r++) {
        u64 P = 1;
        for (uint32_t k = 0; k < np; k++) P = h_mulmod(P, c->mod[nq + k] % c->mod[r], c->mod[r]);
        pinv[r] = h_invmod(P, c->mod[r]);
        pinv_sh[r] = h_shoup(pinv[r], c->mod[r]);
    }
    HE_HIP(c, hipMalloc(&c->d_up_hat, hat.size() * sizeof(u64)));
    HE_HIP(c, hipMalloc(&c->d_dn_hat, dhat.size() * sizeof(u64)));
    HE_HIP(c, hipMalloc(&c->d_pinv, nq * sizeof(u64)));
    HE_HIP(c, hipMalloc(&c->d_pinv_sh, nq * sizeof(u64)));
    HE_HIP(c, hipMemcpy(c->d_up_hat, hat.data(), hat.size() * sizeof(u64), hipMemcpyHostToDevice));
    HE_HIP(c, hipMemcpy(c->d_dn_hat, dhat.data(), dhat.size() * sizeof(u64), hipMemcpyHostToDevice));
    HE_HIP(c, hipMemcpy(c->d_pinv, pinv.data(), nq * sizeof(u64), hipMemcpyHostToDevice));
    HE_HIP(c, hipMemcpy(c->d_pinv_sh, pinv_sh.data(), nq * sizeof(u64), hipMemcpyHostToDevice));
    return HE_OK;
}

void ks_free_tables(he_ctx* c) {
    if (c->d_up_hat) (void)hipFree(c->d_up_hat);
    if (c->d_dn_hat) (void)hipFree(c->d_dn_hat);
    if (c->d_pinv) (void)hipFree(c->d_pinv);
    if (c->d_pinv_sh) (void)hipFree(c->d_pinv_sh);
    if (c->d_qlinv) (void)hipFree(c->d_qlinv);
    if (c->d_qlinv_sh) (void)hipFree(c->d_qlinv_sh);
}

// ---------------------------------------------------------------- host: the engine

static int32_t launch_baseconv(he_ctx* c, const ConvBatch& b, uint32_t nt_max, uint32_t ns_max) {
    dim3 grid((c->N + 2 * KS_THREADS - 1) / (2 * KS_THREADS), (nt_max + CONV_TGT_PER_BLOCK - 1) / CONV_TGT_PER_BLOCK,
              b.njobs * b.reps), block(KS_THREADS);
    if (ns_max <= 8 && c->logN == 16) hipLaunchKernelGGL((baseconv_kernel<true, true>), grid, block, 0, c->stream, b, c->d_mc, c->logN);
    else if (ns_max <= 8) hipLaunchKernelGGL((baseconv_kernel<true, false>), grid, block, 0, c->stream, b, c->d_mc, c->logN);
    else hipLaunchKernelGGL((baseconv_kernel<false, false>), grid, block, 0, c->stream, b, c->d_mc, c->logN);
    HE_HIP(c, hipGetLastError());
    return HE_OK;
}

// How many sources are raised at once and how many jobs share one ModDown launch set.
static void engine_shape(const he_ctx* c, uint32_t level, uint32_t n_src, uint32_t n_jobs, uint32_t& cb, uint32_t& jb) {
    const uint32_t L1 = level + 1, k = c->np;
    cb = std::min<uint32_t>(std::min<uint32_t>(n_src, HE_MAX_SEGS), std::max<uint32_t>(1, HE_MAX_LAUNCH_LIMBS / L1));
    cb = std::min<uint32_t>(cb, 8);
    jb = std::min<uint32_t>(n_jobs, HE_MAX_KS_JOBS);
    jb = std::min<uint32_t>(jb, std::max<uint32_t>(1, HE_MAX_LAUNCH_LIMBS / (2 * L1)));
    jb = std::min<uint32_t>(jb, std::max<uint32_t>(1, HE_MAX_LAUNCH_LIMBS / (2 * k)));
    jb = std::min<uint32_t>(jb, std::max<uint32_t>(1, 4096 / (2 * (L1 + k))));   // source limb offsets are 12 bits
    if (cb == 0) cb = 1;
    if (jb == 0) jb = 1;
}

// raised[cb][beta][R] + tmp_up[cb][L1] + acc[jb][2][R] + tmp_dn[jb][2][k] + conv[jb][2][L1]
size_t ks_engine_ws_elems(const he_ctx* c, uint32_t level, uint32_t n_src, uint32_t n_jobs) {
    uint32_t cb, jb;
    engine_shape(c, level, n_src, n_jobs, cb, jb);
    const size_t L1 = level + 1, k = c->np, R = L1 + k, beta = num_digits(c, level);
    return ((size_t)cb * (beta * R + L1) + (size_t)jb * (2 * R + 2 * k + 2 * L1)) * c->N;
}

// Whether a conversion of `groups` groups (at most `ns` sources and `nt` targets each, `sets` target sets) takes the
// single-launch column path: N = 2^16 only, and only while its work groups (256 per group, a few per compute unit)
// fit the chip about once, beyond which the separate throughput kernels win.
static bool colfuse_ok(const he_ctx* c, uint32_t groups, uint32_t sets, uint32_t ns, uint32_t nt) {
    return c->logN == 16 && groups <= c->cf_max_groups && groups <= CF_MAX_GROUPS && sets <= CF_MAX_SETS && ns <= 8 &&
           nt <= c->cf_max_targets && nt <= HE_MAX_MODULI;
}

// ModUp of `cb` sources at once.  raised [cb][beta][R][N] (own limbs left unwritten), tmp [cb][L1][N].
static int32_t modup_batch(he_ctx* c, const KsSrc* srcs, uint32_t cb, uint32_t level, u64* raised, u64* tmp) {
    const uint32_t N = c->N, L1 = level + 1, R = L1 + c->np, beta = num_digits(c, level), al = c->alpha;
    if (small_ring_path(c, level)) return sr_modup(c, srcs, cb, level, raised);   // one launch: every output limb start to finish
    // coefficient form of all limbs, each pre-multiplied by N^-1 * (Q_j/q_i)^-1
    ScaleList sc;
    for (uint32_t i = 0; i < L1; i++) {
        uint32_t j = i / al, lo = j * al, hi = (j + 1) * al < L1 ? (j + 1) * al : L1, sz = hi - lo;
        u64 qi = c->mod[i];
        scale_entry(c, sc, i, i, h_mulmod(c->h_mc[i].ninv, c->h_up_invhat[(size_t)(j * al + (sz - 1)) * al + (i - lo)], qi));
    }
    // small launches at N = 2^16: the column passes and the conversion run as one launch between the two row passes
    const bool cf_on = colfuse_ok(c, cb * beta, beta, al, R) && cb * beta * R <= HE_MAX_LAUNCH_LIMBS;
    {
        std::vector<uint32_t> mods(cb * L1);
        std::vector<uint8_t> seg(cb * L1);
        std::vector<uint16_t> lim(cb * L1);
        TransformDesc t = {};
        t.fwd = false; t.n_seg = cb; t.dst = tmp; t.n = cb * L1;
        for (uint32_t s = 0; s < cb; s++) {
            t.seg[s] = srcs[s].c1;
            for (uint32_t i = 0; i < L1; i++) { mods[s * L1 + i] = i; seg[s * L1 + i] = (uint8_t)s; lim[s * L1 + i] = (uint16_t)i; }
        }
        t.mod_idx = mods.data(); t.src_seg = seg.data(); t.src_limb = lim.data();
        t.scale = &sc; t.scale_period = L1;
        t.only_pass = cf_on ? 1u : 0u;
        int32_t rc = launch_transform(c, t);
        if (rc != HE_OK) return rc;
    }
    const uint32_t aw = pad8(al);
    if (cf_on) {
        ColFuse cf = {};
        cf.hat_w = aw; cf.n_groups = cb * beta;
        uint32_t passes = 0;
        for (uint32_t j = 0; j < beta; j++) {
            uint32_t lo = j * al, hi = (j + 1) * al < L1 ? (j + 1) * al : L1, sz = hi - lo, nt = 0;
            for (uint32_t r = 0; r < R; r++) {
                if (r >= lo && r < hi) continue;
                cf.tgt_limb[j][nt] = (uint8_t)r;
                cf.tgt_mod[j][nt] = (uint8_t)(r <= level ? r : c->nq + (r - level - 1));
                nt++;
            }
            cf.nt[j] = nt;
            for (uint32_t s = 0; s < cb; s++) {
                const uint32_t g = s * beta + j;
                cf.grp[g].src = tmp + ((size_t)s * L1 + lo) * N;
                cf.grp[g].dst = raised + ((size_t)s * beta + j) * R * N;
                cf.grp[g].hat = c->d_up_hat + (size_t)(j * al + (sz - 1)) * c->M * aw;
                cf.grp[g].ns = sz; cf.grp[g].mod0 = lo; cf.grp[g].sc0 = lo; cf.grp[g].set = j;
                passes += sz + nt;
            }
        }
        int32_t rc = launch_colfuse(c, cf, sc, passes);
        if (rc != HE_OK) return rc;
        std::vector<uint32_t> mods(cb * beta * R);
        for (uint32_t s = 0; s < cb; s++)
            for (uint32_t j = 0; j < beta; j++) {
                uint32_t lo = j * al, hi = (j + 1) * al < L1 ? (j + 1) * al : L1;
                for (uint32_t r = 0; r < R; r++)
                    mods[(s * beta + j) * R + r] = (r >= lo && r < hi) ? 0xFFu : (r <= level ? r : c->nq + (r - level - 1));
            }
        TransformDesc t = {};
        t.fwd = true; t.seg[0] = raised; t.n_seg = 1; t.dst = raised; t.n = cb * beta * R; t.mod_idx = mods.data();
        t.lazy_out = true; t.only_pass = 2;
        rc = launch_transform(c, t);
        if (rc != HE_OK) return rc;
        c->cnt.modup += cb;
        return HE_OK;
    }
    for (uint32_t j0 = 0; j0 < beta; j0 += CONV_MAX_JOBS) {
        ConvBatch b;
        b.njobs = beta - j0 < CONV_MAX_JOBS ? beta - j0 : CONV_MAX_JOBS;
        b.reps = cb;
        b.src_stride = (size_t)L1 * N;
        b.dst_stride = (size_t)beta * R * N;
        uint32_t nt_max = 0, ns_max = 0;
        for (uint32_t jj = 0; jj < b.njobs; jj++) {
            uint32_t j = j0 + jj, lo = j * al, hi = (j + 1) * al < L1 ? (j + 1) * al : L1, sz = hi - lo;
            ConvJob& job = b.job[jj];
            job.src = tmp + (size_t)lo * N;
            job.dst = raised + (size_t)j * R * N;
            job.hat = c->d_up_hat + (size_t)(j * al + (sz - 1)) * c->M * aw;
            job.hat_w = aw;
            job.ns = sz;
            job.nt = 0;
            for (uint32_t r = 0; r < R; r++) {
                if (r >= lo && r < hi) continue;
                job.tgt_limb[job.nt] = (uint8_t)r;
                job.tgt_mod[job.nt] = (uint8_t)(r <= level ? r : c->nq + (r - level - 1));
                job.nt++;
            }
            if (job.nt > nt_max) nt_max = job.nt;
            if (sz > ns_max) ns_max = sz;
        }
        int32_t rc = launch_baseconv(c, b, nt_max, ns_max);
        if (rc != HE_OK) return rc;
    }
    // NTT of every converted limb; own limbs are marked "skip"
    const uint32_t per_src = beta * R;
    std::vector<uint32_t> mods(per_src);
    for (uint32_t j = 0; j < beta; j++) {
        uint32_t lo = j * al, hi = (j + 1) * al < L1 ? (j + 1) * al : L1;
        for (uint32_t r = 0; r < R; r++)
            mods[j * R + r] = (r >= lo && r < hi) ? 0xFFu : (r <= level ? r : c->nq + (r - level - 1));
    }
    if (per_src <= HE_MAX_LAUNCH_LIMBS) {
        const uint32_t per_launch = HE_MAX_LAUNCH_LIMBS / per_src;   // sources per launch
        std::vector<uint32_t> rep;
        for (uint32_t s0 = 0; s0 < cb; s0 += per_launch) {
            uint32_t ns = std::min(per_launch, cb - s0);
            rep.resize((size_t)ns * per_src);
            for (uint32_t s = 0; s < ns; s++) std::copy(mods.begin(), mods.end(), rep.begin() + (size_t)s * per_src);
            TransformDesc t = {};
            t.fwd = true; t.seg[0] = raised + (size_t)s0 * per_src * N; t.n_seg = 1; t.dst = raised + (size_t)s0 * per_src * N;
            t.n = ns * per_src; t.mod_idx = rep.data();
            t.lazy_out = true;      // raised digits are only ever multiplied into 128-bit sums of at most 8 terms
            int32_t rc = launch_transform(c, t);
            if (rc != HE_OK) return rc;
        }
    } else {
        for (uint32_t s = 0; s < cb; s++)
            for (uint32_t o = 0; o < per_src; o += HE_MAX_LAUNCH_LIMBS) {
                uint32_t n = std::min<uint32_t>(HE_MAX_LAUNCH_LIMBS, per_src - o);
                int32_t rc = launch_ntt(c, raised + ((size_t)s * per_src + o) * N, mods.data() + o, n);
                if (rc != HE_OK) return rc;
            }
    }
    c->cnt.modup += cb;
    return HE_OK;
}

// Stand-alone inner product of the jobs described by `ib` (grouped by key): acc [job][2][R][N].
static int32_t launch_inner_product(he_ctx* c, uint32_t level, const IpBatch& ib, uint32_t groups, u64* acc) {
    const uint32_t R = level + 1 + c->np, beta = num_digits(c, level);
    dim3 grid(c->N / KS_THREADS, R, groups), block(KS_THREADS);
    if (beta <= 4)
        hipLaunchKernelGGL(inner_product_kernel<4>, grid, block, 0, c->stream, ib, acc, c->d_mc, c->logN, R, beta, c->M, level,
                           c->nq, c->alpha);
    else if (beta <= 8)
        hipLaunchKernelGGL(inner_product_kernel<8>, grid, block, 0, c->stream, ib, acc, c->d_mc, c->logN, R, beta, c->M, level,
                           c->nq, c->alpha);
    else
        hipLaunchKernelGGL(inner_product_wide_kernel, grid, block, 0, c->stream, ib, acc, c->d_mc, c->logN, R, beta, c->M,
                           level, c->nq, c->alpha);
    HE_HIP(c, hipGetLastError());
    return HE_OK;
}

// The ModDown of J accumulators (each [2][R][N]; on the fused N = 2^16 path they are never stored and `ip` / `ep`
// describe how the transforms compute them): special-prime limbs -> coefficient form (pre-multiplied by
// N^-1 * (P/p_t)^-1), conversion to q_0..q_level, forward transform with the epilogue described by `ep`.
static int32_t moddown_chain(he_ctx* c, uint32_t level, uint32_t J, u64* acc, u64* tmp_dn, u64* conv, const IpPrologue* ip,
                             const ModDownEpilogue& ep) {
    const uint32_t N = c->N, L1 = level + 1, k = c->np, R = L1 + k;
    const bool cf_on = colfuse_ok(c, 2 * J, 1, k, L1) && 2 * J * std::max(k, L1) <= HE_MAX_LAUNCH_LIMBS;
    ScaleList sc;
    for (uint32_t t = 0; t < k; t++) {
        u64 p = c->mod[c->nq + t];
        scale_entry(c, sc, t, c->nq + t, h_mulmod(c->h_mc[c->nq + t].ninv, c->h_dn_invhat[t], p));
    }
    {
        const uint32_t n = J * 2 * k;
        std::vector<uint32_t> mods(n);
        std::vector<uint16_t> lim(n);
        for (uint32_t i = 0; i < n; i++) {
            uint32_t t = i % k, pc = i / k;
            mods[i] = c->nq + t;
            lim[i] = (uint16_t)(pc * R + L1 + t);
        }
        TransformDesc t = {};
        t.fwd = false; t.seg[0] = acc; t.n_seg = 1; t.dst = tmp_dn; t.n = n;
        t.mod_idx = mods.data(); t.src_limb = lim.data(); t.scale = &sc; t.scale_period = k;
        t.ip = ip;
        t.only_pass = cf_on ? 1u : 0u;
        int32_t rc = launch_transform(c, t);
        if (rc != HE_OK) return rc;
    }
    if (cf_on) {
        ColFuse cf = {};
        cf.hat_w = pad8(k); cf.n_groups = 2 * J;
        cf.nt[0] = L1;
        for (uint32_t r = 0; r < L1; r++) { cf.tgt_limb[0][r] = (uint8_t)r; cf.tgt_mod[0][r] = (uint8_t)r; }
        for (uint32_t g = 0; g < 2 * J; g++) {
            cf.grp[g].src = tmp_dn + (size_t)g * k * N;
            cf.grp[g].dst = conv + (size_t)g * L1 * N;
            cf.grp[g].hat = c->d_dn_hat;
            cf.grp[g].ns = k; cf.grp[g].mod0 = c->nq; cf.grp[g].sc0 = 0; cf.grp[g].set = 0;
        }
        int32_t rc = launch_colfuse(c, cf, sc, 2 * J * (k + L1));
        if (rc != HE_OK) return rc;
    } else {
        ConvBatch b;
        b.njobs = 1; b.reps = 2 * J;
        b.src_stride = (size_t)k * N;
        b.dst_stride = (size_t)L1 * N;
        ConvJob& job = b.job[0];
        job.src = tmp_dn; job.dst = conv; job.hat = c->d_dn_hat; job.hat_w = pad8(k); job.ns = k; job.nt = L1;
        for (uint32_t r = 0; r < L1; r++) { job.tgt_limb[r] = (uint8_t)r; job.tgt_mod[r] = (uint8_t)r; }
        int32_t rc = launch_baseconv(c, b, L1, k);
        if (rc != HE_OK) return rc;
    }
    {
        const uint32_t n = J * 2 * L1;
        std::vector<uint32_t> mods(n);
        for (uint32_t i = 0; i < n; i++) mods[i] = i % L1;
        TransformDesc t = {};
        t.fwd = true; t.seg[0] = conv; t.n_seg = 1; t.dst = conv; t.n = n; t.mod_idx = mods.data(); t.ep = &ep;
        t.lazy_out = true;
        t.only_pass = cf_on ? 2u : 0u;
        int32_t rc = launch_transform(c, t);
        if (rc != HE_OK) return rc;
    }
    c->cnt.moddown += J;
    return HE_OK;
}

// Inner product + ModDown of up to HE_MAX_KS_JOBS jobs whose sources are already raised.
// raised_of[i] / srcs give job i's raised digits and source; scratch: acc, tmp_dn, conv.
static int32_t inner_moddown_batch(he_ctx* c, uint32_t level, const KsSrc* srcs, const KsJob* jobs, const u64* const* raised_of,
                                   uint32_t J, u64* acc, u64* tmp_dn, u64* conv) {
    const uint32_t N = c->N, L1 = level + 1, k = c->np, R = L1 + k, beta = num_digits(c, level);
    // group consecutive jobs that use the same key and Galois element (the caller sorts them)
    IpBatch ib;
    uint32_t groups = 0;
    for (uint32_t i = 0; i < J; i++) {
        ib.raised[i] = raised_of[i];
        ib.own[i] = srcs[jobs[i].src].c1;
        if (groups && ib.evk[groups - 1] == jobs[i].evk && ib.g[groups - 1] == jobs[i].g) {
            ib.count[groups - 1]++;
        } else {
            ib.evk[groups] = jobs[i].evk; ib.g[groups] = jobs[i].g; ib.start[groups] = i; ib.count[groups] = 1;
            groups++;
        }
    }
    if (c->prof_on) c->prof_key_limbs += (uint64_t)groups * 2 * beta * R;
    // On the N = 2^16 path no accumulator is materialised: the special-prime limbs of the inner product are
    // computed by the first pass of their inverse transform, the q-limbs inside the ModDown epilogue (they would
    // only be written here and read back there).  Other rings run the stand-alone kernel.
    const bool fused = c->logN == 16 && beta <= 8;
    // small rings: inner product, ModDown and epilogue of every output limb in one work group, one launch
    const bool small = !fused && small_ring_path(c, level);
    IpPrologue ip = {};
    if (fused) {
        ip.beta = beta; ip.R = R; ip.M = c->M; ip.L1 = L1; ip.k = k; ip.nq = c->nq;
        for (uint32_t i = 0; i < J; i++) { ip.raised[i] = raised_of[i]; ip.evk[i] = jobs[i].evk; ip.g[i] = jobs[i].g; }
    } else if (!small) {
        int32_t rc = launch_inner_product(c, level, ib, groups, acc);
        if (rc != HE_OK) return rc;
    }
    ModDownEpilogue ep = {};
    ep.acc = acc; ep.pinv = c->d_pinv; ep.pinv_sh = c->d_pinv_sh; ep.R = R; ep.L1 = L1;
    ep.fused = fused ? 1u : 0u; ep.beta = beta; ep.alpha = c->alpha; ep.M = c->M;
    for (uint32_t i = 0; i < J; i++) {
        const KsSrc& src = srcs[jobs[i].src];
        ep.raised[i] = raised_of[i]; ep.own[i] = src.c1; ep.evk[i] = jobs[i].evk;
        ep.c0[i] = src.c0;
        ep.self0[i] = jobs[i].add_self ? src.s0 : nullptr;
        ep.self1[i] = jobs[i].add_self ? src.s1 : nullptr;
        ep.out0[i] = jobs[i].out0; ep.out1[i] = jobs[i].out1;
        ep.g[i] = jobs[i].g;
        if (ep.c0[i]) c->cnt.automorph += L1;
    }
    int32_t rc = small ? sr_moddown(c, level, J, ep) : moddown_chain(c, level, J, acc, tmp_dn, conv, fused ? &ip : nullptr, ep);
    if (rc != HE_OK) return rc;
    c->cnt.keyswitch += J;
    return HE_OK;
}

int32_t ks_engine(he_ctx* c, uint32_t level, const KsSrc* srcs, uint32_t n_src, const KsJob* jobs, uint32_t n_jobs) {
    if (n_jobs == 0) return HE_OK;
    const uint32_t N = c->N, L1 = level + 1, k = c->np, R = L1 + k, beta = num_digits(c, level);
    if (2 * k > HE_MAX_MODULI) return he_fail(c, HE_ERR_BADARG, "key switch: more than %d special primes", HE_MAX_MODULI / 2);
    int32_t rc = he_ensure_ws(c, ks_engine_ws_elems(c, level, n_src, n_jobs) * sizeof(u64));
    if (rc != HE_OK) return rc;
    uint32_t cb, jb;
    engine_shape(c, level, n_src, n_jobs, cb, jb);
    u64* raised = c->d_ws;
    u64* tmp_up = raised + (size_t)cb * beta * R * N;
    u64* acc = tmp_up + (size_t)cb * L1 * N;
    u64* tmp_dn = acc + (size_t)jb * 2 * R * N;
    u64* conv = tmp_dn + (size_t)jb * 2 * k * N;
    // jobs ordered by source wave, then by key so that equal keys are adjacent
    std::vector<uint32_t> order(n_jobs);
    for (uint32_t i = 0; i < n_jobs; i++) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) {
        uint32_t wa = jobs[a].src / cb, wb = jobs[b].src / cb;
        if (wa != wb) return wa < wb;
        if (jobs[a].evk != jobs[b].evk) return jobs[a].evk < jobs[b].evk;
        return jobs[a].g < jobs[b].g;
    });
    size_t pos = 0;
    for (uint32_t s0 = 0; s0 < n_src; s0 += cb) {
        const uint32_t ns = std::min(cb, n_src - s0);
        size_t end = pos;
        while (end < n_jobs && jobs[order[end]].src / cb == s0 / cb) end++;
        if (end == pos) continue;                       // no job uses these sources
        rc = modup_batch(c, srcs + s0, ns, level, raised, tmp_up);
        if (rc != HE_OK) return rc;
        while (pos < end) {
            uint32_t J = (uint32_t)std::min<size_t>(jb, end - pos);
            // do not split a run of same-key jobs across two launch sets (each set would pass over the key once) when
            // the set can end at a key boundary in its second half instead
            if (pos + J < end && jobs[order[pos + J - 1]].evk == jobs[order[pos + J]].evk) {
                uint32_t b = J;
                while (b > 1 && jobs[order[pos + b - 1]].evk == jobs[order[pos + b]].evk) b--;
                if (2 * b >= J) J = b;
            }
            KsJob chunk[HE_MAX_KS_JOBS];
            const u64* raised_of[HE_MAX_KS_JOBS];
            for (uint32_t i = 0; i < J; i++) {
                chunk[i] = jobs[order[pos + i]];
                raised_of[i] = raised + (size_t)(chunk[i].src - s0) * beta * R * N;
            }
            rc = inner_moddown_batch(c, level, srcs, chunk, raised_of, J, acc, tmp_dn, conv);
            if (rc != HE_OK) return rc;
            pos += J;
        }
    }
    return HE_OK;
}


// ---------------------------------------------------------------- sum of rotations, one ModDown
// out = sum_t Rot(term_t) with the ModDown deferred across the sum: every rotated term is raised and multiplied
// into its key, the products are summed over the raised basis and only the sum is brought down;
// out0 also receives sum_t sigma_g_t(c0_t), and terms with g = 1 are added as they are.

struct RotSumArgs {
    const u64* c0[HE_MAX_SUM_TERMS];     // rotated terms first (n_rot), then the plain ones (n_plain)
    const u64* c1[HE_MAX_SUM_TERMS];     // used for the plain terms only
    uint32_t g[HE_MAX_SUM_TERMS];
    uint32_t n_rot, n_plain;
};
// grid (N/256, L1, 1 or 2).  z = 0: s0[r][n] = sum_rot c0_t[r][sigma-source of n] + sum_plain c0_p[r][n];
// z = 1 (launched only if there are plain terms): s1[r][n] = sum_plain c1_p[r][n].
__global__ __launch_bounds__(KS_THREADS) void rot_sum_kernel(RotSumArgs a, u64* __restrict__ s0, u64* __restrict__ s1, const ModConst* mc,
                                                             uint32_t logN) {
    const uint32_t n = blockIdx.x * KS_THREADS + threadIdx.x, r = blockIdx.y;
    const u64 q = mc[r].q;
    const size_t o = ((size_t)r << logN) + n;
    u64 v = 0;
    if (blockIdx.z == 0) {
        for (uint32_t t = 0; t < a.n_rot; t++) v = addmod(v, a.c0[t][((size_t)r << logN) + galois_src_ks(n, a.g[t], logN)], q);
        for (uint32_t t = a.n_rot; t < a.n_rot + a.n_plain; t++) v = addmod(v, a.c0[t][o], q);
        s0[o] = v;
    } else {
        for (uint32_t t = a.n_rot; t < a.n_rot + a.n_plain; t++) v = addmod(v, a.c1[t][o], q);
        s1[o] = v;
    }
}

// acc[0] (+)= sum_{t=1..n} acc[t], each [2][R][N]; raised-basis limb r = blockIdx.y % R.  grid (N/256, 2R).
__global__ __launch_bounds__(KS_THREADS) void acc_sum_kernel(u64* __restrict__ acc, uint32_t n, uint32_t init, const ModConst* mc,
                                                             uint32_t logN, uint32_t R, uint32_t level, uint32_t nq) {
    const uint32_t i = blockIdx.x * KS_THREADS + threadIdx.x, cr = blockIdx.y, r = cr % R;
    const u64 m = mc[r <= level ? r : nq + (r - level - 1)].q;
    const size_t stride = (size_t)2 * R << logN, o = ((size_t)cr << logN) + i;
    u64 v = init ? 0 : acc[o];
    for (uint32_t t = 1; t <= n; t++) v = addmod(v, acc[t * stride + o], m);
    acc[o] = v;
}

static uint32_t rot_sum_cb(const he_ctx* c, uint32_t level, uint32_t n_rot) {
    uint32_t cb, jb;
    engine_shape(c, level, n_rot ? n_rot : 1, 1, cb, jb);
    return cb;
}
static bool rot_sum_fused(const he_ctx* c, uint32_t level, uint32_t n_rot) {
    return c->logN == 16 && num_digits(c, level) <= 8 && n_rot <= HE_MAX_KS_JOBS;
}

// raised[n_rot][beta][R] + tmp_up[cb][L1] + s0[L1] + s1[L1] + tmp_dn[2][k] + conv[2][L1] (+ acc[1 + min(n_rot,16)][2][R]
// where the accumulators have to be stored)
size_t ks_rotate_sum_ws_elems(const he_ctx* c, uint32_t level, uint32_t n_rot) {
    const size_t L1 = level + 1, k = c->np, R = L1 + k, beta = num_digits(c, level);
    size_t e = (size_t)n_rot * beta * R + (size_t)rot_sum_cb(c, level, n_rot) * L1 + 2 * L1 + 2 * k + 2 * L1;
    if (!rot_sum_fused(c, level, n_rot)) e += (size_t)(1 + std::min<uint32_t>(n_rot, HE_MAX_KS_JOBS)) * 2 * R;
    return e * c->N;
}

int32_t ks_rotate_sum_deferred(he_ctx* c, uint32_t level, const KsSumTerm* terms, uint32_t n_terms, u64* out0, u64* out1, u64* ws) {
    const uint32_t N = c->N, L1 = level + 1, k = c->np, R = L1 + k, beta = num_digits(c, level);
    if (n_terms == 0 || n_terms > HE_MAX_SUM_TERMS) return he_fail(c, HE_ERR_BADARG, "rotation sum: between 1 and %d terms", HE_MAX_SUM_TERMS);
    if (2 * k > HE_MAX_MODULI) return he_fail(c, HE_ERR_BADARG, "key switch: more than %d special primes", HE_MAX_MODULI / 2);
    std::vector<const KsSumTerm*> rot, plain;
    for (uint32_t t = 0; t < n_terms; t++) (terms[t].g == 1 ? plain : rot).push_back(&terms[t]);
    const uint32_t n_rot = (uint32_t)rot.size(), n_plain = (uint32_t)plain.size();
    RotSumArgs ra = {};
    ra.n_rot = n_rot; ra.n_plain = n_plain;
    for (uint32_t t = 0; t < n_rot; t++) { ra.c0[t] = rot[t]->c0; ra.c1[t] = rot[t]->c1; ra.g[t] = rot[t]->g; }
    for (uint32_t t = 0; t < n_plain; t++) { ra.c0[n_rot + t] = plain[t]->c0; ra.c1[n_rot + t] = plain[t]->c1; ra.g[n_rot + t] = 1; }
    if (n_rot == 0) {                                   // nothing to switch: the plain sum is the result
        hipLaunchKernelGGL(rot_sum_kernel, dim3(N / KS_THREADS, L1, 2), dim3(KS_THREADS), 0, c->stream, ra, out0, out1, c->d_mc, c->logN);
        HE_HIP(c, hipGetLastError());
        return HE_OK;
    }
    const uint32_t cb = rot_sum_cb(c, level, n_rot);
    const bool fused = rot_sum_fused(c, level, n_rot);
    u64* raised = ws;
    u64* tmp_up = raised + (size_t)n_rot * beta * R * N;
    u64* s0 = tmp_up + (size_t)cb * L1 * N;
    u64* s1 = s0 + (size_t)L1 * N;
    u64* tmp_dn = s1 + (size_t)L1 * N;
    u64* conv = tmp_dn + (size_t)2 * k * N;
    u64* acc = conv + (size_t)2 * L1 * N;               // stored accumulators: [0] the sum, [1..] one group of terms
    // ModUp of every rotated term's c1; terms that rotate the same polynomial share its raised digits (hoisting)
    std::vector<KsSrc> srcs;
    std::vector<uint32_t> src_of(n_rot);
    for (uint32_t t = 0; t < n_rot; t++) {
        uint32_t u = 0;
        while (u < srcs.size() && srcs[u].c1 != rot[t]->c1) u++;
        if (u == srcs.size()) srcs.push_back({rot[t]->c0, rot[t]->c1, nullptr, nullptr});
        src_of[t] = u;
    }
    const uint32_t n_src = (uint32_t)srcs.size();
    for (uint32_t t0 = 0; t0 < n_src; t0 += cb) {
        int32_t rc = modup_batch(c, srcs.data() + t0, std::min(cb, n_src - t0), level, raised + (size_t)t0 * beta * R * N, tmp_up);
        if (rc != HE_OK) return rc;
    }
    // the rotated c0 parts and the plain terms, summed
    hipLaunchKernelGGL(rot_sum_kernel, dim3(N / KS_THREADS, L1, n_plain ? 2 : 1), dim3(KS_THREADS), 0, c->stream, ra, s0, s1, c->d_mc, c->logN);
    HE_HIP(c, hipGetLastError());
    c->cnt.automorph += (uint64_t)n_rot * L1;
    IpPrologue ip = {};
    ModDownEpilogue ep = {};
    ep.acc = acc; ep.pinv = c->d_pinv; ep.pinv_sh = c->d_pinv_sh; ep.R = R; ep.L1 = L1;
    ep.fused = fused ? 1u : 0u; ep.beta = beta; ep.alpha = c->alpha; ep.M = c->M;
    ep.c0[0] = nullptr; ep.self0[0] = s0; ep.self1[0] = n_plain ? s1 : nullptr;
    ep.out0[0] = out0; ep.out1[0] = out1; ep.g[0] = 1;
    if (fused) {
        ip.beta = beta; ip.R = R; ip.M = c->M; ip.L1 = L1; ip.k = k; ip.nq = c->nq; ip.n_terms = n_rot;
        ep.n_terms = n_rot;
        for (uint32_t t = 0; t < n_rot; t++) {
            ip.raised[t] = ep.raised[t] = raised + (size_t)src_of[t] * beta * R * N;
            ip.evk[t] = ep.evk[t] = rot[t]->evk;
            ip.g[t] = ep.g[t] = rot[t]->g;
            ep.own[t] = rot[t]->c1;
        }
        if (c->prof_on) c->prof_key_limbs += (uint64_t)n_rot * 2 * beta * R;
    } else {
        for (uint32_t t0 = 0; t0 < n_rot; t0 += HE_MAX_KS_JOBS) {
            const uint32_t cnt = std::min<uint32_t>(HE_MAX_KS_JOBS, n_rot - t0);
            IpBatch ib;
            for (uint32_t i = 0; i < cnt; i++) {
                ib.raised[i] = raised + (size_t)src_of[t0 + i] * beta * R * N;
                ib.own[i] = rot[t0 + i]->c1;
                ib.evk[i] = rot[t0 + i]->evk; ib.g[i] = rot[t0 + i]->g; ib.start[i] = i; ib.count[i] = 1;
            }
            int32_t rc = launch_inner_product(c, level, ib, cnt, acc + (size_t)2 * R * N);
            if (rc != HE_OK) return rc;
            hipLaunchKernelGGL(acc_sum_kernel, dim3(N / KS_THREADS, 2 * R), dim3(KS_THREADS), 0, c->stream, acc, cnt, t0 == 0 ? 1u : 0u,
                               c->d_mc, c->logN, R, level, c->nq);
            HE_HIP(c, hipGetLastError());
            if (c->prof_on) c->prof_key_limbs += (uint64_t)cnt * 2 * beta * R;
        }
    }
    int32_t rc = moddown_chain(c, level, 1, acc, tmp_dn, conv, fused ? &ip : nullptr, ep);
    if (rc != HE_OK) return rc;
    c->cnt.keyswitch += n_rot;
    return HE_OK;
}

// ---------------------------------------------------------------- the same sum of rotations of several ciphertexts
// out_j = ct_j' + sum_{t<T} Rot(ct_j; g_t) for j < J with ONE ModUp and ONE ModDown per ciphertext (rotate-and-sum over
// C_a, Section 2.2, evaluated as the sum of its C_a - 1 rotations of the input instead of log2 C_a dependent steps):
//   A_j   = sum_t sum_i sigma_{g_t}(ModUp(c1_j)_i) * evk_t,i
//   out_j = ( sum_t sigma_{g_t}(c0_j) + ModDown(A_j,0) + s0_j , ModDown(A_j,1) + s1_j )     (s0_j, s1_j: addends or null)
// The T keys are shared by all J ciphertexts: the inner products of up to 8 ciphertexts run in one register-tiled kernel
// into stored accumulators, which the ModDown then reads.

// grid (N/256, L1, J): s0_j[r][n] = sum_t c0_j[r][sigma_t-source of n] (+ add_j[r][n])
struct HoistC0 {
    const u64* c0[HE_MAX_KS_JOBS];
    const u64* add[HE_MAX_KS_JOBS];
    u64* s0[HE_MAX_KS_JOBS];
    uint32_t g[HE_MAX_KS_JOBS];
    uint32_t T;
};
// Every Galois element moves values only inside aligned blocks of 256 positions (see hoisted_sum_ip_local_kernel): the
// work group's 256 values are read once into LDS and gathered from there.
__global__ __launch_bounds__(KS_THREADS) void hoist_c0_sum_kernel(HoistC0 a, const ModConst* mc, uint32_t logN) {
    __shared__ u64 tile[KS_THREADS];
    const uint32_t n = blockIdx.x * KS_THREADS + threadIdx.x, r = blockIdx.y, j = blockIdx.z;
    const u64 q = mc[r].q;
    const size_t o = ((size_t)r << logN) + n;
    const u64* c0 = a.c0[j] + ((size_t)r << logN);
    u64 v = a.add[j] ? a.add[j][o] : 0;
    tile[threadIdx.x] = c0[n];
    __syncthreads();
    for (uint32_t t = 0; t < a.T; t++) v = addmod(v, tile[galois_src_ks(n, a.g[t], logN) & (KS_THREADS - 1)], q);
    a.s0[j][o] = v;
}

// Inner products of a hoisted sum for up to HS_JOBS ciphertexts at once, register-tiled: a thread owns one point of
// one raised-basis limb for all the ciphertexts and both components; per (term, digit) it loads the two key values
// once and one digit value per ciphertext, and feeds 2*J multiply-accumulates.
// acc [J][2][R][N] (canonical); init = 0 continues from its contents (more than HS_TERMS terms).
#define HS_JOBS 8
#define HS_TERMS 16
struct HoistIp {
    const u64* raised[HS_JOBS];   // [beta][R][N], own limbs not materialised
    const u64* own[HS_JOBS];      // the switched polynomial [L1][N]
    const u64* evk[HS_TERMS];
    uint32_t g[HS_TERMS];
    uint32_t J, T;
};

// Every Galois element of the list must be 1 modulo 2^(logN-7): such a map moves a value only inside its aligned block
// of 256 positions (the low logN-8 bits of the exponent index g*k + (g-1)/2 are those of k, i.e. the high bits of the
// position stay), which is the case for rotations by multiples of N/512 slots - the rotate-and-sum amounts over up to
// 256 channel blocks (over up to 16 of them the values even stay inside aligned blocks of 16, and the LDS reads below are
// free of bank conflicts).  Then a work group's 256 points need exactly their own 256 values of every digit, for
// every term: they are loaded once into LDS and each term reads them back permuted, so that the only global loads left
// per (term, digit) are the two key values.  LDS: J*beta*2 KiB.  grid (N/256, number of limbs in sel).
//
// Products are taken in halves, three multiplications each: the kernel is bound by its vector instructions (measured:
// they issue nearly all the time with three wavefronts per SIMD), so their count per product is what matters.  With
// h = 27 for moduli of at most 54 bits and h = 30 for wider ones (up to 60 bits), a canonical digit value d = d1*2^h + d0 and a canonical key value
// k = k1*2^h + k0 give d*k = d0*k0 + (d0*k1 + d1*k0)*2^h + d1*k1*2^2h with d0*k1 + d1*k0 = (d0-d1)*(k1-k0) + d0*k0 + d1*k1.
// Three 64-bit accumulators per output take the sums of d0*k0, of d1*k1 and (signed) of (d0-d1)*(k1-k0) directly from
// the 32x32+64-bit multiply-adds, with no carries: three instructions per product, against four multiply-adds and ten
// others (carries, moves) for a 128-bit accumulation.  Every partial product is below 2^2h in magnitude, so after `period` pairs (32 for h = 27, 6
// for h = 30: (period+3)*2^2h < 2^64, and period*2^(2*bits-2h) + 3q < 100q) the middle sum is formed, the carries of the
// low and middle sums move up, the high sum is brought below 3q, and the signed accumulator is set to what keeps the
// identity; the three sums are put together and reduced once at the end.  Digits are made canonical (the forward
// transform may leave them below 69q) and split while they are staged into LDS, the low half in the low word.  JT = size
// of the register tile: ciphertexts a.J..JT-1 repeat ciphertext 0 and are not stored.
#define HSL_MAX_TILES 24      // J * beta digit tiles of 2 KiB: 48 KiB of LDS
#define HSL_RING 2            // (term, digit) pairs whose key values are in registers or on their way
// the raised-basis limbs one launch works on: blockIdx.y indexes this list
struct LimbSel {
    uint32_t r[HE_MAX_MODULI];
};
template <int JT>
__global__ __launch_bounds__(KS_THREADS, 3) void hoisted_sum_ip_local_kernel(HoistIp a, LimbSel sel, u64* __restrict__ acc,
                                                                             const ModConst* mc, uint32_t logN, uint32_t R,
                                                                             uint32_t beta, uint32_t M, uint32_t level, uint32_t nq,
                                                                             uint32_t alpha, uint32_t init) {
    extern __shared__ u64 dig[];                         // a.J * beta tiles of KS_THREADS values
    const uint32_t n = blockIdx.x * KS_THREADS + threadIdx.x, r = sel.r[blockIdx.y];
    const uint32_t mi = r <= level ? r : nq + (r - level - 1);
    const ModConst m = mc[mi];
    const uint32_t mrec = (1u << 24) / ((uint32_t)(m.q >> (m.bits - 8)) + 1);
    const uint32_t h = m.bits > 54 ? 30u : 27u, period = m.bits > 54 ? 6u : 32u;
    const u64 lo_h = (1ull << h) - 1;
    const size_t ro = ((size_t)r << logN) + n, cstride = (size_t)R << logN;
    for (uint32_t j = 0; j < beta; j++) {
        const bool own_digit = r <= level && r / alpha == j;
        const size_t doff = own_digit ? ro : ((size_t)(j * R + r) << logN) + n;
#pragma unroll
        for (int i = 0; i < JT; i++) {
            if ((uint32_t)i < a.J) {
                const u64 v = reduce_small((own_digit ? a.own[i] : a.raised[i])[doff], m.q, m.bits, mrec);
                dig[(j * a.J + i) * KS_THREADS + threadIdx.x] = (v & lo_h) | ((v >> h) << 32);
            }
        }
    }
    // per output and component: low sum, high sum, and the signed sum bm = (middle sum) - low - high
    // (bm is kept modulo 2^64: the middle sum it stands for is below 2^64, so wrap-around arithmetic recovers it)
    u64 b0[JT], b2[JT], a0[JT], a2[JT], bm[JT], am[JT];
#pragma unroll
    for (int i = 0; i < JT; i++) b0[i] = b2[i] = a0[i] = a2[i] = bm[i] = am[i] = 0;
    __syncthreads();
    const size_t kstride = (size_t)M << logN, koff = ((size_t)mi << logN) + n;
    // lane t (mod 16) keeps term t's key address and Galois element: the loop then picks them with a lane read instead
    // of a scalar load from the argument block, whose latency every step would wait for
    uint32_t kp_lo = 0, kp_hi = 0, g_lane = 1;
#pragma unroll
    for (int tt = 0; tt < HS_TERMS; tt++) {
        if ((threadIdx.x & (HS_TERMS - 1)) == (uint32_t)tt) {
            kp_lo = (uint32_t)(uintptr_t)a.evk[tt]; kp_hi = (uint32_t)((uintptr_t)a.evk[tt] >> 32); g_lane = a.g[tt];
        }
    }
    auto key_of = [&](uint32_t term) {
        const uint32_t lo = __builtin_amdgcn_readlane(kp_lo, term), hi = __builtin_amdgcn_readlane(kp_hi, term);
        return (const u64 __attribute__((address_space(1)))*)(((uintptr_t)hi << 32) | lo);   // a global, not a generic, address
    };
    // Software pipeline, pinned with scheduling barriers (left alone, the compiler issues every LDS read right before its
    // use and waits for it).  The register tile is worked in two halves: while one half's products run, the digit values
    // of the other half - of this pair, then of the next pair - are on their way from LDS; the key values of a pair are
    // requested HSL_RING pairs ahead.  Past the end the last key pair is requested again and its products are switched
    // off, so that the loop body has no branch around a load.
    constexpr int HA = (JT + 1) / 2, HB = JT - HA;
    u64 kb[HSL_RING], ka[HSL_RING], dA[HA], dB[HB > 0 ? HB : 1];
    uint32_t tp = 0, jp = 0, pending = 0;
    auto request_key = [&](u64& kbu, u64& kau) {
        const bool more = tp < a.T;
        const auto e = key_of(more ? tp : a.T - 1) + (size_t)(2 * (more ? jp : beta - 1)) * kstride + koff;
        kbu = e[0]; kau = e[kstride];
        if (more && ++jp == beta) { jp = 0; tp++; }
    };
    // (t, j) = the pair whose digits are read next, lsrc = where this thread's value of term t sits in its tile
    uint32_t t = 0, j = 0;
    auto lsrc_of = [&](uint32_t term) {
        return galois_src_ks(n, __builtin_amdgcn_readlane(g_lane, term < a.T ? term : 0), logN) & (KS_THREADS - 1);
    };
    uint32_t lsrc = lsrc_of(0);
    auto read_a = [&]() {
        const u64* dj = dig + (size_t)j * a.J * KS_THREADS + lsrc;
#pragma unroll
        for (int i = 0; i < HA; i++) dA[i] = dj[((uint32_t)i < a.J ? i : 0) * KS_THREADS];
    };
    auto read_b = [&]() {
        const u64* dj = dig + (size_t)j * a.J * KS_THREADS + lsrc;
#pragma unroll
        for (int i = 0; i < HB; i++) dB[i] = dj[((uint32_t)(HA + i) < a.J ? HA + i : 0) * KS_THREADS];
    };
    // the middle sum formed (it is below 2^64, so wrap-around arithmetic gives it exactly), carries moved up (low and
    // middle sums back below 2^h), the high sum, which stays below 100q, brought below 3q, and the signed sum set to
    // middle - low - high again: the value of the three sums together is unchanged modulo q
    auto fold1 = [&](u64& lo, u64& mid_s, u64& hi) {
        u64 mid = mid_s + lo + hi;
        mid += lo >> h; lo &= lo_h;
        hi = reduce_small_lazy(hi + (mid >> h), m.q, m.bits, mrec); mid &= lo_h;
        mid_s = mid - lo - hi;
    };
    auto fold = [&]() {
#pragma unroll
        for (int i = 0; i < JT; i++) { fold1(b0[i], bm[i], b2[i]); fold1(a0[i], am[i], a2[i]); }
        pending = 0;
    };
    // kbd = kb1 - kb0, kad = ka1 - ka0 (signed)
    auto mac = [&](int i, u64 d, uint32_t kb0, uint32_t kb1, int32_t kbd, uint32_t ka0, uint32_t ka1, int32_t kad) {
        const uint32_t d0 = (uint32_t)d, d1 = (uint32_t)(d >> 32);
        const int32_t dd = (int32_t)(d0 - d1);
        b0[i] += (u64)d0 * kb0; b2[i] += (u64)d1 * kb1; bm[i] += (u64)((int64_t)dd * kbd);
        a0[i] += (u64)d0 * ka0; a2[i] += (u64)d1 * ka1; am[i] += (u64)((int64_t)dd * kad);
    };
    auto step = [&](u64& kbu, u64& kau, bool valid) {
        read_b();                                                   // the second half of this pair's digits
        __builtin_amdgcn_sched_barrier(0);
        const u64 kbv = valid ? kbu : 0, kav = valid ? kau : 0;     // a step past the end adds nothing
        const uint32_t kb0 = (uint32_t)(kbv & lo_h), kb1 = (uint32_t)(kbv >> h);
        const uint32_t ka0 = (uint32_t)(kav & lo_h), ka1 = (uint32_t)(kav >> h);
        const int32_t kbd = (int32_t)(kb1 - kb0), kad = (int32_t)(ka1 - ka0);
#pragma unroll
        for (int i = 0; i < HA; i++) mac(i, dA[i], kb0, kb1, kbd, ka0, ka1, kad);
        __builtin_amdgcn_sched_barrier(0);
        if (++j == beta) { j = 0; t++; lsrc = lsrc_of(t); }
        read_a();                                                   // the first half of the next pair's digits
        request_key(kbu, kau);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < HB; i++) mac(HA + i, dB[i], kb0, kb1, kbd, ka0, ka1, kad);
        pending++;
    };
    const uint32_t total = a.T * beta;
#pragma unroll
    for (int u = 0; u < HSL_RING; u++) request_key(kb[u], ka[u]);
    read_a();
    for (uint32_t it = 0; it < total; it += HSL_RING) {  // HSL_RING steps per trip, none of them conditional
        if (pending + HSL_RING > period) fold();
#pragma unroll
        for (int u = 0; u < HSL_RING; u++) step(kb[u], ka[u], it + u < total);
    }
    fold();
#pragma unroll
    for (int i = 0; i < JT; i++) {
        if ((uint32_t)i < a.J) {
            const u64 b1 = bm[i] + b0[i] + b2[i], a1 = am[i] + a0[i] + a2[i];
            const u64 vb = barrett128((u128)b0[i] + ((u128)b1 << h) + ((u128)b2[i] << (2 * h)), m.q, m.mu, m.bits);
            const u64 va = barrett128((u128)a0[i] + ((u128)a1 << h) + ((u128)a2[i] << (2 * h)), m.q, m.mu, m.bits);
            u64* o0 = acc + (size_t)(2 * i) * cstride + ro;
            u64* o1 = acc + (size_t)(2 * i + 1) * cstride + ro;
            *o0 = init ? vb : addmod(vb, *o0, m.q);
            *o1 = init ? va : addmod(va, *o1, m.q);
        }
    }
}

// Whether the Galois elements of a hoisted sum only move values inside aligned blocks of 256 positions, the tile of a
// work group of hoisted_sum_ip_local_kernel.
static bool hoisted_sum_local(const he_ctx* c, uint32_t level, const uint32_t* gs, uint32_t T) {
    if (c->logN < 8 || num_digits(c, level) > HSL_MAX_TILES) return false;
    const uint32_t mask = (1u << (c->logN - 7)) - 1;
    for (uint32_t t = 0; t < T; t++)
        if ((gs[t] & mask) != 1u) return false;
    return true;
}

// ciphertexts per launch set: the engine's limits, the kernel's register tile, and for the LDS form its digit tiles
static uint32_t hoisted_sum_jb(const he_ctx* c, uint32_t level, uint32_t J) {
    uint32_t cb, jb;
    engine_shape(c, level, J, J, cb, jb);
    jb = std::min<uint32_t>(jb, HS_JOBS);
    const uint32_t beta = num_digits(c, level);
    if (beta <= HSL_MAX_TILES) jb = std::min<uint32_t>(jb, HSL_MAX_TILES / beta);
    return jb;
}

size_t ks_hoisted_sum_ws_elems(const he_ctx* c, uint32_t level, uint32_t J, uint32_t T) {
    const size_t L1 = level + 1, k = c->np, R = L1 + k, beta = num_digits(c, level);
    (void)T;
    uint32_t cb, jb;
    engine_shape(c, level, J, J, cb, jb);
    jb = hoisted_sum_jb(c, level, J);
    // raised [jb][beta][R] + tmp_up [cb][L1] + s0 [jb][L1] + acc [jb][2][R] + tmp_dn [jb][2][k] + conv [jb][2][L1]
    return ((size_t)jb * beta * R + (size_t)cb * L1 + (size_t)jb * L1 + (size_t)jb * 2 * R + (size_t)jb * 2 * k + (size_t)jb * 2 * L1) * c->N;
}

int32_t ks_hoisted_sum(he_ctx* c, uint32_t level, const KsSrc* srcs, uint32_t J, const uint32_t* gs, const u64* const* evks, uint32_t T,
                       u64* const* out0, u64* const* out1, u64* ws) {
    const uint32_t N = c->N, L1 = level + 1, k = c->np, R = L1 + k, beta = num_digits(c, level);
    if (T == 0 || T > HE_MAX_SUM_TERMS - 1) return he_fail(c, HE_ERR_BADARG, "hoisted rotation sum: between 1 and %d terms", HE_MAX_SUM_TERMS - 1);
    for (uint32_t t = 0; t < T; t++)
        if (gs[t] == 1 || !evks[t]) return he_fail(c, HE_ERR_BADARG, "hoisted rotation sum: term %u does not rotate or has no key", t);
    if (2 * k > HE_MAX_MODULI) return he_fail(c, HE_ERR_BADARG, "key switch: more than %d special primes", HE_MAX_MODULI / 2);
    if (!hoisted_sum_local(c, level, gs, T))
        return he_fail(c, HE_ERR_BADARG, "hoisted rotation sum: a rotation is not by a multiple of N/512 slots, or more than %d digits",
                       HSL_MAX_TILES);
    uint32_t cb, jb;
    engine_shape(c, level, J, J, cb, jb);
    jb = hoisted_sum_jb(c, level, J);
    u64* raised = ws;
    u64* tmp_up = raised + (size_t)jb * beta * R * N;
    u64* s0 = tmp_up + (size_t)cb * L1 * N;
    u64* acc = s0 + (size_t)jb * L1 * N;
    u64* tmp_dn = acc + (size_t)jb * 2 * R * N;
    u64* conv = tmp_dn + (size_t)jb * 2 * k * N;
    for (uint32_t j0 = 0; j0 < J; j0 += jb) {
        const uint32_t nb = std::min(jb, J - j0);
        for (uint32_t t0 = 0; t0 < nb; t0 += cb) {
            int32_t rc = modup_batch(c, srcs + j0 + t0, std::min(cb, nb - t0), level, raised + (size_t)t0 * beta * R * N, tmp_up);
            if (rc != HE_OK) return rc;
        }
        HoistC0 hc = {};
        hc.T = std::min<uint32_t>(T, HE_MAX_KS_JOBS);
        for (uint32_t j = 0; j < nb; j++) { hc.c0[j] = srcs[j0 + j].c0; hc.s0[j] = s0 + (size_t)j * L1 * N; }
        for (uint32_t t0 = 0; t0 < T; t0 += HE_MAX_KS_JOBS) {                 // the rotated c0 parts, 16 terms per launch
            hc.T = std::min<uint32_t>(HE_MAX_KS_JOBS, T - t0);
            for (uint32_t t = 0; t < hc.T; t++) hc.g[t] = gs[t0 + t];
            for (uint32_t j = 0; j < nb; j++) hc.add[j] = t0 == 0 ? srcs[j0 + j].s0 : hc.s0[j];
            hipLaunchKernelGGL(hoist_c0_sum_kernel, dim3(N / KS_THREADS, L1, nb), dim3(KS_THREADS), 0, c->stream, hc, c->d_mc, c->logN);
            HE_HIP(c, hipGetLastError());
        }
        c->cnt.automorph += (uint64_t)nb * T * L1;
        ModDownEpilogue ep = {};
        ep.acc = acc; ep.pinv = c->d_pinv; ep.pinv_sh = c->d_pinv_sh; ep.R = R; ep.L1 = L1;
        ep.fused = 0; ep.beta = beta; ep.alpha = c->alpha; ep.M = c->M;
        for (uint32_t j = 0; j < nb; j++) {
            ep.c0[j] = nullptr; ep.g[j] = 1;
            ep.self0[j] = s0 + (size_t)j * L1 * N;
            ep.self1[j] = srcs[j0 + j].s1;
            ep.out0[j] = out0[j0 + j]; ep.out1[j] = out1[j0 + j];
        }
        // the inner products of all the chunk's ciphertexts, register-tiled, into stored accumulators
        for (uint32_t t0 = 0; t0 < T; t0 += HS_TERMS) {
            HoistIp hi = {};
            hi.J = nb; hi.T = std::min<uint32_t>(HS_TERMS, T - t0);
            for (uint32_t t = 0; t < hi.T; t++) { hi.evk[t] = evks[t0 + t]; hi.g[t] = gs[t0 + t]; }
            for (uint32_t j = 0; j < nb; j++) { hi.raised[j] = raised + (size_t)j * beta * R * N; hi.own[j] = srcs[j0 + j].c1; }
            {
                // limbs of moduli wider than 54 bits (they move carries every 6 pairs) spread evenly among the others, so
                // that both kinds are resident together
                LimbSel sel;
                {
                    uint32_t wide[HE_MAX_MODULI], narrow[HE_MAX_MODULI], nw = 0, nn = 0, iw = 0, in = 0;
                    for (uint32_t r = 0; r < R; r++) {
                        if (c->h_mc[r <= level ? r : c->nq + (r - level - 1)].bits > 54) wide[nw++] = r; else narrow[nn++] = r;
                    }
                    for (uint32_t i = 0; i < R; i++) {
                        // the i-th slot goes to a wide limb when that keeps wide limbs at nw/R of the slots so far
                        if (iw < nw && (in == nn || (uint64_t)iw * R <= (uint64_t)i * nw)) sel.r[i] = wide[iw++];
                        else sel.r[i] = narrow[in++];
                    }
                }
                const dim3 grid(N / KS_THREADS, R), blk(KS_THREADS);
                const uint32_t init = t0 == 0 ? 1u : 0u;
#define HSL_LAUNCH(JT) hipLaunchKernelGGL(hoisted_sum_ip_local_kernel<JT>, grid, blk, (size_t)nb * beta * KS_THREADS * sizeof(u64), c->stream, hi, sel, acc, c->d_mc, c->logN, R, beta, \
                                          c->M, level, c->nq, c->alpha, init)
                if (nb <= 1) HSL_LAUNCH(1); else if (nb <= 2) HSL_LAUNCH(2); else if (nb <= 4) HSL_LAUNCH(4); else HSL_LAUNCH(8);
#undef HSL_LAUNCH
            }
            HE_HIP(c, hipGetLastError());
        }
        if (c->prof_on) c->prof_key_limbs += (uint64_t)T * 2 * beta * R;
        int32_t rc = moddown_chain(c, level, nb, acc, tmp_dn, conv, nullptr, ep);
        if (rc != HE_OK) return rc;
        c->cnt.keyswitch += (uint64_t)nb * T;
    }
    return HE_OK;
}

// ---------------------------------------------------------------- products kept over the raised basis
// Building blocks of a sum of (plaintext x rotation) terms with one ModDown (the ModDown of Slide_f deferred
// across MulFilter&Sum_f of Algorithm 1): the hoisted inner products of one polynomial with n keys, stored over
// the raised basis, and the ModDown of stored accumulators with addends over the ciphertext primes.

// scratch of ks_raised_products: raised [beta][R][N] + tmp [L1][N]
size_t ks_raised_products_ws_elems(const he_ctx* c, uint32_t level) {
    const size_t L1 = level + 1, R = L1 + c->np, beta = num_digits(c, level);
    return (beta * R + L1) * c->N;
}

// acc[t] = sum_j sigma_{g_t}(ModUp(c1)_j) * evk_t,j for t < n, both components: acc [n][2][R][N], canonical.
int32_t ks_raised_products(he_ctx* c, uint32_t level, const u64* c1, const uint32_t* gs, const u64* const* evks, uint32_t n, u64* acc,
                           u64* ws) {
    const uint32_t N = c->N, L1 = level + 1, R = L1 + c->np, beta = num_digits(c, level);
    u64* raised = ws;
    u64* tmp_up = raised + (size_t)beta * R * N;
    KsSrc src = {nullptr, c1, nullptr, nullptr};
    int32_t rc = modup_batch(c, &src, 1, level, raised, tmp_up);
    if (rc != HE_OK) return rc;
    for (uint32_t t0 = 0; t0 < n; t0 += HE_MAX_KS_JOBS) {
        const uint32_t cnt = std::min<uint32_t>(HE_MAX_KS_JOBS, n - t0);
        IpBatch ib;
        for (uint32_t i = 0; i < cnt; i++) {
            ib.raised[i] = raised; ib.own[i] = c1;
            ib.evk[i] = evks[t0 + i]; ib.g[i] = gs[t0 + i]; ib.start[i] = i; ib.count[i] = 1;
        }
        rc = launch_inner_product(c, level, ib, cnt, acc + (size_t)t0 * 2 * R * N);
        if (rc != HE_OK) return rc;
        if (c->prof_on) c->prof_key_limbs += (uint64_t)cnt * 2 * beta * R;
    }
    c->cnt.keyswitch += n;
    return HE_OK;
}

// scratch of ks_moddown_stored for up to HE_MAX_KS_JOBS accumulators at once: tmp_dn [J][2][k][N] + conv [J][2][L1][N]
size_t ks_moddown_stored_ws_elems(const he_ctx* c, uint32_t level, uint32_t J) {
    const size_t nb = std::min<uint32_t>(J ? J : 1, HE_MAX_KS_JOBS);
    return nb * (2 * c->np + 2 * (level + 1)) * c->N;
}

// out_i = ( ModDown(acc_i,0) + add0_i , ModDown(acc_i,1) + add1_i ) for the J stored accumulators acc [J][2][R][N];
// add0_i / add1_i [L1][N] or null.
int32_t ks_moddown_stored(he_ctx* c, uint32_t level, uint32_t J, u64* acc, const u64* const* add0, const u64* const* add1,
                          u64* const* out0, u64* const* out1, u64* ws) {
    const uint32_t N = c->N, L1 = level + 1, k = c->np, R = L1 + k;
    if (2 * k > HE_MAX_MODULI) return he_fail(c, HE_ERR_BADARG, "key switch: more than %d special primes", HE_MAX_MODULI / 2);
    for (uint32_t j0 = 0; j0 < J; j0 += HE_MAX_KS_JOBS) {
        const uint32_t nb = std::min<uint32_t>(HE_MAX_KS_JOBS, J - j0);
        u64* a = acc + (size_t)j0 * 2 * R * N;
        u64* tmp_dn = ws;
        u64* conv = tmp_dn + (size_t)nb * 2 * k * N;
        ModDownEpilogue ep = {};
        ep.acc = a; ep.pinv = c->d_pinv; ep.pinv_sh = c->d_pinv_sh; ep.R = R; ep.L1 = L1;
        ep.fused = 0; ep.beta = num_digits(c, level); ep.alpha = c->alpha; ep.M = c->M;
        for (uint32_t i = 0; i < nb; i++) {
            ep.c0[i] = nullptr; ep.g[i] = 1;
            ep.self0[i] = add0 ? add0[j0 + i] : nullptr; ep.self1[i] = add1 ? add1[j0 + i] : nullptr;
            ep.out0[i] = out0[j0 + i]; ep.out1[i] = out1[j0 + i];
        }
        int32_t rc = moddown_chain(c, level, nb, a, tmp_dn, conv, nullptr, ep);
        if (rc != HE_OK) return rc;
    }
    return HE_OK;
}

// ---------------------------------------------------------------- rescale

// scratch for rescaling up to HE_MAX_KS_JOBS ciphertexts at once: tmp[2n][N] + delta[n][2][level][N]
size_t rescale_ws_elems(const he_ctx* c, uint32_t level, uint32_t n) {
    uint32_t nb = std::min<uint32_t>(n ? n : 1, HE_MAX_KS_JOBS);
    return (size_t)nb * (2 + 2 * level) * c->N;
}

// cts[i] [2][level+1][N] -> outs[i] [2][level][N] for i < n, batched HE_MAX_KS_JOBS at a time.
int32_t rescale_batch(he_ctx* ctx, const u64* const* cts, u64* const* outs, uint32_t n, uint32_t level, u64* ws) {
    const uint32_t N = ctx->N, L1 = level + 1;
    if (ctx->logN <= 12) return sr_rescale(ctx, cts, outs, n, level);   // limb fits LDS: one launch, no scratch
    // ciphertexts per launch set: the launch-list limit, and (for the fused last step) inputs that lie one after the other
    const uint32_t cap = std::max<uint32_t>(1, std::min<uint32_t>(HE_MAX_KS_JOBS, HE_MAX_LAUNCH_LIMBS / (2 * level)));
    for (uint32_t b0 = 0; b0 < n;) {
        uint32_t nb = 1;
        while (nb < cap && b0 + nb < n && cts[b0 + nb] == cts[b0] + (size_t)nb * 2 * L1 * N) nb++;
        u64* tmp = ws;
        u64* delta = tmp + (size_t)2 * nb * N;
        std::vector<uint32_t> mods(2 * nb, level);
        std::vector<uint8_t> seg(2 * nb);
        std::vector<uint16_t> lim(2 * nb);
        TransformDesc t = {};
        t.fwd = false; t.n_seg = nb; t.dst = tmp; t.n = 2 * nb;
        for (uint32_t i = 0; i < nb; i++) {
            t.seg[i] = cts[b0 + i];
            seg[2 * i] = seg[2 * i + 1] = (uint8_t)i;
            lim[2 * i] = (uint16_t)level; lim[2 * i + 1] = (uint16_t)(L1 + level);
        }
        t.mod_idx = mods.data(); t.src_seg = seg.data(); t.src_limb = lim.data();
        int32_t rc = launch_transform(ctx, t);
        if (rc != HE_OK) return rc;
        // forward transform of -delta whose epilogue writes (c - (-delta)) * q_l^-1: the input limb plays the stored
        // accumulator (component stride level+1 limbs), q_l^-1 mod q_r the constant of the final product.  At N = 2^16
        // the first pass forms -delta from the dropped limb's coefficients as it reads them; otherwise a kernel does.
        const uint32_t total = 2 * nb * level;
        const bool fused_delta = ctx->logN == 16;
        std::vector<uint32_t> dm(total);
        std::vector<uint16_t> dsrc(total);
        for (uint32_t i = 0; i < total; i++) { dm[i] = i % level; dsrc[i] = (uint16_t)(i / level); }
        if (!fused_delta) {
            dim3 grid(N / KS_THREADS, level, 2 * nb), block(KS_THREADS);
            hipLaunchKernelGGL(rescale_delta_kernel, grid, block, 0, ctx->stream, tmp, delta, ctx->d_mc, ctx->logN, level, 1u);
            HE_HIP(ctx, hipGetLastError());
        }
        ModDownEpilogue ep = {};
        ep.acc = cts[b0]; ep.R = L1; ep.L1 = level;
        ep.pinv = ctx->d_qlinv + (size_t)level * ctx->nq; ep.pinv_sh = ctx->d_qlinv_sh + (size_t)level * ctx->nq;
        ep.fused = 0; ep.beta = 1; ep.alpha = ctx->alpha; ep.M = ctx->M;
        for (uint32_t i = 0; i < nb; i++) {
            ep.c0[i] = nullptr; ep.self0[i] = nullptr; ep.self1[i] = nullptr; ep.g[i] = 1;
            ep.out0[i] = outs[b0 + i]; ep.out1[i] = outs[b0 + i] + (size_t)level * N;
        }
        TransformDesc f = {};
        f.fwd = true; f.seg[0] = delta; f.n_seg = 1; f.dst = delta; f.n = total; f.mod_idx = dm.data(); f.ep = &ep;
        f.lazy_out = true;
        if (fused_delta) { f.seg[0] = tmp; f.src_limb = dsrc.data(); f.rescale_from = level + 1; }
        rc = launch_transform(ctx, f);
        if (rc != HE_OK) return rc;
        ctx->cnt.rescale += nb;
        b0 += nb;
    }
    return HE_OK;
}

// ---------------------------------------------------------------- entry points

static bool overlaps(const void* a, size_t ab, const void* b, size_t bb) {
    const char *x = (const char*)a, *y = (const char*)b;
    return x < y + bb && y < x + ab;
}

static int32_t check_ks_ready(he_ctx* c, uint32_t level, const char* who) {
    if (c->np == 0) return he_fail(c, HE_ERR_BADARG, "%s: context has no special primes", who);
    if (level >= c->nq) return he_fail(c, HE_ERR_LEVEL, "%s: level %u above L=%u", who, level, c->nq - 1);
    return HE_OK;
}

extern "C" {

int32_t he_keyswitch(he_ctx* ctx, const uint64_t* d_in, uint32_t level, uint32_t galois_elt_of_key, uint64_t* d_out0,
                     uint64_t* d_out1) {
    return he_guard(ctx, "he_keyswitch: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (!d_in || !d_out0 || !d_out1) return he_fail(ctx, HE_ERR_BADARG, "he_keyswitch: null argument");
    int32_t rc = check_ks_ready(ctx, level, "he_keyswitch");
    if (rc != HE_OK) return rc;
    auto it = ctx->evk.find(galois_elt_of_key);
    if (it == ctx->evk.end()) return he_fail(ctx, HE_ERR_NOKEY, "he_keyswitch: no key registered for Galois element %u", galois_elt_of_key);
    {
        // the last kernel still reads the input while it writes the outputs
        const size_t pb = (size_t)(level + 1) * ctx->N * sizeof(u64);
        if (overlaps(d_in, pb, d_out0, pb) || overlaps(d_in, pb, d_out1, pb) || overlaps(d_out0, pb, d_out1, pb))
            return he_fail(ctx, HE_ERR_BADARG, "he_keyswitch: the outputs overlap the input or each other");
    }
    KsSrc src = {nullptr, (const u64*)d_in, nullptr, nullptr};
    KsJob job = {0, 1, it->second, (u64*)d_out0, (u64*)d_out1, 0};
    return ks_engine(ctx, level, &src, 1, &job, 1);
    });
}

int32_t he_rotate_batch(he_ctx* ctx, const uint64_t* const* h_d_ct, uint32_t n_ct, uint32_t level, const int32_t* h_steps,
                        uint32_t n_steps, uint64_t* const* h_d_out, int32_t hoisted) {
    return he_guard(ctx, "he_rotate_batch: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (n_ct == 0 || n_steps == 0) return HE_OK;
    if (!h_d_ct || !h_steps || !h_d_out) return he_fail(ctx, HE_ERR_BADARG, "he_rotate_batch: null argument");
    int32_t rc = check_ks_ready(ctx, level, "he_rotate_batch");
    if (rc != HE_OK) return rc;
    const uint32_t N = ctx->N, L1 = level + 1;
    const size_t ct_b = (size_t)2 * L1 * N * sizeof(u64);
    // validate everything before any work is enqueued
    std::vector<uint32_t> gs(n_steps);
    std::vector<const u64*> keys(n_steps, nullptr);
    for (uint32_t s = 0; s < n_steps; s++) {
        gs[s] = h_galois_of_step(ctx, h_steps[s]);
        if (gs[s] == 1) continue;
        auto it = ctx->evk.find(gs[s]);
        if (it == ctx->evk.end()) return he_fail(ctx, HE_ERR_NOKEY, "he_rotate_batch: no key for step %d (Galois element %u)", h_steps[s], gs[s]);
        keys[s] = it->second;
    }
    const size_t total = (size_t)n_ct * n_steps;
    for (uint32_t c = 0; c < n_ct; c++)
        if (!h_d_ct[c]) return he_fail(ctx, HE_ERR_BADARG, "he_rotate_batch: ciphertext %u is null", c);
    {   // no output may overlap an input or another output: sort all buffers by address and sweep
        struct Buf { const char* p; bool out; };
        std::vector<Buf> bufs;
        bufs.reserve(total + n_ct);
        for (size_t i = 0; i < total; i++) {
            if (!h_d_out[i]) return he_fail(ctx, HE_ERR_BADARG, "he_rotate_batch: output %zu is null", i);
            bufs.push_back({(const char*)h_d_out[i], true});
        }
        for (uint32_t c = 0; c < n_ct; c++) bufs.push_back({(const char*)h_d_ct[c], false});
        std::sort(bufs.begin(), bufs.end(), [](const Buf& a, const Buf& b) { return a.p < b.p; });
        for (size_t i = 1; i < bufs.size(); i++)
            if (bufs[i].p < bufs[i - 1].p + ct_b && (bufs[i].out || bufs[i - 1].out))
                return he_fail(ctx, HE_ERR_BADARG, "he_rotate_batch: an output overlaps an input or another output");
    }
    std::vector<KsSrc> srcs;
    std::vector<KsJob> jobs;
    for (uint32_t c = 0; c < n_ct; c++)
        for (uint32_t s = 0; s < n_steps; s++)
            if (gs[s] == 1)
                HE_HIP(ctx, hipMemcpyAsync((u64*)h_d_out[(size_t)c * n_steps + s], h_d_ct[c], ct_b, hipMemcpyDeviceToDevice, ctx->stream));
    if (hoisted) {
        // one source per ciphertext; the engine sorts each wave's jobs by key
        for (uint32_t c = 0; c < n_ct; c++) {
            const u64* ct = (const u64*)h_d_ct[c];
            bool have_src = false;
            for (uint32_t s = 0; s < n_steps; s++) {
                if (gs[s] == 1) continue;
                if (!have_src) { srcs.push_back({ct, ct + (size_t)L1 * N, nullptr, nullptr}); have_src = true; }
                u64* out = (u64*)h_d_out[(size_t)c * n_steps + s];
                jobs.push_back({(uint32_t)srcs.size() - 1, gs[s], keys[s], out, out + (size_t)L1 * N, 0});
            }
        }
    } else {
        // one source per rotation, step-major, so that the sources raised together use the same key
        for (uint32_t s = 0; s < n_steps; s++) {
            if (gs[s] == 1) continue;
            for (uint32_t c = 0; c < n_ct; c++) {
                const u64* ct = (const u64*)h_d_ct[c];
                u64* out = (u64*)h_d_out[(size_t)c * n_steps + s];
                srcs.push_back({ct, ct + (size_t)L1 * N, nullptr, nullptr});
                jobs.push_back({(uint32_t)srcs.size() - 1, gs[s], keys[s], out, out + (size_t)L1 * N, 0});
            }
        }
    }
    return ks_engine(ctx, level, srcs.data(), (uint32_t)srcs.size(), jobs.data(), (uint32_t)jobs.size());
    });
}

int32_t he_ws_query_rotate_batch(const he_ctx* ctx, uint32_t level, uint32_t n_ct, uint32_t n_steps, int32_t hoisted,
                                 uint64_t* h_bytes) {
    return he_guard(ctx, "he_ws_query_rotate_batch: host allocation failed", [&]() -> int32_t {
    if (!ctx || !h_bytes) return HE_ERR_BADARG;
    if (level >= ctx->nq) return HE_ERR_LEVEL;
    const uint64_t jobs = (uint64_t)n_ct * n_steps;
    if (jobs > 0xFFFFFFFFull) return HE_ERR_BADARG;
    *h_bytes = jobs == 0 ? 0 : ks_engine_ws_elems(ctx, level, hoisted ? n_ct : (uint32_t)jobs, (uint32_t)jobs) * sizeof(u64);
    return HE_OK;
    });
}

int32_t he_rotate_hoisted(he_ctx* ctx, const uint64_t* d_ct, uint32_t level, const int32_t* h_steps, uint32_t n_steps,
                          uint64_t* const* h_d_out) {
    return he_guard(ctx, "he_rotate_hoisted: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (!d_ct) return he_fail(ctx, HE_ERR_BADARG, "he_rotate_hoisted: null argument");
    const uint64_t* cts[1] = {d_ct};
    return he_rotate_batch(ctx, cts, 1, level, h_steps, n_steps, h_d_out, 1);
    });
}

int32_t he_rotate(he_ctx* ctx, const uint64_t* d_ct, uint32_t level, int32_t step, uint64_t* d_out) {
    return he_guard(ctx, "he_rotate: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (!d_ct || !d_out) return he_fail(ctx, HE_ERR_BADARG, "he_rotate: null argument");
    const uint64_t* cts[1] = {d_ct};
    uint64_t* outs[1] = {d_out};
    return he_rotate_batch(ctx, cts, 1, level, &step, 1, outs, 1);
    });
}

int32_t he_conjugate(he_ctx* ctx, const uint64_t* d_ct, uint32_t level, uint64_t* d_out) {
    return he_guard(ctx, "he_conjugate: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (!d_ct || !d_out) return he_fail(ctx, HE_ERR_BADARG, "he_conjugate: null argument");
    int32_t rc = check_ks_ready(ctx, level, "he_conjugate");
    if (rc != HE_OK) return rc;
    const uint32_t N = ctx->N, L1 = level + 1, g = 2 * N - 1;
    const size_t ct_b = (size_t)2 * L1 * N * sizeof(u64);
    if (overlaps(d_out, ct_b, d_ct, ct_b)) return he_fail(ctx, HE_ERR_BADARG, "he_conjugate: output overlaps the input");
    auto it = ctx->evk.find(g);
    if (it == ctx->evk.end()) return he_fail(ctx, HE_ERR_NOKEY, "he_conjugate: no key registered for Galois element %u", g);
    const u64* ct = (const u64*)d_ct;
    KsSrc src = {ct, ct + (size_t)L1 * N, nullptr, nullptr};
    KsJob job = {0, g, it->second, (u64*)d_out, (u64*)d_out + (size_t)L1 * N, 0};
    return ks_engine(ctx, level, &src, 1, &job, 1);
    });
}

int32_t he_mulct(he_ctx* ctx, const uint64_t* d_a, const uint64_t* d_b, uint32_t level, uint64_t* d_out) {
    return he_guard(ctx, "he_mulct: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (!d_a || !d_b || !d_out) return he_fail(ctx, HE_ERR_BADARG, "he_mulct: null argument");
    int32_t rc = check_ks_ready(ctx, level, "he_mulct");
    if (rc != HE_OK) return rc;
    auto it = ctx->evk.find(0);
    if (it == ctx->evk.end()) return he_fail(ctx, HE_ERR_NOKEY, "he_mulct: no relinearisation key registered (Galois element 0)");
    const uint32_t N = ctx->N, L1 = level + 1;
    const size_t pe = (size_t)L1 * N, ks_e = ks_engine_ws_elems(ctx, level, 1, 1);
    rc = he_ensure_ws(ctx, (ks_e + 3 * pe) * sizeof(u64));
    if (rc != HE_OK) return rc;
    u64* d = ctx->d_ws + ks_e;      // d0, d1, d2 behind the engine's region
    rc = launch_tensor(ctx, (const u64*)d_a, (const u64*)d_b, level, d);
    if (rc != HE_OK) return rc;
    KsSrc src = {nullptr, d + 2 * pe, d, d + pe};
    KsJob job = {0, 1, it->second, (u64*)d_out, (u64*)d_out + pe, 1};
    return ks_engine(ctx, level, &src, 1, &job, 1);
    });
}

int32_t he_rescale(he_ctx* ctx, const uint64_t* d_ct, uint32_t level, uint64_t* d_out) {
    return he_guard(ctx, "he_rescale: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (!d_ct || !d_out) return he_fail(ctx, HE_ERR_BADARG, "he_rescale: null argument");
    if (level == 0 || level >= ctx->nq) return he_fail(ctx, HE_ERR_LEVEL, "he_rescale: level %u outside 1..%u", level, ctx->nq - 1);
    const size_t N = ctx->N;
    if (overlaps(d_out, 2 * level * N * sizeof(u64), d_ct, 2 * (level + 1) * N * sizeof(u64)))
        return he_fail(ctx, HE_ERR_BADARG, "he_rescale: output overlaps the input");
    int32_t rc = he_ensure_ws(ctx, rescale_ws_elems(ctx, level, 1) * sizeof(u64));
    if (rc != HE_OK) return rc;
    const u64* cts[1] = {(const u64*)d_ct};
    u64* outs[1] = {(u64*)d_out};
    return rescale_batch(ctx, cts, outs, 1, level, ctx->d_ws);
    });
}

} // extern "C"
