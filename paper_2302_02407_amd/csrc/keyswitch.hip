// Hybrid key switching with dnum digits (the inner step of CRot; paper Section 2.1 for CRot,
// Appendix for evaluation keys and dnum), hoisted rotations, and rescale.
//
//   ModUp   : digit limbs -> coefficient form (iNTT with the factor (Q_j/q_i)^-1 folded into
//             the N^-1 scaling) -> fast basis conversion to every other limb of
//             {q_0..q_l, p_*} (128-bit accumulation, one Barrett step) -> NTT.
//   inner   : acc_c[r] = sum_j sigma_g(raised_j)[r] * evk_j,c[r]   (sigma_g as a gather).
//   ModDown : p-limbs -> coefficient form (iNTT with (P/p_t)^-1 folded in) -> conversion to
//             q_0..q_l -> NTT -> (acc - conv) * P^-1 (+ sigma_g(c0) for a rotation).
// Neither conversion corrects the overflow multiple; each term is a canonical residue and
// the sum is reduced exactly, so results are defined bit for bit.
#include "modarith.cuh"

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
struct ConvBatch {
    ConvJob job[CONV_MAX_JOBS];
};

// Fast basis conversion.  grid: (N/512, ceil(nt_max/CONV_TGT_PER_BLOCK), jobs); each thread owns two
// adjacent coefficients (16-byte loads and stores).  The block's conversion constants and target
// moduli are staged in LDS once and then read as broadcasts.  With at most 8 source limbs
// (ONE_CHUNK) the pre-scaled sources stay in registers across all targets of the block.
template <bool ONE_CHUNK>
__global__ __launch_bounds__(KS_THREADS) void baseconv_kernel(ConvBatch b, const ModConst* mc, uint32_t logN) {
    __shared__ u64 s_hat[CONV_TGT_PER_BLOCK * 64];
    __shared__ u64 s_q[CONV_TGT_PER_BLOCK], s_mu[CONV_TGT_PER_BLOCK];
    __shared__ uint32_t s_bits[CONV_TGT_PER_BLOCK];
    const ConvJob& job = b.job[blockIdx.z];
    const uint32_t t0 = blockIdx.y * CONV_TGT_PER_BLOCK;
    if (t0 >= job.nt) return;
    const uint32_t nt = min((uint32_t)CONV_TGT_PER_BLOCK, job.nt - t0);
    const uint32_t ns = job.ns, w = job.hat_w;
    for (uint32_t idx = threadIdx.x; idx < nt * w; idx += KS_THREADS) {
        uint32_t tt = idx / w, i = idx - tt * w;
        s_hat[tt * 64 + i] = job.hat[(size_t)job.tgt_mod[t0 + tt] * w + i];
    }
    if (threadIdx.x < nt) {
        const ModConst m = mc[job.tgt_mod[t0 + threadIdx.x]];
        s_q[threadIdx.x] = m.q; s_mu[threadIdx.x] = m.mu; s_bits[threadIdx.x] = m.bits;
    }
    __syncthreads();
    const size_t n = (size_t)(blockIdx.x * KS_THREADS + threadIdx.x) * 2;
    if (n >= ((size_t)1 << logN)) return;      // rings smaller than one block of coefficient pairs
    ulonglong2 y[8];
    if (ONE_CHUNK) {
#pragma unroll
        for (uint32_t i = 0; i < 8; i++)
            y[i] = i < ns ? *reinterpret_cast<const ulonglong2*>(job.src + ((size_t)i << logN) + n) : make_ulonglong2(0, 0);
    }
    for (uint32_t tt = 0; tt < nt; tt++) {
        const u64 q = s_q[tt], mu = s_mu[tt];
        const uint32_t bits = s_bits[tt];
        const u64* h = s_hat + tt * 64;
        u128 a0 = 0, a1 = 0;
        if (ONE_CHUNK) {
#pragma unroll
            for (uint32_t i = 0; i < 8; i++) {
                a0 += (u128)y[i].x * h[i];
                a1 += (u128)y[i].y * h[i];
            }
        } else {
            for (uint32_t i0 = 0; i0 < ns; i0 += 8) {
                if (i0) { a0 = barrett128(a0, q, mu, bits); a1 = barrett128(a1, q, mu, bits); }
                for (uint32_t i = i0; i < min(i0 + 8, ns); i++) {
                    ulonglong2 v = *reinterpret_cast<const ulonglong2*>(job.src + ((size_t)i << logN) + n);
                    a0 += (u128)v.x * h[i];
                    a1 += (u128)v.y * h[i];
                }
            }
        }
        ulonglong2 o = make_ulonglong2(barrett128(a0, q, mu, bits), barrett128(a1, q, mu, bits));
        *reinterpret_cast<ulonglong2*>(job.dst + ((size_t)job.tgt_limb[t0 + tt] << logN) + n) = o;
    }
}

// grid: (N/256, R).  raised [beta][R][N]; evk [dnum][2][M][N]; acc [2][R][N].  A digit's own limbs
// (limb r of digit r/alpha) are never materialised in `raised`: they are read from the input
// polynomial `own` [level+1][N], which is what ModUp would have copied.
__global__ __launch_bounds__(KS_THREADS) void inner_product_kernel(const u64* __restrict__ raised, const u64* __restrict__ own,
                                                                   const u64* __restrict__ evk, u64* __restrict__ acc,
                                                                   const ModConst* mc, uint32_t logN, uint32_t R, uint32_t beta,
                                                                   uint32_t M, uint32_t level, uint32_t nq, uint32_t alpha,
                                                                   uint32_t g) {
    const uint32_t n = blockIdx.x * KS_THREADS + threadIdx.x;
    const uint32_t r = blockIdx.y;
    const uint32_t mi = r <= level ? r : nq + (r - level - 1);
    const ModConst m = mc[mi];
    const uint32_t src = g == 1 ? n : galois_src_ks(n, g, logN);
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
    acc[((size_t)r << logN) + n] = barrett128(a0, m.q, m.mu, m.bits);
    acc[((size_t)(R + r) << logN) + n] = barrett128(a1, m.q, m.mu, m.bits);
}

// grid: (N/256, level+1, 2).  out_c[r] = (acc_c[r] - conv_c[r]) * P^-1 (+ sigma_g(c0)[r] for c = 0).
__global__ __launch_bounds__(KS_THREADS) void moddown_final_kernel(const u64* __restrict__ acc, const u64* __restrict__ conv,
                                                                   const u64* __restrict__ c0, u64* __restrict__ out0,
                                                                   u64* __restrict__ out1, const ModConst* mc,
                                                                   const u64* pinv, const u64* pinv_sh, uint32_t logN,
                                                                   uint32_t R, uint32_t L1, uint32_t g) {
    const uint32_t n = blockIdx.x * KS_THREADS + threadIdx.x;
    const uint32_t r = blockIdx.y, comp = blockIdx.z;
    const u64 q = mc[r].q;
    u64 a = acc[((size_t)(comp * R + r) << logN) + n];
    u64 c = conv[((size_t)(comp * L1 + r) << logN) + n];
    u64 v = shoup_mul(submod(a, c, q), pinv[r], pinv_sh[r], q);
    if (comp == 0 && c0) v = addmod(v, c0[((size_t)r << logN) + (g == 1 ? n : galois_src_ks(n, g, logN))], q);
    (comp ? out1 : out0)[((size_t)r << logN) + n] = v;
}

// ---------------------------------------------------------------- rescale kernels
// grid: (N/256, level, 2).  t = coefficient-form limb `level` of component comp (tmp[comp][N]);
// delta[comp][r] = (h mod q_r) - ((t + h mod q_l) mod q_r), h = floor(q_l/2).
__global__ __launch_bounds__(KS_THREADS) void rescale_delta_kernel(const u64* __restrict__ tmp, u64* __restrict__ delta,
                                                                   const ModConst* mc, uint32_t logN, uint32_t level) {
    const uint32_t n = blockIdx.x * KS_THREADS + threadIdx.x;
    const uint32_t r = blockIdx.y, comp = blockIdx.z;
    const ModConst ml = mc[level], mr = mc[r];
    u64 h = ml.q >> 1;
    u64 t = addmod(tmp[((size_t)comp << logN) + n], h, ml.q);
    u64 tr = barrett64(t, mr.q, mr.mu, mr.bits);
    u64 hr = barrett64(h, mr.q, mr.mu, mr.bits);
    delta[((size_t)(comp * level + r) << logN) + n] = submod(hr, tr, mr.q);
}

// grid: (N/256, level, 2).  out[comp][r] = (ct[comp][r] + delta[comp][r]) * q_l^-1 mod q_r.
__global__ __launch_bounds__(KS_THREADS) void rescale_final_kernel(const u64* __restrict__ ct, const u64* __restrict__ delta,
                                                                   u64* __restrict__ out, const ModConst* mc,
                                                                   const u64* qlinv, const u64* qlinv_sh, uint32_t logN,
                                                                   uint32_t level) {
    const uint32_t n = blockIdx.x * KS_THREADS + threadIdx.x;
    const uint32_t r = blockIdx.y, comp = blockIdx.z;
    const u64 q = mc[r].q;
    u64 a = ct[((size_t)(comp * (level + 1) + r) << logN) + n];
    u64 d = delta[((size_t)(comp * level + r) << logN) + n];
    out[((size_t)(comp * level + r) << logN) + n] = shoup_mul(addmod(a, d, q), qlinv[r], qlinv_sh[r], q);
}

// ---------------------------------------------------------------- host: tables

static uint32_t num_digits(const he_ctx* c, uint32_t level) { return (level + c->alpha) / c->alpha; }
static uint32_t pad8(uint32_t x) { return (x + 7u) & ~7u; }

size_t ks_raised_elems(const he_ctx* c, uint32_t level) {
    return (size_t)num_digits(c, level) * (level + 1 + c->np) * c->N;
}
// tmp_up[level+1] + acc[2][R] + tmp_dn[2][k] + conv[2][level+1]
size_t ks_scratch_elems(const he_ctx* c, uint32_t level) {
    size_t L1 = level + 1, R = L1 + c->np;
    return (L1 + 2 * R + 2 * c->np + 2 * L1) * c->N;
}

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

// ---------------------------------------------------------------- host: ModUp / ModDown

static int32_t launch_baseconv(he_ctx* c, const ConvBatch& b, uint32_t jobs, uint32_t nt_max, uint32_t ns_max) {
    dim3 grid((c->N + 2 * KS_THREADS - 1) / (2 * KS_THREADS), (nt_max + CONV_TGT_PER_BLOCK - 1) / CONV_TGT_PER_BLOCK, jobs), block(KS_THREADS);
    if (ns_max <= 8) hipLaunchKernelGGL(baseconv_kernel<true>, grid, block, 0, c->stream, b, c->d_mc, c->logN);
    else hipLaunchKernelGGL(baseconv_kernel<false>, grid, block, 0, c->stream, b, c->d_mc, c->logN);
    HE_HIP(c, hipGetLastError());
    return HE_OK;
}

// d_poly [level+1][N] NTT form -> d_raised [beta][R][N] NTT form, EXCEPT each digit's own limbs,
// which are left unwritten (the inner product reads them from d_poly).  d_tmp: level+1 limbs.
int32_t modup_impl(he_ctx* c, const u64* d_poly, uint32_t level, u64* d_raised, u64* d_tmp) {
    const uint32_t N = c->N, L1 = level + 1, R = L1 + c->np, beta = num_digits(c, level), al = c->alpha;
    // coefficient form of all limbs, each pre-multiplied by N^-1 * (Q_j/q_i)^-1
    ScaleList sc;
    uint32_t idx[HE_MAX_MODULI];
    uint16_t from[HE_MAX_MODULI];
    for (uint32_t i = 0; i < L1; i++) {
        uint32_t j = i / al, lo = j * al, hi = (j + 1) * al < L1 ? (j + 1) * al : L1, sz = hi - lo;
        u64 qi = c->mod[i];
        u64 s = h_mulmod(c->h_mc[i].ninv, c->h_up_invhat[(size_t)(j * al + (sz - 1)) * al + (i - lo)], qi);
        sc.s[i] = s;
        sc.s_sh[i] = h_shoup(s, qi);
        idx[i] = i;
        from[i] = (uint16_t)i;
    }
    int32_t rc = launch_intt_from(c, d_poly, from, d_tmp, idx, L1, &sc);
    if (rc != HE_OK) return rc;
    const uint32_t aw = pad8(al);
    for (uint32_t j0 = 0; j0 < beta; j0 += CONV_MAX_JOBS) {
        ConvBatch b;
        uint32_t jobs = beta - j0 < CONV_MAX_JOBS ? beta - j0 : CONV_MAX_JOBS, nt_max = 0, ns_max = 0;
        for (uint32_t jj = 0; jj < jobs; jj++) {
            uint32_t j = j0 + jj, lo = j * al, hi = (j + 1) * al < L1 ? (j + 1) * al : L1, sz = hi - lo;
            ConvJob& job = b.job[jj];
            job.src = d_tmp + (size_t)lo * N;
            job.dst = d_raised + (size_t)j * R * N;
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
        rc = launch_baseconv(c, b, jobs, nt_max, ns_max);
        if (rc != HE_OK) return rc;
    }
    // NTT of every converted limb; own limbs are marked "skip"
    uint32_t total = beta * R;
    std::vector<uint32_t> mods(total);
    for (uint32_t j = 0; j < beta; j++) {
        uint32_t lo = j * al, hi = (j + 1) * al < L1 ? (j + 1) * al : L1;
        for (uint32_t r = 0; r < R; r++)
            mods[j * R + r] = (r >= lo && r < hi) ? 0xFFu : (r <= level ? r : c->nq + (r - level - 1));
    }
    for (uint32_t o = 0; o < total; o += HE_MAX_LAUNCH_LIMBS) {
        uint32_t n = total - o < HE_MAX_LAUNCH_LIMBS ? total - o : HE_MAX_LAUNCH_LIMBS;
        rc = launch_ntt(c, d_raised + (size_t)o * N, mods.data() + o, n);
        if (rc != HE_OK) return rc;
    }
    c->cnt.modup += 1;
    return HE_OK;
}

// raised [beta][R][N] (own limbs taken from d_own [level+1][N]) -> (out0, out1) [level+1][N].
// g_perm: Galois element applied to the raised digits (and to c0 if given) as a gather; 1 = none.
// d_scratch: ks_scratch_elems.
int32_t ks_inner_moddown(he_ctx* c, const u64* d_raised, const u64* d_own, uint32_t level, uint32_t g_perm, const u64* d_evk,
                         const u64* d_c0, u64* d_out0, u64* d_out1, u64* d_scratch) {
    const uint32_t N = c->N, L1 = level + 1, k = c->np, R = L1 + k, beta = num_digits(c, level);
    u64* acc = d_scratch + (size_t)L1 * N;       // after tmp_up
    u64* tmp_dn = acc + (size_t)2 * R * N;       // [2][k][N]
    u64* conv = tmp_dn + (size_t)2 * k * N;      // [2][L1][N]
    {
        dim3 grid(N / KS_THREADS, R), block(KS_THREADS);
        hipLaunchKernelGGL(inner_product_kernel, grid, block, 0, c->stream, d_raised, d_own, d_evk, acc, c->d_mc, c->logN, R,
                           beta, c->M, level, c->nq, c->alpha, g_perm);
        HE_HIP(c, hipGetLastError());
    }
    // p-limbs of both accumulators -> coefficient form, pre-multiplied by N^-1 * (P/p_t)^-1
    if (2 * k > HE_MAX_MODULI) return he_fail(c, HE_ERR_BADARG, "key switch: more than %d special primes", HE_MAX_MODULI / 2);
    ScaleList sc;
    uint32_t idx[HE_MAX_MODULI];
    uint16_t from[HE_MAX_MODULI];
    for (uint32_t i = 0; i < 2 * k; i++) {
        uint32_t t = i % k;
        from[i] = (uint16_t)((i / k) * R + L1 + t);
        u64 p = c->mod[c->nq + t];
        u64 s = h_mulmod(c->h_mc[c->nq + t].ninv, c->h_dn_invhat[t], p);
        sc.s[i] = s;
        sc.s_sh[i] = h_shoup(s, p);
        idx[i] = c->nq + t;
    }
    int32_t rc = launch_intt_from(c, acc, from, tmp_dn, idx, 2 * k, &sc);
    if (rc != HE_OK) return rc;
    ConvBatch b;
    for (uint32_t comp = 0; comp < 2; comp++) {
        ConvJob& job = b.job[comp];
        job.src = tmp_dn + (size_t)comp * k * N;
        job.dst = conv + (size_t)comp * L1 * N;
        job.hat = c->d_dn_hat;
        job.hat_w = pad8(k);
        job.ns = k;
        job.nt = L1;
        for (uint32_t r = 0; r < L1; r++) { job.tgt_limb[r] = (uint8_t)r; job.tgt_mod[r] = (uint8_t)r; }
    }
    rc = launch_baseconv(c, b, 2, L1, k);
    if (rc != HE_OK) return rc;
    std::vector<uint32_t> mods(2 * L1);
    for (uint32_t i = 0; i < 2 * L1; i++) mods[i] = i % L1;
    if (c->logN == 16 && 2 * L1 <= HE_MAX_LAUNCH_LIMBS) {
        // the last NTT pass applies (acc - conv) * P^-1 (+ sigma_g(c0)) and writes the outputs itself
        ModDownEpilogue ep;
        ep.acc = acc; ep.c0 = d_c0; ep.out0 = d_out0; ep.out1 = d_out1;
        ep.pinv = c->d_pinv; ep.pinv_sh = c->d_pinv_sh; ep.R = R; ep.L1 = L1; ep.g = g_perm;
        rc = launch_ntt16_moddown(c, conv, mods.data(), 2 * L1, ep);
        if (rc != HE_OK) return rc;
    } else {
        rc = launch_ntt(c, conv, mods.data(), 2 * L1);
        if (rc != HE_OK) return rc;
        dim3 grid(N / KS_THREADS, L1, 2), block(KS_THREADS);
        hipLaunchKernelGGL(moddown_final_kernel, grid, block, 0, c->stream, acc, conv, d_c0, d_out0, d_out1, c->d_mc, c->d_pinv,
                           c->d_pinv_sh, c->logN, R, L1, g_perm);
        HE_HIP(c, hipGetLastError());
    }
    c->cnt.keyswitch += 1;
    if (d_c0) c->cnt.automorph += L1;
    return HE_OK;
}

static bool overlaps(const void* a, size_t ab, const void* b, size_t bb) {
    const char *x = (const char*)a, *y = (const char*)b;
    return x < y + bb && y < x + ab;
}

static int32_t check_ks_ready(he_ctx* c, uint32_t level, const char* who) {
    if (c->np == 0) return he_fail(c, HE_ERR_BADARG, "%s: context has no special primes", who);
    if (level >= c->nq) return he_fail(c, HE_ERR_LEVEL, "%s: level %u above L=%u", who, level, c->nq - 1);
    return he_ensure_ws(c, (ks_raised_elems(c, level) + ks_scratch_elems(c, level)) * sizeof(u64));
}

size_t rescale_ws_elems(const he_ctx* c, uint32_t level) { return (size_t)(2 + 2 * level) * c->N; }

// ct [2][level+1][N] -> out [2][level][N]; ws: tmp[2][N] + delta[2][level][N]
int32_t rescale_impl(he_ctx* ctx, const u64* d_ct, uint32_t level, u64* d_out, u64* ws) {
    const uint32_t N = ctx->N, L1 = level + 1;
    u64* tmp = ws;
    u64* delta = tmp + (size_t)2 * N;
    uint32_t two[2] = {level, level};
    uint16_t from[2] = {(uint16_t)level, (uint16_t)(L1 + level)};
    int32_t rc = launch_intt_from(ctx, d_ct, from, tmp, two, 2, nullptr);
    if (rc != HE_OK) return rc;
    dim3 grid(N / KS_THREADS, level, 2), block(KS_THREADS);
    hipLaunchKernelGGL(rescale_delta_kernel, grid, block, 0, ctx->stream, tmp, delta, ctx->d_mc, ctx->logN, level);
    HE_HIP(ctx, hipGetLastError());
    std::vector<uint32_t> mods(2 * level);
    for (uint32_t i = 0; i < 2 * level; i++) mods[i] = i % level;
    for (uint32_t o = 0; o < 2 * level; o += HE_MAX_LAUNCH_LIMBS) {
        uint32_t n = 2 * level - o < HE_MAX_LAUNCH_LIMBS ? 2 * level - o : HE_MAX_LAUNCH_LIMBS;
        rc = launch_ntt(ctx, delta + (size_t)o * N, mods.data() + o, n);
        if (rc != HE_OK) return rc;
    }
    hipLaunchKernelGGL(rescale_final_kernel, grid, block, 0, ctx->stream, d_ct, delta, d_out, ctx->d_mc,
                       ctx->d_qlinv + (size_t)level * ctx->nq, ctx->d_qlinv_sh + (size_t)level * ctx->nq, ctx->logN, level);
    HE_HIP(ctx, hipGetLastError());
    ctx->cnt.rescale += 1;
    return HE_OK;
}

extern "C" {

int32_t he_keyswitch(he_ctx* ctx, const uint64_t* d_in, uint32_t level, uint32_t galois_elt_of_key, uint64_t* d_out0,
                     uint64_t* d_out1) {
    if (!ctx) return HE_ERR_BADARG;
    if (!d_in || !d_out0 || !d_out1) return he_fail(ctx, HE_ERR_BADARG, "he_keyswitch: null argument");
    int32_t rc = check_ks_ready(ctx, level, "he_keyswitch");
    if (rc != HE_OK) return rc;
    auto it = ctx->evk.find(galois_elt_of_key);
    if (it == ctx->evk.end()) return he_fail(ctx, HE_ERR_NOKEY, "he_keyswitch: no key registered for Galois element %u", galois_elt_of_key);
    u64* raised = ctx->d_ws;
    u64* scratch = raised + ks_raised_elems(ctx, level);
    rc = modup_impl(ctx, (const u64*)d_in, level, raised, scratch);
    if (rc != HE_OK) return rc;
    return ks_inner_moddown(ctx, raised, (const u64*)d_in, level, 1, it->second, nullptr, (u64*)d_out0, (u64*)d_out1, scratch);
}

int32_t he_rotate_hoisted(he_ctx* ctx, const uint64_t* d_ct, uint32_t level, const int32_t* h_steps, uint32_t n_steps,
                          uint64_t* const* h_d_out) {
    if (!ctx) return HE_ERR_BADARG;
    if (!d_ct || (n_steps && (!h_steps || !h_d_out))) return he_fail(ctx, HE_ERR_BADARG, "he_rotate_hoisted: null argument");
    int32_t rc = check_ks_ready(ctx, level, "he_rotate_hoisted");
    if (rc != HE_OK) return rc;
    const uint32_t N = ctx->N, L1 = level + 1;
    const size_t ct_b = (size_t)2 * L1 * N * sizeof(u64);
    // validate everything before any work is enqueued
    std::vector<uint32_t> gs(n_steps);
    std::vector<const u64*> keys(n_steps, nullptr);
    bool any_ks = false;
    for (uint32_t i = 0; i < n_steps; i++) {
        if (!h_d_out[i]) return he_fail(ctx, HE_ERR_BADARG, "he_rotate_hoisted: output %u is null", i);
        if (overlaps(h_d_out[i], ct_b, d_ct, ct_b)) return he_fail(ctx, HE_ERR_BADARG, "he_rotate_hoisted: output %u overlaps the input", i);
        for (uint32_t k = 0; k < i; k++)
            if (overlaps(h_d_out[i], ct_b, h_d_out[k], ct_b)) return he_fail(ctx, HE_ERR_BADARG, "he_rotate_hoisted: outputs %u and %u overlap", k, i);
        gs[i] = h_galois_of_step(ctx, h_steps[i]);
        if (gs[i] == 1) continue;
        auto it = ctx->evk.find(gs[i]);
        if (it == ctx->evk.end()) return he_fail(ctx, HE_ERR_NOKEY, "he_rotate_hoisted: no key for step %d (Galois element %u)", h_steps[i], gs[i]);
        keys[i] = it->second;
        any_ks = true;
    }
    u64* raised = ctx->d_ws;
    u64* scratch = raised + ks_raised_elems(ctx, level);
    if (any_ks) {
        rc = modup_impl(ctx, (const u64*)d_ct + (size_t)L1 * N, level, raised, scratch);
        if (rc != HE_OK) return rc;
    }
    for (uint32_t i = 0; i < n_steps; i++) {
        u64* out = (u64*)h_d_out[i];
        if (gs[i] == 1) {
            HE_HIP(ctx, hipMemcpyAsync(out, d_ct, ct_b, hipMemcpyDeviceToDevice, ctx->stream));
            continue;
        }
        rc = ks_inner_moddown(ctx, raised, (const u64*)d_ct + (size_t)L1 * N, level, gs[i], keys[i], (const u64*)d_ct, out, out + (size_t)L1 * N, scratch);
        if (rc != HE_OK) return rc;
    }
    return HE_OK;
}

int32_t he_rotate(he_ctx* ctx, const uint64_t* d_ct, uint32_t level, int32_t step, uint64_t* d_out) {
    uint64_t* outs[1] = {d_out};
    return he_rotate_hoisted(ctx, d_ct, level, &step, 1, outs);
}

int32_t he_conjugate(he_ctx* ctx, const uint64_t* d_ct, uint32_t level, uint64_t* d_out) {
    if (!ctx) return HE_ERR_BADARG;
    if (!d_ct || !d_out) return he_fail(ctx, HE_ERR_BADARG, "he_conjugate: null argument");
    int32_t rc = check_ks_ready(ctx, level, "he_conjugate");
    if (rc != HE_OK) return rc;
    const uint32_t N = ctx->N, L1 = level + 1, g = 2 * N - 1;
    const size_t ct_b = (size_t)2 * L1 * N * sizeof(u64);
    if (overlaps(d_out, ct_b, d_ct, ct_b)) return he_fail(ctx, HE_ERR_BADARG, "he_conjugate: output overlaps the input");
    auto it = ctx->evk.find(g);
    if (it == ctx->evk.end()) return he_fail(ctx, HE_ERR_NOKEY, "he_conjugate: no key registered for Galois element %u", g);
    u64* raised = ctx->d_ws;
    u64* scratch = raised + ks_raised_elems(ctx, level);
    rc = modup_impl(ctx, (const u64*)d_ct + (size_t)L1 * N, level, raised, scratch);
    if (rc != HE_OK) return rc;
    return ks_inner_moddown(ctx, raised, (const u64*)d_ct + (size_t)L1 * N, level, g, it->second, (const u64*)d_ct, (u64*)d_out, (u64*)d_out + (size_t)L1 * N, scratch);
}

int32_t he_rescale(he_ctx* ctx, const uint64_t* d_ct, uint32_t level, uint64_t* d_out) {
    if (!ctx) return HE_ERR_BADARG;
    if (!d_ct || !d_out) return he_fail(ctx, HE_ERR_BADARG, "he_rescale: null argument");
    if (level == 0 || level >= ctx->nq) return he_fail(ctx, HE_ERR_LEVEL, "he_rescale: level %u outside 1..%u", level, ctx->nq - 1);
    const size_t N = ctx->N;
    if (overlaps(d_out, 2 * level * N * sizeof(u64), d_ct, 2 * (level + 1) * N * sizeof(u64)))
        return he_fail(ctx, HE_ERR_BADARG, "he_rescale: output overlaps the input");
    int32_t rc = he_ensure_ws(ctx, rescale_ws_elems(ctx, level) * sizeof(u64));
    if (rc != HE_OK) return rc;
    return rescale_impl(ctx, (const u64*)d_ct, level, (u64*)d_out, ctx->d_ws);
}

} // extern "C"
