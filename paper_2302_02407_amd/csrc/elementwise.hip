// Coefficient-wise kernels: Galois permutation, MulPt-accumulate, AddCt, and their entry points.
#include <algorithm>

#include "modarith.h"

#define EW_THREADS 256

// Source position of output position j under sigma_g on NTT-form limbs: position j holds the
// evaluation at psi^(2k+1), k = bitrev(j); sigma_g(a) there equals a at exponent
// (2k+1)*g mod 2N, i.e. natural index k' = g*k + (g-1)/2 mod N, stored at bitrev(k').
// Aligned blocks of positions map to aligned blocks, so a wave's 64 loads stay inside one
// 512-byte span.
__device__ __forceinline__ uint32_t galois_src(uint32_t j, uint32_t g, uint32_t logN) {
    uint32_t k = __brev(j) >> (32 - logN);
    uint32_t kp = (g * k + ((g - 1) >> 1)) & ((1u << logN) - 1);
    return __brev(kp) >> (32 - logN);
}

__global__ __launch_bounds__(EW_THREADS) void automorph_ntt_kernel(const u64* __restrict__ in, u64* __restrict__ out,
                                                                   uint32_t logN, uint32_t g) {
    uint32_t j = blockIdx.x * EW_THREADS + threadIdx.x;
    size_t limb = blockIdx.y;
    out[(limb << logN) + j] = in[(limb << logN) + galois_src(j, g, logN)];
}

// Coefficient form: out[t] = +-in[i] with i*g = t (mod 2N) up to the sign from X^N = -1.
__global__ __launch_bounds__(EW_THREADS) void automorph_coef_kernel(const u64* __restrict__ in, u64* __restrict__ out,
                                                                    const ModConst* mc, LimbList ll, uint32_t logN,
                                                                    uint32_t ginv) {
    uint32_t t = blockIdx.x * EW_THREADS + threadIdx.x;
    size_t limb = blockIdx.y;
    u64 q = mc[ll.mod[limb]].q;
    uint32_t N = 1u << logN;
    uint32_t u = (uint32_t)(((u64)t * ginv) & (2ull * N - 1));
    u64 v = in[(limb << logN) + (u & (N - 1))];
    if (u >= N) v = v ? q - v : 0;
    out[(limb << logN) + t] = v;
}

// acc (+)= ct * pt on both components; limb index = blockIdx.y in [0, level+1).
__global__ __launch_bounds__(EW_THREADS) void ptct_mac_kernel(u64* __restrict__ acc, const u64* __restrict__ ct,
                                                              const u64* __restrict__ pt, const ModConst* mc,
                                                              uint32_t logN, uint32_t n_limbs, int init) {
    uint32_t n = blockIdx.x * EW_THREADS + threadIdx.x;
    uint32_t limb = blockIdx.y;
    const ModConst m = mc[limb];
    size_t o0 = ((size_t)limb << logN) + n, o1 = ((size_t)(limb + n_limbs) << logN) + n;
    u64 p = pt[o0];
    u64 r0 = mulmod(ct[o0], p, m), r1 = mulmod(ct[o1], p, m);
    if (!init) {
        r0 = addmod(r0, acc[o0], m.q);
        r1 = addmod(r1, acc[o1], m.q);
    }
    acc[o0] = r0;
    acc[o1] = r1;
}

// acc (+)= sum_i ct_i * sigma_{g_i}(pt_i): the plaintext is permuted as it is read (a plaintext rotation fused into
// the product), products summed in 128 bits and reduced once per 8 terms.  limb = blockIdx.y.
#define MACROT_MAX 16
struct MacRot {
    const u64* ct[MACROT_MAX];   // [2][n_limbs][N]
    const u64* pt[MACROT_MAX];   // [n_limbs][N]
    uint32_t g[MACROT_MAX];
    uint32_t n;
};
__global__ __launch_bounds__(EW_THREADS) void ptct_mac_rot_kernel(u64* __restrict__ acc, MacRot mr, const ModConst* mc, uint32_t logN,
                                                                  uint32_t n_limbs, int init) {
    const uint32_t n = blockIdx.x * EW_THREADS + threadIdx.x;
    const uint32_t limb = blockIdx.y;
    const ModConst m = mc[limb];
    const size_t o0 = ((size_t)limb << logN) + n, o1 = ((size_t)(limb + n_limbs) << logN) + n;
    u128 a0 = init ? 0 : acc[o0], a1 = init ? 0 : acc[o1];
    for (uint32_t i = 0; i < mr.n; i++) {
        if (i && (i & 7) == 0) {
            a0 = barrett128(a0, m.q, m.mu, m.bits);
            a1 = barrett128(a1, m.q, m.mu, m.bits);
        }
        const uint32_t g = mr.g[i];
        const u64 p = mr.pt[i][((size_t)limb << logN) + (g == 1 ? n : galois_src(n, g, logN))];
        a0 += (u128)mr.ct[i][o0] * p;
        a1 += (u128)mr.ct[i][o1] * p;
    }
    acc[o0] = barrett128(a0, m.q, m.mu, m.bits);
    acc[o1] = barrett128(a1, m.q, m.mu, m.bits);
}

__global__ __launch_bounds__(EW_THREADS) void add_kernel(const u64* a, const u64* b, u64* out, const ModConst* mc,
                                                         uint32_t logN, uint32_t n_limbs) {
    uint32_t n = blockIdx.x * EW_THREADS + threadIdx.x;
    uint32_t limb = blockIdx.y % n_limbs;
    u64 q = mc[limb].q;
    size_t o = ((size_t)blockIdx.y << logN) + n;
    out[o] = addmod(a[o], b[o], q);
}

// AddPt: out.c0 = ct.c0 + pt, out.c1 = ct.c1.  grid: (N/256, 2*(level+1)).
__global__ __launch_bounds__(EW_THREADS) void addpt_kernel(const u64* ct, const u64* __restrict__ pt, u64* out, const ModConst* mc,
                                                           uint32_t logN, uint32_t n_limbs) {
    uint32_t n = blockIdx.x * EW_THREADS + threadIdx.x;
    size_t o = ((size_t)blockIdx.y << logN) + n;
    u64 v = ct[o];
    if (blockIdx.y < n_limbs) v = addmod(v, pt[o], mc[blockIdx.y].q);
    out[o] = v;
}

// Tensor product of two ciphertexts (the first half of MulCt): d0 = a0*b0, d1 = a0*b1 + a1*b0,
// d2 = a1*b1, slot-wise per limb.  grid: (N/256, level+1).
__global__ __launch_bounds__(EW_THREADS) void tensor_kernel(const u64* __restrict__ a, const u64* __restrict__ b, u64* __restrict__ d,
                                                            const ModConst* mc, uint32_t logN, uint32_t L1) {
    const uint32_t n = blockIdx.x * EW_THREADS + threadIdx.x;
    const uint32_t limb = blockIdx.y;
    const ModConst m = mc[limb];
    const size_t o0 = ((size_t)limb << logN) + n, o1 = ((size_t)(limb + L1) << logN) + n, o2 = ((size_t)(limb + 2 * L1) << logN) + n;
    const u64 a0 = a[o0], a1 = a[o1], b0 = b[o0], b1 = b[o1];
    d[o0] = mulmod(a0, b0, m);
    d[o1] = barrett128((u128)a0 * b1 + (u128)a1 * b0, m.q, m.mu, m.bits);
    d[o2] = mulmod(a1, b1, m);
}

int32_t launch_tensor(he_ctx* ctx, const u64* a, const u64* b, uint32_t level, u64* d) {
    dim3 grid(ctx->N / EW_THREADS, level + 1), block(EW_THREADS);
    hipLaunchKernelGGL(tensor_kernel, grid, block, 0, ctx->stream, a, b, d, ctx->d_mc, ctx->logN, level + 1);
    HE_HIP(ctx, hipGetLastError());
    return HE_OK;
}

// out_c[r] = ct_c[r] * mul[r] (+ add[r] on component 0).  grid: (N/256, 2*(level+1)).
struct AffineArgs {
    u64 mul[HE_MAX_MODULI], mul_sh[HE_MAX_MODULI], add[HE_MAX_MODULI];
};
__global__ __launch_bounds__(EW_THREADS) void affine_kernel(const u64* ct, u64* out, AffineArgs aa,
                                                            const ModConst* mc, uint32_t logN, uint32_t L1) {
    const uint32_t n = blockIdx.x * EW_THREADS + threadIdx.x;
    const uint32_t r = blockIdx.y % L1, comp = blockIdx.y / L1;
    const u64 q = mc[r].q;
    const size_t o = ((size_t)blockIdx.y << logN) + n;
    u64 v = shoup_mul(ct[o], aa.mul[r], aa.mul_sh[r], q);
    if (comp == 0) v = addmod(v, aa.add[r], q);
    out[o] = v;
}

// k.mul / k.add: canonical residues of limbs 0..level; out may alias ct.
int32_t launch_affine(he_ctx* ctx, const u64* ct, uint32_t level, const AffineConst& k, u64* out) {
    AffineArgs aa;
    for (uint32_t r = 0; r <= level; r++) {
        aa.mul[r] = k.mul[r];
        aa.mul_sh[r] = h_shoup(k.mul[r], ctx->mod[r]);
        aa.add[r] = k.add[r];
    }
    dim3 grid(ctx->N / EW_THREADS, 2 * (level + 1)), block(EW_THREADS);
    hipLaunchKernelGGL(affine_kernel, grid, block, 0, ctx->stream, ct, out, aa, ctx->d_mc, ctx->logN, level + 1);
    HE_HIP(ctx, hipGetLastError());
    return HE_OK;
}

int32_t launch_automorph_ntt(he_ctx* ctx, const u64* in, u64* out, uint32_t n_limbs, uint32_t g) {
    if (n_limbs == 0) return HE_OK;
    dim3 grid(ctx->N / EW_THREADS, n_limbs), block(EW_THREADS);
    hipLaunchKernelGGL(automorph_ntt_kernel, grid, block, 0, ctx->stream, in, out, ctx->logN, g);
    HE_HIP(ctx, hipGetLastError());
    ctx->cnt.automorph += n_limbs;
    return HE_OK;
}

int32_t launch_automorph_coef(he_ctx* ctx, const u64* in, u64* out, const uint32_t* mod_idx, uint32_t n, uint32_t g) {
    if (n == 0) return HE_OK;
    LimbList ll;
    for (uint32_t i = 0; i < n; i++) ll.mod[i] = (uint8_t)mod_idx[i];
    // inverse of g modulo 2N (g odd): g^(N-1) since the unit group of Z_2N has exponent N/2 | N
    uint32_t twoN = 2 * ctx->N;
    u64 ginv = 1, b = g;
    for (uint32_t e = ctx->N - 1; e; e >>= 1) {
        if (e & 1) ginv = ginv * b % twoN;
        b = b * b % twoN;
    }
    dim3 grid(ctx->N / EW_THREADS, n), block(EW_THREADS);
    hipLaunchKernelGGL(automorph_coef_kernel, grid, block, 0, ctx->stream, in, out, ctx->d_mc, ll, ctx->logN, (uint32_t)ginv);
    HE_HIP(ctx, hipGetLastError());
    ctx->cnt.automorph += n;
    return HE_OK;
}

extern "C" {

int32_t he_automorph(he_ctx* ctx, const uint64_t* d_in, uint64_t* d_out, const uint32_t* h_mod_idx,
                     uint32_t n_limbs, uint32_t galois_elt, int32_t ntt_form) {
    return he_guard(ctx, "he_automorph: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (!d_in || !d_out || !h_mod_idx) return he_fail(ctx, HE_ERR_BADARG, "he_automorph: null argument");
    if ((galois_elt & 1u) == 0 || galois_elt >= 2 * ctx->N) return he_fail(ctx, HE_ERR_BADARG, "he_automorph: Galois element %u is not odd and below 2N", galois_elt);
    size_t bytes = (size_t)n_limbs * ctx->N * sizeof(u64);
    const char *a = (const char*)d_in, *b = (const char*)d_out;
    if (a < b + bytes && b < a + bytes) return he_fail(ctx, HE_ERR_BADARG, "he_automorph: input and output overlap");
    for (uint32_t i = 0; i < n_limbs; i++)
        if (h_mod_idx[i] >= ctx->M) return he_fail(ctx, HE_ERR_BADARG, "he_automorph: modulus index out of range");
    for (uint32_t o = 0; o < n_limbs; o += HE_MAX_LAUNCH_LIMBS) {
        uint32_t n = n_limbs - o < HE_MAX_LAUNCH_LIMBS ? n_limbs - o : HE_MAX_LAUNCH_LIMBS;
        const u64* in = (const u64*)d_in + (size_t)o * ctx->N;
        u64* out = (u64*)d_out + (size_t)o * ctx->N;
        int32_t rc = ntt_form ? launch_automorph_ntt(ctx, in, out, n, galois_elt)
                              : launch_automorph_coef(ctx, in, out, h_mod_idx + o, n, galois_elt);
        if (rc != HE_OK) return rc;
    }
    return HE_OK;
    });
}

int32_t he_ptct_mac(he_ctx* ctx, uint64_t* d_acc, const uint64_t* d_ct, const uint64_t* d_pt, uint32_t level, int32_t init) {
    return he_guard(ctx, "he_ptct_mac: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (!d_acc || !d_ct || !d_pt) return he_fail(ctx, HE_ERR_BADARG, "he_ptct_mac: null argument");
    if (level >= ctx->nq) return he_fail(ctx, HE_ERR_LEVEL, "he_ptct_mac: level %u above L=%u", level, ctx->nq - 1);
    {
        // the kernel reads ct and pt through restrict pointers while it writes acc
        const size_t pb = (size_t)(level + 1) * ctx->N * sizeof(u64);
        const char *a = (const char*)d_acc, *c = (const char*)d_ct, *p = (const char*)d_pt;
        if ((a < c + 2 * pb && c < a + 2 * pb) || (a < p + pb && p < a + 2 * pb))
            return he_fail(ctx, HE_ERR_BADARG, "he_ptct_mac: the accumulator overlaps the ciphertext or the plaintext");
    }
    dim3 grid(ctx->N / EW_THREADS, level + 1), block(EW_THREADS);
    hipLaunchKernelGGL(ptct_mac_kernel, grid, block, 0, ctx->stream, (u64*)d_acc, (const u64*)d_ct, (const u64*)d_pt,
                       ctx->d_mc, ctx->logN, level + 1, init);
    HE_HIP(ctx, hipGetLastError());
    ctx->cnt.mac += 1;
    return HE_OK;
    });
}

int32_t he_ptct_mac_rot(he_ctx* ctx, uint64_t* d_acc, const uint64_t* const* h_d_ct, const uint64_t* const* h_d_pt,
                        const uint32_t* h_galois, uint32_t n, uint32_t level, int32_t init) {
    return he_guard(ctx, "he_ptct_mac_rot: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (!d_acc || (n && (!h_d_ct || !h_d_pt || !h_galois))) return he_fail(ctx, HE_ERR_BADARG, "he_ptct_mac_rot: null argument");
    if (level >= ctx->nq) return he_fail(ctx, HE_ERR_LEVEL, "he_ptct_mac_rot: level %u above L=%u", level, ctx->nq - 1);
    const size_t pb = (size_t)(level + 1) * ctx->N * sizeof(u64);
    for (uint32_t i = 0; i < n; i++) {
        if (!h_d_ct[i] || !h_d_pt[i]) return he_fail(ctx, HE_ERR_BADARG, "he_ptct_mac_rot: operand %u is null", i);
        if ((h_galois[i] & 1u) == 0 || h_galois[i] >= 2 * ctx->N)
            return he_fail(ctx, HE_ERR_BADARG, "he_ptct_mac_rot: Galois element %u is not odd and below 2N", h_galois[i]);
        const char *a = (const char*)d_acc, *c = (const char*)h_d_ct[i], *p = (const char*)h_d_pt[i];
        if ((a < c + 2 * pb && c < a + 2 * pb) || (a < p + pb && p < a + 2 * pb))
            return he_fail(ctx, HE_ERR_BADARG, "he_ptct_mac_rot: the accumulator overlaps operand %u", i);
    }
    dim3 grid(ctx->N / EW_THREADS, level + 1), block(EW_THREADS);
    if (n == 0 && init) {                                  // an empty sum: the accumulator is cleared
        MacRot mr = {};
        hipLaunchKernelGGL(ptct_mac_rot_kernel, grid, block, 0, ctx->stream, (u64*)d_acc, mr, ctx->d_mc, ctx->logN, level + 1, 1);
        HE_HIP(ctx, hipGetLastError());
    }
    for (uint32_t i0 = 0; i0 < n; i0 += MACROT_MAX) {
        MacRot mr = {};
        mr.n = std::min<uint32_t>(MACROT_MAX, n - i0);
        for (uint32_t i = 0; i < mr.n; i++) { mr.ct[i] = (const u64*)h_d_ct[i0 + i]; mr.pt[i] = (const u64*)h_d_pt[i0 + i]; mr.g[i] = h_galois[i0 + i]; }
        hipLaunchKernelGGL(ptct_mac_rot_kernel, grid, block, 0, ctx->stream, (u64*)d_acc, mr, ctx->d_mc, ctx->logN, level + 1,
                           (init && i0 == 0) ? 1 : 0);
        HE_HIP(ctx, hipGetLastError());
    }
    ctx->cnt.mac += n;
    for (uint32_t i = 0; i < n; i++) ctx->cnt.automorph += h_galois[i] != 1 ? level + 1 : 0;
    return HE_OK;
    });
}

int32_t he_affine(he_ctx* ctx, const uint64_t* d_ct, uint32_t level, const uint64_t* h_mul, const uint64_t* h_add, uint64_t* d_out) {
    return he_guard(ctx, "he_affine: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (!d_ct || !d_out || !h_mul || !h_add) return he_fail(ctx, HE_ERR_BADARG, "he_affine: null argument");
    if (level >= ctx->nq) return he_fail(ctx, HE_ERR_LEVEL, "he_affine: level %u above L=%u", level, ctx->nq - 1);
    AffineConst k;
    for (uint32_t r = 0; r <= level; r++) {
        if (h_mul[r] >= ctx->mod[r] || h_add[r] >= ctx->mod[r]) return he_fail(ctx, HE_ERR_BADARG, "he_affine: constant of limb %u is not a canonical residue", r);
        k.mul[r] = h_mul[r];
        k.add[r] = h_add[r];
    }
    return launch_affine(ctx, (const u64*)d_ct, level, k, (u64*)d_out);
    });
}

int32_t he_add(he_ctx* ctx, const uint64_t* d_a, const uint64_t* d_b, uint32_t level, uint64_t* d_out) {
    return he_guard(ctx, "he_add: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (!d_a || !d_b || !d_out) return he_fail(ctx, HE_ERR_BADARG, "he_add: null argument");
    if (level >= ctx->nq) return he_fail(ctx, HE_ERR_LEVEL, "he_add: level %u above L=%u", level, ctx->nq - 1);
    dim3 grid(ctx->N / EW_THREADS, 2 * (level + 1)), block(EW_THREADS);
    hipLaunchKernelGGL(add_kernel, grid, block, 0, ctx->stream, (const u64*)d_a, (const u64*)d_b, (u64*)d_out, ctx->d_mc,
                       ctx->logN, level + 1);
    HE_HIP(ctx, hipGetLastError());
    return HE_OK;
    });
}

int32_t he_addpt(he_ctx* ctx, const uint64_t* d_ct, const uint64_t* d_pt, uint32_t level, uint64_t* d_out) {
    return he_guard(ctx, "he_addpt: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (!d_ct || !d_pt || !d_out) return he_fail(ctx, HE_ERR_BADARG, "he_addpt: null argument");
    if (level >= ctx->nq) return he_fail(ctx, HE_ERR_LEVEL, "he_addpt: level %u above L=%u", level, ctx->nq - 1);
    dim3 grid(ctx->N / EW_THREADS, 2 * (level + 1)), block(EW_THREADS);
    hipLaunchKernelGGL(addpt_kernel, grid, block, 0, ctx->stream, (const u64*)d_ct, (const u64*)d_pt, (u64*)d_out, ctx->d_mc,
                       ctx->logN, level + 1);
    HE_HIP(ctx, hipGetLastError());
    return HE_OK;
    });
}

} // extern "C"
