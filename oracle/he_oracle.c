/*
 * CPU oracle for the encrypted-convolution hot path (RNS-CKKS): TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct C: every modular product is (unsigned __int128) a*b % q,
 * every step follows the textbook definition of the operation in the order the scheme
 * states it.  It shares no code, header, table or constant generator with the HIP library.
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * What the paper fixes and what it leaves to the scheme it builds on:
 *   - ring R = Z[X]/(X^N+1), ciphertext = pair of polynomials, N/2 slots (Section 2.1);
 *   - operations AddCt/MulPt/Rescale/CRot (left slot rotation) as black boxes (Section 2.1,
 *     Table 1), key switching with an evaluation key and decomposition number dnum
 *     (Appendix, parameter sets and memory footprint);
 *   - the convolution built from them: SISO (Algorithm 1), rotate-and-sum, CAConv
 *     (Section 3.1).
 * The arithmetic below the black boxes (negacyclic NTT, RNS basis conversion, hybrid key
 * switching, exact rescale) is the standard RNS-CKKS construction; the readings chosen where
 * several valid variants exist are listed next to each function.
 *
 * Layout everywhere: limb-major [poly][limb][N] uint64, canonical residues in [0, q).
 * "NTT form" = evaluations at psi^(2*brv(j)+1), j = 0..N-1 (bit-reversed order).
 * Modulus index space: 0..nq-1 are q_0..q_L, nq..nq+np-1 are p_0..p_{k-1}.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef uint64_t u64;
typedef unsigned __int128 u128;

#define ORC_MAXMOD 64

typedef struct {
    uint32_t logN, N, nq, np, dnum, alpha;
    u64 mod[ORC_MAXMOD];   /* q_0..q_L then p_0..p_{k-1} */
    u64 psi[ORC_MAXMOD];   /* primitive 2N-th root of unity per modulus */
} orc_ctx;

/* ---------------------------------------------------------------- scalar arithmetic */

u64 orc_mulmod(u64 a, u64 b, u64 m) { return (u64)((u128)a * b % m); }
static u64 addmod(u64 a, u64 b, u64 m) { return (u64)(((u128)a + b) % m); }
static u64 submod(u64 a, u64 b, u64 m) { return (u64)(((u128)a + m - b % m) % m); }

u64 orc_powmod(u64 a, u64 e, u64 m) {
    u64 r = 1 % m;
    a %= m;
    while (e) {
        if (e & 1) r = orc_mulmod(r, a, m);
        a = orc_mulmod(a, a, m);
        e >>= 1;
    }
    return r;
}

/* m prime: a^(m-2) */
u64 orc_invmod(u64 a, u64 m) { return orc_powmod(a, m - 2, m); }

static uint32_t brv(uint32_t x, uint32_t bits) {
    uint32_t r = 0;
    for (uint32_t i = 0; i < bits; i++) r |= ((x >> i) & 1u) << (bits - 1 - i);
    return r;
}

/* Root rule: psi = c^((q-1)/2N) for the smallest integer c >= 2 that is a quadratic
 * non-residue mod q (c^((q-1)/2) = -1).  Then psi^N = -1, so psi has order exactly 2N. */
u64 orc_find_psi(u64 q, uint32_t N) {
    for (u64 c = 2;; c++) {
        if (orc_powmod(c, (q - 1) / 2, q) == q - 1) return orc_powmod(c, (q - 1) / (2 * (u64)N), q);
    }
}

/* ---------------------------------------------------------------- context */

orc_ctx* orc_create(uint32_t logN, const u64* q, uint32_t nq, const u64* p, uint32_t np, uint32_t dnum) {
    if (nq + np > ORC_MAXMOD || nq == 0 || dnum == 0) return NULL;
    orc_ctx* c = (orc_ctx*)calloc(1, sizeof(orc_ctx));
    c->logN = logN; c->N = 1u << logN; c->nq = nq; c->np = np; c->dnum = dnum;
    c->alpha = (nq + dnum - 1) / dnum;
    for (uint32_t i = 0; i < nq; i++) c->mod[i] = q[i];
    for (uint32_t i = 0; i < np; i++) c->mod[nq + i] = p[i];
    for (uint32_t i = 0; i < nq + np; i++) c->psi[i] = orc_find_psi(c->mod[i], c->N);
    return c;
}
void orc_destroy(orc_ctx* c) { free(c); }
/* threads the limb-parallel loops will use */
int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
u64 orc_psi(const orc_ctx* c, uint32_t mi) { return c->psi[mi]; }
u64 orc_modulus(const orc_ctx* c, uint32_t mi) { return c->mod[mi]; }

/* ---------------------------------------------------------------- ring definitions */

/* Negacyclic product in Z_q[X]/(X^N+1) by the schoolbook definition:
 * c_k = sum_{i+j=k} a_i b_j - sum_{i+j=k+N} a_i b_j. */
void orc_negacyclic_mul_def(u64 q, uint32_t N, const u64* a, const u64* b, u64* out) {
    for (uint32_t k = 0; k < N; k++) out[k] = 0;
    for (uint32_t i = 0; i < N; i++)
        for (uint32_t j = 0; j < N; j++) {
            u64 t = orc_mulmod(a[i], b[j], q);
            uint32_t k = i + j;
            if (k < N) out[k] = addmod(out[k], t, q);
            else out[k - N] = submod(out[k - N], t, q);
        }
}

/* Forward transform by its definition, O(N^2): out[j] = sum_i a_i psi^((2 brv(j)+1) i). */
void orc_ntt_def(const orc_ctx* c, uint32_t mi, const u64* a, u64* out) {
    u64 q = c->mod[mi];
    for (uint32_t j = 0; j < c->N; j++) {
        u64 x = orc_powmod(c->psi[mi], 2 * (u64)brv(j, c->logN) + 1, q);
        u64 acc = 0, xp = 1;
        for (uint32_t i = 0; i < c->N; i++) {
            acc = addmod(acc, orc_mulmod(a[i], xp, q), q);
            xp = orc_mulmod(xp, x, q);
        }
        out[j] = acc;
    }
}

/* Textbook iterative radix-2 cyclic transform, natural order in and out:
 * A[k] = sum_i a_i w^(ik), w of order N. */
static void cyclic_fft(u64* a, uint32_t logN, u64 w, u64 q) {
    uint32_t N = 1u << logN;
    for (uint32_t i = 0; i < N; i++) {
        uint32_t j = brv(i, logN);
        if (i < j) { u64 t = a[i]; a[i] = a[j]; a[j] = t; }
    }
    for (uint32_t len = 2; len <= N; len <<= 1) {
        u64 wlen = orc_powmod(w, N / len, q);
        for (uint32_t i = 0; i < N; i += len) {
            u64 wk = 1;
            for (uint32_t j = 0; j < len / 2; j++) {
                u64 u = a[i + j], v = orc_mulmod(a[i + j + len / 2], wk, q);
                a[i + j] = addmod(u, v, q);
                a[i + j + len / 2] = submod(u, v, q);
                wk = orc_mulmod(wk, wlen, q);
            }
        }
    }
}

/* Forward negacyclic NTT of one limb, in place, coefficient form -> NTT form:
 * twist by psi^i, cyclic transform with w = psi^2 (gives a(psi^(2k+1)) at index k),
 * then store index k at position brv(k). */
static void ntt_limb(const orc_ctx* c, uint32_t mi, u64* a) {
    u64 q = c->mod[mi], psi = c->psi[mi], pw = 1;
    uint32_t N = c->N;
    for (uint32_t i = 0; i < N; i++) { a[i] = orc_mulmod(a[i] % q, pw, q); pw = orc_mulmod(pw, psi, q); }
    cyclic_fft(a, c->logN, orc_mulmod(psi, psi, q), q);
    for (uint32_t i = 0; i < N; i++) {
        uint32_t j = brv(i, c->logN);
        if (i < j) { u64 t = a[i]; a[i] = a[j]; a[j] = t; }
    }
}

/* Inverse: undo the bit-reversed storage, cyclic transform with w^-1, scale by N^-1 and
 * untwist by psi^-i. */
static void intt_limb(const orc_ctx* c, uint32_t mi, u64* a) {
    u64 q = c->mod[mi], psi = c->psi[mi];
    uint32_t N = c->N;
    for (uint32_t i = 0; i < N; i++) {
        uint32_t j = brv(i, c->logN);
        if (i < j) { u64 t = a[i]; a[i] = a[j]; a[j] = t; }
    }
    u64 winv = orc_invmod(orc_mulmod(psi, psi, q), q);
    cyclic_fft(a, c->logN, winv, q);
    u64 ninv = orc_invmod(N % q, q), pinv = orc_invmod(psi, q), pw = 1;
    for (uint32_t i = 0; i < N; i++) {
        a[i] = orc_mulmod(orc_mulmod(a[i], ninv, q), pw, q);
        pw = orc_mulmod(pw, pinv, q);
    }
}

void orc_ntt(const orc_ctx* c, u64* data, const uint32_t* mod_idx, uint32_t n_limbs) {
#pragma omp parallel for schedule(dynamic)
    for (uint32_t l = 0; l < n_limbs; l++) ntt_limb(c, mod_idx[l], data + (size_t)l * c->N);
}
void orc_intt(const orc_ctx* c, u64* data, const uint32_t* mod_idx, uint32_t n_limbs) {
#pragma omp parallel for schedule(dynamic)
    for (uint32_t l = 0; l < n_limbs; l++) intt_limb(c, mod_idx[l], data + (size_t)l * c->N);
}

/* ---------------------------------------------------------------- automorphism */

/* sigma_g on coefficient form: X^i -> X^(i g); X^N = -1.  g odd. */
void orc_automorph_coef(const orc_ctx* c, const u64* in, u64* out, const uint32_t* mod_idx,
                        uint32_t n_limbs, uint32_t g) {
    uint32_t N = c->N;
    for (uint32_t l = 0; l < n_limbs; l++) {
        u64 q = c->mod[mod_idx[l]];
        const u64* a = in + (size_t)l * N;
        u64* o = out + (size_t)l * N;
        for (uint32_t i = 0; i < N; i++) {
            uint32_t t = (uint32_t)(((u64)i * g) % (2 * (u64)N));
            if (t < N) o[t] = a[i];
            else o[t - N] = (a[i] == 0) ? 0 : q - a[i];
        }
    }
}

/* sigma_g on NTT form: position j holds a(psi^e), e = 2 brv(j)+1.  sigma_g(a)(psi^e) =
 * a(psi^(e g)), which is held at position brv((e g mod 2N - 1)/2). */
void orc_automorph_ntt(const orc_ctx* c, const u64* in, u64* out, uint32_t n_limbs, uint32_t g) {
    uint32_t N = c->N;
    for (uint32_t l = 0; l < n_limbs; l++) {
        const u64* a = in + (size_t)l * N;
        u64* o = out + (size_t)l * N;
        for (uint32_t j = 0; j < N; j++) {
            u64 e = 2 * (u64)brv(j, c->logN) + 1;
            u64 eg = (e * g) % (2 * (u64)N);
            o[j] = a[brv((uint32_t)((eg - 1) / 2), c->logN)];
        }
    }
}

/* ---------------------------------------------------------------- hybrid key switching */

static uint32_t n_digits(const orc_ctx* c, uint32_t level) { return (level + 1 + c->alpha - 1) / c->alpha; }
static uint32_t digit_lo(const orc_ctx* c, uint32_t j) { return j * c->alpha; }
static uint32_t digit_hi(const orc_ctx* c, uint32_t j, uint32_t level) {
    uint32_t h = (j + 1) * c->alpha;
    return h < level + 1 ? h : level + 1;
}
/* modulus index of raised-basis limb r at `level`: q_0..q_level then p_0..p_{k-1} */
static uint32_t raised_mod(const orc_ctx* c, uint32_t level, uint32_t r) {
    return r <= level ? r : c->nq + (r - level - 1);
}

uint32_t orc_num_digits(const orc_ctx* c, uint32_t level) { return n_digits(c, level); }

/* Fast (approximate) basis conversion of coefficient-form limbs x_i over the moduli
 * src[0..ns) to the modulus t:  y_i = x_i * [(S/s_i)^-1]_{s_i} mod s_i  (canonical),
 * out = sum_i y_i * ((S/s_i) mod t) mod t, with S = prod s_i.  No correction of the
 * overflow multiple: the value represented is x + u*S with 0 <= u < ns. */
static void base_convert(const orc_ctx* c, const uint32_t* src, uint32_t ns, const u64* const* x,
                         uint32_t t_idx, u64* out) {
    uint32_t N = c->N;
    u64 t = c->mod[t_idx];
    u64 inv_hat[ORC_MAXMOD], hat_mod_t[ORC_MAXMOD];
    for (uint32_t i = 0; i < ns; i++) {
        u64 si = c->mod[src[i]], hat_si = 1, hat_t = 1;
        for (uint32_t k = 0; k < ns; k++) {
            if (k == i) continue;
            hat_si = orc_mulmod(hat_si, c->mod[src[k]] % si, si);
            hat_t = orc_mulmod(hat_t, c->mod[src[k]] % t, t);
        }
        inv_hat[i] = orc_invmod(hat_si, si);
        hat_mod_t[i] = hat_t;
    }
    for (uint32_t n = 0; n < N; n++) {
        u64 acc = 0;
        for (uint32_t i = 0; i < ns; i++) {
            u64 y = orc_mulmod(x[i][n], inv_hat[i], c->mod[src[i]]);
            acc = addmod(acc, orc_mulmod(y % t, hat_mod_t[i], t), t);
        }
        out[n] = acc;
    }
}

/* ModUp: in = one polynomial [level+1][N] in NTT form.  out = [beta][level+1+k][N] in NTT
 * form: digit j's own limbs copied, every other limb of the raised basis obtained by
 * iNTT(digit limbs) -> base_convert -> NTT.  Digits are the raw limbs (no pre-scaling). */
void orc_modup(const orc_ctx* c, const u64* in, uint32_t level, u64* out) {
    uint32_t N = c->N, R = level + 1 + c->np, beta = n_digits(c, level);
    for (uint32_t j = 0; j < beta; j++) {
        uint32_t lo = digit_lo(c, j), hi = digit_hi(c, j, level), ns = hi - lo;
        u64* coef = (u64*)malloc((size_t)ns * N * sizeof(u64));
        uint32_t src[ORC_MAXMOD];
        const u64* xs[ORC_MAXMOD];
        memcpy(coef, in + (size_t)lo * N, (size_t)ns * N * sizeof(u64));
        for (uint32_t i = 0; i < ns; i++) { src[i] = lo + i; xs[i] = coef + (size_t)i * N; }
        orc_intt(c, coef, src, ns);
        u64* dj = out + (size_t)j * R * N;
#pragma omp parallel for schedule(dynamic)
        for (uint32_t r = 0; r < R; r++) {
            u64* o = dj + (size_t)r * N;
            if (r >= lo && r < hi) {
                memcpy(o, in + (size_t)r * N, N * sizeof(u64));
            } else {
                uint32_t mi = raised_mod(c, level, r);
                base_convert(c, src, ns, xs, mi, o);
                ntt_limb(c, mi, o);
            }
        }
        free(coef);
    }
}

/* Inner product of the raised digits with an evaluation key.
 * digits [beta][level+1+k][N]; evk [dnum][2][nq+np][N] (component 0 = b, 1 = a);
 * acc [2][level+1+k][N]:  acc_c[r] = sum_j digits_j[r] * evk_j,c[r]  mod m_r. */
void orc_inner_product(const orc_ctx* c, const u64* digits, uint32_t level, const u64* evk, u64* acc) {
    uint32_t N = c->N, R = level + 1 + c->np, beta = n_digits(c, level), M = c->nq + c->np;
#pragma omp parallel for schedule(dynamic) collapse(2)
    for (uint32_t comp = 0; comp < 2; comp++)
        for (uint32_t r = 0; r < R; r++) {
            uint32_t mi = raised_mod(c, level, r);
            u64 m = c->mod[mi];
            u64* o = acc + ((size_t)comp * R + r) * N;
            for (uint32_t n = 0; n < N; n++) o[n] = 0;
            for (uint32_t j = 0; j < beta; j++) {
                const u64* d = digits + ((size_t)j * R + r) * N;
                const u64* k = evk + (((size_t)j * 2 + comp) * M + mi) * N;
                for (uint32_t n = 0; n < N; n++) o[n] = addmod(o[n], orc_mulmod(d[n], k[n], m), m);
            }
        }
}

/* ModDown of one polynomial over the raised basis, [level+1+k][N] NTT form -> [level+1][N]:
 * the k special limbs go to coefficient form, are converted (fast conversion, no rounding
 * term) to each q_r, transformed back, and out_r = (acc_r - conv_r) * P^-1 mod q_r. */
void orc_moddown(const orc_ctx* c, const u64* acc, uint32_t level, u64* out) {
    uint32_t N = c->N, k = c->np;
    u64* coef = (u64*)malloc((size_t)k * N * sizeof(u64));
    uint32_t src[ORC_MAXMOD];
    const u64* xs[ORC_MAXMOD];
    memcpy(coef, acc + (size_t)(level + 1) * N, (size_t)k * N * sizeof(u64));
    for (uint32_t t = 0; t < k; t++) { src[t] = c->nq + t; xs[t] = coef + (size_t)t * N; }
    orc_intt(c, coef, src, k);
#pragma omp parallel for schedule(dynamic)
    for (uint32_t r = 0; r <= level; r++) {
        u64 q = c->mod[r], pinv = 1;
        for (uint32_t t = 0; t < k; t++) pinv = orc_mulmod(pinv, c->mod[c->nq + t] % q, q);
        pinv = orc_invmod(pinv, q);
        u64* o = out + (size_t)r * N;
        base_convert(c, src, k, xs, r, o);
        ntt_limb(c, r, o);
        const u64* a = acc + (size_t)r * N;
        for (uint32_t n = 0; n < N; n++) o[n] = orc_mulmod(submod(a[n], o[n], q), pinv, q);
    }
    free(coef);
}

/* Key switch of one polynomial d (NTT form, [level+1][N]) with the key `evk`:
 * (out0, out1) with out0 + out1*s = d*s' + small.  No automorphism applied. */
void orc_keyswitch(const orc_ctx* c, const u64* in, uint32_t level, const u64* evk, u64* out0, u64* out1) {
    uint32_t N = c->N, R = level + 1 + c->np, beta = n_digits(c, level);
    u64* digits = (u64*)malloc((size_t)beta * R * N * sizeof(u64));
    u64* acc = (u64*)malloc((size_t)2 * R * N * sizeof(u64));
    orc_modup(c, in, level, digits);
    orc_inner_product(c, digits, level, evk, acc);
    orc_moddown(c, acc, level, out0);
    orc_moddown(c, acc + (size_t)R * N, level, out1);
    free(digits); free(acc);
}

/* Rotation from already-raised digits of c1 (the shared part of a hoisted rotation):
 * acc = sum_j sigma_g(raised_j) * evk_{g,j};  (ks0, ks1) = ModDown(acc);
 * out = (sigma_g(c0) + ks0, ks1).  The automorphism acts on the raised digits, before
 * ModDown; that order is part of the contract because ModDown does not commute with it. */
void orc_rotate_from_raised(const orc_ctx* c, const u64* ct, const u64* raised, uint32_t level, uint32_t g,
                            const u64* evk, u64* out) {
    uint32_t N = c->N, R = level + 1 + c->np, beta = n_digits(c, level), L1 = level + 1;
    u64* rot = (u64*)malloc((size_t)beta * R * N * sizeof(u64));
    u64* acc = (u64*)malloc((size_t)2 * R * N * sizeof(u64));
    u64* s0 = (u64*)malloc((size_t)L1 * N * sizeof(u64));
    orc_automorph_ntt(c, raised, rot, beta * R, g);
    orc_inner_product(c, rot, level, evk, acc);
    orc_moddown(c, acc, level, out);
    orc_moddown(c, acc + (size_t)R * N, level, out + (size_t)L1 * N);
    orc_automorph_ntt(c, ct, s0, L1, g);
    for (uint32_t r = 0; r < L1; r++)
        for (uint32_t n = 0; n < N; n++)
            out[(size_t)r * N + n] = addmod(out[(size_t)r * N + n], s0[(size_t)r * N + n], c->mod[r]);
    free(rot); free(acc); free(s0);
}

/* out[l] = a[l] + b[l] mod the modulus listed for limb l (used to add key-switch accumulators over the
 * raised basis q_0..q_level, p_*). */
void orc_add_limbs(const orc_ctx* c, const u64* a, const u64* b, const uint32_t* mod_idx, uint32_t n_limbs, u64* out) {
    for (uint32_t l = 0; l < n_limbs; l++) {
        u64 m = c->mod[mod_idx[l]];
        for (uint32_t n = 0; n < c->N; n++) {
            size_t i = (size_t)l * c->N + n;
            out[i] = addmod(a[i], b[i], m);
        }
    }
}

/* Rotation of a ciphertext ct = [2][level+1][N] by Galois element g with its key. */
void orc_rotate(const orc_ctx* c, const u64* ct, uint32_t level, uint32_t g, const u64* evk, u64* out) {
    uint32_t N = c->N, R = level + 1 + c->np, beta = n_digits(c, level);
    u64* raised = (u64*)malloc((size_t)beta * R * N * sizeof(u64));
    orc_modup(c, ct + (size_t)(level + 1) * N, level, raised);
    orc_rotate_from_raised(c, ct, raised, level, g, evk, out);
    free(raised);
}

/* ---------------------------------------------------------------- MulPt-accumulate, rescale */

/* acc.c0 (+)= ct.c0 * pt, acc.c1 (+)= ct.c1 * pt, slot-wise in NTT form, per limb mod q_i.
 * acc, ct: [2][level+1][N]; pt: [level+1][N]; init != 0 overwrites acc. */
void orc_ptct_mac(const orc_ctx* c, u64* acc, const u64* ct, const u64* pt, uint32_t level, int init) {
    uint32_t N = c->N, L1 = level + 1;
    for (uint32_t comp = 0; comp < 2; comp++)
        for (uint32_t r = 0; r < L1; r++) {
            u64 q = c->mod[r];
            size_t off = ((size_t)comp * L1 + r) * N;
            for (uint32_t n = 0; n < N; n++) {
                u64 t = orc_mulmod(ct[off + n], pt[(size_t)r * N + n], q);
                acc[off + n] = init ? t : addmod(acc[off + n], t, q);
            }
        }
}

/* Rescale by q_level with exact rounding: per coefficient round(c / q_level) (half up).
 * h = floor(q_level/2); t = (c_level + h) mod q_level in coefficient form;
 * out_i = (c_i + h - t) * q_level^-1 mod q_i for i < level.  ct [2][level+1][N] -> out [2][level][N]. */
void orc_rescale(const orc_ctx* c, const u64* ct, uint32_t level, u64* out) {
    uint32_t N = c->N, L1 = level + 1;
    u64 ql = c->mod[level], h = ql / 2;
    for (uint32_t comp = 0; comp < 2; comp++) {
        u64* t = (u64*)malloc((size_t)N * sizeof(u64));
        memcpy(t, ct + ((size_t)comp * L1 + level) * N, N * sizeof(u64));
        intt_limb(c, level, t);
        for (uint32_t n = 0; n < N; n++) t[n] = addmod(t[n], h, ql);
#pragma omp parallel for schedule(dynamic)
        for (uint32_t r = 0; r < level; r++) {
            u64 q = c->mod[r], qinv = orc_invmod(ql % q, q);
            u64* d = (u64*)malloc((size_t)N * sizeof(u64));
            for (uint32_t n = 0; n < N; n++) d[n] = submod(h % q, t[n] % q, q);
            ntt_limb(c, r, d);
            const u64* a = ct + ((size_t)comp * L1 + r) * N;
            u64* o = out + ((size_t)comp * level + r) * N;
            for (uint32_t n = 0; n < N; n++) o[n] = orc_mulmod(addmod(a[n], d[n], q), qinv, q);
            free(d);
        }
        free(t);
    }
}

/* MulCt (paper Section 2.1): tensor product d0 = a0*b0, d1 = a0*b1 + a1*b0, d2 = a1*b1 (slot-wise,
 * NTT form), then relinearisation of d2 with the key for s^2 -> s: out = (d0 + ks0, d1 + ks1).
 * a, b, out: [2][level+1][N].  The level does not change; the caller rescales. */
void orc_mulct(const orc_ctx* c, const u64* a, const u64* b, uint32_t level, const u64* rlk, u64* out) {
    uint32_t N = c->N, L1 = level + 1;
    size_t pe = (size_t)L1 * N;
    u64* d2 = (u64*)malloc(pe * sizeof(u64));
    u64* k0 = (u64*)malloc(pe * sizeof(u64));
    u64* k1 = (u64*)malloc(pe * sizeof(u64));
    for (uint32_t r = 0; r < L1; r++) {
        u64 q = c->mod[r];
        for (uint32_t n = 0; n < N; n++) {
            size_t i = (size_t)r * N + n;
            u64 a0 = a[i], a1 = a[pe + i], b0 = b[i], b1 = b[pe + i];
            out[i] = orc_mulmod(a0, b0, q);
            out[pe + i] = addmod(orc_mulmod(a0, b1, q), orc_mulmod(a1, b0, q), q);
            d2[i] = orc_mulmod(a1, b1, q);
        }
    }
    orc_keyswitch(c, d2, level, rlk, k0, k1);
    for (uint32_t r = 0; r < L1; r++)
        for (uint32_t n = 0; n < N; n++) {
            size_t i = (size_t)r * N + n;
            out[i] = addmod(out[i], k0[i], c->mod[r]);
            out[pe + i] = addmod(out[pe + i], k1[i], c->mod[r]);
        }
    free(d2); free(k0); free(k1);
}

/* out_c[r] = ct_c[r] * mul[r]  (+ add[r] at every position of c0: a constant polynomial has a
 * constant transform).  mul, add: canonical residues per limb.  Covers negation, multiplication by
 * an integer constant and adding a constant to every slot. */
void orc_affine(const orc_ctx* c, const u64* ct, uint32_t level, const u64* mul, const u64* add, u64* out) {
    uint32_t N = c->N, L1 = level + 1;
    for (uint32_t comp = 0; comp < 2; comp++)
        for (uint32_t r = 0; r < L1; r++) {
            u64 q = c->mod[r];
            size_t off = ((size_t)comp * L1 + r) * N;
            for (uint32_t n = 0; n < N; n++) {
                u64 v = orc_mulmod(ct[off + n], mul[r], q);
                if (comp == 0) v = addmod(v, add[r], q);
                out[off + n] = v;
            }
        }
}

/* out = a + b on [2][level+1][N] */
void orc_add(const orc_ctx* c, const u64* a, const u64* b, uint32_t level, u64* out) {
    uint32_t N = c->N, L1 = level + 1;
    for (uint32_t comp = 0; comp < 2; comp++)
        for (uint32_t r = 0; r < L1; r++) {
            size_t off = ((size_t)comp * L1 + r) * N;
            for (uint32_t n = 0; n < N; n++) out[off + n] = addmod(a[off + n], b[off + n], c->mod[r]);
        }
}

/* AddPt (Section 2.1): the plaintext is added to c0 slot-wise per limb; c1 is copied. */
void orc_addpt(const orc_ctx* c, const u64* ct, const u64* pt, uint32_t level, u64* out) {
    uint32_t N = c->N, L1 = level + 1;
    for (uint32_t r = 0; r < L1; r++)
        for (uint32_t n = 0; n < N; n++) {
            out[(size_t)r * N + n] = addmod(ct[(size_t)r * N + n], pt[(size_t)r * N + n], c->mod[r]);
            out[((size_t)L1 + r) * N + n] = ct[((size_t)L1 + r) * N + n];
        }
}

/* ---------------------------------------------------------------- client side (tests only) */

/* Signed coefficients -> canonical residues of the listed moduli, coefficient form. */
void orc_reduce_signed(const orc_ctx* c, const int64_t* m, const uint32_t* mod_idx, uint32_t n_limbs, u64* out) {
    for (uint32_t l = 0; l < n_limbs; l++) {
        u64 q = c->mod[mod_idx[l]];
        for (uint32_t n = 0; n < c->N; n++) {
            int64_t v = m[n];
            out[(size_t)l * c->N + n] = v >= 0 ? (u64)v % q : (q - ((u64)(-v) % q)) % q;
        }
    }
}

/* Pointwise a*b mod q per limb (NTT form). */
void orc_pointwise_mul(const orc_ctx* c, const u64* a, const u64* b, const uint32_t* mod_idx, uint32_t n_limbs, u64* out) {
    for (uint32_t l = 0; l < n_limbs; l++) {
        u64 q = c->mod[mod_idx[l]];
        for (uint32_t n = 0; n < c->N; n++) {
            size_t i = (size_t)l * c->N + n;
            out[i] = orc_mulmod(a[i], b[i], q);
        }
    }
}

/* Evaluation key for switching s' -> s over the full basis q_0..q_L, p_0..p_{k-1}:
 * for digit j and limb r:  a_j uniform (given, taken as NTT form),
 * b_j = -a_j*s + e_j + [r is a q-limb of digit j] * (P mod q_r) * s'.
 * s, sprime: signed coefficient vectors [N]; a: [dnum][M][N]; e: signed [dnum][N];
 * evk out: [dnum][2][M][N] NTT form (0 = b, 1 = a). */
void orc_make_evk(const orc_ctx* c, const int64_t* s, const int64_t* sprime, const u64* a, const int64_t* e, u64* evk) {
    uint32_t N = c->N, M = c->nq + c->np;
    uint32_t idx[ORC_MAXMOD];
    for (uint32_t r = 0; r < M; r++) idx[r] = r;
    u64* sh = (u64*)malloc((size_t)M * N * sizeof(u64));
    u64* sph = (u64*)malloc((size_t)M * N * sizeof(u64));
    u64* eh = (u64*)malloc((size_t)M * N * sizeof(u64));
    orc_reduce_signed(c, s, idx, M, sh); orc_ntt(c, sh, idx, M);
    orc_reduce_signed(c, sprime, idx, M, sph); orc_ntt(c, sph, idx, M);
    for (uint32_t j = 0; j < c->dnum; j++) {
        orc_reduce_signed(c, e + (size_t)j * N, idx, M, eh); orc_ntt(c, eh, idx, M);
        uint32_t lo = j * c->alpha, hi = (j + 1) * c->alpha < c->nq ? (j + 1) * c->alpha : c->nq;
        for (uint32_t r = 0; r < M; r++) {
            u64 m = c->mod[r], Pm = 1;
            for (uint32_t t = 0; t < c->np; t++) Pm = orc_mulmod(Pm, c->mod[c->nq + t] % m, m);
            const u64* aj = a + ((size_t)j * M + r) * N;
            u64* bo = evk + (((size_t)j * 2 + 0) * M + r) * N;
            u64* ao = evk + (((size_t)j * 2 + 1) * M + r) * N;
            int in_digit = (r >= lo && r < hi);
            for (uint32_t n = 0; n < N; n++) {
                u64 v = submod(eh[(size_t)r * N + n], orc_mulmod(aj[n], sh[(size_t)r * N + n], m), m);
                if (in_digit) v = addmod(v, orc_mulmod(Pm, sph[(size_t)r * N + n], m), m);
                bo[n] = v;
                ao[n] = aj[n];
            }
        }
    }
    free(sh); free(sph); free(eh);
}

/* Secret-key encryption at `level`: c1 = a (uniform, given, NTT form), c0 = -a*s + e + m.
 * m, e, s signed coefficient vectors.  ct out [2][level+1][N] NTT form. */
void orc_encrypt(const orc_ctx* c, const int64_t* m, const int64_t* s, const u64* a, const int64_t* e,
                 uint32_t level, u64* ct) {
    uint32_t N = c->N, L1 = level + 1;
    uint32_t idx[ORC_MAXMOD];
    for (uint32_t r = 0; r < L1; r++) idx[r] = r;
    u64* sh = (u64*)malloc((size_t)L1 * N * sizeof(u64));
    int64_t* me = (int64_t*)malloc((size_t)N * sizeof(int64_t));
    for (uint32_t n = 0; n < N; n++) me[n] = m[n] + e[n];
    orc_reduce_signed(c, s, idx, L1, sh); orc_ntt(c, sh, idx, L1);
    orc_reduce_signed(c, me, idx, L1, ct); orc_ntt(c, ct, idx, L1);
    for (uint32_t r = 0; r < L1; r++)
        for (uint32_t n = 0; n < N; n++) {
            size_t i = (size_t)r * N + n;
            ct[i] = submod(ct[i], orc_mulmod(a[i], sh[i], c->mod[r]), c->mod[r]);
            ct[(size_t)L1 * N + i] = a[i];
        }
    free(sh); free(me);
}

/* Phase c0 + c1*s on the limbs listed (indices < level+1), returned in coefficient form
 * as canonical residues [n_limbs][N]. */
void orc_phase(const orc_ctx* c, const u64* ct, uint32_t level, const int64_t* s, const uint32_t* limbs,
               uint32_t n_limbs, u64* out) {
    uint32_t N = c->N, L1 = level + 1;
    for (uint32_t l = 0; l < n_limbs; l++) {
        uint32_t r = limbs[l];
        u64 q = c->mod[r];
        u64* sh = (u64*)malloc((size_t)N * sizeof(u64));
        orc_reduce_signed(c, s, &r, 1, sh); ntt_limb(c, r, sh);
        u64* o = out + (size_t)l * N;
        for (uint32_t n = 0; n < N; n++)
            o[n] = addmod(ct[(size_t)r * N + n], orc_mulmod(ct[((size_t)L1 + r) * N + n], sh[n], q), q);
        intt_limb(c, r, o);
        free(sh);
    }
}
