/*
 * he_mi355x.h - C ABI of the MI355X (gfx950) library for the homomorphic convolution layer
 * over RNS-CKKS ciphertexts: slot rotations (Galois automorphism + hybrid key switching),
 * plaintext-ciphertext multiply-accumulate and rescale, all resting on batched negacyclic
 * NTT/iNTT over 64-bit RNS limbs.
 *
 * The paper (HyPHEN, arXiv 2302.02407) states the problem as sequences of RNS-CKKS
 * operations - CRot, MulPt, MulCt, AddCt, Rescale (Section 2.1, Table 1), assembled into SISO
 * convolution (Algorithm 1), rotate-and-sum (Section 2.2), channel-aligned convolution
 * CAConv (Section 3.1) and replication-aligned convolution RAConv in its reordered form
 * (Algorithm 2) - and takes the operations themselves from an RNS-CKKS library with
 * hybrid key switching (decomposition number dnum; Appendix, parameter sets).  Each entry
 * point below is one of those operations or one stage inside CRot.
 *
 * Conventions (all entry points)
 *  - Pointers named d_* are DEVICE pointers, h_* are HOST pointers.  The caller owns every
 *    buffer it passes; the context owns only its precomputed tables and its workspace.
 *  - A polynomial limb is N = 2^logN uint64 residues in [0, m) of one modulus m.  Buffers are
 *    limb-major: [poly][limb][N].  A ciphertext at level l is [2][l+1][N] (c0 then c1) over
 *    q_0..q_l.
 *  - "NTT form": position j holds the evaluation at psi^(2*bitrev(j)+1), psi the primitive
 *    2N-th root of the modulus given by he_ctx_psi.  Ciphertexts, plaintexts and keys are in
 *    NTT form unless a call says otherwise.
 *  - Modulus index space: 0..nq-1 = q_0..q_L (ciphertext primes), nq..nq+np-1 = special primes.
 *  - Every call returns HE_OK (0) or a negative he_status; he_last_error() gives the text.
 *    Calls never abort and never throw (a failed host allocation inside a call comes back as
 *    HE_ERR_ALLOC).  Work is enqueued on the context's HIP stream and is
 *    NOT synchronised on return unless stated.
 *  - A context is not thread-safe; calls on one context must not overlap (they share its
 *    workspace).
 */
#ifndef HE_MI355X_H
#define HE_MI355X_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct he_ctx he_ctx;

typedef enum {
    HE_OK = 0,
    HE_ERR_BADARG = -1, /* null pointer, size or index out of range, even Galois element ... */
    HE_ERR_LEVEL = -2,  /* level outside 0..L (or 1..L for rescale) */
    HE_ERR_NOKEY = -3,  /* no evaluation key registered for the Galois element */
    HE_ERR_ALLOC = -4,  /* device or host allocation failed */
    HE_ERR_HIP = -5     /* a HIP runtime call or kernel launch failed */
} he_status;

/* Operation counts since creation / last reset (paper: cost table of the convolutions counts
 * rotations per stage; these let a caller check CAConv issues f^2-1 Slide + n_o*log2(C_a) RaS
 * key switches and no other). */
typedef struct {
    uint64_t keyswitch;   /* key-switch inner products executed (one per rotation / relinearisation) */
    uint64_t modup;       /* digit decompositions (ModUp of one polynomial) */
    uint64_t ntt_limbs;   /* forward limb transforms */
    uint64_t intt_limbs;  /* inverse limb transforms */
    uint64_t mac;         /* plaintext-ciphertext products accumulated */
    uint64_t rescale;     /* ciphertext rescales */
    uint64_t automorph;   /* limb permutations (explicit calls and c0 of rotations) */
    uint64_t moddown;     /* ModDowns of an accumulator pair (equals keyswitch unless a sum of rotations shared one) */
} he_counters_t;

/* Geometry and operands of one channel-aligned convolution (paper Section 3.1, CAConv on the
 * data format pi_CA = {C_a, H, W, R_g}; slot(c,h,w,r) = ((c*H+h)*W+w)*R + r, C_a*H*W*R = N/2).
 * d_weights[o*f*f + t] is the filter plaintext of output ciphertext o and tap t (row-major
 * taps, dy outer, dx inner, both from -(f-1)/2), NTT form at `level`, [level+1][N]. */
typedef struct {
    uint32_t C_a, H, W, R;       /* slot layout of the input ciphertext */
    uint32_t f;                  /* odd filter width (1, 3, 5, ...) */
    uint32_t n_out;              /* number of output ciphertexts */
    uint32_t level;              /* level of the input; outputs are at level-1 */
    uint32_t skip_ras;           /* != 0: stop after the Rescale (no rotate-and-sum over C_a, no keys needed for it); the
                                    caller sums later with he_ras, e.g. after merging outputs into the stride gap */
    uint32_t deferred_taps;      /* != 0: Slide_f and MulFilter&Sum_f (Algorithm 1) share ONE ModDown per output: the
                                    hoisted key-switch inner products of the f^2-1 rotated taps stay over the raised
                                    basis q_0..q_level, p_0..p_{k-1}, the filter plaintexts multiply them there, and
                                    only each output's sum is brought down (the un-switched parts, plaintext times
                                    rotated c0 and the tap that does not rotate, are added over the ciphertext
                                    primes).  Every weight plaintext is then [level+1+k][N]: the same integer
                                    polynomial reduced modulo the ciphertext primes first, then the special primes.
                                    Same values up to rounding (one ModDown rounding per output instead of one per
                                    tap scaled by the plaintext), different bits; n_out ModDowns instead of f^2-1. */
    uint32_t hoisted_ras;        /* != 0: the rotate-and-sum over C_a (Section 2.2) is evaluated as the sum of the C_a-1
                                    rotations of each rescaled output by i*H*W*R slots (i = 1..C_a-1) plus the output
                                    itself, with ONE ModUp and ONE ModDown per output and every key shared by all
                                    outputs, instead of log2(C_a) dependent rotate-and-add steps.  Needs the C_a-1 keys
                                    (not only the log2(C_a) power-of-two ones); C_a <= 49.  Same sum, one ModDown
                                    rounding instead of log2(C_a); bits differ from the stepwise form. */
    const uint64_t* const* h_d_weights; /* host array of n_out*f*f device pointers */
} he_conv_plan;

/* Operands of one replication-aligned convolution in its reordered form (Section 3.1 RAConv,
 * Algorithm 2).  The n_in inputs are in the format CAConv leaves (every channel block holds
 * the same image); h_d_weights[i*f*f + t] is the filter plaintext of input i and tap t,
 * prepared rotated the opposite way to the tap (so that it can meet the input before the
 * rotation), NTT form at `level`, [level+1][N].  Tap (dy,dx) rotates by (dy*W+dx)*R slots. */
typedef struct {
    uint32_t n_in;               /* number of input ciphertexts */
    uint32_t W, R;               /* image row length and inner slot stride */
    uint32_t f;                  /* odd filter width */
    uint32_t level;              /* level of the inputs; the output is at level-1 */
    uint32_t deferred_moddown;   /* 0: every off-centre tap is rotated completely, then added; 1: Slide_1&Sum_f as
                                    he_rotate_sum with deferred != 0 (one ModDown for the sum of the f^2-1 rotations) */
    const uint64_t* const* h_d_weights; /* host array of n_in*f*f device pointers */
} he_raconv_plan;

/* Create a context: ring degree 2^logN (8 <= logN <= 17), ciphertext primes q[0..nq),
 * special primes p[0..np) (np may be 0 if no key switching is used), decomposition number
 * dnum (alpha = ceil(nq/dnum) limbs per digit, needs np >= 1 for key switching).  Every
 * modulus must be a prime = 1 mod 2N, 2^20 < m < 2^60, pairwise distinct.  Builds the root
 * tables (psi = c^((m-1)/2N), c the smallest quadratic non-residue of m), conversion
 * constants and a device workspace sized for level L.  hip_stream is a hipStream_t (NULL =
 * the default stream) on which all work of this context is enqueued.  Synchronises once. */
int32_t he_ctx_create(he_ctx** out, uint32_t logN, const uint64_t* h_q, uint32_t nq,
                      const uint64_t* h_p, uint32_t np, uint32_t dnum, void* hip_stream);
int32_t he_ctx_destroy(he_ctx* ctx);
/* Text of the last error on this context (ctx may be NULL: last creation error). */
const char* he_last_error(const he_ctx* ctx);
/* psi of modulus `mod_idx` (tests compare the root choice against their own). */
int32_t he_ctx_psi(const he_ctx* ctx, uint32_t mod_idx, uint64_t* h_psi_out);
int32_t he_counters(const he_ctx* ctx, he_counters_t* h_out);
int32_t he_counters_reset(he_ctx* ctx);
/* Timing of the transform kernels (the dominant kernels of every entry point) with a HIP event
 * pair around each launch on the context's stream.  he_profile_begin starts collecting;
 * he_profile_end synchronises the stream, sums the spans and stops.  transform_limb_passes
 * counts limbs per launch (a full NTT of one limb at N > 2^12 is two launches = two passes).
 * inner_product_digit_limbs counts the raised-digit limbs that passes carrying the key-switch
 * inner product have to read besides their own limb (N = 2^16 path; 0 elsewhere).
 * pass_* split the same launches by kind: 0 forward column pass, 1 forward row pass, 2 forward row
 * pass carrying the inner product of the q-limbs and the ModDown epilogue, 3 inverse row pass,
 * 4 inverse row pass computing the inner product of the special-prime limbs, 5 inverse column pass.
 * key_limbs_read counts the evaluation-key limbs the inner products had to read in the order the
 * engine ran them (one pass over a key per group of same-key jobs of a launch set). */
typedef struct {
    uint64_t transform_launches;
    uint64_t transform_limb_passes;
    uint64_t inner_product_digit_limbs;
    double transform_ms;
    uint64_t pass_launches[6];
    uint64_t pass_limbs[6];
    double pass_ms[6];
    uint64_t key_limbs_read;
} he_profile_t;
int32_t he_profile_begin(he_ctx* ctx);
int32_t he_profile_end(he_ctx* ctx, he_profile_t* h_out);
/* Vector-ALU roof of the transforms on this GPU, measured: radix-2 butterflies per second when the
 * register blocks of the N = 2^16 passes (Shoup twiddle product from 32-bit multiplies, lazy ranges)
 * run back to back out of registers: forward and inverse on the first ciphertext prime, forward on
 * the first modulus wider than 57 bits (0 if there is none).  Synchronises the stream. */
typedef struct {
    double fwd_butterflies_per_s;
    double inv_butterflies_per_s;
    double fwd_wide_butterflies_per_s;
} he_alu_probe_t;
int32_t he_probe_alu(he_ctx* ctx, he_alu_probe_t* h_out);
/* Identifies the build: hash of the library's sources taken when it was compiled (so that counter
 * summaries taken on one build are not quoted for another). */
const char* he_build_id(void);
/* Block until everything enqueued on the context's stream has finished. */
int32_t he_sync(he_ctx* ctx);

/* Workspace.  The context owns one device workspace.  It is sized at creation for every call that works
 * on one ciphertext at the top level (he_keyswitch, he_rotate, he_conjugate, he_rotate_hoisted, he_mulct,
 * he_rescale); the batched calls and the convolutions may need more and then grow it on entry, which
 * synchronises the stream, frees and reallocates.  To keep that out of a timed or latency-critical
 * region, ask the matching he_ws_query_* for the size (bytes, host output) and call he_ws_reserve once
 * beforehand.  he_ws_reserve never shrinks the workspace; he_ws_bytes reports its current size.
 * The queries return HE_ERR_LEVEL / HE_ERR_BADARG for shapes the call itself would refuse. */
int32_t he_ws_bytes(const he_ctx* ctx, uint64_t* h_bytes);
int32_t he_ws_reserve(he_ctx* ctx, uint64_t bytes);

/* Forward / inverse negacyclic NTT of n_limbs limbs in place (ring of Section 2.1).
 * d_data: [n_limbs][N]; h_mod_idx[i] = modulus index of limb i.  he_ntt: coefficient form in,
 * NTT form out; he_intt the inverse (including the factor N^-1).  Inputs must be canonical;
 * outputs are canonical. */
int32_t he_ntt(he_ctx* ctx, uint64_t* d_data, const uint32_t* h_mod_idx, uint32_t n_limbs);
int32_t he_intt(he_ctx* ctx, uint64_t* d_data, const uint32_t* h_mod_idx, uint32_t n_limbs);

/* Galois automorphism a(X) -> a(X^g) on every limb (the slot permutation inside CRot,
 * Section 2.1): g odd, 0 < g < 2N; g = 5^r mod 2N rotates slots left by r, g = 2N-1
 * conjugates.  ntt_form != 0: pure index permutation of NTT-form limbs; ntt_form == 0:
 * signed index map on coefficient-form limbs.  d_out must not overlap d_in. */
int32_t he_automorph(he_ctx* ctx, const uint64_t* d_in, uint64_t* d_out, const uint32_t* h_mod_idx,
                     uint32_t n_limbs, uint32_t galois_elt, int32_t ntt_form);

/* Register the evaluation key that switches sigma_g(s) -> s (galois_elt = g) or s^2 -> s
 * (galois_elt = 0).  d_evk: [dnum][2][nq+np][N] NTT form, component 0 = b, 1 = a, limb order
 * q_0..q_L, p_0..p_{k-1}; digit j carries P*s' on the q-limbs j*alpha..(j+1)*alpha-1.  Every
 * residue must be canonical (below its modulus): the inner products split key values in halves
 * and do not reduce them first; the buffer is not checked.  The caller keeps the buffer alive
 * and unchanged while it is registered; registering again replaces the pointer. */
int32_t he_evk_register(he_ctx* ctx, uint32_t galois_elt, const uint64_t* d_evk);

/* Hybrid key switching of one polynomial (the inner step of CRot and of relinearisation;
 * paper Appendix, evaluation keys and dnum): d_in [level+1][N] NTT form;
 * (d_out0, d_out1), each [level+1][N], satisfy out0 + out1*s = in*s' + small error for the
 * key registered under galois_elt_of_key.  Steps: ModUp of each digit (iNTT, fast basis
 * conversion without overflow correction, NTT), inner product with the key over
 * q_0..q_level,p_*, ModDown (conversion of the p-part without rounding term, times P^-1).
 * No automorphism is applied.  The outputs must not overlap the input or each other. */
int32_t he_keyswitch(he_ctx* ctx, const uint64_t* d_in, uint32_t level, uint32_t galois_elt_of_key,
                     uint64_t* d_out0, uint64_t* d_out1);

/* Rotations of one ciphertext by several slot amounts sharing a single ModUp of c1 (what
 * Slide_f of Algorithm 1 needs: all f^2 rotations of one input).  d_ct [2][level+1][N];
 * h_steps[i] = left-rotation amount (negative = right; reduced mod N/2; 0 = plain copy, no
 * key needed); h_d_out[i] = device buffer [2][level+1][N] for rotation i (must not overlap
 * d_ct or each other).  Per step with g = 5^step: acc = sum_j sigma_g(raised_j) * evk_g,j;
 * (ks0, ks1) = ModDown(acc); out = (sigma_g(c0) + ks0, ks1). */
int32_t he_rotate_hoisted(he_ctx* ctx, const uint64_t* d_ct, uint32_t level, const int32_t* h_steps,
                          uint32_t n_steps, uint64_t* const* h_d_out);
/* Batched CRot: every ciphertext h_d_ct[c] (c < n_ct, all [2][level+1][N] at `level`) rotated by
 * every amount h_steps[s] (s < n_steps); h_d_out[c*n_steps + s] receives CRot(ct_c; steps_s).
 * hoisted != 0: one ModUp per ciphertext shared by its n_steps rotations; hoisted == 0: one ModUp
 * per rotation (the cost of n_ct*n_steps independent CRot calls; the results are the same bits).
 * Launches are shared across the batch and rotations that use the same key share one pass over
 * it.  No output may overlap an input or another output.  Workspace grows with the batch. */
int32_t he_rotate_batch(he_ctx* ctx, const uint64_t* const* h_d_ct, uint32_t n_ct, uint32_t level,
                        const int32_t* h_steps, uint32_t n_steps, uint64_t* const* h_d_out, int32_t hoisted);
int32_t he_ws_query_rotate_batch(const he_ctx* ctx, uint32_t level, uint32_t n_ct, uint32_t n_steps, int32_t hoisted,
                                 uint64_t* h_bytes);
/* Slide_1 & Sum_f of Algorithm 2: d_out = sum over t < n_ct of CRot(h_d_ct[t]; h_steps[t]), all ciphertexts
 * [2][level+1][N] at `level` (a step of 0 adds the ciphertext as it is), 1 <= n_ct <= 49; d_out must not overlap an
 * input.  deferred == 0: every rotation is completed on its own (same bits as he_rotate followed by he_add).
 * deferred != 0: the rotations share ONE ModDown - each term's raised digits are multiplied into its key, the
 * products are summed over q_0..q_level,p_*, and the sum is brought down once; out0 also gets the sum of the rotated c0
 * parts.  The result encrypts the same sum with one ModDown's rounding instead of one per rotation, and differs in
 * bits from the deferred == 0 result.  Terms that rotate the same ciphertext (the same pointer) share its ModUp.
 * Grows the workspace with n_ct (all raised digits are live at once). */
int32_t he_rotate_sum(he_ctx* ctx, const uint64_t* const* h_d_ct, uint32_t n_ct, uint32_t level, const int32_t* h_steps,
                      uint64_t* d_out, int32_t deferred);
/* CRot(ct; step): identical bits to he_rotate_hoisted with n_steps = 1. */
int32_t he_rotate(he_ctx* ctx, const uint64_t* d_ct, uint32_t level, int32_t step, uint64_t* d_out);
/* Slot-wise complex conjugation (Galois element 2N-1, key registered under 2N-1). */
int32_t he_conjugate(he_ctx* ctx, const uint64_t* d_ct, uint32_t level, uint64_t* d_out);

/* MulPt + AddCt (MulFilter&Sum_f of Algorithm 1, one tap): acc.c0 (+)= ct.c0*pt,
 * acc.c1 (+)= ct.c1*pt, slot-wise per limb.  d_acc, d_ct [2][level+1][N]; d_pt [level+1][N];
 * init != 0 overwrites d_acc instead of accumulating.  d_acc may not overlap d_ct / d_pt. */
int32_t he_ptct_mac(he_ctx* ctx, uint64_t* d_acc, const uint64_t* d_ct, const uint64_t* d_pt,
                    uint32_t level, int32_t init);

/* d_acc (= | +=) sum_{i<n} ct_i * sigma_{g_i}(pt_i): MulPt-accumulate with each plaintext rotated as it is read (PRot
 * of Table 1 fused into the product, no key involved).  This is the operation PRCR needs (paper Section 3.3: a
 * weight plaintext whose fragments are arranged circularly is reused through plaintext rotations instead of being
 * stored once per use).  h_d_ct[i] [2][level+1][N] and h_d_pt[i] [level+1][N] are device pointers in host arrays,
 * NTT form; h_galois[i] is odd and below 2N (1 = no rotation; 5^step mod 2N rotates the slots left by step).
 * init != 0 overwrites d_acc, else accumulates into its canonical contents.  d_acc may not overlap
 * any operand (HE_ERR_BADARG).  n = 0 with init != 0 clears d_acc. */
int32_t he_ptct_mac_rot(he_ctx* ctx, uint64_t* d_acc, const uint64_t* const* h_d_ct, const uint64_t* const* h_d_pt,
                        const uint32_t* h_galois, uint32_t n, uint32_t level, int32_t init);
/* AddCt: d_out = d_a + d_b on [2][level+1][N]; d_out may alias d_a or d_b. */
int32_t he_add(he_ctx* ctx, const uint64_t* d_a, const uint64_t* d_b, uint32_t level, uint64_t* d_out);

/* AddPt (Section 2.1): d_out.c0 = d_ct.c0 + d_pt slot-wise per limb, d_out.c1 = d_ct.c1.  d_ct, d_out
 * [2][level+1][N]; d_pt [level+1][N] at the scale of the ciphertext; d_out may alias d_ct. */
int32_t he_addpt(he_ctx* ctx, const uint64_t* d_ct, const uint64_t* d_pt, uint32_t level, uint64_t* d_out);

/* MulCt (Section 2.1): ciphertext-ciphertext multiplication = slot-wise tensor product
 * d0 = a0*b0, d1 = a0*b1 + a1*b0, d2 = a1*b1 followed by relinearisation of d2 with the key
 * registered under Galois element 0 (s^2 -> s): out = (d0 + ks0, d1 + ks1).  d_a, d_b, d_out:
 * [2][level+1][N]; d_out may alias d_a or d_b.  The level is unchanged (the caller rescales);
 * the scale is the product of the input scales. */
int32_t he_mulct(he_ctx* ctx, const uint64_t* d_a, const uint64_t* d_b, uint32_t level, uint64_t* d_out);
/* Slot-wise affine map with constants: out_c[r] = ct_c[r]*h_mul[r] (+ h_add[r] at every position of
 * c0; a constant polynomial has a constant NTT).  h_mul, h_add: level+1 canonical residues (host).
 * Covers negation (q_r - 1), multiplication by an integer constant, and AddPt of a constant.
 * d_out may alias d_ct. */
int32_t he_affine(he_ctx* ctx, const uint64_t* d_ct, uint32_t level, const uint64_t* h_mul,
                  const uint64_t* h_add, uint64_t* d_out);

/* Rescale (Section 2.1): divide by q_level with exact rounding (half up) per coefficient and
 * drop that limb: d_ct [2][level+1][N] -> d_out [2][level][N], 1 <= level <= L. */
int32_t he_rescale(he_ctx* ctx, const uint64_t* d_ct, uint32_t level, uint64_t* d_out);

/* he_rescale for callers that cannot allocate device memory - code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc/hipFree.  Same arguments, same result bit for bit; its
 * scratch ((2 + 2*level) * N residues) lives in a static device array of HE_NOALLOC_SCRATCH_BYTES that
 * each GPU the library runs on holds until the process ends, instead of in the context's workspace.
 * The call allocates and frees nothing on the device and never synchronises.  Levels whose scratch
 * exceeds the array (level > 15 at N = 2^16) are refused with HE_ERR_BADARG, as is a call while
 * he_profile_begin is active (launch timing creates events).  The context's device must be the current
 * device.  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 * streams, two contexts, two threads) race; serialise them.  Nothing in the array has to survive or be
 * cleared between calls. */
#define HE_NOALLOC_SCRATCH_BYTES (16u << 20)
int32_t he_rescale_noalloc(he_ctx* ctx, const uint64_t* d_ct, uint32_t level, uint64_t* d_out);

/* Channel-aligned convolution CAConv (Section 3.1; Algorithm 1 for Slide_f and
 * MulFilter&Sum_f): Slide_f = hoisted rotations by (dy*W+dx)*R for the f^2 taps; for each
 * output o: sum over taps of rotated input * weight plaintext, Rescale, then rotate-and-sum
 * over C_a with amounts H*W*R*2^t, t < log2(C_a).  d_ct_in [2][level+1][N];
 * h_d_ct_out[o] = device buffer [2][level][N].  Needs keys for every non-zero tap amount and
 * every rotate-and-sum amount.  Grows the context workspace on first use (allocates). */
int32_t he_conv2d(he_ctx* ctx, const he_conv_plan* plan, const uint64_t* d_ct_in, uint64_t* const* h_d_ct_out);
int32_t he_ws_query_conv2d(const he_ctx* ctx, const he_conv_plan* plan, uint64_t* h_bytes);

/* Rotate-and-sum on a batch of ciphertexts (Section 2.2 RaS_{c_i}; Section 3.2 and the cost table of Section 3.1
 * for the sums and re-replications inside the gap, RaS_g / IR_g): for every step s in the order given,
 * ct <- ct + CRot(ct; h_steps[s]), applied to the n_ct ciphertexts h_d_ct[i] ([2][level+1][N]) at once (one launch
 * set per step; the ciphertexts share the step's key pass); results in h_d_out[i], inputs unchanged.  No output may
 * overlap an input or another output.  n_ct*n_steps key switches.  Grows the workspace with n_ct. */
int32_t he_ras(he_ctx* ctx, const uint64_t* const* h_d_ct, uint32_t n_ct, uint32_t level, const int32_t* h_steps,
               uint32_t n_steps, uint64_t* const* h_d_out);

/* Replication-aligned convolution, reordered (Section 3.1; Algorithm 2): MulFilter&Sum_ci -
 * for every tap the sum over the n_in inputs of input x inversely rotated filter plaintext
 * (additions only) - then Slide_1&Sum_f - one rotation per off-centre tap (f^2-1 in all) and
 * additions - then one Rescale.  h_d_ct_in[i] = device buffer [2][level+1][N]; d_ct_out
 * [2][level][N], must not overlap an input.  Needs keys for every non-zero tap amount.
 * Grows the context workspace on first use (allocates). */
int32_t he_raconv(he_ctx* ctx, const he_raconv_plan* plan, const uint64_t* const* h_d_ct_in, uint64_t* d_ct_out);
int32_t he_ws_query_raconv(const he_ctx* ctx, const he_raconv_plan* plan, uint64_t* h_bytes);

/* Fused CAConv -> Square -> RAConv block (Algorithm 3; Section 3.1 for the two convolutions, Section 3.4 for
 * the square activation).  n_ca channel-aligned ciphertexts in (input k holds channels k*C_a .. (k+1)*C_a-1, one
 * per block, R replicas each), n_ca channel-aligned ciphertexts out (output l holds output channels
 * l*C_a .. (l+1)*C_a-1; with R > 1 replica position r holds the partial sum over the intermediate channels of
 * class r, as he_raconv leaves it), n_ra replication-aligned ciphertexts in between (intermediate j carries
 * channel (j*R + r) mod c_mid in replica r).  Order of operations, as the algorithm states it: Slide_f of every
 * input; then for the intermediates, `group` at a time, MulFilter&Sum_f over all inputs and taps, Rescale,
 * rotate-and-sum over C_a, multiplication by the integer k_in (the lift to the square's working scale; its
 * residues per limb are given), Square = MulCt with itself + Rescale, and MulFilter&Sum_ci of the result into
 * the f^2 accumulators of every output ("forwarding": only the n_ca*f^2 rotated inputs and the n_ca*f^2
 * accumulators stay alive, plus `group` intermediates); finally Slide_1&Sum_f and Rescale per output.
 * group = 1 is the algorithm's loop exactly; larger groups batch the launches of several intermediates (0 or
 * >= n_ra: all at once).  Every group size gives the same bits.  Inputs [2][level+1][N] at `level` >= 3, outputs
 * [2][level-2][N] at level-3.  h_d_w_ca[(j*n_ca + k)*f*f + t]: filter plaintext of (intermediate j, input k,
 * tap t) at `level`; h_d_w_ra[(l*n_ra + j)*f*f + t]: inversely rotated filter plaintext of (output l,
 * intermediate j, tap t) at level-2.  Needs the keys of the tap rotations, of the rotate-and-sum amounts
 * H*W*R*2^t and the relinearisation key (Galois element 0).  Outputs must not overlap inputs. */
typedef struct {
    uint32_t C_a, H, W, R;
    uint32_t f;
    uint32_t n_ca, n_ra;
    uint32_t level;
    uint32_t group;
    uint32_t deferred_moddown;   /* Slide_1&Sum_f with one ModDown per output (see he_rotate_sum) */
    uint32_t hoisted_ras;        /* rotate-and-sum over C_a as one hoisted sum per intermediate (see he_conv_plan); needs
                                    the keys of i*H*W*R for every i < C_a */
    const uint64_t* h_k_in;      /* `level` canonical residues: k_in mod q_0 .. q_(level-1) */
    const uint64_t* const* h_d_w_ca;
    const uint64_t* const* h_d_w_ra;
} he_block_plan;
int32_t he_ca_ra_block(he_ctx* ctx, const he_block_plan* plan, const uint64_t* const* h_d_ct_in, uint64_t* const* h_d_ct_out);
int32_t he_ws_query_ca_ra_block(const he_ctx* ctx, const he_block_plan* plan, uint64_t* h_bytes);

#ifdef __cplusplus
}
#endif
#endif /* HE_MI355X_H */
