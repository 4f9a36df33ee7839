// Internal declarations shared by the translation units of the library (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <map>
#include <new>
#include <string>
#include <vector>

#include "../../include/he_mi355x.h"

typedef unsigned long long u64;
typedef unsigned __int128 u128;

#define HE_MAX_MODULI 64        // nq + np
#define HE_MAX_LAUNCH_LIMBS 512 // limbs described by one kernel-argument list

// Per-modulus constants, resident on the device (array indexed by modulus index).
struct ModConst {
    u64 q;          // the prime
    u64 q2;         // 2q
    u64 mu;         // floor(2^(bits+63) / q): Barrett constant for inputs < 2^(bits+63)
    u64 ninv;       // N^-1 mod q
    u64 ninv_sh;    // Shoup companion floor(ninv * 2^64 / q)
    u64 ninv_w;     // N^-1 * psi^-(N/2): scaling folded into the twiddle of the last inverse stage
    u64 ninv_w_sh;
    u64 one_sh;     // floor(2^64 / q): Shoup companion of the constant 1 (a quotient step for any 64-bit value)
    uint32_t bits;  // bit length of q
    uint32_t pad;
};

// Modulus index of each limb of a launch, passed by value in the kernel arguments.
struct LimbList {
    uint8_t mod[HE_MAX_LAUNCH_LIMBS];
};

// Optional per-limb output scaling of an inverse transform (replaces the plain N^-1).
struct ScaleList {
    u64 s[HE_MAX_MODULI];
    u64 s_sh[HE_MAX_MODULI];
    u64 w[HE_MAX_MODULI];      // s * psi^-(N/2) mod q (the last inverse stage's twiddle, pre-scaled)
    u64 w_sh[HE_MAX_MODULI];
};

struct ProfSpan {
    hipEvent_t e0, e1;
    uint32_t limbs;   // limbs transformed by the launch between the two events
    uint32_t digit_limbs; // raised-digit limbs a pass that carries the key-switch inner product has to read
    uint32_t kind;        // he_profile_t::pass_ms index: 0 fwd column, 1 fwd row, 2 fwd row + inner product/epilogue,
                          // 3 inv row, 4 inv row + inner product, 5 inv column
};

struct he_ctx {
    uint32_t logN, N, nq, np, dnum, alpha, M; // M = nq + np
    hipStream_t stream;
    int device;
    u64 mod[HE_MAX_MODULI];
    u64 psi[HE_MAX_MODULI];
    u64 itw1[HE_MAX_MODULI];    // psi^-(N/2), the single twiddle of inverse stage 0
    ModConst h_mc[HE_MAX_MODULI];
    // device tables
    ModConst* d_mc;    // [M]
    u64* d_tw;         // [M][N]  psi^bitrev(i)
    u64* d_tw_sh;      // [M][N]  Shoup companions
    u64* d_itw;        // [M][N]  psi^-bitrev(i)
    u64* d_itw_sh;     // [M][N]
    // basis-conversion tables (keyswitch.hip); present when np > 0
    u64* d_up_hat;     // [dnum][alpha][alpha][M]: (Q_j/q_i) mod m for digit j holding sz limbs, [j][sz-1][i][m]
    std::vector<u64> h_up_invhat; // [dnum][alpha][alpha]: ((Q_j/q_i)^-1 mod q_i), [j][sz-1][i]
    u64* d_dn_hat;     // [np][M]: (P/p_t) mod m  (only m < nq used)
    std::vector<u64> h_dn_invhat; // [np]: (P/p_t)^-1 mod p_t
    u64* d_pinv;       // [nq] P^-1 mod q_r
    u64* d_pinv_sh;    // [nq] Shoup companions
    // rescale tables: q_l^-1 mod q_r for r < l, [nq][nq]
    u64* d_qlinv;
    u64* d_qlinv_sh;
    // workspace (grown on demand)
    u64* d_ws;
    size_t ws_bytes;
    std::map<uint32_t, const u64*> evk; // Galois element -> device key
    he_counters_t cnt;
    bool prof_on;                       // time every transform launch with an event pair
    std::vector<ProfSpan> prof_events;
    uint64_t prof_key_limbs;            // key limbs the inner products had to read while timing was on (one pass per key per chunk)
    uint32_t cf_max_groups, cf_max_targets;   // N = 2^16 latency path: largest conversion (groups, targets per group) that takes the single-launch column kernel
    std::string err;
};

// ---- host helpers (ctx.hip)
int32_t he_fail(he_ctx* ctx, int32_t code, const char* fmt, ...);
int32_t he_ensure_ws(he_ctx* ctx, size_t bytes);
u64 h_mulmod(u64 a, u64 b, u64 m);
u64 h_powmod(u64 a, u64 e, u64 m);
u64 h_invmod(u64 a, u64 m);
u64 h_shoup(u64 w, u64 m);
uint32_t h_galois_of_step(const he_ctx* ctx, int32_t step);

// Every extern "C" body runs inside he_guard: no C++ exception (a failed host allocation in a
// std::vector / std::map / std::string) crosses the C ABI; it comes back as HE_ERR_ALLOC.
void he_fail_nothrow(he_ctx* ctx, const char* msg) noexcept;
template <class F>
static inline int32_t he_guard(const he_ctx* ctx, const char* who, F&& body) noexcept {
    try {
        return body();
    } catch (const std::bad_alloc&) {
        he_fail_nothrow(const_cast<he_ctx*>(ctx), who);
        return HE_ERR_ALLOC;
    } catch (...) {
        he_fail_nothrow(const_cast<he_ctx*>(ctx), who);
        return HE_ERR_ALLOC;
    }
}

#define HE_HIP(ctx, call)                                                                            \
    do {                                                                                             \
        hipError_t e__ = (call);                                                                     \
        if (e__ != hipSuccess) return he_fail(ctx, HE_ERR_HIP, "%s: %s", #call, hipGetErrorString(e__)); \
    } while (0)

int32_t he_noalloc_init_device(he_ctx* ctx, int device);   // noalloc.hip: address of the static scratch on this GPU

// ---- internal device-work launchers (all enqueue on ctx->stream, none synchronises)
#define HE_MAX_SEGS 16      // distinct source allocations one transform launch can read from
#define HE_MAX_KS_JOBS 16   // key-switch jobs whose ModDown runs in one set of launches

// Epilogue of ModDown fused into the last pass of the forward transform of the converted p-part
// (separate kernel on the generic path).  The launch covers J jobs x 2 components x L1 limbs:
// limb i -> job i/(2*L1), component (i/L1)&1, limb r = i%L1;
//   out_c[r] = (acc_c[r] - ntt) * P^-1  (+ c0[r] gathered by the Galois map of g for component 0)
//              (+ self_c[r], ungathered: the ciphertext itself for a rotate-and-sum step, the
//                 tensor-product parts d0, d1 for a relinearisation).
struct ModDownEpilogue {
    const u64* acc;      // [J][2][R][N]
    const u64* pinv;     // [nq]
    const u64* pinv_sh;
    uint32_t R, L1;
    const u64* c0[HE_MAX_KS_JOBS];      // [L1][N] or nullptr (plain key switch)
    const u64* self0[HE_MAX_KS_JOBS];   // [L1][N] or nullptr: added to out0 as is
    const u64* self1[HE_MAX_KS_JOBS];   // [L1][N] or nullptr: added to out1 as is
    u64* out0[HE_MAX_KS_JOBS];
    u64* out1[HE_MAX_KS_JOBS];
    uint32_t g[HE_MAX_KS_JOBS];
    // N = 2^16 path only.  fused != 0: the q-limbs of acc are never materialised; the epilogue computes
    // acc_c[r] = sum_j digit_j[r] (gathered by the Galois map) * evk_j,c[r] itself, digit j's own limbs
    // taken from the switched polynomial.  beta <= 8.
    uint32_t fused, beta, alpha, M;
    // n_terms > 0 (fused only): the launch serves ONE output whose accumulator is the sum over n_terms
    // (polynomial, Galois element, key) terms, a sum of rotations brought down by one ModDown; raised/own/evk/g
    // are then indexed by term, c0[0] must be null (the rotated c0 parts arrive summed through self0[0]).
    uint32_t n_terms;
    const u64* raised[HE_MAX_KS_JOBS];  // [beta][R][N]
    const u64* own[HE_MAX_KS_JOBS];     // [L1][N]
    const u64* evk[HE_MAX_KS_JOBS];     // [dnum][2][M][N]
};

// Key-switch inner product of the special-prime limbs computed by the first pass of their inverse transform
// (N = 2^16 path): limb i of the launch is job i/(2k), component (i/k)&1, special prime i%k; its input value at
// position n is sum_j raised_j[L1 + i%k][galois(n)] * evk_j,comp[nq + i%k][n] and is never stored.  beta <= 8.
struct IpPrologue {
    const u64* raised[HE_MAX_KS_JOBS];  // [beta][R][N]
    const u64* evk[HE_MAX_KS_JOBS];     // [dnum][2][M][N]
    uint32_t g[HE_MAX_KS_JOBS];
    uint32_t beta, R, M, L1, k, nq;
    uint32_t n_terms;                   // as in ModDownEpilogue: > 0 = one output, arrays indexed by term
};

// One batched transform launch (both passes).  Limb i is read at seg[src_seg[i]] + src_limb[i]*N
// by the first pass and lives at dst + i*N afterwards; mod_idx[i] == 0xFF leaves limb i alone.
struct TransformDesc {
    bool fwd;
    const u64* seg[HE_MAX_SEGS];
    uint32_t n_seg;
    u64* dst;
    uint32_t n;                  // <= HE_MAX_LAUNCH_LIMBS
    const uint32_t* mod_idx;     // [n]
    const uint8_t* src_seg;      // [n] or nullptr (all segment 0)
    const uint16_t* src_limb;    // [n] (< 4096) or nullptr (identity)
    const ScaleList* scale;      // inverse only: limb i is multiplied by scale[i % scale_period]
    uint32_t scale_period;       //   (must include N^-1); nullptr = plain N^-1
    const ModDownEpilogue* ep;   // forward only, or nullptr
    const IpPrologue* ip;        // inverse on the N = 2^16 path only, or nullptr: inputs are computed, not read
    bool lazy_out;               // forward only: outputs may stay unreduced (below 2^7 q) where the
                                 // consumers' 128-bit accumulations leave room; internal buffers only
    uint32_t only_pass;          // N = 2^16 path: 0 = both passes; 1 = the first pass only (inverse: rows, reading the
                                 // sources; forward: columns); 2 = the second pass only, in place at dst
    uint32_t rescale_from;       // N = 2^16 path, forward only: l + 1 when the sources are coefficient-form limbs of
                                 // modulus l and limb i (modulus r) transforms ((t + h) mod q_l) mod q_r - (h mod q_r),
                                 // h = floor(q_l / 2): the rounding term of Rescale, negated; 0 = sources as they are
};

// N = 2^16 latency path: [inverse column pass -> basis conversion -> forward column pass] of several groups in one launch.
// Group g: sources src + i*N (i < ns, moduli mod0 + i, output scaling sc entry sc0 + i) in the state the inverse row
// pass leaves them; targets of its set: target t has modulus tgt_mod[set][t] and is written, in the state the forward
// column pass leaves it, at dst + tgt_limb[set][t]*N; conversion constants hat[modulus*hat_w + i].
#define CF_MAX_GROUPS 32
#define CF_MAX_SETS 4
// Per-group fields are all 32 or 64 bits wide on purpose.  The group index is uniform, so the compiler reads these
// through scalar loads, and it is free to split an aligned address into a base register and an offset register
// that are each misaligned (it did, for byte-sized per-group arrays: base = args + g, offset = 7g).  The hardware
// drops the two low bits of each register separately, and the load then returns the wrong words.
struct CfGroup {
    const u64* src;
    u64* dst;
    const u64* hat;
    uint32_t ns, mod0, sc0, set;
};
struct ColFuse {
    CfGroup grp[CF_MAX_GROUPS];
    uint32_t hat_w, n_groups;
    uint32_t nt[CF_MAX_SETS];
    uint8_t tgt_limb[CF_MAX_SETS][HE_MAX_MODULI];     // indexed per wavefront: vector loads
    uint8_t tgt_mod[CF_MAX_SETS][HE_MAX_MODULI];
};
int32_t launch_colfuse(he_ctx* ctx, const ColFuse& cf, const ScaleList& sc, uint32_t limb_passes);   // ntt16.hip
// fills w / w_sh of entry i from s (modulus index mi)
void scale_entry(const he_ctx* c, ScaleList& sc, uint32_t i, uint32_t mi, u64 s);
int32_t launch_transform(he_ctx* ctx, const TransformDesc& d);
int32_t launch_transform16(he_ctx* ctx, const TransformDesc& d);   // N = 2^16 fast path
int32_t probe_butterfly_rates(he_ctx* ctx, u64* d_out, uint32_t groups, double rate_out[3]);   // ntt16.hip
int32_t launch_moddown_final(he_ctx* ctx, const u64* conv, uint32_t n_jobs, const ModDownEpilogue& ep);

// in-place conveniences
int32_t launch_ntt(he_ctx* ctx, u64* d, const uint32_t* mod_idx, uint32_t n);
int32_t launch_intt(he_ctx* ctx, u64* d, const uint32_t* mod_idx, uint32_t n, const ScaleList* scale);
int32_t launch_automorph_ntt(he_ctx* ctx, const u64* in, u64* out, uint32_t n_limbs, uint32_t g);
struct AffineConst {
    u64 mul[HE_MAX_MODULI], add[HE_MAX_MODULI];
};
int32_t launch_affine(he_ctx* ctx, const u64* ct, uint32_t level, const AffineConst& k, u64* out);   // out may alias ct
int32_t launch_tensor(he_ctx* ctx, const u64* a, const u64* b, uint32_t level, u64* d);   // d = [d0][d1][d2], each [level+1][N]
int32_t launch_automorph_coef(he_ctx* ctx, const u64* in, u64* out, const uint32_t* mod_idx, uint32_t n, uint32_t g);

// key switching engine (keyswitch.hip)
int32_t ks_init_tables(he_ctx* ctx);
void ks_free_tables(he_ctx* ctx);
struct KsSrc {
    const u64* c0;   // [level+1][N] or nullptr (plain key switch: nothing rotated is added to out0)
    const u64* c1;   // [level+1][N]: the polynomial that is raised and switched
    const u64* s0;   // [level+1][N] or nullptr: addends for jobs with add_self
    const u64* s1;
};
struct KsJob {
    uint32_t src;        // index into the sources
    uint32_t g;          // Galois element applied to the raised digits and to c0 (1 = none)
    const u64* evk;      // key used
    u64* out0;           // [level+1][N]
    u64* out1;
    uint32_t add_self;   // out0 += src.s0, out1 += src.s1 (rotate-and-sum step, relinearisation)
};
// Runs every job: one ModUp per source, then inner product + ModDown per job, batched.
int32_t ks_engine(he_ctx* ctx, uint32_t level, const KsSrc* srcs, uint32_t n_src, const KsJob* jobs, uint32_t n_jobs);
size_t ks_engine_ws_elems(const he_ctx* c, uint32_t level, uint32_t n_src, uint32_t n_jobs);
// Sum of rotations with one ModDown for the whole sum.  Terms with g == 1 are added as they are (evk unused).
#define HE_MAX_SUM_TERMS 49
struct KsSumTerm {
    const u64* c0;   // [level+1][N]
    const u64* c1;
    uint32_t g;
    const u64* evk;
};
size_t ks_rotate_sum_ws_elems(const he_ctx* c, uint32_t level, uint32_t n_rot);
int32_t ks_rotate_sum_deferred(he_ctx* c, uint32_t level, const KsSumTerm* terms, uint32_t n_terms, u64* out0, u64* out1, u64* ws);
// sum over T shared (Galois element, key) terms of the rotations of each of J ciphertexts, one ModUp and one ModDown per
// ciphertext; srcs[j] = {c0_j, c1_j, addend0_j or null, addend1_j or null} (keyswitch.hip)
size_t ks_hoisted_sum_ws_elems(const he_ctx* c, uint32_t level, uint32_t J, uint32_t T);
int32_t ks_hoisted_sum(he_ctx* c, uint32_t level, const KsSrc* srcs, uint32_t J, const uint32_t* gs, const u64* const* evks, uint32_t T,
                       u64* const* out0, u64* const* out1, u64* ws);
// Hoisted inner products kept over the raised basis, and the ModDown of stored accumulators (keyswitch.hip)
size_t ks_raised_products_ws_elems(const he_ctx* c, uint32_t level);
int32_t ks_raised_products(he_ctx* c, uint32_t level, const u64* c1, const uint32_t* gs, const u64* const* evks, uint32_t n, u64* acc, u64* ws);
size_t ks_moddown_stored_ws_elems(const he_ctx* c, uint32_t level, uint32_t J);
int32_t ks_moddown_stored(he_ctx* c, uint32_t level, uint32_t J, u64* acc, const u64* const* add0, const u64* const* add1,
                          u64* const* out0, u64* const* out1, u64* ws);
// Latency path for rings whose limb fits one work group's LDS (smallring.hip)
bool small_ring_path(const he_ctx* c, uint32_t level);
int32_t sr_modup(he_ctx* c, const KsSrc* srcs, uint32_t cb, uint32_t level, u64* raised);
int32_t sr_moddown(he_ctx* c, uint32_t level, uint32_t J, const ModDownEpilogue& ep);
int32_t sr_rescale(he_ctx* c, const u64* const* cts, u64* const* outs, uint32_t n, uint32_t level);
size_t rescale_ws_elems(const he_ctx* c, uint32_t level, uint32_t n);
int32_t rescale_batch(he_ctx* ctx, const u64* const* cts, u64* const* outs, uint32_t n, uint32_t level, u64* ws);
