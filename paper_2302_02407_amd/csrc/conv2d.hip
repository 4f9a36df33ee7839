// Channel-aligned convolution CAConv (paper Section 3.1) assembled from Slide_f and
// MulFilter&Sum_f (Algorithm 1), Rescale (Section 2.1) and rotate-and-sum over C_a
// (Section 2.2), and replication-aligned convolution RAConv in its reordered form
// (Algorithm 2), all enqueued on the context's stream with no host synchronisation.
#include <algorithm>

#include "modarith.h"

#define CV_THREADS 256
#define CV_MAX_TAPS 49

#define CV_MAX_OUT_PER_LAUNCH 16

struct MacTaps {
    const u64* ct[CV_MAX_TAPS];                          // rotated inputs [2][CL][N]
    uint32_t n_taps, n_out;
    uint32_t c1_tap;                                     // 0xFFFFFFFF: every tap has both components; else only this tap
                                                         // has a second component (the others are [CL][N])
    u64* acc[CV_MAX_OUT_PER_LAUNCH];                     // one accumulator [2][CL][N] per output
};
struct MacWeights {
    const u64* pt[CV_MAX_OUT_PER_LAUNCH * 9];            // [out][tap] filter plaintexts [L1][N] (9-tap fast path)
};

// MulFilter&Sum_f for several output ciphertexts at once (9 taps or fewer): the rotated inputs of a
// coefficient are loaded once and reused for every output, acc_o,c[limb] = sum_t ct_t,c[limb] *
// pt_o,t[limb], summed in 128 bits and reduced once per 8 taps.  grid: (N/256, CL).  Operands and outputs have CL
// limbs per component: the level+1 ciphertext primes, followed by the special primes when the operands are
// key-switch inner products still over the raised basis (CL = level+1+k).
__global__ __launch_bounds__(CV_THREADS) void mac_taps9_kernel(MacTaps taps, MacWeights w, const ModConst* mc, uint32_t logN,
                                                               uint32_t CL, uint32_t level, uint32_t nq) {
    const uint32_t n = blockIdx.x * CV_THREADS + threadIdx.x;
    const uint32_t limb = blockIdx.y;
    const ModConst m = mc[limb <= level ? limb : nq + (limb - level - 1)];
    const size_t o0 = ((size_t)limb << logN) + n, o1 = ((size_t)(limb + CL) << logN) + n;
    u64 c0[9], c1[9];
#pragma unroll
    for (uint32_t t = 0; t < 9; t++) {
        c0[t] = t < taps.n_taps ? taps.ct[t][o0] : 0;
        c1[t] = (t < taps.n_taps && (taps.c1_tap == 0xFFFFFFFFu || taps.c1_tap == t)) ? taps.ct[t][o1] : 0;
    }
    for (uint32_t o = 0; o < taps.n_out; o++) {
        u128 a0 = 0, a1 = 0;
#pragma unroll
        for (uint32_t t = 0; t < 9; t++) {
            if (t == 8) {
                a0 = barrett128(a0, m.q, m.mu, m.bits);
                a1 = barrett128(a1, m.q, m.mu, m.bits);
            }
            if (t < taps.n_taps) {
                u64 p = w.pt[o * 9 + t][o0];
                a0 += (u128)c0[t] * p;
                a1 += (u128)c1[t] * p;
            }
        }
        taps.acc[o][o0] = barrett128(a0, m.q, m.mu, m.bits);
        taps.acc[o][o1] = barrett128(a1, m.q, m.mu, m.bits);
    }
}

struct MacTapsAny {
    const u64* ct[CV_MAX_TAPS];
    const u64* pt[CV_MAX_TAPS];
    uint32_t n, init;
    uint32_t c1_tap;                                     // as in MacTaps
};
// Any number of (ciphertext, plaintext) products, one output per launch; init = 0 continues from the
// accumulator's current (canonical) contents.  CL, level, nq as in mac_taps9_kernel.
__global__ __launch_bounds__(CV_THREADS) void mac_taps_kernel(MacTapsAny taps, u64* __restrict__ acc, const ModConst* mc,
                                                              uint32_t logN, uint32_t CL, uint32_t level, uint32_t nq) {
    const uint32_t n = blockIdx.x * CV_THREADS + threadIdx.x;
    const uint32_t limb = blockIdx.y;
    const ModConst m = mc[limb <= level ? limb : nq + (limb - level - 1)];
    const size_t o0 = ((size_t)limb << logN) + n, o1 = ((size_t)(limb + CL) << logN) + n;
    u128 a0 = taps.init ? 0 : acc[o0], a1 = taps.init ? 0 : acc[o1];
    for (uint32_t t = 0; t < taps.n; t++) {
        if (t && (t & 7) == 0) {
            a0 = barrett128(a0, m.q, m.mu, m.bits);
            a1 = barrett128(a1, m.q, m.mu, m.bits);
        }
        u64 p = taps.pt[t][o0];
        a0 += (u128)taps.ct[t][o0] * p;
        if (taps.c1_tap == 0xFFFFFFFFu || taps.c1_tap == t) a1 += (u128)taps.ct[t][o1] * p;
    }
    acc[o0] = barrett128(a0, m.q, m.mu, m.bits);
    acc[o1] = barrett128(a1, m.q, m.mu, m.bits);
}

// Slot amounts of the f^2 taps (dy outer, dx inner, both from -(f-1)/2), reduced to [0, slots).
static std::vector<uint32_t> tap_slot_steps(uint32_t W, uint32_t R, uint32_t f, uint32_t slots) {
    std::vector<uint32_t> steps(f * f);
    const int32_t half = (int32_t)(f - 1) / 2;
    for (uint32_t t = 0; t < f * f; t++) {
        const int32_t dy = (int32_t)(t / f) - half, dx = (int32_t)(t % f) - half;
        int64_t step = ((int64_t)dy * W + dx) * R;
        steps[t] = (uint32_t)(((step % (int64_t)slots) + slots) % slots);
    }
    return steps;
}

// he_conv2d workspace: [key-switch engine region][rescale scratch][rotated inputs][n_out accumulators at `level`]
// [n_out temporaries at level-1]
// With the ModDown deferred across the taps the rotated inputs are replaced by (at the start of the region, where the
// engine's scratch of the rotate-and-sum steps lives later): [ModUp scratch][n_rot inner products over the raised
// basis][accumulators of one chunk of outputs over the raised basis][ModDown scratch][n_rot rotated c0][the chunk's
// plain parts].
static size_t conv2d_deferred_elems(const he_ctx* ctx, uint32_t level, uint32_t n_rot, uint32_t n_out) {
    const size_t N = ctx->N, L1 = level + 1, R = L1 + ctx->np, nb = std::min<uint32_t>(n_out, HE_MAX_KS_JOBS);
    return ks_raised_products_ws_elems(ctx, level) + (size_t)n_rot * 2 * R * N + nb * 2 * R * N + ks_moddown_stored_ws_elems(ctx, level, (uint32_t)nb) +
           (size_t)n_rot * L1 * N + nb * 2 * L1 * N;
}
static size_t conv2d_ws_elems(const he_ctx* ctx, uint32_t level, uint32_t n_rot, uint32_t n_out, bool deferred_taps = false,
                              uint32_t hoisted_ras_terms = 0) {
    const size_t N = ctx->N, ct_e = (size_t)2 * (level + 1) * N, ct_lo_e = (size_t)2 * level * N;
    // scratch of the rotate-and-sum stage: the engine's (one step at a time) or the hoisted sum's
    const size_t ras_e = hoisted_ras_terms ? ks_hoisted_sum_ws_elems(ctx, level - 1, n_out, hoisted_ras_terms)
                                           : ks_engine_ws_elems(ctx, level - 1, n_out, n_out);
    if (deferred_taps && n_rot) {
        const size_t head = std::max(conv2d_deferred_elems(ctx, level, n_rot, n_out), ras_e);
        return head + rescale_ws_elems(ctx, level, n_out) + (size_t)n_out * ct_e + (size_t)n_out * ct_lo_e;
    }
    const size_t ks_e = std::max(n_rot ? ks_engine_ws_elems(ctx, level, 1, n_rot) : 0, ras_e);
    return ks_e + rescale_ws_elems(ctx, level, n_out) + (size_t)(n_rot + n_out) * ct_e + (size_t)n_out * ct_lo_e;
}
// terms of the hoisted rotate-and-sum of a plan (0: the log2 C_a dependent steps are used)
static uint32_t hoisted_ras_terms(const he_conv_plan* plan) {
    return (plan->hoisted_ras && !plan->skip_ras && plan->C_a > 1) ? plan->C_a - 1 : 0;
}

extern "C" int32_t he_ws_query_conv2d(const he_ctx* ctx, const he_conv_plan* plan, uint64_t* h_bytes) {
    return he_guard(ctx, "he_ws_query_conv2d: host allocation failed", [&]() -> int32_t {
    if (!ctx || !plan || !h_bytes) return HE_ERR_BADARG;
    if (plan->level == 0 || plan->level >= ctx->nq) return HE_ERR_LEVEL;
    if ((plan->f & 1u) == 0 || plan->f * plan->f > CV_MAX_TAPS || plan->n_out == 0) return HE_ERR_BADARG;
    uint32_t n_rot = 0;
    for (uint32_t st : tap_slot_steps(plan->W, plan->R, plan->f, ctx->N / 2)) n_rot += st != 0;
    *h_bytes = conv2d_ws_elems(ctx, plan->level, n_rot, plan->n_out, plan->deferred_taps != 0, hoisted_ras_terms(plan)) * sizeof(u64);
    return HE_OK;
    });
}

extern "C" int32_t he_conv2d(he_ctx* ctx, const he_conv_plan* plan, const uint64_t* d_ct_in, uint64_t* const* h_d_ct_out) {
    return he_guard(ctx, "he_conv2d: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (!plan || !d_ct_in || !h_d_ct_out || !plan->h_d_weights) return he_fail(ctx, HE_ERR_BADARG, "he_conv2d: null argument");
    const uint32_t N = ctx->N, slots = N / 2, level = plan->level, f = plan->f, taps = f * f;
    if (ctx->np == 0) return he_fail(ctx, HE_ERR_BADARG, "he_conv2d: context has no special primes");
    if (level == 0 || level >= ctx->nq) return he_fail(ctx, HE_ERR_LEVEL, "he_conv2d: level %u outside 1..%u", level, ctx->nq - 1);
    if ((f & 1u) == 0 || taps > CV_MAX_TAPS) return he_fail(ctx, HE_ERR_BADARG, "he_conv2d: filter width %u must be odd and at most 7", f);
    if (plan->C_a == 0 || (plan->C_a & (plan->C_a - 1))) return he_fail(ctx, HE_ERR_BADARG, "he_conv2d: C_a must be a power of two");
    if ((u64)plan->C_a * plan->H * plan->W * plan->R != slots) return he_fail(ctx, HE_ERR_BADARG, "he_conv2d: C_a*H*W*R must equal N/2");
    if (plan->n_out == 0) return he_fail(ctx, HE_ERR_BADARG, "he_conv2d: n_out is zero");
    const uint32_t L1 = level + 1;
    // rotation amounts: Slide_f taps (dy outer, dx inner) and rotate-and-sum over C_a
    std::vector<uint32_t> tap_g(taps), ras_g;
    std::vector<const u64*> tap_key(taps, nullptr), ras_key;
    const int32_t half = (int32_t)(f - 1) / 2;
    for (uint32_t t = 0; t < taps; t++) {
        int32_t dy = (int32_t)(t / f) - half, dx = (int32_t)(t % f) - half;
        int64_t step = ((int64_t)dy * plan->W + dx) * plan->R;
        step = ((step % (int64_t)slots) + slots) % slots;
        tap_g[t] = h_galois_of_step(ctx, (int32_t)step);
        if (tap_g[t] != 1) {
            auto it = ctx->evk.find(tap_g[t]);
            if (it == ctx->evk.end()) return he_fail(ctx, HE_ERR_NOKEY, "he_conv2d: no key for tap rotation %lld", (long long)step);
            tap_key[t] = it->second;
        }
    }
    const uint32_t ras_T = hoisted_ras_terms(plan);
    if (ras_T > HE_MAX_SUM_TERMS - 1) return he_fail(ctx, HE_ERR_BADARG, "he_conv2d: hoisted_ras supports C_a up to %d", HE_MAX_SUM_TERMS);
    for (uint32_t s = 1; s < plan->C_a && !plan->skip_ras; s = ras_T ? s + 1 : s << 1) {
        uint32_t step = plan->H * plan->W * plan->R * s;
        uint32_t g = h_galois_of_step(ctx, (int32_t)step);
        auto it = ctx->evk.find(g);
        if (it == ctx->evk.end()) return he_fail(ctx, HE_ERR_NOKEY, "he_conv2d: no key for rotate-and-sum amount %u", step);
        ras_g.push_back(g);
        ras_key.push_back(it->second);
    }
    for (uint32_t i = 0; i < plan->n_out * taps; i++)
        if (!plan->h_d_weights[i]) return he_fail(ctx, HE_ERR_BADARG, "he_conv2d: weight plaintext %u is null", i);
    for (uint32_t o = 0; o < plan->n_out; o++)
        if (!h_d_ct_out[o]) return he_fail(ctx, HE_ERR_BADARG, "he_conv2d: output %u is null", o);
    const uint32_t lo = level - 1;                       // level after the rescale
    const uint32_t n_out = plan->n_out, n_ras = (uint32_t)ras_g.size();
    uint32_t n_rot = 0;
    for (uint32_t t = 0; t < taps; t++) n_rot += tap_g[t] != 1;
    const size_t ct_e = (size_t)2 * L1 * N, ct_lo_e = (size_t)2 * level * N;
    const bool deferred_taps = plan->deferred_taps != 0 && n_rot > 0;
    if (deferred_taps && n_rot + 1 != taps)
        return he_fail(ctx, HE_ERR_BADARG, "he_conv2d: deferred_taps needs exactly one tap that does not rotate (%u of %u do)", taps - n_rot, taps);
    const size_t total = conv2d_ws_elems(ctx, level, n_rot, n_out, deferred_taps, ras_T);
    int32_t rc = he_ensure_ws(ctx, total * sizeof(u64));
    if (rc != HE_OK) return rc;
    // laid out from the end of the region: [engine ...][rescale scratch][rotated inputs][accumulators][temporaries]
    u64* tmp = ctx->d_ws + total - (size_t)n_out * ct_lo_e;  // [n_out] ciphertexts at level lo
    u64* acc = tmp - (size_t)n_out * ct_e;                   // [n_out] ciphertexts at `level`
    u64* slid = acc - (size_t)(deferred_taps ? 0 : n_rot) * ct_e;   // [n_rot] rotated inputs
    u64* rs_ws = slid - rescale_ws_elems(ctx, level, n_out);
    const u64* ct_in = (const u64*)d_ct_in;

    if (deferred_taps) {
        // Slide_f and MulFilter&Sum_f with one ModDown per output: the plaintexts (given over the raised basis)
        // multiply the hoisted inner products before these are brought down
        const uint32_t k = ctx->np, R = L1 + k;
        u64* prod_ws = ctx->d_ws;
        u64* A = prod_ws + ks_raised_products_ws_elems(ctx, level);              // [n_rot][2][R][N]
        const uint32_t nb_max = std::min<uint32_t>(n_out, HE_MAX_KS_JOBS);
        u64* ACC = A + (size_t)n_rot * 2 * R * N;                                // [nb][2][R][N]
        u64* md_ws = ACC + (size_t)nb_max * 2 * R * N;
        u64* rot0 = md_ws + ks_moddown_stored_ws_elems(ctx, level, nb_max);      // [n_rot][L1][N]
        u64* plain = rot0 + (size_t)n_rot * L1 * N;                              // [nb][2][L1][N]
        std::vector<uint32_t> gs, rot_tap;                                       // the rotated taps, in tap order
        std::vector<const u64*> keys;
        uint32_t centre = 0xFFFFFFFFu;
        for (uint32_t t = 0; t < taps; t++) {
            if (tap_g[t] == 1) { centre = t; continue; }
            gs.push_back(tap_g[t]); keys.push_back(tap_key[t]); rot_tap.push_back(t);
        }
        rc = ks_raised_products(ctx, level, ct_in + (size_t)L1 * N, gs.data(), keys.data(), n_rot, A, prod_ws);
        if (rc != HE_OK) return rc;
        for (uint32_t i = 0; i < n_rot; i++) {
            rc = launch_automorph_ntt(ctx, ct_in, rot0 + (size_t)i * L1 * N, L1, gs[i]);
            if (rc != HE_OK) return rc;
        }
        // operand of tap t in the plain part: the rotated c0 (one component) or the input itself (both)
        std::vector<const u64*> plain_ct(taps);
        for (uint32_t i = 0; i < n_rot; i++) plain_ct[rot_tap[i]] = rot0 + (size_t)i * L1 * N;
        if (centre != 0xFFFFFFFFu) plain_ct[centre] = ct_in;
        dim3 block(CV_THREADS), grid_r(N / CV_THREADS, R), grid_q(N / CV_THREADS, L1);
        for (uint32_t o0 = 0; o0 < n_out; o0 += nb_max) {
            const uint32_t nb = std::min<uint32_t>(nb_max, n_out - o0);
            if (n_rot <= 9 && taps <= 9) {
                MacTaps mt;
                MacWeights mw;
                mt.n_taps = n_rot; mt.n_out = nb; mt.c1_tap = 0xFFFFFFFFu;
                for (uint32_t i = 0; i < n_rot; i++) mt.ct[i] = A + (size_t)i * 2 * R * N;
                for (uint32_t o = 0; o < nb; o++) {
                    mt.acc[o] = ACC + (size_t)o * 2 * R * N;
                    for (uint32_t i = 0; i < n_rot; i++) mw.pt[o * 9 + i] = (const u64*)plan->h_d_weights[(size_t)(o0 + o) * taps + rot_tap[i]];
                }
                hipLaunchKernelGGL(mac_taps9_kernel, grid_r, block, 0, ctx->stream, mt, mw, ctx->d_mc, ctx->logN, R, level, ctx->nq);
                HE_HIP(ctx, hipGetLastError());
                mt.n_taps = taps; mt.c1_tap = centre;
                for (uint32_t t = 0; t < taps; t++) mt.ct[t] = plain_ct[t];
                for (uint32_t o = 0; o < nb; o++) {
                    mt.acc[o] = plain + (size_t)o * 2 * L1 * N;
                    for (uint32_t t = 0; t < taps; t++) mw.pt[o * 9 + t] = (const u64*)plan->h_d_weights[(size_t)(o0 + o) * taps + t];
                }
                hipLaunchKernelGGL(mac_taps9_kernel, grid_q, block, 0, ctx->stream, mt, mw, ctx->d_mc, ctx->logN, L1, level, ctx->nq);
                HE_HIP(ctx, hipGetLastError());
            } else {
                for (uint32_t o = 0; o < nb; o++) {
                    MacTapsAny mt;
                    mt.n = n_rot; mt.init = 1; mt.c1_tap = 0xFFFFFFFFu;
                    for (uint32_t i = 0; i < n_rot; i++) {
                        mt.ct[i] = A + (size_t)i * 2 * R * N;
                        mt.pt[i] = (const u64*)plan->h_d_weights[(size_t)(o0 + o) * taps + rot_tap[i]];
                    }
                    hipLaunchKernelGGL(mac_taps_kernel, grid_r, block, 0, ctx->stream, mt, ACC + (size_t)o * 2 * R * N, ctx->d_mc, ctx->logN, R, level, ctx->nq);
                    HE_HIP(ctx, hipGetLastError());
                    mt.n = taps; mt.c1_tap = centre;
                    for (uint32_t t = 0; t < taps; t++) { mt.ct[t] = plain_ct[t]; mt.pt[t] = (const u64*)plan->h_d_weights[(size_t)(o0 + o) * taps + t]; }
                    hipLaunchKernelGGL(mac_taps_kernel, grid_q, block, 0, ctx->stream, mt, plain + (size_t)o * 2 * L1 * N, ctx->d_mc, ctx->logN, L1, level, ctx->nq);
                    HE_HIP(ctx, hipGetLastError());
                }
            }
            std::vector<const u64*> a0(nb), a1(nb);
            std::vector<u64*> o_0(nb), o_1(nb);
            for (uint32_t o = 0; o < nb; o++) {
                a0[o] = plain + (size_t)o * 2 * L1 * N;
                a1[o] = centre != 0xFFFFFFFFu ? a0[o] + (size_t)L1 * N : nullptr;
                o_0[o] = acc + (size_t)(o0 + o) * ct_e;
                o_1[o] = o_0[o] + (size_t)L1 * N;
            }
            rc = ks_moddown_stored(ctx, level, nb, ACC, a0.data(), a1.data(), o_0.data(), o_1.data(), md_ws);
            if (rc != HE_OK) return rc;
        }
        ctx->cnt.mac += (uint64_t)taps * n_out;
    }
    // Slide_f: one ModUp of c1 shared by all taps
    std::vector<const u64*> tap_ct(taps);
    if (!deferred_taps) {
        KsSrc src = {ct_in, ct_in + (size_t)L1 * N, nullptr, nullptr};
        std::vector<KsJob> jobs;
        uint32_t nb = 0;
        for (uint32_t t = 0; t < taps; t++) {
            if (tap_g[t] == 1) { tap_ct[t] = ct_in; continue; }
            u64* out = slid + (size_t)nb++ * ct_e;
            jobs.push_back({0, tap_g[t], tap_key[t], out, out + (size_t)L1 * N, 0});
            tap_ct[t] = out;
        }
        rc = ks_engine(ctx, level, &src, 1, jobs.data(), (uint32_t)jobs.size());
        if (rc != HE_OK) return rc;
    }
    // MulFilter&Sum_f for all outputs, then Rescale of all outputs.  The rotate-and-sum steps
    // ping-pong between the caller's output buffers and the temporaries; start so that the last
    // step lands in the output.
    std::vector<u64*> cur(n_out), nxt(n_out);
    for (uint32_t o = 0; o < n_out; o++) {
        u64* a = (u64*)h_d_ct_out[o];
        u64* b = tmp + (size_t)o * ct_lo_e;
        const uint32_t n_pp = ras_T ? 1u : n_ras;          // buffer swaps until the result must sit in the output
        cur[o] = (n_pp & 1u) ? b : a;
        nxt[o] = (n_pp & 1u) ? a : b;
    }
    {
        dim3 grid(N / CV_THREADS, L1), block(CV_THREADS);
        if (deferred_taps) {
            // the accumulators are already in place
        } else if (taps <= 9) {
            for (uint32_t o0 = 0; o0 < n_out; o0 += CV_MAX_OUT_PER_LAUNCH) {
                MacTaps mt;
                MacWeights mw;
                mt.n_taps = taps; mt.c1_tap = 0xFFFFFFFFu;
                mt.n_out = std::min<uint32_t>(CV_MAX_OUT_PER_LAUNCH, n_out - o0);
                for (uint32_t t = 0; t < taps; t++) mt.ct[t] = tap_ct[t];
                for (uint32_t o = 0; o < mt.n_out; o++) {
                    mt.acc[o] = acc + (size_t)(o0 + o) * ct_e;
                    for (uint32_t t = 0; t < taps; t++) mw.pt[o * 9 + t] = (const u64*)plan->h_d_weights[(size_t)(o0 + o) * taps + t];
                }
                hipLaunchKernelGGL(mac_taps9_kernel, grid, block, 0, ctx->stream, mt, mw, ctx->d_mc, ctx->logN, L1, level, ctx->nq);
                HE_HIP(ctx, hipGetLastError());
            }
        } else {
            for (uint32_t o = 0; o < n_out; o++) {
                MacTapsAny mt;
                mt.n = taps; mt.init = 1; mt.c1_tap = 0xFFFFFFFFu;
                for (uint32_t t = 0; t < taps; t++) { mt.ct[t] = tap_ct[t]; mt.pt[t] = (const u64*)plan->h_d_weights[(size_t)o * taps + t]; }
                hipLaunchKernelGGL(mac_taps_kernel, grid, block, 0, ctx->stream, mt, acc + (size_t)o * ct_e, ctx->d_mc, ctx->logN, L1, level, ctx->nq);
                HE_HIP(ctx, hipGetLastError());
            }
        }
        if (!deferred_taps) ctx->cnt.mac += (uint64_t)taps * n_out;
        std::vector<const u64*> accs(n_out);
        for (uint32_t o = 0; o < n_out; o++) accs[o] = acc + (size_t)o * ct_e;
        rc = rescale_batch(ctx, accs.data(), cur.data(), n_out, level, rs_ws);
        if (rc != HE_OK) return rc;
    }
    if (ras_T) {
        // rotate-and-sum as the sum of the C_a - 1 rotations of each rescaled output, sharing one ModUp and one
        // ModDown per output and the keys between the outputs
        std::vector<KsSrc> srcs(n_out);
        std::vector<u64*> o0(n_out), o1(n_out);
        for (uint32_t o = 0; o < n_out; o++) {
            srcs[o] = {cur[o], cur[o] + (size_t)level * N, cur[o], cur[o] + (size_t)level * N};
            o0[o] = nxt[o]; o1[o] = nxt[o] + (size_t)level * N;
        }
        rc = ks_hoisted_sum(ctx, lo, srcs.data(), n_out, ras_g.data(), ras_key.data(), ras_T, o0.data(), o1.data(), ctx->d_ws);
        if (rc != HE_OK) return rc;
        return HE_OK;
    }
    // rotate-and-sum over the outermost channel dimension: every step is one batch over all
    // outputs (same key), the addition ct + Rot(ct) is done by the ModDown epilogue
    for (uint32_t s = 0; s < n_ras; s++) {
        std::vector<KsSrc> srcs(n_out);
        std::vector<KsJob> jobs(n_out);
        for (uint32_t o = 0; o < n_out; o++) {
            srcs[o] = {cur[o], cur[o] + (size_t)level * N, cur[o], cur[o] + (size_t)level * N};
            jobs[o] = {o, ras_g[s], ras_key[s], nxt[o], nxt[o] + (size_t)level * N, 1};
        }
        rc = ks_engine(ctx, lo, srcs.data(), n_out, jobs.data(), n_out);
        if (rc != HE_OK) return rc;
        std::swap(cur, nxt);
    }
    return HE_OK;
    });
}

// ---------------------------------------------------------------- RAConv (Algorithm 2)
#define RA_IN_PER_LAUNCH 16

struct RaMac {
    const u64* ct[RA_IN_PER_LAUNCH];                     // input ciphertexts [2][L1][N]
    const u64* pt[RA_IN_PER_LAUNCH * 9];                 // [input][tap] inversely rotated filter plaintexts [L1][N]
    u64* acc[9];                                         // one accumulator ciphertext per tap
    uint32_t n_in, n_taps, init;
};

// MulFilter&Sum_ci for up to 9 taps: the coefficients of the (at most NI) inputs are loaded once and kept in registers;
// each tap's accumulator is then their sum of products with that tap's plaintexts, in 128 bits with one Barrett step
// per 8 inputs, so that only two sums are live at a time.  init = 0 continues from the accumulators' current
// (canonical) contents.  grid: (N/256, L1).
template <int NI>
__global__ __launch_bounds__(CV_THREADS) void ra_mac9_kernel(RaMac a, const ModConst* mc, uint32_t logN, uint32_t L1) {
    const uint32_t n = blockIdx.x * CV_THREADS + threadIdx.x;
    const uint32_t limb = blockIdx.y;
    const ModConst m = mc[limb];
    const size_t o0 = ((size_t)limb << logN) + n, o1 = ((size_t)(limb + L1) << logN) + n;
    u64 c0[NI], c1[NI];
#pragma unroll
    for (int i = 0; i < NI; i++) {
        c0[i] = (uint32_t)i < a.n_in ? a.ct[i][o0] : 0;
        c1[i] = (uint32_t)i < a.n_in ? a.ct[i][o1] : 0;
    }
    for (uint32_t t = 0; t < a.n_taps; t++) {
        u128 s0 = a.init ? 0 : a.acc[t][o0], s1 = a.init ? 0 : a.acc[t][o1];
#pragma unroll
        for (int i = 0; i < NI; i++) {
            if (i == 8) {
                s0 = barrett128(s0, m.q, m.mu, m.bits);
                s1 = barrett128(s1, m.q, m.mu, m.bits);
            }
            if ((uint32_t)i < a.n_in) {
                const u64 p = a.pt[i * 9 + t][o0];
                s0 += (u128)c0[i] * p;
                s1 += (u128)c1[i] * p;
            }
        }
        a.acc[t][o0] = barrett128(s0, m.q, m.mu, m.bits);
        a.acc[t][o1] = barrett128(s1, m.q, m.mu, m.bits);
    }
}

static void launch_ra_mac9(he_ctx* ctx, const RaMac& a, dim3 grid, dim3 block, uint32_t L1) {
    if (a.n_in <= 8) hipLaunchKernelGGL(ra_mac9_kernel<8>, grid, block, 0, ctx->stream, a, ctx->d_mc, ctx->logN, L1);
    else hipLaunchKernelGGL(ra_mac9_kernel<RA_IN_PER_LAUNCH>, grid, block, 0, ctx->stream, a, ctx->d_mc, ctx->logN, L1);
}

struct SumList {
    const u64* in[CV_MAX_TAPS];
    uint32_t n;
};
// Sum_f: out = sum of n ciphertexts [2][L1][N] (AddCt only).  grid: (N/256, 2*L1).
__global__ __launch_bounds__(CV_THREADS) void sum_cts_kernel(SumList l, u64* out, const ModConst* mc, uint32_t logN,
                                                             uint32_t L1) {
    const uint32_t n = blockIdx.x * CV_THREADS + threadIdx.x;
    const uint32_t pl = blockIdx.y, limb = pl >= L1 ? pl - L1 : pl;
    const u64 q = mc[limb].q;
    const size_t o = ((size_t)pl << logN) + n;
    u64 acc = l.in[0][o];
    for (uint32_t k = 1; k < l.n; k++) acc = csub(acc + l.in[k][o], q);
    out[o] = acc;
}

// Slide_1 & Sum_f (Algorithm 2): total = sum_t Rot(term_t) over ciphertexts at `level`, term t rotated by the Galois
// element g[t] with key[t] (g = 1: added as it is).  deferred = false: one complete rotation per term, then
// additions; deferred = true: one ModDown for the whole sum.  `total` may alias term 0 only when !deferred.
// ws: slide1_sum_ws_elems elements.
static size_t slide1_sum_ws_elems(const he_ctx* ctx, uint32_t level, uint32_t n_rot, bool deferred) {
    if (n_rot == 0) return 0;
    if (deferred) return ks_rotate_sum_ws_elems(ctx, level, n_rot);
    return ks_engine_ws_elems(ctx, level, n_rot, n_rot) + (size_t)n_rot * 2 * (level + 1) * ctx->N;
}

static int32_t slide1_sum(he_ctx* ctx, uint32_t level, const u64* const* cts, const uint32_t* g, const u64* const* key, uint32_t n,
                          bool deferred, u64* total, u64* ws) {
    const uint32_t N = ctx->N, L1 = level + 1;
    const size_t ct_e = (size_t)2 * L1 * N;
    uint32_t n_rot = 0;
    for (uint32_t t = 0; t < n; t++) n_rot += g[t] != 1;
    if (deferred && n_rot) {
        std::vector<KsSumTerm> terms(n);
        for (uint32_t t = 0; t < n; t++) terms[t] = {cts[t], cts[t] + (size_t)L1 * N, g[t], key[t]};
        return ks_rotate_sum_deferred(ctx, level, terms.data(), n, total, total + (size_t)L1 * N, ws);
    }
    SumList sl;
    sl.n = 0;
    if (n_rot) {
        u64* rot = ws + ks_engine_ws_elems(ctx, level, n_rot, n_rot);   // [n_rot] rotated terms behind the engine's region
        std::vector<KsSrc> srcs;
        std::vector<KsJob> jobs;
        for (uint32_t t = 0; t < n; t++) {
            if (g[t] == 1) { sl.in[sl.n++] = cts[t]; continue; }
            u64* out = rot + (size_t)srcs.size() * ct_e;
            jobs.push_back({(uint32_t)srcs.size(), g[t], key[t], out, out + (size_t)L1 * N, 0});
            srcs.push_back({cts[t], cts[t] + (size_t)L1 * N, nullptr, nullptr});
            sl.in[sl.n++] = out;
        }
        int32_t rc = ks_engine(ctx, level, srcs.data(), (uint32_t)srcs.size(), jobs.data(), (uint32_t)jobs.size());
        if (rc != HE_OK) return rc;
    } else {
        for (uint32_t t = 0; t < n; t++) sl.in[sl.n++] = cts[t];
    }
    hipLaunchKernelGGL(sum_cts_kernel, dim3(N / CV_THREADS, 2 * L1), dim3(CV_THREADS), 0, ctx->stream, sl, total, ctx->d_mc, ctx->logN, L1);
    HE_HIP(ctx, hipGetLastError());
    return HE_OK;
}

extern "C" int32_t he_rotate_sum(he_ctx* ctx, const uint64_t* const* h_d_ct, uint32_t n_ct, uint32_t level, const int32_t* h_steps,
                                 uint64_t* d_out, int32_t deferred) {
    return he_guard(ctx, "he_rotate_sum: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (!h_d_ct || !h_steps || !d_out) return he_fail(ctx, HE_ERR_BADARG, "he_rotate_sum: null argument");
    if (n_ct == 0 || n_ct > CV_MAX_TAPS) return he_fail(ctx, HE_ERR_BADARG, "he_rotate_sum: between 1 and %d terms", CV_MAX_TAPS);
    if (ctx->np == 0) return he_fail(ctx, HE_ERR_BADARG, "he_rotate_sum: context has no special primes");
    if (level >= ctx->nq) return he_fail(ctx, HE_ERR_LEVEL, "he_rotate_sum: level %u above L=%u", level, ctx->nq - 1);
    const uint32_t N = ctx->N, L1 = level + 1;
    const size_t ct_b = (size_t)2 * L1 * N * sizeof(u64);
    std::vector<uint32_t> g(n_ct);
    std::vector<const u64*> key(n_ct, nullptr), cts(n_ct);
    uint32_t n_rot = 0;
    for (uint32_t t = 0; t < n_ct; t++) {
        if (!h_d_ct[t]) return he_fail(ctx, HE_ERR_BADARG, "he_rotate_sum: ciphertext %u is null", t);
        const char *a = (const char*)h_d_ct[t], *b = (const char*)d_out;
        if (a < b + ct_b && b < a + ct_b) return he_fail(ctx, HE_ERR_BADARG, "he_rotate_sum: the output overlaps ciphertext %u", t);
        cts[t] = (const u64*)h_d_ct[t];
        g[t] = h_galois_of_step(ctx, h_steps[t]);
        if (g[t] == 1) continue;
        auto it = ctx->evk.find(g[t]);
        if (it == ctx->evk.end()) return he_fail(ctx, HE_ERR_NOKEY, "he_rotate_sum: no key for step %d (Galois element %u)", h_steps[t], g[t]);
        key[t] = it->second;
        n_rot++;
    }
    int32_t rc = he_ensure_ws(ctx, slide1_sum_ws_elems(ctx, level, n_rot, deferred != 0) * sizeof(u64));
    if (rc != HE_OK) return rc;
    return slide1_sum(ctx, level, cts.data(), g.data(), key.data(), n_ct, deferred != 0, (u64*)d_out, ctx->d_ws);
    });
}

// he_raconv workspace: [Slide_1 & Sum_f region][rescale scratch][taps accumulators][the sum (deferred only)]
static size_t raconv_ws_elems(const he_ctx* ctx, uint32_t level, uint32_t taps, uint32_t n_rot, bool deferred) {
    const size_t ct_e = (size_t)2 * (level + 1) * ctx->N;
    return slide1_sum_ws_elems(ctx, level, n_rot, deferred) + rescale_ws_elems(ctx, level, 1) + (size_t)(taps + (deferred ? 1 : 0)) * ct_e;
}

extern "C" int32_t he_ws_query_raconv(const he_ctx* ctx, const he_raconv_plan* plan, uint64_t* h_bytes) {
    return he_guard(ctx, "he_ws_query_raconv: host allocation failed", [&]() -> int32_t {
    if (!ctx || !plan || !h_bytes) return HE_ERR_BADARG;
    if (plan->level == 0 || plan->level >= ctx->nq) return HE_ERR_LEVEL;
    if ((plan->f & 1u) == 0 || plan->f * plan->f > CV_MAX_TAPS || plan->n_in == 0) return HE_ERR_BADARG;
    uint32_t n_rot = 0;
    for (uint32_t st : tap_slot_steps(plan->W, plan->R, plan->f, ctx->N / 2)) n_rot += st != 0;
    *h_bytes = raconv_ws_elems(ctx, plan->level, plan->f * plan->f, n_rot, plan->deferred_moddown != 0) * sizeof(u64);
    return HE_OK;
    });
}

extern "C" int32_t he_raconv(he_ctx* ctx, const he_raconv_plan* plan, const uint64_t* const* h_d_ct_in, uint64_t* d_ct_out) {
    return he_guard(ctx, "he_raconv: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (!plan || !h_d_ct_in || !d_ct_out || !plan->h_d_weights) return he_fail(ctx, HE_ERR_BADARG, "he_raconv: null argument");
    const uint32_t N = ctx->N, slots = N / 2, level = plan->level, f = plan->f, taps = f * f, n_in = plan->n_in;
    if (ctx->np == 0) return he_fail(ctx, HE_ERR_BADARG, "he_raconv: context has no special primes");
    if (level == 0 || level >= ctx->nq) return he_fail(ctx, HE_ERR_LEVEL, "he_raconv: level %u outside 1..%u", level, ctx->nq - 1);
    if ((f & 1u) == 0 || taps > CV_MAX_TAPS) return he_fail(ctx, HE_ERR_BADARG, "he_raconv: filter width %u must be odd and at most 7", f);
    if (n_in == 0) return he_fail(ctx, HE_ERR_BADARG, "he_raconv: n_in is zero");
    if (plan->W == 0 || plan->R == 0 || (u64)plan->W * plan->R * f > slots)
        return he_fail(ctx, HE_ERR_BADARG, "he_raconv: row length %u x stride %u does not fit the slots", plan->W, plan->R);
    const uint32_t L1 = level + 1;
    const bool deferred = plan->deferred_moddown != 0;
    const std::vector<uint32_t> steps = tap_slot_steps(plan->W, plan->R, f, slots);
    std::vector<uint32_t> tap_g(taps);
    std::vector<const u64*> tap_key(taps, nullptr);
    uint32_t n_rot = 0;
    for (uint32_t t = 0; t < taps; t++) {
        tap_g[t] = h_galois_of_step(ctx, (int32_t)steps[t]);
        if (tap_g[t] != 1) {
            auto it = ctx->evk.find(tap_g[t]);
            if (it == ctx->evk.end()) return he_fail(ctx, HE_ERR_NOKEY, "he_raconv: no key for tap rotation %u", steps[t]);
            tap_key[t] = it->second;
            n_rot++;
        }
    }
    for (uint32_t i = 0; i < n_in; i++)
        if (!h_d_ct_in[i]) return he_fail(ctx, HE_ERR_BADARG, "he_raconv: input %u is null", i);
    for (uint32_t i = 0; i < n_in * taps; i++)
        if (!plan->h_d_weights[i]) return he_fail(ctx, HE_ERR_BADARG, "he_raconv: weight plaintext %u is null", i);
    const size_t ct_e = (size_t)2 * L1 * N;
    const size_t sl_e = slide1_sum_ws_elems(ctx, level, n_rot, deferred), rs_e = rescale_ws_elems(ctx, level, 1);
    int32_t rc = he_ensure_ws(ctx, raconv_ws_elems(ctx, level, taps, n_rot, deferred) * sizeof(u64));
    if (rc != HE_OK) return rc;
    u64* rs_ws = ctx->d_ws + sl_e;
    u64* acc = rs_ws + rs_e;                              // [taps] ciphertexts at `level`
    u64* total = deferred ? acc + (size_t)taps * ct_e : acc;   // not deferred: the sum overwrites the first accumulator
                                                               // (each element is read before it is written)
    // MulFilter&Sum_ci: per tap, the sum over all inputs of input x inversely rotated filter
    {
        dim3 grid(N / CV_THREADS, L1), block(CV_THREADS);
        for (uint32_t t0 = 0; t0 < taps; t0 += 9) {
            for (uint32_t i0 = 0; i0 < n_in; i0 += RA_IN_PER_LAUNCH) {
                RaMac a;
                a.n_taps = std::min<uint32_t>(9, taps - t0);
                a.n_in = std::min<uint32_t>(RA_IN_PER_LAUNCH, n_in - i0);
                a.init = i0 == 0;
                for (uint32_t t = 0; t < a.n_taps; t++) a.acc[t] = acc + (size_t)(t0 + t) * ct_e;
                for (uint32_t i = 0; i < a.n_in; i++) {
                    a.ct[i] = (const u64*)h_d_ct_in[i0 + i];
                    for (uint32_t t = 0; t < a.n_taps; t++) a.pt[i * 9 + t] = (const u64*)plan->h_d_weights[(size_t)(i0 + i) * taps + t0 + t];
                }
                launch_ra_mac9(ctx, a, grid, block, L1);
                HE_HIP(ctx, hipGetLastError());
            }
        }
        ctx->cnt.mac += (uint64_t)taps * n_in;
    }
    // Slide_1&Sum_f: one rotation per off-centre tap (each accumulator is its own source) and additions
    const u64* rin = acc;
    if (taps > 1) {
        std::vector<const u64*> cts(taps);
        for (uint32_t t = 0; t < taps; t++) cts[t] = acc + (size_t)t * ct_e;
        rc = slide1_sum(ctx, level, cts.data(), tap_g.data(), tap_key.data(), taps, deferred, total, ctx->d_ws);
        if (rc != HE_OK) return rc;
        rin = total;
    }
    u64* rout = (u64*)d_ct_out;
    return rescale_batch(ctx, &rin, &rout, 1, level, rs_ws);
    });
}

// ---------------------------------------------------------------- fused block (Algorithm 3)
struct BlockShape {
    uint32_t taps, n_rot, n_ras, G;
    size_t eng_e, rs_e, ct1_e, ct4_e, grp_e, total;
};
static BlockShape block_shape(const he_ctx* ctx, const he_block_plan* p, uint32_t n_rot) {
    BlockShape b;
    const size_t N = ctx->N;
    const uint32_t level = p->level;
    b.taps = p->f * p->f; b.n_rot = n_rot;
    b.n_ras = 0;
    for (uint32_t s = 1; s < p->C_a; s <<= 1) b.n_ras++;
    b.G = (p->group == 0 || p->group > p->n_ra) ? p->n_ra : p->group;
    const size_t ct_hi = 2 * (size_t)(level + 1) * N, ct_mid = 2 * (size_t)level * N, ct_lo = 2 * (size_t)(level - 1) * N;
    b.eng_e = n_rot ? ks_engine_ws_elems(ctx, level, p->n_ca, p->n_ca * n_rot) : 0;
    b.eng_e = std::max(b.eng_e, (p->hoisted_ras && p->C_a > 1) ? ks_hoisted_sum_ws_elems(ctx, level - 1, b.G, p->C_a - 1)
                                                                : ks_engine_ws_elems(ctx, level - 1, b.G, b.G));
    b.eng_e = std::max(b.eng_e, slide1_sum_ws_elems(ctx, level - 2, n_rot, p->deferred_moddown != 0));
    b.rs_e = rescale_ws_elems(ctx, level, b.G);
    b.ct1_e = (size_t)p->n_ca * n_rot * ct_hi;
    b.ct4_e = (size_t)p->n_ca * b.taps * ct_lo;
    // per forwarded group: accumulators at `level`, two buffers at level-1 (rotate-and-sum ping-pong, then the square),
    // the tensor product (3 polynomials per ciphertext at level-1), the squares at level-2; plus one sum at level-2
    b.grp_e = (size_t)b.G * (ct_hi + 2 * ct_mid + 3 * (ct_mid / 2) + ct_lo) + ct_lo;
    b.total = b.eng_e + b.rs_e + b.ct1_e + b.ct4_e + b.grp_e;
    return b;
}

static int32_t block_check(const he_ctx* ctx, const he_block_plan* p) {
    if (p->level < 3 || p->level >= ctx->nq) return HE_ERR_LEVEL;
    if ((p->f & 1u) == 0 || p->f * p->f > CV_MAX_TAPS || p->n_ca == 0 || p->n_ra == 0) return HE_ERR_BADARG;
    if (p->C_a == 0 || (p->C_a & (p->C_a - 1)) || (u64)p->C_a * p->H * p->W * p->R != ctx->N / 2) return HE_ERR_BADARG;
    if ((u64)p->n_ca * p->f * p->f > 4096) return HE_ERR_BADARG;
    return HE_OK;
}

extern "C" int32_t he_ws_query_ca_ra_block(const he_ctx* ctx, const he_block_plan* plan, uint64_t* h_bytes) {
    return he_guard(ctx, "he_ws_query_ca_ra_block: host allocation failed", [&]() -> int32_t {
    if (!ctx || !plan || !h_bytes) return HE_ERR_BADARG;
    int32_t rc = block_check(ctx, plan);
    if (rc != HE_OK) return rc;
    uint32_t n_rot = 0;
    for (uint32_t st : tap_slot_steps(plan->W, plan->R, plan->f, ctx->N / 2)) n_rot += st != 0;
    *h_bytes = block_shape(ctx, plan, n_rot).total * sizeof(u64);
    return HE_OK;
    });
}

extern "C" int32_t he_ca_ra_block(he_ctx* ctx, const he_block_plan* plan, const uint64_t* const* h_d_ct_in, uint64_t* const* h_d_ct_out) {
    return he_guard(ctx, "he_ca_ra_block: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (!plan || !h_d_ct_in || !h_d_ct_out || !plan->h_d_w_ca || !plan->h_d_w_ra || !plan->h_k_in)
        return he_fail(ctx, HE_ERR_BADARG, "he_ca_ra_block: null argument");
    if (ctx->np == 0) return he_fail(ctx, HE_ERR_BADARG, "he_ca_ra_block: context has no special primes");
    int32_t rc = block_check(ctx, plan);
    if (rc == HE_ERR_LEVEL) return he_fail(ctx, rc, "he_ca_ra_block: level %u outside 3..%u", plan->level, ctx->nq - 1);
    if (rc != HE_OK) return he_fail(ctx, rc, "he_ca_ra_block: bad geometry (odd f <= 7, C_a a power of two, C_a*H*W*R = N/2, n_ca, n_ra > 0)");
    const uint32_t N = ctx->N, slots = N / 2, level = plan->level, f = plan->f, taps = f * f, n_ca = plan->n_ca, n_ra = plan->n_ra;
    const uint32_t lv = level - 1, lo = level - 2;
    const bool deferred = plan->deferred_moddown != 0;
    // keys: Slide taps, rotate-and-sum amounts, relinearisation
    const std::vector<uint32_t> steps = tap_slot_steps(plan->W, plan->R, f, slots);
    std::vector<uint32_t> tap_g(taps), ras_g;
    std::vector<const u64*> tap_key(taps, nullptr), ras_key;
    uint32_t n_rot = 0;
    for (uint32_t t = 0; t < taps; t++) {
        tap_g[t] = h_galois_of_step(ctx, (int32_t)steps[t]);
        if (tap_g[t] == 1) continue;
        auto it = ctx->evk.find(tap_g[t]);
        if (it == ctx->evk.end()) return he_fail(ctx, HE_ERR_NOKEY, "he_ca_ra_block: no key for tap rotation %u", steps[t]);
        tap_key[t] = it->second;
        n_rot++;
    }
    const bool hoisted_ras = plan->hoisted_ras != 0 && plan->C_a > 1;
    if (hoisted_ras && plan->C_a > HE_MAX_SUM_TERMS) return he_fail(ctx, HE_ERR_BADARG, "he_ca_ra_block: hoisted_ras supports C_a up to %d", HE_MAX_SUM_TERMS);
    for (uint32_t s = 1; s < plan->C_a; s = hoisted_ras ? s + 1 : s << 1) {
        const uint32_t step = plan->H * plan->W * plan->R * s, g = h_galois_of_step(ctx, (int32_t)step);
        auto it = ctx->evk.find(g);
        if (it == ctx->evk.end()) return he_fail(ctx, HE_ERR_NOKEY, "he_ca_ra_block: no key for rotate-and-sum amount %u", step);
        ras_g.push_back(g);
        ras_key.push_back(it->second);
    }
    auto rl = ctx->evk.find(0);
    if (rl == ctx->evk.end()) return he_fail(ctx, HE_ERR_NOKEY, "he_ca_ra_block: no relinearisation key registered (Galois element 0)");
    for (uint32_t k = 0; k < n_ca; k++)
        if (!h_d_ct_in[k] || !h_d_ct_out[k]) return he_fail(ctx, HE_ERR_BADARG, "he_ca_ra_block: input or output %u is null", k);
    for (size_t i = 0; i < (size_t)n_ra * n_ca * taps; i++)
        if (!plan->h_d_w_ca[i] || !plan->h_d_w_ra[i]) return he_fail(ctx, HE_ERR_BADARG, "he_ca_ra_block: weight plaintext %zu is null", i);
    for (uint32_t r = 0; r <= lv; r++)
        if (plan->h_k_in[r] >= ctx->mod[r]) return he_fail(ctx, HE_ERR_BADARG, "he_ca_ra_block: k_in of limb %u is not a canonical residue", r);
    const BlockShape bs = block_shape(ctx, plan, n_rot);
    rc = he_ensure_ws(ctx, bs.total * sizeof(u64));
    if (rc != HE_OK) return rc;
    const uint32_t G = bs.G, n_ras = bs.n_ras;
    const size_t ct_hi = 2 * (size_t)(level + 1) * N, ct_mid = 2 * (size_t)level * N, ct_lo = 2 * (size_t)lv * N, pe_mid = (size_t)level * N;
    u64* rs_ws = ctx->d_ws + bs.eng_e;
    u64* ct1 = rs_ws + bs.rs_e;                           // [n_ca][n_rot] rotated inputs at `level`
    u64* ct4 = ct1 + bs.ct1_e;                            // [n_ca][taps] accumulators at level-2
    u64* acc = ct4 + bs.ct4_e;                            // [G] at `level`
    u64* pa = acc + (size_t)G * ct_hi;                    // [G] at level-1
    u64* pb = pa + (size_t)G * ct_mid;                    // [G] at level-1
    u64* tens = pb + (size_t)G * ct_mid;                  // [G][3] polynomials at level-1
    u64* ct3 = tens + (size_t)G * 3 * pe_mid;             // [G] squares at level-2
    u64* total = ct3 + (size_t)G * ct_lo;                 // one sum at level-2

    // Slide_f of every input: one ModUp per input shared by its taps, all inputs in one batch
    std::vector<const u64*> slid((size_t)n_ca * taps);
    {
        std::vector<KsSrc> srcs(n_ca);
        std::vector<KsJob> jobs;
        for (uint32_t k = 0; k < n_ca; k++) {
            const u64* in = (const u64*)h_d_ct_in[k];
            srcs[k] = {in, in + (size_t)(level + 1) * N, nullptr, nullptr};
            uint32_t nb = 0;
            for (uint32_t t = 0; t < taps; t++) {
                if (tap_g[t] == 1) { slid[(size_t)k * taps + t] = in; continue; }
                u64* out = ct1 + ((size_t)k * n_rot + nb++) * ct_hi;
                jobs.push_back({k, tap_g[t], tap_key[t], out, out + (size_t)(level + 1) * N, 0});
                slid[(size_t)k * taps + t] = out;
            }
        }
        if (!jobs.empty()) {
            rc = ks_engine(ctx, level, srcs.data(), n_ca, jobs.data(), (uint32_t)jobs.size());
            if (rc != HE_OK) return rc;
        }
    }
    AffineConst kin;                                      // integer lift before the square, per limb
    for (uint32_t r = 0; r <= lv; r++) { kin.mul[r] = plan->h_k_in[r]; kin.add[r] = 0; }
    for (uint32_t j0 = 0; j0 < n_ra; j0 += G) {
        const uint32_t g = std::min(G, n_ra - j0);
        // MulFilter&Sum_f over every input and tap, for the g intermediates of this group
        {
            dim3 grid(N / CV_THREADS, level + 1), block(CV_THREADS);
            if (n_ca == 1 && taps <= 9) {
                for (uint32_t o0 = 0; o0 < g; o0 += CV_MAX_OUT_PER_LAUNCH) {
                    MacTaps mt;
                    MacWeights mw;
                    mt.n_taps = taps; mt.c1_tap = 0xFFFFFFFFu;
                    mt.n_out = std::min<uint32_t>(CV_MAX_OUT_PER_LAUNCH, g - o0);
                    for (uint32_t t = 0; t < taps; t++) mt.ct[t] = slid[t];
                    for (uint32_t o = 0; o < mt.n_out; o++) {
                        mt.acc[o] = acc + (size_t)(o0 + o) * ct_hi;
                        for (uint32_t t = 0; t < taps; t++) mw.pt[o * 9 + t] = (const u64*)plan->h_d_w_ca[(size_t)(j0 + o0 + o) * taps + t];
                    }
                    hipLaunchKernelGGL(mac_taps9_kernel, grid, block, 0, ctx->stream, mt, mw, ctx->d_mc, ctx->logN, level + 1, level, ctx->nq);
                    HE_HIP(ctx, hipGetLastError());
                }
            } else {
                const size_t terms = (size_t)n_ca * taps;
                for (uint32_t o = 0; o < g; o++)
                    for (size_t i0 = 0; i0 < terms; i0 += CV_MAX_TAPS) {
                        MacTapsAny mt;
                        mt.n = (uint32_t)std::min<size_t>(CV_MAX_TAPS, terms - i0);
                        mt.init = i0 == 0; mt.c1_tap = 0xFFFFFFFFu;
                        for (uint32_t i = 0; i < mt.n; i++) {
                            mt.ct[i] = slid[i0 + i];                                       // [k][tap] flattened
                            mt.pt[i] = (const u64*)plan->h_d_w_ca[(size_t)(j0 + o) * terms + i0 + i];
                        }
                        hipLaunchKernelGGL(mac_taps_kernel, grid, block, 0, ctx->stream, mt, acc + (size_t)o * ct_hi, ctx->d_mc, ctx->logN, level + 1, level, ctx->nq);
                        HE_HIP(ctx, hipGetLastError());
                    }
            }
            ctx->cnt.mac += (uint64_t)g * n_ca * taps;
        }
        // Rescale, then rotate-and-sum over C_a (ping-pong so that the last step lands in pa)
        std::vector<const u64*> accs(g);
        std::vector<u64*> cur(g), nxt(g);
        for (uint32_t o = 0; o < g; o++) {
            accs[o] = acc + (size_t)o * ct_hi;
            u64 *a = pa + (size_t)o * ct_mid, *b = pb + (size_t)o * ct_mid;
            const uint32_t n_pp = hoisted_ras ? 1u : n_ras;
            cur[o] = (n_pp & 1u) ? b : a;
            nxt[o] = (n_pp & 1u) ? a : b;
        }
        rc = rescale_batch(ctx, accs.data(), cur.data(), g, level, rs_ws);
        if (rc != HE_OK) return rc;
        if (hoisted_ras) {
            // one hoisted sum of the C_a - 1 rotations per intermediate (one ModUp, one ModDown each)
            std::vector<KsSrc> srcs(g);
            std::vector<u64*> o0(g), o1(g);
            for (uint32_t o = 0; o < g; o++) {
                srcs[o] = {cur[o], cur[o] + pe_mid, cur[o], cur[o] + pe_mid};
                o0[o] = nxt[o]; o1[o] = nxt[o] + pe_mid;
            }
            rc = ks_hoisted_sum(ctx, lv, srcs.data(), g, ras_g.data(), ras_key.data(), plan->C_a - 1, o0.data(), o1.data(), ctx->d_ws);
            if (rc != HE_OK) return rc;
            std::swap(cur, nxt);
        }
        for (uint32_t s = 0; s < n_ras && !hoisted_ras; s++) {
            std::vector<KsSrc> srcs(g);
            std::vector<KsJob> jobs(g);
            for (uint32_t o = 0; o < g; o++) {
                srcs[o] = {cur[o], cur[o] + pe_mid, cur[o], cur[o] + pe_mid};
                jobs[o] = {o, ras_g[s], ras_key[s], nxt[o], nxt[o] + pe_mid, 1};
            }
            rc = ks_engine(ctx, lv, srcs.data(), g, jobs.data(), g);
            if (rc != HE_OK) return rc;
            std::swap(cur, nxt);
        }
        // Square: integer lift, tensor product, relinearisation of all g at once, Rescale -> ct3
        {
            std::vector<KsSrc> srcs(g);
            std::vector<KsJob> jobs(g);
            std::vector<const u64*> sq(g);
            std::vector<u64*> outs(g);
            for (uint32_t o = 0; o < g; o++) {
                u64* u = cur[o];                          // == pa + o*ct_mid
                rc = launch_affine(ctx, u, lv, kin, u);
                if (rc != HE_OK) return rc;
                u64* d = tens + (size_t)o * 3 * pe_mid;
                rc = launch_tensor(ctx, u, u, lv, d);
                if (rc != HE_OK) return rc;
                u64* res = nxt[o];                        // the other level-1 buffer
                srcs[o] = {nullptr, d + 2 * pe_mid, d, d + pe_mid};
                jobs[o] = {o, 1, rl->second, res, res + pe_mid, 1};
                sq[o] = res;
                outs[o] = ct3 + (size_t)o * ct_lo;
            }
            rc = ks_engine(ctx, lv, srcs.data(), g, jobs.data(), g);
            if (rc != HE_OK) return rc;
            rc = rescale_batch(ctx, sq.data(), outs.data(), g, lv, rs_ws);
            if (rc != HE_OK) return rc;
        }
        // forwarded into the f^2 accumulators of every output: MulFilter&Sum_ci with the inversely rotated filters
        {
            dim3 grid(N / CV_THREADS, lo + 1), block(CV_THREADS);
            for (uint32_t l = 0; l < n_ca; l++)
                for (uint32_t t0 = 0; t0 < taps; t0 += 9)
                    for (uint32_t i0 = 0; i0 < g; i0 += RA_IN_PER_LAUNCH) {
                        RaMac a;
                        a.n_taps = std::min<uint32_t>(9, taps - t0);
                        a.n_in = std::min<uint32_t>(RA_IN_PER_LAUNCH, g - i0);
                        a.init = (j0 == 0 && i0 == 0);
                        for (uint32_t t = 0; t < a.n_taps; t++) a.acc[t] = ct4 + ((size_t)l * taps + t0 + t) * ct_lo;
                        for (uint32_t i = 0; i < a.n_in; i++) {
                            a.ct[i] = ct3 + (size_t)(i0 + i) * ct_lo;
                            for (uint32_t t = 0; t < a.n_taps; t++)
                                a.pt[i * 9 + t] = (const u64*)plan->h_d_w_ra[((size_t)l * n_ra + j0 + i0 + i) * taps + t0 + t];
                        }
                        launch_ra_mac9(ctx, a, grid, block, lo + 1);
                        HE_HIP(ctx, hipGetLastError());
                    }
            ctx->cnt.mac += (uint64_t)g * n_ca * taps;
        }
    }
    // Slide_1&Sum_f of every output's accumulators, then its Rescale
    for (uint32_t l = 0; l < n_ca; l++) {
        std::vector<const u64*> cts(taps);
        for (uint32_t t = 0; t < taps; t++) cts[t] = ct4 + ((size_t)l * taps + t) * ct_lo;
        const u64* rin = cts[0];
        if (taps > 1) {
            u64* tot = deferred ? total : (u64*)cts[0];
            rc = slide1_sum(ctx, lo, cts.data(), tap_g.data(), tap_key.data(), taps, deferred, tot, ctx->d_ws);
            if (rc != HE_OK) return rc;
            rin = tot;
        }
        u64* rout = (u64*)h_d_ct_out[l];
        rc = rescale_batch(ctx, &rin, &rout, 1, lo, rs_ws);
        if (rc != HE_OK) return rc;
    }
    return HE_OK;
    });
}

// ---------------------------------------------------------------- batched rotate-and-sum
extern "C" int32_t he_ras(he_ctx* ctx, const uint64_t* const* h_d_ct, uint32_t n_ct, uint32_t level, const int32_t* h_steps,
                          uint32_t n_steps, uint64_t* const* h_d_out) {
    return he_guard(ctx, "he_ras: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (n_ct == 0) return HE_OK;
    if (!h_d_ct || !h_d_out || (n_steps && !h_steps)) return he_fail(ctx, HE_ERR_BADARG, "he_ras: null argument");
    if (ctx->np == 0) return he_fail(ctx, HE_ERR_BADARG, "he_ras: context has no special primes");
    if (level >= ctx->nq) return he_fail(ctx, HE_ERR_LEVEL, "he_ras: level %u above L=%u", level, ctx->nq - 1);
    const uint32_t N = ctx->N, L1 = level + 1;
    const size_t ct_e = (size_t)2 * L1 * N, ct_b = ct_e * sizeof(u64);
    std::vector<uint32_t> gs(n_steps);
    std::vector<const u64*> keys(n_steps);
    for (uint32_t s = 0; s < n_steps; s++) {
        gs[s] = h_galois_of_step(ctx, h_steps[s]);
        if (gs[s] == 1) return he_fail(ctx, HE_ERR_BADARG, "he_ras: step %u is a multiple of the slot count", s);
        auto it = ctx->evk.find(gs[s]);
        if (it == ctx->evk.end()) return he_fail(ctx, HE_ERR_NOKEY, "he_ras: no key for step %d (Galois element %u)", h_steps[s], gs[s]);
        keys[s] = it->second;
    }
    {   // no output may overlap an input or another output
        struct Buf { const char* p; bool out; };
        std::vector<Buf> bufs;
        for (uint32_t i = 0; i < n_ct; i++) {
            if (!h_d_ct[i] || !h_d_out[i]) return he_fail(ctx, HE_ERR_BADARG, "he_ras: ciphertext %u is null", i);
            bufs.push_back({(const char*)h_d_ct[i], false});
            bufs.push_back({(const char*)h_d_out[i], true});
        }
        std::sort(bufs.begin(), bufs.end(), [](const Buf& a, const Buf& b) { return a.p < b.p; });
        for (size_t i = 1; i < bufs.size(); i++)
            if (bufs[i].p < bufs[i - 1].p + ct_b && (bufs[i].out || bufs[i - 1].out))
                return he_fail(ctx, HE_ERR_BADARG, "he_ras: an output overlaps an input or another output");
    }
    if (n_steps == 0) {
        for (uint32_t i = 0; i < n_ct; i++) HE_HIP(ctx, hipMemcpyAsync(h_d_out[i], h_d_ct[i], ct_b, hipMemcpyDeviceToDevice, ctx->stream));
        return HE_OK;
    }
    // workspace: [engine region][n_ct temporaries]; the steps ping-pong so that the last one lands in the outputs
    const size_t ks_e = ks_engine_ws_elems(ctx, level, n_ct, n_ct);
    int32_t rc = he_ensure_ws(ctx, (ks_e + (n_steps > 1 ? (size_t)n_ct * ct_e : 0)) * sizeof(u64));
    if (rc != HE_OK) return rc;
    u64* tmp = ctx->d_ws + ks_e;
    std::vector<const u64*> cur(n_ct);
    for (uint32_t i = 0; i < n_ct; i++) cur[i] = (const u64*)h_d_ct[i];
    for (uint32_t s = 0; s < n_steps; s++) {
        const bool to_out = ((n_steps - 1 - s) & 1u) == 0;
        std::vector<KsSrc> srcs(n_ct);
        std::vector<KsJob> jobs(n_ct);
        std::vector<const u64*> nxt(n_ct);
        for (uint32_t i = 0; i < n_ct; i++) {
            u64* dst = to_out ? (u64*)h_d_out[i] : tmp + (size_t)i * ct_e;
            srcs[i] = {cur[i], cur[i] + (size_t)L1 * N, cur[i], cur[i] + (size_t)L1 * N};
            jobs[i] = {i, gs[s], keys[s], dst, dst + (size_t)L1 * N, 1};
            nxt[i] = dst;
        }
        rc = ks_engine(ctx, level, srcs.data(), n_ct, jobs.data(), n_ct);
        if (rc != HE_OK) return rc;
        cur = nxt;
    }
    return HE_OK;
    });
}
