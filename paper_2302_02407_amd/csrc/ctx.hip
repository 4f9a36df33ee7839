// Context: parameter validation, root/twiddle tables, device constants, workspace, errors.
#include <stdarg.h>
#include <new>
#include <stdio.h>
#include <string.h>

#include "he_internal.h"

static std::string g_create_err;

int32_t he_fail(he_ctx* ctx, int32_t code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    if (ctx) ctx->err = buf; else g_create_err = buf;
    return code;
}

void he_fail_nothrow(he_ctx* ctx, const char* msg) noexcept {
    try {
        if (ctx) ctx->err = msg; else g_create_err = msg;
    } catch (...) {
    }
}

u64 h_mulmod(u64 a, u64 b, u64 m) { return (u64)((u128)a * b % m); }
u64 h_powmod(u64 a, u64 e, u64 m) {
    u64 r = 1 % m;
    a %= m;
    for (; e; e >>= 1) {
        if (e & 1) r = h_mulmod(r, a, m);
        a = h_mulmod(a, a, m);
    }
    return r;
}
u64 h_invmod(u64 a, u64 m) { return h_powmod(a % m, m - 2, m); }
u64 h_shoup(u64 w, u64 m) { return (u64)(((u128)w << 64) / m); }

static bool h_is_prime(u64 n) {
    if (n < 2) return false;
    static const u64 bases[] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
    for (u64 b : bases) {
        if (n % b == 0) return n == b;
    }
    u64 d = n - 1;
    int r = 0;
    while ((d & 1) == 0) { d >>= 1; r++; }
    for (u64 a : bases) {
        u64 x = h_powmod(a, d, n);
        if (x == 1 || x == n - 1) continue;
        bool comp = true;
        for (int i = 1; i < r; i++) {
            x = h_mulmod(x, x, n);
            if (x == n - 1) { comp = false; break; }
        }
        if (comp) return false;
    }
    return true;
}

static uint32_t bitrev(uint32_t x, uint32_t bits) {
    uint32_t r = 0;
    for (uint32_t i = 0; i < bits; i++) r |= ((x >> i) & 1u) << (bits - 1 - i);
    return r;
}

uint32_t h_galois_of_step(const he_ctx* ctx, int32_t step) {
    int64_t half = ctx->N / 2;
    int64_t s = ((int64_t)step % half + half) % half;
    return (uint32_t)h_powmod(5, (u64)s, 2 * (u64)ctx->N);
}

void scale_entry(const he_ctx* c, ScaleList& sc, uint32_t i, uint32_t mi, u64 s) {
    const u64 m = c->mod[mi];
    sc.s[i] = s;
    sc.s_sh[i] = h_shoup(s, m);
    sc.w[i] = h_mulmod(s, c->itw1[mi], m);
    sc.w_sh[i] = h_shoup(sc.w[i], m);
}

int32_t he_ensure_ws(he_ctx* ctx, size_t bytes) {
    if (bytes <= ctx->ws_bytes) return HE_OK;
    if (ctx->d_ws) {
        HE_HIP(ctx, hipStreamSynchronize(ctx->stream));
        HE_HIP(ctx, hipFree(ctx->d_ws));
        ctx->d_ws = nullptr;
        ctx->ws_bytes = 0;
    }
    if (hipMalloc(&ctx->d_ws, bytes) != hipSuccess) {
        (void)hipGetLastError();
        return he_fail(ctx, HE_ERR_ALLOC, "workspace allocation of %zu bytes failed", bytes);
    }
    ctx->ws_bytes = bytes;
    return HE_OK;
}

extern "C" {

const char* he_last_error(const he_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_err.c_str(); }

int32_t he_ctx_create(he_ctx** out, uint32_t logN, const uint64_t* h_q, uint32_t nq, const uint64_t* h_p,
                      uint32_t np, uint32_t dnum, void* hip_stream) {
    return he_guard(nullptr, "he_ctx_create: host allocation failed", [&]() -> int32_t {
    if (!out) return he_fail(nullptr, HE_ERR_BADARG, "he_ctx_create: out is null");
    *out = nullptr;
    if (logN < 8 || logN > 17) return he_fail(nullptr, HE_ERR_BADARG, "he_ctx_create: logN %u outside 8..17", logN);
    if (!h_q || nq == 0 || (np && !h_p)) return he_fail(nullptr, HE_ERR_BADARG, "he_ctx_create: missing prime list");
    if (nq + np > HE_MAX_MODULI) return he_fail(nullptr, HE_ERR_BADARG, "he_ctx_create: more than %d moduli", HE_MAX_MODULI);
    if (dnum == 0 || dnum > nq) return he_fail(nullptr, HE_ERR_BADARG, "he_ctx_create: dnum %u outside 1..nq", dnum);
    uint32_t N = 1u << logN, M = nq + np;
    for (uint32_t i = 0; i < M; i++) {
        u64 m = i < nq ? h_q[i] : h_p[i - nq];
        if (m <= (1ull << 20) || m >= (1ull << 60)) return he_fail(nullptr, HE_ERR_BADARG, "he_ctx_create: modulus %u out of range (2^20, 2^60)", i);
        if (m % (2ull * N) != 1) return he_fail(nullptr, HE_ERR_BADARG, "he_ctx_create: modulus %u is not 1 mod 2N", i);
        if (!h_is_prime(m)) return he_fail(nullptr, HE_ERR_BADARG, "he_ctx_create: modulus %u is not prime", i);
        for (uint32_t k = 0; k < i; k++) {
            u64 mk = k < nq ? h_q[k] : h_p[k - nq];
            if (mk == m) return he_fail(nullptr, HE_ERR_BADARG, "he_ctx_create: modulus %u repeats modulus %u", i, k);
        }
    }
    // host tables first, so that a failed host allocation leaves nothing behind
    std::vector<u64> tw((size_t)M * N), tw_sh((size_t)M * N), itw((size_t)M * N), itw_sh((size_t)M * N);
    he_ctx* c = new (std::nothrow) he_ctx();
    if (!c) return he_fail(nullptr, HE_ERR_ALLOC, "he_ctx_create: host allocation failed");
    struct Owner {                                      // destroys the half-built context on every early exit
        he_ctx* c;
        ~Owner() { if (c) he_ctx_destroy(c); }
    } own{c};
    c->logN = logN; c->N = N; c->nq = nq; c->np = np; c->dnum = dnum; c->M = M;
    c->alpha = (nq + dnum - 1) / dnum;
    c->stream = (hipStream_t)hip_stream;
    c->d_mc = nullptr; c->d_tw = c->d_tw_sh = c->d_itw = c->d_itw_sh = nullptr;
    c->d_ws = nullptr; c->ws_bytes = 0;
    c->d_up_hat = c->d_dn_hat = c->d_pinv = c->d_pinv_sh = c->d_qlinv = c->d_qlinv_sh = nullptr;
    memset(&c->cnt, 0, sizeof(c->cnt));
    c->prof_on = false;
    // latency path of the N = 2^16 conversions; HE_COLFUSE_GROUPS=0 switches it off (for measurements)
    c->cf_max_groups = 4; c->cf_max_targets = 16;
    if (const char* e = getenv("HE_COLFUSE_GROUPS")) c->cf_max_groups = (uint32_t)strtoul(e, nullptr, 10);
    if (const char* e = getenv("HE_COLFUSE_TARGETS")) c->cf_max_targets = (uint32_t)strtoul(e, nullptr, 10);
    if (hipGetDevice(&c->device) != hipSuccess) {
        return he_fail(nullptr, HE_ERR_HIP, "he_ctx_create: no HIP device");
    }
    // tables on the host
    for (uint32_t i = 0; i < M; i++) {
        u64 m = i < nq ? h_q[i] : h_p[i - nq];
        c->mod[i] = m;
        u64 g = 2;
        while (h_powmod(g, (m - 1) / 2, m) != m - 1) g++;       // smallest quadratic non-residue
        u64 psi = h_powmod(g, (m - 1) / (2ull * N), m);
        c->psi[i] = psi;
        u64 ipsi = h_invmod(psi, m);
        u64 pw = 1, ipw = 1;
        u64* t = &tw[(size_t)i * N]; u64* ts = &tw_sh[(size_t)i * N];
        u64* it = &itw[(size_t)i * N]; u64* its = &itw_sh[(size_t)i * N];
        for (uint32_t e = 0; e < N; e++) {                      // psi^e stored at bitrev(e)
            uint32_t pos = bitrev(e, logN);
            t[pos] = pw; ts[pos] = h_shoup(pw, m);
            it[pos] = ipw; its[pos] = h_shoup(ipw, m);
            pw = h_mulmod(pw, psi, m);
            ipw = h_mulmod(ipw, ipsi, m);
        }
        ModConst& mc = c->h_mc[i];
        mc.q = m; mc.q2 = 2 * m;
        mc.bits = 64 - __builtin_clzll(m);
        mc.mu = (u64)(((u128)1 << (mc.bits + 63)) / m);
        mc.ninv = h_invmod(N % m, m);
        mc.ninv_sh = h_shoup(mc.ninv, m);
        c->itw1[i] = h_powmod(ipsi, N / 2, m);
        mc.ninv_w = h_mulmod(mc.ninv, c->itw1[i], m);
        mc.ninv_w_sh = h_shoup(mc.ninv_w, m);
        mc.one_sh = h_shoup(1, m);
        mc.pad = 0;
    }
    size_t tb = (size_t)M * N * sizeof(u64);
    hipError_t e = hipSuccess;
    if (e == hipSuccess) e = hipMalloc(&c->d_mc, sizeof(ModConst) * M);
    if (e == hipSuccess) e = hipMalloc(&c->d_tw, tb);
    if (e == hipSuccess) e = hipMalloc(&c->d_tw_sh, tb);
    if (e == hipSuccess) e = hipMalloc(&c->d_itw, tb);
    if (e == hipSuccess) e = hipMalloc(&c->d_itw_sh, tb);
    if (e == hipSuccess) e = hipMemcpy(c->d_mc, c->h_mc, sizeof(ModConst) * M, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c->d_tw, tw.data(), tb, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c->d_tw_sh, tw_sh.data(), tb, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c->d_itw, itw.data(), tb, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c->d_itw_sh, itw_sh.data(), tb, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        he_fail(nullptr, e == hipErrorOutOfMemory ? HE_ERR_ALLOC : HE_ERR_HIP, "he_ctx_create: %s", hipGetErrorString(e));
        return e == hipErrorOutOfMemory ? HE_ERR_ALLOC : HE_ERR_HIP;
    }
    {
        int32_t rc = ks_init_tables(c);
        if (rc != HE_OK) {
            g_create_err = c->err;
                return rc;
        }
    }
    {
        int32_t rc = he_noalloc_init_device(c, c->device);
        if (rc != HE_OK) {
            g_create_err = c->err;
            return rc;
        }
    }
    // workspace for every one-ciphertext call at the top level: one key switch (raised digits +
    // temporaries) with the three tensor-product polynomials of a ct x ct multiplication behind it, or
    // one rescale; only the batched calls and the convolutions can need more (he_ws_reserve)
    if (np > 0) {
        size_t elems = ks_engine_ws_elems(c, nq - 1, 1, 1) + (size_t)3 * nq * N;
        if (nq > 1) elems = elems > rescale_ws_elems(c, nq - 1, 1) ? elems : rescale_ws_elems(c, nq - 1, 1);
        int32_t rc = he_ensure_ws(c, elems * sizeof(u64));
        if (rc != HE_OK) {
            g_create_err = c->err;
                return rc;
        }
    }
    own.c = nullptr;
    *out = c;
    return HE_OK;
    });
}

int32_t he_ctx_destroy(he_ctx* c) {
    return he_guard(c, "he_ctx_destroy: host allocation failed", [&]() -> int32_t {
    if (!c) return HE_OK;
    (void)hipStreamSynchronize(c->stream);
    if (c->d_mc) (void)hipFree(c->d_mc);
    if (c->d_tw) (void)hipFree(c->d_tw);
    if (c->d_tw_sh) (void)hipFree(c->d_tw_sh);
    if (c->d_itw) (void)hipFree(c->d_itw);
    if (c->d_itw_sh) (void)hipFree(c->d_itw_sh);
    if (c->d_ws) (void)hipFree(c->d_ws);
    for (auto& s : c->prof_events) { (void)hipEventDestroy(s.e0); (void)hipEventDestroy(s.e1); }
    ks_free_tables(c);
    delete c;
    return HE_OK;
    });
}

int32_t he_ctx_psi(const he_ctx* ctx, uint32_t mod_idx, uint64_t* h_psi_out) {
    return he_guard(ctx, "he_ctx_psi: host allocation failed", [&]() -> int32_t {
    if (!ctx || !h_psi_out || mod_idx >= ctx->M) return HE_ERR_BADARG;
    *h_psi_out = ctx->psi[mod_idx];
    return HE_OK;
    });
}

int32_t he_counters(const he_ctx* ctx, he_counters_t* h_out) {
    return he_guard(ctx, "he_counters: host allocation failed", [&]() -> int32_t {
    if (!ctx || !h_out) return HE_ERR_BADARG;
    *h_out = ctx->cnt;
    return HE_OK;
    });
}

int32_t he_counters_reset(he_ctx* ctx) {
    return he_guard(ctx, "he_counters_reset: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    memset(&ctx->cnt, 0, sizeof(ctx->cnt));
    return HE_OK;
    });
}

int32_t he_profile_begin(he_ctx* ctx) {
    return he_guard(ctx, "he_profile_begin: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    for (auto& s : ctx->prof_events) { (void)hipEventDestroy(s.e0); (void)hipEventDestroy(s.e1); }
    ctx->prof_events.clear();
    ctx->prof_key_limbs = 0;
    ctx->prof_on = true;
    return HE_OK;
    });
}

int32_t he_profile_end(he_ctx* ctx, he_profile_t* h_out) {
    return he_guard(ctx, "he_profile_end: host allocation failed", [&]() -> int32_t {
    if (!ctx || !h_out) return HE_ERR_BADARG;
    ctx->prof_on = false;
    HE_HIP(ctx, hipStreamSynchronize(ctx->stream));
    memset(h_out, 0, sizeof(*h_out));
    for (auto& s : ctx->prof_events) {
        float ms = 0.f;
        HE_HIP(ctx, hipEventElapsedTime(&ms, s.e0, s.e1));
        h_out->transform_launches += 1;
        h_out->transform_limb_passes += s.limbs;
        h_out->inner_product_digit_limbs += s.digit_limbs;
        h_out->transform_ms += ms;
        const uint32_t kd = s.kind < 6 ? s.kind : 0;
        h_out->pass_launches[kd] += 1;
        h_out->pass_limbs[kd] += s.limbs;
        h_out->pass_ms[kd] += ms;
        (void)hipEventDestroy(s.e0);
        (void)hipEventDestroy(s.e1);
    }
    h_out->key_limbs_read = ctx->prof_key_limbs;
    ctx->prof_events.clear();
    return HE_OK;
    });
}

int32_t he_probe_alu(he_ctx* ctx, he_alu_probe_t* h_out) {
    return he_guard(ctx, "he_probe_alu: host allocation failed", [&]() -> int32_t {
    if (!ctx || !h_out) return HE_ERR_BADARG;
    const uint32_t groups = 256 * 16;                    // 16 work groups of 256 threads per compute unit
    int32_t rc = he_ensure_ws(ctx, (size_t)groups * 256 * sizeof(u64));
    if (rc != HE_OK) return rc;
    double r[3];
    rc = probe_butterfly_rates(ctx, ctx->d_ws, groups, r);
    if (rc != HE_OK) return rc;
    h_out->fwd_butterflies_per_s = r[0];
    h_out->inv_butterflies_per_s = r[1];
    h_out->fwd_wide_butterflies_per_s = r[2];
    return HE_OK;
    });
}

#ifndef HE_BUILD_ID
#define HE_BUILD_ID "unknown"
#endif
const char* he_build_id(void) { return HE_BUILD_ID; }

int32_t he_sync(he_ctx* ctx) {
    return he_guard(ctx, "he_sync: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    HE_HIP(ctx, hipStreamSynchronize(ctx->stream));
    return HE_OK;
    });
}

int32_t he_ws_bytes(const he_ctx* ctx, uint64_t* h_bytes) {
    return he_guard(ctx, "he_ws_bytes: host allocation failed", [&]() -> int32_t {
    if (!ctx || !h_bytes) return HE_ERR_BADARG;
    *h_bytes = ctx->ws_bytes;
    return HE_OK;
    });
}

int32_t he_ws_reserve(he_ctx* ctx, uint64_t bytes) {
    return he_guard(ctx, "he_ws_reserve: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    return he_ensure_ws(ctx, (size_t)bytes);
    });
}

int32_t he_evk_register(he_ctx* ctx, uint32_t galois_elt, const uint64_t* d_evk) {
    return he_guard(ctx, "he_evk_register: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (!d_evk) return he_fail(ctx, HE_ERR_BADARG, "he_evk_register: null key");
    if (galois_elt != 0 && ((galois_elt & 1u) == 0 || galois_elt >= 2 * ctx->N))
        return he_fail(ctx, HE_ERR_BADARG, "he_evk_register: Galois element %u is not odd and below 2N", galois_elt);
    if (ctx->np == 0) return he_fail(ctx, HE_ERR_BADARG, "he_evk_register: context has no special primes");
    ctx->evk[galois_elt] = (const u64*)d_evk;
    return HE_OK;
    });
}

} // extern "C"
