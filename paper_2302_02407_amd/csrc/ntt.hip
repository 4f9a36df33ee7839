// Batched negacyclic NTT / iNTT over RNS limbs (ring Z_q[X]/(X^N+1), paper Section 2.1).
//
// Forward: decimation-in-time butterflies with the 2N-th root folded into the twiddles
// (natural-order coefficients in, bit-reversed evaluations out); inverse: the mirrored
// decimation-in-frequency network.  Butterflies keep residues lazily reduced (forward in
// [0,4q), inverse in [0,2q)) and multiply by twiddles with Shoup's precomputed quotients;
// only the last pass canonicalises.
//
// This file serves every ring size except N = 2^16 (which has its own two-launch kernels).  Rings up
// to N = 2^12 are one pass with the whole limb (at most 32 KiB) staged in LDS; larger rings take two
// passes over tiles of 2^12 elements:
//   pass A ("strided"): the first logN-12 stages; a tile is ROWS = 2^(logN-12) rows of
//                       COLS = 4096/ROWS adjacent columns of the 4096-wide row-major view;
//   pass B ("contiguous"): the last 12 stages; a tile is 4096 consecutive elements.
// Both passes run the same butterfly loop on the tile-local index space.
#include "modarith.h"

#define NTT_THREADS 1024
#define NTT_LOG_TILE_MAX 12

struct NttArgs {
    u64* data;
    const ModConst* mc;
    const u64* tw;     // [M][N] forward or inverse table
    const u64* tw_sh;  // Shoup companions
    uint32_t logN;
    uint32_t log_tile; // min(logN, 12)
    uint32_t s_begin;  // stages [s_begin, s_end) of this pass, ascending stage index
    uint32_t s_end;
    uint32_t strided;  // 1 = pass A layout, 0 = pass B layout
    uint32_t last;     // 1 = this pass produces the final (canonical) output
};

__device__ __forceinline__ uint32_t tile_global_index(uint32_t e, uint32_t tile, uint32_t log_tile, uint32_t log_rows,
                                                      uint32_t strided) {
    if (!strided) return (tile << log_tile) + e;
    uint32_t log_cols = log_tile - log_rows;
    uint32_t r = e >> log_cols, c = e & ((1u << log_cols) - 1);
    return (r << log_tile) + (tile << log_cols) + c;
}

// Where the first pass of a transform reads limb i: segment (limb[i] >> 12) at limb offset (limb[i] & 0xFFF);
// the result always lands at data + i*N, and a second pass works in place there.
struct TileSrc {
    const u64* seg[HE_MAX_SEGS];
    uint16_t limb[HE_MAX_LAUNCH_LIMBS];
};

template <bool FWD, bool CUSTOM_SCALE>
__global__ __launch_bounds__(NTT_THREADS) void ntt_tile_kernel(NttArgs a, LimbList ll, ScaleList sc, uint32_t scale_period, TileSrc ts,
                                                               uint32_t gather) {
    __shared__ u64 sm[1u << NTT_LOG_TILE_MAX];
    const uint32_t tile_elems = 1u << a.log_tile;
    const uint32_t tiles_per_limb = 1u << (a.logN - a.log_tile);
    const uint32_t limb = blockIdx.x / tiles_per_limb, tile = blockIdx.x % tiles_per_limb;
    const uint32_t mi = ll.mod[limb];
    if (mi == 0xFFu) return; // limb marked "leave untouched" (uniform for the whole workgroup)
    const ModConst m = a.mc[mi];
    const u64 q = m.q, q2 = m.q2;
    const uint32_t N = 1u << a.logN;
    u64* base = a.data + (size_t)limb * N;
    const u64* tw = a.tw + (size_t)mi * N;
    const u64* tw_sh = a.tw_sh + (size_t)mi * N;
    const uint32_t log_rows = a.logN - a.log_tile; // rows of the strided view

    const u64* in = base;
    if (gather) {
        const uint32_t sl = ts.limb[limb];
        in = ts.seg[sl >> 12] + (size_t)(sl & 0xFFFu) * N;
    }
    for (uint32_t e = threadIdx.x; e < tile_elems; e += NTT_THREADS)
        sm[e] = in[tile_global_index(e, tile, a.log_tile, log_rows, a.strided)];
    __syncthreads();

    const uint32_t half = tile_elems >> 1;
    if (FWD) {
        for (uint32_t s = a.s_begin; s < a.s_end; s++) {
            // global distance t = N >> (s+1); local distance: strided tiles keep 1 of every 2^log_rows..., see header
            uint32_t log_t_local = a.strided ? (a.log_tile - 1 - s) : (a.logN - 1 - s);
            uint32_t t_local = 1u << log_t_local;
            uint32_t groups_in_tile_log = a.log_tile - 1 - log_t_local;
            uint32_t group_base = a.strided ? 0 : (tile << groups_in_tile_log);
            for (uint32_t b = threadIdx.x; b < half; b += NTT_THREADS) {
                uint32_t i = b >> log_t_local, off = b & (t_local - 1);
                uint32_t e0 = (i << (log_t_local + 1)) + off, e1 = e0 + t_local;
                uint32_t k = (1u << s) + group_base + i;
                u64 w = tw[k], w_sh = tw_sh[k];
                u64 x = sm[e0], y = sm[e1];
                x = csub(x, q2);
                u64 v = shoup_lazy(y, w, w_sh, q);
                sm[e0] = x + v;
                sm[e1] = x - v + q2;
            }
            __syncthreads();
        }
    } else {
        for (uint32_t s = a.s_end; s-- > a.s_begin;) {
            uint32_t log_t_local = a.strided ? (a.log_tile - 1 - s) : (a.logN - 1 - s);
            uint32_t t_local = 1u << log_t_local;
            uint32_t groups_in_tile_log = a.log_tile - 1 - log_t_local;
            uint32_t group_base = a.strided ? 0 : (tile << groups_in_tile_log);
            for (uint32_t b = threadIdx.x; b < half; b += NTT_THREADS) {
                uint32_t i = b >> log_t_local, off = b & (t_local - 1);
                uint32_t e0 = (i << (log_t_local + 1)) + off, e1 = e0 + t_local;
                uint32_t k = (1u << s) + group_base + i;
                u64 w = tw[k], w_sh = tw_sh[k];
                u64 x = sm[e0], y = sm[e1];
                sm[e0] = csub(x + y, q2);
                sm[e1] = shoup_lazy(x - y + q2, w, w_sh, q);
            }
            __syncthreads();
        }
    }

    u64 scale = 0, scale_sh = 0;
    if (!FWD && a.last) {
        scale = CUSTOM_SCALE ? sc.s[limb % scale_period] : m.ninv;
        scale_sh = CUSTOM_SCALE ? sc.s_sh[limb % scale_period] : m.ninv_sh;
    }
    for (uint32_t e = threadIdx.x; e < tile_elems; e += NTT_THREADS) {
        u64 v = sm[e];
        if (a.last) {
            if (FWD) v = csub(csub(v, q2), q);
            else v = csub(shoup_lazy(v, scale, scale_sh, q), q);
        }
        base[tile_global_index(e, tile, a.log_tile, log_rows, a.strided)] = v;
    }
}

template <bool FWD>
static int32_t run_transform(he_ctx* ctx, u64* d, const uint32_t* mod_idx, uint32_t n, const ScaleList* scale, uint32_t scale_period,
                             const TileSrc& ts) {
    if (n == 0) return HE_OK;
    if (n > HE_MAX_LAUNCH_LIMBS) return he_fail(ctx, HE_ERR_BADARG, "transform: too many limbs in one launch");
    LimbList ll;
    uint32_t live = 0;
    for (uint32_t i = 0; i < n; i++) {
        if (mod_idx[i] == 0xFFu) { ll.mod[i] = 0xFF; continue; } // internal marker: skip this limb
        if (mod_idx[i] >= ctx->M) return he_fail(ctx, HE_ERR_BADARG, "transform: modulus index %u out of range", mod_idx[i]);
        ll.mod[i] = (uint8_t)mod_idx[i];
        live++;
    }
    ScaleList sc;
    if (scale) sc = *scale;
    NttArgs a;
    a.data = d; a.mc = ctx->d_mc;
    a.tw = FWD ? ctx->d_tw : ctx->d_itw;
    a.tw_sh = FWD ? ctx->d_tw_sh : ctx->d_itw_sh;
    a.logN = ctx->logN;
    a.log_tile = ctx->logN < NTT_LOG_TILE_MAX ? ctx->logN : NTT_LOG_TILE_MAX;
    uint32_t sA = ctx->logN - a.log_tile; // number of strided stages
    dim3 grid(n << (ctx->logN - a.log_tile)), block(NTT_THREADS);
    // forward: pass A (stages 0..sA) then pass B; inverse: pass B then pass A
    uint32_t gather = 1;                                 // only the first pass that runs reads the sources
    for (int pass = 0; pass < 2; pass++) {
        bool strided = FWD ? (pass == 0) : (pass == 1);
        if (strided && sA == 0) continue;
        a.strided = strided ? 1 : 0;
        a.s_begin = strided ? 0 : sA;
        a.s_end = strided ? sA : ctx->logN;
        a.last = (FWD ? !strided : (strided || sA == 0)) ? 1 : 0;
        hipEvent_t e0 = nullptr, e1 = nullptr;
        if (ctx->prof_on) {
            HE_HIP(ctx, hipEventCreate(&e0));
            HE_HIP(ctx, hipEventCreate(&e1));
            HE_HIP(ctx, hipEventRecord(e0, ctx->stream));
        }
        if (scale)
            hipLaunchKernelGGL((ntt_tile_kernel<FWD, true>), grid, block, 0, ctx->stream, a, ll, sc, scale_period ? scale_period : 1u, ts,
                               gather);
        else
            hipLaunchKernelGGL((ntt_tile_kernel<FWD, false>), grid, block, 0, ctx->stream, a, ll, sc, 1u, ts, gather);
        HE_HIP(ctx, hipGetLastError());
        gather = 0;
        if (ctx->prof_on) {
            HE_HIP(ctx, hipEventRecord(e1, ctx->stream));
            ctx->prof_events.push_back({e0, e1, live, 0u, FWD ? (strided ? 0u : 1u) : (strided ? 5u : 3u)});
        }
    }
    if (FWD) ctx->cnt.ntt_limbs += live; else ctx->cnt.intt_limbs += live;
    return HE_OK;
}

// Generic ring sizes: the first pass reads the source limbs where they are; the ModDown epilogue runs as
// its own kernel.
static int32_t launch_transform_generic(he_ctx* ctx, const TransformDesc& d) {
    if (d.rescale_from) return he_fail(ctx, HE_ERR_BADARG, "transform: the Rescale rounding term is only read on the N = 2^16 path");
    TileSrc ts;
    for (uint32_t s = 0; s < HE_MAX_SEGS; s++) ts.seg[s] = s < d.n_seg ? d.seg[s] : d.seg[0];
    for (uint32_t i = 0; i < d.n; i++) {
        uint32_t seg = d.src_seg ? d.src_seg[i] : 0, lim = d.src_limb ? d.src_limb[i] : i;
        if (seg >= HE_MAX_SEGS || seg >= d.n_seg || lim >= 4096) return he_fail(ctx, HE_ERR_BADARG, "transform: source limb out of range");
        ts.limb[i] = (uint16_t)((seg << 12) | lim);
    }
    int32_t rc = d.fwd ? run_transform<true>(ctx, d.dst, d.mod_idx, d.n, nullptr, 1, ts)
                       : run_transform<false>(ctx, d.dst, d.mod_idx, d.n, d.scale, d.scale_period, ts);
    if (rc != HE_OK) return rc;
    if (d.fwd && d.ep) return launch_moddown_final(ctx, d.dst, d.n / (2 * d.ep->L1), *d.ep);
    return HE_OK;
}

int32_t launch_transform(he_ctx* ctx, const TransformDesc& d) {
    if (d.n == 0) return HE_OK;
    if (d.n > HE_MAX_LAUNCH_LIMBS) return he_fail(ctx, HE_ERR_BADARG, "transform: too many limbs in one launch");
    if (d.scale && (d.scale_period == 0 || d.scale_period > HE_MAX_MODULI)) return he_fail(ctx, HE_ERR_BADARG, "transform: bad scale period");
    return ctx->logN == 16 ? launch_transform16(ctx, d) : launch_transform_generic(ctx, d);
}

int32_t launch_ntt(he_ctx* ctx, u64* d, const uint32_t* mod_idx, uint32_t n) {
    TransformDesc t = {};
    t.fwd = true; t.seg[0] = d; t.n_seg = 1; t.dst = d; t.n = n; t.mod_idx = mod_idx;
    return launch_transform(ctx, t);
}
int32_t launch_intt(he_ctx* ctx, u64* d, const uint32_t* mod_idx, uint32_t n, const ScaleList* scale) {
    TransformDesc t = {};
    t.fwd = false; t.seg[0] = d; t.n_seg = 1; t.dst = d; t.n = n; t.mod_idx = mod_idx;
    t.scale = scale; t.scale_period = scale ? n : 0;
    return launch_transform(ctx, t);
}

extern "C" {

int32_t he_ntt(he_ctx* ctx, uint64_t* d_data, const uint32_t* h_mod_idx, uint32_t n_limbs) {
    return he_guard(ctx, "he_ntt: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (n_limbs == 0) return HE_OK;
    if (!d_data || !h_mod_idx) return he_fail(ctx, HE_ERR_BADARG, "he_ntt: null argument");
    for (uint32_t i = 0; i < n_limbs; i++)
        if (h_mod_idx[i] >= ctx->M) return he_fail(ctx, HE_ERR_BADARG, "he_ntt: modulus index %u out of range", h_mod_idx[i]);
    for (uint32_t o = 0; o < n_limbs; o += HE_MAX_LAUNCH_LIMBS) {
        uint32_t n = n_limbs - o < HE_MAX_LAUNCH_LIMBS ? n_limbs - o : HE_MAX_LAUNCH_LIMBS;
        int32_t rc = launch_ntt(ctx, (u64*)d_data + (size_t)o * ctx->N, h_mod_idx + o, n);
        if (rc != HE_OK) return rc;
    }
    return HE_OK;
    });
}

int32_t he_intt(he_ctx* ctx, uint64_t* d_data, const uint32_t* h_mod_idx, uint32_t n_limbs) {
    return he_guard(ctx, "he_intt: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (n_limbs == 0) return HE_OK;
    if (!d_data || !h_mod_idx) return he_fail(ctx, HE_ERR_BADARG, "he_intt: null argument");
    for (uint32_t i = 0; i < n_limbs; i++)
        if (h_mod_idx[i] >= ctx->M) return he_fail(ctx, HE_ERR_BADARG, "he_intt: modulus index %u out of range", h_mod_idx[i]);
    for (uint32_t o = 0; o < n_limbs; o += HE_MAX_LAUNCH_LIMBS) {
        uint32_t n = n_limbs - o < HE_MAX_LAUNCH_LIMBS ? n_limbs - o : HE_MAX_LAUNCH_LIMBS;
        int32_t rc = launch_intt(ctx, (u64*)d_data + (size_t)o * ctx->N, h_mod_idx + o, n, nullptr);
        if (rc != HE_OK) return rc;
    }
    return HE_OK;
    });
}

} // extern "C"
