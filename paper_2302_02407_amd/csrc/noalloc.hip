// Entry point for callers that cannot allocate device memory (code under HIP graph capture, tight
// serving loops, harnesses that forbid hipMalloc): he_rescale_noalloc is he_rescale with its scratch
// (the coefficient form of the dropped limb and the per-limb correction terms) taken from a fixed
// device array instead of the context's growable workspace.
#include "he_internal.h"

// (2 + 2*level) * N residues are needed: 16 MiB covers level <= 15 at N = 2^16 and every level of the
// smaller rings.  Each GPU the library runs on holds its own copy until the process ends.
#define HE_NOALLOC_SCRATCH_ELEMS ((size_t)HE_NOALLOC_SCRATCH_BYTES / sizeof(u64))
static __device__ __align__(256) u64 scratch[HE_NOALLOC_SCRATCH_ELEMS];

// The array's name is only a host-side handle; its device address differs per GPU and is looked up once
// per device (with that device current) and kept here.
#define HE_NOALLOC_MAX_DEVICES 64
static u64* g_scratch_ptr[HE_NOALLOC_MAX_DEVICES];

int32_t he_noalloc_init_device(he_ctx* ctx, int device) {
    if (device < 0 || device >= HE_NOALLOC_MAX_DEVICES) return he_fail(ctx, HE_ERR_BADARG, "device index %d out of range", device);
    if (g_scratch_ptr[device]) return HE_OK;
    int cur = -1;
    HE_HIP(ctx, hipGetDevice(&cur));
    if (cur != device) return he_fail(ctx, HE_ERR_BADARG, "device %d is not the current device (%d)", device, cur);
    u64* ptr = nullptr;
    HE_HIP(ctx, hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return he_fail(ctx, HE_ERR_HIP, "hipGetSymbolAddress returned a null address for the static scratch array");
    g_scratch_ptr[device] = ptr;
    return HE_OK;
}

extern "C" int32_t he_rescale_noalloc(he_ctx* ctx, const uint64_t* d_ct, uint32_t level, uint64_t* d_out) {
    return he_guard(ctx, "he_rescale_noalloc: host allocation failed", [&]() -> int32_t {
    if (!ctx) return HE_ERR_BADARG;
    if (!d_ct || !d_out) return he_fail(ctx, HE_ERR_BADARG, "he_rescale_noalloc: null argument");
    if (level == 0 || level >= ctx->nq) return he_fail(ctx, HE_ERR_LEVEL, "he_rescale_noalloc: level %u outside 1..%u", level, ctx->nq - 1);
    const size_t N = ctx->N;
    const size_t need = rescale_ws_elems(ctx, level, 1);
    if (need > HE_NOALLOC_SCRATCH_ELEMS)
        return he_fail(ctx, HE_ERR_BADARG, "he_rescale_noalloc: level %u at N=%zu needs %zu bytes of scratch, the static array holds %zu",
                       level, N, need * sizeof(u64), (size_t)HE_NOALLOC_SCRATCH_BYTES);
    if (ctx->prof_on) return he_fail(ctx, HE_ERR_BADARG, "he_rescale_noalloc: launch timing is on (it creates events); call he_profile_end first");
    {
        const char *a = (const char*)d_out, *b = (const char*)d_ct;
        if (a < b + 2 * (level + 1) * N * sizeof(u64) && b < a + 2 * level * N * sizeof(u64))
            return he_fail(ctx, HE_ERR_BADARG, "he_rescale_noalloc: output overlaps the input");
    }
    int32_t rc = he_noalloc_init_device(ctx, ctx->device);   // already done by he_ctx_create; a lookup otherwise
    if (rc != HE_OK) return rc;
    u64* ptr = g_scratch_ptr[ctx->device];
    // every scratch element that is read has been written earlier in the same call (the inverse transform
    // writes the coefficient form, the correction kernel writes every term before it is transformed), so
    // nothing has to be cleared between calls
    const u64* cts[1] = {(const u64*)d_ct};
    u64* outs[1] = {(u64*)d_out};
    return rescale_batch(ctx, cts, outs, 1, level, ptr);
    });
}
