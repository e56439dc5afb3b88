// An entry point that allocates nothing, for callers that cannot call hipMalloc: code under HIP graph capture,
// tight serving loops, harnesses that forbid allocation.  It is ensi_rotate on a workspace that is not allocated
// but linked: a file-scope device array of fixed size, which every GPU the library runs on holds from the moment
// the code object is loaded until the process ends.
#include <string.h>

#include "api_util.h"
#include "common.h"

// 96 MiB: one ciphertext of the N = 2^16 ring at up to 16 + 4 limbs in four digits (80 MiB of intermediates), or a
// batch at smaller parameters.
#define ENSI_STATIC_SCRATCH_BYTES ((size_t)96 << 20)
#define ENSI_STATIC_MAX_BATCH 64
#define ENSI_STATIC_MAX_DEVICES 64

static __device__ __align__(256) unsigned char scratch[ENSI_STATIC_SCRATCH_BYTES];

// In host code the array's name is only a handle for the runtime: the device address of each GPU's copy comes from
// hipGetSymbolAddress, asked once per device with that device current, and is what kernels and copies are given.
static void *scratch_of_device[ENSI_STATIC_MAX_DEVICES];

int ensi_static_init(ensi_ctx *ctx) {
    ctx->static_scratch = nullptr;
    ctx->static_scratch_bytes = 0;
    if (ctx->device < 0 || ctx->device >= ENSI_STATIC_MAX_DEVICES) return ENSI_OK;  // the static entry point will refuse
    if (!scratch_of_device[ctx->device]) {
        int cur = -1;
        if (hipGetDevice(&cur) != hipSuccess || cur != ctx->device) ENSI_FAIL(ctx, ENSI_E_HIP, "the context's device is not current");
        void *ptr = nullptr;
        hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) ENSI_FAIL(ctx, ENSI_E_HIP, "hipGetSymbolAddress of the static workspace failed: %s", hipGetErrorString(e));
        scratch_of_device[ctx->device] = ptr;
    }
    ctx->static_scratch = scratch_of_device[ctx->device];
    ctx->static_scratch_bytes = ENSI_STATIC_SCRATCH_BYTES;
    return ENSI_OK;
}

extern "C" int ensi_rotate_static(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *in, const int32_t *steps, ensi_ct *out, void *stream) {
    if (!ctx || !gk || !in || !steps || !out) return ENSI_E_BADARG;
    if (in->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "a batch of prepared weights is read by ensi_ccmm_segment and ensi_ccmm_av only");
    if (in->n != out->n) ENSI_FAIL(ctx, ENSI_E_SHAPE, "rotate: batch sizes differ (%d vs %d)", in->n, out->n);
    if (in->limbs != out->limbs) ENSI_FAIL(ctx, ENSI_E_LEVEL, "rotate: levels differ (%d vs %d limbs)", in->limbs, out->limbs);
    if (in->d == out->d) ENSI_FAIL(ctx, ENSI_E_BADARG, "rotate: in and out must not overlap");
    if (!ctx->static_scratch) ENSI_FAIL(ctx, ENSI_E_HIP, "the static workspace is not available on this device");
    if (ctx->profiling) ENSI_FAIL(ctx, ENSI_E_BADARG, "the per-kernel timers create events: switch them off for the allocation-free call");
    hipStream_t st = (hipStream_t)stream;
    const int N = ctx->N, l1 = in->limbs, ext = l1 + ctx->K, n = in->n;
    // workspace layout inside the static array: descriptors, then the four arrays of the key switch
    const size_t rw = raised_words(ctx, l1);
    const size_t desc_bytes = (((size_t)n * sizeof(RotDesc)) + 255) & ~(size_t)255;
    const size_t w_digits = (size_t)n * rw, w_u = (size_t)n * 2 * ext * N, w_y = (size_t)n * l1 * N, w_ysp = (size_t)n * 2 * ctx->K * N;
    const size_t need = desc_bytes + (w_digits + w_u + w_y + w_ysp) * sizeof(u64);
    if (n > ENSI_STATIC_MAX_BATCH || need > ctx->static_scratch_bytes)
        ENSI_FAIL(ctx, ENSI_E_SHAPE, "rotate_static: %d ciphertexts at %d limbs need %zu bytes of workspace; the static workspace holds %zu (at most %d per call)",
                  n, l1, need, ctx->static_scratch_bytes, ENSI_STATIC_MAX_BATCH);
    // the constants of every level were built when the context was created; a missing set would mean an allocation here
    if (ctx->ks16 ? !ctx->ks16c.count(l1) : (!ctx->modup.count(l1) || !ctx->moddown.count(l1)))
        ENSI_FAIL(ctx, ENSI_E_LEVEL, "no key-switch constants for %d limbs", l1);
    unsigned char *base = (unsigned char *)ctx->static_scratch;
    RotDesc *d_desc = (RotDesc *)base;
    KsWorkspace ws;
    ws.digits = (u64 *)(base + desc_bytes);
    ws.u = ws.digits + w_digits;
    ws.y = ws.u + w_u;
    ws.ysp = ws.y + w_y;
    RotDesc desc[ENSI_STATIC_MAX_BATCH];
    const size_t in_ct = (size_t)2 * in->limbs_alloc * N, out_ct = (size_t)2 * out->limbs_alloc * N;
    for (int c = 0; c < n; c++) {
        const u32 g = galois_element(ctx, steps[c]);
        auto it = gk->keys.find(g);
        if (it == gk->keys.end()) ENSI_FAIL(ctx, ENSI_E_NOKEY, "rotate: no Galois key for step %d", steps[c]);
        memset(&desc[c], 0, sizeof(RotDesc));
        desc[c].c0 = in->d + (size_t)c * in_ct;
        desc[c].digits = ws.digits + (size_t)c * rw;
        desc[c].key = it->second;
        desc[c].out = out->d + (size_t)c * out_ct;
        desc[c].g = g;
        desc[c].g_inv = inv_mod_2n(g, N);
    }
    // through the pinned ring the context allocated at creation (a slot holds 64 KiB, the descriptors at most 3 KiB)
    if ((size_t)n * sizeof(RotDesc) > ctx->stage[ctx->stage_next].cap) ENSI_FAIL(ctx, ENSI_E_SHAPE, "descriptor table larger than a staging slot");
    ENSI_HIP(ctx, host_to_device(ctx, d_desc, desc, (size_t)n * sizeof(RotDesc), st));
    int rc;
    // every word of the workspace that a kernel reads is written earlier in this same call (digits and inner factors by the
    // raise, accumulators by the inner product, special-limb residues by the first ModDown kernel): nothing has to start at zero
    if ((rc = raise_cts(ctx, l1, in->d, in_ct, in->limbs_alloc, n, st, &ws))) return rc;
    if ((rc = run_rotations(ctx, d_desc, n, l1, in->limbs_alloc, out->limbs_alloc, st, 1, nullptr, &ws))) return rc;
    out->scale = in->scale;
    ENSI_HIP(ctx, hipGetLastError());
    return ENSI_OK;
}
