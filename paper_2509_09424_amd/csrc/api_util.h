// Small host-side helpers shared by the translation units that hold the C ABI.
#pragma once
#include <algorithm>
#include <vector>

#include "common.h"
// ------------------------------------------------------------------ utilities

struct DevBuf {
    void *p = nullptr;
    DevBuf() {}
    DevBuf(const DevBuf &) = delete;
    ~DevBuf() {
        if (p) (void)hipFree(p);
    }
    hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 8); }
    template <class T>
    T *as() { return (T *)p; }
};

template <class T>
inline hipError_t upload(T **d, const std::vector<T> &h) {
    hipError_t e = hipMalloc((void **)d, std::max<size_t>(h.size() * sizeof(T), 8));
    if (e != hipSuccess) return e;
    return hipMemcpy(*d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice);
}

inline LimbMap make_map(const ensi_ctx *ctx, int l1, bool with_p) {
    LimbMap m;
    m.n = l1 + (with_p ? ctx->K : 0);
    for (int e = 0; e < ENSI_MAX_EXT; e++) m.prime[e] = 0;
    for (int e = 0; e < m.n; e++) m.prime[e] = e < l1 ? e : ctx->L + (e - l1);
    return m;
}

inline u32 galois_element(const ensi_ctx *ctx, int32_t step) {
    const int n = ctx->N / 2;
    int k = step % n;
    if (k < 0) k += n;
    return ctx->rot_exp[k];
}
inline u32 inv_mod_2n(u32 g, int N) {
    // g odd: Newton iteration modulo a power of two
    u32 x = g;
    for (int i = 0; i < 5; i++) x *= 2 - g * x;
    return x & (2 * (u32)N - 1);
}

inline int grow(ensi_ctx *ctx, u64 **p, size_t *have, size_t need) {
    if (*have >= need) return ENSI_OK;
    if (*p) ENSI_HIP(ctx, hipFree(*p));
    *p = nullptr;
    *have = 0;
    hipError_t e = hipMalloc((void **)p, need * sizeof(u64));
    if (e != hipSuccess) ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation of %zu bytes failed: %s", need * sizeof(u64), hipGetErrorString(e));
    *have = need;
    return ENSI_OK;
}



// The library's own sampler of small polynomials (api_keys.hip): operating-system randomness when the context's
// seed is 0, a deterministic test generator otherwise.  Return an ENSI_E_* code.
int sample_ternary(ensi_ctx *ctx, int8_t *out, size_t n);
int sample_error(ensi_ctx *ctx, int8_t *out, size_t n);

// dst (device) <- src (host, any memory) on the stream, through the context's ring of pinned buffers: returns at once,
// never waits for the stream, and src may be reused or freed as soon as the call returns.
hipError_t host_to_device(ensi_ctx *ctx, void *dst, const void *src, size_t bytes, hipStream_t st);

// ---- key switching, shared by the entry points (api.hip) -------------------------------------------------
// Intermediates of a batch of key switches: raised digits (raised_words per ciphertext), accumulators
// (2 (l1+K) N words per rotation), inner factors of the basis conversion (l1 N per ciphertext, fused path),
// centred special-limb residues (2 K N per rotation, fused path).
struct KsWorkspace {
    u64 *digits, *u, *y, *ysp;
};
size_t raised_words(const ensi_ctx *ctx, int l1);
int get_modup(ensi_ctx *ctx, int l1, const ModUpConst **out);
int get_moddown(ensi_ctx *ctx, int l1, const ModDownConst **out);
int get_ks16(ensi_ctx *ctx, int l1, const Ks16Const **out);
int raise_cts(ensi_ctx *ctx, int l1, const u64 *ct_base, size_t ct_stride_words, int limb_stride, int n_ct, hipStream_t st,
              const KsWorkspace *ws = nullptr);
int run_rotations(ensi_ctx *ctx, const RotDesc *d_desc, int n_rot, int l1, int limb_stride_in, int limb_stride_out, hipStream_t st,
                  int members = 1, const RotDesc *h_desc = nullptr, const KsWorkspace *ws = nullptr);

// Resolves the device address of the statically linked workspace for the context's device (api_static.hip).
int ensi_static_init(ensi_ctx *ctx);
// Allocates every slot of the staging ring and its event now, so that later small uploads allocate nothing.
int stage_prealloc(ensi_ctx *ctx);

// ---- helpers defined in one translation unit of the C ABI and used by others ---------------------------------
// api.hip
int encode_window(ensi_ctx *ctx, const double *slots, int n_pt, int n_slots, int slot0, int slot_step, int limbs, double scale,
                  ensi_pt **out);
int rot_chunk();                           // ciphertexts per group of a batched rotation
int ensure_desc(ensi_ctx *ctx, size_t n);  // grows the context's descriptor table to n entries
// api_matmul.hip
void free_plan(MatmulPlan *p);
// Constants of the scalar-multiply + rescale step at l1 limbs (integer set and fp64 set), uploaded to the context's
// small-constants workspace; kr = the integer the limbs are multiplied by before the division (1: plain rescale).
int upload_rescale_consts(ensi_ctx *ctx, int l1, double kr, bool negative, hipStream_t st, const u64 **d_consts, const double **d_fconsts,
                          bool *fp_out);
// api_pmult.hip: out_o = Rescale(sum of the terms [begin[o], begin[o+1]) of src (x) plaintext)
int pmult_core(ensi_ctx *ctx, const std::vector<PmTerm> &terms_in, const std::vector<int32_t> &begin, int l1, int limb_stride_in,
               const ensi_pt *pt, ensi_ct *out, hipStream_t st);
