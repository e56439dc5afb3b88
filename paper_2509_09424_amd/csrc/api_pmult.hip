// Host side of the plaintext multiplication summed and rescaled once, and of what stands on it: the merge of
// block-placed outputs and the secure RoPE protocol (Alg. 2).
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <set>

#include "api_util.h"
#include "common.h"
#include "hostmath.h"

// ------------------------------------------------------- plaintext multiplication
extern "C" int ensi_set_pmult_mode(ensi_ctx *ctx, int32_t mode) {
    if (!ctx || mode < 0 || mode > 1) return ENSI_E_BADARG;
    ctx->pmult_mode = mode;
    return ENSI_OK;
}

// Builds the multiplier form of a plaintext batch on first use: transform domain, Montgomery residues (generic
// kernels) or doubles in the register order of the row pass (N = 2^16 kernels).
static int pt_prepare(ensi_ctx *ctx, const ensi_pt *pt, bool fused, hipStream_t st) {
    if (fused ? pt->d_fp != nullptr : pt->d_mont != nullptr) return ENSI_OK;
    const int rows = pt->n * pt->limbs;
    const size_t bytes = (size_t)rows * ctx->N * 8;
    u64 *buf = nullptr;
    if (hipMalloc((void **)&buf, bytes) != hipSuccess) ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation failed for the transformed plaintext");
    const LimbMap map = make_map(ctx, pt->limbs, false);
    hipError_t e = hipMemcpyAsync(buf, pt->d, bytes, hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess) {
        launch_ntt(ctx, buf, rows, map, false, st);
        if (fused) {
            u64 *f = nullptr;
            if (hipMalloc((void **)&f, bytes) != hipSuccess) {
                (void)hipFree(buf);
                ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation failed for the transformed plaintext");
            }
            launch_pm16_pt_format(ctx, buf, rows, f, st);
            e = hipStreamSynchronize(st);
            (void)hipFree(buf);
            buf = nullptr;
            if (e == hipSuccess) pt->d_fp = f;
            else (void)hipFree(f);
        } else {
            launch_to_mont(ctx, buf, rows, map, st);
            e = hipGetLastError();
            if (e == hipSuccess) pt->d_mont = buf;
        }
    }
    if (e != hipSuccess) {
        if (buf) (void)hipFree(buf);
        ENSI_FAIL(ctx, ENSI_E_HIP, "plaintext transform failed: %s", hipGetErrorString(e));
    }
    return ENSI_OK;
}

// out_o = Rescale(sum_{t in [begin[o], begin[o+1])} src_t (x) pt_t) for every output o; sources have l1 limbs at
// stride limb_stride_in.  Outputs are handled in groups whose transformed sources fit a bounded workspace.
int pmult_core(ensi_ctx *ctx, const std::vector<PmTerm> &terms_in, const std::vector<int32_t> &begin, int l1, int limb_stride_in,
                      const ensi_pt *pt, ensi_ct *out, hipStream_t st) {
    std::vector<PmTerm> terms(terms_in);  // the slots are filled in below
    const int N = ctx->N, n_out = (int)begin.size() - 1;
    if (l1 < 2) ENSI_FAIL(ctx, ENSI_E_LEVEL, "plaintext multiplication: no limb left to drop");
    if (pt->limbs < l1) ENSI_FAIL(ctx, ENSI_E_LEVEL, "plaintext has %d limbs, ciphertexts have %d", pt->limbs, l1);
    if (out->limbs != l1 - 1) ENSI_FAIL(ctx, ENSI_E_LEVEL, "output must be one level below the input (%d vs %d limbs)", out->limbs, l1);
    if (out->n != n_out) ENSI_FAIL(ctx, ENSI_E_SHAPE, "output batch holds %d ciphertexts, need %d", out->n, n_out);
    for (const PmTerm &t : terms)
        if (t.pt < 0 || t.pt >= pt->n) ENSI_FAIL(ctx, ENSI_E_BADARG, "plaintext index %d outside the batch of %d", t.pt, pt->n);
    const bool fused = ctx->ks16 && ctx->pmult_mode != 1;
    int rc;
    if ((rc = pt_prepare(ctx, pt, fused, st))) return rc;

    // groups of outputs: at most 8 GiB of transformed sources and of sums, at least one output.  Per group its distinct
    // sources are numbered in order of first use: a source that enters several products (one ciphertext under several
    // masks) is transformed once.
    const size_t term_words = (size_t)2 * l1 * N;
    // a group's sources index one grid dimension of the transform kernels (at most 65535)
    const size_t max_src = std::min<size_t>(65535, std::max<size_t>(1, ((size_t)1 << 30) / term_words));
    for (int o = 0; o < n_out; o++)
        if (begin[o + 1] - begin[o] > 65535) ENSI_FAIL(ctx, ENSI_E_SHAPE, "output %d sums %d products, at most 65535", o, begin[o + 1] - begin[o]);
    std::vector<int> cut(1, 0);
    std::vector<int32_t> owner;
    std::vector<size_t> owner_base(1, 0);
    size_t need_a = 1, need_b = 0;
    for (int o0 = 0; o0 < n_out;) {
        std::map<const u64 *, int> slot;
        int o1 = o0;
        for (; o1 < n_out && (size_t)(o1 - o0) < max_src; o1++) {
            if (o1 > o0) {  // would this output's new sources still fit?
                std::set<const u64 *> fresh;
                for (int t = begin[o1]; t < begin[o1 + 1]; t++)
                    if (!slot.count(terms[t].src)) fresh.insert(terms[t].src);
                if (slot.size() + fresh.size() > max_src) break;
            }
            for (int t = begin[o1]; t < begin[o1 + 1]; t++) {
                auto it = slot.emplace(terms[t].src, (int)slot.size());
                if (it.second) owner.push_back(t);
                terms[t].slot = it.first->second;
            }
        }
        cut.push_back(o1);
        owner_base.push_back(owner.size());
        need_a = std::max(need_a, slot.size());
        need_b = std::max(need_b, (size_t)(o1 - o0));
        o0 = o1;
    }
    if ((rc = grow(ctx, &ctx->ws_pa, &ctx->ws_pa_words, need_a * term_words))) return rc;
    if ((rc = grow(ctx, &ctx->ws_pb, &ctx->ws_pb_words, need_b * term_words))) return rc;
    if ((rc = grow(ctx, &ctx->ws_pl, &ctx->ws_pl_words, need_b * 2 * N))) return rc;
    const size_t tw = terms.size() * (sizeof(PmTerm) / 8), bw = (begin.size() + 1) / 2, ow = (owner.size() + 1) / 2;
    if ((rc = grow(ctx, &ctx->ws_pt, &ctx->ws_pt_words, tw + bw + ow + 2))) return rc;
    if (!terms.empty()) ENSI_HIP(ctx, host_to_device(ctx, ctx->ws_pt, terms.data(), terms.size() * sizeof(PmTerm), st));
    ENSI_HIP(ctx, host_to_device(ctx, ctx->ws_pt + tw, begin.data(), begin.size() * 4, st));
    if (!owner.empty()) ENSI_HIP(ctx, host_to_device(ctx, ctx->ws_pt + tw + bw, owner.data(), owner.size() * 4, st));

    const u64 ql = ctx->primes[l1 - 1];
    PmRescale rs;
    const u64 *d_consts = nullptr;
    const double *d_fconsts = nullptr;
    if (fused) {
        for (int i = 0; i < ENSI_MAX_EXT; i++) rs.w[i] = rs.wp[i] = 0.0;
        for (int i = 0; i < l1 - 1; i++) {
            const u64 q = ctx->primes[i];
            rs.w[i] = (double)hm_invmod(ql % q, q);
            rs.wp[i] = rs.w[i] / (double)q;
        }
    } else {
        bool fp;
        if ((rc = upload_rescale_consts(ctx, l1, 1.0, false, st, &d_consts, &d_fconsts, &fp))) return rc;
        if (!fp) d_fconsts = nullptr;
    }
    for (size_t k = 0; k + 1 < cut.size(); k++) {
        const int o0 = cut[k], o1 = cut[k + 1];
        PmGroup g;
        g.terms = (const PmTerm *)ctx->ws_pt;
        g.begin = (const int32_t *)(ctx->ws_pt + tw) + o0;
        g.t_base = begin[o0];
        g.n_terms = begin[o1] - begin[o0];
        g.n_out = o1 - o0;
        g.owner = (const int32_t *)(ctx->ws_pt + tw + bw) + owner_base[k];
        g.n_src = (int)(owner_base[k + 1] - owner_base[k]);
        g.l1 = l1;
        g.limb_stride_in = limb_stride_in;
        g.pt = fused ? pt->d_fp : pt->d_mont;
        g.pt_limbs = pt->limbs;
        g.ws_a = ctx->ws_pa;
        g.ws_b = ctx->ws_pb;
        g.ws_last = ctx->ws_pl;
        g.out_stride = (size_t)2 * out->limbs_alloc * N;
        g.out = out->d + (size_t)o0 * g.out_stride;
        g.limb_stride_out = out->limbs_alloc;
        if (fused) launch_pm16(ctx, g, rs, st);
        else launch_pm_generic(ctx, g, d_consts, d_fconsts, st);
    }
    ENSI_HIP(ctx, hipGetLastError());
    return ENSI_OK;
}

extern "C" int ensi_pmult_sum_rescale(ensi_ctx *ctx, const ensi_ct *in, const ensi_pt *pt, const int32_t *begin, const int32_t *term_ct,
                                      const int32_t *term_pt, int32_t n_out, ensi_ct *out, void *stream) {
    if (!ctx || !in || !pt || !begin || !out || n_out < 1) return ENSI_E_BADARG;
    if (in->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "a batch of prepared weights is read by ensi_ccmm_segment and ensi_ccmm_av only");
    if (begin[0] != 0) ENSI_FAIL(ctx, ENSI_E_BADARG, "term offsets must start at 0");
    for (int o = 0; o < n_out; o++)
        if (begin[o + 1] < begin[o]) ENSI_FAIL(ctx, ENSI_E_BADARG, "term offsets must not decrease");
    const int T = begin[n_out];
    if (T > 0 && (!term_ct || !term_pt)) return ENSI_E_BADARG;
    if (in->d == out->d) ENSI_FAIL(ctx, ENSI_E_BADARG, "plaintext multiplication: in and out must not overlap");
    const size_t in_ct = (size_t)2 * in->limbs_alloc * ctx->N;
    std::vector<PmTerm> terms(T);
    for (int t = 0; t < T; t++) {
        if (term_ct[t] < 0 || term_ct[t] >= in->n) ENSI_FAIL(ctx, ENSI_E_BADARG, "term %d names ciphertext %d of %d", t, term_ct[t], in->n);
        terms[t].src = in->d + (size_t)term_ct[t] * in_ct;
        terms[t].pt = term_pt[t];
        terms[t].slot = 0;
    }
    std::vector<int32_t> b(begin, begin + n_out + 1);
    int rc;
    if ((rc = pmult_core(ctx, terms, b, in->limbs, in->limbs_alloc, pt, out, (hipStream_t)stream))) return rc;
    out->scale = in->scale * pt->scale / (double)ctx->primes[in->limbs - 1];
    return ENSI_OK;
}

// ------------------------------------------------------------ merge of placed outputs
extern "C" int ensi_block_masks(ensi_ctx *ctx, int32_t s, int32_t c_tot, int32_t limbs, ensi_pt **out) {
    if (!ctx || !out || s < 1 || c_tot < 1 || limbs < 2 || limbs > ctx->L) return ENSI_E_BADARG;
    if ((int64_t)s * c_tot > ctx->N / 2) ENSI_FAIL(ctx, ENSI_E_SHAPE, "%d blocks of %d slots exceed the %d slots", c_tot, s, ctx->N / 2);
    std::vector<double> ones((size_t)c_tot * s, 1.0);
    return encode_window(ctx, ones.data(), c_tot, s, 0, s, limbs, (double)ctx->primes[limbs - 1], out);
}

extern "C" int ensi_merge(ensi_ctx *ctx, const ensi_ct *in, const ensi_pt *masks, int32_t c_tot, ensi_ct *out, void *stream) {
    if (!ctx || !in || !masks || !out || c_tot < 1) return ENSI_E_BADARG;
    if (in->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "a batch of prepared weights is read by ensi_ccmm_segment and ensi_ccmm_av only");
    if (masks->n < c_tot) ENSI_FAIL(ctx, ENSI_E_SHAPE, "merge: %d masks for %d blocks", masks->n, c_tot);
    if (in->d == out->d) ENSI_FAIL(ctx, ENSI_E_BADARG, "merge: in and out must not overlap");
    const int n_out = (in->n + c_tot - 1) / c_tot;
    const size_t in_ct = (size_t)2 * in->limbs_alloc * ctx->N;
    std::vector<PmTerm> terms(in->n);
    std::vector<int32_t> begin(n_out + 1);
    for (int i = 0; i < in->n; i++) terms[i] = {in->d + (size_t)i * in_ct, i % c_tot, 0};
    for (int o = 0; o <= n_out; o++) begin[o] = std::min(o * c_tot, in->n);
    int rc;
    if ((rc = pmult_core(ctx, terms, begin, in->limbs, in->limbs_alloc, masks, out, (hipStream_t)stream))) return rc;
    out->scale = in->scale * masks->scale / (double)ctx->primes[in->limbs - 1];
    return ENSI_OK;
}

// --------------------------------------------------------------------- Alg. 2 (RoPE)
extern "C" int ensi_rope_plaintexts(ensi_ctx *ctx, const double *cos_v, const double *sin_v, int32_t n_slots, int32_t limbs, ensi_pt **out) {
    if (!ctx || !cos_v || !sin_v || !out || n_slots < 1 || n_slots > ctx->N / 2 || limbs < 2 || limbs > ctx->L) return ENSI_E_BADARG;
    // cos, neg (.) sin, pos (.) sin with neg = (-1,0,-1,0,...), pos = (0,1,0,1,...): selections, no arithmetic
    std::vector<double> v((size_t)3 * n_slots);
    for (int j = 0; j < n_slots; j++) {
        v[j] = cos_v[j];
        v[(size_t)n_slots + j] = (j & 1) ? 0.0 : -sin_v[j];
        v[(size_t)2 * n_slots + j] = (j & 1) ? sin_v[j] : 0.0;
    }
    return encode_window(ctx, v.data(), 3, n_slots, 0, 0, limbs, (double)ctx->primes[limbs - 1], out);
}

extern "C" int ensi_rope(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *in, const ensi_pt *pt, ensi_ct *out, void *stream) {
    if (!ctx || !gk || !in || !pt || !out) return ENSI_E_BADARG;
    if (in->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "a batch of prepared weights is read by ensi_ccmm_segment and ensi_ccmm_av only");
    if (pt->n < 3) ENSI_FAIL(ctx, ENSI_E_SHAPE, "rope: the plaintext batch must hold cos, neg*sin and pos*sin");
    if (in->n != out->n) ENSI_FAIL(ctx, ENSI_E_SHAPE, "rope: batch sizes differ (%d vs %d)", in->n, out->n);
    if (in->limbs < 2 || out->limbs != in->limbs - 1) ENSI_FAIL(ctx, ENSI_E_LEVEL, "rope: output must be one level below the input");
    if (in->d == out->d) ENSI_FAIL(ctx, ENSI_E_BADARG, "rope: in and out must not overlap");
    hipStream_t st = (hipStream_t)stream;
    const int N = ctx->N, l1 = in->limbs, ext = l1 + ctx->K, n = in->n, ls = in->limbs_alloc;
    const int steps[2] = {1, -1};
    u32 g[2];
    const u64 *key[2];
    for (int e = 0; e < 2; e++) {
        g[e] = galois_element(ctx, steps[e]);
        auto it = gk->keys.find(g[e]);
        if (it == gk->keys.end()) ENSI_FAIL(ctx, ENSI_E_NOKEY, "rope: no Galois key for step %d", steps[e]);
        key[e] = it->second;
    }
    const int chunk = std::min(n, rot_chunk() / 2);
    const size_t rw = raised_words(ctx, l1), ct_words = (size_t)2 * ls * N;
    int rc;
    if ((rc = grow(ctx, &ctx->ws_digits, &ctx->ws_digits_words, (size_t)chunk * rw))) return rc;
    if ((rc = grow(ctx, &ctx->ws_u, &ctx->ws_u_words, (size_t)2 * chunk * 2 * ext * N))) return rc;
    if ((rc = grow(ctx, &ctx->ws_rot, &ctx->ws_rot_words, (size_t)2 * chunk * ct_words))) return rc;
    if ((rc = ensure_desc(ctx, (size_t)2 * chunk))) return rc;
    const size_t out_ct = (size_t)2 * out->limbs_alloc * N;
    ensi_ct part = *out;  // a window of the output batch
    part.owns = false;
    for (int c0 = 0; c0 < n; c0 += chunk) {
        const int cnt = std::min(chunk, n - c0);
        // both rotations of every input share that input's raised digits; rotations by the same key are neighbours
        std::vector<RotDesc> desc(2 * cnt);
        for (int e = 0; e < 2; e++)
            for (int k = 0; k < cnt; k++) {
                RotDesc &d = desc[e * cnt + k];
                d.c0 = in->d + (size_t)(c0 + k) * ct_words;
                d.digits = ctx->ws_digits + (size_t)k * rw;
                d.key = key[e];
                d.out = ctx->ws_rot + (size_t)(2 * k + e) * ct_words;
                d.g = g[e];
                d.g_inv = inv_mod_2n(g[e], N);
            }
        ENSI_HIP(ctx, host_to_device(ctx, ctx->ws_desc, desc.data(), desc.size() * sizeof(RotDesc), st));
        if ((rc = raise_cts(ctx, l1, in->d + (size_t)c0 * ct_words, ct_words, ls, cnt, st))) return rc;
        if ((rc = run_rotations(ctx, ctx->ws_desc, 2 * cnt, l1, ls, ls, st))) return rc;
        // y = q (x) cos + Rot(q; 1) (x) (neg sin) + Rot(q; -1) (x) (pos sin), rescaled once
        std::vector<PmTerm> terms(3 * cnt);
        std::vector<int32_t> begin(cnt + 1);
        for (int k = 0; k < cnt; k++) {
            begin[k] = 3 * k;
            terms[3 * k] = {in->d + (size_t)(c0 + k) * ct_words, 0, 0};
            terms[3 * k + 1] = {ctx->ws_rot + (size_t)(2 * k) * ct_words, 1, 0};
            terms[3 * k + 2] = {ctx->ws_rot + (size_t)(2 * k + 1) * ct_words, 2, 0};
        }
        begin[cnt] = 3 * cnt;
        part.d = out->d + (size_t)c0 * out_ct;
        part.n = cnt;
        if ((rc = pmult_core(ctx, terms, begin, l1, ls, pt, &part, st))) return rc;
    }
    out->scale = in->scale * pt->scale / (double)ctx->primes[l1 - 1];
    ENSI_HIP(ctx, hipGetLastError());
    return ENSI_OK;
}

