// Host side of Mult (tensor products, relinearisation, rescale) and of the CCMM section: element extraction and the
// ciphertext-ciphertext matrix products in their several forms.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <set>

#include "api_util.h"
#include "common.h"
#include "hostmath.h"

// ----------------------------------------------- ciphertext-ciphertext products
extern "C" int ensi_ct_drop_limbs(ensi_ct *ct, int32_t limbs) {
    if (!ct || limbs < 1 || limbs > ct->limbs) return ENSI_E_BADARG;
    ct->limbs = limbs;
    return ENSI_OK;
}

// out_o = Rescale(Relin(sum_{t in [begin[o], begin[o+1])} a_t (x) b_t)); operands have l1 limbs.  Outputs are
// handled in groups of at most one rotation chunk whose operand polynomials fit a bounded workspace.
// a_pre: the a operands already hold their transform (limb stride l1): they are read in place.  rescale = false stops
// after the relinearisation: the outputs keep l1 limbs and the product's scale.
// grid_x, grid_y > 0: the caller states that output x * grid_y + y sums a_(j,x) (x) b_(j,y) over j, with every output's terms
// in the same order of j; where the fp64 kernels apply and the outputs make one group, the tiled multiply-add is used.
static int mult_core(ensi_ctx *ctx, const u64 *rkey, const std::vector<MmTerm> &terms, const std::vector<int32_t> &begin, int l1,
                     int limb_stride_a, int limb_stride_b, ensi_ct *out, hipStream_t st, bool a_pre = false, bool rescale = true,
                     int grid_x = 0, int grid_y = 0) {
    const int N = ctx->N, n_out = (int)begin.size() - 1, ext = l1 + ctx->K;
    if (l1 < 2) ENSI_FAIL(ctx, ENSI_E_LEVEL, "ciphertext multiplication: no limb left to drop");
    if (out->limbs != (rescale ? l1 - 1 : l1))
        ENSI_FAIL(ctx, ENSI_E_LEVEL, "output must be %s the operands (%d vs %d limbs)", rescale ? "one level below" : "at the level of", out->limbs, l1);
    if (out->n != n_out) ENSI_FAIL(ctx, ENSI_E_SHAPE, "output batch holds %d ciphertexts, need %d", out->n, n_out);
    for (int o = 0; o < n_out; o++)
        if (begin[o + 1] - begin[o] > 65535) ENSI_FAIL(ctx, ENSI_E_SHAPE, "output %d sums %d products, at most 65535", o, begin[o + 1] - begin[o]);
    // groups of outputs: at most 24 GiB of transformed operands (a group's distinct operand ciphertexts, by address:
    // one that enters several products is gathered and transformed once), at most 65535 products, at least one output
    const size_t max_ops = std::max<size_t>(2, ((size_t)3 << 30) / ((size_t)2 * l1 * N));
    // (a grid of up to 256 outputs is kept in one group, so that the tiled multiply-add applies)
    const int max_out = (grid_x > 0 && grid_x * grid_y == n_out && n_out <= 256) ? std::max(n_out, 64) : ctx->ks16 ? rot_chunk() : 64;
    if (a_pre && limb_stride_a != l1) ENSI_FAIL(ctx, ENSI_E_LEVEL, "prepared operands have %d limbs, the product runs at %d", limb_stride_a, l1);
    std::vector<int> cut(1, 0);
    std::vector<MmOperand> ops;
    std::vector<MmPair> pairs(terms.size());
    std::vector<size_t> op_base(1, 0);
    std::vector<int> n_gather;  // per group: operands to gather and transform (they come first in the group's list)
    size_t need_a = 1, need_o = 0;
    for (int o0 = 0; o0 < n_out;) {
        std::map<std::pair<const u64 *, int>, int> id;
        std::vector<MmOperand> gops;
        int o1 = o0, n_np = 0;
        for (; o1 < n_out && o1 - o0 < max_out && begin[o1 + 1] - begin[o0] <= 65535; o1++) {
            if (o1 > o0) {  // would this output's new operands still fit?
                std::map<std::pair<const u64 *, int>, int> fresh;
                for (int t = begin[o1]; t < begin[o1 + 1]; t++) {
                    const auto ka = std::make_pair(terms[t].a, terms[t].stride_a ? terms[t].stride_a : limb_stride_a), kb = std::make_pair(terms[t].b, limb_stride_b);
                    if (!a_pre && !id.count(ka)) fresh.emplace(ka, 0);
                    if (!id.count(kb)) fresh.emplace(kb, 0);
                }
                if ((size_t)n_np + fresh.size() > max_ops) break;
            }
            for (int t = begin[o1]; t < begin[o1 + 1]; t++) {
                const int sa = terms[t].stride_a ? terms[t].stride_a : limb_stride_a;
                auto ia = id.emplace(std::make_pair(terms[t].a, sa), (int)id.size());
                if (ia.second) {
                    gops.push_back({terms[t].a, nullptr, sa, a_pre ? 1 : 0});
                    n_np += a_pre ? 0 : 1;
                }
                auto ib = id.emplace(std::make_pair(terms[t].b, limb_stride_b), (int)id.size());
                if (ib.second) {
                    gops.push_back({terms[t].b, nullptr, limb_stride_b, 0});
                    n_np++;
                }
                pairs[t] = {ia.first->second, ib.first->second};
            }
        }
        // operands to transform first, prepared ones after them
        std::vector<int> where(gops.size());
        int at_np = 0, at_pre = n_np;
        for (size_t u = 0; u < gops.size(); u++) where[u] = gops[u].pre ? at_pre++ : at_np++;
        std::vector<MmOperand> sorted(gops.size());
        for (size_t u = 0; u < gops.size(); u++) sorted[where[u]] = gops[u];
        for (int t = begin[o0]; t < begin[o1]; t++) pairs[t] = {where[pairs[t].a], where[pairs[t].b]};
        ops.insert(ops.end(), sorted.begin(), sorted.end());
        n_gather.push_back(n_np);
        cut.push_back(o1);
        op_base.push_back(ops.size());
        need_a = std::max(need_a, (size_t)n_np);
        need_o = std::max(need_o, (size_t)(o1 - o0));
        o0 = o1;
    }
    int rc;
    const size_t rw = raised_words(ctx, l1);
    if ((rc = grow(ctx, &ctx->ws_ma, &ctx->ws_ma_words, need_a * 2 * l1 * N))) return rc;
    if ((rc = grow(ctx, &ctx->ws_md, &ctx->ws_md_words, need_o * 3 * l1 * N))) return rc;
    if ((rc = grow(ctx, &ctx->ws_me, &ctx->ws_me_words, need_o * 2 * l1 * N))) return rc;
    if ((rc = grow(ctx, &ctx->ws_digits, &ctx->ws_digits_words, need_o * rw))) return rc;
    if ((rc = grow(ctx, &ctx->ws_u, &ctx->ws_u_words, need_o * 2 * ext * N))) return rc;
    if ((rc = ensure_desc(ctx, need_o))) return rc;
    for (size_t k = 0; k + 1 < op_base.size(); k++)
        for (size_t u = op_base[k]; u < op_base[k + 1]; u++)
            ops[u].t = ops[u].pre ? ops[u].p : ctx->ws_ma + (u - op_base[k]) * 2 * l1 * N;
    const size_t ow = ops.size() * (sizeof(MmOperand) / 8), pw = pairs.size() * (sizeof(MmPair) / 8), bw = (begin.size() + 1) / 2;
    if ((rc = grow(ctx, &ctx->ws_mt, &ctx->ws_mt_words, ow + pw + bw + 2))) return rc;
    if (!ops.empty()) ENSI_HIP(ctx, host_to_device(ctx, ctx->ws_mt, ops.data(), ops.size() * sizeof(MmOperand), st));
    if (!pairs.empty()) ENSI_HIP(ctx, host_to_device(ctx, ctx->ws_mt + ow, pairs.data(), pairs.size() * sizeof(MmPair), st));
    ENSI_HIP(ctx, host_to_device(ctx, ctx->ws_mt + ow + pw, begin.data(), begin.size() * 4, st));
    const u64 *d_consts;
    const double *d_fconsts;
    bool fp;
    if ((rc = upload_rescale_consts(ctx, l1, 1.0, false, st, &d_consts, &d_fconsts, &fp))) return rc;
    for (size_t k = 0; k + 1 < cut.size(); k++) {
        const int o0 = cut[k], o1 = cut[k + 1], cnt = o1 - o0;
        MmGroup g;
        g.ops = (const MmOperand *)ctx->ws_mt + op_base[k];
        g.pairs = (const MmPair *)(ctx->ws_mt + ow) + begin[o0];
        g.begin = (const int32_t *)(ctx->ws_mt + ow + pw) + o0;
        g.t_base = begin[o0];
        g.n_terms = begin[o1] - begin[o0];
        g.n_ops = n_gather[k];
        g.n_out = cnt;
        g.l1 = l1;
        g.limbs_out = rescale ? l1 - 1 : l1;
        g.grid_x = g.grid_y = 0;
        bool even = grid_x > 0 && grid_y > 0 && cut.size() == 2 && grid_x * grid_y == n_out && ctx->ks16 && n_out > 0;
        for (int o = 1; o < n_out && even; o++) even = begin[o + 1] - begin[o] == begin[1] - begin[0];
        if (even && begin[1] > begin[0]) {
            g.grid_x = grid_x;
            g.grid_y = grid_y;
        }
        g.ws_a = ctx->ws_ma;
        g.ws_d = ctx->ws_md;
        g.ws_e = ctx->ws_me;
        g.out_stride = (size_t)2 * out->limbs_alloc * N;
        g.out = out->d + (size_t)o0 * g.out_stride;
        g.limb_stride_out = out->limbs_alloc;
        launch_mm_tensor(ctx, g, st);
        // relinearisation: (d0, d2) of every output goes through the key switch like a ciphertext (c0, c1) under
        // the identity automorphism; the result is (d0 + KS_0(d2), KS_1(d2))
        std::vector<RotDesc> desc(cnt);
        for (int c = 0; c < cnt; c++) {
            desc[c].c0 = ctx->ws_md + (size_t)c * 3 * l1 * N;
            desc[c].digits = ctx->ws_digits + (size_t)c * rw;
            desc[c].key = rkey;
            desc[c].out = ctx->ws_me + (size_t)c * 2 * l1 * N;
            desc[c].g = 1;
            desc[c].g_inv = 1;
        }
        ENSI_HIP(ctx, host_to_device(ctx, ctx->ws_desc, desc.data(), cnt * sizeof(RotDesc), st));
        if ((rc = raise_cts(ctx, l1, ctx->ws_md, (size_t)3 * l1 * N, l1, cnt, st))) return rc;
        if ((rc = run_rotations(ctx, ctx->ws_desc, cnt, l1, l1, l1, st))) return rc;
        launch_mm_add_d1(ctx, g, st);
        if (rescale) launch_rescale(ctx, ctx->ws_me, cnt, l1, l1, d_consts, fp ? d_fconsts : nullptr, st);
        launch_mm_scatter(ctx, g, st);
    }
    ENSI_HIP(ctx, hipGetLastError());
    return ENSI_OK;
}

static int relin_key(ensi_ctx *ctx, const ensi_gk *rk, const u64 **key) {
    auto it = rk->keys.find(1u);
    if (it == rk->keys.end()) ENSI_FAIL(ctx, ENSI_E_NOKEY, "the key set holds no evaluation key (ensi_relin_keygen)");
    *key = it->second;
    return ENSI_OK;
}

extern "C" int ensi_mult_sum_relin_rescale(ensi_ctx *ctx, const ensi_gk *rk, const ensi_ct *a, const ensi_ct *b, const int32_t *begin,
                                           const int32_t *term_a, const int32_t *term_b, int32_t n_out, ensi_ct *out, void *stream) {
    if (!ctx || !rk || !a || !b || !begin || !out || n_out < 1) return ENSI_E_BADARG;
    if (a->prepared || b->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "a batch of prepared weights is read by ensi_ccmm_segment and ensi_ccmm_av only");
    if (a->limbs != b->limbs) ENSI_FAIL(ctx, ENSI_E_LEVEL, "operands at different levels (%d vs %d limbs)", a->limbs, b->limbs);
    if (begin[0] != 0) ENSI_FAIL(ctx, ENSI_E_BADARG, "term offsets must start at 0");
    for (int o = 0; o < n_out; o++)
        if (begin[o + 1] < begin[o]) ENSI_FAIL(ctx, ENSI_E_BADARG, "term offsets must not decrease");
    const int T = begin[n_out];
    if (T > 0 && (!term_a || !term_b)) return ENSI_E_BADARG;
    if (a->d == out->d || b->d == out->d) ENSI_FAIL(ctx, ENSI_E_BADARG, "ciphertext multiplication: operands and out must not overlap");
    const u64 *key;
    int rc;
    if ((rc = relin_key(ctx, rk, &key))) return rc;
    const size_t a_ct = (size_t)2 * a->limbs_alloc * ctx->N, b_ct = (size_t)2 * b->limbs_alloc * ctx->N;
    std::vector<MmTerm> terms(T);
    for (int t = 0; t < T; t++) {
        if (term_a[t] < 0 || term_a[t] >= a->n || term_b[t] < 0 || term_b[t] >= b->n)
            ENSI_FAIL(ctx, ENSI_E_BADARG, "term %d names ciphertexts %d of %d and %d of %d", t, term_a[t], a->n, term_b[t], b->n);
        terms[t].a = a->d + (size_t)term_a[t] * a_ct;
        terms[t].b = b->d + (size_t)term_b[t] * b_ct;
    }
    std::vector<int32_t> bg(begin, begin + n_out + 1);
    if ((rc = mult_core(ctx, key, terms, bg, a->limbs, a->limbs_alloc, b->limbs_alloc, out, (hipStream_t)stream))) return rc;
    out->scale = a->scale * b->scale / (double)ctx->primes[a->limbs - 1];
    return ENSI_OK;
}

// ------------------------------------------------------------------------ CCMM
extern "C" int ensi_one_hot_masks(ensi_ctx *ctx, int32_t count, int32_t limbs, ensi_pt **out) {
    if (!ctx || !out || count < 1 || count > ctx->N / 2 || limbs < 2 || limbs > ctx->L) return ENSI_E_BADARG;
    std::vector<double> ones(count, 1.0);
    return encode_window(ctx, ones.data(), count, 1, 0, 1, limbs, (double)ctx->primes[limbs - 1], out);
}

// The rotate-and-add fill t <- sum_{e < r_end / r_begin} Rot(t; sign * e * r_begin): groups of steps taken together.
// While two doublings remain they are one step of radix four, t <- t + Rot(t; r) + Rot(t; 2r) + Rot(t; 3r), whose
// three rotations share one ModUp of t; a last single doubling is t <- t + Rot(t; r).
static std::vector<std::vector<int>> fill_groups(int r_begin, int r_end, int sign) {
    std::vector<std::vector<int>> groups;
    for (int r = r_begin; r < r_end;) {
        if (2 * r < r_end) {
            groups.push_back({sign * r, sign * 2 * r, sign * 3 * r});
            r *= 4;
        } else {
            groups.push_back({sign * r});
            r *= 2;
        }
    }
    return groups;
}

extern "C" int ensi_fill_steps(int32_t r_begin, int32_t r_end, int32_t sign, int32_t *steps_out, int32_t cap) {
    if (r_begin < 1 || r_end < r_begin || (sign != 1 && sign != -1) || (cap > 0 && !steps_out)) return ENSI_E_BADARG;
    int n = 0;
    for (const auto &grp : fill_groups(r_begin, r_end, sign))
        for (int st : grp) {
            if (n < cap) steps_out[n] = st;
            n++;
        }
    return n;
}

// The fill in place on a batch.  The rotations of a group share the raise of t and are switched back together (one
// inverse transform and one ModDown per group).  On the fused path the last key-switch kernel adds the group's
// result to t directly (legal in place: every read of t happens in the raise kernels); otherwise the group's
// result goes through a workspace and is added by a separate kernel.
static int doubling_steps(ensi_ctx *ctx, const ensi_gk *gk, ensi_ct *t, int r_begin, int r_end, hipStream_t st, int sign = 1) {
    const int N = ctx->N, n = t->n, l1 = t->limbs, ext = l1 + ctx->K;
    const auto groups = fill_groups(r_begin, r_end, sign);
    if (groups.empty()) return ENSI_OK;
    int rc;
    const bool fused = ctx->ks16;
    const int chunk = std::min(n, fused ? rot_chunk() : 16);
    const size_t rw = raised_words(ctx, l1), ct_words = (size_t)2 * t->limbs_alloc * N, tmp_words = (size_t)2 * l1 * N;
    if ((rc = grow(ctx, &ctx->ws_digits, &ctx->ws_digits_words, (size_t)chunk * rw))) return rc;
    if ((rc = grow(ctx, &ctx->ws_u, &ctx->ws_u_words, (size_t)chunk * 3 * 2 * ext * N))) return rc;
    if (!fused && (rc = grow(ctx, &ctx->ws_rtmp, &ctx->ws_rtmp_words, (size_t)chunk * tmp_words))) return rc;
    // descriptors of all groups in one copy; per group and chunk: ciphertext c, member e at base + c * members + e
    std::vector<RotDesc> desc;
    std::vector<size_t> base;  // per (group, chunk) in launch order
    for (const auto &grp : groups) {
        std::vector<std::pair<u32, const u64 *>> gk_of;
        for (int step : grp) {
            const u32 g = galois_element(ctx, step);
            auto it = gk->keys.find(g);
            if (it == gk->keys.end()) ENSI_FAIL(ctx, ENSI_E_NOKEY, "no Galois key for step %d", step);
            gk_of.push_back({g, it->second});
        }
        for (int c0 = 0; c0 < n; c0 += chunk) {
            base.push_back(desc.size());
            for (int c = c0; c < std::min(n, c0 + chunk); c++)
                for (const auto &ge : gk_of) {
                    RotDesc d = {};
                    d.c0 = t->d + (size_t)c * ct_words;
                    d.digits = ctx->ws_digits + (size_t)(c - c0) * rw;
                    d.key = ge.second;
                    d.out = fused ? t->d + (size_t)c * ct_words : ctx->ws_rtmp + (size_t)(c - c0) * tmp_words;
                    d.g = ge.first;
                    d.g_inv = inv_mod_2n(ge.first, N);
                    d.accumulate = fused ? 1 : 0;
                    desc.push_back(d);
                }
        }
    }
    if ((rc = ensure_desc(ctx, desc.size()))) return rc;
    ENSI_HIP(ctx, host_to_device(ctx, ctx->ws_desc, desc.data(), desc.size() * sizeof(RotDesc), st));
    size_t k = 0;
    for (const auto &grp : groups) {
        const int members = (int)grp.size();
        for (int c0 = 0; c0 < n; c0 += chunk, k++) {
            const int cnt = std::min(chunk, n - c0);
            if ((rc = raise_cts(ctx, l1, t->d + (size_t)c0 * ct_words, ct_words, t->limbs_alloc, cnt, st))) return rc;
            if ((rc = run_rotations(ctx, ctx->ws_desc + base[k], cnt * members, l1, t->limbs_alloc, fused ? t->limbs_alloc : l1, st, members,
                                    desc.data() + base[k])))
                return rc;
            if (!fused) launch_ct_add(ctx, t->d + (size_t)c0 * ct_words, t->limbs_alloc, ctx->ws_rtmp, l1, l1, cnt, st);
        }
    }
    return ENSI_OK;
}

// rep_o = Rescale(in[src[o]] (x) masks[mask_idx[o]]): n ciphertexts with in.limbs - 1 limbs
static int mask_rescale(ensi_ctx *ctx, const ensi_ct *in, const std::vector<int32_t> &src, const ensi_pt *masks,
                        const std::vector<int32_t> &mask_idx, ensi_ct *rep, hipStream_t st) {
    const int N = ctx->N, n = (int)src.size(), l1 = in->limbs;
    const size_t in_ct = (size_t)2 * in->limbs_alloc * N;
    std::vector<PmTerm> terms(n);
    std::vector<int32_t> begin(n + 1);
    for (int o = 0; o < n; o++) {
        if (src[o] < 0 || src[o] >= in->n) ENSI_FAIL(ctx, ENSI_E_BADARG, "ciphertext index %d outside the batch of %d", src[o], in->n);
        terms[o] = {in->d + (size_t)src[o] * in_ct, mask_idx[o], 0};
        begin[o] = o;
    }
    begin[n] = n;
    int rc;
    if ((rc = pmult_core(ctx, terms, begin, l1, in->limbs_alloc, masks, rep, st))) return rc;
    rep->scale = in->scale * masks->scale / (double)ctx->primes[l1 - 1];
    return ENSI_OK;
}

// rep_o = the value in slot mask_idx[o] of in[src[o]], copied into every slot: one product with the one-hot mask
// and one rescale, then log2(N/2) steps t <- t + Rot(t; 2^r).
static int replicate_core(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *in, const std::vector<int32_t> &src, const ensi_pt *masks,
                          const std::vector<int32_t> &mask_idx, ensi_ct *rep, hipStream_t st) {
    int rc;
    if ((rc = mask_rescale(ctx, in, src, masks, mask_idx, rep, st))) return rc;
    return doubling_steps(ctx, gk, rep, 1, ctx->N / 2, st);
}

extern "C" int ensi_replicate(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *in, const int32_t *src, const ensi_pt *masks,
                              const int32_t *mask_idx, int32_t n_out, ensi_ct *out, void *stream) {
    if (!ctx || !gk || !in || !src || !masks || !mask_idx || !out || n_out < 1) return ENSI_E_BADARG;
    if (in->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "a batch of prepared weights is read by ensi_ccmm_segment and ensi_ccmm_av only");
    if (in->limbs < 2 || out->limbs != in->limbs - 1) ENSI_FAIL(ctx, ENSI_E_LEVEL, "replicate: output must be one level below the input");
    if (out->n != n_out) ENSI_FAIL(ctx, ENSI_E_SHAPE, "replicate: output batch holds %d ciphertexts, need %d", out->n, n_out);
    if (in->d == out->d) ENSI_FAIL(ctx, ENSI_E_BADARG, "replicate: in and out must not overlap");
    std::vector<int32_t> s(src, src + n_out), mi(mask_idx, mask_idx + n_out);
    int rc = replicate_core(ctx, gk, in, s, masks, mi, out, (hipStream_t)stream);
    if (rc) return rc;
    ENSI_HIP(ctx, hipGetLastError());
    return ENSI_OK;
}

extern "C" int ensi_periodic_masks(ensi_ctx *ctx, int32_t period, int32_t count, int32_t limbs, ensi_pt **out) {
    if (!ctx || !out || period < 1 || (period & (period - 1)) || period > ctx->N / 2 || count < 1 || count > period || limbs < 2 || limbs > ctx->L)
        return ENSI_E_BADARG;
    const int n = ctx->N / 2;
    std::vector<double> z((size_t)count * n, 0.0);
    for (int j = 0; j < count; j++)
        for (int p = j; p < n; p += period) z[(size_t)j * n + p] = 1.0;
    return encode_window(ctx, z.data(), count, n, 0, 0, limbs, (double)ctx->primes[limbs - 1], out);
}

extern "C" int ensi_ccmm(ensi_ctx *ctx, const ensi_gk *rk, const ensi_gk *gk, const ensi_ct *A, const ensi_ct *B, const ensi_pt *masks,
                         int32_t period, ensi_ct *out, void *stream) {
    if (!ctx || !rk || !gk || !A || !B || !masks || !out) return ENSI_E_BADARG;
    if (A->prepared || B->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "a batch of prepared weights is read by ensi_ccmm_segment and ensi_ccmm_av only");
    const int N = ctx->N, d = A->n, m = B->n, l1 = B->limbs;
    if (period < 1 || (period & (period - 1)) || period > N / 2 || period < d)
        ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: the period must be a power of two between the inner dimension %d and %d", d, N / 2);
    if (A->limbs != l1) ENSI_FAIL(ctx, ENSI_E_LEVEL, "ccmm: A and B at different levels (%d vs %d limbs)", A->limbs, l1);
    if (l1 < 3 || out->limbs != l1 - 2) ENSI_FAIL(ctx, ENSI_E_LEVEL, "ccmm: output must be two levels below the operands");
    if (out->n != m) ENSI_FAIL(ctx, ENSI_E_SHAPE, "ccmm: output batch holds %d ciphertexts, need %d", out->n, m);
    if (masks->n < d) ENSI_FAIL(ctx, ENSI_E_SHAPE, "ccmm: %d masks for %d rows of B", masks->n, d);
    if (A->d == out->d || B->d == out->d) ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: operands and out must not overlap");
    hipStream_t st = (hipStream_t)stream;
    const u64 *key;
    int rc;
    if ((rc = relin_key(ctx, rk, &key))) return rc;
    const int lo = l1 - 1;
    // outputs in groups: up to `per` columns of B at a time, their d replicated elements side by side
    const int per = std::max(1, std::min(m, 512 / d));
    const size_t u_words = (size_t)per * 2 * l1 * N;
    if ((rc = grow(ctx, &ctx->ws_rep, &ctx->ws_rep_words, u_words + (size_t)per * d * 2 * lo * N))) return rc;
    const size_t a_ct = (size_t)2 * A->limbs_alloc * N, b_ct = (size_t)2 * B->limbs_alloc * N, out_ct = (size_t)2 * out->limbs_alloc * N;
    for (int i0 = 0; i0 < m; i0 += per) {
        const int cnt = std::min(per, m - i0);
        // giant steps, once per column: u[p] = b[p mod period]
        ensi_ct u;
        u.ctx = ctx;
        u.n = cnt;
        u.limbs = u.limbs_alloc = l1;
        u.scale = B->scale;
        u.d = ctx->ws_rep;
        u.owns = false;
        for (int c = 0; c < cnt; c++)
            for (int poly = 0; poly < 2; poly++)
                ENSI_HIP(ctx, hipMemcpyAsync(u.d + ((size_t)c * 2 + poly) * l1 * N, B->d + (size_t)(i0 + c) * b_ct + (size_t)poly * B->limbs_alloc * N,
                                             (size_t)l1 * N * 8, hipMemcpyDeviceToDevice, st));
        if ((rc = doubling_steps(ctx, gk, &u, period, N / 2, st))) return rc;
        // baby steps, per element: mask the slots congruent to j, fill every window of `period` slots
        ensi_ct rep;
        rep.ctx = ctx;
        rep.n = cnt * d;
        rep.limbs = rep.limbs_alloc = lo;
        rep.scale = 1.0;
        rep.d = ctx->ws_rep + u_words;
        rep.owns = false;
        std::vector<int32_t> src(cnt * d), mi(cnt * d);
        for (int c = 0; c < cnt; c++)
            for (int j = 0; j < d; j++) {
                src[c * d + j] = c;
                mi[c * d + j] = j;
            }
        if ((rc = mask_rescale(ctx, &u, src, masks, mi, &rep, st))) return rc;
        if ((rc = doubling_steps(ctx, gk, &rep, 1, period, st))) return rc;
        // c_i = sum_j a_j (x) rep_(i,j); a_j is read at the level of the replicated elements (its last limb dropped)
        std::vector<MmTerm> terms(cnt * d);
        std::vector<int32_t> begin(cnt + 1);
        for (int c = 0; c < cnt; c++) {
            begin[c] = c * d;
            for (int j = 0; j < d; j++) terms[c * d + j] = {A->d + (size_t)j * a_ct, rep.d + (size_t)(c * d + j) * 2 * lo * N};
        }
        begin[cnt] = cnt * d;
        ensi_ct part = *out;
        part.owns = false;
        part.d = out->d + (size_t)i0 * out_ct;
        part.n = cnt;
        if ((rc = mult_core(ctx, key, terms, begin, lo, A->limbs_alloc, lo, &part, st))) return rc;
        out->scale = A->scale * rep.scale / (double)ctx->primes[lo - 1];
    }
    ENSI_HIP(ctx, hipGetLastError());
    return ENSI_OK;
}

// --------------------------------------------- CCMM, several heads per ciphertext
extern "C" int ensi_block_start_mask(ensi_ctx *ctx, int32_t s, int32_t limbs, ensi_pt **out) {
    if (!ctx || !out || s < 1 || (s & (s - 1)) || s > ctx->N / 2 || limbs < 2 || limbs > ctx->L) return ENSI_E_BADARG;
    const int n = ctx->N / 2;
    std::vector<double> z(n, 0.0);
    for (int p = 0; p < n; p += s) z[p] = 1.0;
    return encode_window(ctx, z.data(), 1, n, 0, 0, limbs, (double)ctx->primes[limbs - 1], out);
}

// out[c * d + j] = Rot(B_j; cols[c]) for c < cnt, j < d: the d ciphertexts of B are raised in groups of up to 16 and
// every group serves all its rotations (rotations by the same amount, hence the same key, are neighbours).  A
// column index 0 is a plain copy.  out: cnt * d ciphertexts at limb stride l1.
static int rotate_columns(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *B, const int32_t *cols, int cnt, u64 *out, hipStream_t st) {
    const int N = ctx->N, d = B->n, l1 = B->limbs, ext = l1 + ctx->K;
    const size_t b_ct = (size_t)2 * B->limbs_alloc * N, o_ct = (size_t)2 * l1 * N, rw = raised_words(ctx, l1);
    const int GS = std::min(d, 16), per = std::max(1, rot_chunk() * 2 / GS);  // rotation amounts per launch
    int rc;
    if ((rc = grow(ctx, &ctx->ws_digits, &ctx->ws_digits_words, (size_t)GS * rw))) return rc;
    if ((rc = grow(ctx, &ctx->ws_u, &ctx->ws_u_words, (size_t)GS * per * 2 * ext * N))) return rc;
    if ((rc = ensure_desc(ctx, (size_t)GS * per))) return rc;
    std::vector<const u64 *> key(cnt, nullptr);
    std::vector<u32> gel(cnt, 1);
    for (int c = 0; c < cnt; c++) {
        if (cols[c] == 0) continue;
        gel[c] = galois_element(ctx, cols[c]);
        auto it = gk->keys.find(gel[c]);
        if (it == gk->keys.end()) ENSI_FAIL(ctx, ENSI_E_NOKEY, "no Galois key for step %d", cols[c]);
        key[c] = it->second;
    }
    for (int j0 = 0; j0 < d; j0 += GS) {
        const int gs = std::min(GS, d - j0);
        bool raised = false;
        for (int c0 = 0; c0 < cnt; c0 += per) {
            std::vector<RotDesc> desc;
            for (int c = c0; c < std::min(cnt, c0 + per); c++)
                for (int j = 0; j < gs; j++) {
                    u64 *dst = out + (size_t)(c * d + j0 + j) * o_ct;
                    const u64 *src = B->d + (size_t)(j0 + j) * b_ct;
                    if (cols[c] == 0) {
                        for (int poly = 0; poly < 2; poly++)
                            ENSI_HIP(ctx, hipMemcpyAsync(dst + (size_t)poly * l1 * N, src + (size_t)poly * B->limbs_alloc * N, (size_t)l1 * N * 8,
                                                         hipMemcpyDeviceToDevice, st));
                        continue;
                    }
                    RotDesc r = {};
                    r.c0 = src;
                    r.digits = ctx->ws_digits + (size_t)j * rw;
                    r.key = key[c];
                    r.out = dst;
                    r.g = gel[c];
                    r.g_inv = inv_mod_2n(gel[c], N);
                    desc.push_back(r);
                }
            if (desc.empty()) continue;
            if (!raised) {
                if ((rc = raise_cts(ctx, l1, B->d + (size_t)j0 * b_ct, b_ct, B->limbs_alloc, gs, st))) return rc;
                raised = true;
            }
            ENSI_HIP(ctx, host_to_device(ctx, ctx->ws_desc, desc.data(), desc.size() * sizeof(RotDesc), st));
            if ((rc = run_rotations(ctx, ctx->ws_desc, (int)desc.size(), l1, B->limbs_alloc, l1, st))) return rc;
        }
    }
    return ENSI_OK;
}

extern "C" int ensi_ccmm_blocks(ensi_ctx *ctx, const ensi_gk *rk, const ensi_gk *gk, const ensi_ct *A, const ensi_ct *B, int32_t s,
                                const int32_t *cols, int32_t n_cols, const ensi_pt *mask, ensi_ct *out, void *stream) {
    if (!ctx || !rk || !gk || !A || !B || !cols || !mask || !out || n_cols < 1) return ENSI_E_BADARG;
    if (A->prepared || B->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "a batch of prepared weights is read by ensi_ccmm_segment and ensi_ccmm_av only");
    const int N = ctx->N, d = A->n, l1 = B->limbs;
    if (s < 1 || (s & (s - 1)) || s > N / 2) ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: the block length must be a power of two up to %d", N / 2);
    if (B->n != d) ENSI_FAIL(ctx, ENSI_E_SHAPE, "ccmm: A has %d columns, B has %d rows", d, B->n);
    if (A->limbs != l1) ENSI_FAIL(ctx, ENSI_E_LEVEL, "ccmm: A and B at different levels (%d vs %d limbs)", A->limbs, l1);
    if (l1 < 3 || out->limbs != l1 - 2) ENSI_FAIL(ctx, ENSI_E_LEVEL, "ccmm: output must be two levels below the operands");
    if (out->n != n_cols) ENSI_FAIL(ctx, ENSI_E_SHAPE, "ccmm: output batch holds %d ciphertexts, need %d", out->n, n_cols);
    for (int c = 0; c < n_cols; c++)
        if (cols[c] < 0 || cols[c] >= s) ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: output column %d outside a block of %d", cols[c], s);
    if (A->d == out->d || B->d == out->d) ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: operands and out must not overlap");
    hipStream_t st = (hipStream_t)stream;
    const u64 *key;
    int rc;
    if ((rc = relin_key(ctx, rk, &key))) return rc;
    const int lo = l1 - 1;
    const int per = std::max(1, std::min((int)n_cols, 512 / d));
    if ((rc = grow(ctx, &ctx->ws_rot, &ctx->ws_rot_words, (size_t)per * d * 2 * l1 * N))) return rc;
    if ((rc = grow(ctx, &ctx->ws_rep, &ctx->ws_rep_words, (size_t)per * d * 2 * lo * N))) return rc;
    const size_t a_ct = (size_t)2 * A->limbs_alloc * N, out_ct = (size_t)2 * out->limbs_alloc * N;
    for (int i0 = 0; i0 < n_cols; i0 += per) {
        const int cnt = std::min(per, n_cols - i0);
        // slot i of every block to the block's first slot
        if ((rc = rotate_columns(ctx, gk, B, cols + i0, cnt, ctx->ws_rot, st))) return rc;
        ensi_ct al;
        al.ctx = ctx;
        al.n = cnt * d;
        al.limbs = al.limbs_alloc = l1;
        al.scale = B->scale;
        al.d = ctx->ws_rot;
        al.owns = false;
        // keep the block starts, then fill every block upwards
        ensi_ct rep = al;
        rep.limbs = rep.limbs_alloc = lo;
        rep.d = ctx->ws_rep;
        std::vector<int32_t> src(cnt * d), mi(cnt * d, 0);
        for (int k = 0; k < cnt * d; k++) src[k] = k;
        if ((rc = mask_rescale(ctx, &al, src, mask, mi, &rep, st))) return rc;
        if ((rc = doubling_steps(ctx, gk, &rep, 1, s, st, -1))) return rc;
        std::vector<MmTerm> terms(cnt * d);
        std::vector<int32_t> begin(cnt + 1);
        for (int c = 0; c < cnt; c++) {
            begin[c] = c * d;
            for (int j = 0; j < d; j++) terms[c * d + j] = {A->d + (size_t)j * a_ct, rep.d + (size_t)(c * d + j) * 2 * lo * N};
        }
        begin[cnt] = cnt * d;
        ensi_ct part = *out;
        part.owns = false;
        part.d = out->d + (size_t)i0 * out_ct;
        part.n = cnt;
        if ((rc = mult_core(ctx, key, terms, begin, lo, A->limbs_alloc, lo, &part, st))) return rc;
        out->scale = A->scale * rep.scale / (double)ctx->primes[lo - 1];
    }
    ENSI_HIP(ctx, hipGetLastError());
    return ENSI_OK;
}

// ---------------------- CCMM, several heads per ciphertext, extraction in giant and baby steps
extern "C" int ensi_block_head_mask(ensi_ctx *ctx, int32_t s, int32_t period, int32_t limbs, ensi_pt **out) {
    if (!ctx || !out || s < 1 || (s & (s - 1)) || s > ctx->N / 2 || period < 1 || (period & (period - 1)) || period > s || limbs < 2 ||
        limbs > ctx->L)
        return ENSI_E_BADARG;
    const int n = ctx->N / 2;
    std::vector<double> z(n, 0.0);
    for (int p = 0; p < n; p += s)
        for (int x = 0; x < period; x++) z[p + x] = 1.0;
    return encode_window(ctx, z.data(), 1, n, 0, 0, limbs, (double)ctx->primes[limbs - 1], out);
}

struct RotJob {
    int src;       // index into the source batch
    int32_t step;  // rotation amount; 0 = copy
    u64 *dst;      // destination ciphertext, limb stride l1
};

// dst_k = Rot(src batch[job.src]; job.step) for every job: the sources are raised in groups of up to 16 neighbours
// and each raise serves all the rotations of its ciphertexts (jobs of a group ordered by amount, so that rotations
// with the same key are neighbours).  Source batch: ciphertext stride src_ct words, limb stride limb_stride_in.
static int rotate_jobs(ensi_ctx *ctx, const ensi_gk *gk, const u64 *src, size_t src_ct, int limb_stride_in, int n_src, int l1,
                       std::vector<RotJob> jobs, hipStream_t st) {
    const int N = ctx->N, ext = l1 + ctx->K;
    const size_t rw = raised_words(ctx, l1);
    const int GS = 16, per = std::max(1, rot_chunk() * 2 / GS);
    int rc;
    if ((rc = grow(ctx, &ctx->ws_digits, &ctx->ws_digits_words, (size_t)GS * rw))) return rc;
    if ((rc = grow(ctx, &ctx->ws_u, &ctx->ws_u_words, (size_t)GS * per * 2 * ext * N))) return rc;
    if ((rc = ensure_desc(ctx, (size_t)GS * per))) return rc;
    for (const RotJob &j : jobs)
        if (j.src < 0 || j.src >= n_src) ENSI_FAIL(ctx, ENSI_E_BADARG, "rotation source %d outside the batch of %d", j.src, n_src);
    std::stable_sort(jobs.begin(), jobs.end(), [&](const RotJob &a, const RotJob &b) {
        const int ga = a.src / GS, gb = b.src / GS;
        return ga != gb ? ga < gb : a.step != b.step ? a.step < b.step : a.src < b.src;
    });
    for (size_t k0 = 0; k0 < jobs.size();) {
        const int grp = jobs[k0].src / GS;
        size_t k1 = k0;
        int lo = n_src, hi = -1;
        bool any = false;
        while (k1 < jobs.size() && jobs[k1].src / GS == grp) {
            if (jobs[k1].step) {
                lo = std::min(lo, jobs[k1].src);
                hi = std::max(hi, jobs[k1].src);
                any = true;
            }
            k1++;
        }
        if (any && (rc = raise_cts(ctx, l1, src + (size_t)lo * src_ct, src_ct, limb_stride_in, hi - lo + 1, st))) return rc;
        std::vector<RotDesc> desc;
        auto flush = [&]() -> int {
            if (desc.empty()) return ENSI_OK;
            if (host_to_device(ctx, ctx->ws_desc, desc.data(), desc.size() * sizeof(RotDesc), st) != hipSuccess)
                ENSI_FAIL(ctx, ENSI_E_HIP, "descriptor copy failed");
            const int r = run_rotations(ctx, ctx->ws_desc, (int)desc.size(), l1, limb_stride_in, l1, st);
            desc.clear();
            return r;
        };
        for (size_t k = k0; k < k1; k++) {
            const RotJob &j = jobs[k];
            const u64 *from = src + (size_t)j.src * src_ct;
            if (j.step == 0) {
                for (int poly = 0; poly < 2; poly++)
                    ENSI_HIP(ctx, hipMemcpyAsync(j.dst + (size_t)poly * l1 * N, from + (size_t)poly * limb_stride_in * N, (size_t)l1 * N * 8,
                                                 hipMemcpyDeviceToDevice, st));
                continue;
            }
            const u32 g = galois_element(ctx, j.step);
            auto it = gk->keys.find(g);
            if (it == gk->keys.end()) ENSI_FAIL(ctx, ENSI_E_NOKEY, "no Galois key for step %d", j.step);
            RotDesc r = {};
            r.c0 = from;
            r.digits = ctx->ws_digits + (size_t)(j.src - lo) * rw;
            r.key = it->second;
            r.out = j.dst;
            r.g = g;
            r.g_inv = inv_mod_2n(g, N);
            desc.push_back(r);
            if ((int)desc.size() == GS * per && (rc = flush())) return rc;
        }
        if ((rc = flush())) return rc;
        k0 = k1;
    }
    return ENSI_OK;
}

// Giant steps of the block-wise extraction: for every (ciphertext b of B, segment g) of `segs`, Rot(b; g period) brings
// the segment to the start of every block, the head mask keeps its `period` slots (one product, one rescale) and the
// fill with steps -period, -2 period, ... repeats it through the block.  seg: a view whose storage (segs.size()
// ciphertexts at B.limbs - 1 limbs) the caller provides; ws_rot must hold segs.size() ciphertexts at B.limbs limbs.
static int spread_segments(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *B, const std::vector<std::pair<int, int>> &segs, int s, int period,
                           const ensi_pt *mask_head, ensi_ct *seg, hipStream_t st) {
    const int S = (int)segs.size(), N = ctx->N, l1 = B->limbs;
    seg->n = S;
    if (!S) return ENSI_OK;
    int r;
    std::vector<RotJob> jobs(S);
    for (int k = 0; k < S; k++) jobs[k] = {segs[k].first, segs[k].second * period, ctx->ws_rot + (size_t)k * 2 * l1 * N};
    if ((r = rotate_jobs(ctx, gk, B->d, (size_t)2 * B->limbs_alloc * N, B->limbs_alloc, B->n, l1, jobs, st))) return r;
    ensi_ct al;
    al.ctx = ctx;
    al.owns = false;
    al.n = S;
    al.limbs = al.limbs_alloc = l1;
    al.scale = B->scale;
    al.d = ctx->ws_rot;
    std::vector<int32_t> src(S), mi(S, 0);
    for (int k = 0; k < S; k++) src[k] = k;
    if ((r = mask_rescale(ctx, &al, src, mask_head, mi, seg, st))) return r;
    return doubling_steps(ctx, gk, seg, period, s, st, -1);
}

extern "C" int ensi_ccmm_bsgs(ensi_ctx *ctx, const ensi_gk *rk, const ensi_gk *gk, const ensi_ct *A, const ensi_ct *B, int32_t s,
                              int32_t period, const int32_t *begin, const int32_t *term_a, const int32_t *term_b, const int32_t *term_slot,
                              int32_t n_out, const ensi_pt *mask_head, const ensi_pt *mask_start, ensi_ct *out, void *stream) {
    if (!ctx || !rk || !gk || !A || !B || !begin || !mask_head || !mask_start || !out || n_out < 1) return ENSI_E_BADARG;
    if (A->prepared || B->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "a batch of prepared weights is read by ensi_ccmm_segment and ensi_ccmm_av only");
    const int N = ctx->N, l1 = B->limbs;
    if (s < 1 || (s & (s - 1)) || s > N / 2) ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: the block length must be a power of two up to %d", N / 2);
    if (period < 1 || (period & (period - 1)) || period > s) ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: the period must be a power of two up to the block length");
    if (A->limbs != l1) ENSI_FAIL(ctx, ENSI_E_LEVEL, "ccmm: A and B at different levels (%d vs %d limbs)", A->limbs, l1);
    if (l1 < 4 || out->limbs != l1 - 3) ENSI_FAIL(ctx, ENSI_E_LEVEL, "ccmm: output must be three levels below the operands");
    if (out->n != n_out) ENSI_FAIL(ctx, ENSI_E_SHAPE, "ccmm: output batch holds %d ciphertexts, need %d", out->n, n_out);
    if (mask_head->n < 1 || mask_start->n < 1 || mask_head->limbs < l1 || mask_start->limbs < l1 - 1)
        ENSI_FAIL(ctx, ENSI_E_LEVEL, "ccmm: the masks need %d and %d limbs", l1, l1 - 1);
    if (begin[0] != 0) ENSI_FAIL(ctx, ENSI_E_BADARG, "term offsets must start at 0");
    for (int o = 0; o < n_out; o++)
        if (begin[o + 1] < begin[o]) ENSI_FAIL(ctx, ENSI_E_BADARG, "term offsets must not decrease");
    const int T = begin[n_out];
    if (T > 0 && (!term_a || !term_b || !term_slot)) return ENSI_E_BADARG;
    for (int t = 0; t < T; t++)
        if (term_a[t] < 0 || term_a[t] >= A->n || term_b[t] < 0 || term_b[t] >= B->n || term_slot[t] < 0 || term_slot[t] >= s)
            ENSI_FAIL(ctx, ENSI_E_BADARG, "term %d names ciphertexts %d of %d and %d of %d, slot %d of %d", t, term_a[t], A->n, term_b[t], B->n,
                      term_slot[t], s);
    if (A->d == out->d || B->d == out->d) ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: operands and out must not overlap");
    hipStream_t st = (hipStream_t)stream;
    const u64 *key;
    int rc;
    if ((rc = relin_key(ctx, rk, &key))) return rc;
    const int l2 = l1 - 1, l3 = l1 - 2;
    const size_t a_ct = (size_t)2 * A->limbs_alloc * N, out_ct = (size_t)2 * out->limbs_alloc * N;
    const size_t seg_ct = (size_t)2 * l2 * N, rep_ct = (size_t)2 * l3 * N;

    // groups of outputs whose distinct elements fit the workspace (an output is never split: its products are
    // relinearised together); the segments are formed once for the whole call when there are at most 1024 of them,
    // else once per group
    const size_t cap = 512, cap_seg = 1024;
    struct Chunk {
        int o0, o1;
        std::vector<std::pair<int, int>> segs, els;  // (b, g) and (b, slot), in order of first use
        std::vector<int> el_seg, term_el;            // segment of each element; element of each term from begin[o0] on
    };
    std::vector<std::pair<int, int>> all_segs;
    std::map<std::pair<int, int>, int> all_seg_id;
    for (int t = 0; t < T; t++) {
        const std::pair<int, int> g(term_b[t], term_slot[t] / period);
        if (all_seg_id.emplace(g, (int)all_segs.size()).second) all_segs.push_back(g);
    }
    const bool shared = all_segs.size() <= cap_seg;
    std::vector<Chunk> chunks;
    for (int o0 = 0; o0 < n_out;) {
        Chunk c;
        c.o0 = o0;
        std::map<std::pair<int, int>, int> seg_id, el_id;
        int o = o0;
        for (; o < n_out; o++) {
            size_t fresh = 0;
            std::set<std::pair<int, int>> seen;
            for (int t = begin[o]; t < begin[o + 1]; t++) {
                const std::pair<int, int> e(term_b[t], term_slot[t]);
                if (!el_id.count(e) && seen.insert(e).second) fresh++;
            }
            if (o > o0 && c.els.size() + fresh > cap) break;
            for (int t = begin[o]; t < begin[o + 1]; t++) {
                const std::pair<int, int> e(term_b[t], term_slot[t]), g(term_b[t], term_slot[t] / period);
                auto ie = el_id.find(e);
                if (ie == el_id.end()) {
                    int sid;
                    if (shared) {
                        sid = all_seg_id[g];
                    } else {
                        auto ig = seg_id.find(g);
                        if (ig == seg_id.end()) {
                            ig = seg_id.emplace(g, (int)c.segs.size()).first;
                            c.segs.push_back(g);
                        }
                        sid = ig->second;
                    }
                    ie = el_id.emplace(e, (int)c.els.size()).first;
                    c.els.push_back(e);
                    c.el_seg.push_back(sid);
                }
                c.term_el.push_back(ie->second);
            }
        }
        c.o1 = o;
        o0 = o;
        chunks.push_back(std::move(c));
    }
    size_t max_seg = shared ? std::max<size_t>(1, all_segs.size()) : 1, max_el = 1;
    for (const Chunk &c : chunks) {
        max_seg = std::max(max_seg, c.segs.size());
        max_el = std::max(max_el, c.els.size());
    }
    if ((rc = grow(ctx, &ctx->ws_rot, &ctx->ws_rot_words, std::max(max_seg * 2 * l1 * N, max_el * seg_ct)))) return rc;
    if ((rc = grow(ctx, &ctx->ws_rep, &ctx->ws_rep_words, max_seg * seg_ct + max_el * rep_ct))) return rc;

    ensi_ct view;
    view.ctx = ctx;
    view.owns = false;
    ensi_ct seg = view;
    seg.limbs = seg.limbs_alloc = l2;
    seg.d = ctx->ws_rep;
    seg.scale = B->scale * mask_head->scale / (double)ctx->primes[l1 - 1];
    auto spread = [&](const std::vector<std::pair<int, int>> &segs) -> int { return spread_segments(ctx, gk, B, segs, s, period, mask_head, &seg, st); };
    if (shared && (rc = spread(all_segs))) return rc;

    for (const Chunk &c : chunks) {
        const int E = (int)c.els.size();
        if (!shared && (rc = spread(c.segs))) return rc;
        // baby steps: element b of every period to the period's start, kept by the period-start mask, copied through the period
        ensi_ct al = view, rep = view;
        std::vector<RotJob> jobs(E);
        for (int k = 0; k < E; k++) jobs[k] = {c.el_seg[k], c.els[k].second % period, ctx->ws_rot + (size_t)k * seg_ct};
        if (E && (rc = rotate_jobs(ctx, gk, seg.d, seg_ct, l2, seg.n, l2, jobs, st))) return rc;
        al.n = E;
        al.limbs = al.limbs_alloc = l2;
        al.scale = seg.scale;
        al.d = ctx->ws_rot;
        rep.n = E;
        rep.limbs = rep.limbs_alloc = l3;
        rep.d = ctx->ws_rep + max_seg * seg_ct;
        rep.scale = seg.scale * mask_start->scale / (double)ctx->primes[l2 - 1];
        if (E) {
            std::vector<int32_t> src(E), mi(E, 0);
            for (int k = 0; k < E; k++) src[k] = k;
            if ((rc = mask_rescale(ctx, &al, src, mask_start, mi, &rep, st))) return rc;
            if ((rc = doubling_steps(ctx, gk, &rep, 1, period, st, -1))) return rc;
        }
        const int tb = begin[c.o0], cnt = c.o1 - c.o0;
        std::vector<MmTerm> terms(begin[c.o1] - tb);
        std::vector<int32_t> bg(cnt + 1);
        for (int o = 0; o <= cnt; o++) bg[o] = begin[c.o0 + o] - tb;
        for (size_t t = 0; t < terms.size(); t++) terms[t] = {A->d + (size_t)term_a[tb + t] * a_ct, rep.d + (size_t)c.term_el[t] * rep_ct};
        ensi_ct part = *out;
        part.owns = false;
        part.d = out->d + (size_t)c.o0 * out_ct;
        part.n = cnt;
        if ((rc = mult_core(ctx, key, terms, bg, l3, A->limbs_alloc, l3, &part, st))) return rc;
        out->scale = A->scale * rep.scale / (double)ctx->primes[l3 - 1];
    }
    ENSI_HIP(ctx, hipGetLastError());
    return ENSI_OK;
}

// ------------- CCMM, several heads per ciphertext: a whole segment of output columns from its diagonals
extern "C" int ensi_segment_masks(ensi_ctx *ctx, int32_t s, int32_t period, int32_t limbs, ensi_pt **out) {
    if (!ctx || !out || s < 1 || (s & (s - 1)) || s > ctx->N / 2 || period < 1 || (period & (period - 1)) || period > s || limbs < 2 ||
        limbs > ctx->L)
        return ENSI_E_BADARG;
    const int n = ctx->N / 2;
    std::vector<double> z((size_t)3 * period * n, 0.0);
    for (int kind = 0; kind < 3; kind++)
        for (int r = 0; r < period; r++) {
            double *m = z.data() + ((size_t)kind * period + r) * n;
            for (int b0 = 0; b0 < n; b0 += s) {
                if (kind == 2) m[b0 + s - period + r] = 1.0;
                else
                    for (int x = r; x < s - (kind == 1 ? period : 0); x += period) m[b0 + x] = 1.0;
            }
        }
    return encode_window(ctx, z.data(), 3 * period, n, 0, 0, limbs, (double)ctx->primes[limbs - 1], out);
}

// Baby and giant steps over the 2P - 1 diagonals of a segment: diagonal q has rotation amount q (q < P) or q - 2P + 1
// (the one used in the last slots of a block) = e1 + t with 0 <= e1 < baby and t a multiple of baby.
static void diagonal_schedule(int P, int baby, std::vector<int> &e1, std::vector<int> &t) {
    e1.resize(2 * P - 1);
    t.resize(2 * P - 1);
    for (int q = 0; q < 2 * P - 1; q++) {
        const int amount = q < P ? q : q - 2 * P + 1;
        e1[q] = ((amount % baby) + baby) % baby;
        t[q] = amount - e1[q];
    }
}

// The left operand of ensi_ccmm_segment moved by minus every giant step, once for all segments:
// out[j nT + k] = Rot(A_j; -giant_k) on the first l - 1 limbs, giant_k ascending = -P, -P + baby, ..., P - baby.
extern "C" int ensi_ccmm_left_giant_steps(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *A, int32_t period, int32_t baby, int32_t prepare,
                                          ensi_ct *out, void *stream) {
    if (!ctx || !gk || !A || !out) return ENSI_E_BADARG;
    if (A->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "the operand is already prepared");
    const int N = ctx->N, P = period, d = A->n, l2 = A->limbs - 1;
    if (P < 1 || (P & (P - 1)) || P > N / 2) ENSI_FAIL(ctx, ENSI_E_BADARG, "the period must be a power of two");
    if (baby < 1 || (baby & (baby - 1)) || baby > P) ENSI_FAIL(ctx, ENSI_E_BADARG, "the baby-step range must be a power of two up to the period");
    std::vector<int> e1, t;
    diagonal_schedule(P, baby, e1, t);
    std::vector<int> giant(t);
    std::sort(giant.begin(), giant.end());
    giant.erase(std::unique(giant.begin(), giant.end()), giant.end());
    const int nT = (int)giant.size();
    if (l2 < 1 || out->limbs != l2 || out->limbs_alloc != l2) ENSI_FAIL(ctx, ENSI_E_LEVEL, "the output batch must be allocated one level below the input");
    if (out->n != d * nT) ENSI_FAIL(ctx, ENSI_E_SHAPE, "output batch holds %d ciphertexts, need %d", out->n, d * nT);
    if (A->d == out->d) ENSI_FAIL(ctx, ENSI_E_BADARG, "in and out must not overlap");
    hipStream_t st = (hipStream_t)stream;
    const size_t o_ct = (size_t)2 * l2 * N;
    std::vector<RotJob> jobs;
    for (int j = 0; j < d; j++)
        for (int k = 0; k < nT; k++) jobs.push_back({j, -giant[k], out->d + ((size_t)j * nT + k) * o_ct});
    int rc;
    out->prepared = false;
    if ((rc = rotate_jobs(ctx, gk, A->d, (size_t)2 * A->limbs_alloc * N, A->limbs_alloc, d, l2, jobs, st))) return rc;
    out->scale = A->scale;
    if (prepare) {
        launch_ntt(ctx, out->d, out->n * 2 * l2, make_map(ctx, l2, false), false, st);
        out->prepared = true;
    }
    ENSI_HIP(ctx, hipGetLastError());
    return ENSI_OK;
}

extern "C" int ensi_ccmm_segment(ensi_ctx *ctx, const ensi_gk *rk, const ensi_gk *gk, const ensi_ct *A, const ensi_ct *B, int32_t s,
                                 int32_t period, int32_t baby, int32_t g, const ensi_pt *mask_head, const ensi_pt *masks, ensi_ct *out,
                                 void *stream) {
    if (!ctx || !rk || !gk || !A || !B || !mask_head || !masks || !out) return ENSI_E_BADARG;
    if (B->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "a batch of prepared weights is read by ensi_ccmm_segment and ensi_ccmm_av only");
    const int N = ctx->N, d = B->n, l1 = B->limbs, P = period;
    if (s < 1 || (s & (s - 1)) || s > N / 2) ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: the block length must be a power of two up to %d", N / 2);
    if (P < 1 || (P & (P - 1)) || P > s) ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: the period must be a power of two up to the block length");
    if (baby < 1 || (baby & (baby - 1)) || baby > P) ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: the baby-step range must be a power of two up to the period");
    if (g < 0 || g >= s / P) ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: segment %d outside a block of %d segments", g, s / P);
    // A one level below B: the columns already moved by their giant steps (ensi_ccmm_left_giant_steps), 2P / baby to a column
    const bool a_given = A->limbs == l1 - 1;
    if (!a_given && A->limbs != l1) ENSI_FAIL(ctx, ENSI_E_LEVEL, "ccmm: A and B at different levels (%d vs %d limbs)", A->limbs, l1);
    const int n_giant = baby == 1 ? 2 * P - 1 : 2 * P / baby;  // distinct giant steps of the diagonals
    if (A->n != (a_given ? d * n_giant : d)) ENSI_FAIL(ctx, ENSI_E_SHAPE, "ccmm: A holds %d ciphertexts, B has %d rows", A->n, d);
    if (A->prepared && !a_given) ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: a prepared A must come from ensi_ccmm_left_giant_steps");
    if (l1 < 4 || out->limbs != l1 - 3) ENSI_FAIL(ctx, ENSI_E_LEVEL, "ccmm: output must be three levels below the operands");
    if (out->n != P) ENSI_FAIL(ctx, ENSI_E_SHAPE, "ccmm: output batch holds %d ciphertexts, need %d", out->n, P);
    if (mask_head->n < 1 || mask_head->limbs < l1 || masks->n < 3 * P || masks->limbs < l1 - 2)
        ENSI_FAIL(ctx, ENSI_E_LEVEL, "ccmm: the head mask needs %d limbs, the %d sorting masks %d", l1, 3 * P, l1 - 2);
    if (d > 65535) ENSI_FAIL(ctx, ENSI_E_SHAPE, "ccmm: at most 65535 products per diagonal");
    if (A->d == out->d || B->d == out->d) ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: operands and out must not overlap");
    hipStream_t st = (hipStream_t)stream;
    const u64 *key;
    int rc;
    if ((rc = relin_key(ctx, rk, &key))) return rc;
    const int l2 = l1 - 1, l3 = l1 - 2, n_diag = 2 * P - 1;
    const size_t a_ct = (size_t)2 * A->limbs_alloc * N, seg_ct = (size_t)2 * l2 * N;
    std::vector<int> e1, t;
    diagonal_schedule(P, baby, e1, t);
    std::vector<int> giant(t);  // the distinct giant steps, ascending
    std::sort(giant.begin(), giant.end());
    giant.erase(std::unique(giant.begin(), giant.end()), giant.end());
    const int nT = (int)giant.size();
    auto giant_index = [&](int v) { return (int)(std::lower_bound(giant.begin(), giant.end(), v) - giant.begin()); };
    // The sums are laid out as a grid: entry x * baby + y pairs giant step giant[x] with baby step y (amount giant[x] + y);
    // where no diagonal has that amount (one entry when baby > 1) the entry is formed all the same and not used.
    const int n_sum = nT * baby;
    std::vector<int> diag_at(n_sum, -1);
    for (int q = 0; q < n_diag; q++) diag_at[giant_index(t[q]) * baby + e1[q]] = q;
    // ws_rot: [rotated w: d (baby - 1)][rotated a: d (nT - 1)][rotated sums: n_sum], all at l2 limbs; the first stage
    // (aligning rotations at l1 limbs) uses its start.  ws_rep: [segs: d][sums: n_sum].
    const size_t n_w = (size_t)d * (baby - 1), n_a = a_given ? 0 : (size_t)d * (nT - 1);
    if ((rc = grow(ctx, &ctx->ws_rot, &ctx->ws_rot_words, std::max((size_t)d * 2 * l1 * N, (n_w + n_a + n_sum) * seg_ct)))) return rc;
    if ((rc = grow(ctx, &ctx->ws_rep, &ctx->ws_rep_words, ((size_t)d + n_sum) * seg_ct))) return rc;
    ensi_ct seg;
    seg.ctx = ctx;
    seg.owns = false;
    seg.limbs = seg.limbs_alloc = l2;
    seg.d = ctx->ws_rep;
    seg.scale = B->scale * mask_head->scale / (double)ctx->primes[l1 - 1];
    std::vector<std::pair<int, int>> segs(d);
    for (int j = 0; j < d; j++) segs[j] = {j, g};
    if ((rc = spread_segments(ctx, gk, B, segs, s, P, mask_head, &seg, st))) return rc;
    // baby steps of the spread operands, minus the giant steps of the columns of A (read at l2 limbs)
    u64 *w_rot = ctx->ws_rot, *a_rot = w_rot + n_w * seg_ct, *s_rot = a_rot + n_a * seg_ct;
    std::vector<RotJob> jobs;
    for (int j = 0; j < d; j++)
        for (int b = 1; b < baby; b++) jobs.push_back({j, b, w_rot + ((size_t)j * (baby - 1) + (b - 1)) * seg_ct});
    if (!jobs.empty() && (rc = rotate_jobs(ctx, gk, seg.d, seg_ct, l2, d, l2, jobs, st))) return rc;
    jobs.clear();
    std::vector<int> a_slot(nT, -1);  // position of each nonzero giant step among the rotated copies of a column
    int x_plain = 0;                  // the grid row without a giant step
    for (int gi = 0, k = 0; gi < nT; gi++) {
        if (giant[gi]) a_slot[gi] = k++;
        else x_plain = gi;
    }
    for (int j = 0; j < d && !a_given; j++)
        for (int gi = 0; gi < nT; gi++)
            if (giant[gi]) jobs.push_back({j, -giant[gi], a_rot + ((size_t)j * (nT - 1) + a_slot[gi]) * seg_ct});
    if (!jobs.empty() && (rc = rotate_jobs(ctx, gk, A->d, a_ct, A->limbs_alloc, d, l2, jobs, st))) return rc;
    // the sums: relinearised, at the product's scale (the rotated columns of A have limb stride l2, the unrotated ones A's own)
    ensi_ct sums = seg;
    sums.n = n_sum;
    sums.d = ctx->ws_rep + (size_t)d * seg_ct;
    sums.scale = A->scale * seg.scale;
    {
        std::vector<MmTerm> terms;
        std::vector<int32_t> begin(1, 0);
        for (int x = 0; x < nT; x++)
            for (int y = 0; y < baby; y++) {
                for (int j = 0; j < d; j++) {
                    MmTerm tm;
                    if (a_given) {
                        tm.a = A->d + ((size_t)j * nT + x) * a_ct;
                        tm.stride_a = A->limbs_alloc;
                    } else {
                        tm.a = giant[x] ? a_rot + ((size_t)j * (nT - 1) + a_slot[x]) * seg_ct : A->d + (size_t)j * a_ct;
                        tm.stride_a = giant[x] ? l2 : A->limbs_alloc;
                    }
                    tm.b = y ? w_rot + ((size_t)j * (baby - 1) + (y - 1)) * seg_ct : seg.d + (size_t)j * seg_ct;
                    terms.push_back(tm);
                }
                begin.push_back((int32_t)terms.size());
            }
        if ((rc = mult_core(ctx, key, terms, begin, l2, A->limbs_alloc, l2, &sums, st, A->prepared, false, nT, baby))) return rc;
    }
    // giant steps of the sums, then the rescale of every diagonal (in place; limb stride l2): the row without a giant step
    // where it is, the rows before and after it in their rotated copies
    jobs.clear();
    for (int k = 0; k < n_sum; k++)
        if (diag_at[k] >= 0 && giant[k / baby]) jobs.push_back({k, giant[k / baby], s_rot + (size_t)k * seg_ct});
    if (!jobs.empty() && (rc = rotate_jobs(ctx, gk, sums.d, seg_ct, l2, n_sum, l2, jobs, st))) return rc;
    const u64 *d_consts;
    const double *d_fconsts;
    bool fp;
    if ((rc = upload_rescale_consts(ctx, l2, 1.0, false, st, &d_consts, &d_fconsts, &fp))) return rc;
    launch_rescale(ctx, sums.d + (size_t)x_plain * baby * seg_ct, baby, l2, l2, d_consts, fp ? d_fconsts : nullptr, st);
    if (x_plain > 0) launch_rescale(ctx, s_rot, x_plain * baby, l2, l2, d_consts, fp ? d_fconsts : nullptr, st);
    if (x_plain + 1 < nT)
        launch_rescale(ctx, s_rot + (size_t)(x_plain + 1) * baby * seg_ct, (nT - x_plain - 1) * baby, l2, l2, d_consts, fp ? d_fconsts : nullptr, st);
    std::vector<const u64 *> diag(n_diag);
    for (int k = 0; k < n_sum; k++)
        if (diag_at[k] >= 0) diag[diag_at[k]] = (giant[k / baby] ? s_rot : sums.d) + (size_t)k * seg_ct;
    const double diag_scale = sums.scale / (double)ctx->primes[l2 - 1];
    // sorting: slot x of D_e holds column (x + e) mod P; column c takes the class r = (c - e) mod P of D_e, and from D'_e
    // where that class meets the last e slots of a block
    std::vector<PmTerm> pt;
    std::vector<int32_t> pb(P + 1);
    for (int c = 0; c < P; c++) {
        pb[c] = (int32_t)pt.size();
        for (int e = 0; e < P; e++) {
            const int r = ((c - e) % P + P) % P;
            if (e && r >= P - e) {
                pt.push_back({diag[e], P + r, 0});
                pt.push_back({diag[P - 1 + e], 2 * P + r, 0});
            } else {
                pt.push_back({diag[e], r, 0});
            }
        }
    }
    pb[P] = (int32_t)pt.size();
    if ((rc = pmult_core(ctx, pt, pb, l3, l2, masks, out, st))) return rc;
    out->scale = diag_scale * masks->scale / (double)ctx->primes[l3 - 1];
    ENSI_HIP(ctx, hipGetLastError());
    return ENSI_OK;
}

// ------------- CCMM, several heads per ciphertext: weights times V from diagonalised weights
extern "C" int ensi_diagonalise_weights(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *A, int32_t s, int32_t period, int32_t baby,
                                        const ensi_pt *masks, int32_t prepare, ensi_ct *out, void *stream) {
    if (!ctx || !gk || !A || !masks || !out) return ENSI_E_BADARG;
    if (A->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "the weights are already prepared");
    const int N = ctx->N, P = period, l1 = A->limbs;
    if (s < 1 || (s & (s - 1)) || s > N / 2) ENSI_FAIL(ctx, ENSI_E_BADARG, "the block length must be a power of two up to %d", N / 2);
    if (P < 1 || (P & (P - 1)) || P > s) ENSI_FAIL(ctx, ENSI_E_BADARG, "the period must be a power of two up to the block length");
    if (baby < 1 || (baby & (baby - 1)) || baby > P) ENSI_FAIL(ctx, ENSI_E_BADARG, "the baby-step range must be a power of two up to the period");
    if (A->n < P || A->n % P) ENSI_FAIL(ctx, ENSI_E_SHAPE, "the weights come in whole segments of %d columns, got %d", P, A->n);
    const int n_seg = A->n / P, n_diag = 2 * P - 1, l2 = l1 - 1;
    if (l1 < 2 || out->limbs != l2) ENSI_FAIL(ctx, ENSI_E_LEVEL, "output must be one level below the input");
    if (out->limbs_alloc != l2) ENSI_FAIL(ctx, ENSI_E_SHAPE, "the output batch must be allocated at %d limbs", l2);
    if (out->n != n_seg * n_diag) ENSI_FAIL(ctx, ENSI_E_SHAPE, "output batch holds %d ciphertexts, need %d", out->n, n_seg * n_diag);
    if (masks->n < 3 * P || masks->limbs < l1) ENSI_FAIL(ctx, ENSI_E_LEVEL, "need %d sorting masks at %d limbs", 3 * P, l1);
    if (A->d == out->d) ENSI_FAIL(ctx, ENSI_E_BADARG, "in and out must not overlap");
    hipStream_t st = (hipStream_t)stream;
    const size_t a_ct = (size_t)2 * A->limbs_alloc * N, d_ct = (size_t)2 * l2 * N;
    std::vector<PmTerm> pt;
    std::vector<int32_t> pb(1, 0);
    for (int g = 0; g < n_seg; g++) {
        const u64 *col = A->d + (size_t)g * P * a_ct;
        for (int e = 0; e < P; e++) {  // diagonal e: column (x + e) mod P in slot x, without the block's last e slots
            for (int c = 0; c < P; c++) {
                const int r = ((c - e) % P + P) % P;
                pt.push_back({col + (size_t)c * a_ct, (e && r >= P - e) ? P + r : r, 0});
            }
            pb.push_back((int32_t)pt.size());
        }
        for (int e = 1; e < P; e++) {  // diagonal P - 1 + e: the same column in those last e slots
            for (int c = 0; c < P; c++) {
                const int r = ((c - e) % P + P) % P;
                if (r >= P - e) pt.push_back({col + (size_t)c * a_ct, 2 * P + r, 0});
            }
            pb.push_back((int32_t)pt.size());
        }
    }
    int rc;
    if ((rc = grow(ctx, &ctx->ws_rot, &ctx->ws_rot_words, (size_t)out->n * d_ct))) return rc;
    ensi_ct tmp = *out;
    tmp.owns = false;
    tmp.prepared = false;
    tmp.d = ctx->ws_rot;
    out->prepared = false;
    if ((rc = pmult_core(ctx, pt, pb, l1, A->limbs_alloc, masks, &tmp, st))) return rc;
    out->scale = A->scale * masks->scale / (double)ctx->primes[l1 - 1];
    // every diagonal moves by minus its giant step
    std::vector<int> e1, t;
    diagonal_schedule(P, baby, e1, t);
    std::vector<RotJob> jobs(out->n);
    for (int k = 0; k < out->n; k++) jobs[k] = {k, -t[k % n_diag], out->d + (size_t)k * d_ct};
    if ((rc = rotate_jobs(ctx, gk, tmp.d, d_ct, l2, out->n, l2, jobs, st))) return rc;
    if (prepare) {
        // left in the transform domain, where every column of V multiplies it: ensi_ccmm_av reads it in place
        launch_ntt(ctx, out->d, out->n * 2 * l2, make_map(ctx, l2, false), false, st);
        out->prepared = true;
    }
    ENSI_HIP(ctx, hipGetLastError());
    return ENSI_OK;
}

extern "C" int ensi_ccmm_av(ensi_ctx *ctx, const ensi_gk *rk, const ensi_gk *gk, const ensi_ct *Ad, const ensi_ct *V, int32_t s, int32_t period,
                            int32_t baby, int32_t g0, const ensi_pt *mask_head, ensi_ct *out, void *stream) {
    if (!ctx || !rk || !gk || !Ad || !V || !mask_head || !out) return ENSI_E_BADARG;
    if (V->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "a batch of prepared weights is read by ensi_ccmm_segment and ensi_ccmm_av only");
    const int N = ctx->N, P = period, l1 = V->limbs, m = V->n;
    if (s < 1 || (s & (s - 1)) || s > N / 2) ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: the block length must be a power of two up to %d", N / 2);
    if (P < 1 || (P & (P - 1)) || P > s) ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: the period must be a power of two up to the block length");
    if (baby < 1 || (baby & (baby - 1)) || baby > P) ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: the baby-step range must be a power of two up to the period");
    const int n_diag = 2 * P - 1;
    if (Ad->n < n_diag || Ad->n % n_diag) ENSI_FAIL(ctx, ENSI_E_SHAPE, "ccmm: the diagonalised weights come %d to a segment, got %d", n_diag, Ad->n);
    const int n_seg = Ad->n / n_diag;
    if (g0 < 0 || g0 + n_seg > s / P) ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: segments %d .. %d outside a block of %d segments", g0, g0 + n_seg - 1, s / P);
    if (l1 < 3 || Ad->limbs != l1 - 1) ENSI_FAIL(ctx, ENSI_E_LEVEL, "ccmm: the diagonalised weights must be one level below V (%d vs %d limbs)", Ad->limbs, l1);
    if (out->limbs != l1 - 2) ENSI_FAIL(ctx, ENSI_E_LEVEL, "ccmm: output must be two levels below V");
    if (out->n != m) ENSI_FAIL(ctx, ENSI_E_SHAPE, "ccmm: output batch holds %d ciphertexts, need %d", out->n, m);
    if (mask_head->n < 1 || mask_head->limbs < l1) ENSI_FAIL(ctx, ENSI_E_LEVEL, "ccmm: the head mask needs %d limbs", l1);
    if ((size_t)n_seg * n_diag > 65535) ENSI_FAIL(ctx, ENSI_E_SHAPE, "ccmm: %d segments give more than 65535 products per sum", n_seg);
    if (Ad->d == out->d || V->d == out->d) ENSI_FAIL(ctx, ENSI_E_BADARG, "ccmm: operands and out must not overlap");
    hipStream_t st = (hipStream_t)stream;
    const u64 *key;
    int rc;
    if ((rc = relin_key(ctx, rk, &key))) return rc;
    const int l2 = l1 - 1, l3 = l1 - 2;
    const size_t ad_ct = (size_t)2 * Ad->limbs_alloc * N, seg_ct = (size_t)2 * l2 * N, out_ct = (size_t)2 * out->limbs_alloc * N;
    std::vector<int> e1, t;
    diagonal_schedule(P, baby, e1, t);
    std::vector<int> giant(t);  // the distinct giant steps, ascending
    std::sort(giant.begin(), giant.end());
    giant.erase(std::unique(giant.begin(), giant.end()), giant.end());
    const int nT = (int)giant.size();
    // outputs whose rotated operands are held at once
    const int per = std::max(1, std::min(m, 1536 / (n_seg * std::max(1, baby - 1))));
    const size_t n_sg = (size_t)per * n_seg, n_rot = n_sg * (baby - 1), n_sum = (size_t)per * nT;
    if ((rc = grow(ctx, &ctx->ws_rot, &ctx->ws_rot_words, std::max(n_sg * 2 * l1 * N, std::max(std::max<size_t>(n_rot, 1), n_sum) * seg_ct)))) return rc;
    if ((rc = grow(ctx, &ctx->ws_rep, &ctx->ws_rep_words, (n_sg + n_sum) * seg_ct))) return rc;
    for (int i0 = 0; i0 < m; i0 += per) {
        const int cnt = std::min(per, m - i0);
        ensi_ct seg;
        seg.ctx = ctx;
        seg.owns = false;
        seg.limbs = seg.limbs_alloc = l2;
        seg.d = ctx->ws_rep;
        seg.scale = V->scale * mask_head->scale / (double)ctx->primes[l1 - 1];
        std::vector<std::pair<int, int>> segs;
        for (int i = 0; i < cnt; i++)
            for (int k = 0; k < n_seg; k++) segs.push_back({i0 + i, g0 + k});
        if ((rc = spread_segments(ctx, gk, V, segs, s, P, mask_head, &seg, st))) return rc;
        // baby steps: every spread operand rotated by 1 .. baby - 1 on one raise
        std::vector<RotJob> jobs;
        for (int sg = 0; sg < cnt * n_seg; sg++)
            for (int b = 1; b < baby; b++) jobs.push_back({sg, b, ctx->ws_rot + ((size_t)sg * (baby - 1) + (b - 1)) * seg_ct});
        if (!jobs.empty() && (rc = rotate_jobs(ctx, gk, seg.d, seg_ct, l2, cnt * n_seg, l2, jobs, st))) return rc;
        // one sum per output and giant step: the products of all segments' diagonals that share it
        std::vector<MmTerm> terms;
        std::vector<int32_t> begin(1, 0);
        for (int i = 0; i < cnt; i++)
            for (int g = 0; g < nT; g++) {
                for (int k = 0; k < n_seg; k++) {
                    const int sg = i * n_seg + k;
                    for (int q = 0; q < n_diag; q++) {
                        if (t[q] != giant[g]) continue;
                        const u64 *b = e1[q] ? ctx->ws_rot + ((size_t)sg * (baby - 1) + (e1[q] - 1)) * seg_ct : seg.d + (size_t)sg * seg_ct;
                        terms.push_back({Ad->d + ((size_t)k * n_diag + q) * ad_ct, b});
                    }
                }
                begin.push_back((int32_t)terms.size());
            }
        // relinearised, not yet rescaled: the giant steps act at the product's scale
        ensi_ct sums = seg;
        sums.n = cnt * nT;
        sums.limbs = sums.limbs_alloc = l2;
        sums.d = ctx->ws_rep + n_sg * seg_ct;
        sums.scale = Ad->scale * seg.scale;
        if ((rc = mult_core(ctx, key, terms, begin, l2, Ad->limbs_alloc, l2, &sums, st, Ad->prepared, false))) return rc;
        // giant steps: every sum rotated by its own (the rotated baby steps are no longer needed), added up per output
        // in the slot of the output's first sum, rescaled once
        jobs.clear();
        for (int i = 0; i < cnt; i++)
            for (int g = 0; g < nT; g++)
                if (giant[g]) jobs.push_back({i * nT + g, giant[g], ctx->ws_rot + ((size_t)i * nT + g) * seg_ct});
        if (!jobs.empty() && (rc = rotate_jobs(ctx, gk, sums.d, seg_ct, l2, cnt * nT, l2, jobs, st))) return rc;
        const u64 *d_consts;
        const double *d_fconsts;
        bool fp;
        if ((rc = upload_rescale_consts(ctx, l2, 1.0, false, st, &d_consts, &d_fconsts, &fp))) return rc;
        for (int i = 0; i < cnt; i++) {
            // the sum with giant step 0 stays where it is and collects the others; if there is none, the first rotated one does
            int home = -1;
            for (int g = 0; g < nT; g++)
                if (!giant[g]) home = g;
            u64 *acc = home >= 0 ? sums.d + ((size_t)i * nT + home) * seg_ct : ctx->ws_rot + (size_t)i * nT * seg_ct;
            for (int g = 0; g < nT; g++) {
                if (g == (home >= 0 ? home : 0)) continue;
                launch_ct_add(ctx, acc, l2, ctx->ws_rot + ((size_t)i * nT + g) * seg_ct, l2, l2, 1, st);
            }
            launch_rescale(ctx, acc, 1, l2, l2, d_consts, fp ? d_fconsts : nullptr, st);
            u64 *dst = out->d + (size_t)(i0 + i) * out_ct;
            for (int poly = 0; poly < 2; poly++)
                ENSI_HIP(ctx, hipMemcpyAsync(dst + (size_t)poly * out->limbs_alloc * N, acc + (size_t)poly * l2 * N, (size_t)l3 * N * 8,
                                             hipMemcpyDeviceToDevice, st));
        }
        out->scale = sums.scale / (double)ctx->primes[l2 - 1];
    }
    ENSI_HIP(ctx, hipGetLastError());
    return ENSI_OK;
}

