// Host side of Alg. 1 (PCMM): the plan of a weight matrix, the unpack rotations and the signed sums, the scalar-multiply +
// rescale step between two layers, and the C ABI entry points around them.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <set>

#include "api_util.h"
#include "common.h"
#include "hostmath.h"

// ------------------------------------------------------------------------ PCMM
static u64 hash_weights(const int8_t *W, size_t n, u64 h) {
    size_t i = 0;
    for (; i + 8 <= n; i += 8) {
        u64 w;
        memcpy(&w, W + i, 8);
        h = (h ^ w) * 0x100000001B3ULL;
        h ^= h >> 29;
    }
    for (; i < n; i++) h = (h ^ (u64)(uint8_t)W[i]) * 0x100000001B3ULL;
    return h;
}

void free_plan(MatmulPlan *p) {
    if (!p) return;
    if (p->d_masks) (void)hipFree(p->d_masks);
    if (p->d_wt) (void)hipFree(p->d_wt);
    if (p->d_bias) (void)hipFree(p->d_bias);
    if (p->d_bias_fp) (void)hipFree(p->d_bias_fp);
    delete p;
}

// Builds (or finds) the plan of Y = X W: which (packed input G, rotation amount rho)
// operands exist, and the weight of each operand in each output,
//   W'[v][i] = W[G*c_tot + (rho + p_i) mod c_tot][i],   p_i = placement block of output i.
static int build_plan(ensi_ctx *ctx, const int8_t *W, int s, int d, int m, int placement, int c_tot, int n_in, int l1, u64 h,
                      MatmulPlan **out) {
    for (size_t k = 0; k < (size_t)d * m; k++)
        if (W[k] < -1 || W[k] > 1) ENSI_FAIL(ctx, ENSI_E_BADARG, "weight %zu is %d, outside {-1,0,1}", k, (int)W[k]);
    MatmulPlan *p = new MatmulPlan();
    p->hash = h;
    p->l1 = l1;
    p->w_copy.assign(W, W + (size_t)d * m);
    p->s = s; p->d = d; p->m = m; p->placement = placement; p->c_tot = c_tot; p->n_in = n_in;
    p->vid.assign((size_t)n_in * c_tot, -1);
    for (int j = 0; j < d; j++) {
        const int G = j / c_tot, b = j % c_tot;
        const int8_t *row = W + (size_t)j * m;
        for (int i = 0; i < m; i++) {
            if (!row[i]) continue;
            const int pb = placement == ENSI_PLACE_ZERO ? 0 : i % c_tot;
            int rho = b - pb;
            if (rho < 0) rho += c_tot;
            p->vid[(size_t)G * c_tot + rho] = 0;
        }
    }
    p->n_v = p->n_rot = 0;
    for (int G = 0; G < n_in; G++)
        for (int rho = 1; rho < c_tot; rho++)
            if (p->vid[(size_t)G * c_tot + rho] == 0) p->n_rot++;
    if (p->n_rot == 0) {
        // no rotation anywhere: the operands are the inputs themselves, in place (operand G = input G)
        for (int G = 0; G < n_in; G++) p->vid[(size_t)G * c_tot] = G;
        p->n_v = n_in;
    } else {
        for (int G = 0; G < n_in; G++)
            for (int rho = 0; rho < c_tot; rho++)
                if (p->vid[(size_t)G * c_tot + rho] == 0) p->vid[(size_t)G * c_tot + rho] = p->n_v++;
    }
    const int n_v = p->n_v;
    // matrix-core layout is valid when a 32-word tile stays inside a limb and the exact
    // signed sum of n_v residues fits a signed 64-bit word
    int qbits = 0;
    for (int i = 0; i < l1; i++) qbits = std::max(qbits, 64 - __builtin_clzll(ctx->primes[i]));
    // |sum of n_v residues| <= n_v * (2^qbits - 1) must stay below 2^63
    // (and a plane sum of n_v bytes, shifted by eight bits, has to fit a signed 32-bit word: n_v <= 32768)
    const bool mfma_ok = ctx->N >= 32 && n_v >= 1 && n_v <= 32768 && qbits <= 56 && (u64)n_v <= ((u64)1 << (63 - qbits));
    p->planes = 0;
    p->n_kpad = (std::max(n_v, 1) + 255) / 256 * 256;  // whole groups of eight 32-operand steps
    p->m_pad = (m + 255) / 256 * 256;
    const int tiles = (m + 31) / 32;
    std::vector<u32> masks((size_t)tiles * std::max(n_v, 1) * 2, 0);
    std::vector<int8_t> wt;
    std::vector<int32_t> bias;
    if (mfma_ok) {
        const int need = (qbits + 7) / 8;
        p->planes = need <= 5 ? 5 : 7;  // qbits <= 56: never more than seven byte planes
        wt.assign((size_t)p->m_pad * p->n_kpad, 0);
        bias.assign(p->m_pad, 0);
    }
    for (int j = 0; j < d; j++) {
        const int G = j / c_tot, b = j % c_tot;
        const int8_t *row = W + (size_t)j * m;
        for (int i = 0; i < m; i++) {
            if (!row[i]) continue;
            const int pb = placement == ENSI_PLACE_ZERO ? 0 : i % c_tot;
            int rho = b - pb;
            if (rho < 0) rho += c_tot;
            const int v = p->vid[(size_t)G * c_tot + rho];
            masks[((size_t)(i / 32) * n_v + v) * 2 + (row[i] > 0 ? 0 : 1)] |= 1u << (i % 32);
            if (mfma_ok) {
                // fragment order: [output tile of 256][step of 32 operands][wave][block of 32][lane][16 bytes],
                // lane = 32*(operand half of the step) + output within the block
                const size_t cell = ((((size_t)(i / 256) * (p->n_kpad / 32) + v / 32) * 4 + (i % 256) / 64) * 2 + (i % 64) / 32) * 64 +
                                    ((v % 32) / 16) * 32 + i % 32;
                wt[cell * 16 + v % 16] = row[i];
                bias[i] += row[i];
            }
        }
    }
    if (mfma_ok)
        for (int i = 0; i < m; i++) bias[i] *= 128;  // every byte is fed to the matrix pipe as u - 128
    hipError_t e1 = upload(&p->d_masks, masks), e2 = hipSuccess, e3 = hipSuccess, e4 = hipSuccess;
    if (mfma_ok) {
        e2 = upload(&p->d_wt, wt);
        e3 = upload(&p->d_bias, bias);
        if (qbits <= 50) {
            // the recombination in double precision adds the offset term already reduced: b * sum_p 256^p mod q_limb
            std::vector<double> bias_fp((size_t)l1 * p->m_pad, 0.0);
            __int128 ones = 0;
            for (int pl = 0; pl < p->planes; pl++) ones |= (__int128)1 << (8 * pl);
            for (int limb = 0; limb < l1; limb++) {
                const __int128 q = (__int128)ctx->primes[limb];
                for (int i = 0; i < m; i++) {
                    __int128 r = ((__int128)bias[i] * ones) % q;
                    if (r < 0) r += q;
                    bias_fp[(size_t)limb * p->m_pad + i] = (double)(u64)r;
                }
            }
            e4 = upload(&p->d_bias_fp, bias_fp);
        }
    }
    if (e1 != hipSuccess || e2 != hipSuccess || e3 != hipSuccess || e4 != hipSuccess) {
        free_plan(p);
        ENSI_FAIL(ctx, ENSI_E_NOMEM, "uploading the matmul plan failed");
    }
    *out = p;
    return ENSI_OK;
}

// The plan of (W, s, d, m, placement) at l1 limbs from the context's cache (the weights of a layer are the same call
// after call), built on a miss.  A hit is a match of the 64-bit hash confirmed by comparing the weights byte by byte.
// Callers that want neither the hash nor the comparison inside their step prepare the weights once
// (ensi_weights_prepare).
static int get_plan(ensi_ctx *ctx, const int8_t *W, int s, int d, int m, int placement, int c_tot, int n_in, int l1,
                    MatmulPlan **out) {
    u64 h = 0xCBF29CE484222325ULL ^ ((u64)s << 40) ^ ((u64)d << 20) ^ (u64)m ^ ((u64)placement << 60) ^ ((u64)l1 << 52);
    h = hash_weights(W, (size_t)d * m, h);
    for (size_t k = 0; k < ctx->plans.size(); k++) {
        MatmulPlan *p = ctx->plans[k];
        if (p->hash == h && p->s == s && p->d == d && p->m == m && p->placement == placement && p->l1 == l1 &&
            p->w_copy.size() == (size_t)d * m && memcmp(p->w_copy.data(), W, (size_t)d * m) == 0) {
            *out = p;
            return ENSI_OK;
        }
    }
    MatmulPlan *p = nullptr;
    int rc = build_plan(ctx, W, s, d, m, placement, c_tot, n_in, l1, h, &p);
    if (rc) return rc;
    if (ctx->plans.size() >= 8) {
        (void)hipDeviceSynchronize();  // the evicted plan's device arrays may still be read by work in flight
        free_plan(ctx->plans.front());
        ctx->plans.erase(ctx->plans.begin());
    }
    ctx->plans.push_back(p);
    *out = p;
    return ENSI_OK;
}

extern "C" int ensi_set_accumulate_mode(ensi_ctx *ctx, int32_t mode) {
    if (!ctx || mode < 0 || mode > 2) return ENSI_E_BADARG;
    ctx->accumulate_mode = mode;
    return ENSI_OK;
}

extern "C" int ensi_matrix_rate_probe(ensi_ctx *ctx, double seconds, double *ops_per_second, void *stream) {
    if (!ctx || !ops_per_second || !(seconds > 0) || seconds > 2.0) return ENSI_E_BADARG;
    return launch_matrix_rate(ctx, seconds, ops_per_second, (hipStream_t)stream);
}

// Shape and level checks shared by the entry points of Alg. 1.
static int matmul_check(ensi_ctx *ctx, const ensi_ct *in, int32_t s, int32_t d, int32_t m, int32_t placement, const ensi_ct *out, int *c_tot_out,
                        int *n_in_out) {
    if (in->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "a batch of prepared weights is read by ensi_ccmm_segment and ensi_ccmm_av only");
    if (placement != ENSI_PLACE_ZERO && placement != ENSI_PLACE_DIAGONAL) ENSI_FAIL(ctx, ENSI_E_BADARG, "unknown placement %d", placement);
    const int n_slots = ctx->N / 2;
    if (n_slots % s) ENSI_FAIL(ctx, ENSI_E_SHAPE, "tokens per column (%d) must divide the slot count %d", s, n_slots);
    const int c_tot = n_slots / s;
    const int n_in = (d + c_tot - 1) / c_tot;
    if (in->n != n_in) ENSI_FAIL(ctx, ENSI_E_SHAPE, "expected %d packed input ciphertexts for d=%d, c_tot=%d, got %d", n_in, d, c_tot, in->n);
    if (out->n != m) ENSI_FAIL(ctx, ENSI_E_SHAPE, "output batch holds %d ciphertexts, need %d", out->n, m);
    if (in->limbs != out->limbs) ENSI_FAIL(ctx, ENSI_E_LEVEL, "matmul: levels differ (%d vs %d limbs)", in->limbs, out->limbs);
    if (in->d == out->d) ENSI_FAIL(ctx, ENSI_E_BADARG, "matmul: in and out must not overlap");
    *c_tot_out = c_tot;
    *n_in_out = n_in;
    return ENSI_OK;
}

static int matmul_run(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *in, MatmulPlan *plan, ensi_ct *out, void *stream);

extern "C" int ensi_ternary_matmul(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *in, int32_t s, int32_t d, const int8_t *W,
                                   int32_t m, int32_t placement, ensi_ct *out, void *stream) {
    if (!ctx || !in || !W || !out || s < 1 || d < 1 || m < 1) return ENSI_E_BADARG;
    int rc, c_tot, n_in;
    if ((rc = matmul_check(ctx, in, s, d, m, placement, out, &c_tot, &n_in))) return rc;
    MatmulPlan *plan;
    if ((rc = get_plan(ctx, W, s, d, m, placement, c_tot, n_in, in->limbs, &plan))) return rc;
    return matmul_run(ctx, gk, in, plan, out, stream);
}

extern "C" int ensi_weights_prepare(ensi_ctx *ctx, const int8_t *W, int32_t s, int32_t d, int32_t m, int32_t placement, int32_t limbs,
                                    ensi_wt **out) {
    if (!ctx || !W || !out || s < 1 || d < 1 || m < 1 || limbs < 1 || limbs > ctx->L) return ENSI_E_BADARG;
    *out = nullptr;
    if (placement != ENSI_PLACE_ZERO && placement != ENSI_PLACE_DIAGONAL) ENSI_FAIL(ctx, ENSI_E_BADARG, "unknown placement %d", placement);
    const int n_slots = ctx->N / 2;
    if (n_slots % s) ENSI_FAIL(ctx, ENSI_E_SHAPE, "tokens per column (%d) must divide the slot count %d", s, n_slots);
    const int c_tot = n_slots / s, n_in = (d + c_tot - 1) / c_tot;
    MatmulPlan *plan = nullptr;
    int rc = build_plan(ctx, W, s, d, m, placement, c_tot, n_in, limbs, 0, &plan);
    if (rc) return rc;
    plan->w_copy.clear();  // a prepared plan is never looked up by its weights
    plan->w_copy.shrink_to_fit();
    ensi_wt *wt = new ensi_wt();
    wt->ctx = ctx;
    wt->plan = plan;
    wt->limbs = limbs;
    *out = wt;
    return ENSI_OK;
}
extern "C" void ensi_weights_free(ensi_wt *wt) {
    if (!wt) return;
    (void)hipDeviceSynchronize();  // the plan's device arrays may still be read by work in flight
    free_plan(wt->plan);
    delete wt;
}

extern "C" int ensi_ternary_matmul_prepared(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *in, const ensi_wt *wt, ensi_ct *out, void *stream) {
    if (!ctx || !in || !wt || !out || wt->ctx != ctx) return ENSI_E_BADARG;
    const MatmulPlan *p = wt->plan;
    if (in->limbs != wt->limbs) ENSI_FAIL(ctx, ENSI_E_LEVEL, "weights were prepared for %d limbs, the input has %d", wt->limbs, in->limbs);
    int rc, c_tot, n_in;
    if ((rc = matmul_check(ctx, in, p->s, p->d, p->m, p->placement, out, &c_tot, &n_in))) return rc;
    return matmul_run(ctx, gk, in, wt->plan, out, stream);
}

// Unpack rotations and the signed sums of Alg. 1 for a validated call.
static int matmul_run(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *in, MatmulPlan *plan, ensi_ct *out, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    const int N = ctx->N, s = plan->s, m = plan->m, c_tot = plan->c_tot, n_in = plan->n_in;
    const int l1 = in->limbs, ext = l1 + ctx->K;
    const size_t in_ct = (size_t)2 * in->limbs_alloc * N;
    int rc;
    const int n_v = plan->n_v, n_rot = plan->n_rot;
    const std::vector<int> &vid = plan->vid;

    // ---- keys for every needed rotation amount
    std::vector<const u64 *> key_of(c_tot, nullptr);
    std::vector<u32> g_of(c_tot, 1);
    for (int rho = 1; rho < c_tot && n_rot; rho++) {
        bool need = false;
        for (int G = 0; G < n_in && !need; G++) need = vid[(size_t)G * c_tot + rho] >= 0;
        if (!need) continue;
        if (!gk) ENSI_FAIL(ctx, ENSI_E_NOKEY, "matmul needs rotations but no key set was given");
        const u32 g = galois_element(ctx, rho * s);
        auto it = gk->keys.find(g);
        if (it == gk->keys.end()) ENSI_FAIL(ctx, ENSI_E_NOKEY, "matmul: no Galois key for step %d", rho * s);
        key_of[rho] = it->second;
        g_of[rho] = g;
    }
    // ---- workspaces.  With rotations, operand v is written to slot v of ws_virt (inputs used
    // unrotated are copied there); without, the operands are the input batch itself.
    const int chunk = 128;
    const u64 *xbase = in->d;
    if (n_rot) {
        const int GS = std::min(n_in, 16);  // packed inputs raised together (about 48 MiB of digits each at 16 limbs)
        const size_t rw = raised_words(ctx, l1);
        if ((rc = grow(ctx, &ctx->ws_digits, &ctx->ws_digits_words, (size_t)GS * rw))) return rc;
        if ((rc = grow(ctx, &ctx->ws_u, &ctx->ws_u_words, (size_t)std::min(chunk, n_rot) * 2 * ext * N))) return rc;
        if ((rc = grow(ctx, &ctx->ws_virt, &ctx->ws_virt_words, (size_t)n_v * in_ct))) return rc;
        if ((rc = ensure_desc(ctx, n_rot))) return rc;
        xbase = ctx->ws_virt;
        // Packed inputs are raised GS at a time and their rotations ordered by amount, so that the GS
        // rotations that use one key sit next to each other in a launch: the blocks that read a key tile then
        // run at nearly the same time on one XCD and all but the first read are served by its L2.
        std::vector<RotDesc> desc;
        std::vector<std::pair<int, int>> groups;  // (first descriptor, count) per group of GS packed inputs
        for (int G0 = 0; G0 < n_in; G0 += GS) {
            const int first = (int)desc.size();
            for (int rho = 0; rho < c_tot; rho++) {
                for (int G = G0; G < std::min(G0 + GS, n_in); G++) {
                    const int v = vid[(size_t)G * c_tot + rho];
                    if (v < 0) continue;
                    u64 *slot = ctx->ws_virt + (size_t)v * in_ct;
                    if (rho == 0) {
                        ENSI_HIP(ctx, hipMemcpyAsync(slot, in->d + (size_t)G * in_ct, in_ct * sizeof(u64), hipMemcpyDeviceToDevice, st));
                        continue;
                    }
                    RotDesc ds = {};
                    ds.c0 = in->d + (size_t)G * in_ct;
                    ds.digits = ctx->ws_digits + (size_t)(G - G0) * rw;
                    ds.key = key_of[rho];
                    ds.out = slot;
                    ds.g = g_of[rho];
                    ds.g_inv = inv_mod_2n(ds.g, N);
                    desc.push_back(ds);
                }
            }
            groups.push_back({first, (int)desc.size() - first});
        }
        ENSI_HIP(ctx, host_to_device(ctx, ctx->ws_desc, desc.data(), desc.size() * sizeof(RotDesc), st));
        // ---- unpack: one ModUp per packed input, shared by all its rotations
        for (size_t gi = 0; gi < groups.size(); gi++) {
            if (!groups[gi].second) continue;
            const int G0 = (int)gi * GS, cnt_in = std::min(GS, n_in - G0);
            if ((rc = raise_cts(ctx, l1, in->d + (size_t)G0 * in_ct, in_ct, in->limbs_alloc, cnt_in, st))) return rc;
            for (int o = 0; o < groups[gi].second; o += chunk) {
                const int cnt = std::min(chunk, groups[gi].second - o);
                if ((rc = run_rotations(ctx, ctx->ws_desc + groups[gi].first + o, cnt, l1, in->limbs_alloc, in->limbs_alloc, st))) return rc;
            }
        }
    }
    // ---- Alg. 1: signed sums
    const bool use_mfma = plan->planes > 0 && ctx->accumulate_mode != 1;
    if (use_mfma) {
        if ((rc = launch_accumulate_mfma(ctx, xbase, in_ct, n_v, plan->n_kpad, plan->d_wt, plan->d_bias, plan->d_bias_fp, plan->planes, m, l1, in->limbs_alloc,
                                         out->d, out->limbs_alloc, nullptr, st)))
            return rc;
    } else
        launch_accumulate(ctx, xbase, in_ct, n_v, plan->d_masks, m, l1, in->limbs_alloc, out->d, out->limbs_alloc, st);
    out->scale = in->scale;
    ENSI_HIP(ctx, hipGetLastError());
    return ENSI_OK;
}

// -------------------------------------------------------------------- rescale
// Constants of the scalar-multiply + rescale step at l1 limbs, uploaded to ws_plan: integer set [5][l1]
// (k mod q_i, Shoup(k), q_l^{-1} mod q_i, Shoup(.), q_l mod q_i) followed by the fp64 set [5][l1] (k, k/q, q_l^{-1},
// q_l^{-1}/q, 1/q), the latter only meaningful when every active prime is below 2^50 (*fp).
// kr: magnitude of the integer constant the limbs are multiplied by before the division (1: plain rescale)
static double rescale_constant(const ensi_ctx *ctx, int l1, double kappa) {
    return floor(fabs(kappa) * (double)ctx->primes[l1 - 1] + 0.5);
}
int upload_rescale_consts(ensi_ctx *ctx, int l1, double kr, bool negative, hipStream_t st, const u64 **d_consts,
                                 const double **d_fconsts, bool *fp_out) {
    const u64 ql = ctx->primes[l1 - 1];
    const u64 kabs = (u64)kr;
    std::vector<u64> consts(5 * (size_t)l1, 0);
    for (int i = 0; i < l1; i++) {
        const u64 q = ctx->primes[i];
        u64 k = kabs % q;
        if (negative && k) k = q - k;
        consts[i] = k;
        consts[l1 + i] = hm_shoup(k, q);
        if (i < l1 - 1) {
            consts[2 * l1 + i] = hm_invmod(ql % q, q);
            consts[3 * l1 + i] = hm_shoup(consts[2 * l1 + i], q);
            consts[4 * l1 + i] = ql % q;
        }
    }
    bool fp = true;
    for (int i = 0; i < l1; i++) fp = fp && ctx->primes[i] < ((u64)1 << 50);
    std::vector<double> fconsts(5 * (size_t)l1, 0.0);
    for (int i = 0; i < l1 && fp; i++) {
        const double q = (double)ctx->primes[i];
        fconsts[i] = (double)consts[i];
        fconsts[l1 + i] = (double)consts[i] / q;
        fconsts[2 * l1 + i] = (double)consts[2 * l1 + i];
        fconsts[3 * l1 + i] = (double)consts[2 * l1 + i] / q;
        fconsts[4 * l1 + i] = 1.0 / q;
    }
    int rc;
    if ((rc = grow(ctx, &ctx->ws_plan, &ctx->ws_plan_words, 2 * consts.size()))) return rc;
    ENSI_HIP(ctx, host_to_device(ctx, ctx->ws_plan, consts.data(), consts.size() * 8, st));
    ENSI_HIP(ctx, host_to_device(ctx, ctx->ws_plan + consts.size(), fconsts.data(), fconsts.size() * 8, st));
    *d_consts = ctx->ws_plan;
    *d_fconsts = (const double *)(ctx->ws_plan + consts.size());
    *fp_out = fp;
    return ENSI_OK;
}

extern "C" int ensi_mul_scalar_rescale(ensi_ctx *ctx, ensi_ct *ct, double kappa, void *stream) {
    if (!ctx || !ct || !(fabs(kappa) > 0) || fabs(kappa) >= 1.0) return ENSI_E_BADARG;
    if (ct->limbs < 2) ENSI_FAIL(ctx, ENSI_E_LEVEL, "rescale: no limb left to drop");
    hipStream_t st = (hipStream_t)stream;
    const int l1 = ct->limbs;
    const u64 *d_consts;
    const double *d_fconsts;
    bool fp;
    const double kr = rescale_constant(ctx, l1, kappa);
    int rc;
    if ((rc = upload_rescale_consts(ctx, l1, kr, kappa < 0, st, &d_consts, &d_fconsts, &fp))) return rc;
    launch_rescale(ctx, ct->d, ct->n, l1, ct->limbs_alloc, d_consts, fp ? d_fconsts : nullptr, st);
    ct->limbs = l1 - 1;
    ct->scale = ct->scale * kr / (fabs(kappa) * (double)ctx->primes[l1 - 1]);
    ENSI_HIP(ctx, hipGetLastError());
    return ENSI_OK;
}

// The fused step for a validated call; plan: the second layer's plan at in->limbs - 1 limbs.
static int rescale_matmul_run(ensi_ctx *ctx, ensi_ct *in, double kappa, MatmulPlan *plan, ensi_ct *out, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    const int N = ctx->N, d = in->n, l1_in = in->limbs, l1 = l1_in - 1, m = plan->m;
    int rc;
    bool fp = true;
    for (int i = 0; i < l1_in; i++) fp = fp && ctx->primes[i] < ((u64)1 << 50);
    if (!fp || plan->planes == 0 || ctx->accumulate_mode == 1) {
        // no fused form for these parameters: the two steps one after the other
        if ((rc = ensi_mul_scalar_rescale(ctx, in, kappa, stream))) return rc;
        return matmul_run(ctx, nullptr, in, plan, out, stream);
    }
    const u64 *d_consts;
    const double *d_fconsts;
    const double kr = rescale_constant(ctx, l1_in, kappa);
    if ((rc = upload_rescale_consts(ctx, l1_in, kr, kappa < 0, st, &d_consts, &d_fconsts, &fp))) return rc;
    if ((rc = launch_accumulate_mfma(ctx, in->d, (size_t)2 * in->limbs_alloc * N, d, plan->n_kpad, plan->d_wt, plan->d_bias, plan->d_bias_fp, plan->planes, m, l1,
                                     in->limbs_alloc, out->d, out->limbs_alloc, d_fconsts, st)))
        return rc;
    in->limbs = l1;
    in->scale = in->scale * kr / (fabs(kappa) * (double)ctx->primes[l1_in - 1]);
    out->scale = in->scale;
    ENSI_HIP(ctx, hipGetLastError());
    return ENSI_OK;
}

static int rescale_matmul_check(ensi_ctx *ctx, const ensi_ct *in, double kappa, int32_t m, const ensi_ct *out) {
    if (!(fabs(kappa) > 0) || fabs(kappa) >= 1.0) return ENSI_E_BADARG;
    if (in->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "a batch of prepared weights is read by ensi_ccmm_segment and ensi_ccmm_av only");
    if (in->limbs < 2) ENSI_FAIL(ctx, ENSI_E_LEVEL, "rescale: no limb left to drop");
    if (out->limbs != in->limbs - 1) ENSI_FAIL(ctx, ENSI_E_LEVEL, "output must be one level below the input (%d vs %d limbs)", out->limbs, in->limbs);
    if (out->n != m) ENSI_FAIL(ctx, ENSI_E_SHAPE, "output batch holds %d ciphertexts, need %d", out->n, m);
    if (in->d == out->d) ENSI_FAIL(ctx, ENSI_E_BADARG, "matmul: in and out must not overlap");
    return ENSI_OK;
}

extern "C" int ensi_rescale_ternary_matmul(ensi_ctx *ctx, ensi_ct *in, double kappa, const int8_t *W, int32_t m, ensi_ct *out,
                                           void *stream) {
    if (!ctx || !in || !W || !out || m < 1) return ENSI_E_BADARG;
    int rc;
    if ((rc = rescale_matmul_check(ctx, in, kappa, m, out))) return rc;
    MatmulPlan *plan;
    if ((rc = get_plan(ctx, W, ctx->N / 2, in->n, m, ENSI_PLACE_ZERO, 1, in->n, in->limbs - 1, &plan))) return rc;
    return rescale_matmul_run(ctx, in, kappa, plan, out, stream);
}

extern "C" int ensi_rescale_ternary_matmul_prepared(ensi_ctx *ctx, ensi_ct *in, double kappa, const ensi_wt *wt, ensi_ct *out, void *stream) {
    if (!ctx || !in || !wt || !out || wt->ctx != ctx) return ENSI_E_BADARG;
    const MatmulPlan *p = wt->plan;
    int rc;
    if ((rc = rescale_matmul_check(ctx, in, kappa, p->m, out))) return rc;
    if (p->c_tot != 1 || p->placement != ENSI_PLACE_ZERO || p->d != in->n)
        ENSI_FAIL(ctx, ENSI_E_SHAPE, "the weights must be prepared for one column per ciphertext (s = N/2), d = %d, placement zero", in->n);
    if (wt->limbs != in->limbs - 1) ENSI_FAIL(ctx, ENSI_E_LEVEL, "weights were prepared for %d limbs, the rescaled input has %d", wt->limbs, in->limbs - 1);
    return rescale_matmul_run(ctx, in, kappa, wt->plan, out, stream);
}

