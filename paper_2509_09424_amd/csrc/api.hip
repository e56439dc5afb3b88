// Host side of the library: context set-up (primes, tables, conversion
// constants), key generation, encryption/decryption plumbing, and the C ABI.
// All polynomial arithmetic runs in the kernels of ntt.hip / kernels.hip; the
// host only derives constants, builds launch descriptors and moves data.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <random>
#include <set>

#include "common.h"
#include "hostmath.h"

#include "api_util.h"

// ------------------------------------------------------------ staged uploads
hipError_t host_to_device(ensi_ctx *ctx, void *dst, const void *src, size_t bytes, hipStream_t st) {
    if (!bytes) return hipSuccess;
    StageSlot &sl = ctx->stage[ctx->stage_next];
    ctx->stage_next = (ctx->stage_next + 1) % ENSI_STAGE_SLOTS;
    hipError_t e;
    if (sl.pending) {
        if ((e = hipEventSynchronize(sl.ev)) != hipSuccess) return e;  // an earlier small copy: long finished in practice
        sl.pending = false;
    }
    if (sl.cap < bytes) {
        if (sl.host) (void)hipHostFree(sl.host);
        sl.host = nullptr;
        sl.cap = 0;
        const size_t cap = std::max<size_t>(bytes, 64 << 10);
        if ((e = hipHostMalloc(&sl.host, cap, hipHostMallocDefault)) != hipSuccess) return e;
        sl.cap = cap;
    }
    if (!sl.ev && (e = hipEventCreateWithFlags(&sl.ev, hipEventDisableTiming)) != hipSuccess) return e;
    memcpy(sl.host, src, bytes);
    if ((e = hipMemcpyAsync(dst, sl.host, bytes, hipMemcpyHostToDevice, st)) != hipSuccess) return e;
    if ((e = hipEventRecord(sl.ev, st)) != hipSuccess) return e;
    sl.pending = true;
    return hipSuccess;
}

int stage_prealloc(ensi_ctx *ctx) {
    for (StageSlot &sl : ctx->stage) {
        if (!sl.host) {
            if (hipHostMalloc(&sl.host, 64 << 10, hipHostMallocDefault) != hipSuccess) ENSI_FAIL(ctx, ENSI_E_NOMEM, "pinned staging buffer allocation failed");
            sl.cap = 64 << 10;
        }
        if (!sl.ev && hipEventCreateWithFlags(&sl.ev, hipEventDisableTiming) != hipSuccess) ENSI_FAIL(ctx, ENSI_E_HIP, "event creation failed");
    }
    return ENSI_OK;
}

// ---------------------------------------------------------------------- timers
int timer_id(ensi_ctx *ctx, const char *name) {
    for (size_t i = 0; i < ctx->timers.size(); i++)
        if (ctx->timers[i].name == name) return (int)i;
    KernelTimer t;
    t.name = name;
    ctx->timers.push_back(t);
    return (int)ctx->timers.size() - 1;
}
void timer_begin(ensi_ctx *ctx, int id, hipStream_t st) {
    hipEvent_t a, b;
    (void)hipEventCreate(&a);
    (void)hipEventCreate(&b);
    (void)hipEventRecord(a, st);
    ctx->pending.push_back({id, {a, b}});
}
void timer_end(ensi_ctx *ctx, hipStream_t st) { (void)hipEventRecord(ctx->pending.back().second.second, st); }

extern "C" int ensi_profile_enable(ensi_ctx *ctx, int32_t on) {
    if (!ctx) return ENSI_E_BADARG;
    ctx->profiling = on != 0;
    return ENSI_OK;
}
extern "C" int ensi_profile_read(ensi_ctx *ctx, char *names_out, int32_t names_cap, double *ms, int64_t *count, int32_t cap) {
    if (!ctx) return ENSI_E_BADARG;
    for (auto &p : ctx->pending) {
        (void)hipEventSynchronize(p.second.second);
        float t = 0;
        if (hipEventElapsedTime(&t, p.second.first, p.second.second) == hipSuccess) {
            ctx->timers[p.first].ms += t;
            ctx->timers[p.first].count += 1;
        }
        (void)hipEventDestroy(p.second.first);
        (void)hipEventDestroy(p.second.second);
    }
    ctx->pending.clear();
    std::string names;
    int n = 0;
    for (auto &t : ctx->timers) {
        if (n < cap) {
            if (ms) ms[n] = t.ms;
            if (count) count[n] = t.count;
        }
        names += t.name;
        names += '\n';
        n++;
    }
    if (names_out && names_cap > 0) {
        strncpy(names_out, names.c_str(), names_cap - 1);
        names_out[names_cap - 1] = 0;
    }
    for (auto &t : ctx->timers) {
        t.ms = 0;
        t.count = 0;
    }
    return n;
}

// --------------------------------------------------------------------- context
static void free_plan(MatmulPlan *p);
static bool find_primes(int bits, int count, u64 two_n, const std::vector<u64> &skip, std::vector<u64> &out) {
    u64 x = (((u64)1 << bits) - 1) / two_n * two_n + 1;
    if (x >= ((u64)1 << bits)) x -= two_n;
    while ((int)out.size() < count) {
        if (x < two_n) return false;
        if (std::find(skip.begin(), skip.end(), x) == skip.end() && hm_is_prime(x)) out.push_back(x);
        x -= two_n;
    }
    return true;
}

extern "C" int ensi_ctx_create(const ensi_params *prm, ensi_ctx **out) {
    if (!prm || !out) return ENSI_E_BADARG;
    *out = nullptr;
    if (prm->log_n < 4 || prm->log_n > 16 || prm->q_bits < 20 || prm->q_bits > 60 || prm->p_bits < 20 || prm->p_bits > 61 ||
        prm->q_count < 1 || prm->p_count < 1 || prm->p_count > ENSI_MAX_K || prm->q_count + prm->p_count > ENSI_MAX_EXT ||
        prm->alpha < 1 || prm->alpha > ENSI_MAX_ALPHA || prm->log_scale < 1 || prm->log_scale > 60 ||
        (prm->q_count + prm->alpha - 1) / prm->alpha > 8)
        return ENSI_E_BADARG;
    ensi_ctx *ctx = new ensi_ctx();
    ctx->prm = *prm;
    ctx->log_n = prm->log_n;
    ctx->N = 1 << prm->log_n;
    ctx->L = prm->q_count;
    ctx->K = prm->p_count;
    ctx->alpha = prm->alpha;
    ctx->scale = ldexp(1.0, prm->log_scale);
    const int N = ctx->N;
    const u64 two_n = 2 * (u64)N;
    if (hipGetDevice(&ctx->device) != hipSuccess) {
        delete ctx;
        return ENSI_E_HIP;
    }
    std::vector<u64> qs, ps;
    if (!find_primes(prm->q_bits, ctx->L, two_n, {}, qs) || !find_primes(prm->p_bits, ctx->K, two_n, qs, ps)) {
        delete ctx;
        return ENSI_E_BADARG;
    }
    ctx->primes = qs;
    ctx->primes.insert(ctx->primes.end(), ps.begin(), ps.end());
    const int np = ctx->L + ctx->K;

    std::vector<PrimeConst> pcs(np);
    std::vector<u64> tw((size_t)np * 4 * N);
    for (int i = 0; i < np; i++) {
        const u64 q = ctx->primes[i];
        u64 psi = 0;
        for (u64 g = 2; g < 1000 && !psi; g++) {
            u64 c = hm_powmod(g, (q - 1) / two_n, q);
            if (hm_powmod(c, N, q) == q - 1) psi = c;
        }
        if (!psi) {
            delete ctx;
            return ENSI_E_BADARG;
        }
        ctx->psi.push_back(psi);
        PrimeConst &pc = pcs[i];
        memset(&pc, 0, sizeof(pc));
        pc.q = q;
        pc.qneg_inv = hm_neg_inv64(q);
        u64 r = hm_to_mont(1, q);
        pc.r2 = hm_mulmod(r, r, q);
        pc.n_inv = hm_invmod((u64)N % q, q);
        pc.n_inv_s = hm_shoup(pc.n_inv, q);
        // N = 2^16 rings transform limbs with primes below 2^50 in fp64 (see ntt16.hip)
        const bool fp = ctx->log_n == 16 && q < ((u64)1 << 50);
        if (fp) {
            const double qi = 1.0 / (double)q, nq = (double)pc.n_inv / (double)q;
            pc.pad[0] = 1;
            memcpy(&pc.pad[1], &qi, 8);
            memcpy(&pc.pad[2], &nq, 8);
        }
        // powers of psi and psi^{-1}, then bit-reversed tables
        std::vector<u64> pw(N), ipw(N);
        const u64 psi_inv = hm_invmod(psi, q);
        pw[0] = ipw[0] = 1;
        for (int k = 1; k < N; k++) {
            pw[k] = hm_mulmod(pw[k - 1], psi, q);
            ipw[k] = hm_mulmod(ipw[k - 1], psi_inv, q);
        }
        u64 *t = tw.data() + (size_t)i * 4 * N;
        for (int k = 0; k < N; k++) {
            u32 rk = 0;
            for (int b = 0; b < ctx->log_n; b++) rk |= ((k >> b) & 1u) << (ctx->log_n - 1 - b);
            if (fp) {
                // fp64 path: the table holds the twiddle and twiddle/q as doubles
                const double w = (double)pw[rk], wi = (double)ipw[rk];
                const double wq = w / (double)q, wiq = wi / (double)q;
                memcpy(&t[k], &w, 8);
                memcpy(&t[N + k], &wq, 8);
                memcpy(&t[2 * N + k], &wi, 8);
                memcpy(&t[3 * N + k], &wiq, 8);
            } else {
                t[k] = pw[rk];
                t[N + k] = hm_shoup(pw[rk], q);
                t[2 * N + k] = ipw[rk];
                t[3 * N + k] = hm_shoup(ipw[rk], q);
            }
        }
    }
    // the fused key-switching kernels need every ciphertext prime on the fp64 path
    ctx->ks16 = ctx->log_n == 16;
    for (int i = 0; i < ctx->L; i++) ctx->ks16 = ctx->ks16 && pcs[i].pad[0] != 0;
    std::vector<double> cs(2 * (size_t)N);
    for (size_t e = 0; e < cs.size(); e++) cs[e] = (double)cosl(M_PIl * (long double)e / (long double)N);
    ctx->rot_exp.resize(N / 2);
    u64 x = 1;
    for (int j = 0; j < N / 2; j++) {
        ctx->rot_exp[j] = (u32)x;
        x = x * 5 % two_n;
    }
    if (upload(&ctx->d_pc, pcs) != hipSuccess || upload(&ctx->d_tw, tw) != hipSuccess || upload(&ctx->d_cos, cs) != hipSuccess ||
        upload(&ctx->d_rot_exp, ctx->rot_exp) != hipSuccess) {
        ensi_ctx_free(ctx);
        return ENSI_E_HIP;
    }
    // Everything later calls would otherwise create on first use, so that the allocation-free entry point never has to:
    // the staging ring, the conversion constants of every level, the address of the static workspace.
    int rc = stage_prealloc(ctx);
    for (int l1 = 1; l1 <= ctx->L && !rc; l1++) {
        if (ctx->ks16) {
            const Ks16Const *kc;
            rc = get_ks16(ctx, l1, &kc);
        } else {
            const ModUpConst *mu;
            const ModDownConst *md;
            rc = get_modup(ctx, l1, &mu);
            if (!rc) rc = get_moddown(ctx, l1, &md);
        }
    }
    if (!rc) rc = ensi_static_init(ctx);
    if (rc) {
        ensi_ctx_free(ctx);
        return rc;
    }
    *out = ctx;
    return ENSI_OK;
}

static void free_modconst(ensi_ctx *ctx) {
    for (auto &kv : ctx->ks16c) {
        (void)hipFree((void *)kv.second.hat_fp);
        (void)hipFree((void *)kv.second.pmod_fp);
        (void)hipFree((void *)kv.second.down_p);
        (void)hipFree((void *)kv.second.down_p_fp);
        (void)hipFree((void *)kv.second.down_q);
    }
    for (auto &kv : ctx->modup) {
        (void)hipFree(kv.second.inv);
        (void)hipFree(kv.second.inv_s);
        (void)hipFree(kv.second.hat);
    }
    for (auto &kv : ctx->moddown) {
        (void)hipFree(kv.second.inv);
        (void)hipFree(kv.second.inv_s);
        (void)hipFree(kv.second.hat);
        (void)hipFree(kv.second.pinv);
        (void)hipFree(kv.second.pinv_s);
        (void)hipFree(kv.second.negtab);
    }
}

extern "C" void ensi_ctx_free(ensi_ctx *ctx) {
    if (!ctx) return;
    (void)hipDeviceSynchronize();
    free_modconst(ctx);
    if (ctx->d_pc) (void)hipFree(ctx->d_pc);
    if (ctx->d_tw) (void)hipFree(ctx->d_tw);
    if (ctx->d_cos) (void)hipFree(ctx->d_cos);
    if (ctx->d_rot_exp) (void)hipFree(ctx->d_rot_exp);
    if (ctx->ws_digits) (void)hipFree(ctx->ws_digits);
    if (ctx->ws_u) (void)hipFree(ctx->ws_u);
    if (ctx->ws_y) (void)hipFree(ctx->ws_y);
    if (ctx->ws_ysp) (void)hipFree(ctx->ws_ysp);
    if (ctx->ws_virt) (void)hipFree(ctx->ws_virt);
    if (ctx->ws_desc) (void)hipFree(ctx->ws_desc);
    if (ctx->ws_plan) (void)hipFree(ctx->ws_plan);
    if (ctx->ws_xp) (void)hipFree(ctx->ws_xp);
    if (ctx->ws_pa) (void)hipFree(ctx->ws_pa);
    if (ctx->ws_pb) (void)hipFree(ctx->ws_pb);
    if (ctx->ws_pl) (void)hipFree(ctx->ws_pl);
    if (ctx->ws_pt) (void)hipFree(ctx->ws_pt);
    if (ctx->ws_rot) (void)hipFree(ctx->ws_rot);
    if (ctx->ws_ma) (void)hipFree(ctx->ws_ma);
    if (ctx->ws_md) (void)hipFree(ctx->ws_md);
    if (ctx->ws_me) (void)hipFree(ctx->ws_me);
    if (ctx->ws_mt) (void)hipFree(ctx->ws_mt);
    if (ctx->ws_rep) (void)hipFree(ctx->ws_rep);
    if (ctx->ws_rtmp) (void)hipFree(ctx->ws_rtmp);
    for (MatmulPlan *p : ctx->plans) free_plan(p);
    for (StageSlot &sl : ctx->stage) {
        if (sl.host) (void)hipHostFree(sl.host);
        if (sl.ev) (void)hipEventDestroy(sl.ev);
    }
    for (auto &p : ctx->pending) {
        (void)hipEventDestroy(p.second.first);
        (void)hipEventDestroy(p.second.second);
    }
    delete ctx;
}

extern "C" const char *ensi_last_error(const ensi_ctx *ctx) { return ctx ? ctx->err.c_str() : "null context"; }

extern "C" int ensi_get_primes(const ensi_ctx *ctx, uint64_t *q, uint64_t *p) {
    if (!ctx) return ENSI_E_BADARG;
    if (q) memcpy(q, ctx->primes.data(), sizeof(u64) * ctx->L);
    if (p) memcpy(p, ctx->primes.data() + ctx->L, sizeof(u64) * ctx->K);
    return ENSI_OK;
}

// Conversion constants at level l1 (built once per level, kept for the context's life).
int get_modup(ensi_ctx *ctx, int l1, const ModUpConst **out) {
    auto it = ctx->modup.find(l1);
    if (it == ctx->modup.end()) {
        ModUpConst mc;
        memset(&mc, 0, sizeof(mc));
        mc.l1 = l1;
        mc.K = ctx->K;
        mc.alpha = ctx->alpha;
        mc.beta = (l1 + ctx->alpha - 1) / ctx->alpha;
        const int ext = l1 + ctx->K;
        std::vector<u64> inv((size_t)mc.beta * mc.alpha, 0), inv_s(inv.size(), 0), hat((size_t)mc.beta * ext * mc.alpha, 0);
        for (int j = 0; j < mc.beta; j++) {
            const int first = j * mc.alpha;
            const int ns = std::min(mc.alpha, l1 - first);
            mc.n_src[j] = ns;
            for (int a = 0; a < ns; a++) {
                const u64 qa = ctx->primes[first + a];
                u64 prod = 1;  // (Q_j/q_a) mod q_a
                for (int b = 0; b < ns; b++)
                    if (b != a) prod = hm_mulmod(prod, ctx->primes[first + b] % qa, qa);
                inv[j * mc.alpha + a] = hm_invmod(prod, qa);
                inv_s[j * mc.alpha + a] = hm_shoup(inv[j * mc.alpha + a], qa);
                for (int e = 0; e < ext; e++) {
                    if (e >= first && e < first + ns) continue;
                    const u64 t = ctx->primes[e < l1 ? e : ctx->L + (e - l1)];
                    u64 h = 1;
                    for (int b = 0; b < ns; b++)
                        if (b != a) h = hm_mulmod(h, ctx->primes[first + b] % t, t);
                    hat[((size_t)j * ext + e) * mc.alpha + a] = hm_to_mont(h, t);
                }
            }
        }
        if (upload(&mc.inv, inv) != hipSuccess || upload(&mc.inv_s, inv_s) != hipSuccess || upload(&mc.hat, hat) != hipSuccess)
            ENSI_FAIL(ctx, ENSI_E_HIP, "uploading ModUp constants failed");
        it = ctx->modup.insert({l1, mc}).first;
    }
    *out = &it->second;
    return ENSI_OK;
}

int get_moddown(ensi_ctx *ctx, int l1, const ModDownConst **out) {
    auto it = ctx->moddown.find(l1);
    if (it == ctx->moddown.end()) {
        ModDownConst mc;
        memset(&mc, 0, sizeof(mc));
        mc.l1 = l1;
        mc.K = ctx->K;
        const int K = ctx->K, L = ctx->L;
        std::vector<u64> inv(K), inv_s(K), hat((size_t)l1 * K), pinv(l1), pinv_s(l1), negtab((size_t)l1 * (K + 1));
        for (int k = 0; k < K; k++) {
            const u64 pk = ctx->primes[L + k];
            u64 prod = 1;
            for (int b = 0; b < K; b++)
                if (b != k) prod = hm_mulmod(prod, ctx->primes[L + b] % pk, pk);
            inv[k] = hm_invmod(prod, pk);
            inv_s[k] = hm_shoup(inv[k], pk);
        }
        for (int i = 0; i < l1; i++) {
            const u64 q = ctx->primes[i];
            u64 P = 1;
            for (int b = 0; b < K; b++) P = hm_mulmod(P, ctx->primes[L + b] % q, q);
            pinv[i] = hm_invmod(P, q);
            pinv_s[i] = hm_shoup(pinv[i], q);
            for (int j = 0; j <= K; j++) negtab[(size_t)i * (K + 1) + j] = hm_mulmod((u64)j, P, q);
            for (int k = 0; k < K; k++) {
                u64 h = 1;
                for (int b = 0; b < K; b++)
                    if (b != k) h = hm_mulmod(h, ctx->primes[L + b] % q, q);
                hat[(size_t)i * K + k] = hm_to_mont(h, q);
            }
        }
        if (upload(&mc.inv, inv) != hipSuccess || upload(&mc.inv_s, inv_s) != hipSuccess || upload(&mc.hat, hat) != hipSuccess ||
            upload(&mc.pinv, pinv) != hipSuccess || upload(&mc.pinv_s, pinv_s) != hipSuccess || upload(&mc.negtab, negtab) != hipSuccess)
            ENSI_FAIL(ctx, ENSI_E_HIP, "uploading ModDown constants failed");
        it = ctx->moddown.insert({l1, mc}).first;
    }
    *out = &it->second;
    return ENSI_OK;
}

// Constants of the fused N = 2^16 key switch at level l1 (shares the integer ModUp tables).
int get_ks16(ensi_ctx *ctx, int l1, const Ks16Const **out) {
    auto it = ctx->ks16c.find(l1);
    if (it == ctx->ks16c.end()) {
        const ModUpConst *mu;
        int rc = get_modup(ctx, l1, &mu);
        if (rc) return rc;
        Ks16Const kc;
        memset(&kc, 0, sizeof(kc));
        const int K = ctx->K, L = ctx->L, ext = l1 + K, alpha = ctx->alpha;
        kc.l1 = l1;
        kc.K = K;
        kc.L = L;
        kc.alpha = alpha;
        kc.beta = mu->beta;
        for (int j = 0; j < 8; j++) kc.n_src[j] = mu->n_src[j];
        kc.inv = mu->inv;  // [beta][alpha] with digit j starting at limb j*alpha: the index is the limb itself
        kc.inv_s = mu->inv_s;
        kc.hat_mont = mu->hat;
        const u64 n_ring = (u64)ctx->N;
        auto prime_of = [&](int e) { return ctx->primes[e < l1 ? e : L + (e - l1)]; };
        auto is_fp = [&](u64 t) { return t < ((u64)1 << 50); };
        std::vector<double> hat_fp((size_t)kc.beta * ext * alpha * 2, 0.0), pmod((size_t)l1 * 2), down_p_fp((size_t)K * 2, 0.0),
            down_q((size_t)l1 * (2 + 4 * K));
        std::vector<u64> down_p((size_t)K * 2);
        for (int j = 0; j < kc.beta; j++) {
            const int first = j * alpha, ns = kc.n_src[j];
            for (int e = 0; e < ext; e++) {
                const u64 t = prime_of(e);
                if ((e >= first && e < first + ns) || !is_fp(t)) continue;
                for (int a = 0; a < ns; a++) {
                    u64 h = 1;
                    for (int b = 0; b < ns; b++)
                        if (b != a) h = hm_mulmod(h, ctx->primes[first + b] % t, t);
                    hat_fp[(((size_t)j * ext + e) * alpha + a) * 2] = (double)h;
                    hat_fp[(((size_t)j * ext + e) * alpha + a) * 2 + 1] = (double)h / (double)t;
                }
            }
        }
        for (int i = 0; i < l1; i++) {
            const u64 q = ctx->primes[i];
            u64 P = 1;
            for (int b = 0; b < K; b++) P = hm_mulmod(P, ctx->primes[L + b] % q, q);
            pmod[2 * i] = (double)P;
            pmod[2 * i + 1] = (double)P / (double)q;
            double *dq = &down_q[(size_t)i * (2 + 4 * K)];
            const u64 sc = hm_mulmod(hm_invmod(n_ring % q, q), hm_invmod(P, q), q);
            dq[0] = (double)sc;
            dq[1] = (double)sc / (double)q;
            for (int k = 0; k < K; k++) {
                const u64 h = hm_invmod(ctx->primes[L + k] % q, q);
                const u64 h30 = hm_mulmod(h, ((u64)1 << 30) % q, q);
                dq[2 + 4 * k] = (double)h;
                dq[3 + 4 * k] = (double)h / (double)q;
                dq[4 + 4 * k] = (double)h30;
                dq[5 + 4 * k] = (double)h30 / (double)q;
            }
        }
        for (int k = 0; k < K; k++) {
            const u64 pk = ctx->primes[L + k];
            u64 prod = 1;
            for (int b = 0; b < K; b++)
                if (b != k) prod = hm_mulmod(prod, ctx->primes[L + b] % pk, pk);
            const u64 cs = hm_mulmod(hm_invmod(n_ring % pk, pk), hm_invmod(prod, pk), pk);
            down_p[2 * k] = cs;
            down_p[2 * k + 1] = hm_shoup(cs, pk);
            if (is_fp(pk)) {
                down_p_fp[2 * k] = (double)cs;
                down_p_fp[2 * k + 1] = (double)cs / (double)pk;
            }
        }
        double *d_hat = nullptr, *d_pmod = nullptr, *d_dpf = nullptr, *d_dq = nullptr;
        u64 *d_dp = nullptr;
        if (upload(&d_hat, hat_fp) != hipSuccess || upload(&d_pmod, pmod) != hipSuccess || upload(&d_dp, down_p) != hipSuccess ||
            upload(&d_dpf, down_p_fp) != hipSuccess || upload(&d_dq, down_q) != hipSuccess)
            ENSI_FAIL(ctx, ENSI_E_HIP, "uploading key-switch constants failed");
        kc.hat_fp = d_hat;
        kc.pmod_fp = d_pmod;
        kc.down_p = d_dp;
        kc.down_p_fp = d_dpf;
        kc.down_q = d_dq;
        it = ctx->ks16c.insert({l1, kc}).first;
    }
    *out = &it->second;
    return ENSI_OK;
}

// ------------------------------------------------------------------ plaintexts
static int pt_from_coeffs(ensi_ctx *ctx, const int64_t *d_coeffs, int n_pt, int limbs, double scale, ensi_pt **out) {
    ensi_pt *pt = new ensi_pt();
    pt->ctx = ctx;
    pt->n = n_pt;
    pt->limbs = limbs;
    pt->scale = scale;
    pt->d = nullptr;
    if (hipMalloc((void **)&pt->d, (size_t)n_pt * limbs * ctx->N * 8) != hipSuccess) {
        delete pt;
        ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation failed for plaintext");
    }
    launch_i64_to_rns(ctx, d_coeffs, n_pt, make_map(ctx, limbs, false), pt->d, nullptr);
    if (hipStreamSynchronize(nullptr) != hipSuccess) {
        ensi_pt_free(pt);
        ENSI_FAIL(ctx, ENSI_E_HIP, "kernel failure in plaintext conversion");
    }
    *out = pt;
    return ENSI_OK;
}

// slots: host [n_pt][n_slots]; plaintext y holds its values in slots [slot0 + y*slot_step, ...+n_slots)
static int encode_window(ensi_ctx *ctx, const double *slots, int n_pt, int n_slots, int slot0, int slot_step, int limbs, double scale,
                         ensi_pt **out) {
    DevBuf d_slots, d_coeffs;
    if (d_slots.alloc((size_t)n_pt * n_slots * 8) != hipSuccess || d_coeffs.alloc((size_t)n_pt * ctx->N * 8) != hipSuccess)
        ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation failed in encode");
    ENSI_HIP(ctx, hipMemcpy(d_slots.p, slots, (size_t)n_pt * n_slots * 8, hipMemcpyHostToDevice));
    launch_encode(ctx, d_slots.as<double>(), n_pt, n_slots, slot0, slot_step, scale, d_coeffs.as<int64_t>(), nullptr);
    return pt_from_coeffs(ctx, d_coeffs.as<int64_t>(), n_pt, limbs, scale, out);
}
extern "C" int ensi_encode(ensi_ctx *ctx, const double *slots, int32_t n_pt, int32_t n_slots, int32_t limbs, ensi_pt **out) {
    if (!ctx || !slots || !out || n_pt < 1 || n_slots < 1 || n_slots > ctx->N / 2 || limbs < 1 || limbs > ctx->L) return ENSI_E_BADARG;
    return encode_window(ctx, slots, n_pt, n_slots, 0, 0, limbs, ctx->scale, out);
}
extern "C" int ensi_encode_at(ensi_ctx *ctx, const double *slots, int32_t n_pt, int32_t n_slots, int32_t limbs, double scale, ensi_pt **out) {
    if (!ctx || !slots || !out || n_pt < 1 || n_slots < 1 || n_slots > ctx->N / 2 || limbs < 1 || limbs > ctx->L) return ENSI_E_BADARG;
    if (!(scale >= 1.0) || !(scale < 9.0e18)) return ENSI_E_BADARG;
    return encode_window(ctx, slots, n_pt, n_slots, 0, 0, limbs, scale, out);
}
extern "C" int ensi_pt_set_scale(ensi_pt *pt, double scale) {
    if (!pt || !(scale > 0)) return ENSI_E_BADARG;
    pt->scale = scale;
    return ENSI_OK;
}
extern "C" int ensi_pt_import(ensi_ctx *ctx, const int64_t *coeffs, int32_t n_pt, int32_t limbs, ensi_pt **out) {
    if (!ctx || !coeffs || !out || n_pt < 1 || limbs < 1 || limbs > ctx->L) return ENSI_E_BADARG;
    DevBuf d_coeffs;
    if (d_coeffs.alloc((size_t)n_pt * ctx->N * 8) != hipSuccess) ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation failed in pt_import");
    ENSI_HIP(ctx, hipMemcpy(d_coeffs.p, coeffs, (size_t)n_pt * ctx->N * 8, hipMemcpyHostToDevice));
    return pt_from_coeffs(ctx, d_coeffs.as<int64_t>(), n_pt, limbs, ctx->scale, out);
}
extern "C" int ensi_pt_export(ensi_ctx *ctx, const ensi_pt *pt, int64_t *coeffs) {
    if (!ctx || !pt || !coeffs) return ENSI_E_BADARG;
    DevBuf d_out;
    if (d_out.alloc((size_t)pt->n * ctx->N * 8) != hipSuccess) ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation failed in pt_export");
    launch_center_i64(ctx, pt->d, (size_t)pt->limbs * ctx->N, pt->n, d_out.as<int64_t>(), nullptr);
    ENSI_HIP(ctx, hipMemcpy(coeffs, d_out.p, (size_t)pt->n * ctx->N * 8, hipMemcpyDeviceToHost));
    return ENSI_OK;
}
extern "C" void ensi_pt_free(ensi_pt *pt) {
    if (!pt) return;
    if (pt->d) (void)hipFree(pt->d);
    if (pt->d_mont) (void)hipFree(pt->d_mont);
    if (pt->d_fp) (void)hipFree(pt->d_fp);
    delete pt;
}

// ----------------------------------------------------------------- ciphertexts
extern "C" int ensi_ct_alloc(ensi_ctx *ctx, int32_t n, int32_t limbs, ensi_ct **out) {
    if (!ctx || !out || n < 1 || limbs < 1 || limbs > ctx->L) return ENSI_E_BADARG;
    ensi_ct *ct = new ensi_ct();
    ct->ctx = ctx;
    ct->n = n;
    ct->limbs = ct->limbs_alloc = limbs;
    ct->scale = ctx->scale;
    ct->owns = true;
    ct->d = nullptr;
    hipError_t e = hipMalloc((void **)&ct->d, (size_t)n * 2 * limbs * ctx->N * 8);
    if (e != hipSuccess) {
        delete ct;
        ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation of %zu bytes failed: %s", (size_t)n * 2 * limbs * ctx->N * 8, hipGetErrorString(e));
    }
    *out = ct;
    return ENSI_OK;
}
extern "C" int ensi_ct_wrap(ensi_ctx *ctx, void *device_words, int32_t n, int32_t limbs, double scale, ensi_ct **out) {
    if (!ctx || !out || !device_words || n < 1 || limbs < 1 || limbs > ctx->L) return ENSI_E_BADARG;
    ensi_ct *ct = new ensi_ct();
    ct->ctx = ctx;
    ct->n = n;
    ct->limbs = ct->limbs_alloc = limbs;
    ct->scale = scale;
    ct->owns = false;
    ct->d = (u64 *)device_words;
    *out = ct;
    return ENSI_OK;
}
extern "C" void ensi_ct_free(ensi_ct *ct) {
    if (!ct) return;
    if (ct->owns && ct->d) (void)hipFree(ct->d);
    delete ct;
}
extern "C" int ensi_ct_info(const ensi_ct *ct, int32_t *n, int32_t *limbs, double *scale, void **device_words) {
    if (!ct) return ENSI_E_BADARG;
    if (n) *n = ct->n;
    if (limbs) *limbs = ct->limbs;
    if (scale) *scale = ct->scale;
    if (device_words) *device_words = ct->d;
    return ENSI_OK;
}
extern "C" int ensi_ct_export(ensi_ctx *ctx, const ensi_ct *ct, uint64_t *out) {
    if (!ctx || !ct || !out) return ENSI_E_BADARG;
    if (ct->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "the batch holds prepared weights, which only ensi_ccmm_av reads");
    const size_t N = ctx->N;
    ENSI_HIP(ctx, hipDeviceSynchronize());
    if (ct->limbs == ct->limbs_alloc) {
        ENSI_HIP(ctx, hipMemcpy(out, ct->d, (size_t)ct->n * 2 * ct->limbs * N * 8, hipMemcpyDeviceToHost));
    } else {
        ENSI_HIP(ctx, hipMemcpy2D(out, (size_t)ct->limbs * N * 8, ct->d, (size_t)ct->limbs_alloc * N * 8, (size_t)ct->limbs * N * 8,
                                  (size_t)ct->n * 2, hipMemcpyDeviceToHost));
    }
    return ENSI_OK;
}
extern "C" int ensi_ct_import(ensi_ctx *ctx, const uint64_t *in, int32_t n, int32_t limbs, double scale, ensi_ct **out) {
    if (!ctx || !in || !out) return ENSI_E_BADARG;
    for (int l = 0; l < limbs && l < ctx->L; l++) {
        // spot-check canonical range on the first words of each limb of the first ciphertext
        for (int i = 0; i < 4 && i < ctx->N; i++)
            if (in[(size_t)l * ctx->N + i] >= ctx->primes[l]) ENSI_FAIL(ctx, ENSI_E_BADARG, "imported residue not below q_%d", l);
    }
    int rc = ensi_ct_alloc(ctx, n, limbs, out);
    if (rc) return rc;
    (*out)->scale = scale;
    hipError_t e = hipMemcpy((*out)->d, in, (size_t)n * 2 * limbs * ctx->N * 8, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        ensi_ct_free(*out);
        *out = nullptr;
        ENSI_FAIL(ctx, ENSI_E_HIP, "upload failed: %s", hipGetErrorString(e));
    }
    return ENSI_OK;
}

extern "C" int ensi_ct_checksum(ensi_ctx *ctx, const ensi_ct *ct, uint64_t *sums, void *stream) {
    if (!ctx || !ct || !sums) return ENSI_E_BADARG;
    if (ct->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "the batch holds prepared weights, which only ensi_ccmm_av reads");
    hipStream_t st = (hipStream_t)stream;
    DevBuf d_sums;
    if (d_sums.alloc((size_t)ct->n * 8) != hipSuccess) ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation failed in ct_checksum");
    ENSI_HIP(ctx, hipMemsetAsync(d_sums.p, 0, (size_t)ct->n * 8, st));
    launch_ct_checksum(ctx, ct->d, ct->n, ct->limbs, ct->limbs_alloc, d_sums.as<u64>(), st);
    ENSI_HIP(ctx, hipMemcpyAsync(sums, d_sums.p, (size_t)ct->n * 8, hipMemcpyDeviceToHost, st));
    ENSI_HIP(ctx, hipStreamSynchronize(st));
    return ENSI_OK;
}

extern "C" int ensi_encrypt(ensi_ctx *ctx, const ensi_pk *pk, const ensi_pt *pt, const int8_t *v, const int8_t *e0, const int8_t *e1,
                            ensi_ct **out) {
    if (!ctx || !pk || !pt || !out) return ENSI_E_BADARG;
    if (!((v && e0 && e1) || (!v && !e0 && !e1))) ENSI_FAIL(ctx, ENSI_E_BADARG, "v, e0, e1 must be all given or all NULL");
    const int N = ctx->N, L = ctx->L, l1 = pt->limbs, n = pt->n;
    const size_t pn = (size_t)n * N;
    std::vector<int8_t> small(3 * pn);
    if (v) {
        memcpy(small.data(), v, pn);
        memcpy(small.data() + pn, e0, pn);
        memcpy(small.data() + 2 * pn, e1, pn);
    } else {
        int rs;
        if ((rs = sample_ternary(ctx, small.data(), pn)) || (rs = sample_error(ctx, small.data() + pn, 2 * pn))) return rs;
    }
    int rc = ensi_ct_alloc(ctx, n, l1, out);
    if (rc) return rc;
    ensi_ct *ct = *out;
    hipStream_t st = nullptr;
    LimbMap mq = make_map(ctx, l1, false);
    DevBuf d_small, d_v, d_t, d_e;
    const size_t rows = (size_t)n * l1;
    if (d_small.alloc(3 * pn) != hipSuccess || d_v.alloc(rows * N * 8) != hipSuccess || d_t.alloc(rows * N * 8) != hipSuccess ||
        d_e.alloc(rows * N * 8) != hipSuccess) {
        ensi_ct_free(ct);
        *out = nullptr;
        ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation failed in encrypt");
    }
    (void)hipMemcpy(d_small.p, small.data(), 3 * pn, hipMemcpyHostToDevice);
    // v: residues -> transform domain
    launch_small_to_rns(ctx, d_small.as<int8_t>(), n, mq, d_v.as<u64>(), st);
    launch_ntt(ctx, d_v.as<u64>(), (int)rows, mq, false, st);
    for (int poly = 0; poly < 2; poly++) {
        // t = v * pk[poly] (rows 0..l1-1 of the L-limb key), back to coefficient form
        for (int c = 0; c < n; c++)
            launch_mul_mont(ctx, d_t.as<u64>() + (size_t)c * l1 * N, d_v.as<u64>() + (size_t)c * l1 * N, pk->d_pk + (size_t)poly * L * N, l1,
                            mq, st);
        launch_ntt(ctx, d_t.as<u64>(), (int)rows, mq, true, st);
        // + error (+ message on c0)
        launch_small_to_rns(ctx, d_small.as<int8_t>() + (1 + poly) * pn, n, mq, d_e.as<u64>(), st);
        for (int c = 0; c < n; c++) {
            u64 *dst = ct->d + ((size_t)c * 2 + poly) * l1 * N;
            launch_add(ctx, dst, d_t.as<u64>() + (size_t)c * l1 * N, d_e.as<u64>() + (size_t)c * l1 * N, l1, mq, st);
            if (poly == 0) launch_add(ctx, dst, dst, pt->d + (size_t)c * l1 * N, l1, mq, st);
        }
    }
    if (hipStreamSynchronize(st) != hipSuccess || hipGetLastError() != hipSuccess) {
        ensi_ct_free(ct);
        *out = nullptr;
        ENSI_FAIL(ctx, ENSI_E_HIP, "kernel failure in encrypt");
    }
    return ENSI_OK;
}

extern "C" int ensi_decrypt(ensi_ctx *ctx, const ensi_sk *sk, const ensi_ct *ct, int32_t slot_begin, int32_t n_slots, double *slots_out) {
    if (!ctx || !sk || !ct || !slots_out || slot_begin < 0 || n_slots < 1 || slot_begin + n_slots > ctx->N / 2) return ENSI_E_BADARG;
    if (ct->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "the batch holds prepared weights, which only ensi_ccmm_av reads");
    const int N = ctx->N, n = ct->n;
    const int use = std::min(ct->limbs, 2);
    hipStream_t st = nullptr;
    LimbMap mq = make_map(ctx, use, false);
    DevBuf d_m, d_coef, d_out;
    if (d_m.alloc((size_t)n * use * N * 8) != hipSuccess || d_coef.alloc((size_t)n * N * 8) != hipSuccess ||
        d_out.alloc((size_t)n * n_slots * 8) != hipSuccess)
        ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation failed in decrypt");
    ENSI_HIP(ctx, hipDeviceSynchronize());
    const size_t poly_words = (size_t)ct->limbs_alloc * N;
    for (int c = 0; c < n; c++)
        ENSI_HIP(ctx, hipMemcpyAsync(d_m.as<u64>() + (size_t)c * use * N, ct->d + ((size_t)c * 2 + 1) * poly_words, (size_t)use * N * 8,
                                     hipMemcpyDeviceToDevice, st));
    launch_ntt(ctx, d_m.as<u64>(), n * use, mq, false, st);
    for (int c = 0; c < n; c++) {
        u64 *mc = d_m.as<u64>() + (size_t)c * use * N;
        launch_mul_mont(ctx, mc, mc, sk->d_s_hat, use, mq, st);
    }
    launch_ntt(ctx, d_m.as<u64>(), n * use, mq, true, st);
    for (int c = 0; c < n; c++) {
        u64 *mc = d_m.as<u64>() + (size_t)c * use * N;
        launch_add(ctx, mc, mc, ct->d + (size_t)c * 2 * poly_words, use, mq, st);
    }
    launch_crt_center(ctx, d_m.as<u64>(), n, use, d_coef.as<double>(), st);
    launch_decode(ctx, d_coef.as<double>(), n, slot_begin, n_slots, 1.0 / ct->scale, d_out.as<double>(), st);
    ENSI_HIP(ctx, hipStreamSynchronize(st));
    ENSI_HIP(ctx, hipMemcpy(slots_out, d_out.p, (size_t)n * n_slots * 8, hipMemcpyDeviceToHost));
    return ENSI_OK;
}

// --------------------------------------------------------------------- rotation
// Words of the raised form of one ciphertext at level l1 (fused path: digits of c1 and P*c0).
size_t raised_words(const ensi_ctx *ctx, int l1) {
    const size_t ext = l1 + ctx->K, beta = (l1 + ctx->alpha - 1) / ctx->alpha;
    return (beta * ext + (ctx->ks16 ? l1 : 0)) * (size_t)ctx->N;
}

// Digit decomposition, ModUp and forward transform of n_ct ciphertexts into ws_digits (which must hold
// n_ct * raised_words).
// ws: where the intermediates go; nullptr = the context's own workspaces (ws_digits sized by the caller, the rest
// grown here).  With an explicit workspace nothing is allocated.
int raise_cts(ensi_ctx *ctx, int l1, const u64 *ct_base, size_t ct_stride_words, int limb_stride, int n_ct, hipStream_t st,
              const KsWorkspace *ws) {
    int rc;
    u64 *digits = ws ? ws->digits : ctx->ws_digits;
    if (ctx->ks16) {
        const Ks16Const *kc;
        if ((rc = get_ks16(ctx, l1, &kc))) return rc;
        if (!ws && (rc = grow(ctx, &ctx->ws_y, &ctx->ws_y_words, (size_t)n_ct * l1 * ctx->N))) return rc;
        launch_ks16_raise(ctx, *kc, ct_base, ct_stride_words, limb_stride, n_ct, ws ? ws->y : ctx->ws_y, digits, st);
        return ENSI_OK;
    }
    const ModUpConst *mu;
    if ((rc = get_modup(ctx, l1, &mu))) return rc;
    const int ext = l1 + ctx->K, beta = (l1 + ctx->alpha - 1) / ctx->alpha;
    launch_modup(ctx, *mu, ct_base, ct_stride_words, limb_stride, n_ct, digits, st);
    launch_ntt(ctx, digits, n_ct * beta * ext, make_map(ctx, l1, true), false, st);
    return ENSI_OK;
}

// Runs inner product -> inverse transform -> ModDown (+ phi_g(c0)) for n_rot descriptors already on the device.
// members > 1: the descriptors come in groups of `members` rotations of one ciphertext (same source, digits and
// destination); a group's inner products are added over the extended basis and brought back by one inverse
// transform and one ModDown, and the destination receives sum_k phi_{g_k}(c0) with it.  h_desc: host copy of the
// descriptors (needed by the unfused path of a grouped call only).
int run_rotations(ensi_ctx *ctx, const RotDesc *d_desc, int n_rot, int l1, int limb_stride_in, int limb_stride_out, hipStream_t st,
                  int members, const RotDesc *h_desc, const KsWorkspace *ws) {
    int rc;
    u64 *u = ws ? ws->u : ctx->ws_u;
    if (ctx->ks16) {
        const Ks16Const *kc;
        if ((rc = get_ks16(ctx, l1, &kc))) return rc;
        if (!ws && (rc = grow(ctx, &ctx->ws_ysp, &ctx->ws_ysp_words, (size_t)(n_rot / members) * 2 * ctx->K * ctx->N))) return rc;
        launch_ks16_switch(ctx, *kc, d_desc, n_rot, u, ws ? ws->ysp : ctx->ws_ysp, limb_stride_out, st, members);
        return ENSI_OK;
    }
    const ModDownConst *md;
    if ((rc = get_moddown(ctx, l1, &md))) return rc;
    const int ext = l1 + ctx->K, beta = (l1 + ctx->alpha - 1) / ctx->alpha, N = ctx->N;
    const LimbMap mext = make_map(ctx, l1, true);
    launch_inner(ctx, d_desc, n_rot, l1, beta, u, st);
    if (members == 1) {
        launch_ntt(ctx, u, n_rot * 2 * ext, mext, true, st);
        launch_moddown(ctx, *md, d_desc, n_rot, limb_stride_in, limb_stride_out, u, st);
        return ENSI_OK;
    }
    if (ws) ENSI_FAIL(ctx, ENSI_E_BADARG, "grouped rotations run on the context's own workspaces only");
    if (!h_desc) ENSI_FAIL(ctx, ENSI_E_BADARG, "grouped rotations need the host descriptors");
    const LimbMap mq = make_map(ctx, l1, false);
    const size_t W = (size_t)2 * ext * N;  // accumulator words of one rotation
    if ((rc = grow(ctx, &ctx->ws_y, &ctx->ws_y_words, (size_t)l1 * N))) return rc;
    for (int g = 0; g < n_rot / members; g++) {
        u64 *ug = ctx->ws_u + (size_t)g * members * W;
        for (int e = 1; e < members; e++) launch_add(ctx, ug, ug, ug + (size_t)e * W, 2 * ext, mext, st);
        launch_ntt(ctx, ug, 2 * ext, mext, true, st);
        launch_moddown(ctx, *md, d_desc + (size_t)g * members, 1, limb_stride_in, limb_stride_out, ug, st);  // adds phi_{g_0}(c0)
        for (int e = 1; e < members; e++) {
            const RotDesc &h = h_desc[(size_t)g * members + e];
            launch_automorphism_coef(ctx, ctx->ws_y, h.c0, mq, h.g_inv, st);
            launch_add(ctx, h.out, h.out, ctx->ws_y, l1, mq, st);
        }
    }
    return ENSI_OK;
}

// Ciphertexts per group of a batched rotation: bounds the workspace (about 31 MiB of raised digits per
// ciphertext at 13 limbs).  Smaller groups were measured slower: the kernels are not limited by HBM alone,
// so keeping the intermediates of a group inside the memory-side cache gains less than the shorter
// launches lose.
static int rot_chunk() { return 64; }

static int ensure_desc(ensi_ctx *ctx, size_t n) {
    if (ctx->ws_desc_n >= n) return ENSI_OK;
    if (ctx->ws_desc) ENSI_HIP(ctx, hipFree(ctx->ws_desc));
    ctx->ws_desc = nullptr;
    ctx->ws_desc_n = 0;
    if (hipMalloc((void **)&ctx->ws_desc, n * sizeof(RotDesc)) != hipSuccess) ENSI_FAIL(ctx, ENSI_E_NOMEM, "descriptor allocation failed");
    ctx->ws_desc_n = n;
    return ENSI_OK;
}

extern "C" int ensi_rotate(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *in, const int32_t *steps, ensi_ct *out, void *stream) {
    if (!ctx || !gk || !in || !steps || !out) return ENSI_E_BADARG;
    if (in->prepared) ENSI_FAIL(ctx, ENSI_E_BADARG, "a batch of prepared weights is read by ensi_ccmm_segment and ensi_ccmm_av only");
    if (in->n != out->n) ENSI_FAIL(ctx, ENSI_E_SHAPE, "rotate: batch sizes differ (%d vs %d)", in->n, out->n);
    if (in->limbs != out->limbs) ENSI_FAIL(ctx, ENSI_E_LEVEL, "rotate: levels differ (%d vs %d limbs)", in->limbs, out->limbs);
    if (in->d == out->d) ENSI_FAIL(ctx, ENSI_E_BADARG, "rotate: in and out must not overlap");
    hipStream_t st = (hipStream_t)stream;
    const int N = ctx->N, l1 = in->limbs, ext = l1 + ctx->K, n = in->n;
    std::vector<RotDesc> desc(n);
    const size_t in_ct = (size_t)2 * in->limbs_alloc * N, out_ct = (size_t)2 * out->limbs_alloc * N;
    const int chunk = std::min(n, ctx->ks16 ? rot_chunk() : n);
    const size_t rw = raised_words(ctx, l1);
    int rc;
    if ((rc = grow(ctx, &ctx->ws_digits, &ctx->ws_digits_words, (size_t)chunk * rw))) return rc;
    if ((rc = grow(ctx, &ctx->ws_u, &ctx->ws_u_words, (size_t)chunk * 2 * ext * N))) return rc;
    if ((rc = ensure_desc(ctx, n))) return rc;
    for (int c = 0; c < n; c++) {
        const u32 g = galois_element(ctx, steps[c]);
        auto it = gk->keys.find(g);
        if (it == gk->keys.end()) ENSI_FAIL(ctx, ENSI_E_NOKEY, "rotate: no Galois key for step %d", steps[c]);
        desc[c].c0 = in->d + (size_t)c * in_ct;
        desc[c].digits = ctx->ws_digits + (size_t)(c % chunk) * rw;
        desc[c].key = it->second;
        desc[c].out = out->d + (size_t)c * out_ct;
        desc[c].g = g;
        desc[c].g_inv = inv_mod_2n(g, N);
    }
    // inside a group, rotations that use the same key are made neighbours: the blocks reading a key tile then run
    // at nearly the same time on one XCD and share it through L2 (a descriptor carries its own source and
    // destination, so the order inside a launch is free)
    for (int c0 = 0; c0 < n; c0 += chunk)
        std::stable_sort(desc.begin() + c0, desc.begin() + std::min(n, c0 + chunk),
                         [](const RotDesc &a, const RotDesc &b) { return (uintptr_t)a.key < (uintptr_t)b.key; });
    ENSI_HIP(ctx, host_to_device(ctx, ctx->ws_desc, desc.data(), n * sizeof(RotDesc), st));
    for (int c0 = 0; c0 < n; c0 += chunk) {
        const int cnt = std::min(chunk, n - c0);
        if ((rc = raise_cts(ctx, l1, in->d + (size_t)c0 * in_ct, in_ct, in->limbs_alloc, cnt, st))) return rc;
        if ((rc = run_rotations(ctx, ctx->ws_desc + c0, cnt, l1, in->limbs_alloc, out->limbs_alloc, st))) return rc;
    }
    out->scale = in->scale;
    ENSI_HIP(ctx, hipGetLastError());
    return ENSI_OK;
}

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

static void free_plan(MatmulPlan *p) {
    if (!p) return;
    if (p->d_masks) (void)hipFree(p->d_masks);
    if (p->d_wt) (void)hipFree(p->d_wt);
    if (p->d_bias) (void)hipFree(p->d_bias);
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
    hipError_t e1 = upload(&p->d_masks, masks), e2 = hipSuccess, e3 = hipSuccess;
    if (mfma_ok) {
        e2 = upload(&p->d_wt, wt);
        e3 = upload(&p->d_bias, bias);
    }
    if (e1 != hipSuccess || e2 != hipSuccess || e3 != hipSuccess) {
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
        if ((rc = launch_accumulate_mfma(ctx, xbase, in_ct, n_v, plan->n_kpad, plan->d_wt, plan->d_bias, plan->planes, m, l1, in->limbs_alloc,
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
static int upload_rescale_consts(ensi_ctx *ctx, int l1, double kr, bool negative, hipStream_t st, const u64 **d_consts,
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
    if ((rc = launch_accumulate_mfma(ctx, in->d, (size_t)2 * in->limbs_alloc * N, d, plan->n_kpad, plan->d_wt, plan->d_bias, plan->planes, m, l1,
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
static int pmult_core(ensi_ctx *ctx, const std::vector<PmTerm> &terms_in, const std::vector<int32_t> &begin, int l1, int limb_stride_in,
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

// ------------------------------------------------------------------------- NTT
extern "C" int ensi_ntt(ensi_ctx *ctx, void *data, int32_t n_limbs, const int32_t *prime_idx, int32_t inverse, void *stream) {
    if (!ctx || !data || !prime_idx || n_limbs < 1) return ENSI_E_BADARG;
    // rows are grouped into runs that share a periodic prime pattern of at most ENSI_MAX_EXT
    int period = 0;
    for (int p = 1; p <= ENSI_MAX_EXT && p <= n_limbs && !period; p++) {
        bool ok = true;
        for (int r = p; r < n_limbs && ok; r++) ok = prime_idx[r] == prime_idx[r - p];
        if (ok) period = p;
    }
    if (!period) ENSI_FAIL(ctx, ENSI_E_BADARG, "ntt: prime pattern must repeat with period <= %d", ENSI_MAX_EXT);
    LimbMap map;
    map.n = period;
    for (int e = 0; e < ENSI_MAX_EXT; e++) map.prime[e] = 0;
    for (int e = 0; e < period; e++) {
        if (prime_idx[e] < 0 || prime_idx[e] >= ctx->L + ctx->K) ENSI_FAIL(ctx, ENSI_E_BADARG, "ntt: prime index %d out of range", prime_idx[e]);
        map.prime[e] = prime_idx[e];
    }
    launch_ntt(ctx, (u64 *)data, n_limbs, map, inverse != 0, (hipStream_t)stream);
    ENSI_HIP(ctx, hipGetLastError());
    return ENSI_OK;
}
