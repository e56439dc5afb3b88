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
int encode_window(ensi_ctx *ctx, const double *slots, int n_pt, int n_slots, int slot0, int slot_step, int limbs, double scale,
                         ensi_pt **out) {
    DevBuf d_slots, d_coeffs;
    if (d_slots.alloc((size_t)n_pt * n_slots * 8) != hipSuccess || d_coeffs.alloc((size_t)n_pt * ctx->N * 8) != hipSuccess)
        ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation failed in encode");
    ENSI_HIP(ctx, hipMemcpy(d_slots.p, slots, (size_t)n_pt * n_slots * 8, hipMemcpyHostToDevice));
    ENSI_HIP(ctx, launch_encode(ctx, d_slots.as<double>(), n_pt, n_slots, slot0, slot_step, scale, d_coeffs.as<int64_t>(), nullptr));
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
    ENSI_HIP(ctx, launch_decode(ctx, d_coef.as<double>(), n, slot_begin, n_slots, 1.0 / ct->scale, d_out.as<double>(), st));
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
int rot_chunk() { return 64; }

int ensure_desc(ensi_ctx *ctx, size_t n) {
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
