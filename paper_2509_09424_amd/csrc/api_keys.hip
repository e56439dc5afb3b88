// Host side of the library, keys: sampling of the small polynomials, KeyGen (Preliminaries), the hybrid
// key-switching keys of Rot and Mult, and the import/export of key material in coefficient form.
#include <math.h>
#include <stdio.h>
#include <string.h>
#include <sys/random.h>

#include <algorithm>
#include <random>

#include "api_util.h"
#include "common.h"
#include "hostmath.h"

// ------------------------------------------------------------------ sampling
// The library's own sampler, used only where the caller passes NULL randomness.  With params.seed == 0
// the small polynomials (secret key, encryption masks, errors) are drawn from the operating system's
// cryptographic generator; a non-zero seed selects a deterministic generator for reproducible tests and
// benchmarks, whose output anyone who knows the (public) seed can recompute.
namespace {
struct SmallSampler {
    bool os;
    std::mt19937_64 gen;
    unsigned char buf[4096];
    size_t have = 0, pos = 0;
    bool failed = false;
    SmallSampler(ensi_ctx *ctx) : os(ctx->prm.seed == 0), gen(ctx->prm.seed * 0x9E3779B97F4A7C15ULL + (++ctx->sampler_ctr)) {}
    u64 next64() {
        if (!os) return gen();
        if (pos + 8 > have) {
            size_t got = 0;
            while (got < sizeof(buf)) {
                ssize_t r = getrandom(buf + got, sizeof(buf) - got, 0);
                if (r <= 0) {
                    failed = true;
                    memset(buf + got, 0, sizeof(buf) - got);
                    break;
                }
                got += (size_t)r;
            }
            have = sizeof(buf);
            pos = 0;
        }
        u64 v;
        memcpy(&v, buf + pos, 8);
        pos += 8;
        return v;
    }
    double unit() { return ((double)(next64() >> 11) + 0.5) * (1.0 / 9007199254740992.0); }  // (0, 1)
};
}  // namespace

int sample_ternary(ensi_ctx *ctx, int8_t *out, size_t n) {
    SmallSampler sm(ctx);
    size_t i = 0;
    while (i < n) {
        u64 w = sm.next64();
        // two bits per draw, the value 3 rejected: exactly uniform on {-1, 0, 1}
        for (int k = 0; k < 32 && i < n; k++, w >>= 2)
            if ((w & 3) != 3) out[i++] = (int8_t)((int)(w & 3) - 1);
    }
    if (sm.failed) ENSI_FAIL(ctx, ENSI_E_BADARG, "the operating system's random generator is not available");
    return ENSI_OK;
}
int sample_error(ensi_ctx *ctx, int8_t *out, size_t n) {
    SmallSampler sm(ctx);
    // rounded Gaussian, sigma 3.2, clipped at +-19 (Box-Muller on 53-bit uniforms)
    for (size_t i = 0; i < n; i += 2) {
        const double r = sqrt(-2.0 * log(sm.unit())) * 3.2, t = 2.0 * M_PI * sm.unit();
        const double v[2] = {r * cos(t), r * sin(t)};
        for (int k = 0; k < 2 && i + k < n; k++) out[i + k] = (int8_t)std::max(-19.0, std::min(19.0, nearbyint(v[k])));
    }
    if (sm.failed) ENSI_FAIL(ctx, ENSI_E_BADARG, "the operating system's random generator is not available");
    return ENSI_OK;
}

// ------------------------------------------------------------------------ keys
// Secret key handle from its ternary coefficients: residues over Q_L + P -> transform domain -> Montgomery form.
static int make_sk(ensi_ctx *ctx, const std::vector<int8_t> &sv, ensi_sk **out) {
    const int N = ctx->N, ext = ctx->L + ctx->K;
    for (int i = 0; i < N; i++)
        if (sv[i] < -1 || sv[i] > 1) ENSI_FAIL(ctx, ENSI_E_BADARG, "secret coefficient %d outside {-1,0,1}", i);
    hipStream_t st = nullptr;
    LimbMap mext = make_map(ctx, ctx->L, true);
    DevBuf d_small;
    ensi_sk *sk = new ensi_sk();
    sk->ctx = ctx;
    sk->s = sv;
    sk->d_s_hat = nullptr;
    if (d_small.alloc((size_t)N) != hipSuccess || hipMalloc((void **)&sk->d_s_hat, (size_t)ext * N * 8) != hipSuccess) {
        ensi_sk_free(sk);
        ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation failed for the secret key");
    }
    (void)hipMemcpy(d_small.p, sv.data(), N, hipMemcpyHostToDevice);
    launch_small_to_rns(ctx, d_small.as<int8_t>(), 1, mext, sk->d_s_hat, st);
    launch_ntt(ctx, sk->d_s_hat, ext, mext, false, st);
    launch_to_mont(ctx, sk->d_s_hat, ext, mext, st);
    if (hipStreamSynchronize(st) != hipSuccess || hipGetLastError() != hipSuccess) {
        ensi_sk_free(sk);
        ENSI_FAIL(ctx, ENSI_E_HIP, "kernel failure while building the secret key");
    }
    *out = sk;
    return ENSI_OK;
}

extern "C" int ensi_keygen(ensi_ctx *ctx, const int8_t *s, const int8_t *e, uint64_t seed_a, ensi_sk **sk_out, ensi_pk **pk_out) {
    if (!ctx || !sk_out || !pk_out) return ENSI_E_BADARG;
    const int N = ctx->N, L = ctx->L;
    std::vector<int8_t> sv(N), ev(N);
    int rc;
    if (s) memcpy(sv.data(), s, N);
    else if ((rc = sample_ternary(ctx, sv.data(), N))) return rc;
    if (e) memcpy(ev.data(), e, N);
    else if ((rc = sample_error(ctx, ev.data(), N))) return rc;
    ensi_sk *sk = nullptr;
    if ((rc = make_sk(ctx, sv, &sk))) return rc;

    hipStream_t st = nullptr;
    LimbMap mq = make_map(ctx, L, false);
    DevBuf d_small, d_e, d_a;
    ensi_pk *pk = new ensi_pk();
    pk->ctx = ctx;
    pk->d_pk = nullptr;
    auto fail = [&](int code) {
        ensi_sk_free(sk);
        ensi_pk_free(pk);
        return code;
    };
    if (d_small.alloc((size_t)N) != hipSuccess || d_e.alloc((size_t)L * N * 8) != hipSuccess || d_a.alloc((size_t)L * N * 8) != hipSuccess ||
        hipMalloc((void **)&pk->d_pk, (size_t)2 * L * N * 8) != hipSuccess) {
        ctx->err = "device allocation failed in keygen";
        return fail(ENSI_E_NOMEM);
    }
    (void)hipMemcpy(d_small.p, ev.data(), N, hipMemcpyHostToDevice);
    // pk = (-a s + e, a) over Q_L
    u64 *pk_b = pk->d_pk, *pk_a = pk->d_pk + (size_t)L * N;
    launch_uniform(ctx, d_a.as<u64>(), mq, seed_a, 1, st);
    launch_ntt(ctx, d_a.as<u64>(), L, mq, false, st);
    launch_small_to_rns(ctx, d_small.as<int8_t>(), 1, mq, d_e.as<u64>(), st);
    launch_ntt(ctx, d_e.as<u64>(), L, mq, false, st);
    launch_key_assemble(ctx, pk_b, d_a.as<u64>(), sk->d_s_hat, d_e.as<u64>(), nullptr, nullptr, mq, st);
    (void)hipMemcpyAsync(pk_a, d_a.p, (size_t)L * N * 8, hipMemcpyDeviceToDevice, st);
    launch_to_mont(ctx, pk_a, L, mq, st);
    if (hipStreamSynchronize(st) != hipSuccess || hipGetLastError() != hipSuccess) {
        ctx->err = "kernel failure in keygen";
        return fail(ENSI_E_HIP);
    }
    *sk_out = sk;
    *pk_out = pk;
    return ENSI_OK;
}
extern "C" void ensi_sk_free(ensi_sk *sk) {
    if (!sk) return;
    if (sk->d_s_hat) (void)hipFree(sk->d_s_hat);
    delete sk;
}
extern "C" void ensi_pk_free(ensi_pk *pk) {
    if (!pk) return;
    if (pk->d_pk) (void)hipFree(pk->d_pk);
    delete pk;
}

// Scratch of the switching-key generation (one secret, any number of keys).
struct KeygenScratch {
    DevBuf d_s, d_target, d_e8, d_e, d_fac, d_s8;
};
static int keygen_scratch(ensi_ctx *ctx, const ensi_sk *sk, KeygenScratch &k, hipStream_t st) {
    const int N = ctx->N, ext = ctx->L + ctx->K;
    if (k.d_s.alloc((size_t)ext * N * 8) != hipSuccess || k.d_target.alloc((size_t)ext * N * 8) != hipSuccess || k.d_e8.alloc(N) != hipSuccess ||
        k.d_e.alloc((size_t)ext * N * 8) != hipSuccess || k.d_fac.alloc((size_t)ext * 8) != hipSuccess || k.d_s8.alloc(N) != hipSuccess)
        ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation failed in key generation");
    (void)hipMemcpy(k.d_s8.p, sk->s.data(), N, hipMemcpyHostToDevice);
    launch_small_to_rns(ctx, k.d_s8.as<int8_t>(), 1, make_map(ctx, ctx->L, true), k.d_s.as<u64>(), st);  // coefficient form of s
    return ENSI_OK;
}
// key <- hybrid key-switching key from the secret in k.d_target (transform domain, ordinary residues) to s:
// per digit j, (b_j, a_j) with b_j = -a_j s + e_j + [P]_{q_i} target on the limbs of digit j.  e: host
// int8[beta][N] or NULL; a_j is the uniform stream stream_base | j.
static int make_switch_key(ensi_ctx *ctx, const ensi_sk *sk, KeygenScratch &k, const int8_t *e, uint64_t seed_a, u64 stream_base, u64 *key,
                            hipStream_t st) {
    const int N = ctx->N, L = ctx->L, K = ctx->K, ext = L + K;
    const int beta = (L + ctx->alpha - 1) / ctx->alpha;
    LimbMap mext = make_map(ctx, L, true);
    std::vector<int8_t> ev(N);
    for (int j = 0; j < beta; j++) {
        u64 *kb = key + (size_t)(j * 2) * ext * N, *ka = kb + (size_t)ext * N;
        if (e) memcpy(ev.data(), e + (size_t)j * N, N);
        else if (sample_error(ctx, ev.data(), N)) return ENSI_E_BADARG;
        (void)hipMemcpyAsync(k.d_e8.p, ev.data(), N, hipMemcpyHostToDevice, st);
        (void)hipStreamSynchronize(st);
        launch_small_to_rns(ctx, k.d_e8.as<int8_t>(), 1, mext, k.d_e.as<u64>(), st);
        launch_ntt(ctx, k.d_e.as<u64>(), ext, mext, false, st);
        launch_uniform(ctx, ka, mext, seed_a, stream_base | (u64)j, st);
        launch_ntt(ctx, ka, ext, mext, false, st);
        std::vector<u64> fac(ext, 0);
        for (int i = j * ctx->alpha; i < std::min((j + 1) * ctx->alpha, L); i++) {
            const u64 q = ctx->primes[i];
            u64 P = 1;
            for (int b = 0; b < K; b++) P = hm_mulmod(P, ctx->primes[L + b] % q, q);
            fac[i] = hm_to_mont(P, q);
        }
        (void)hipMemcpyAsync(k.d_fac.p, fac.data(), ext * 8, hipMemcpyHostToDevice, st);
        (void)hipStreamSynchronize(st);
        launch_key_assemble(ctx, kb, ka, sk->d_s_hat, k.d_e.as<u64>(), k.d_target.as<u64>(), k.d_fac.as<u64>(), mext, st);
        launch_to_mont(ctx, ka, ext, mext, st);
    }
    if (ctx->ks16) launch_ks16_key_format(ctx, key, beta, st);
    return ENSI_OK;
}

extern "C" int ensi_galois_keygen(ensi_ctx *ctx, const ensi_sk *sk, const int32_t *steps, int32_t n_steps, const int8_t *e,
                                  uint64_t seed_a, ensi_gk **out) {
    if (!ctx || !sk || !out || (n_steps > 0 && !steps) || n_steps < 0) return ENSI_E_BADARG;
    const int N = ctx->N, L = ctx->L, K = ctx->K, ext = L + K;
    const int beta = (L + ctx->alpha - 1) / ctx->alpha;
    hipStream_t st = nullptr;
    LimbMap mext = make_map(ctx, L, true);
    ensi_gk *gk = new ensi_gk();
    gk->ctx = ctx;
    KeygenScratch k;
    int rc;
    if ((rc = keygen_scratch(ctx, sk, k, st))) {
        ensi_gk_free(gk);
        return rc;
    }
    for (int t = 0; t < n_steps; t++) {
        const u32 g = galois_element(ctx, steps[t]);
        if (gk->keys.count(g)) continue;
        u64 *key = nullptr;
        if (hipMalloc((void **)&key, (size_t)beta * 2 * ext * N * 8) != hipSuccess) {
            ensi_gk_free(gk);
            ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation of a Galois key failed");
        }
        gk->keys[g] = key;
        // phi_g(s), transform domain
        launch_automorphism_coef(ctx, k.d_target.as<u64>(), k.d_s.as<u64>(), mext, inv_mod_2n(g, N), st);
        launch_ntt(ctx, k.d_target.as<u64>(), ext, mext, false, st);
        if ((rc = make_switch_key(ctx, sk, k, e ? e + (size_t)t * beta * N : nullptr, seed_a, ((u64)2 << 56) | ((u64)g << 8), key, st))) {
            ensi_gk_free(gk);
            return rc;
        }
    }
    if (hipStreamSynchronize(st) != hipSuccess || hipGetLastError() != hipSuccess) {
        ensi_gk_free(gk);
        ENSI_FAIL(ctx, ENSI_E_HIP, "kernel failure in galois_keygen");
    }
    *out = gk;
    return ENSI_OK;
}

// Evaluation key of Mult: switches from s^2 to s.  Stored in a key set under the element 1 (the identity
// automorphism), which is how the key-switch kernels are driven for a relinearisation.
extern "C" int ensi_relin_keygen(ensi_ctx *ctx, const ensi_sk *sk, const int8_t *e, uint64_t seed_a, ensi_gk **out) {
    if (!ctx || !sk || !out) return ENSI_E_BADARG;
    const int N = ctx->N, L = ctx->L, K = ctx->K, ext = L + K;
    const int beta = (L + ctx->alpha - 1) / ctx->alpha;
    hipStream_t st = nullptr;
    LimbMap mext = make_map(ctx, L, true);
    ensi_gk *gk = new ensi_gk();
    gk->ctx = ctx;
    KeygenScratch k;
    int rc;
    if ((rc = keygen_scratch(ctx, sk, k, st))) {
        ensi_gk_free(gk);
        return rc;
    }
    u64 *key = nullptr;
    if (hipMalloc((void **)&key, (size_t)beta * 2 * ext * N * 8) != hipSuccess) {
        ensi_gk_free(gk);
        ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation of the evaluation key failed");
    }
    gk->keys[1u] = key;
    // s^2, transform domain: NTT(s) (.) NTT(s), the second factor in Montgomery form
    launch_ntt(ctx, k.d_s.as<u64>(), ext, mext, false, st);
    launch_mul_mont(ctx, k.d_target.as<u64>(), k.d_s.as<u64>(), sk->d_s_hat, ext, mext, st);
    if ((rc = make_switch_key(ctx, sk, k, e, seed_a, (u64)3 << 56, key, st))) {
        ensi_gk_free(gk);
        return rc;
    }
    if (hipStreamSynchronize(st) != hipSuccess || hipGetLastError() != hipSuccess) {
        ensi_gk_free(gk);
        ENSI_FAIL(ctx, ENSI_E_HIP, "kernel failure in relin_keygen");
    }
    *out = gk;
    return ENSI_OK;
}
extern "C" void ensi_gk_free(ensi_gk *gk) {
    if (!gk) return;
    for (auto &kv : gk->keys) (void)hipFree(kv.second);
    delete gk;
}


// ------------------------------------------------------------ import / export
// Key material crosses the boundary in coefficient form as canonical residues: the client generates keys, the
// server holds only the public ones (paper: System model; Preliminaries, KeyGen).  On the device keys live in the
// transform domain in the format the kernels read; these calls convert both ways with the library's own kernels.

// Host words -> a device buffer, checked to be canonical residues (row r modulo prime map.prime[r % map.n]).
static int upload_residues(ensi_ctx *ctx, u64 *dst, const uint64_t *words, int n_rows, const LimbMap &map, const char *what) {
    const size_t bytes = (size_t)n_rows * ctx->N * 8;
    DevBuf d_bad;
    if (d_bad.alloc(4) != hipSuccess) ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation failed in %s", what);
    ENSI_HIP(ctx, hipMemset(d_bad.p, 0, 4));
    ENSI_HIP(ctx, hipMemcpy(dst, words, bytes, hipMemcpyHostToDevice));
    launch_count_noncanonical(ctx, dst, n_rows, map, d_bad.as<unsigned int>(), nullptr);
    unsigned int bad = 0;
    ENSI_HIP(ctx, hipMemcpy(&bad, d_bad.p, 4, hipMemcpyDeviceToHost));
    if (bad) ENSI_FAIL(ctx, ENSI_E_BADARG, "%s: %u words are not residues below their prime", what, bad);
    return ENSI_OK;
}

extern "C" int ensi_sk_import(ensi_ctx *ctx, const int8_t *s, ensi_sk **sk) {
    if (!ctx || !s || !sk) return ENSI_E_BADARG;
    *sk = nullptr;
    std::vector<int8_t> sv(s, s + ctx->N);
    return make_sk(ctx, sv, sk);
}
extern "C" int ensi_sk_export(ensi_ctx *ctx, const ensi_sk *sk, int8_t *s) {
    if (!ctx || !sk || !s) return ENSI_E_BADARG;
    memcpy(s, sk->s.data(), ctx->N);
    return ENSI_OK;
}

extern "C" int ensi_pk_export(ensi_ctx *ctx, const ensi_pk *pk, uint64_t *words) {
    if (!ctx || !pk || !words) return ENSI_E_BADARG;
    const int N = ctx->N, L = ctx->L;
    const size_t bytes = (size_t)2 * L * N * 8;
    LimbMap mq = make_map(ctx, L, false);
    DevBuf d_t;
    if (d_t.alloc(bytes) != hipSuccess) ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation failed in pk_export");
    ENSI_HIP(ctx, hipDeviceSynchronize());
    ENSI_HIP(ctx, hipMemcpy(d_t.p, pk->d_pk, bytes, hipMemcpyDeviceToDevice));
    launch_key_to_plain(ctx, d_t.as<u64>(), 2 * L, mq, false, nullptr);
    launch_ntt(ctx, d_t.as<u64>(), 2 * L, mq, true, nullptr);
    ENSI_HIP(ctx, hipMemcpy(words, d_t.p, bytes, hipMemcpyDeviceToHost));
    return ENSI_OK;
}
extern "C" int ensi_pk_import(ensi_ctx *ctx, const uint64_t *words, ensi_pk **out) {
    if (!ctx || !words || !out) return ENSI_E_BADARG;
    *out = nullptr;
    const int N = ctx->N, L = ctx->L;
    LimbMap mq = make_map(ctx, L, false);
    ensi_pk *pk = new ensi_pk();
    pk->ctx = ctx;
    pk->d_pk = nullptr;
    if (hipMalloc((void **)&pk->d_pk, (size_t)2 * L * N * 8) != hipSuccess) {
        ensi_pk_free(pk);
        ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation failed in pk_import");
    }
    int rc = upload_residues(ctx, pk->d_pk, words, 2 * L, mq, "pk_import");
    if (rc) {
        ensi_pk_free(pk);
        return rc;
    }
    launch_ntt(ctx, pk->d_pk, 2 * L, mq, false, nullptr);
    launch_to_mont(ctx, pk->d_pk, 2 * L, mq, nullptr);
    if (hipStreamSynchronize(nullptr) != hipSuccess || hipGetLastError() != hipSuccess) {
        ensi_pk_free(pk);
        ENSI_FAIL(ctx, ENSI_E_HIP, "kernel failure in pk_import");
    }
    *out = pk;
    return ENSI_OK;
}

extern "C" int ensi_gk_elements(const ensi_gk *gk, int32_t *elements_out, int32_t cap) {
    if (!gk || cap < 0 || (cap > 0 && !elements_out)) return ENSI_E_BADARG;
    int n = 0;
    for (auto &kv : gk->keys) {
        if (n < cap) elements_out[n] = (int32_t)kv.first;
        n++;
    }
    return n;
}

extern "C" int ensi_gk_export(ensi_ctx *ctx, const ensi_gk *gk, int32_t step, uint64_t *words) {
    if (!ctx || !gk || !words) return ENSI_E_BADARG;
    const int N = ctx->N, ext = ctx->L + ctx->K, beta = (ctx->L + ctx->alpha - 1) / ctx->alpha;
    auto it = gk->keys.find(galois_element(ctx, step));
    if (it == gk->keys.end()) ENSI_FAIL(ctx, ENSI_E_NOKEY, "gk_export: the key set holds no key for step %d", step);
    const size_t bytes = (size_t)beta * 2 * ext * N * 8;
    LimbMap mext = make_map(ctx, ctx->L, true);
    DevBuf d_t;
    if (d_t.alloc(bytes) != hipSuccess) ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation failed in gk_export");
    ENSI_HIP(ctx, hipDeviceSynchronize());
    ENSI_HIP(ctx, hipMemcpy(d_t.p, it->second, bytes, hipMemcpyDeviceToDevice));
    launch_key_to_plain(ctx, d_t.as<u64>(), beta * 2 * ext, mext, ctx->ks16, nullptr);
    launch_ntt(ctx, d_t.as<u64>(), beta * 2 * ext, mext, true, nullptr);
    ENSI_HIP(ctx, hipMemcpy(words, d_t.p, bytes, hipMemcpyDeviceToHost));
    return ENSI_OK;
}

extern "C" int ensi_gk_import(ensi_ctx *ctx, ensi_gk **gk_io, int32_t step, const uint64_t *words) {
    if (!ctx || !gk_io || !words) return ENSI_E_BADARG;
    const int N = ctx->N, ext = ctx->L + ctx->K, beta = (ctx->L + ctx->alpha - 1) / ctx->alpha;
    if (*gk_io && (*gk_io)->ctx != ctx) ENSI_FAIL(ctx, ENSI_E_BADARG, "gk_import: the key set belongs to another context");
    const u32 g = galois_element(ctx, step);
    LimbMap mext = make_map(ctx, ctx->L, true);
    u64 *key = nullptr;
    if (hipMalloc((void **)&key, (size_t)beta * 2 * ext * N * 8) != hipSuccess) ENSI_FAIL(ctx, ENSI_E_NOMEM, "device allocation of a key failed");
    int rc = upload_residues(ctx, key, words, beta * 2 * ext, mext, "gk_import");
    if (rc) {
        (void)hipFree(key);
        return rc;
    }
    launch_ntt(ctx, key, beta * 2 * ext, mext, false, nullptr);
    launch_to_mont(ctx, key, beta * 2 * ext, mext, nullptr);
    if (ctx->ks16) launch_ks16_key_format(ctx, key, beta, nullptr);
    if (hipStreamSynchronize(nullptr) != hipSuccess || hipGetLastError() != hipSuccess) {
        (void)hipFree(key);
        ENSI_FAIL(ctx, ENSI_E_HIP, "kernel failure in gk_import");
    }
    ensi_gk *gk = *gk_io;
    if (!gk) {
        gk = new ensi_gk();
        gk->ctx = ctx;
        *gk_io = gk;
    }
    auto it = gk->keys.find(g);
    if (it != gk->keys.end()) {
        (void)hipDeviceSynchronize();  // a replaced key may still be read by work in flight
        (void)hipFree(it->second);
    }
    gk->keys[g] = key;
    return ENSI_OK;
}
