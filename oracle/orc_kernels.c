/*
 * CPU oracle for the encrypted ternary matmul path -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct integer routines over Z_q[X]/(X^N+1) with
 * q < 2^62 held in 64-bit words.  Every modular product is the definition
 * itself: a 128-bit product followed by the C remainder operator.  No
 * Montgomery, Barrett or Shoup forms, no blocking, no fusion.  Nothing in the
 * GPU library includes, links or calls this file; only the tests, the smoke
 * check and the benchmark's cpu_baseline leg do.
 *
 * The ring and its RNS representation are those of the paper's Preliminaries
 * (RNS-CKKS: R_Q = Z_Q[X]/(X^N'+1), Q a product of distinct primes).  The
 * paper calls library routines for everything below the Rot/Add primitives, so
 * the number-theoretic transform, the basis conversions and the key-switching
 * steps here follow the standard published definitions (Cheon et al. full-RNS
 * CKKS; Han-Ki hybrid key switching), each pinned by tests against big-integer
 * arithmetic and the schoolbook negacyclic product.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef unsigned __int128 u128;
typedef __int128 i128;

static inline uint64_t mulmod(uint64_t a, uint64_t b, uint64_t q) {
    return (uint64_t)(((u128)a * b) % q);
}
static inline uint64_t addmod(uint64_t a, uint64_t b, uint64_t q) {
    uint64_t s = a + b; /* a,b < q < 2^62: no wrap */
    return s >= q ? s - q : s;
}
static inline uint64_t submod(uint64_t a, uint64_t b, uint64_t q) {
    return a >= b ? a - b : a + q - b;
}

uint64_t orc_powmod(uint64_t a, uint64_t e, uint64_t q) {
    uint64_t r = 1 % q;
    a %= q;
    while (e) {
        if (e & 1) r = mulmod(r, a, q);
        a = mulmod(a, a, q);
        e >>= 1;
    }
    return r;
}

static uint32_t bitrev(uint32_t x, int bits) {
    uint32_t r = 0;
    for (int i = 0; i < bits; i++) r |= ((x >> i) & 1u) << (bits - 1 - i);
    return r;
}

/* Cyclic length-N DFT over Z_q with root w (w^N = 1), natural order in and out:
 * textbook iterative radix-2 decimation in time. */
static void cyclic_dft(uint64_t *a, int log_n, uint64_t q, uint64_t w) {
    const uint32_t n = 1u << log_n;
    for (uint32_t i = 0; i < n; i++) {
        uint32_t j = bitrev(i, log_n);
        if (i < j) { uint64_t t = a[i]; a[i] = a[j]; a[j] = t; }
    }
    uint64_t *wp = (uint64_t *)malloc(sizeof(uint64_t) * (n / 2 + 1));
    wp[0] = 1;
    for (uint32_t i = 1; i < n / 2 + 1; i++) wp[i] = mulmod(wp[i - 1], w, q);
    for (uint32_t len = 2; len <= n; len <<= 1) {
        uint32_t half = len / 2, step = n / len;
        for (uint32_t base = 0; base < n; base += len)
            for (uint32_t k = 0; k < half; k++) {
                uint64_t u = a[base + k];
                uint64_t v = mulmod(a[base + k + half], wp[k * step], q);
                a[base + k] = addmod(u, v, q);
                a[base + k + half] = submod(u, v, q);
            }
    }
    free(wp);
}

/* Negacyclic transform of one limb: out[k] = sum_i a[i] * psi^{(2k+1) i} mod q,
 * natural order.  psi is a primitive 2N-th root of unity mod q.  Computed as the
 * cyclic DFT (root psi^2) of the twisted sequence a[i]*psi^i. */
static void ntt_limb(uint64_t *a, int log_n, uint64_t q, uint64_t psi) {
    const uint32_t n = 1u << log_n;
    uint64_t p = 1;
    for (uint32_t i = 0; i < n; i++) { a[i] = mulmod(a[i], p, q); p = mulmod(p, psi, q); }
    cyclic_dft(a, log_n, q, mulmod(psi, psi, q));
}

/* Inverse of ntt_limb. */
static void intt_limb(uint64_t *a, int log_n, uint64_t q, uint64_t psi) {
    const uint32_t n = 1u << log_n;
    uint64_t psi_inv = orc_powmod(psi, q - 2, q);
    uint64_t n_inv = orc_powmod(n % q, q - 2, q);
    cyclic_dft(a, log_n, q, mulmod(psi_inv, psi_inv, q));
    uint64_t p = n_inv;
    for (uint32_t i = 0; i < n; i++) { a[i] = mulmod(a[i], p, q); p = mulmod(p, psi_inv, q); }
}

/* a: [n_limbs][N]; limb l uses prime q[l] and root psi[l]. */
void orc_ntt(uint64_t *a, int n_limbs, int log_n, const uint64_t *q, const uint64_t *psi, int inverse) {
    const size_t n = (size_t)1 << log_n;
#pragma omp parallel for schedule(dynamic)
    for (int l = 0; l < n_limbs; l++) {
        if (inverse) intt_limb(a + l * n, log_n, q[l], psi[l]);
        else ntt_limb(a + l * n, log_n, q[l], psi[l]);
    }
}

/* Schoolbook product in Z_q[X]/(X^N+1): c = a*b with X^N = -1. */
void orc_negacyclic_naive(uint64_t *c, const uint64_t *a, const uint64_t *b, int n, uint64_t q) {
    memset(c, 0, sizeof(uint64_t) * n);
    for (int i = 0; i < n; i++)
        for (int j = 0; j < n; j++) {
            uint64_t t = mulmod(a[i], b[j], q);
            int k = i + j;
            if (k < n) c[k] = addmod(c[k], t, q);
            else c[k - n] = submod(c[k - n], t, q);
        }
}

/* limb-wise c = a (.) b, [n_limbs][N] */
void orc_pointwise_mul(uint64_t *c, const uint64_t *a, const uint64_t *b, int n_limbs, int n, const uint64_t *q) {
#pragma omp parallel for
    for (int l = 0; l < n_limbs; l++)
        for (int i = 0; i < n; i++) {
            size_t o = (size_t)l * n + i;
            c[o] = mulmod(a[o], b[o], q[l]);
        }
}
/* acc += a (.) b */
void orc_pointwise_mac(uint64_t *acc, const uint64_t *a, const uint64_t *b, int n_limbs, int n, const uint64_t *q) {
#pragma omp parallel for
    for (int l = 0; l < n_limbs; l++)
        for (int i = 0; i < n; i++) {
            size_t o = (size_t)l * n + i;
            acc[o] = addmod(acc[o], mulmod(a[o], b[o], q[l]), q[l]);
        }
}
void orc_add(uint64_t *c, const uint64_t *a, const uint64_t *b, int n_limbs, int n, const uint64_t *q) {
#pragma omp parallel for
    for (int l = 0; l < n_limbs; l++)
        for (int i = 0; i < n; i++) {
            size_t o = (size_t)l * n + i;
            c[o] = addmod(a[o], b[o], q[l]);
        }
}
void orc_sub(uint64_t *c, const uint64_t *a, const uint64_t *b, int n_limbs, int n, const uint64_t *q) {
#pragma omp parallel for
    for (int l = 0; l < n_limbs; l++)
        for (int i = 0; i < n; i++) {
            size_t o = (size_t)l * n + i;
            c[o] = submod(a[o], b[o], q[l]);
        }
}
/* c = a * scalar[l] per limb */
void orc_mul_scalar(uint64_t *c, const uint64_t *a, const uint64_t *scalar, int n_limbs, int n, const uint64_t *q) {
#pragma omp parallel for
    for (int l = 0; l < n_limbs; l++)
        for (int i = 0; i < n; i++) {
            size_t o = (size_t)l * n + i;
            c[o] = mulmod(a[o], scalar[l], q[l]);
        }
}

/* Galois automorphism a(X) -> a(X^g) in coefficient form (g odd): coefficient i
 * moves to position i*g mod 2N; positions >= N wrap with a sign flip since
 * X^N = -1.  This is the ring map under which slot vectors rotate (the paper's
 * Rot, Preliminaries) when g = 5^k. */
void orc_automorphism(uint64_t *out, const uint64_t *in, int n_limbs, int n, uint64_t g, const uint64_t *q) {
#pragma omp parallel for
    for (int l = 0; l < n_limbs; l++)
        for (int i = 0; i < n; i++) {
            uint64_t j = ((uint64_t)i * g) % (2 * (uint64_t)n);
            uint64_t v = in[(size_t)l * n + i];
            if (j < (uint64_t)n) out[(size_t)l * n + j] = v;
            else out[(size_t)l * n + (j - n)] = v ? q[l] - v : 0;
        }
}

/* Fast basis conversion.  Source limbs in[a][.] mod qs[a], a < A.  For every target
 * modulus t[k]:
 *   out[k][i] = sum_a  y_a * hat_mod_t[k][a]   mod t[k],   y_a = in[a][i] * inv[a] mod qs[a]
 * where inv[a] = (Qs/qs[a])^{-1} mod qs[a], hat_mod_t[k][a] = (Qs/qs[a]) mod t[k].
 * centered = 0: y_a is taken in [0, qs[a])            (the sum is x + u*Qs, 0 <= u < A);
 * centered = 1: y_a is taken in (-qs[a]/2, qs[a]/2]   (the sum is x + u*Qs, |u| <= A/2, zero mean).
 * No floating-point correction of u in either case. */
void orc_bconv(uint64_t *out, const uint64_t *in, int A, int T, int n, const uint64_t *qs, const uint64_t *inv,
               const uint64_t *hat_mod_t, const uint64_t *t, int centered) {
#pragma omp parallel for
    for (int k = 0; k < T; k++)
        for (int i = 0; i < n; i++) {
            uint64_t acc = 0;
            for (int a = 0; a < A; a++) {
                uint64_t y = mulmod(in[(size_t)a * n + i], inv[a], qs[a]);
                uint64_t h = hat_mod_t[(size_t)k * A + a];
                if (centered && y > qs[a] / 2)
                    acc = submod(acc, mulmod(qs[a] - y, h, t[k]), t[k]); /* y - qs[a] is negative */
                else
                    acc = addmod(acc, mulmod(y, h, t[k]), t[k]);
            }
            out[(size_t)k * n + i] = acc;
        }
}

/* Small signed coefficients (ternary secrets, rounded-Gaussian errors) to RNS. */
void orc_small_to_rns(uint64_t *out, const int8_t *in, int n_limbs, int n, const uint64_t *q) {
    for (int l = 0; l < n_limbs; l++)
        for (int i = 0; i < n; i++) {
            int v = in[i];
            out[(size_t)l * n + i] = v >= 0 ? (uint64_t)v : q[l] - (uint64_t)(-v);
        }
}
/* Signed 64-bit coefficients (encoded plaintexts) to RNS. */
void orc_i64_to_rns(uint64_t *out, const int64_t *in, int n_limbs, int n, const uint64_t *q) {
    for (int l = 0; l < n_limbs; l++)
        for (int i = 0; i < n; i++) {
            int64_t v = in[i];
            uint64_t m = (uint64_t)(v >= 0 ? v : -v) % q[l];
            out[(size_t)l * n + i] = (v >= 0 || m == 0) ? m : q[l] - m;
        }
}

/* Counter-based uniform generator shared BY SPECIFICATION (not by code) with the
 * GPU library.  A sample is two consecutive outputs of SplitMix64 (Steele, Lea,
 * Flood, "Fast splittable pseudorandom number generators", 2014) read as one
 * 128-bit number and reduced mod q; the generator's starting state is a key
 * derived from (seed, stream, prime index) with the same finaliser:
 *   mix(z): z^=z>>30; z*=0xBF58476D1CE4E5B9; z^=z>>27; z*=0x94D049BB133111EB; z^=z>>31
 *   SplitMix64: state += G; output = mix(state),   G = 0x9E3779B97F4A7C15
 *   key = mix(mix(mix(seed) + stream) + prime_id)
 *   sample_i = (output_{2i+1}*2^64 + output_{2i+2}) mod q   of the generator started at key
 * The key derivation and the two-words-per-sample layout are this build's own
 * format; the generator is the published one (orc_splitmix64 is pinned to its
 * published output vectors). */
static inline uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27; z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}
static inline uint64_t splitmix64_next(uint64_t *state) {
    *state += 0x9E3779B97F4A7C15ULL;
    return mix64(*state);
}
/* The first n outputs of SplitMix64 started at `state`. */
void orc_splitmix64(uint64_t *out, int n, uint64_t state) {
    for (int i = 0; i < n; i++) out[i] = splitmix64_next(&state);
}
void orc_uniform(uint64_t *out, int n, uint64_t seed, uint64_t stream, uint64_t prime_id, uint64_t q) {
    uint64_t state = mix64(mix64(mix64(seed) + stream) + prime_id);
    for (int i = 0; i < n; i++) {
        uint64_t hi = splitmix64_next(&state);
        uint64_t lo = splitmix64_next(&state);
        out[i] = (uint64_t)((((u128)hi << 64) | lo) % q);
    }
}

/* CRT-combine two residues and centre: value in (-q0*q1/2, q0*q1/2], as double.
 * Garner: v = r0 + q0 * ((r1 - r0) * q0^{-1} mod q1). */
void orc_crt2_center(double *out, const uint64_t *r0, const uint64_t *r1, uint64_t q0, uint64_t q1, int n) {
    uint64_t q0_inv = orc_powmod(q0 % q1, q1 - 2, q1);
    u128 big = (u128)q0 * q1;
    for (int i = 0; i < n; i++) {
        uint64_t d = submod(r1[i] % q1, r0[i] % q1, q1);
        uint64_t t = mulmod(d, q0_inv, q1);
        u128 v = (u128)r0[i] + (u128)q0 * t;
        if (v > big / 2) out[i] = -(double)(big - v);
        else out[i] = (double)v;
    }
}
void orc_center1(double *out, const uint64_t *r0, uint64_t q0, int n) {
    for (int i = 0; i < n; i++) out[i] = r0[i] > q0 / 2 ? -(double)(q0 - r0[i]) : (double)r0[i];
}

/* Alg. 1 (PCMM) inner loop for one output ciphertext, over a flat array of limb
 * words: y starts at zero; for every listed term, y = y (+) x or y (-) x
 * limb-wise mod q.  srcs[k] points at the k-th term's [n_limbs][N] words. */
void orc_signed_accumulate(uint64_t *y, const uint64_t *const *srcs, const int8_t *signs, int n_terms, int n_limbs,
                           int n, const uint64_t *q) {
#pragma omp parallel for
    for (int l = 0; l < n_limbs; l++) {
        uint64_t *yl = y + (size_t)l * n;
        for (int i = 0; i < n; i++) yl[i] = 0;
        for (int k = 0; k < n_terms; k++) {
            const uint64_t *x = srcs[k] + (size_t)l * n;
            if (signs[k] > 0) for (int i = 0; i < n; i++) yl[i] = addmod(yl[i], x[i], q[l]);
            else if (signs[k] < 0) for (int i = 0; i < n; i++) yl[i] = submod(yl[i], x[i], q[l]);
        }
    }
}
