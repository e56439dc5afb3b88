// Host-side exact modular helpers (context set-up only; never on the hot path).
#pragma once
#include <stdint.h>

#include "modarith.h"

static inline u64 hm_mulmod(u64 a, u64 b, u64 q) { return (u64)(((u128)a * b) % q); }
static inline u64 hm_powmod(u64 a, u64 e, u64 q) {
    u64 r = 1 % q;
    a %= q;
    while (e) {
        if (e & 1) r = hm_mulmod(r, a, q);
        a = hm_mulmod(a, a, q);
        e >>= 1;
    }
    return r;
}
// q prime
static inline u64 hm_invmod(u64 a, u64 q) { return hm_powmod(a, q - 2, q); }
// floor(w * 2^64 / q), w < q
static inline u64 hm_shoup(u64 w, u64 q) { return (u64)((((u128)w) << 64) / q); }
// w * 2^64 mod q
static inline u64 hm_to_mont(u64 w, u64 q) { return (u64)((((u128)w) << 64) % q); }
// -q^{-1} mod 2^64, q odd (Newton iteration)
static inline u64 hm_neg_inv64(u64 q) {
    u64 x = q;  // correct to 3 bits
    for (int i = 0; i < 6; i++) x *= 2 - q * x;
    return (u64)0 - x;
}
static inline bool hm_is_prime(u64 n) {
    if (n < 2) return false;
    static const u64 bases[] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
    for (u64 b : bases) {
        if (n % b == 0) return n == b;
    }
    u64 d = n - 1;
    int r = 0;
    while ((d & 1) == 0) {
        d >>= 1;
        r++;
    }
    for (u64 b : bases) {
        u64 y = hm_powmod(b, d, n);
        if (y == 1 || y == n - 1) continue;
        bool comp = true;
        for (int i = 1; i < r; i++) {
            y = hm_mulmod(y, y, n);
            if (y == n - 1) {
                comp = false;
                break;
            }
        }
        if (comp) return false;
    }
    return true;
}
