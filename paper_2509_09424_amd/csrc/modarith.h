// Modular arithmetic on 64-bit words for primes q < 2^62.
//
// Three product forms are used by the kernels:
//   * Shoup products for multiplications by precomputed constants (twiddles,
//     basis-conversion inverses): w' = floor(w * 2^64 / q) is stored beside w and
//     x*w mod q costs one high product and two low products, result in [0, 2q);
//   * Montgomery reduction of 128-bit accumulators (key inner product, basis
//     conversion sums): constants are stored as c*2^64 mod q so that the reduced
//     sum comes out in ordinary form;
//   * plain add/sub with one conditional correction.
// All results that leave a kernel are canonical residues in [0, q).
#pragma once
#include <stdint.h>

typedef uint64_t u64;
typedef uint32_t u32;
typedef unsigned __int128 u128;

#define ENSI_HD __host__ __device__ __forceinline__

ENSI_HD u64 mulhi64(u64 a, u64 b) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __umul64hi(a, b);
#else
    return (u64)(((u128)a * b) >> 64);
#endif
}

ENSI_HD u64 add_mod(u64 a, u64 b, u64 q) {
    u64 s = a + b;
    return s >= q ? s - q : s;
}
ENSI_HD u64 sub_mod(u64 a, u64 b, u64 q) { return a >= b ? a - b : a + q - b; }
ENSI_HD u64 neg_mod(u64 a, u64 q) { return a ? q - a : 0; }
ENSI_HD u64 csub(u64 a, u64 q) { return a >= q ? a - q : a; }

// x * w mod q in [0, 2q) for any 64-bit x; ws = floor(w * 2^64 / q), w < q.
ENSI_HD u64 mul_shoup_lazy(u64 x, u64 w, u64 ws, u64 q) {
    u64 t = mulhi64(x, ws);
    return x * w - t * q;
}
ENSI_HD u64 mul_shoup(u64 x, u64 w, u64 ws, u64 q) { return csub(mul_shoup_lazy(x, w, ws, q), q); }

// 128-bit accumulator
struct acc128 {
    u64 lo, hi;
};
ENSI_HD void mac128(acc128 &a, u64 x, u64 y) {
    u64 lo = x * y;
    u64 hi = mulhi64(x, y);
    a.lo += lo;
    a.hi += hi + (a.lo < lo ? 1 : 0);
}
// T * 2^-64 mod q, canonical, for T < q * 2^64;  qneg_inv = -q^{-1} mod 2^64.
ENSI_HD u64 mont_reduce(acc128 a, u64 q, u64 qneg_inv) {
    u64 m = a.lo * qneg_inv;
    u64 t = a.hi + mulhi64(m, q) + (a.lo != 0 ? 1 : 0);
    return csub(t, q);
}
// a * b * 2^-64 mod q
ENSI_HD u64 mont_mul(u64 a, u64 b, u64 q, u64 qneg_inv) {
    acc128 t = {0, 0};
    mac128(t, a, b);
    return mont_reduce(t, q, qneg_inv);
}
