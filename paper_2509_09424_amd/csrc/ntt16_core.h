// Arithmetic and register-level building blocks of the N = 2^16 transform, shared by the
// plain transform kernels and the fused key-switching kernels.
//
// A limb is viewed as 256 x 256 (row-major).  The 16 stages of the Cooley-Tukey network
// (Gentleman-Sande for the inverse) are cut 4 + 4 | 4 + 4: the column pass covers the
// stages whose butterflies span rows, the row pass those inside a row, and each pass is
// two radix-16 steps held in registers with one exchange through LDS in between.
//
// Two arithmetic back ends with the same interface:
//   ArithFp   primes below 2^50: residues are exact integers held in doubles; a product
//             x*w mod p is  h = x*w; l = fma(x,w,-h); q = rint(x*(w/p)); r = fma(-q,p,h)+l
//             (exact: h - q*p and l are integers below 2^53).  Values stay within +-8p and
//             are brought back to |x| <= p/2 with x - rint(x/p)*p between steps.
//   ArithInt  wider primes: 64-bit Shoup/Harvey lazy butterflies.
#pragma once
#include "common.h"

struct ArithInt {
    typedef u64 T;
    u64 q, two_q, ninv, ninv_s;
    __device__ __forceinline__ void init(const PrimeConst &pc) {
        q = pc.q;
        two_q = 2 * pc.q;
        ninv = pc.n_inv;
        ninv_s = pc.n_inv_s;
    }
    __device__ __forceinline__ T load(u64 x) const { return x; }
    __device__ __forceinline__ T center(T x) const { return x; }
    __device__ __forceinline__ void ct(T &x, T &y, u64 w, u64 ws) const {  // in/out [0,4q)
        const T xs = csub(x, two_q);
        const T t = mul_shoup_lazy(y, w, ws, q);
        x = xs + t;
        y = xs - t + two_q;
    }
    __device__ __forceinline__ void gs(T &u, T &v, u64 w, u64 ws) const {  // in/out [0,2q)
        const T s = csub(u + v, two_q);
        v = mul_shoup_lazy(u - v + two_q, w, ws, q);
        u = s;
    }
    __device__ __forceinline__ T mid(T x) const { return x; }
    __device__ __forceinline__ u64 store_fwd(T x) const { return csub(csub(x, two_q), q); }
    __device__ __forceinline__ u64 store_inv(T x) const { return csub(x, q); }
    __device__ __forceinline__ u64 store_inv_scaled(T x) const { return mul_shoup(x, ninv, ninv_s, q); }
    // workspace word after a forward pass: the canonical residue
    __device__ __forceinline__ u64 store_ws_fwd(T x) const { return store_fwd(x); }
};

struct ArithFp {
    typedef double T;
    double p, pinv, ninv, ninv_p;
    __device__ __forceinline__ void init(const PrimeConst &pc) {
        p = (double)pc.q;
        pinv = __longlong_as_double((long long)pc.pad[1]);
        ninv = (double)pc.n_inv;
        ninv_p = __longlong_as_double((long long)pc.pad[2]);
    }
    __device__ __forceinline__ T load(u64 x) const { return (double)x; }
    __device__ __forceinline__ T mid(T x) const { return fma(-rint(x * pinv), p, x); }  // -> |x| <= p/2
    __device__ __forceinline__ T center(T x) const { return mid(x); }
    __device__ __forceinline__ T mulmod(T y, T w, T wp) const {  // |y| < 2^53 -> |result| < 2.5p, exact integer
        const double h = y * w;
        const double l = fma(y, w, -h);
        const double q = rint(y * wp);
        return fma(-q, p, h) + l;
    }
    // x*k mod p for a multiplier without a precomputed k/p: |x| <= p/2, 0 <= k < p -> |result| < 0.7p, exact integer
    __device__ __forceinline__ T mulmod_np(T x, T k) const {
        const double h = x * k;
        const double l = fma(x, k, -h);
        const double q = rint(h * pinv);
        return fma(-q, p, h) + l;
    }
    __device__ __forceinline__ void ct(T &x, T &y, u64 w, u64 ws) const {
        const T t = mulmod(y, __longlong_as_double((long long)w), __longlong_as_double((long long)ws));
        y = x - t;
        x = x + t;
    }
    __device__ __forceinline__ void gs(T &u, T &v, u64 w, u64 ws) const {
        const T s = u + v;
        v = mulmod(u - v, __longlong_as_double((long long)w), __longlong_as_double((long long)ws));
        u = s;
    }
    __device__ __forceinline__ u64 canon(T x) const {
        T r = mid(x);
        r = r < 0.0 ? r + p : r;
        return (u64)r;
    }
    __device__ __forceinline__ u64 store_fwd(T x) const { return canon(x); }
    __device__ __forceinline__ u64 store_inv(T x) const { return canon(x); }
    __device__ __forceinline__ u64 store_inv_scaled(T x) const { return canon(mulmod(mid(x), ninv, ninv_p)); }
    // workspace word after a forward pass: the bits of the double, |x| <= p/2
    __device__ __forceinline__ u64 store_ws_fwd(T x) const { return (u64)__double_as_longlong(mid(x)); }
};

// Four Cooley-Tukey stages on 16 elements whose local index i is the 4 index bits of the step
// (bit 3 = largest distance).  tw/tws: the prime's forward table and its companion.
template <class A>
__device__ __forceinline__ void ct4(const A &ar, typename A::T *v, const u64 *tw, const u64 *tws, u32 mbase) {
#pragma unroll
    for (int k = 0; k < 4; k++) {
        const int d = 8 >> k;
#pragma unroll
        for (int g = 0; g < (1 << k); g++) {
            const u64 w = tw[(mbase << k) + g], ws = tws[(mbase << k) + g];
#pragma unroll
            for (int o = 0; o < d; o++) {
                const int i0 = g * 2 * d + o;
                ar.ct(v[i0], v[i0 + d], w, ws);
            }
        }
    }
}
// ct4 with the step's 15 twiddles (value, companion) already at hand: entry (1 << k) - 1 + g serves local stage k,
// butterfly group g.  TAB is anything indexable that yields .x (value) and .y (companion) as 64-bit words -- a table
// in LDS shared by the threads of a row, or a per-thread array in registers -- so that a kernel that runs the same
// step on several limbs in a row fetches the twiddles once.
template <class A, class TAB>
__device__ __forceinline__ void ct4_tab(const A &ar, typename A::T *v, const TAB &tab) {
#pragma unroll
    for (int k = 0; k < 4; k++) {
        const int d = 8 >> k;
#pragma unroll
        for (int g = 0; g < (1 << k); g++) {
            const u64 w = tab[(1 << k) - 1 + g].x, ws = tab[(1 << k) - 1 + g].y;
#pragma unroll
            for (int o = 0; o < d; o++) {
                const int i0 = g * 2 * d + o;
                ar.ct(v[i0], v[i0 + d], w, ws);
            }
        }
    }
}
// The 15 twiddles of a step with base index mbase, in ct4_tab's order.
struct TwRegs {
    ulonglong2 t[15];
    __device__ __forceinline__ const ulonglong2 &operator[](int i) const { return t[i]; }
    __device__ __forceinline__ void load(const u64 *tw, const u64 *tws, u32 mbase) {
#pragma unroll
        for (int k = 0; k < 4; k++)
#pragma unroll
            for (int g = 0; g < (1 << k); g++) t[(1 << k) - 1 + g] = make_ulonglong2(tw[(mbase << k) + g], tws[(mbase << k) + g]);
    }
};

// The inverse of ct4 up to the factor 16 (inverse table).
template <class A>
__device__ __forceinline__ void gs4(const A &ar, typename A::T *v, const u64 *tw, const u64 *tws, u32 mbase) {
#pragma unroll
    for (int k = 3; k >= 0; k--) {
        const int d = 8 >> k;
#pragma unroll
        for (int g = 0; g < (1 << k); g++) {
            const u64 w = tw[(mbase << k) + g], ws = tws[(mbase << k) + g];
#pragma unroll
            for (int o = 0; o < d; o++) {
                const int i0 = g * 2 * d + o;
                ar.gs(v[i0], v[i0 + d], w, ws);
            }
        }
    }
}
// gs4 with the step's twiddles at hand (see ct4_tab).
template <class A, class TAB>
__device__ __forceinline__ void gs4_tab(const A &ar, typename A::T *v, const TAB &tab) {
#pragma unroll
    for (int k = 3; k >= 0; k--) {
        const int d = 8 >> k;
#pragma unroll
        for (int g = 0; g < (1 << k); g++) {
            const u64 w = tab[(1 << k) - 1 + g].x, ws = tab[(1 << k) - 1 + g].y;
#pragma unroll
            for (int o = 0; o < d; o++) {
                const int i0 = g * 2 * d + o;
                ar.gs(v[i0], v[i0 + d], w, ws);
            }
        }
    }
}
// Thread (rho = tid / 16, j) of a 256-thread block puts entry j < 15 of row rho's step table (base index mbase_row,
// which depends on the row only) into tab[rho * 16 + j]; the caller synchronises before the first use.
__device__ __forceinline__ void row_table_to_lds(ulonglong2 *tab, const u64 *tw, const u64 *tws, u32 mbase_row, int rho, int j) {
    if (j < 15) {
        const int k = 31 - __clz(j + 1), g = j + 1 - (1 << k);
        const u32 idx = (mbase_row << k) + g;
        tab[rho * 16 + j] = make_ulonglong2(tw[idx], tws[idx]);
    }
}

// ---- pass bodies on registers ------------------------------------------------------
// Column pass, thread (c = tid % 16, jj = tid / 16) of a 256-thread block working on 16
// adjacent columns; lds holds 4096 words.
//   forward: on entry v[i] = row jj + 16 i of the thread's column, on exit v[i] = row 16 jj + i.
//   inverse: on entry v[i] = row 16 jj + i (|v| <= p/2 for ArithFp, [0,2q) for ArithInt), on exit
//            v[i] = row jj + 16 i, not yet multiplied by 1/N.
// Neither synchronises after its last LDS read: the caller must, before the tile is reused.
template <class A>
__device__ __forceinline__ void cols_fwd_regs(const A &ar, typename A::T *v, const u64 *tw, const u64 *tws, void *lds, int c, int jj) {
    typename A::T *l = (typename A::T *)lds;
    ct4(ar, v, tw, tws, 1u);
#pragma unroll
    for (int i = 0; i < 16; i++) l[(jj + 16 * i) * 16 + c] = ar.mid(v[i]);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; i++) v[i] = l[(16 * jj + i) * 16 + c];
    ct4(ar, v, tw, tws, 16u + jj);
}
template <class A>
__device__ __forceinline__ void cols_inv_regs(const A &ar, typename A::T *v, const u64 *tw, const u64 *tws, void *lds, int c, int jj) {
    typename A::T *l = (typename A::T *)lds;
    gs4(ar, v, tw, tws, 16u + jj);
#pragma unroll
    for (int i = 0; i < 16; i++) l[(16 * jj + i) * 16 + c] = ar.mid(v[i]);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; i++) v[i] = l[(jj + 16 * i) * 16 + c];
    gs4(ar, v, tw, tws, 1u);
}

// The same two passes with their twiddles in LDS.  A column tile uses 15 pairs that are the same for every thread
// (first forward step, base index 1) and 15 pairs per thread row jj (base index 16 + jj); read straight from the
// table in memory they are 60 loads per thread for 16 values.  col_tables_to_lds puts them into tab (COL_TAB_PAIRS
// entries: slot 0 = base 1, slot 1 + jj = base 16 + jj, 16 entries per slot of which 15 are used); the caller
// synchronises between the fill and the first use.
#define COL_TAB_PAIRS (17 * 16)
__device__ __forceinline__ void col_tables_to_lds(ulonglong2 *tab, const u64 *tw, const u64 *tws, int tid) {
    for (int t = tid; t < COL_TAB_PAIRS; t += 256) {
        const int slot = t >> 4, ent = t & 15;
        if (ent < 15) {
            const int k = 31 - __clz(ent + 1), g = ent + 1 - (1 << k);
            const u32 mbase = slot == 0 ? 1u : 16u + (u32)(slot - 1);
            const u32 idx = (mbase << k) + g;
            tab[t] = make_ulonglong2(tw[idx], tws[idx]);
        }
    }
}
template <class A>
__device__ __forceinline__ void cols_fwd_regs_t(const A &ar, typename A::T *v, const ulonglong2 *tab, void *lds, int c, int jj) {
    typename A::T *l = (typename A::T *)lds;
    ct4_tab(ar, v, tab);
#pragma unroll
    for (int i = 0; i < 16; i++) l[(jj + 16 * i) * 16 + c] = ar.mid(v[i]);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; i++) v[i] = l[(16 * jj + i) * 16 + c];
    ct4_tab(ar, v, tab + 16 * (1 + jj));
}
template <class A>
__device__ __forceinline__ void cols_inv_regs_t(const A &ar, typename A::T *v, const ulonglong2 *tab, void *lds, int c, int jj) {
    typename A::T *l = (typename A::T *)lds;
    gs4_tab(ar, v, tab + 16 * (1 + jj));
#pragma unroll
    for (int i = 0; i < 16; i++) l[(16 * jj + i) * 16 + c] = ar.mid(v[i]);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; i++) v[i] = l[(jj + 16 * i) * 16 + c];
    gs4_tab(ar, v, tab);
}

// Row pass, thread (rho = tid / 16, j = tid % 16) of a 256-thread block working on 16 whole
// rows r0 .. r0+15 (r = r0 + rho); lds holds 4096 + 256 words (one pad word per 16).
//   forward: on entry v[i] = element j + 16 i of row rho, on exit v[i] = element 16 j + i.
//   inverse: on entry v[i] = element 16 j + i, on exit v[i] = element j + 16 i.
__device__ __forceinline__ int rpad(int p) { return p + (p >> 4); }

template <class A>
__device__ __forceinline__ void rows_fwd_regs(const A &ar, typename A::T *v, const u64 *tw, const u64 *tws, void *lds, int rho, int j, u32 r) {
    typename A::T *l = (typename A::T *)lds;
    ct4(ar, v, tw, tws, 256u + r);
#pragma unroll
    for (int i = 0; i < 16; i++) l[rpad(rho * 256 + j + 16 * i)] = ar.mid(v[i]);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; i++) v[i] = l[rpad(rho * 256 + 16 * j + i)];
    ct4(ar, v, tw, tws, (256u + r) * 16u + j);
}
template <class A>
__device__ __forceinline__ void rows_inv_regs(const A &ar, typename A::T *v, const u64 *tw, const u64 *tws, void *lds, int rho, int j, u32 r) {
    typename A::T *l = (typename A::T *)lds;
    gs4(ar, v, tw, tws, (256u + r) * 16u + j);
#pragma unroll
    for (int i = 0; i < 16; i++) l[rpad(rho * 256 + 16 * j + i)] = ar.mid(v[i]);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; i++) v[i] = l[rpad(rho * 256 + j + 16 * i)];
    gs4(ar, v, tw, tws, 256u + r);
}
