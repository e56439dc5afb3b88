// Rotation (paper, Preliminaries: Rot) for the ring N = 2^16 with ciphertext primes below 2^50:
// automorphism plus hybrid key switching in five kernels that keep every intermediate in
// the layout and number format of the transform passes around it.
//
//   k_ks16_pre         y_a = c1_a * (Q_j/q_a)^-1 mod q_a for every ciphertext limb (the inner factor
//                      of the fast basis conversion), once per input ciphertext
//   k_ks16_up_fcols    ModUp fused into the forward column pass: each block forms its 256 x 16
//                      tile of the raised digit  sum_a y_a * (Q_j/q_a) mod t  (or copies the limb
//                      inside its own digit) in registers and runs the column pass on it.  The
//                      same kernel transforms P * c0, so that phi_g(c0) can be added in the
//                      transform domain (ModDown divides it by P again, exactly)
//   k_ks16_frows       forward row pass of the raised digits and of P * c0
//   k_ks16_inner_irows automorphism (a permutation of transform-domain positions that maps rows
//                      onto rows, applied on the read side) + inner product with the key +
//                      P * phi_g(c0), fused into the inverse row pass
//   k_ks16_icols_special, k_ks16_icols_down
//                      inverse column pass fused with ModDown: the K special limbs are transformed
//                      first and left as centred residues y_k = [u * (P/p_k)^-1]_{p_k}; every
//                      ciphertext limb is then transformed and leaves as
//                      u * P^-1 - sum_k y_k * p_k^-1  mod q_i
//
// Number formats between the kernels (workspaces only, never visible outside the library):
// limbs of primes below 2^50 hold doubles (exact integers, |x| <= p/2); limbs of wider primes
// hold canonical 64-bit residues.  The key holds doubles in [0,p) on the former and Montgomery
// residues on the latter.  All results that leave the last kernel are canonical residues and
// equal, word for word, what the unfused sequence (ModUp, transform, inner product, inverse
// transform, ModDown, + phi_g(c0)) gives.
#include "common.h"
#include "ntt16_core.h"

#define KS_THREADS 256
#define KS_N 65536
#ifndef KS_BATCH
#define KS_BATCH 8  // positions whose operands are loaded together in the inner product
#endif

__device__ __forceinline__ int ks_ext_prime(int e, int l1, int L) { return e < l1 ? e : L + (e - l1); }
__device__ __forceinline__ double as_f64(u64 x) { return __longlong_as_double((long long)x); }
__device__ __forceinline__ u64 as_u64(double x) { return (u64)__double_as_longlong(x); }

// ------------------------------------------------------------------ inner factor of ModUp
// grid (N/256, l1, n_ct)
__global__ __launch_bounds__(KS_THREADS) void k_ks16_pre(Ks16Const kc, const PrimeConst *pcs, const u64 *ct_base, size_t ct_stride,
                                                         int limb_stride, u64 *ybuf) {
    const int idx = blockIdx.x * KS_THREADS + threadIdx.x;
    const int a = blockIdx.y, ct = blockIdx.z;
    const u64 *c1 = ct_base + (size_t)ct * ct_stride + (size_t)limb_stride * KS_N;
    const u64 q = pcs[a].q;
    ybuf[((size_t)ct * kc.l1 + a) * KS_N + idx] = mul_shoup(c1[(size_t)a * KS_N + idx], kc.inv[a], kc.inv_s[a], q);
}

// ------------------------------------------------------------------ ModUp + forward column pass
// grid (16, beta*ext + l1, n_ct): row R < beta*ext is limb R % ext of raised digit R / ext, the last
// l1 rows are P * c0.  dig: [n_ct][beta*ext + l1][N].
__global__ __launch_bounds__(KS_THREADS) void k_ks16_up_fcols(Ks16Const kc, const PrimeConst *pcs, const u64 *tw_all, const u64 *ct_base,
                                                              size_t ct_stride, int limb_stride, const u64 *ybuf, u64 *dig) {
    __shared__ u64 lds[4096];
    const int tid = threadIdx.x, c = tid & 15, jj = tid >> 4;
    const int R = blockIdx.y, ct = blockIdx.z;
    const int l1 = kc.l1, ext = l1 + kc.K, n_rows = kc.beta * ext + l1;
    const u64 *c0 = ct_base + (size_t)ct * ct_stride;
    const u64 *c1 = c0 + (size_t)limb_stride * KS_N;
    const u64 *y = ybuf + (size_t)ct * l1 * KS_N;
    const size_t col = (size_t)blockIdx.x * 16 + c;
    u64 *out = dig + ((size_t)ct * n_rows + R) * KS_N + col;
    int prime, j = 0, e = 0;
    bool digit_row = R < kc.beta * ext;
    if (digit_row) {
        j = R / ext;
        e = R - j * ext;
        prime = ks_ext_prime(e, l1, kc.L);
    } else {
        prime = R - kc.beta * ext;
    }
    const PrimeConst pc = pcs[prime];
    const u64 *tw = tw_all + (size_t)prime * 4 * KS_N;
    const int first = j * kc.alpha, ns = digit_row ? kc.n_src[j] : 0;
    if (pc.pad[0]) {
        ArithFp ar;
        ar.init(pc);
        double v[16];
        if (!digit_row) {
            const double pm = kc.pmod_fp[2 * prime], pm_p = kc.pmod_fp[2 * prime + 1];
#pragma unroll
            for (int i = 0; i < 16; i++) v[i] = ar.mid(ar.mulmod((double)c0[(size_t)prime * KS_N + (size_t)(jj + 16 * i) * 256 + col], pm, pm_p));
        } else if (e >= first && e < first + ns) {
#pragma unroll
            for (int i = 0; i < 16; i++) v[i] = (double)c1[(size_t)e * KS_N + (size_t)(jj + 16 * i) * 256 + col];
        } else {
            const double *hat = kc.hat_fp + ((size_t)j * ext + e) * kc.alpha * 2;
#pragma unroll
            for (int i = 0; i < 16; i++) v[i] = 0.0;
            for (int a = 0; a < ns; a++) {
                const double h = hat[2 * a], hp = hat[2 * a + 1];
                const u64 *ya = y + (size_t)(first + a) * KS_N + col;
#pragma unroll
                for (int i = 0; i < 16; i++) v[i] += ar.mulmod((double)ya[(size_t)(jj + 16 * i) * 256], h, hp);
            }
#pragma unroll
            for (int i = 0; i < 16; i++) v[i] = ar.mid(v[i]);
        }
        cols_fwd_regs(ar, v, tw, tw + KS_N, lds, c, jj);
#pragma unroll
        for (int i = 0; i < 16; i++) out[(size_t)(16 * jj + i) * 256] = as_u64(ar.mid(v[i]));
    } else {
        // a wide prime is always a conversion target (ciphertext primes are below 2^50 on this path)
        ArithInt ar;
        ar.init(pc);
        u64 v[16];
        const u64 *hat = kc.hat_mont + ((size_t)j * ext + e) * kc.alpha;
        acc128 acc[16];
#pragma unroll
        for (int i = 0; i < 16; i++) acc[i] = {0, 0};
        for (int a = 0; a < ns; a++) {
            const u64 h = hat[a];
            const u64 *ya = y + (size_t)(first + a) * KS_N + col;
#pragma unroll
            for (int i = 0; i < 16; i++) mac128(acc[i], ya[(size_t)(jj + 16 * i) * 256], h);
        }
#pragma unroll
        for (int i = 0; i < 16; i++) v[i] = mont_reduce(acc[i], pc.q, pc.qneg_inv);
        cols_fwd_regs(ar, v, tw, tw + KS_N, lds, c, jj);
#pragma unroll
        for (int i = 0; i < 16; i++) out[(size_t)(16 * jj + i) * 256] = ar.store_fwd(v[i]);
    }
}

// ------------------------------------------------------------------ forward row pass (in place)
// grid (16 * (beta*ext + l1) * ceil(n_ct / KS_FROWS_GROUP)).  A block runs one 16-row tile of one limb for up to
// KS_FROWS_GROUP ciphertexts in a row: the twiddles of the tile -- the larger part of what a single tile loads, 15
// pairs per row for the first step and 15 pairs per thread for the second -- are fetched once (first step: LDS,
// second step: registers), and the next ciphertext's tile is requested before the current one is transformed.
#define KS_FROWS_GROUP 8  // measured: 4 -> 0.91 ms, 8 -> 0.83 ms, 16 -> 0.86 ms per 64 raised ciphertexts (one tile at a time: 1.12 ms)
template <class A>
__device__ __forceinline__ void frows_body(u64 *g, size_t ct_stride, int n_here, const u64 *tw, const PrimeConst &pc, u64 *lds, ulonglong2 *tw1,
                                           int r0) {
    A ar;
    ar.init(pc);
    const int tid = threadIdx.x, rho = tid >> 4, j = tid & 15;
    const u32 r = (u32)(r0 + rho);
    row_table_to_lds(tw1, tw, tw + KS_N, 256u + r, rho, j);
    TwRegs tw2;
    tw2.load(tw, tw + KS_N, (256u + r) * 16u + j);
    typename A::T v[16], nv[16];
    typename A::T *l = (typename A::T *)lds;
    {
        const typename A::T *gt = (const typename A::T *)g;
#pragma unroll
        for (int i = 0; i < 16; i++) nv[i] = gt[rho * 256 + j + 16 * i];
    }
    __syncthreads();  // tw1 is complete
    const ulonglong2 *tab = tw1 + rho * 16;
#pragma unroll 1
    for (int c = 0; c < n_here; c++) {
#pragma unroll
        for (int i = 0; i < 16; i++) v[i] = nv[i];
        if (c + 1 < n_here) {
            const typename A::T *gt = (const typename A::T *)(g + (size_t)(c + 1) * ct_stride);
#pragma unroll
            for (int i = 0; i < 16; i++) nv[i] = gt[rho * 256 + j + 16 * i];
        }
        ct4_tab(ar, v, tab);
#pragma unroll
        for (int i = 0; i < 16; i++) l[rpad(rho * 256 + j + 16 * i)] = ar.mid(v[i]);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 16; i++) v[i] = l[rpad(rho * 256 + 16 * j + i)];
        ct4_tab(ar, v, tw2);
#pragma unroll
        for (int i = 0; i < 16; i++) lds[rpad(rho * 256 + 16 * j + i)] = ar.store_ws_fwd(v[i]);
        __syncthreads();
        u64 *go = g + (size_t)c * ct_stride;
#pragma unroll
        for (int i = 0; i < 16; i++) go[tid + 256 * i] = lds[rpad(tid + 256 * i)];
        __syncthreads();  // the tile is reused by the next ciphertext's exchange
    }
}

// (two blocks per CU: with a third the register file forces spills and the pass takes half as long again)
__global__ __launch_bounds__(KS_THREADS, 2) void k_ks16_frows(Ks16Const kc, const PrimeConst *pcs, const u64 *tw_all, u64 *dig, int n_ct) {
    __shared__ u64 lds[4096 + 256];
    __shared__ ulonglong2 tw1[16 * 16];
    // The ciphertext group runs fastest: blocks that share a tile of the twiddle table (same limb, same rows) are
    // launched together and fetch it from memory once per XCD.
    const int n_grp = (n_ct + KS_FROWS_GROUP - 1) / KS_FROWS_GROUP;
    const int grp = blockIdx.x % n_grp, tile = (blockIdx.x / n_grp) & 15, R = blockIdx.x / (n_grp * 16);
    const int l1 = kc.l1, ext = l1 + kc.K, n_rows = kc.beta * ext + l1;
    const int prime = R < kc.beta * ext ? ks_ext_prime(R % ext, l1, kc.L) : R - kc.beta * ext;
    const PrimeConst pc = pcs[prime];
    const u64 *tw = tw_all + (size_t)prime * 4 * KS_N;
    const int r0 = tile * 16, ct0 = grp * KS_FROWS_GROUP;
    const int n_here = min(KS_FROWS_GROUP, n_ct - ct0);
    const size_t ct_stride = (size_t)n_rows * KS_N;
    u64 *g = dig + ((size_t)ct0 * n_rows + R) * KS_N + (size_t)r0 * 256;
    if (pc.pad[0]) frows_body<ArithFp>(g, ct_stride, n_here, tw, pc, lds, tw1, r0);
    else frows_body<ArithInt>(g, ct_stride, n_here, tw, pc, lds, tw1, r0);
}

// ---------------------------------------- automorphism + key inner product + inverse row pass
// grid (16, n_rot, ext): limb slowest, so that the blocks in flight share one limb of the digits.
// Transform-domain position k holds the evaluation at psi^(2*bitrev(k)+1); phi_g(d)(psi^e) =
// d(psi^(e*g)), so output position k reads position bitrev(((2*bitrev(k)+1)*g mod 2N - 1)/2), which
// lies in one source row for all 256 positions of an output row.
__device__ __forceinline__ u32 ks_perm(u32 k, u32 g) {
    const u32 ex = 2 * (__brev(k) >> 16) + 1;
    const u32 es = (ex * g) & (2 * KS_N - 1);
    return __brev((es - 1) >> 1) >> 16;
}

// FP: the limbs of primes below 2^50 (fp64 arithmetic) or the wider ones (integer arithmetic); the two
// are separate kernels so that each gets its own register allocation.  limb_list holds the extended-
// basis limb index of each grid slot z.
struct LimbList {
    int32_t n;
    int32_t e[ENSI_MAX_EXT];
};

// members > 1: the block adds the inner products of `members` consecutive descriptors (rotations of one ciphertext:
// same digits, their own Galois element and key) before the inverse pass, so that the group is brought back to
// the ciphertext basis by one inverse transform and one ModDown; grid y then counts groups.
template <bool FP>
__global__ __launch_bounds__(KS_THREADS, FP ? 3 : 2) void k_ks16_inner_irows(Ks16Const kc, const RotDesc *desc, const PrimeConst *pcs, const u64 *tw_all,
                                                                 u64 *u, LimbList limbs, int members) {
    __shared__ u64 lds[(FP ? 1 : 2) * (4096 + 256)];
    __shared__ ulonglong2 tw1[16 * 16];
    const int tid = threadIdx.x, rho = tid >> 4, j16 = tid & 15;
    const int rot = blockIdx.y, e = limbs.e[blockIdx.z];
    const int l1 = kc.l1, ext = l1 + kc.K, ext_full = kc.L + kc.K, beta = kc.beta;
    const int prime = ks_ext_prime(e, l1, kc.L);
    const PrimeConst pc = pcs[prime];
    const u64 *tw = tw_all + (size_t)prime * 4 * KS_N + 2 * KS_N;
    const int r0 = blockIdx.x * 16;
    const size_t kstride = (size_t)ext_full * KS_N;  // words between b_j and a_j, and half the distance between digits
    u64 *uo = u + ((size_t)rot * 2 * ext + e) * KS_N + (size_t)r0 * 256;
    if (FP) {
        ArithFp ar;
        ar.init(pc);
        double a0[16], a1[16];
#pragma unroll
        for (int i = 0; i < 16; i++) a0[i] = a1[i] = 0.0;
#pragma unroll 1
        for (int mem = 0; mem < members; mem++) {
        const RotDesc d = desc[rot * members + mem];
        const u64 *dg = d.digits + (size_t)e * KS_N;
        const u64 *key = d.key + (size_t)prime * KS_N + (size_t)r0 * 256 + tid;
        u32 ks[16];
#pragma unroll
        for (int i = 0; i < 16; i++) ks[i] = ks_perm((u32)((r0 + i) * 256 + tid), d.g);
        const u64 *c0h = d.digits + ((size_t)beta * ext + e) * KS_N;
        if (e < l1) {
#pragma unroll
            for (int i = 0; i < 16; i++) a0[i] += as_f64(c0h[ks[i]]);
        }
        // one digit at a time; the operands of KS_BATCH positions are loaded together, then consumed
#pragma unroll 1
        for (int jd = 0; jd < beta; jd++) {
            const u64 *dj = dg + (size_t)jd * ext * KS_N;
            const u64 *kj = key + (size_t)jd * 2 * kstride;
#pragma unroll
            for (int h = 0; h < 16; h += KS_BATCH) {
                double x[KS_BATCH], k0[KS_BATCH], k1[KS_BATCH];
#pragma unroll
                for (int i = 0; i < KS_BATCH; i++) {
                    x[i] = as_f64(dj[ks[h + i]]);
                    k0[i] = as_f64(kj[(h + i) * 256]);
                    k1[i] = as_f64(kj[kstride + (h + i) * 256]);
                }
#pragma unroll
                for (int i = 0; i < KS_BATCH; i++) {
                    a0[h + i] += ar.mulmod_np(x[i], k0[i]);
                    a1[h + i] += ar.mulmod_np(x[i], k1[i]);
                }
            }
        }
        if (members > 1) {
            // a member adds up to beta + 1 terms below 0.7 p: reduced between members, the sums stay exact integers
#pragma unroll
            for (int i = 0; i < 16; i++) {
                a0[i] = ar.mid(a0[i]);
                a1[i] = ar.mid(a1[i]);
            }
        }
        }
        // Inverse row pass of both sums.  Its twiddles are fetched once for the two polynomials: the 15 pairs of the
        // second step (per row) into LDS, the 15 pairs of the first step (per thread) into registers.
        double *l = (double *)lds;
        double v[16];
        row_table_to_lds(tw1, tw, tw + KS_N, 256u + (u32)(r0 + rho), rho, j16);
        TwRegs tw2;
        tw2.load(tw, tw + KS_N, (256u + (u32)(r0 + rho)) * 16u + j16);
        const ulonglong2 *tab = tw1 + rho * 16;
#pragma unroll
        for (int poly = 0; poly < 2; poly++) {
            if (poly) __syncthreads();
#pragma unroll
            for (int i = 0; i < 16; i++) l[rpad(tid + 256 * i)] = ar.mid(poly ? a1[i] : a0[i]);
            __syncthreads();  // (also makes tw1 visible)
#pragma unroll
            for (int i = 0; i < 16; i++) v[i] = l[rpad(rho * 256 + 16 * j16 + i)];
            gs4_tab(ar, v, tw2);
#pragma unroll
            for (int i = 0; i < 16; i++) l[rpad(rho * 256 + 16 * j16 + i)] = ar.mid(v[i]);
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 16; i++) v[i] = l[rpad(rho * 256 + j16 + 16 * i)];
            gs4_tab(ar, v, tab);
            u64 *o = uo + (size_t)poly * ext * KS_N + rho * 256 + j16;
#pragma unroll
            for (int i = 0; i < 16; i++) o[16 * i] = as_u64(ar.mid(v[i]));
        }
    } else {
        // Montgomery products summed in 128 bits, reduced once per four digits (4 * 2^120 < p * 2^64).  The
        // sums of eight positions at a time go straight to LDS (one tile per polynomial).
        ArithInt ar;
        ar.init(pc);
        u64 *lds1 = lds + 4096 + 256;
#pragma unroll 1
        for (int h = 0; h < 16; h += 8) {
            u64 t0[8], t1[8];
#pragma unroll
            for (int i = 0; i < 8; i++) t0[i] = t1[i] = 0;
#pragma unroll 1
            for (int mem = 0; mem < members; mem++) {
            const RotDesc d = desc[rot * members + mem];
            const u64 *dg = d.digits + (size_t)e * KS_N;
            const u64 *key = d.key + (size_t)prime * KS_N + (size_t)r0 * 256 + tid;
#pragma unroll 1
            for (int j0 = 0; j0 < beta; j0 += 4) {
                acc128 s0[8], s1[8];
#pragma unroll
                for (int i = 0; i < 8; i++) {
                    s0[i] = {0, 0};
                    s1[i] = {0, 0};
                }
#pragma unroll 1
                for (int jd = j0; jd < beta && jd < j0 + 4; jd++) {
                    const u64 *dj = dg + (size_t)jd * ext * KS_N;
                    const u64 *kj = key + (size_t)jd * 2 * kstride + h * 256;
                    u64 x[8], k0[8], k1[8];
#pragma unroll
                    for (int i = 0; i < 8; i++) {
                        x[i] = dj[ks_perm((u32)((r0 + h + i) * 256 + tid), d.g)];
                        k0[i] = kj[i * 256];
                        k1[i] = kj[kstride + i * 256];
                    }
#pragma unroll
                    for (int i = 0; i < 8; i++) {
                        mac128(s0[i], x[i], k0[i]);
                        mac128(s1[i], x[i], k1[i]);
                    }
                }
#pragma unroll
                for (int i = 0; i < 8; i++) {
                    t0[i] = add_mod(t0[i], mont_reduce(s0[i], pc.q, pc.qneg_inv), pc.q);
                    t1[i] = add_mod(t1[i], mont_reduce(s1[i], pc.q, pc.qneg_inv), pc.q);
                }
            }
            }
#pragma unroll
            for (int i = 0; i < 8; i++) {
                lds[rpad(tid + 256 * (h + i))] = t0[i];
                lds1[rpad(tid + 256 * (h + i))] = t1[i];
            }
        }
        row_table_to_lds(tw1, tw, tw + KS_N, 256u + (u32)(r0 + rho), rho, j16);
        TwRegs tw2;
        tw2.load(tw, tw + KS_N, (256u + (u32)(r0 + rho)) * 16u + j16);
        const ulonglong2 *tab = tw1 + rho * 16;
        __syncthreads();
        u64 v[16];
#pragma unroll 1
        for (int poly = 0; poly < 2; poly++) {
            u64 *lp = poly ? lds1 : lds;
#pragma unroll
            for (int i = 0; i < 16; i++) v[i] = lp[rpad(rho * 256 + 16 * j16 + i)];
            gs4_tab(ar, v, tw2);
#pragma unroll
            for (int i = 0; i < 16; i++) lp[rpad(rho * 256 + 16 * j16 + i)] = v[i];
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 16; i++) v[i] = lp[rpad(rho * 256 + j16 + 16 * i)];
            gs4_tab(ar, v, tab);
            u64 *o = uo + (size_t)poly * ext * KS_N + rho * 256 + j16;
#pragma unroll
            for (int i = 0; i < 16; i++) o[16 * i] = ar.store_inv(v[i]);
        }
    }
}

// ------------------------------------------------------ inverse column pass + ModDown
// Two kernels.  k_ks16_icols_special transforms the K special limbs of both accumulators and leaves,
// per coefficient, the centred residue y = [u * (P/p_k)^-1]_{p_k} split as y = hi * 2^30 + lo (lo in the
// low word, hi signed in the high word of one 64-bit word).  k_ks16_icols_down then handles one
// ciphertext limb of one column tile per block: inverse column pass, then
//   out = u * N^-1 P^-1 - sum_k (lo_k * p_k^-1 + hi_k * 2^30 p_k^-1)  mod q_i
// in fp64 (every factor is below 2^30 or a precomputed constant with its quotient).  Blocks that
// share a tile (the l1 limbs) are adjacent in the grid, so the y words are read from HBM once.

// grid (16, 2K, n_rot); ysp: [n_rot][2][K][N]
__global__ __launch_bounds__(KS_THREADS) void k_ks16_icols_special(Ks16Const kc, const PrimeConst *pcs, const u64 *tw_all, const u64 *u,
                                                                   u64 *ysp) {
    __shared__ u64 lds[4096];
    const int tid = threadIdx.x, c = tid & 15, jj = tid >> 4;
    const int K = kc.K, ext = kc.l1 + K;
    const int poly = blockIdx.y / K, k = blockIdx.y - poly * K, rot = blockIdx.z;
    const size_t col = (size_t)blockIdx.x * 16 + c;
    const int prime = kc.L + k;
    const PrimeConst pc = pcs[prime];
    const u64 *tw = tw_all + (size_t)prime * 4 * KS_N + 2 * KS_N;
    const u64 *src = u + (((size_t)rot * 2 + poly) * ext + kc.l1 + k) * KS_N + col;
    u64 *dst = ysp + (((size_t)rot * 2 + poly) * K + k) * KS_N + col;
    int64_t y[16];
    if (pc.pad[0]) {
        ArithFp ar;
        ar.init(pc);
        double v[16];
#pragma unroll
        for (int i = 0; i < 16; i++) v[i] = as_f64(src[(size_t)(16 * jj + i) * 256]);
        cols_inv_regs(ar, v, tw, tw + KS_N, lds, c, jj);
        const double cs = kc.down_p_fp[2 * k], cs_p = kc.down_p_fp[2 * k + 1];
#pragma unroll
        for (int i = 0; i < 16; i++) y[i] = (int64_t)ar.mid(ar.mulmod(ar.mid(v[i]), cs, cs_p));
    } else {
        ArithInt ar;
        ar.init(pc);
        u64 v[16];
#pragma unroll
        for (int i = 0; i < 16; i++) v[i] = src[(size_t)(16 * jj + i) * 256];
        cols_inv_regs(ar, v, tw, tw + KS_N, lds, c, jj);
        const u64 cs = kc.down_p[2 * k], cs_s = kc.down_p[2 * k + 1];
#pragma unroll
        for (int i = 0; i < 16; i++) {
            const u64 yv = mul_shoup(v[i], cs, cs_s, pc.q);
            y[i] = yv > pc.q / 2 ? (int64_t)yv - (int64_t)pc.q : (int64_t)yv;
        }
    }
#pragma unroll
    for (int i = 0; i < 16; i++) {
        const u32 lo = (u32)(y[i] & 0x3fffffff);
        const u32 hi = (u32)(int32_t)(y[i] >> 30);
        dst[(size_t)(jj + 16 * i) * 256] = ((u64)hi << 32) | lo;
    }
}

// grid (l1, 32, n_rot): blockIdx.y = poly * 16 + column tile
__global__ __launch_bounds__(KS_THREADS) void k_ks16_icols_down(Ks16Const kc, const RotDesc *desc, const PrimeConst *pcs, const u64 *tw_all,
                                                                const u64 *u, const u64 *ysp, int limb_stride_out, int members) {
    __shared__ u64 lds[4096];
    __shared__ ulonglong2 ctab[COL_TAB_PAIRS];
    const int tid = threadIdx.x, c = tid & 15, jj = tid >> 4;
    const int limb = blockIdx.x, poly = blockIdx.y >> 4, rot = blockIdx.z;
    const int l1 = kc.l1, K = kc.K, ext = l1 + K;
    const size_t col = (size_t)(blockIdx.y & 15) * 16 + c;
    const u64 *src = u + (((size_t)rot * 2 + poly) * ext + limb) * KS_N + col;
    const u64 *ys = ysp + ((size_t)rot * 2 + poly) * K * KS_N + col;
    const RotDesc dl = desc[rot * members];  // the group's first descriptor carries the destination
    u64 *out = dl.out + ((size_t)poly * limb_stride_out + limb) * KS_N + col;
    const PrimeConst pc = pcs[limb];
    const u64 *tw = tw_all + (size_t)limb * 4 * KS_N + 2 * KS_N;
    ArithFp ar;
    ar.init(pc);
    double v[16];
    col_tables_to_lds(ctab, tw, tw + KS_N, tid);
#pragma unroll
    for (int i = 0; i < 16; i++) v[i] = as_f64(src[(size_t)(16 * jj + i) * 256]);
    __syncthreads();
    cols_inv_regs_t(ar, v, ctab, lds, c, jj);
    const double *dq = kc.down_q + (size_t)limb * (2 + 4 * K);
    const double sc = dq[0], sc_p = dq[1];
#pragma unroll
    for (int i = 0; i < 16; i++) v[i] = ar.mulmod(ar.mid(v[i]), sc, sc_p);
#pragma unroll
    for (int k = 0; k < ENSI_MAX_K; k++) {
        if (k < K) {
            const double h_lo = dq[2 + 4 * k], h_lo_p = dq[3 + 4 * k], h_hi = dq[4 + 4 * k], h_hi_p = dq[5 + 4 * k];
            u64 w[16];
#pragma unroll
            for (int i = 0; i < 16; i++) w[i] = ys[(size_t)k * KS_N + (size_t)(jj + 16 * i) * 256];
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const double lo = (double)(int)(u32)w[i];
                const double hi = (double)(int)(u32)(w[i] >> 32);
                v[i] -= ar.mulmod(lo, h_lo, h_lo_p) + ar.mulmod(hi, h_hi, h_hi_p);
            }
        }
    }
    if (dl.accumulate) {
        // out <- out + result: `out` may be the rotation's own source (every read of the source happened in the
        // raise kernels, which have finished), which turns t <- t + Rot(t; r) into one pass
        const u64 q = pc.q;
#pragma unroll
        for (int i = 0; i < 16; i++) {
            u64 *o = out + (size_t)(jj + 16 * i) * 256;
            *o = add_mod(*o, ar.canon(v[i]), q);
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < 16; i++) out[(size_t)(jj + 16 * i) * 256] = ar.canon(v[i]);
}

// ---------------------------------------------------------------- key format
// In place on one key [beta][2][L+K][N] that holds Montgomery residues everywhere: limbs of
// primes below 2^50 become doubles in [0,p).  grid (N/256, L+K, 2*beta)
__global__ __launch_bounds__(KS_THREADS) void k_ks16_key_format(u64 *key, const PrimeConst *pcs, int ext_full) {
    const int idx = blockIdx.x * KS_THREADS + threadIdx.x;
    const int prime = blockIdx.y;
    const PrimeConst pc = pcs[prime];
    if (!pc.pad[0]) return;
    u64 *w = key + ((size_t)blockIdx.z * ext_full + prime) * KS_N + idx;
    acc128 t = {*w, 0};
    *w = as_u64((double)mont_reduce(t, pc.q, pc.qneg_inv));
}

// ---------------------------------------------------------------- launchers
void launch_ks16_key_format(ensi_ctx *ctx, u64 *key, int beta_full, hipStream_t st) {
    dim3 grid(KS_N / KS_THREADS, ctx->L + ctx->K, 2 * beta_full);
    hipLaunchKernelGGL(k_ks16_key_format, grid, dim3(KS_THREADS), 0, st, key, ctx->d_pc, ctx->L + ctx->K);
}

void launch_ks16_raise(ensi_ctx *ctx, const Ks16Const &kc, const u64 *ct_base, size_t ct_stride_words, int limb_stride, int n_ct,
                       u64 *ybuf, u64 *dig, hipStream_t st) {
    const int n_rows = kc.beta * (kc.l1 + kc.K) + kc.l1;
    {
        ScopedTimer t(ctx, "ks_pre", st);
        hipLaunchKernelGGL(k_ks16_pre, dim3(KS_N / KS_THREADS, kc.l1, n_ct), dim3(KS_THREADS), 0, st, kc, ctx->d_pc, ct_base,
                           ct_stride_words, limb_stride, ybuf);
    }
    {
        ScopedTimer t(ctx, "ks_modup_fcols", st);
        hipLaunchKernelGGL(k_ks16_up_fcols, dim3(16, n_rows, n_ct), dim3(KS_THREADS), 0, st, kc, ctx->d_pc, ctx->d_tw, ct_base,
                           ct_stride_words, limb_stride, ybuf, dig);
    }
    {
        ScopedTimer t(ctx, "ks_frows", st);
        hipLaunchKernelGGL(k_ks16_frows, dim3(16 * n_rows * ((n_ct + KS_FROWS_GROUP - 1) / KS_FROWS_GROUP)), dim3(KS_THREADS), 0, st, kc, ctx->d_pc, ctx->d_tw,
                           dig, n_ct);
    }
}

void launch_ks16_switch(ensi_ctx *ctx, const Ks16Const &kc, const RotDesc *d_desc, int n_rot, u64 *u, u64 *ysp, int limb_stride_out,
                        hipStream_t st, int members) {
    // n_rot descriptors in groups of `members` (1: every rotation on its own); u and ysp are indexed by group
    const int n_grp = n_rot / members;
    // limbs of wide primes (integer arithmetic, ALU-bound) first, then the fp64 limbs (memory-bound)
    LimbList wide, fp;
    wide.n = fp.n = 0;
    for (int e = 0; e < kc.l1 + kc.K; e++) {
        const u64 q = ctx->primes[e < kc.l1 ? e : kc.L + (e - kc.l1)];
        LimbList &dst = q < ((u64)1 << 50) ? fp : wide;
        dst.e[dst.n++] = e;
    }
    if (wide.n) {
        ScopedTimer t(ctx, "ks_inner_irows_wide", st);
        hipLaunchKernelGGL(k_ks16_inner_irows<false>, dim3(16, n_grp, wide.n), dim3(KS_THREADS), 0, st, kc, d_desc, ctx->d_pc, ctx->d_tw, u, wide,
                           members);
    }
    if (fp.n) {
        ScopedTimer t(ctx, "ks_inner_irows", st);
        hipLaunchKernelGGL(k_ks16_inner_irows<true>, dim3(16, n_grp, fp.n), dim3(KS_THREADS), 0, st, kc, d_desc, ctx->d_pc, ctx->d_tw, u, fp, members);
    }
    {
        ScopedTimer t(ctx, "ks_icols_special", st);
        hipLaunchKernelGGL(k_ks16_icols_special, dim3(16, 2 * kc.K, n_grp), dim3(KS_THREADS), 0, st, kc, ctx->d_pc, ctx->d_tw, u, ysp);
    }
    {
        ScopedTimer t(ctx, "ks_icols_moddown", st);
        hipLaunchKernelGGL(k_ks16_icols_down, dim3(kc.l1, 32, n_grp), dim3(KS_THREADS), 0, st, kc, d_desc, ctx->d_pc, ctx->d_tw, u, ysp,
                           limb_stride_out, members);
    }
}
