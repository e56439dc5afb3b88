// Key-switching, accumulate, rescale and the small element-wise kernels.
//
// Rotation (paper, Preliminaries: Rot) = automorphism X -> X^g plus hybrid key
// switching.  The steps, in the order they are applied here:
//   k_modup    digit decomposition of c1 and fast basis conversion of every digit
//              to Q_l + P (coefficient form)
//   (transform of the raised digits, ntt.hip)
//   k_inner    automorphism (a permutation of transform-domain positions, read
//              side) fused with the inner product against the key
//   (inverse transform of the two accumulators)
//   k_moddown  division by P with basis conversion P -> Q_l, fused with the
//              addition of phi_g(c0)
// Alg. 1 (PCMM) itself is k_accumulate: signed sums of ciphertext limb words.
#include "common.h"
#include "hostmath.h"

#define EW_THREADS 256

__device__ __forceinline__ int ext_prime(int e, int l1, int L) { return e < l1 ? e : L + (e - l1); }

// ------------------------------------------------------------------ ModUp
// grid (N/256, n_ct).  c1 of ciphertext c starts at ct_base + c*ct_stride + limb_stride*N.
__global__ __launch_bounds__(EW_THREADS) void k_modup(ModUpConst mc, const PrimeConst *pc, int L, int N, const u64 *ct_base,
                                                      size_t ct_stride, int limb_stride, u64 *digits) {
    const int idx = blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int ct = blockIdx.y;
    const int ext = mc.l1 + mc.K;
    const u64 *c1 = ct_base + (size_t)ct * ct_stride + (size_t)limb_stride * N;
    u64 *out = digits + (size_t)ct * mc.beta * ext * N;
    for (int j = 0; j < mc.beta; j++) {
        const int first = j * mc.alpha, ns = mc.n_src[j];
        u64 y[ENSI_MAX_ALPHA], x[ENSI_MAX_ALPHA];
        for (int a = 0; a < ENSI_MAX_ALPHA; a++) {
            if (a < ns) {
                x[a] = c1[(size_t)(first + a) * N + idx];
                y[a] = mul_shoup(x[a], mc.inv[j * mc.alpha + a], mc.inv_s[j * mc.alpha + a], pc[first + a].q);
            }
        }
        for (int e = 0; e < ext; e++) {
            u64 r;
            if (e >= first && e < first + ns) {
                r = x[e - first];
            } else {
                const PrimeConst p = pc[ext_prime(e, mc.l1, L)];
                const u64 *hat = mc.hat + ((size_t)j * ext + e) * mc.alpha;
                acc128 acc = {0, 0};
                for (int a = 0; a < ENSI_MAX_ALPHA; a++)
                    if (a < ns) mac128(acc, y[a], hat[a]);
                r = mont_reduce(acc, p.q, p.qneg_inv);
            }
            out[((size_t)j * ext + e) * N + idx] = r;
        }
    }
}

void launch_modup(ensi_ctx *ctx, const ModUpConst &mc, const u64 *ct_base, size_t ct_stride_words, int limb_stride,
                  int n_ct, u64 *digits, hipStream_t st) {
    ScopedTimer t(ctx, "modup", st);
    dim3 grid((ctx->N + EW_THREADS - 1) / EW_THREADS, n_ct);
    hipLaunchKernelGGL(k_modup, grid, dim3(EW_THREADS), 0, st, mc, ctx->d_pc, ctx->L, ctx->N, ct_base, ct_stride_words,
                       limb_stride, digits);
}

// -------------------------------------------------- automorphism + inner product
// grid (N/256, l1+K, n_rot).  Transform-domain position k holds the evaluation at
// psi^(2*bitrev(k)+1); phi_g(d)(psi^e) = d(psi^(e*g)), so output position k reads
// position bitrev(((2*bitrev(k)+1)*g mod 2N - 1)/2).  With 256 consecutive
// positions per block the sources stay inside one 256-word row of the operand.
__global__ __launch_bounds__(EW_THREADS) void k_inner(const RotDesc *desc, const PrimeConst *pc, int L, int K, int log_n,
                                                      int l1, int beta, u64 *u) {
    const int N = 1 << log_n;
    const int k = blockIdx.x * EW_THREADS + threadIdx.x;
    if (k >= N) return;
    const int e = blockIdx.y;
    const int ext = l1 + K, ext_full = L + K;
    const RotDesc d = desc[blockIdx.z];
    const int prime = ext_prime(e, l1, L);
    const PrimeConst p = pc[prime];
    const u32 sh = 32 - log_n;
    const u32 ex = 2 * (__brev((u32)k) >> sh) + 1;
    const u32 es = (u32)(((u64)ex * d.g) & (2 * (u64)N - 1));
    const u32 ks = __brev((es - 1) >> 1) >> sh;
    u64 t0 = 0, t1 = 0;
    for (int j0 = 0; j0 < beta; j0 += 4) {
        acc128 a0 = {0, 0}, a1 = {0, 0};
        for (int j = j0; j < beta && j < j0 + 4; j++) {
            const u64 x = d.digits[((size_t)j * ext + e) * N + ks];
            const u64 *kj = d.key + ((size_t)j * 2 * ext_full + prime) * N + k;
            mac128(a0, x, kj[0]);
            mac128(a1, x, kj[(size_t)ext_full * N]);
        }
        t0 = add_mod(t0, mont_reduce(a0, p.q, p.qneg_inv), p.q);
        t1 = add_mod(t1, mont_reduce(a1, p.q, p.qneg_inv), p.q);
    }
    u64 *uo = u + ((size_t)blockIdx.z * 2 * ext + e) * N + k;
    uo[0] = t0;
    uo[(size_t)ext * N] = t1;
}

void launch_inner(ensi_ctx *ctx, const RotDesc *d_desc, int n_rot, int l1, int beta, u64 *u, hipStream_t st) {
    ScopedTimer t(ctx, "inner_product", st);
    dim3 grid((ctx->N + EW_THREADS - 1) / EW_THREADS, l1 + ctx->K, n_rot);
    hipLaunchKernelGGL(k_inner, grid, dim3(EW_THREADS), 0, st, d_desc, ctx->d_pc, ctx->L, ctx->K, ctx->log_n, l1, beta, u);
}

// --------------------------------------------------------- ModDown + phi_g(c0)
// grid (N/256, n_rot).  u: [n_rot][2][l1+K][N] coefficient form.
__global__ __launch_bounds__(EW_THREADS) void k_moddown(ModDownConst mc, const RotDesc *desc, const PrimeConst *pc, int L, int N,
                                                        int limb_stride_in, int limb_stride_out, const u64 *u) {
    const int idx = blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= N) return;
    const RotDesc d = desc[blockIdx.y];
    const int ext = mc.l1 + mc.K;
    // source coefficient of phi_g(c0) for output position idx
    const u32 i0 = (u32)(((u64)idx * d.g_inv) & (2 * (u64)N - 1));
    const bool neg = i0 >= (u32)N;
    const u32 isrc = neg ? i0 - N : i0;
    for (int poly = 0; poly < 2; poly++) {
        const u64 *up = u + ((size_t)blockIdx.y * 2 + poly) * ext * N;
        // residues [u * (P/p_k)^-1]_{p_k}; the conversion takes them centred, i.e. every residue above
        // p_k/2 stands for itself minus p_k, which changes the converted value by -(P mod q_i)
        u64 y[ENSI_MAX_K];
        int n_neg = 0;
        for (int k = 0; k < ENSI_MAX_K; k++)
            if (k < mc.K) {
                const u64 pk = pc[L + k].q;
                y[k] = mul_shoup(up[(size_t)(mc.l1 + k) * N + idx], mc.inv[k], mc.inv_s[k], pk);
                n_neg += y[k] > pk / 2 ? 1 : 0;
            }
        for (int i = 0; i < mc.l1; i++) {
            const PrimeConst p = pc[i];
            acc128 acc = {0, 0};
            for (int k = 0; k < ENSI_MAX_K; k++)
                if (k < mc.K) mac128(acc, y[k], mc.hat[i * mc.K + k]);
            u64 r = sub_mod(mont_reduce(acc, p.q, p.qneg_inv), mc.negtab[i * (mc.K + 1) + n_neg], p.q);
            u64 v = mul_shoup(sub_mod(up[(size_t)i * N + idx], r, p.q), mc.pinv[i], mc.pinv_s[i], p.q);
            if (poly == 0) {
                u64 c = d.c0[(size_t)i * N + isrc];
                v = add_mod(v, neg ? neg_mod(c, p.q) : c, p.q);
            }
            d.out[((size_t)poly * limb_stride_out + i) * N + idx] = v;
        }
    }
}

void launch_moddown(ensi_ctx *ctx, const ModDownConst &mc, const RotDesc *d_desc, int n_rot, int limb_stride_in,
                    int limb_stride_out, const u64 *u, hipStream_t st) {
    ScopedTimer t(ctx, "moddown", st);
    dim3 grid((ctx->N + EW_THREADS - 1) / EW_THREADS, n_rot);
    hipLaunchKernelGGL(k_moddown, grid, dim3(EW_THREADS), 0, st, mc, d_desc, ctx->d_pc, ctx->L, ctx->N, limb_stride_in,
                       limb_stride_out, u);
}

// ------------------------------------------------------------ Alg. 1 accumulate
// y_i = sum_v W'[v][i] x_v over limb words, W' in {-1,0,+1} given as two 32-bit
// masks (+1 bits, -1 bits) per (output tile of 32, operand v).  Each thread owns
// one word position and 32 output accumulators; the weight bits are uniform over
// the block, so zero weights are skipped by uniform branches.  Sums are kept as
// wrapping signed 64-bit integers and reduced every `red_every` operands.
#define ACC_T 32
__global__ __launch_bounds__(EW_THREADS) void k_accumulate(const u64 *xbase, size_t xstride, int n_v, const u32 *masks, int m,
                                                           const PrimeConst *pc, int N, int l1, int limb_stride_in, u64 *out,
                                                           int limb_stride_out, int red_every) {
    const size_t w = (size_t)blockIdx.y * EW_THREADS + threadIdx.x;  // word within the active limbs of one ciphertext
    const size_t per_poly = (size_t)l1 * N;
    if (w >= 2 * per_poly) return;
    const int poly = (int)(w / per_poly);
    const size_t rem = w - (size_t)poly * per_poly;
    const int limb = (int)(rem / N);
    const u64 q = pc[limb].q;
    const size_t off_in = (size_t)poly * limb_stride_in * N + rem;
    const size_t off_out = (size_t)poly * limb_stride_out * N + rem;
    const int tile = blockIdx.x;
    const u32 *mk = masks + (size_t)tile * n_v * 2;
    int64_t acc[ACC_T];
#pragma unroll
    for (int t = 0; t < ACC_T; t++) acc[t] = 0;
    int since = 0;
    for (int v = 0; v < n_v; v++) {
        const u32 pm = mk[2 * v], mm = mk[2 * v + 1];
        if ((pm | mm) == 0) continue;
        const int64_t x = (int64_t)xbase[(size_t)v * xstride + off_in];
#pragma unroll
        for (int t = 0; t < ACC_T; t++) {
            if (pm & (1u << t)) acc[t] += x;
            else if (mm & (1u << t)) acc[t] -= x;
        }
        if (++since == red_every) {
            since = 0;
#pragma unroll
            for (int t = 0; t < ACC_T; t++) {
                int64_t a = acc[t];
                u64 r = (u64)(a < 0 ? -a : a) % q;
                acc[t] = (int64_t)((a < 0 && r) ? q - r : r);
            }
        }
    }
    const size_t ct_words_out = (size_t)2 * limb_stride_out * N;
#pragma unroll
    for (int t = 0; t < ACC_T; t++) {
        const int i = tile * ACC_T + t;
        if (i < m) {
            int64_t a = acc[t];
            u64 r = (u64)(a < 0 ? -a : a) % q;
            out[(size_t)i * ct_words_out + off_out] = (a < 0 && r) ? q - r : r;
        }
    }
}

void launch_accumulate(ensi_ctx *ctx, const u64 *xbase, size_t xstride, int n_v, const u32 *d_masks, int m, int l1,
                       int limb_stride_in, u64 *out, int limb_stride_out, hipStream_t st) {
    ScopedTimer t(ctx, "accumulate", st);
    int qbits = 0;
    for (int i = 0; i < l1; i++) {
        int b = 64 - __builtin_clzll(ctx->primes[i]);
        if (b > qbits) qbits = b;
    }
    int red_every = qbits >= 62 ? 1 : (int)std::min<int64_t>((int64_t)1 << (62 - qbits), 1 << 30);
    if (red_every > 1) red_every -= 1;  // the carried residue counts as one operand
    size_t words = (size_t)2 * l1 * ctx->N;
    dim3 grid((m + ACC_T - 1) / ACC_T, (unsigned)((words + EW_THREADS - 1) / EW_THREADS));
    hipLaunchKernelGGL(k_accumulate, grid, dim3(EW_THREADS), 0, st, xbase, xstride, n_v, d_masks, m, ctx->d_pc, ctx->N, l1,
                       limb_stride_in, out, limb_stride_out, red_every);
}

// ------------------------------------------------------- scalar multiply + rescale
// consts: [5][l1]: k mod q_i, Shoup(k), q_l^{-1} mod q_i, Shoup(.), q_l mod q_i  (rows 2..4 unused at i = l1-1)
// grid (N/256, 2, n_ct)
__global__ __launch_bounds__(EW_THREADS) void k_rescale(u64 *ct, int l1, int limb_stride, int N, const PrimeConst *pc,
                                                        const u64 *consts) {
    const int idx = blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= N) return;
    u64 *c = ct + ((size_t)blockIdx.z * 2 + blockIdx.y) * limb_stride * N;
    const int last = l1 - 1;
    const u64 ql = pc[last].q;
    const u64 xl = mul_shoup(c[(size_t)last * N + idx], consts[last], consts[l1 + last], ql);
    const bool neg = xl > ql / 2;
    // the update is in place, so the compiler must assume every store may feed the next load; limbs are
    // therefore loaded four at a time ahead of their stores to keep several loads in flight
    for (int i0 = 0; i0 < last; i0 += 4) {
        u64 in[4];
#pragma unroll
        for (int j = 0; j < 4; j++)
            if (i0 + j < last) in[j] = c[(size_t)(i0 + j) * N + idx];
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int i = i0 + j;
            if (i < last) {
                const u64 q = pc[i].q;
                const u64 v = mul_shoup(in[j], consts[i], consts[l1 + i], q);
                u64 r = xl;
                if (r >= q) {
                    r -= q;
                    if (r >= q) r %= q;
                }
                // centred representative of limb l: values above q_l/2 stand for themselves minus q_l
                if (neg) r = sub_mod(r, consts[4 * l1 + i], q);
                c[(size_t)i * N + idx] = mul_shoup(sub_mod(v, r, q), consts[2 * l1 + i], consts[3 * l1 + i], q);
            }
        }
    }
}

// The same step in fp64 for primes below 2^50 (64-bit integer multiplies are several times slower than
// fp64 FMAs here): residues are exact integers in doubles and x*w mod q is
// h = x*w; l = fma(x,w,-h); t = rint(x*(w/q)); r = fma(-t,q,h) + l, exact because h - t*q and l are
// integers below 2^53.  fconsts: [5][l1] doubles: k mod q_i, (k mod q_i)/q_i, q_l^{-1} mod q_i, that/q_i, 1/q_i.
// All limbs of a coefficient are loaded before the first store, so the in-place update keeps l1 loads in
// flight per thread.  grid (N/256, 2, n_ct)
struct FpMod {
    double q, qinv;
    __device__ __forceinline__ double mid(double x) const { return fma(-rint(x * qinv), q, x); }
    __device__ __forceinline__ double mulmod(double x, double w, double wq) const {
        const double h = x * w;
        const double l = fma(x, w, -h);
        const double t = rint(x * wq);
        return fma(-t, q, h) + l;
    }
};
template <int MAXL>
__global__ __launch_bounds__(EW_THREADS) void k_rescale_fp(u64 *ct, int l1, int limb_stride, int N, const PrimeConst *pc, const double *fc) {
    const int idx = blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= N) return;
    u64 *c = ct + ((size_t)blockIdx.z * 2 + blockIdx.y) * limb_stride * N + idx;
    const int last = l1 - 1;
    u64 in[MAXL];
#pragma unroll
    for (int i = 0; i < MAXL; i++)
        if (i < l1) in[i] = c[(size_t)i * N];
    FpMod ml = {(double)pc[last].q, fc[4 * l1 + last]};
    double xl = 0.0;
#pragma unroll
    for (int i = 0; i < MAXL; i++)
        if (i == last) xl = ml.mid(ml.mulmod((double)in[i], fc[last], fc[l1 + last]));  // centred [c_l * k]_{q_l}
#pragma unroll
    for (int i = 0; i < MAXL; i++) {
        if (i < last) {
            FpMod m = {(double)pc[i].q, fc[4 * l1 + i]};
            const double v = m.mulmod((double)in[i], fc[i], fc[l1 + i]) - m.mid(xl);
            double r = m.mid(m.mulmod(m.mid(v), fc[2 * l1 + i], fc[3 * l1 + i]));
            r = r < 0.0 ? r + m.q : r;
            c[(size_t)i * N] = (u64)r;
        }
    }
}

void launch_rescale(ensi_ctx *ctx, u64 *ct, int n_ct, int l1, int limb_stride, const u64 *d_consts, const double *d_fconsts,
                    hipStream_t st) {
    ScopedTimer t(ctx, "mul_scalar_rescale", st);
    dim3 grid((ctx->N + EW_THREADS - 1) / EW_THREADS, 2, n_ct);
    if (d_fconsts && l1 <= 16)
        hipLaunchKernelGGL(k_rescale_fp<16>, grid, dim3(EW_THREADS), 0, st, ct, l1, limb_stride, ctx->N, ctx->d_pc, d_fconsts);
    else if (d_fconsts)
        hipLaunchKernelGGL(k_rescale_fp<ENSI_MAX_EXT>, grid, dim3(EW_THREADS), 0, st, ct, l1, limb_stride, ctx->N, ctx->d_pc, d_fconsts);
    else
        hipLaunchKernelGGL(k_rescale, grid, dim3(EW_THREADS), 0, st, ct, l1, limb_stride, ctx->N, ctx->d_pc, d_consts);
}

// ------------------------------------------------------------- element-wise
// rows are limb rows of N words; row r uses prime map.prime[r % map.n]
__global__ __launch_bounds__(EW_THREADS) void k_small_to_rns(const int8_t *in, LimbMap map, const PrimeConst *pc, int N, u64 *out) {
    const int idx = blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int row = blockIdx.y;
    const int poly = row / map.n;
    const u64 q = pc[map.prime[row % map.n]].q;
    const int v = in[(size_t)poly * N + idx];
    out[(size_t)row * N + idx] = v >= 0 ? (u64)v : q - (u64)(-v);
}
void launch_small_to_rns(ensi_ctx *ctx, const int8_t *d_in, int n_poly, const LimbMap &map, u64 *out, hipStream_t st) {
    dim3 grid((ctx->N + EW_THREADS - 1) / EW_THREADS, n_poly * map.n);
    hipLaunchKernelGGL(k_small_to_rns, grid, dim3(EW_THREADS), 0, st, d_in, map, ctx->d_pc, ctx->N, out);
}

__global__ __launch_bounds__(EW_THREADS) void k_i64_to_rns(const int64_t *in, LimbMap map, const PrimeConst *pc, int N, u64 *out) {
    const int idx = blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int row = blockIdx.y;
    const int poly = row / map.n;
    const u64 q = pc[map.prime[row % map.n]].q;
    const int64_t v = in[(size_t)poly * N + idx];
    const u64 r = (u64)(v < 0 ? -v : v) % q;
    out[(size_t)row * N + idx] = (v < 0 && r) ? q - r : r;
}
void launch_i64_to_rns(ensi_ctx *ctx, const int64_t *d_in, int n_poly, const LimbMap &map, u64 *out, hipStream_t st) {
    dim3 grid((ctx->N + EW_THREADS - 1) / EW_THREADS, n_poly * map.n);
    hipLaunchKernelGGL(k_i64_to_rns, grid, dim3(EW_THREADS), 0, st, d_in, map, ctx->d_pc, ctx->N, out);
}

// Counter-based uniform residues (see the generator's specification in ensi.h).
__device__ __forceinline__ u64 mix64(u64 z) {
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}
__global__ __launch_bounds__(EW_THREADS) void k_uniform(u64 *out, LimbMap map, const PrimeConst *pc, int N, u64 seed, u64 stream_id) {
    const int idx = blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int row = blockIdx.y;
    const int prime = map.prime[row];
    const PrimeConst p = pc[prime];
    const u64 G = 0x9E3779B97F4A7C15ULL;
    const u64 key = mix64(mix64(mix64(seed) + stream_id) + (u64)prime);
    const u64 hi = mix64(key + G * (2 * (u64)idx + 1));
    const u64 lo = mix64(key + G * (2 * (u64)idx + 2));
    // (hi * 2^64 + lo) mod q = hi * (2^64 mod q) + lo:  mont_mul(hi mod q, r2) = hi * 2^64 mod q
    const u64 h = mont_mul(hi % p.q, p.r2, p.q, p.qneg_inv);
    out[(size_t)row * N + idx] = add_mod(h, lo % p.q, p.q);
}
void launch_uniform(ensi_ctx *ctx, u64 *out, const LimbMap &map, u64 seed, u64 stream_id, hipStream_t st) {
    dim3 grid((ctx->N + EW_THREADS - 1) / EW_THREADS, map.n);
    hipLaunchKernelGGL(k_uniform, grid, dim3(EW_THREADS), 0, st, out, map, ctx->d_pc, ctx->N, seed, stream_id);
}

__global__ __launch_bounds__(EW_THREADS) void k_mul_mont(u64 *out, const u64 *a, const u64 *b, LimbMap map, const PrimeConst *pc, int N) {
    const int idx = blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int row = blockIdx.y;
    const PrimeConst p = pc[map.prime[row % map.n]];
    const size_t o = (size_t)row * N + idx;
    out[o] = mont_mul(a[o], b[o], p.q, p.qneg_inv);
}
void launch_mul_mont(ensi_ctx *ctx, u64 *out, const u64 *a, const u64 *b_mont, int n_rows, const LimbMap &map, hipStream_t st) {
    dim3 grid((ctx->N + EW_THREADS - 1) / EW_THREADS, n_rows);
    hipLaunchKernelGGL(k_mul_mont, grid, dim3(EW_THREADS), 0, st, out, a, b_mont, map, ctx->d_pc, ctx->N);
}

__global__ __launch_bounds__(EW_THREADS) void k_add(u64 *out, const u64 *a, const u64 *b, LimbMap map, const PrimeConst *pc, int N) {
    const int idx = blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int row = blockIdx.y;
    const u64 q = pc[map.prime[row % map.n]].q;
    const size_t o = (size_t)row * N + idx;
    out[o] = add_mod(a[o], b[o], q);
}
void launch_add(ensi_ctx *ctx, u64 *out, const u64 *a, const u64 *b, int n_rows, const LimbMap &map, hipStream_t st) {
    dim3 grid((ctx->N + EW_THREADS - 1) / EW_THREADS, n_rows);
    hipLaunchKernelGGL(k_add, grid, dim3(EW_THREADS), 0, st, out, a, b, map, ctx->d_pc, ctx->N);
}

__global__ __launch_bounds__(EW_THREADS) void k_to_mont(u64 *data, LimbMap map, const PrimeConst *pc, int N) {
    const int idx = blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int row = blockIdx.y;
    const PrimeConst p = pc[map.prime[row % map.n]];
    const size_t o = (size_t)row * N + idx;
    data[o] = mont_mul(data[o], p.r2, p.q, p.qneg_inv);
}
void launch_to_mont(ensi_ctx *ctx, u64 *data, int n_rows, const LimbMap &map, hipStream_t st) {
    dim3 grid((ctx->N + EW_THREADS - 1) / EW_THREADS, n_rows);
    hipLaunchKernelGGL(k_to_mont, grid, dim3(EW_THREADS), 0, st, data, map, ctx->d_pc, ctx->N);
}

// Stored key words back to ordinary residues, in place: limbs that the fused N = 2^16 kernels keep as doubles in
// [0,p) (fp_format, primes below 2^50) are converted, every other word leaves Montgomery form.
__global__ __launch_bounds__(EW_THREADS) void k_key_to_plain(u64 *data, LimbMap map, const PrimeConst *pc, int N, int fp_format) {
    const int idx = blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int row = blockIdx.y;
    const PrimeConst p = pc[map.prime[row % map.n]];
    const size_t o = (size_t)row * N + idx;
    if (fp_format && p.pad[0]) {
        data[o] = (u64)__longlong_as_double((long long)data[o]);
    } else {
        acc128 t = {data[o], 0};
        data[o] = mont_reduce(t, p.q, p.qneg_inv);
    }
}
void launch_key_to_plain(ensi_ctx *ctx, u64 *data, int n_rows, const LimbMap &map, bool fp_format, hipStream_t st) {
    dim3 grid((ctx->N + EW_THREADS - 1) / EW_THREADS, n_rows);
    hipLaunchKernelGGL(k_key_to_plain, grid, dim3(EW_THREADS), 0, st, data, map, ctx->d_pc, ctx->N, fp_format ? 1 : 0);
}

// Number of words of a batch of limb rows that are not canonical residues (>= their prime), added to *bad.
__global__ __launch_bounds__(EW_THREADS) void k_count_noncanonical(const u64 *data, LimbMap map, const PrimeConst *pc, int N, unsigned int *bad) {
    const int idx = blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int row = blockIdx.y;
    if (data[(size_t)row * N + idx] >= pc[map.prime[row % map.n]].q) atomicAdd(bad, 1u);
}
void launch_count_noncanonical(ensi_ctx *ctx, const u64 *data, int n_rows, const LimbMap &map, unsigned int *d_bad, hipStream_t st) {
    dim3 grid((ctx->N + EW_THREADS - 1) / EW_THREADS, n_rows);
    hipLaunchKernelGGL(k_count_noncanonical, grid, dim3(EW_THREADS), 0, st, data, map, ctx->d_pc, ctx->N, d_bad);
}

// Wrap-around 64-bit sum of the active limb words of every ciphertext of a batch: sums[c] += sum of the words of
// ciphertext c ([2][limb_stride][N], first l1 limbs of each polynomial).  grid (ceil(N / (EW_THREADS * 8)), 2 * l1, n).
__global__ __launch_bounds__(EW_THREADS) void k_ct_checksum(const u64 *ct, int l1, int limb_stride, int N, unsigned long long *sums) {
    __shared__ unsigned long long part[EW_THREADS / 64];
    const int c = blockIdx.z, poly = blockIdx.y / l1, limb = blockIdx.y - poly * l1;
    const u64 *row = ct + (((size_t)c * 2 + poly) * limb_stride + limb) * N;
    unsigned long long acc = 0;
    for (int i = blockIdx.x * EW_THREADS * 8 + threadIdx.x; i < N && i < (int)(blockIdx.x + 1) * EW_THREADS * 8; i += EW_THREADS) acc += row[i];
    for (int off = 32; off; off >>= 1) acc += __shfl_down(acc, off, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long t = 0;
        for (int w = 0; w < EW_THREADS / 64; w++) t += part[w];
        atomicAdd(&sums[c], t);
    }
}
void launch_ct_checksum(ensi_ctx *ctx, const u64 *ct, int n, int l1, int limb_stride, u64 *d_sums, hipStream_t st) {
    dim3 grid((ctx->N + EW_THREADS * 8 - 1) / (EW_THREADS * 8), 2 * l1, n);
    hipLaunchKernelGGL(k_ct_checksum, grid, dim3(EW_THREADS), 0, st, ct, l1, limb_stride, ctx->N, (unsigned long long *)d_sums);
}

// b = -a*s + e + factor[row]*sg  (transform domain); s_mont is in Montgomery form;
// b is written in Montgomery form.  One row per limb of map.
__global__ __launch_bounds__(EW_THREADS) void k_key_assemble(u64 *b_out, const u64 *a, const u64 *s_mont, const u64 *e, const u64 *sg,
                                                             const u64 *factor, LimbMap map, const PrimeConst *pc, int N) {
    const int idx = blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int row = blockIdx.y;
    const PrimeConst p = pc[map.prime[row]];
    const size_t o = (size_t)row * N + idx;
    u64 as = mont_mul(a[o], s_mont[o], p.q, p.qneg_inv);  // a*s
    u64 b = add_mod(neg_mod(as, p.q), e[o], p.q);
    if (sg != nullptr && factor[row] != 0) {
        // factor is stored in Montgomery form: mont_mul(sg, factor*R) = sg*factor
        b = add_mod(b, mont_mul(sg[o], factor[row], p.q, p.qneg_inv), p.q);
    }
    b_out[o] = mont_mul(b, p.r2, p.q, p.qneg_inv);
}
void launch_key_assemble(ensi_ctx *ctx, u64 *b_out, const u64 *a, const u64 *s_mont, const u64 *e, const u64 *sg,
                         const u64 *d_factor, const LimbMap &map, hipStream_t st) {
    dim3 grid((ctx->N + EW_THREADS - 1) / EW_THREADS, map.n);
    hipLaunchKernelGGL(k_key_assemble, grid, dim3(EW_THREADS), 0, st, b_out, a, s_mont, e, sg, d_factor, map, ctx->d_pc, ctx->N);
}

// Coefficient-form automorphism: out[k] = +-in[k * g^{-1} mod 2N].
__global__ __launch_bounds__(EW_THREADS) void k_automorphism_coef(u64 *out, const u64 *in, LimbMap map, const PrimeConst *pc, int N, u32 g_inv) {
    const int idx = blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int row = blockIdx.y;
    const u64 q = pc[map.prime[row % map.n]].q;
    const u32 i0 = (u32)(((u64)idx * g_inv) & (2 * (u64)N - 1));
    const u64 v = in[(size_t)row * N + (i0 >= (u32)N ? i0 - N : i0)];
    out[(size_t)row * N + idx] = i0 >= (u32)N ? neg_mod(v, q) : v;
}
void launch_automorphism_coef(ensi_ctx *ctx, u64 *out, const u64 *in, const LimbMap &map, u32 g_inv, hipStream_t st) {
    dim3 grid((ctx->N + EW_THREADS - 1) / EW_THREADS, map.n);
    hipLaunchKernelGGL(k_automorphism_coef, grid, dim3(EW_THREADS), 0, st, out, in, map, ctx->d_pc, ctx->N, g_inv);
}

// ---------------------------------------------------------------- encode / decode
// Column-wise SIMD encoding pi (paper, Preliminaries), in fp64:
//   coefficient k = round_half_away((2*scale/N) * sum_j z_j cos(pi * 5^j * k / N))        (encode)
//   slot j        = (1/scale) * sum_k m_k cos(pi * 5^j * k / N)                           (decode)
// Both sums are the real part of one length-2N discrete Fourier transform of a real vector: encode transforms the
// vector that holds z_j at index 5^j mod 2N and reads outputs 0..N-1, decode transforms (m_0..m_{N-1}, 0..0) and reads
// outputs 5^j mod 2N.  The transform is a self-sorting radix-2 Stockham FFT, one pass per launch over the whole batch
// (log2(2N) passes of 2N complex doubles each way: tens of microseconds per plaintext where the defining sums took
// hundreds of milliseconds); twiddles come from the context's table of cos(pi e / N), which holds the 2N-th roots.
// Rounding error: below 1e-13 * ||input||_2 per output, far under one half of a coefficient at every scale in use.
constexpr int FFT_CHUNK = 128;  // plaintexts per batch of transforms: 2 x 128 x 2N x 16 B of workspace (512 MiB at N = 2^16)

__global__ __launch_bounds__(EW_THREADS) void k_fft_pass(const double2 *x, double2 *y, int n2, int s, const double *cos_tab) {
    const int t = blockIdx.x * EW_THREADS + threadIdx.x;
    if (t >= n2 / 2) return;
    x += (size_t)blockIdx.y * n2;
    y += (size_t)blockIdx.y * n2;
    const int q = t & (s - 1), idx = t - q;  // idx = p * s with p = t / s: the twiddle is exp(-2 pi i idx / n2)
    const double2 a = x[t], b = x[t + n2 / 2];
    const double c = cos_tab[idx], sn = cos_tab[(idx - n2 / 4) & (n2 - 1)];
    const double dr = a.x - b.x, di = a.y - b.y;
    const size_t o = (size_t)q + 2 * (size_t)idx;
    y[o] = make_double2(a.x + b.x, a.y + b.y);
    y[o + s] = make_double2(dr * c + di * sn, di * c - dr * sn);
}
// Plaintext y of the chunk holds its n_slots values in slots [slot0 + (y0 + y)*slot_step, ... + n_slots); x is zero beforehand.
__global__ __launch_bounds__(EW_THREADS) void k_fft_scatter_slots(const double *slots, int n_slots, int slot0, int slot_step, int y0,
                                                                  const u32 *rot_exp, int n2, double2 *x) {
    const int j = blockIdx.x * EW_THREADS + threadIdx.x;
    if (j >= n_slots) return;
    const int y = y0 + blockIdx.y;
    x[(size_t)blockIdx.y * n2 + rot_exp[slot0 + (size_t)y * slot_step + j]] = make_double2(slots[(size_t)y * n_slots + j], 0.0);
}
__global__ __launch_bounds__(EW_THREADS) void k_fft_round_coeffs(const double2 *f, int N, double factor, int64_t *coeffs) {
    const int k = blockIdx.x * EW_THREADS + threadIdx.x;
    if (k >= N) return;
    const double m = f[(size_t)blockIdx.y * 2 * N + k].x * factor;
    const double r = floor(fabs(m) + 0.5);
    coeffs[(size_t)blockIdx.y * N + k] = (int64_t)(m < 0 ? -r : r);
}
__global__ __launch_bounds__(EW_THREADS) void k_fft_load_coeffs(const double *coeffs, int N, double2 *x) {
    const int k = blockIdx.x * EW_THREADS + threadIdx.x;
    if (k >= 2 * N) return;
    x[(size_t)blockIdx.y * 2 * N + k] = make_double2(k < N ? coeffs[(size_t)blockIdx.y * N + k] : 0.0, 0.0);
}
__global__ __launch_bounds__(EW_THREADS) void k_fft_gather_slots(const double2 *f, int n2, const u32 *rot_exp, int slot_begin, int n_slots,
                                                                 double inv_scale, double *out) {
    const int j = blockIdx.x * EW_THREADS + threadIdx.x;
    if (j >= n_slots) return;
    out[(size_t)blockIdx.y * n_slots + j] = f[(size_t)blockIdx.y * n2 + rot_exp[slot_begin + j]].x * inv_scale;
}
// All passes over `count` transforms; returns the buffer that holds the result (a or b).
static double2 *fft_passes(ensi_ctx *ctx, double2 *a, double2 *b, int count, hipStream_t st) {
    const int n2 = 2 * ctx->N;
    dim3 grid((n2 / 2 + EW_THREADS - 1) / EW_THREADS, count);
    for (int s = 1; s < n2; s *= 2) {
        hipLaunchKernelGGL(k_fft_pass, grid, dim3(EW_THREADS), 0, st, a, b, n2, s, ctx->d_cos);
        std::swap(a, b);
    }
    return a;
}
static hipError_t fft_workspace(ensi_ctx *ctx, int n, double2 **a, double2 **b) {
    const size_t bytes = (size_t)std::min(n, FFT_CHUNK) * 2 * ctx->N * sizeof(double2);
    *a = *b = nullptr;
    hipError_t e = hipMalloc((void **)a, bytes);
    if (e == hipSuccess) e = hipMalloc((void **)b, bytes);
    if (e != hipSuccess && *a) {
        (void)hipFree(*a);
        *a = nullptr;
    }
    return e;
}
hipError_t launch_encode(ensi_ctx *ctx, const double *d_slots, int n_pt, int n_slots, int slot0, int slot_step, double scale,
                         int64_t *d_coeffs, hipStream_t st) {
    const int N = ctx->N, n2 = 2 * N;
    double2 *a, *b;
    hipError_t e = fft_workspace(ctx, n_pt, &a, &b);
    if (e != hipSuccess) return e;
    for (int y0 = 0; y0 < n_pt && e == hipSuccess; y0 += FFT_CHUNK) {
        const int cnt = std::min(FFT_CHUNK, n_pt - y0);
        e = hipMemsetAsync(a, 0, (size_t)cnt * n2 * sizeof(double2), st);
        hipLaunchKernelGGL(k_fft_scatter_slots, dim3((n_slots + EW_THREADS - 1) / EW_THREADS, cnt), dim3(EW_THREADS), 0, st, d_slots, n_slots,
                           slot0, slot_step, y0, ctx->d_rot_exp, n2, a);
        const double2 *f = fft_passes(ctx, a, b, cnt, st);
        hipLaunchKernelGGL(k_fft_round_coeffs, dim3((N + EW_THREADS - 1) / EW_THREADS, cnt), dim3(EW_THREADS), 0, st, f, N, 2.0 * scale / N,
                           d_coeffs + (size_t)y0 * N);
    }
    const hipError_t e2 = hipStreamSynchronize(st);
    (void)hipFree(a);
    (void)hipFree(b);
    return e != hipSuccess ? e : e2;
}

// Garner CRT of limbs 0 and 1 (rows 0,1 of each [n_used][N] block), centred, as double.
// big = q0*q1 is passed as (big_hi, big_lo).
__global__ __launch_bounds__(EW_THREADS) void k_crt_center(const u64 *m, int n_used, int N, u64 q0, u64 q1, u64 q0_inv_mont,
                                                           u64 q1_neg_inv, u64 big_hi, u64 big_lo, double *out) {
    const int idx = blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= N) return;
    const u64 *mm = m + (size_t)blockIdx.y * n_used * N;
    const u64 r0 = mm[idx];
    double v;
    if (n_used == 1) {
        v = r0 > q0 / 2 ? -(double)(q0 - r0) : (double)r0;
    } else {
        const u64 r1 = mm[(size_t)N + idx];
        const u64 d = sub_mod(r1, r0 % q1, q1);
        const u64 t = mont_mul(d, q0_inv_mont, q1, q1_neg_inv);  // (r1-r0) * q0^{-1} mod q1
        // val = r0 + q0*t  (< q0*q1 < 2^124)
        u64 lo = q0 * t, hi = mulhi64(q0, t);
        lo += r0;
        hi += lo < r0 ? 1 : 0;
        // half = floor(big/2); negative branch when val > half
        const u64 half_hi = big_hi >> 1, half_lo = (big_lo >> 1) | (big_hi << 63);
        const bool neg = hi > half_hi || (hi == half_hi && lo > half_lo);
        if (neg) {  // val = big - val
            const u64 nlo = big_lo - lo;
            hi = big_hi - hi - (big_lo < lo ? 1 : 0);
            lo = nlo;
        }
        v = (double)hi * 18446744073709551616.0 + (double)lo;
        if (neg) v = -v;
    }
    out[(size_t)blockIdx.y * N + idx] = v;
}
void launch_crt_center(ensi_ctx *ctx, const u64 *m, int n_ct, int n_limbs_used, double *out, hipStream_t st) {
    const u64 q0 = ctx->primes[0];
    u64 q1 = 0, q0_inv_mont = 0, q1_neg_inv = 0, big_hi = 0, big_lo = 0;
    if (n_limbs_used >= 2) {
        q1 = ctx->primes[1];
        u64 q0_inv = hm_invmod(q0 % q1, q1);
        q0_inv_mont = (u64)((((u128)q0_inv) << 64) % q1);
        q1_neg_inv = hm_neg_inv64(q1);
        u128 big = (u128)q0 * q1;
        big_hi = (u64)(big >> 64);
        big_lo = (u64)big;
    }
    dim3 grid((ctx->N + EW_THREADS - 1) / EW_THREADS, n_ct);
    hipLaunchKernelGGL(k_crt_center, grid, dim3(EW_THREADS), 0, st, m, n_limbs_used, ctx->N, q0, q1, q0_inv_mont, q1_neg_inv,
                       big_hi, big_lo, out);
}

__global__ __launch_bounds__(EW_THREADS) void k_center_i64(const u64 *m, size_t stride, int N, u64 q0, int64_t *out) {
    const int idx = blockIdx.x * EW_THREADS + threadIdx.x;
    if (idx >= N) return;
    const u64 r = m[(size_t)blockIdx.y * stride + idx];
    out[(size_t)blockIdx.y * N + idx] = r > q0 / 2 ? -(int64_t)(q0 - r) : (int64_t)r;
}
void launch_center_i64(ensi_ctx *ctx, const u64 *m, size_t stride_words, int n, int64_t *out, hipStream_t st) {
    dim3 grid((ctx->N + EW_THREADS - 1) / EW_THREADS, n);
    hipLaunchKernelGGL(k_center_i64, grid, dim3(EW_THREADS), 0, st, m, stride_words, ctx->N, ctx->primes[0], out);
}

// z_j = (1/scale) sum_k m_k cos(pi 5^j k / N) for j in [slot_begin, slot_begin+n_slots): the same transform, read at 5^j.
hipError_t launch_decode(ensi_ctx *ctx, const double *d_coeffs, int n_ct, int slot_begin, int n_slots, double inv_scale, double *d_out,
                         hipStream_t st) {
    const int N = ctx->N, n2 = 2 * N;
    double2 *a, *b;
    hipError_t e = fft_workspace(ctx, n_ct, &a, &b);
    if (e != hipSuccess) return e;
    for (int y0 = 0; y0 < n_ct; y0 += FFT_CHUNK) {
        const int cnt = std::min(FFT_CHUNK, n_ct - y0);
        hipLaunchKernelGGL(k_fft_load_coeffs, dim3((n2 + EW_THREADS - 1) / EW_THREADS, cnt), dim3(EW_THREADS), 0, st,
                           d_coeffs + (size_t)y0 * N, N, a);
        const double2 *f = fft_passes(ctx, a, b, cnt, st);
        hipLaunchKernelGGL(k_fft_gather_slots, dim3((n_slots + EW_THREADS - 1) / EW_THREADS, cnt), dim3(EW_THREADS), 0, st, f, n2,
                           ctx->d_rot_exp, slot_begin, n_slots, inv_scale, d_out + (size_t)y0 * n_slots);
    }
    e = hipStreamSynchronize(st);
    (void)hipFree(a);
    (void)hipFree(b);
    return e;
}
