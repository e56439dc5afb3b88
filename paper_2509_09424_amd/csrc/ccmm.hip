// Ciphertext-ciphertext multiplication (paper, Preliminaries: Multiplication, Mult) for the ciphertext-
// ciphertext matrix product of the CCMM section:  out_o = Rescale(Relin(sum_t a_t (x) b_t)).
//
// The tensor product of two ciphertexts is three polynomials (d0, d1, d2) = (a0 b0, a0 b1 + a1 b0, a1 b1),
// products in R_{Q_l}, i.e. pointwise in the transform domain.  The products of one output are added there,
// transformed back once, d2 is key-switched from s^2 to s with the evaluation key (the same raise / inner
// product / ModDown kernels as a rotation, with the identity automorphism, fed (d0, d2) as if it were a
// ciphertext so that d0 is added on the way), d1 is added and the result rescaled.
//
// Kernels here: the gather of the two polynomials of every distinct operand of a group (an operand that enters
// several products is transformed once), the multiply-add that forms
// (d0, d2, d1) per output, the addition of d1 and a strided ciphertext addition (used by the rotate-and-add
// steps of the element replication).  Transforms, key switch, rescale and the final strided copy are the
// library's existing kernels.
#include "common.h"
#include "ntt16_core.h"

#define MM_THREADS 256

// grid (ceil(N/256) * n_ops, 2*l1): ws_a[u][p*l1+i][N] <- polynomial p, limb i of distinct operand u
__global__ __launch_bounds__(MM_THREADS) void k_mm_gather(MmGroup g, int N, int nb) {
    const int u = blockIdx.x / nb;
    const int idx = (blockIdx.x - u * nb) * MM_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int y = blockIdx.y, p = y / g.l1, i = y - p * g.l1;
    const MmOperand op = g.ops[u];
    g.ws_a[((size_t)u * 2 * g.l1 + y) * N + idx] = op.p[((size_t)p * op.limb_stride + i) * N + idx];
}

// grid (ceil(N/256), l1, n_out): ws_d[o][0|1|2][i][N] <- d0, d2, d1 (transform domain).  Operands are ordinary
// residues: a Montgomery product carries a factor 2^-64, removed once per sum with 2^128 mod q.
__global__ __launch_bounds__(MM_THREADS) void k_mm_tensor_mac(MmGroup g, int N, const PrimeConst *pcs) {
    const int idx = blockIdx.x * MM_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int i = blockIdx.y, o = blockIdx.z;
    const PrimeConst pc = pcs[i];
    const u64 q = pc.q, qn = pc.qneg_inv;
    const int t0 = g.begin[o], t1 = g.begin[o + 1];
    u64 d0 = 0, d1 = 0, d2 = 0;
    const size_t poly = (size_t)g.l1 * N;
    for (int t = t0; t < t1; t++) {
        const MmPair pr = g.pairs[t - g.t_base];
        const u64 *xa = g.ops[pr.a].t + (size_t)i * N + idx;
        const u64 *xb = g.ops[pr.b].t + (size_t)i * N + idx;
        const u64 a0 = xa[0], a1 = xa[poly], b0 = xb[0], b1 = xb[poly];
        d0 = add_mod(d0, mont_mul(a0, b0, q, qn), q);
        d1 = add_mod(d1, add_mod(mont_mul(a0, b1, q, qn), mont_mul(a1, b0, q, qn), q), q);
        d2 = add_mod(d2, mont_mul(a1, b1, q, qn), q);
    }
    u64 *out = g.ws_d + ((size_t)o * 3 * g.l1 + i) * N + idx;
    out[0] = mont_mul(d0, pc.r2, q, qn);
    out[poly] = mont_mul(d2, pc.r2, q, qn);
    out[2 * poly] = mont_mul(d1, pc.r2, q, qn);
}

// The same sums for outputs that form a grid (MmGroup.grid_x, grid_y), primes below 2^50: a block forms a tile of 4 x 2
// outputs for 256 words of one limb, so that every operand word it reads enters 2 or 4 products (the plain kernel reads
// four operand words per product, most of them again and again for other outputs), and multiplies in fp64 on exact
// integers.  grid (ceil(N/256), l1, tiles_x * tiles_y).
#define MM_TX 4
#define MM_TY 2
__global__ __launch_bounds__(MM_THREADS) void k_mm_grid_mac_fp(MmGroup g, int N, const PrimeConst *pcs) {
    const int idx = blockIdx.x * MM_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int i = blockIdx.y;
    const int tiles_y = (g.grid_y + MM_TY - 1) / MM_TY;
    const int x0 = (blockIdx.z / tiles_y) * MM_TX, y0 = (blockIdx.z % tiles_y) * MM_TY;
    ArithFp ar;
    ar.init(pcs[i]);
    const double half = 0.5 * ar.p;
    const size_t poly = (size_t)g.l1 * N, off = (size_t)i * N + idx;
    const int J = g.begin[1] - g.begin[0];
    // term j of output (x, y0) names the left operand of row x, term j of output (x0, y) the right operand of column y
    const MmPair *pa[MM_TX], *pb[MM_TY];
#pragma unroll
    for (int x = 0; x < MM_TX; x++) pa[x] = g.pairs + (g.begin[(x0 + x < g.grid_x ? x0 + x : x0) * g.grid_y + y0] - g.t_base);
#pragma unroll
    for (int y = 0; y < MM_TY; y++) pb[y] = g.pairs + (g.begin[x0 * g.grid_y + (y0 + y < g.grid_y ? y0 + y : y0)] - g.t_base);
    double d0[MM_TX][MM_TY], d1[MM_TX][MM_TY], d2[MM_TX][MM_TY];
#pragma unroll
    for (int x = 0; x < MM_TX; x++)
#pragma unroll
        for (int y = 0; y < MM_TY; y++) d0[x][y] = d1[x][y] = d2[x][y] = 0.0;
    for (int j = 0; j < J; j++) {
        double a0[MM_TX], a1[MM_TX], b0[MM_TY], b1[MM_TY];
#pragma unroll
        for (int x = 0; x < MM_TX; x++) {
            const u64 *p = g.ops[pa[x][j].a].t + off;
            const double v0 = (double)p[0], v1 = (double)p[poly];
            a0[x] = v0 > half ? v0 - ar.p : v0;  // the left factor centred: |a| <= p/2
            a1[x] = v1 > half ? v1 - ar.p : v1;
        }
#pragma unroll
        for (int y = 0; y < MM_TY; y++) {
            const u64 *p = g.ops[pb[y][j].b].t + off;
            b0[y] = (double)p[0];
            b1[y] = (double)p[poly];
        }
#pragma unroll
        for (int x = 0; x < MM_TX; x++)
#pragma unroll
            for (int y = 0; y < MM_TY; y++) {
                d0[x][y] += ar.mulmod_np(a0[x], b0[y]);
                d1[x][y] += ar.mulmod_np(a0[x], b1[y]) + ar.mulmod_np(a1[x], b0[y]);
                d2[x][y] += ar.mulmod_np(a1[x], b1[y]);
            }
        if ((j & 3) == 3) {
#pragma unroll
            for (int x = 0; x < MM_TX; x++)
#pragma unroll
                for (int y = 0; y < MM_TY; y++) {
                    d0[x][y] = ar.mid(d0[x][y]);
                    d1[x][y] = ar.mid(d1[x][y]);
                    d2[x][y] = ar.mid(d2[x][y]);
                }
        }
    }
#pragma unroll
    for (int x = 0; x < MM_TX; x++)
#pragma unroll
        for (int y = 0; y < MM_TY; y++) {
            if (x0 + x >= g.grid_x || y0 + y >= g.grid_y) continue;
            u64 *out = g.ws_d + ((size_t)((x0 + x) * g.grid_y + y0 + y) * 3 * g.l1 + i) * N + idx;
            out[0] = ar.canon(d0[x][y]);
            out[poly] = ar.canon(d2[x][y]);
            out[2 * poly] = ar.canon(d1[x][y]);
        }
}

// grid (ceil(N/256), l1, n_out): ws_e[o][1][i] += ws_d[o][2][i]  (d1 joins the second polynomial)
__global__ __launch_bounds__(MM_THREADS) void k_mm_add_d1(MmGroup g, int N, const PrimeConst *pcs) {
    const int idx = blockIdx.x * MM_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int i = blockIdx.y, o = blockIdx.z;
    u64 *e = g.ws_e + ((size_t)o * 2 * g.l1 + g.l1 + i) * N + idx;
    *e = add_mod(*e, g.ws_d[((size_t)o * 3 * g.l1 + 2 * g.l1 + i) * N + idx], pcs[i].q);
}

// grid (ceil(N/256), 2*l1, n): a[c][poly][i] += b[c][poly][i] on batches with their own limb strides
__global__ __launch_bounds__(MM_THREADS) void k_ct_add(u64 *a, int stride_a, const u64 *b, int stride_b, int l1, int N, const PrimeConst *pcs) {
    const int idx = blockIdx.x * MM_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int y = blockIdx.y, p = y / l1, i = y - p * l1, c = blockIdx.z;
    u64 *x = a + ((size_t)c * 2 * stride_a + (size_t)p * stride_a + i) * N + idx;
    *x = add_mod(*x, b[((size_t)c * 2 * stride_b + (size_t)p * stride_b + i) * N + idx], pcs[i].q);
}

// grid (ceil(N/256), 2*limbs_out, n_out): the first limbs_out limbs of ws_e (limb stride l1) to the output ciphertexts
__global__ __launch_bounds__(MM_THREADS) void k_mm_scatter(MmGroup g, int N) {
    const int idx = blockIdx.x * MM_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int lo = g.limbs_out;
    const int y = blockIdx.y, c = y / lo, i = y - c * lo, o = blockIdx.z;
    g.out[(size_t)o * g.out_stride + ((size_t)c * g.limb_stride_out + i) * N + idx] = g.ws_e[((size_t)o * 2 * g.l1 + c * g.l1 + i) * N + idx];
}

static LimbMap mm_map(int l1) {
    LimbMap m;
    m.n = l1;
    for (int e = 0; e < ENSI_MAX_EXT; e++) m.prime[e] = e < l1 ? e : 0;
    return m;
}

// gather -> forward transform -> tensor multiply-add -> inverse transform: leaves (d0, d2, d1) of every output of
// the group in ws_d, coefficient form
void launch_mm_tensor(ensi_ctx *ctx, const MmGroup &g, hipStream_t st) {
    const int N = ctx->N, nb = (N + MM_THREADS - 1) / MM_THREADS;
    const LimbMap map = mm_map(g.l1);
    if (g.n_ops > 0) {
        if (ctx->log_n == 16) {
            // the forward column pass reads the operands where they lie
            launch_ntt16_gather(ctx, g.ws_a, g.ops, g.n_ops, g.l1, st);
        } else {
            {
                ScopedTimer t(ctx, "mm_gather", st);
                hipLaunchKernelGGL(k_mm_gather, dim3((unsigned)nb * g.n_ops, 2 * g.l1), dim3(MM_THREADS), 0, st, g, N, nb);
            }
            launch_ntt(ctx, g.ws_a, g.n_ops * 2 * g.l1, map, false, st);
        }
    }
    {
        ScopedTimer t(ctx, "mm_tensor_mac", st);
        if (g.grid_x > 0) {
            const int tiles = ((g.grid_x + MM_TX - 1) / MM_TX) * ((g.grid_y + MM_TY - 1) / MM_TY);
            hipLaunchKernelGGL(k_mm_grid_mac_fp, dim3(nb, g.l1, tiles), dim3(MM_THREADS), 0, st, g, N, ctx->d_pc);
        } else {
            hipLaunchKernelGGL(k_mm_tensor_mac, dim3(nb, g.l1, g.n_out), dim3(MM_THREADS), 0, st, g, N, ctx->d_pc);
        }
    }
    launch_ntt(ctx, g.ws_d, g.n_out * 3 * g.l1, map, true, st);
}

void launch_mm_add_d1(ensi_ctx *ctx, const MmGroup &g, hipStream_t st) {
    const int N = ctx->N, nb = (N + MM_THREADS - 1) / MM_THREADS;
    ScopedTimer t(ctx, "mm_add_d1", st);
    hipLaunchKernelGGL(k_mm_add_d1, dim3(nb, g.l1, g.n_out), dim3(MM_THREADS), 0, st, g, N, ctx->d_pc);
}

void launch_ct_add(ensi_ctx *ctx, u64 *a, int stride_a, const u64 *b, int stride_b, int l1, int n, hipStream_t st) {
    const int N = ctx->N, nb = (N + MM_THREADS - 1) / MM_THREADS;
    ScopedTimer t(ctx, "ct_add", st);
    hipLaunchKernelGGL(k_ct_add, dim3(nb, 2 * l1, n), dim3(MM_THREADS), 0, st, a, stride_a, b, stride_b, l1, N, ctx->d_pc);
}

void launch_mm_scatter(ensi_ctx *ctx, const MmGroup &g, hipStream_t st) {
    const int N = ctx->N, nb = (N + MM_THREADS - 1) / MM_THREADS;
    ScopedTimer t(ctx, "mm_scatter", st);
    hipLaunchKernelGGL(k_mm_scatter, dim3(nb, 2 * g.limbs_out, g.n_out), dim3(MM_THREADS), 0, st, g, N);
}
