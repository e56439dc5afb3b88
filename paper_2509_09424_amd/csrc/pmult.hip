// Plaintext multiplication (paper, Preliminaries: Multiplication, PMult) of many ciphertexts, summed per
// output and rescaled once:  out_o = Rescale( sum_{t in terms(o)} src_t (x) pt_t ).  This is the shape of the
// secure RoPE protocol (Alg. 2: three products per output) and of the mask-and-add merge of block-placed
// outputs (c_tot products per output).
//
// A product in R_Q is a pointwise product in the transform domain, so per output limb the work is: forward
// transform of every source limb, multiply by the (pre-transformed) plaintext limb and add, one inverse
// transform, then the rescale across limbs.  Two implementations:
//
//   generic  any ring size and prime: gather the sources, the library's transform, a Montgomery
//            multiply-add kernel, the inverse transform, the integer or fp64 rescale kernel, a strided copy.
//   pm16     N = 2^16 with ciphertext primes below 2^50, four kernels that keep every intermediate in the
//            layout and number format (exact integers in doubles) of the transform passes around it:
//              k_pm16_fcols            forward column pass of every source limb, read straight from the
//                                      source ciphertexts
//              k_pm16_frows_mac_irows  per output limb and 16-row tile: forward row pass of each term in
//                                      registers, multiply by the plaintext (stored in the register order
//                                      of that pass, so its loads are contiguous), accumulate, and run the
//                                      inverse row pass on the sum -- the products never reach memory
//              k_pm16_icols_last       inverse column pass of the limb the rescale drops, left as the
//                                      centred residue [c_l]
//              k_pm16_icols_rescale    inverse column pass of every other limb fused with
//                                      (c_i - [c_l]) q_l^{-1} mod q_i, written to the output ciphertext
// Both produce canonical residues and agree word for word.
#include "common.h"
#include "ntt16_core.h"

#define PM_THREADS 256
#define PM_N 65536
#ifndef PM_MAC_BLOCKS
#define PM_MAC_BLOCKS 2
#endif

__device__ __forceinline__ double pm_f64(u64 x) { return __longlong_as_double((long long)x); }
__device__ __forceinline__ u64 pm_u64(double x) { return (u64)__double_as_longlong(x); }

// ===================================================================== generic path
// grid (ceil(N/256), 2*l1, n_src): ws_a[slot][c*l1+i][N] <- limb i of component c of the group's distinct source `slot`
__global__ __launch_bounds__(PM_THREADS) void k_pm_gather(PmGroup g, int N) {
    const int idx = blockIdx.x * PM_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int y = blockIdx.y, c = y / g.l1, i = y - c * g.l1, t = blockIdx.z;
    const u64 *src = g.terms[g.owner[t]].src + ((size_t)c * g.limb_stride_in + i) * N;
    g.ws_a[((size_t)t * 2 * g.l1 + y) * N + idx] = src[idx];
}

// grid (ceil(N/256), 2*l1, n_out): ws_b[o][y][N] <- sum_t ws_a[t][y] * pt[t][i]  (transform domain)
__global__ __launch_bounds__(PM_THREADS) void k_pm_mac(PmGroup g, int N, const PrimeConst *pcs) {
    const int idx = blockIdx.x * PM_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int y = blockIdx.y, i = y % g.l1, o = blockIdx.z;
    const u64 q = pcs[i].q, qn = pcs[i].qneg_inv;
    const int t0 = g.begin[o], t1 = g.begin[o + 1];
    u64 acc = 0;
    for (int t = t0; t < t1; t++) {
        const u64 a = g.ws_a[((size_t)g.terms[t].slot * 2 * g.l1 + y) * N + idx];
        const u64 b = g.pt[((size_t)g.terms[t].pt * g.pt_limbs + i) * N + idx];
        acc = add_mod(acc, mont_mul(a, b, q, qn), q);
    }
    g.ws_b[((size_t)o * 2 * g.l1 + y) * N + idx] = acc;
}

// grid (ceil(N/256), 2*(l1-1), n_out): the rescaled limbs of ws_b (limb stride l1) to the output ciphertexts
__global__ __launch_bounds__(PM_THREADS) void k_pm_scatter(PmGroup g, int N) {
    const int idx = blockIdx.x * PM_THREADS + threadIdx.x;
    if (idx >= N) return;
    const int lo = g.l1 - 1;
    const int y = blockIdx.y, c = y / lo, i = y - c * lo, o = blockIdx.z;
    g.out[(size_t)o * g.out_stride + ((size_t)c * g.limb_stride_out + i) * N + idx] = g.ws_b[((size_t)o * 2 * g.l1 + c * g.l1 + i) * N + idx];
}

static LimbMap pm_map(int l1) {
    LimbMap m;
    m.n = l1;
    for (int e = 0; e < ENSI_MAX_EXT; e++) m.prime[e] = e < l1 ? e : 0;
    return m;
}

// d_consts / d_fconsts: the rescale constants with the scalar set to one
void launch_pm_generic(ensi_ctx *ctx, const PmGroup &g, const u64 *d_consts, const double *d_fconsts, hipStream_t st) {
    const int N = ctx->N, nb = (N + PM_THREADS - 1) / PM_THREADS;
    const LimbMap map = pm_map(g.l1);
    if (g.n_src > 0) {
        ScopedTimer t(ctx, "pm_gather", st);
        hipLaunchKernelGGL(k_pm_gather, dim3(nb, 2 * g.l1, g.n_src), dim3(PM_THREADS), 0, st, g, N);
    }
    if (g.n_src > 0) launch_ntt(ctx, g.ws_a, g.n_src * 2 * g.l1, map, false, st);
    {
        ScopedTimer t(ctx, "pm_mac", st);
        hipLaunchKernelGGL(k_pm_mac, dim3(nb, 2 * g.l1, g.n_out), dim3(PM_THREADS), 0, st, g, N, ctx->d_pc);
    }
    launch_ntt(ctx, g.ws_b, g.n_out * 2 * g.l1, map, true, st);
    launch_rescale(ctx, g.ws_b, g.n_out, g.l1, g.l1, d_consts, d_fconsts, st);
    {
        ScopedTimer t(ctx, "pm_scatter", st);
        hipLaunchKernelGGL(k_pm_scatter, dim3(nb, 2 * (g.l1 - 1), g.n_out), dim3(PM_THREADS), 0, st, g, N);
    }
}

// ===================================================================== N = 2^16, fp64 arithmetic
// Plaintext in the order the row pass holds it: within the 16-row tile b, thread (rho, j) = tid owns, as its
// i-th value, position 16 j + i of row rho; that value is stored at b*4096 + i*256 + tid, as a double.
// grid (16, n_rows)
__global__ __launch_bounds__(PM_THREADS) void k_pm16_pt_format(const u64 *in, u64 *out) {
    const int tid = threadIdx.x, rho = tid >> 4, j = tid & 15;
    const size_t base = (size_t)blockIdx.y * PM_N + (size_t)blockIdx.x * 4096;
#pragma unroll
    for (int i = 0; i < 16; i++) out[base + i * 256 + tid] = pm_u64((double)in[base + rho * 256 + 16 * j + i]);
}
void launch_pm16_pt_format(ensi_ctx *ctx, const u64 *ntt_form, int n_rows, u64 *out, hipStream_t st) {
    (void)ctx;
    hipLaunchKernelGGL(k_pm16_pt_format, dim3(16, n_rows), dim3(PM_THREADS), 0, st, ntt_form, out);
}

// grid (16, 2*l1, n_src)
__global__ __launch_bounds__(PM_THREADS) void k_pm16_fcols(PmGroup g, const PrimeConst *pcs, const u64 *tw_all) {
    __shared__ u64 lds[4096];
    const int tid = threadIdx.x, c16 = tid & 15, jj = tid >> 4;
    const int y = blockIdx.y, c = y / g.l1, i = y - c * g.l1, t = blockIdx.z;
    const size_t col = (size_t)blockIdx.x * 16 + c16;
    const u64 *src = g.terms[g.owner[t]].src + ((size_t)c * g.limb_stride_in + i) * PM_N + col;
    u64 *out = g.ws_a + ((size_t)t * 2 * g.l1 + y) * PM_N + col;
    ArithFp ar;
    ar.init(pcs[i]);
    const u64 *tw = tw_all + (size_t)i * 4 * PM_N;
    double v[16];
#pragma unroll
    for (int k = 0; k < 16; k++) v[k] = (double)src[(size_t)(jj + 16 * k) * 256];
    cols_fwd_regs(ar, v, tw, tw + PM_N, lds, c16, jj);
#pragma unroll
    for (int k = 0; k < 16; k++) out[(size_t)(16 * jj + k) * 256] = pm_u64(ar.mid(v[k]));
}

// Four Cooley-Tukey stages like ct4, with the 15 twiddles (value, companion) of the step read from a table in LDS:
// entry (1 << k) - 1 + g serves stage k, butterfly group g.
__device__ __forceinline__ void pm_ct4_tab(const ArithFp &ar, double *v, const ulonglong2 *tab) {
#pragma unroll
    for (int k = 0; k < 4; k++) {
        const int d = 8 >> k;
#pragma unroll
        for (int gq = 0; gq < (1 << k); gq++) {
            const ulonglong2 w = tab[(1 << k) - 1 + gq];
#pragma unroll
            for (int o = 0; o < d; o++) {
                const int i0 = gq * 2 * d + o;
                ar.ct(v[i0], v[i0 + d], w.x, w.y);
            }
        }
    }
}

// grid (16 * 2*l1 * n_out).  The operand of the next term is fetched while the current forward pass runs.  The
// twiddles of a pass's first step depend on the row only and sit in LDS (the 16 threads of a row read the same
// word); those of the second step differ per thread and stay in registers across all terms.
__global__ __launch_bounds__(PM_THREADS, PM_MAC_BLOCKS) void k_pm16_frows_mac_irows(PmGroup g, const PrimeConst *pcs, const u64 *tw_all) {
    __shared__ u64 lds[4096 + 256];
    __shared__ ulonglong2 tw1[16 * 16];
    const int tid = threadIdx.x, rho = tid >> 4, j = tid & 15;
    // Workgroups are dealt to the eight XCDs in turn.  The two polynomials of an output tile multiply by the same
    // plaintext tile, so their blocks are made consecutive on one XCD (ids n and n + 8) and the second read of
    // the tile is served by that XCD's L2.
    const u32 id = blockIdx.x, q = (id >> 4) * 8 + (id & 7);
    const int cpoly = (id >> 3) & 1, tile = q & 15, i = (q >> 4) % g.l1, o = (q >> 4) / g.l1;
    const int y = cpoly * g.l1 + i;
    const int r0 = tile * 16;
    ArithFp ar;
    ar.init(pcs[i]);
    const u64 *twf = tw_all + (size_t)i * 4 * PM_N, *twi = twf + 2 * PM_N;
    const u32 r = (u32)(r0 + rho);
    if (j < 15) {
        const int k = 31 - __clz(j + 1), gq = j + 1 - (1 << k);
        const u32 idx = ((256u + r) << k) + gq;
        tw1[rho * 16 + j] = make_ulonglong2(twf[idx], twf[PM_N + idx]);
    }
    const ulonglong2 *tab = tw1 + rho * 16;
    const int t0 = g.begin[o], t1 = g.begin[o + 1];
    double acc[16], nv[16];
#pragma unroll
    for (int k = 0; k < 16; k++) acc[k] = 0.0;
    const size_t term = (size_t)2 * g.l1 * PM_N;  // words per term in ws_a
    const size_t a_off = (size_t)y * PM_N + (size_t)r0 * 256 + rho * 256 + j;
    const size_t b_off = (size_t)i * PM_N + (size_t)tile * 4096 + tid;
    if (t0 < t1) {
        const u64 *a = g.ws_a + (size_t)g.terms[t0].slot * term + a_off;
#pragma unroll
        for (int k = 0; k < 16; k++) nv[k] = pm_f64(a[16 * k]);
    }
    double *l = (double *)lds;
    __syncthreads();
#pragma unroll 1
    for (int t = t0; t < t1; t++) {
        const u64 *b = g.pt + (size_t)g.terms[t].pt * g.pt_limbs * PM_N + b_off;
        double v[16], w[16];
#pragma unroll
        for (int k = 0; k < 16; k++) w[k] = pm_f64(b[256 * k]);
#pragma unroll
        for (int k = 0; k < 16; k++) v[k] = nv[k];
        if (t + 1 < t1) {
            const u64 *a = g.ws_a + (size_t)g.terms[t + 1].slot * term + a_off;
#pragma unroll
            for (int k = 0; k < 16; k++) nv[k] = pm_f64(a[16 * k]);
        }
        // forward row pass (the steps of rows_fwd_regs)
        pm_ct4_tab(ar, v, tab);
#pragma unroll
        for (int k = 0; k < 16; k++) l[rpad(rho * 256 + j + 16 * k)] = ar.mid(v[k]);
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; k++) v[k] = l[rpad(rho * 256 + 16 * j + k)];
        ct4(ar, v, twf, twf + PM_N, (256u + r) * 16u + j);
#pragma unroll
        for (int k = 0; k < 16; k++) acc[k] += ar.mulmod_np(ar.mid(v[k]), w[k]);
        // a product is below 0.7 q in magnitude: eight of them stay exact in a double
        if (((t - t0) & 7) == 7) {
#pragma unroll
            for (int k = 0; k < 16; k++) acc[k] = ar.mid(acc[k]);
        }
        __syncthreads();  // the tile is reused by the next exchange
    }
    double v[16];
#pragma unroll
    for (int k = 0; k < 16; k++) v[k] = ar.mid(acc[k]);
    rows_inv_regs(ar, v, twi, twi + PM_N, lds, rho, j, r);
    u64 *out = g.ws_b + (size_t)o * term + a_off;
#pragma unroll
    for (int k = 0; k < 16; k++) out[16 * k] = pm_u64(ar.mid(v[k]));
}

// grid (16, 2, n_out): ws_last[o][c][N] <- centred residue of limb l1-1 (coefficient form)
__global__ __launch_bounds__(PM_THREADS) void k_pm16_icols_last(PmGroup g, const PrimeConst *pcs, const u64 *tw_all) {
    __shared__ u64 lds[4096];
    const int tid = threadIdx.x, c16 = tid & 15, jj = tid >> 4;
    const int c = blockIdx.y, o = blockIdx.z, i = g.l1 - 1;
    const size_t col = (size_t)blockIdx.x * 16 + c16;
    const u64 *src = g.ws_b + ((size_t)o * 2 * g.l1 + c * g.l1 + i) * PM_N + col;
    u64 *dst = g.ws_last + ((size_t)o * 2 + c) * PM_N + col;
    ArithFp ar;
    ar.init(pcs[i]);
    const u64 *tw = tw_all + (size_t)i * 4 * PM_N + 2 * PM_N;
    double v[16];
#pragma unroll
    for (int k = 0; k < 16; k++) v[k] = pm_f64(src[(size_t)(16 * jj + k) * 256]);
    cols_inv_regs(ar, v, tw, tw + PM_N, lds, c16, jj);
#pragma unroll
    for (int k = 0; k < 16; k++) dst[(size_t)(jj + 16 * k) * 256] = pm_u64(ar.mid(ar.mulmod(ar.mid(v[k]), ar.ninv, ar.ninv_p)));
}

// grid (16, 2*(l1-1), n_out)
__global__ __launch_bounds__(PM_THREADS) void k_pm16_icols_rescale(PmGroup g, PmRescale rs, const PrimeConst *pcs, const u64 *tw_all) {
    __shared__ u64 lds[4096];
    const int tid = threadIdx.x, c16 = tid & 15, jj = tid >> 4;
    const int lo = g.l1 - 1;
    const int y = blockIdx.y, c = y / lo, i = y - c * lo, o = blockIdx.z;
    const size_t col = (size_t)blockIdx.x * 16 + c16;
    const u64 *src = g.ws_b + ((size_t)o * 2 * g.l1 + c * g.l1 + i) * PM_N + col;
    const u64 *last = g.ws_last + ((size_t)o * 2 + c) * PM_N + col;
    u64 *dst = g.out + (size_t)o * g.out_stride + ((size_t)c * g.limb_stride_out + i) * PM_N + col;
    ArithFp ar;
    ar.init(pcs[i]);
    const u64 *tw = tw_all + (size_t)i * 4 * PM_N + 2 * PM_N;
    const double w = rs.w[i], wp = rs.wp[i];
    double v[16], tl[16];
#pragma unroll
    for (int k = 0; k < 16; k++) v[k] = pm_f64(src[(size_t)(16 * jj + k) * 256]);
#pragma unroll
    for (int k = 0; k < 16; k++) tl[k] = pm_f64(last[(size_t)(jj + 16 * k) * 256]);
    cols_inv_regs(ar, v, tw, tw + PM_N, lds, c16, jj);
#pragma unroll
    for (int k = 0; k < 16; k++) {
        const double x = ar.mid(ar.mulmod(ar.mid(v[k]), ar.ninv, ar.ninv_p));
        const double z = ar.mid(x - ar.mid(tl[k]));
        dst[(size_t)(jj + 16 * k) * 256] = ar.canon(ar.mulmod(z, w, wp));
    }
}

void launch_pm16(ensi_ctx *ctx, const PmGroup &g, const PmRescale &rs, hipStream_t st) {
    if (g.n_src > 0) {
        ScopedTimer t(ctx, "pm_fcols", st);
        hipLaunchKernelGGL(k_pm16_fcols, dim3(16, 2 * g.l1, g.n_src), dim3(PM_THREADS), 0, st, g, ctx->d_pc, ctx->d_tw);
    }
    {
        ScopedTimer t(ctx, "pm_frows_mac_irows", st);
        hipLaunchKernelGGL(k_pm16_frows_mac_irows, dim3(16 * 2 * g.l1 * g.n_out), dim3(PM_THREADS), 0, st, g, ctx->d_pc, ctx->d_tw);
    }
    {
        ScopedTimer t(ctx, "pm_icols_last", st);
        hipLaunchKernelGGL(k_pm16_icols_last, dim3(16, 2, g.n_out), dim3(PM_THREADS), 0, st, g, ctx->d_pc, ctx->d_tw);
    }
    {
        ScopedTimer t(ctx, "pm_icols_rescale", st);
        hipLaunchKernelGGL(k_pm16_icols_rescale, dim3(16, 2 * (g.l1 - 1), g.n_out), dim3(PM_THREADS), 0, st, g, rs, ctx->d_pc, ctx->d_tw);
    }
}
