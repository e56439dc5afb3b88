// Negacyclic number-theoretic transform over word primes, batched over limb rows.
//
// The paper leaves the transform to its CKKS library; it is the ring product
// of R_Q = Z_Q[X]/(X^N+1) (Preliminaries, RNS-CKKS) evaluated limb by limb.
//
// A limb of N = N1*N2 coefficients is viewed as an N1 x N2 matrix (row-major).
// The forward transform (Cooley-Tukey, twiddles psi^bitrev(k), natural order in,
// bit-reversed order out) runs its first log N1 stages down the columns and the
// remaining log N2 stages inside rows; the inverse (Gentleman-Sande) undoes them
// in the opposite order.  Each pass stages a 4096-word tile in LDS, so a limb
// makes two round trips through HBM per transform.  Position k of the forward
// output holds the evaluation at psi^(2*bitrev(k)+1).
//
// Butterflies keep values lazily in [0,4q) (forward) / [0,2q) (inverse); the
// last pass of either direction writes canonical residues.
#include <algorithm>

#include "common.h"

#define NTT_TILE_LOG 12
#define NTT_TILE (1 << NTT_TILE_LOG)
#define NTT_THREADS 256

struct NttGeom {
    int log_n, log_n1, log_n2;
    int log_c;  // columns per tile in the column pass
    int log_r;  // rows per tile in the row pass
};

static NttGeom ntt_geom(int log_n) {
    NttGeom g;
    g.log_n = log_n;
    g.log_n2 = log_n / 2;
    g.log_n1 = log_n - g.log_n2;
    int tile = log_n < NTT_TILE_LOG ? log_n : NTT_TILE_LOG;
    g.log_c = tile - g.log_n1;
    g.log_r = tile - g.log_n2;
    return g;
}

// Column pass: all N1 rows x C columns.  FWD: stages 0..log_n1-1 (forward
// direction); otherwise the same stages in reverse with inverse butterflies and
// the final 1/N scaling.
template <bool FWD>
__global__ __launch_bounds__(NTT_THREADS) void k_ntt_cols(u64 *data, const u64 *tw_all, const PrimeConst *pc, LimbMap map,
                                                          NttGeom g) {
    __shared__ u64 lds[NTT_TILE];
    const int tid = threadIdx.x;
    const int inst = blockIdx.y;
    const int prime = map.prime[inst % map.n];
    const size_t N = (size_t)1 << g.log_n;
    const int N1 = 1 << g.log_n1, N2 = 1 << g.log_n2, C = 1 << g.log_c;
    const u64 q = pc[prime].q, two_q = 2 * q;
    const u64 *tw = tw_all + (size_t)prime * 4 * N + (FWD ? 0 : 2 * N);
    const u64 *tws = tw + N;
    u64 *base = data + (size_t)inst * N + (size_t)blockIdx.x * C;
    const int tile = N1 * C;

    for (int e = tid; e < tile; e += NTT_THREADS) lds[e] = base[(size_t)(e >> g.log_c) * N2 + (e & (C - 1))];
    __syncthreads();

    if (FWD) {
        for (int s = 0; s < g.log_n1; s++) {
            const int log_t = g.log_n1 - 1 - s;  // rows between butterfly partners = 2^log_t
            for (int b = tid; b < tile / 2; b += NTT_THREADS) {
                int c = b & (C - 1), rb = b >> g.log_c;
                int i = rb >> log_t, k = rb & ((1 << log_t) - 1);
                int i0 = ((((i << 1) << log_t) + k) << g.log_c) + c;
                int i1 = i0 + (1 << (log_t + g.log_c));
                u64 w = tw[(1 << s) + i], ws = tws[(1 << s) + i];
                u64 X = csub(lds[i0], two_q);
                u64 T = mul_shoup_lazy(lds[i1], w, ws, q);
                lds[i0] = X + T;
                lds[i1] = X - T + two_q;
            }
            __syncthreads();
        }
        for (int e = tid; e < tile; e += NTT_THREADS) base[(size_t)(e >> g.log_c) * N2 + (e & (C - 1))] = lds[e];
    } else {
        for (int s = g.log_n1 - 1; s >= 0; s--) {
            const int log_t = g.log_n1 - 1 - s;
            for (int b = tid; b < tile / 2; b += NTT_THREADS) {
                int c = b & (C - 1), rb = b >> g.log_c;
                int i = rb >> log_t, k = rb & ((1 << log_t) - 1);
                int i0 = ((((i << 1) << log_t) + k) << g.log_c) + c;
                int i1 = i0 + (1 << (log_t + g.log_c));
                u64 w = tw[(1 << s) + i], ws = tws[(1 << s) + i];
                u64 U = lds[i0], V = lds[i1];
                lds[i0] = csub(U + V, two_q);
                lds[i1] = mul_shoup_lazy(U - V + two_q, w, ws, q);
            }
            __syncthreads();
        }
        const u64 ni = pc[prime].n_inv, nis = pc[prime].n_inv_s;
        for (int e = tid; e < tile; e += NTT_THREADS)
            base[(size_t)(e >> g.log_c) * N2 + (e & (C - 1))] = mul_shoup(lds[e], ni, nis, q);
    }
}

// Row pass: R whole rows (contiguous R*N2 words).  FWD: stages log_n1..log_n-1
// and the final reduction to [0,q); otherwise the first log_n2 inverse stages.
template <bool FWD>
__global__ __launch_bounds__(NTT_THREADS) void k_ntt_rows(u64 *data, const u64 *tw_all, const PrimeConst *pc, LimbMap map,
                                                          NttGeom g) {
    __shared__ u64 lds[NTT_TILE];
    const int tid = threadIdx.x;
    const int inst = blockIdx.y;
    const int prime = map.prime[inst % map.n];
    const size_t N = (size_t)1 << g.log_n;
    const int N1 = 1 << g.log_n1, N2 = 1 << g.log_n2, R = 1 << g.log_r;
    const u64 q = pc[prime].q, two_q = 2 * q;
    const u64 *tw = tw_all + (size_t)prime * 4 * N + (FWD ? 0 : 2 * N);
    const u64 *tws = tw + N;
    const int r0 = blockIdx.x * R;
    u64 *base = data + (size_t)inst * N + (size_t)r0 * N2;
    const int tile = R * N2;

    for (int e = tid; e < tile; e += NTT_THREADS) lds[e] = base[e];
    __syncthreads();

    if (FWD) {
        for (int s = 0; s < g.log_n2; s++) {
            const int log_t = g.log_n2 - 1 - s;
            for (int b = tid; b < tile / 2; b += NTT_THREADS) {
                int row = b >> (g.log_n2 - 1), bb = b & ((N2 >> 1) - 1);
                int i = bb >> log_t, k = bb & ((1 << log_t) - 1);
                int i0 = (row << g.log_n2) + ((i << 1) << log_t) + k;
                int i1 = i0 + (1 << log_t);
                int ti = ((N1 + r0 + row) << s) + i;
                u64 w = tw[ti], ws = tws[ti];
                u64 X = csub(lds[i0], two_q);
                u64 T = mul_shoup_lazy(lds[i1], w, ws, q);
                lds[i0] = X + T;
                lds[i1] = X - T + two_q;
            }
            __syncthreads();
        }
        for (int e = tid; e < tile; e += NTT_THREADS) base[e] = csub(csub(lds[e], two_q), q);
    } else {
        for (int s = g.log_n2 - 1; s >= 0; s--) {
            const int log_t = g.log_n2 - 1 - s;
            for (int b = tid; b < tile / 2; b += NTT_THREADS) {
                int row = b >> (g.log_n2 - 1), bb = b & ((N2 >> 1) - 1);
                int i = bb >> log_t, k = bb & ((1 << log_t) - 1);
                int i0 = (row << g.log_n2) + ((i << 1) << log_t) + k;
                int i1 = i0 + (1 << log_t);
                int ti = ((N1 + r0 + row) << s) + i;
                u64 w = tw[ti], ws = tws[ti];
                u64 U = lds[i0], V = lds[i1];
                lds[i0] = csub(U + V, two_q);
                lds[i1] = mul_shoup_lazy(U - V + two_q, w, ws, q);
            }
            __syncthreads();
        }
        for (int e = tid; e < tile; e += NTT_THREADS) base[e] = lds[e];
    }
}

static void launch_ntt_chunk(ensi_ctx *ctx, u64 *data, int n_inst, const LimbMap &map, bool inverse, hipStream_t st) {
    NttGeom g = ntt_geom(ctx->log_n);
    dim3 grid_c(1u << (g.log_n2 - g.log_c), n_inst), grid_r(1u << (g.log_n1 - g.log_r), n_inst);
    if (!inverse) {
        {
            ScopedTimer t(ctx, "ntt_fwd_cols", st);
            hipLaunchKernelGGL(k_ntt_cols<true>, grid_c, dim3(NTT_THREADS), 0, st, data, ctx->d_tw, ctx->d_pc, map, g);
        }
        {
            ScopedTimer t(ctx, "ntt_fwd_rows", st);
            hipLaunchKernelGGL(k_ntt_rows<true>, grid_r, dim3(NTT_THREADS), 0, st, data, ctx->d_tw, ctx->d_pc, map, g);
        }
    } else {
        {
            ScopedTimer t(ctx, "ntt_inv_rows", st);
            hipLaunchKernelGGL(k_ntt_rows<false>, grid_r, dim3(NTT_THREADS), 0, st, data, ctx->d_tw, ctx->d_pc, map, g);
        }
        {
            ScopedTimer t(ctx, "ntt_inv_cols", st);
            hipLaunchKernelGGL(k_ntt_cols<false>, grid_c, dim3(NTT_THREADS), 0, st, data, ctx->d_tw, ctx->d_pc, map, g);
        }
    }
}

// Rows beyond the grid's y limit are transformed in several launches, each a whole
// number of periods of the prime map.
void launch_ntt(ensi_ctx *ctx, u64 *data, int n_inst, const LimbMap &map, bool inverse, hipStream_t st) {
    if (ctx->log_n == 16) {
        launch_ntt16(ctx, data, n_inst, map, inverse, st);
        return;
    }
    const int max_rows = (32768 / map.n) * map.n;
    for (int done = 0; done < n_inst; done += max_rows)
        launch_ntt_chunk(ctx, data + (size_t)done * ctx->N, std::min(max_rows, n_inst - done), map, inverse, st);
}
