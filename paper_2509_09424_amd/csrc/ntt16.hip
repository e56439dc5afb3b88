// Negacyclic NTT for N = 2^16: two passes of 256-point transforms, each done as two
// radix-16 steps held in registers with one exchange through LDS in between.
//
// Same transform, stage order, twiddle tables (psi^bitrev(k)) and output order as the
// generic kernels in ntt.hip: the 16 stages of the Cooley-Tukey network (Gentleman-
// Sande for the inverse) are cut 4 + 4 | 4 + 4.  Viewing a limb as 256 x 256 (row-
// major), the column pass covers the stages whose butterflies span rows and the row
// pass those inside a row.  In a 4-stage step a thread owns 16 elements whose
// indices differ in the 4 bits the step works on; the twiddle of local stage k and
// local butterfly group g is table[(Mbase << k) + g] with
//   Mbase = 1 | 16 + j | 256 + r | (256 + r) * 16 + j
// for column step 1 | column step 2 | row step 1 | row step 2 (j: the thread's slot
// of 16, r: the row).
//
// Arithmetic.  64-bit integer multiplies are a quarter-rate, multi-instruction affair
// on this chip while fp64 FMAs run at full rate, so limbs whose prime is below 2^50
// are transformed in fp64: residues are held as exact integers in doubles and a
// product x*w mod p is  h = x*w; l = fma(x,w,-h); q = rint(x*(w/p)); r = fma(-q,p,h)+l
// (exact: h - q*p and l are integers below 2^53).  Values are kept lazily within
// +-8p and brought back with x - rint(x/p)*p between steps.  The special primes
// (60 bits) use the integer Shoup/Harvey butterflies.  Both produce canonical
// residues, so results are bit-identical to the generic kernels.
#include <algorithm>

#include "common.h"
#include "ntt16_core.h"

#define N16_THREADS 256
#define N16_LOG 16

// ---- column pass: tile = 256 rows x 16 columns; thread (c = tid%16, j = tid/16)
// gin: where the forward pass reads its tile (the same place as g for a transform in place)
template <bool FWD, class A>
__device__ __forceinline__ void cols_body(u64 *g, const u64 *gin, const u64 *tw, const u64 *tws, const PrimeConst &pc, u64 *lds) {
    A ar;
    ar.init(pc);
    const int tid = threadIdx.x, c = tid & 15, j = tid >> 4;
    typename A::T v[16];
    if (FWD) {
#pragma unroll
        for (int i = 0; i < 16; i++) v[i] = ar.load(gin[(size_t)(j + 16 * i) * 256 + c]);
        ct4(ar, v, tw, tws, 1u);
#pragma unroll
        for (int i = 0; i < 16; i++) ((typename A::T *)lds)[(j + 16 * i) * 16 + c] = ar.mid(v[i]);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 16; i++) v[i] = ((typename A::T *)lds)[(16 * j + i) * 16 + c];
        ct4(ar, v, tw, tws, 16u + j);
#pragma unroll
        for (int i = 0; i < 16; i++) g[(size_t)(16 * j + i) * 256 + c] = ar.store_fwd(v[i]);
    } else {
#pragma unroll
        for (int i = 0; i < 16; i++) v[i] = ar.center(ar.load(g[(size_t)(16 * j + i) * 256 + c]));
        gs4(ar, v, tw, tws, 16u + j);
#pragma unroll
        for (int i = 0; i < 16; i++) ((typename A::T *)lds)[(16 * j + i) * 16 + c] = ar.mid(v[i]);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 16; i++) v[i] = ((typename A::T *)lds)[(j + 16 * i) * 16 + c];
        gs4(ar, v, tw, tws, 1u);
#pragma unroll
        for (int i = 0; i < 16; i++) g[(size_t)(j + 16 * i) * 256 + c] = ar.store_inv_scaled(v[i]);
    }
}

// ---- row pass: tile = 16 contiguous rows; thread (rho = tid/16, j = tid%16).  LDS positions are
// padded by one word per 16 so that both the strided and the contiguous 16-element patterns are
// conflict-free; global traffic is fully coalesced (the contiguous-per-thread layout only ever
// touches LDS).
// A block runs its tile for up to N16_ROWS_GROUP limbs of the same prime (n_here of them, inst_stride words apart):
// the tile's twiddles -- 15 pairs per row for one step, 15 pairs per thread for the other, more bytes than the tile
// itself -- are fetched once (LDS and registers), and the next limb's tile is requested before the current one is
// transformed.
#define N16_ROWS_GROUP 8

template <bool FWD, class A>
__device__ __forceinline__ void rows_body(u64 *g, size_t inst_stride, int n_here, const u64 *tw, const u64 *tws, const PrimeConst &pc, u64 *lds,
                                          ulonglong2 *tw1, int r0) {
    A ar;
    ar.init(pc);
    const int tid = threadIdx.x, rho = tid >> 4, j = tid & 15;
    const u32 r = (u32)(r0 + rho);
    typename A::T v[16];
    typename A::T *l = (typename A::T *)lds;
    row_table_to_lds(tw1, tw, tws, 256u + r, rho, j);
    TwRegs tw2;
    tw2.load(tw, tws, (256u + r) * 16u + j);
    const ulonglong2 *tab = tw1 + rho * 16;
    u64 nv[16];
    if (FWD) {
#pragma unroll
        for (int i = 0; i < 16; i++) nv[i] = g[rho * 256 + j + 16 * i];
        __syncthreads();  // tw1 is complete
#pragma unroll 1
        for (int c = 0; c < n_here; c++) {
#pragma unroll
            for (int i = 0; i < 16; i++) v[i] = ar.load(nv[i]);
            if (c + 1 < n_here) {
                const u64 *gn = g + (size_t)(c + 1) * inst_stride;
#pragma unroll
                for (int i = 0; i < 16; i++) nv[i] = gn[rho * 256 + j + 16 * i];
            }
            ct4_tab(ar, v, tab);
#pragma unroll
            for (int i = 0; i < 16; i++) l[rpad(rho * 256 + j + 16 * i)] = ar.mid(v[i]);
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 16; i++) v[i] = l[rpad(rho * 256 + 16 * j + i)];
            ct4_tab(ar, v, tw2);
#pragma unroll
            for (int i = 0; i < 16; i++) lds[rpad(rho * 256 + 16 * j + i)] = ar.store_fwd(v[i]);
            __syncthreads();
            u64 *go = g + (size_t)c * inst_stride;
#pragma unroll
            for (int i = 0; i < 16; i++) go[tid + 256 * i] = lds[rpad(tid + 256 * i)];
            __syncthreads();  // the tile is reused by the next limb's exchange
        }
    } else {
#pragma unroll
        for (int i = 0; i < 16; i++) nv[i] = g[tid + 256 * i];
#pragma unroll 1
        for (int c = 0; c < n_here; c++) {
#pragma unroll
            for (int i = 0; i < 16; i++) lds[rpad(tid + 256 * i)] = nv[i];
            __syncthreads();  // (also covers tw1 on the first round)
            if (c + 1 < n_here) {
                const u64 *gn = g + (size_t)(c + 1) * inst_stride;
#pragma unroll
                for (int i = 0; i < 16; i++) nv[i] = gn[tid + 256 * i];
            }
#pragma unroll
            for (int i = 0; i < 16; i++) v[i] = ar.center(ar.load(lds[rpad(rho * 256 + 16 * j + i)]));
            gs4_tab(ar, v, tw2);
#pragma unroll
            for (int i = 0; i < 16; i++) l[rpad(rho * 256 + 16 * j + i)] = ar.mid(v[i]);
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 16; i++) v[i] = l[rpad(rho * 256 + j + 16 * i)];
            gs4_tab(ar, v, tab);
            u64 *go = g + (size_t)c * inst_stride;
#pragma unroll
            for (int i = 0; i < 16; i++) go[rho * 256 + j + 16 * i] = ar.store_inv(v[i]);
            __syncthreads();  // the tile is reused by the next limb's staging
        }
    }
}

template <bool FWD>
__global__ __launch_bounds__(N16_THREADS) void k_ntt16_cols(u64 *data, const u64 *tw_all, const PrimeConst *pcs, LimbMap map) {
    __shared__ u64 lds[4096];
    const int inst = blockIdx.y;
    const int prime = map.prime[inst % map.n];
    const PrimeConst pc = pcs[prime];
    const size_t N = (size_t)1 << N16_LOG;
    const u64 *tw = tw_all + (size_t)prime * 4 * N + (FWD ? 0 : 2 * N);
    u64 *g = data + (size_t)inst * N + (size_t)blockIdx.x * 16;
    if (pc.pad[0]) cols_body<FWD, ArithFp>(g, g, tw, tw + N, pc, lds);
    else cols_body<FWD, ArithInt>(g, g, tw, tw + N, pc, lds);
}

// Forward column pass that reads every limb from its operand ciphertext and writes the operand array of the
// ciphertext products: row inst = (operand u, polynomial p, limb i) of data <- ops[u].p[p][i], column-transformed.
// l1 limbs per polynomial, limb i under prime i.
__global__ __launch_bounds__(N16_THREADS) void k_ntt16_cols_gather(u64 *data, const MmOperand *ops, int l1, const u64 *tw_all,
                                                                    const PrimeConst *pcs) {
    __shared__ u64 lds[4096];
    const int inst = blockIdx.y;
    const int u = inst / (2 * l1), y = inst - u * 2 * l1, p = y / l1, prime = y - p * l1;
    const PrimeConst pc = pcs[prime];
    const size_t N = (size_t)1 << N16_LOG;
    const u64 *tw = tw_all + (size_t)prime * 4 * N;
    const MmOperand op = ops[u];
    const u64 *gin = op.p + ((size_t)p * op.limb_stride + prime) * N + (size_t)blockIdx.x * 16;
    u64 *g = data + (size_t)inst * N + (size_t)blockIdx.x * 16;
    if (pc.pad[0]) cols_body<true, ArithFp>(g, gin, tw, tw + N, pc, lds);
    else cols_body<true, ArithInt>(g, gin, tw, tw + N, pc, lds);
}

// grid (16, map.n * n_groups): instance inst = slot + map.n * (N16_ROWS_GROUP * group + c), c < N16_ROWS_GROUP, lies under
// prime map.prime[slot]; n_inst instances in all.
template <bool FWD>
__global__ __launch_bounds__(N16_THREADS, 2) void k_ntt16_rows(u64 *data, const u64 *tw_all, const PrimeConst *pcs, LimbMap map, int n_inst) {
    __shared__ u64 lds[4096 + 256];
    __shared__ ulonglong2 tw1[16 * 16];
    const int slot = blockIdx.y % map.n, group = blockIdx.y / map.n;
    const int inst0 = slot + map.n * N16_ROWS_GROUP * group;
    if (inst0 >= n_inst) return;
    const int n_here = min(N16_ROWS_GROUP, (n_inst - inst0 + map.n - 1) / map.n);
    const int prime = map.prime[slot];
    const PrimeConst pc = pcs[prime];
    const size_t N = (size_t)1 << N16_LOG;
    const u64 *tw = tw_all + (size_t)prime * 4 * N + (FWD ? 0 : 2 * N);
    const int r0 = blockIdx.x * 16;
    u64 *g = data + (size_t)inst0 * N + (size_t)r0 * 256;
    if (pc.pad[0]) rows_body<FWD, ArithFp>(g, (size_t)map.n * N, n_here, tw, tw + N, pc, lds, tw1, r0);
    else rows_body<FWD, ArithInt>(g, (size_t)map.n * N, n_here, tw, tw + N, pc, lds, tw1, r0);
}

// Grid of the row pass over n_inst instances whose primes repeat with period `period`.
static dim3 rows_grid(int n_inst, int period) {
    const int reps = (n_inst + period - 1) / period;  // instances per prime slot (the last ones may be missing)
    return dim3(16, period * ((reps + N16_ROWS_GROUP - 1) / N16_ROWS_GROUP));
}

// Forward transform of n_ops operand ciphertexts (two polynomials of l1 limbs each, limb i under prime i) from where they
// lie into data[n_ops][2][l1][N]: the column pass gathers, the row pass runs in place.  ops: device array.
void launch_ntt16_gather(ensi_ctx *ctx, u64 *data, const MmOperand *ops, int n_ops, int l1, hipStream_t st) {
    LimbMap map;
    map.n = l1;
    for (int e = 0; e < ENSI_MAX_EXT; e++) map.prime[e] = e < l1 ? e : 0;
    const int per = 32768 / (2 * l1);  // operands per launch (grid y below 65536)
    for (int done = 0; done < n_ops; done += per) {
        const int cnt = std::min(per, n_ops - done);
        u64 *d = data + (size_t)done * 2 * l1 * ctx->N;
        dim3 grid(16, cnt * 2 * l1);
        {
            ScopedTimer t(ctx, "ntt_fwd_cols", st);
            hipLaunchKernelGGL(k_ntt16_cols_gather, grid, dim3(N16_THREADS), 0, st, d, ops + done, l1, ctx->d_tw, ctx->d_pc);
        }
        {
            ScopedTimer t(ctx, "ntt_fwd_rows", st);
            hipLaunchKernelGGL(k_ntt16_rows<true>, rows_grid(cnt * 2 * l1, map.n), dim3(N16_THREADS), 0, st, d, ctx->d_tw, ctx->d_pc, map, cnt * 2 * l1);
        }
    }
}

void launch_ntt16(ensi_ctx *ctx, u64 *data, int n_inst, const LimbMap &map, bool inverse, hipStream_t st) {
    const int max_rows = (32768 / map.n) * map.n;
    for (int done = 0; done < n_inst; done += max_rows) {
        const int cnt = std::min(max_rows, n_inst - done);
        u64 *d = data + (size_t)done * ctx->N;
        dim3 grid(16, cnt);
        if (!inverse) {
            {
                ScopedTimer t(ctx, "ntt_fwd_cols", st);
                hipLaunchKernelGGL(k_ntt16_cols<true>, grid, dim3(N16_THREADS), 0, st, d, ctx->d_tw, ctx->d_pc, map);
            }
            {
                ScopedTimer t(ctx, "ntt_fwd_rows", st);
                hipLaunchKernelGGL(k_ntt16_rows<true>, rows_grid(cnt, map.n), dim3(N16_THREADS), 0, st, d, ctx->d_tw, ctx->d_pc, map, cnt);
            }
        } else {
            {
                ScopedTimer t(ctx, "ntt_inv_rows", st);
                hipLaunchKernelGGL(k_ntt16_rows<false>, rows_grid(cnt, map.n), dim3(N16_THREADS), 0, st, d, ctx->d_tw, ctx->d_pc, map, cnt);
            }
            {
                ScopedTimer t(ctx, "ntt_inv_cols", st);
                hipLaunchKernelGGL(k_ntt16_cols<false>, grid, dim3(N16_THREADS), 0, st, d, ctx->d_tw, ctx->d_pc, map);
            }
        }
    }
}
