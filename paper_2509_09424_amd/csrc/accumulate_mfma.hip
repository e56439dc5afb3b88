// Alg. 1 (PCMM) as a dense integer contraction on the matrix cores.
//
// y_i = sum_v W'[v][i] * x_v over limb words, W' in {-1,0,+1}.  The paper's point is
// that these products need no ciphertext multiplication; on this chip the cheapest
// way to form the signed sums is still the int8 matrix pipe: every 64-bit limb word
// is split into byte planes, each plane is contracted against the ternary weights
// with V_MFMA_I32_32X32X32_I8 (exact 32-bit integer sums), and the planes are
// recombined with shifts and reduced mod q once per output word.  The result is
// bit-identical to the sequence of modular additions and subtractions.
//
// Bytes are unsigned; the matrix pipe is signed, so each byte u is fed as u-128
// (u xor 0x80) and the constant 128 * sum_v W'[v][i] * sum_b 256^b is added back per
// output (`bias`, wrapped 64-bit).
//
// Work split: a workgroup (4 waves) owns 256 outputs x 32 consecutive words; each
// wave owns 64 outputs (two 32x32 blocks) for all byte planes.  Per step of 32
// operands the workgroup loads 32x32 words, transposes them into byte planes in
// LDS (cell = 16 operands of one word of one plane), and every wave multiplies its
// weight fragments (read straight from global memory, v-contiguous layout) with
// the shared plane fragments.  Workgroups that share the same 32 words (different
// output tiles) are given consecutive slots on one XCD so the operand words are
// fetched from HBM once and served from that XCD's L2 afterwards.
#include "common.h"

typedef int v4i __attribute__((vector_size(16)));
typedef int v16i __attribute__((vector_size(64)));

#define AM_THREADS 256
#define AM_TILE_M 256
#define AM_TILE_N 32
#define AM_TILE_K 32

// Byte b of four dwords gathered into one dword (4x4 byte transpose, two stages).
__device__ __forceinline__ void transpose4(u32 a0, u32 a1, u32 a2, u32 a3, u32 *p) {
    u32 t0 = __builtin_amdgcn_perm(a1, a0, 0x05010400u);
    u32 t1 = __builtin_amdgcn_perm(a1, a0, 0x07030602u);
    u32 t2 = __builtin_amdgcn_perm(a3, a2, 0x05010400u);
    u32 t3 = __builtin_amdgcn_perm(a3, a2, 0x07030602u);
    p[0] = __builtin_amdgcn_perm(t2, t0, 0x05040100u);
    p[1] = __builtin_amdgcn_perm(t2, t0, 0x07060302u);
    p[2] = __builtin_amdgcn_perm(t3, t1, 0x05040100u);
    p[3] = __builtin_amdgcn_perm(t3, t1, 0x07060302u);
}

// signed 64-bit T (|T| < 2^62, |T|/q < 2^31) to its canonical residue mod q
__device__ __forceinline__ u64 reduce_signed(int64_t t, u64 q, double q_inv) {
    const int k = (int)rint((double)t * q_inv);
    int64_t r = t - (int64_t)k * (int64_t)q;
    if (r < 0) r += (int64_t)q;
    if (r < 0) r += (int64_t)q;
    if (r >= (int64_t)q) r -= (int64_t)q;
    return (u64)r;
}

template <int PLANES>
__global__ __launch_bounds__(AM_THREADS) void k_accumulate_mfma(const u64 *const *vptr, int n_v, int n_kpad, const int8_t *wt,
                                                                const int64_t *bias, int m, const PrimeConst *pc, int N, int l1,
                                                                int limb_stride_in, u64 *out, int limb_stride_out, int n_tiles_n,
                                                                int n_tiles_m) {
    __shared__ v4i lds[2][PLANES * 64];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6, g = lane >> 5, nl = lane & 31;
    // XCD-aware tile assignment: workgroup b runs on XCD b%8; consecutive local slots share the word tile
    const int b = blockIdx.x, xcd = b & 7, loc = b >> 3;
    const int m_tile = loc % n_tiles_m;
    const int nt = (loc / n_tiles_m) * 8 + xcd;
    if (nt >= n_tiles_n) return;
    const size_t word0 = (size_t)nt * AM_TILE_N;
    const size_t per_poly = (size_t)l1 * N;
    const int poly = (int)(word0 / per_poly);
    const size_t rem = word0 - (size_t)poly * per_poly;
    const int limb = (int)(rem / N);
    const size_t off_in = (size_t)poly * limb_stride_in * N + rem;
    const size_t off_out = (size_t)poly * limb_stride_out * N + rem;
    // loader role: word ln of the tile, operands 4*k4 .. 4*k4+3 of the step
    const int ln = tid & 31, k4 = tid >> 5;
    // weight fragments: rows (outputs) i0 + nl and i0 + 32 + nl, 16 consecutive operands starting at 16*g
    const int i0 = m_tile * AM_TILE_M + wv * 64;
    const int8_t *wa0 = wt + (size_t)(i0 + nl) * n_kpad + 16 * g;
    const int8_t *wa1 = wa0 + (size_t)32 * n_kpad;

    v16i acc[PLANES][2];
#pragma unroll
    for (int p = 0; p < PLANES; p++)
#pragma unroll
        for (int mb = 0; mb < 2; mb++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[p][mb][r] = 0;

    const int nk = n_kpad / AM_TILE_K;
    u64 x[4];
#pragma unroll
    for (int j = 0; j < 4; j++) {
        int v = 4 * k4 + j;
        v = v < n_v ? v : n_v - 1;
        x[j] = vptr[v][off_in + ln];
    }
    v4i a0 = *(const v4i *)wa0, a1 = *(const v4i *)wa1;

    for (int ks = 0; ks < nk; ks++) {
        // byte planes of the four loaded words -> LDS
        u32 pl[8];
        transpose4((u32)x[0], (u32)x[1], (u32)x[2], (u32)x[3], pl);
        transpose4((u32)(x[0] >> 32), (u32)(x[1] >> 32), (u32)(x[2] >> 32), (u32)(x[3] >> 32), pl + 4);
        int *cells = (int *)lds[ks & 1];
#pragma unroll
        for (int p = 0; p < PLANES; p++) cells[(p * 64 + (k4 >> 2) * 32 + ln) * 4 + (k4 & 3)] = (int)(pl[p] ^ 0x80808080u);
        __syncthreads();
        v4i a0n = a0, a1n = a1;
        if (ks + 1 < nk) {
            const int kb = (ks + 1) * AM_TILE_K;
#pragma unroll
            for (int j = 0; j < 4; j++) {
                int v = kb + 4 * k4 + j;
                v = v < n_v ? v : n_v - 1;
                x[j] = vptr[v][off_in + ln];
            }
            a0n = *(const v4i *)(wa0 + kb);
            a1n = *(const v4i *)(wa1 + kb);
        }
#pragma unroll
        for (int p = 0; p < PLANES; p++) {
            const v4i bf = lds[ks & 1][p * 64 + g * 32 + nl];
            acc[p][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, bf, acc[p][0], 0, 0, 0);
            acc[p][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, bf, acc[p][1], 0, 0, 0);
        }
        a0 = a0n;
        a1 = a1n;
    }

    // recombine planes, add the offset term, reduce mod q, store.  Accumulator register r of
    // a lane holds output row 8*(r/4) + 4*(lane/32) + r%4 of the 32x32 block, column lane%32.
    const u64 q = pc[limb].q;
    const double q_inv = 1.0 / (double)q;
    const size_t ct_words_out = (size_t)2 * limb_stride_out * N;
#pragma unroll
    for (int mb = 0; mb < 2; mb++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
            const int i = i0 + mb * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
            if (i < m) {
                int64_t t = bias[i];
#pragma unroll
                for (int p = 0; p < PLANES; p++) t += (int64_t)((u64)(int64_t)acc[p][mb][r] << (8 * p));
                out[(size_t)i * ct_words_out + off_out + nl] = reduce_signed(t, q, q_inv);
            }
        }
}

void launch_accumulate_mfma(ensi_ctx *ctx, const u64 *const *d_vptr, int n_v, int n_kpad, const int8_t *d_wt, const int64_t *d_bias,
                            int planes, int m, int l1, int limb_stride_in, u64 *out, int limb_stride_out, hipStream_t st) {
    ScopedTimer t(ctx, "accumulate_mfma", st);
    const size_t words = (size_t)2 * l1 * ctx->N;
    const int n_tiles_n = (int)(words / AM_TILE_N);
    const int n_tiles_m = (m + AM_TILE_M - 1) / AM_TILE_M;
    const unsigned grid = 8u * (unsigned)((n_tiles_n + 7) / 8) * (unsigned)n_tiles_m;
#define AM_LAUNCH(P)                                                                                                           \
    hipLaunchKernelGGL(k_accumulate_mfma<P>, dim3(grid), dim3(AM_THREADS), 0, st, d_vptr, n_v, n_kpad, d_wt, d_bias, m, ctx->d_pc, \
                       ctx->N, l1, limb_stride_in, out, limb_stride_out, n_tiles_n, n_tiles_m)
    if (planes <= 5) AM_LAUNCH(5);
    else if (planes <= 7) AM_LAUNCH(7);
    else AM_LAUNCH(8);
#undef AM_LAUNCH
}
