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
// (u xor 0x80) and 128 * sum_v W'[v][i] (`bias`) is added back to every plane of
// output i when the planes are recombined.
//
// Operand v is the ciphertext at xbase + v*xstride words (the unpack phase writes its
// rotations straight into that array).
//
// Work split.  A work item is 256 outputs x 32 consecutive words; inside it each of
// the 4 waves owns 64 outputs (two 32x32 blocks) for all byte planes and walks the
// operands in steps of 32.  Per step:
//   * the raw 32x32 operand words and the wave's two weight fragments arrive in LDS
//     by asynchronous global->LDS copies issued AM_DEPTH steps earlier (rings of
//     AM_DEPTH+1 slots; no registers are held while they are in flight);
//   * the words of step k+1 are transposed into byte planes (cell = 16 operands of
//     one word of one plane; one pad cell per 8 so dword writes hit distinct banks)
//     in the shadow of the matrix instructions of step k;
//   * one barrier.
// The grid is persistent: one workgroup per CU, 32 per XCD.  Items that share their
// 32 words (different output tiles) are consecutive in one XCD's list and the
// workers of that XCD take the list round-robin, so they read the same operand words
// at nearly the same time and all but the first read are served by that XCD's L2.
#include "common.h"

#include <ensi_dma.h>

typedef int v4i __attribute__((vector_size(16)));
typedef int v16i __attribute__((vector_size(64)));

#define AM_THREADS 256
#define AM_TILE_M 256
#define AM_TILE_N 32
#define AM_TILE_K 32
#define AM_DEPTH 7
#define AM_RING (AM_DEPTH + 1)  // power of two; the step loop is unrolled by it so every LDS offset is a constant
#define AM_PLANE_CELLS 72       // 64 cells of 16 bytes + 8 pad cells
#define AM_XBLOCK 1040          // 4 operand rows of 32 words (one copy) + 16 bytes so that blocks start 4 banks apart
#define AM_XSLOT (8 * AM_XBLOCK)  // raw operand words of one step
#define AM_ASLOT 2048           // one wave's two weight fragments of one step

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

// signed 64-bit T (|T| < 2^63, |T|/q < 2^31) to its canonical residue mod q
__device__ __forceinline__ u64 reduce_signed(int64_t t, u64 q, double q_inv) {
    const int k = (int)rint((double)t * q_inv);
    int64_t r = t - (int64_t)k * (int64_t)q;
    if (r < 0) r += (int64_t)q;
    if (r < 0) r += (int64_t)q;
    if (r >= (int64_t)q) r -= (int64_t)q;
    return (u64)r;
}

__device__ __forceinline__ int am_cell(int g, int n) {
    const int c = g * 32 + n;
    return c + (c >> 3);
}

template <int PLANES>
struct AmLayout {
    static constexpr int plane_bytes = PLANES * AM_PLANE_CELLS * 16;
    static constexpr int planes_off = 0;                              // [2][plane_bytes]
    static constexpr int xring_off = 2 * plane_bytes;                 // [AM_RING][AM_XSLOT]
    static constexpr int aring_off = xring_off + AM_RING * AM_XSLOT;  // [4 waves][AM_RING][AM_ASLOT]
    static constexpr int bias_off = aring_off + 4 * AM_RING * AM_ASLOT;  // [256] offset terms of the item's outputs
    static constexpr int total = bias_off + AM_TILE_M * 4;
};

template <int PLANES>
__global__ __launch_bounds__(AM_THREADS) void k_accumulate_mfma(const u64 *xbase, u32 xstride, int n_v, int n_kpad, const v4i *wfrag,
                                                                const int32_t *bias, int m, const PrimeConst *pc, int N, int l1,
                                                                int limb_stride_in, u64 *out, int limb_stride_out, int n_tiles_n,
                                                                int n_tiles_m, int workers_per_xcd, int m_group) {
    HIP_DYNAMIC_SHARED(char, smem)
    typedef AmLayout<PLANES> LY;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6, g = lane >> 5, nl = lane & 31;
    // transposer role: operands 4*k4..4*k4+3 of the step (= copy block k4), word ln.  k4 varies fastest so
    // that one wave's dword writes cover all banks.
    const int k4 = tid & 7, ln = tid >> 3;
    const int nk = n_kpad / AM_TILE_K;
    const u32 smem0 = lds_addr(smem);
    // wave-uniform LDS byte addresses of this wave's copy targets (slot 0)
    const u32 x_lds = (u32)__builtin_amdgcn_readfirstlane((int)(smem0 + LY::xring_off + 2 * wv * AM_XBLOCK));
    const u32 a_lds = (u32)__builtin_amdgcn_readfirstlane((int)(smem0 + LY::aring_off + wv * AM_RING * AM_ASLOT));
    const char *a_rd = smem + LY::aring_off + wv * AM_RING * AM_ASLOT + lane * 16;
    const char *x_rd = smem + LY::xring_off + k4 * AM_XBLOCK + ln * 8;
    int *p_wr = (int *)(smem + LY::planes_off) + am_cell(k4 >> 2, ln) * 4 + (k4 & 3);
    const v4i *p_rd = (const v4i *)(smem + LY::planes_off) + am_cell(g, nl);
    const size_t per_poly = (size_t)l1 * N;
    const size_t ct_words_out = (size_t)2 * limb_stride_out * N;
    const int xcd = blockIdx.x & 7, worker = blockIdx.x >> 3;
    const int n_nt = (n_tiles_n + 7) / 8;  // word tiles of this XCD
    const int items = n_nt * n_tiles_m;
    const int per_group = n_nt * m_group, last_group = (n_tiles_m - 1) / m_group;
    const u64 step_bytes = (u64)AM_TILE_K * xstride * sizeof(u64);

    for (int item = worker; item < items; item += workers_per_xcd) {
        // items are ordered: group of m_group output tiles, word tile, output tile inside the group; the
        // workers of an XCD therefore share both operand words and weight fragments through its L2
        const int mg = item / per_group < last_group ? item / per_group : last_group;
        const int j = item - mg * per_group;
        const int gsize = n_tiles_m - mg * m_group < m_group ? n_tiles_m - mg * m_group : m_group;
        const int m_tile = mg * m_group + j % gsize;
        const int nt = (j / gsize) * 8 + xcd;
        if (nt >= n_tiles_n) continue;
        const size_t word0 = (size_t)nt * AM_TILE_N;
        const int poly = (int)(word0 / per_poly);
        const size_t rem = word0 - (size_t)poly * per_poly;
        const int limb = (int)(rem / N);
        const size_t off_in = (size_t)poly * limb_stride_in * N + rem;
        const size_t off_out = (size_t)poly * limb_stride_out * N + rem;
        const int i0 = m_tile * AM_TILE_M + wv * 64;
        // copy addressing: one copy moves 4 operand rows of 32 words; lane -> (row lane/16, words 2*(lane%16)..+1).
        // Running per-lane pointers walk the operands in step order; they are only used (and advanced) for
        // steps that lie wholly inside the n_v operands, the ragged remainder is clamped lane by lane.
        const u64 *xlane = xbase + off_in + 2 * (lane & 15);
        const int row0 = 8 * wv + (lane >> 4);
        const char *px0 = (const char *)(xlane + (u64)(u32)row0 * (u64)xstride);
        const char *px1 = px0 + 4 * (u64)xstride * sizeof(u64);
        const char *pa = (const char *)(wfrag + ((size_t)m_tile * nk * 4 + wv) * 128 + lane);

        // one of the wave's two copies of the raw words of `step` -> ring slot (copy c = rows 4c..4c+3 of the wave's 8)
        auto issue_x = [&](int step, int slot, int c) {
            const u32 dst = x_lds + (u32)slot * AM_XSLOT + c * AM_XBLOCK;
            if ((step + 1) * AM_TILE_K <= n_v) {
                dma_load16(c ? px1 : px0, dst);
            } else {
                const int st = step < nk ? step : nk - 1;
                int v = st * AM_TILE_K + row0 + 4 * c;
                v = v < n_v ? v : n_v - 1;
                dma_load16(xlane + (u64)(u32)v * (u64)xstride, dst);
            }
            if (c == 1 && (step + 1) * AM_TILE_K <= n_v) {
                px0 += step_bytes;
                px1 += step_bytes;
            }
        };
        // one of the wave's two weight fragments of `step` -> ring slot
        auto issue_a = [&](int step, int slot, int c) {
            dma_load16(pa + c * 1024, a_lds + (u32)slot * AM_ASLOT + c * 1024);
            if (c == 1) pa += step + 1 < nk ? 8192 : 0;
        };
        auto raw_words = [&](int slot, u64 *w) {
            const char *src = x_rd + slot * AM_XSLOT;
#pragma unroll
            for (int j = 0; j < 4; j++) w[j] = *(const u64 *)(src + j * 256);
        };
        auto write_planes = [&](int parity, const u32 *pl) {
            int *cells = p_wr + parity * (LY::plane_bytes / 4);
#pragma unroll
            for (int p = 0; p < PLANES; p++) cells[p * AM_PLANE_CELLS * 4] = (int)(pl[p] ^ 0x80808080u);
        };
        auto build_planes = [&](int slot, int parity) {
            u64 w[4];
            u32 pl[8];
            raw_words(slot, w);
            transpose4((u32)w[0], (u32)w[1], (u32)w[2], (u32)w[3], pl);
            transpose4((u32)(w[0] >> 32), (u32)(w[1] >> 32), (u32)(w[2] >> 32), (u32)(w[3] >> 32), pl + 4);
            write_planes(parity, pl);
        };

        v16i acc[PLANES][2];
#pragma unroll
        for (int p = 0; p < PLANES; p++)
#pragma unroll
            for (int mb = 0; mb < 2; mb++)
#pragma unroll
                for (int r = 0; r < 16; r++) acc[p][mb][r] = 0;

        // drain the previous item's loads and stores: inside the step loop only the copies are in flight
        wait_vmcnt<0>();
        __syncthreads();  // every wave is done with the LDS contents of the previous item
        ((int *)(smem + LY::bias_off))[tid] = bias[m_tile * AM_TILE_M + tid];
        // Copies are issued in one fixed order, "iteration j issues X(j+9) then A(j+8)", from j = -9 on, so that
        // waiting until at most 24 copies are outstanding always means: everything of iteration j-6 has landed.
        issue_x(0, 0, 0);
        issue_x(0, 0, 1);
#pragma unroll
        for (int t = 0; t < AM_DEPTH; t++) {  // iterations -8 .. -2
            issue_x(t + 1, t + 1, 0);
            issue_x(t + 1, t + 1, 1);
            issue_a(t, t, 0);
            issue_a(t, t, 1);
        }
        wait_vmcnt<4 * (AM_DEPTH - 1)>();  // X(0), X(1), A(0) have landed
        __syncthreads();
        build_planes(0, 0);
        build_planes(1, 1);
        __syncthreads();  // planes(0), planes(1) visible; X(0) consumed by everyone
        issue_x(AM_RING, 0, 0);  // iteration -1
        issue_x(AM_RING, 0, 1);
        issue_a(AM_DEPTH, AM_DEPTH, 0);
        issue_a(AM_DEPTH, AM_DEPTH, 1);
        // fragments of step 0 into registers
        v4i bfc[PLANES], a0c, a1c;
#pragma unroll
        for (int p = 0; p < PLANES; p++) bfc[p] = p_rd[p * AM_PLANE_CELLS];
        a0c = *(const v4i *)a_rd;
        a1c = *(const v4i *)(a_rd + 1024);
        wait_vmcnt<4 * (AM_DEPTH - 1)>();  // X(2), A(1) have landed
        __syncthreads();

        // nk is a multiple of AM_RING (the plan pads the operand count with zero weights).
        // Step ks multiplies from registers filled during step ks-1; meanwhile it reads the fragments of step
        // ks+1 (planes buffer (ks+1)&1, A slot (ks+1)%RING), builds the planes of step ks+2 from the raw words
        // in X slot (ks+2)%RING into planes buffer ks&1 (whose contents are already in registers), and issues
        // the copies X(ks+9) -> slot of X(ks+1) and A(ks+8) -> slot of A(ks).  Scheduling fences keep the LDS
        // reads, the copies and the vector work spread between the matrix instructions.
        for (int ks0 = 0; ks0 < nk; ks0 += AM_RING) {
#pragma unroll
            for (int s = 0; s < AM_RING; s++) {
                const int ks = ks0 + s;
                const v4i *pbn = p_rd + ((s + 1) & 1) * (LY::plane_bytes / 16);
                const char *arn = a_rd + ((s + 1) % AM_RING) * AM_ASLOT;
                v4i bfn[PLANES], a0n, a1n;
                u64 xw[4];
                u32 pl[8];
                a0n = *(const v4i *)arn;
                a1n = *(const v4i *)(arn + 1024);
                raw_words((s + 2) % AM_RING, xw);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int p = 0; p < PLANES; p++) {
                    acc[p][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0c, bfc[p], acc[p][0], 0, 0, 0);
                    acc[p][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1c, bfc[p], acc[p][1], 0, 0, 0);
                    bfn[p] = pbn[p * AM_PLANE_CELLS];
                    if (p == 0) issue_x(ks + AM_RING + 1, (s + 1) % AM_RING, 0);
                    if (p == 1) {
                        issue_x(ks + AM_RING + 1, (s + 1) % AM_RING, 1);
                        transpose4((u32)xw[0], (u32)xw[1], (u32)xw[2], (u32)xw[3], pl);
                    }
                    if (p == 2) {
                        issue_a(ks + AM_RING, s, 0);
                        transpose4((u32)(xw[0] >> 32), (u32)(xw[1] >> 32), (u32)(xw[2] >> 32), (u32)(xw[3] >> 32), pl + 4);
                    }
                    if (p == 3) {
                        issue_a(ks + AM_RING, s, 1);
                        write_planes(s & 1, pl);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                wait_vmcnt<4 * (AM_DEPTH - 1)>();  // X(ks+3) and A(ks+2) have landed
                __syncthreads();
#pragma unroll
                for (int p = 0; p < PLANES; p++) bfc[p] = bfn[p];
                a0c = a0n;
                a1c = a1n;
            }
        }

        // Recombine planes, add the offset term 128 * sum_v W'[v][i] * sum_p 256^p, reduce mod q, store.
        // Accumulator register r of a lane holds output row 8*(r/4) + 4*(lane/32) + r%4 of the 32x32
        // block, column lane%32.  The accumulators go through LDS (all rings and planes are dead by
        // now) so that the recombination can be a rolled loop with few live registers.
        wait_vmcnt<0>();
        __syncthreads();
        const u64 q = pc[limb].q;
        const double q_inv = 1.0 / (double)q;
        u64 ones = 0;
#pragma unroll
        for (int p = 0; p < PLANES; p++) ones |= (u64)1 << (8 * p);
        v4i *scr = (v4i *)smem + tid;  // chunk (p, c) of this thread at scr[(p*4 + c) * 256]
        const int *bl = (const int *)(smem + LY::bias_off);
#pragma unroll
        for (int mb = 0; mb < 2; mb++) {
#pragma unroll
            for (int p = 0; p < PLANES; p++)
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    v4i t4 = {acc[p][mb][4 * c], acc[p][mb][4 * c + 1], acc[p][mb][4 * c + 2], acc[p][mb][4 * c + 3]};
                    scr[(p * 4 + c) * AM_THREADS] = t4;
                }
#pragma unroll 1
            for (int c = 0; c < 4; c++) {
                const int ib = i0 + mb * 32 + 8 * c + 4 * g;  // rows ib .. ib+3
                int64_t t[4];
#pragma unroll
                for (int e = 0; e < 4; e++) t[e] = (int64_t)((u64)(int64_t)bl[ib - m_tile * AM_TILE_M + e] * ones);
#pragma unroll
                for (int p = 0; p < PLANES; p++) {
                    const v4i t4 = scr[(p * 4 + c) * AM_THREADS];
#pragma unroll
                    for (int e = 0; e < 4; e++) t[e] += (int64_t)((u64)(int64_t)t4[e] << (8 * p));
                }
#pragma unroll
                for (int e = 0; e < 4; e++)
                    if (ib + e < m) out[(size_t)(ib + e) * ct_words_out + off_out + nl] = reduce_signed(t[e], q, q_inv);
            }
        }
    }
    wait_vmcnt<0>();  // no copy may still be in flight into LDS when the workgroup ends
}

template <int P>
static void am_launch(ensi_ctx *ctx, unsigned grid, hipStream_t st, const u64 *xbase, u32 xstride, int n_v, int n_kpad, const v4i *wfrag,
                      const int32_t *bias, int m, int l1, int limb_stride_in, u64 *out, int limb_stride_out, int n_tiles_n, int n_tiles_m,
                      int workers, int m_group) {
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void *)k_accumulate_mfma<P>, hipFuncAttributeMaxDynamicSharedMemorySize, AmLayout<P>::total);
        attr_set = true;
    }
    hipLaunchKernelGGL(k_accumulate_mfma<P>, dim3(grid), dim3(AM_THREADS), AmLayout<P>::total, st, xbase, xstride, n_v, n_kpad, wfrag, bias, m,
                       ctx->d_pc, ctx->N, l1, limb_stride_in, out, limb_stride_out, n_tiles_n, n_tiles_m, workers, m_group);
}

void launch_accumulate_mfma(ensi_ctx *ctx, const u64 *xbase, size_t xstride, int n_v, int n_kpad, const int8_t *d_wt, const int32_t *d_bias,
                            int planes, int m, int l1, int limb_stride_in, u64 *out, int limb_stride_out, hipStream_t st) {
    ScopedTimer t(ctx, "accumulate_mfma", st);
    const size_t words = (size_t)2 * l1 * ctx->N;
    const int n_tiles_n = (int)(words / AM_TILE_N);
    const int n_tiles_m = (m + AM_TILE_M - 1) / AM_TILE_M;
    static int n_cu = 0;
    if (!n_cu) {
        hipDeviceProp_t prop;
        n_cu = hipGetDeviceProperties(&prop, ctx->device) == hipSuccess ? prop.multiProcessorCount : 256;
        if (n_cu < 8) n_cu = 8;
    }
    const int workers = n_cu / 8;  // one persistent workgroup per CU; workgroup b runs on XCD b % 8
    const unsigned grid = 8u * (unsigned)workers;
    const v4i *wf = (const v4i *)d_wt;
    const int m_group = 8;  // 8 output tiles x 4 word tiles in flight per XCD
    if (planes <= 5)
        am_launch<5>(ctx, grid, st, xbase, (u32)xstride, n_v, n_kpad, wf, d_bias, m, l1, limb_stride_in, out, limb_stride_out, n_tiles_n, n_tiles_m, workers, m_group);
    else
        am_launch<7>(ctx, grid, st, xbase, (u32)xstride, n_v, n_kpad, wf, d_bias, m, l1, limb_stride_in, out, limb_stride_out, n_tiles_n, n_tiles_m, workers, m_group);
}
