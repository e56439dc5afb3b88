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
// Two kernels.  k_byte_planes runs once per operand array: it splits every 32 x 32 tile
// (32 operands x 32 consecutive words) into its byte planes, already in the register
// layout of the matrix instruction's second operand (lane = 32*(operand/16) + word, 16
// operand bytes per lane), so that the tile of one plane is 1 KiB that a single
// asynchronous global->LDS copy drops in place.  Tiles are stored [word tile][step]
// [plane]: a work item of the contraction streams one contiguous run.  The split is done
// once instead of once per output tile (10 to 27 times at the benchmark shapes), which
// takes the byte shuffling, the plane stores and a second LDS buffer out of the
// contraction's inner loop.  The plane array of a whole operand array can exceed the
// memory left, so the host works through the coefficients in slices (a slice holds a
// range of 32-coefficient tiles of every limb of both polynomials).  The split can apply
// the scalar-multiply + rescale step between two layers on the fly (k_byte_planes<.., true>):
// the rescaled operands then never exist as 64-bit words in memory.
//
// k_accumulate_mfma.  A work item is 256 outputs x 32 consecutive words; inside it each
// of the 4 waves owns 64 outputs (two 32x32 blocks) for all byte planes and walks the
// operands in steps of 32.  Per step:
//   * the step's plane tiles and the wave's two weight fragments arrive in LDS by
//     asynchronous global->LDS copies issued AM_RING steps earlier (rings of AM_RING
//     slots; no registers are held while they are in flight);
//   * the fragments of step k+1 are read from LDS while the matrix instructions of
//     step k run from registers;
//   * one barrier.
// The step loop holds no vector-ALU instruction besides the matrix instructions: the running source addresses of the
// copies are wave-uniform and live in scalar registers (a lane adds 16 * lane through the instruction's offset
// operand).  Vector instructions issued between matrix instructions slow the matrix pipe down measurably -- four 64-bit
// address updates per step cost 5 % of the kernel, an in-loop unpacking of 2-bit weights (22 instructions) 10 %.
// The grid is persistent: one workgroup per CU, 32 per XCD.  Items that share their
// 32 words (different output tiles) are consecutive in one XCD's list and the
// workers of that XCD take the list round-robin, so they read the same plane tiles
// at nearly the same time and all but the first read are served by that XCD's L2.
#include <algorithm>

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
#define AM_BSLOT 8192           // plane tiles of one step (1 KiB each, PLANES of 8 used)
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

// The same recombination for primes below 2^50, in double precision on exact integers (no 64-bit integer
// multiplies, which take many quarter-rate instructions on this chip).  S_p: the plane sums from the matrix
// pipe; the true plane sums are T_p = S_p + b with b = 128 * (column sum of the weights), and the result is
// sum_p T_p 2^(8p) mod q = (sum_p S_p 2^(8p) + B) mod q with B = b * sum_p 2^(8p) mod q, which the host supplies
// per output and limb as a double in [0, q).  |S_p| <= 2^22 for up to 32768 operands, so planes are first paired
// in 32-bit integers (S_p + 2^8 S_(p+1) < 2^31) and the pairs combined into lo + 2^32 hi with |lo| < 2^48 and
// |hi| < 2^38.1 -- every product by a power of two and every sum below 2^53 is exact in a double.  One reduction:
// k = rint((lo + B + 2^32 hi) / q) from two rounded products (off by far less than one half except within 2^-30 of
// a tie), then 2^32 hi - k q, an integer below 2^52 in magnitude that the fused multiply-add returns exactly, plus
// lo + B: a representative within (1/2 + 2^-30) q of zero, shifted into [0, q).
template <int PLANES>
__device__ __forceinline__ u64 recombine_fp(const int (&S)[PLANES], double B, double q, double q_inv) {
    const int c01 = S[0] + (S[1] << 8), c23 = S[2] + (S[3] << 8);
    const double lb = fma((double)c23, 65536.0, (double)c01) + B;
    double hi;
    if (PLANES == 7) {
        const int c45 = S[4] + (S[5] << 8);
        hi = fma((double)S[6], 65536.0, (double)c45);
    } else {
        hi = (double)S[4];
    }
    const double x = hi * 4294967296.0;
    const double k = rint(fma(lb, q_inv, x * q_inv));
    double u = fma(-k, q, x) + lb;
    u = u < 0.0 ? u + q : u;
    // an integer in [0, 2^52) plus 2^52 has that integer as its mantissa
    return (u64)__double_as_longlong(u + 4503599627370496.0) & 0xFFFFFFFFFFFFFull;
}

// ---------------------------------------------------------------- byte planes of the operands
// Slice-local word tile: nt_local = pl * cw + ctile, pl = poly * l1 + limb, ctile = coefficient tile - c0.
// Thread (k4 = tid / 32, ln = tid % 32) handles operands 4*k4 .. 4*k4+3 of a step, word ln: its four
// words give one dword (4 operand bytes) of every plane.  A plane tile is staged in LDS and written out as
// whole 16-byte lane entries.  Bytes are stored as u - 128 (u xor 0x80); operands beyond n_v are zero
// words (their weights are zero).
struct AmFp {  // fp64 arithmetic on exact integers modulo a prime below 2^50 (as in the rescale kernel)
    double q, qinv;
    __device__ __forceinline__ double mid(double x) const { return fma(-rint(x * qinv), q, x); }
    __device__ __forceinline__ double mulmod(double x, double w, double wq) const {
        const double h = x * w;
        const double l = fma(x, w, -h);
        const double t = rint(x * wq);
        return fma(-t, q, h) + l;
    }
};

template <int PLANES, int STEPS>
__device__ __forceinline__ void planes_out(const u64 (&w)[STEPS][4], u32 (*stage)[PLANES * 256], int dst, v4i *out, int tid) {
#pragma unroll
    for (int s8 = 0; s8 < STEPS; s8++) {
        u32 pl[8];
        transpose4((u32)w[s8][0], (u32)w[s8][1], (u32)w[s8][2], (u32)w[s8][3], pl);
        transpose4((u32)(w[s8][0] >> 32), (u32)(w[s8][1] >> 32), (u32)(w[s8][2] >> 32), (u32)(w[s8][3] >> 32), pl + 4);
        u32 *st = stage[s8 & 1];
#pragma unroll
        for (int p = 0; p < PLANES; p++) st[p * 256 + dst] = pl[p] ^ 0x80808080u;
        __syncthreads();  // (the other staging buffer was read before the previous barrier)
        const v4i *sv = (const v4i *)st;
        for (int e = tid; e < PLANES * 64; e += AM_THREADS) out[(size_t)s8 * PLANES * 64 + e] = sv[e];
    }
}

// grid (cw, nk / 8, 2 * l1); each block converts 8 steps of one word tile.
template <int PLANES>
__global__ __launch_bounds__(AM_THREADS) void k_byte_planes(const u64 *xbase, u32 xstride, int n_v, int nk, int N, int l1, int limb_stride_in,
                                                            int c0, int cw, char *xp) {
    __shared__ u32 stage[2][PLANES * 256];
    const int tid = threadIdx.x, k4 = tid >> 5, ln = tid & 31;
    const int pl = blockIdx.z, poly = pl / l1, limb = pl - poly * l1;
    const u64 *xw = xbase + ((size_t)poly * limb_stride_in + limb) * N + (size_t)(c0 + blockIdx.x) * AM_TILE_N + ln;
    // destination dword of this thread inside a plane tile: lane (k4/4)*32 + ln, dword k4 % 4
    const int dst = ((k4 >> 2) * 32 + ln) * 4 + (k4 & 3);
    v4i *out = (v4i *)(xp + (((size_t)pl * cw + blockIdx.x) * nk + (size_t)blockIdx.y * 8) * PLANES * 1024);
    // all 32 words of the block's 8 steps are requested before the first is used
    u64 w[8][4];
#pragma unroll
    for (int s8 = 0; s8 < 8; s8++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int v = (blockIdx.y * 8 + s8) * AM_TILE_K + 4 * k4 + j;
            w[s8][j] = v < n_v ? xw[(size_t)v * xstride] : 0;
        }
    planes_out<PLANES, 8>(w, stage, dst, out, tid);
}

// The same with the scalar-multiply + rescale step applied on the way: the operands are read at l1 + 1
// limbs, c <- c * k, limb l1 dropped with rounding to nearest (c_i <- (c_i k - [c_l k]) q_l^-1 mod q_i with
// the centred representative of limb l1), and the planes of the l1 remaining limbs written.  fc: [5][l1+1]
// doubles: k mod q_i, that / q_i, q_l^-1 mod q_i, that / q_i, 1 / q_i.  grid (cw, nk / 4, 2): a block keeps
// the centred last-limb residues of its 32 coefficients x 128 operands in registers and walks the limbs
// (4 steps per block keep the register count low enough for four blocks per CU).
#define AM_RS_STEPS 4
template <int PLANES>
__global__ __launch_bounds__(AM_THREADS) void k_byte_planes_rescale(const u64 *xbase, u32 xstride, int n_v, int nk, int N, int l1,
                                                                    int limb_stride_in, int c0, int cw, char *xp, const PrimeConst *pc,
                                                                    const double *fc) {
    __shared__ u32 stage[2][PLANES * 256];
    const int tid = threadIdx.x, k4 = tid >> 5, ln = tid & 31;
    const int poly = blockIdx.z, lin = l1 + 1;
    const u64 *xw = xbase + (size_t)poly * limb_stride_in * N + (size_t)(c0 + blockIdx.x) * AM_TILE_N + ln;
    const int dst = ((k4 >> 2) * 32 + ln) * 4 + (k4 & 3);
    u64 w[AM_RS_STEPS][4];
    double xl[AM_RS_STEPS][4];
    // operand rows of this thread: row[s8] + j * xstride for j < n_live[s8] (a multiple of four operands except in
    // the last step of a ragged operand count; dead operands re-read row j = 0 and are zeroed before the split)
    const u64 *row[AM_RS_STEPS];
    int n_live[AM_RS_STEPS];
#pragma unroll
    for (int s8 = 0; s8 < AM_RS_STEPS; s8++) {
        const int v0 = (blockIdx.y * AM_RS_STEPS + s8) * AM_TILE_K + 4 * k4;
        n_live[s8] = min(max(n_v - v0, 0), 4);
        row[s8] = xw + (size_t)(n_live[s8] ? v0 : 0) * xstride;
    }
    {
        const AmFp ml = {(double)pc[l1].q, fc[4 * lin + l1]};
        const double kl = fc[l1], kl_q = fc[lin + l1];
#pragma unroll
        for (int s8 = 0; s8 < AM_RS_STEPS; s8++)
#pragma unroll
            for (int j = 0; j < 4; j++) w[s8][j] = row[s8][(size_t)(j < n_live[s8] ? j : 0) * xstride + (size_t)l1 * N];
#pragma unroll
        for (int s8 = 0; s8 < AM_RS_STEPS; s8++)
#pragma unroll
            for (int j = 0; j < 4; j++) xl[s8][j] = ml.mid(ml.mulmod((double)w[s8][j], kl, kl_q));
    }
    for (int limb = 0; limb < l1; limb++) {
        const AmFp m = {(double)pc[limb].q, fc[4 * lin + limb]};
        const double k = fc[limb], k_q = fc[lin + limb], qi = fc[2 * lin + limb], qi_q = fc[3 * lin + limb];
#pragma unroll
        for (int s8 = 0; s8 < AM_RS_STEPS; s8++)
#pragma unroll
            for (int j = 0; j < 4; j++) w[s8][j] = row[s8][(size_t)(j < n_live[s8] ? j : 0) * xstride + (size_t)limb * N];
#pragma unroll
        for (int s8 = 0; s8 < AM_RS_STEPS; s8++)
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const double t = m.mulmod((double)w[s8][j], k, k_q) - m.mid(xl[s8][j]);
                double r = m.mid(m.mulmod(m.mid(t), qi, qi_q));
                r = r < 0.0 ? r + m.q : r;
                w[s8][j] = j < n_live[s8] ? (u64)r : 0;
            }
        v4i *out = (v4i *)(xp + ((((size_t)poly * l1 + limb) * cw + blockIdx.x) * nk + (size_t)blockIdx.y * AM_RS_STEPS) * PLANES * 1024);
        __syncthreads();  // the staging buffers of the previous limb have been written out
        planes_out<PLANES, AM_RS_STEPS>(w, stage, dst, out, tid);
    }
}

// primes of the active limbs and their reciprocals, passed by value so that the recombination reads them with
// scalar loads (a vector load there would make the compiler wait for every copy in flight)
struct AmPrimes {
    u64 q[ENSI_MAX_EXT];
    double q_inv[ENSI_MAX_EXT];
};

template <int PLANES>
struct AmLayout {
    static constexpr int bring_off = 0;                                  // [AM_RING][AM_BSLOT]
    static constexpr int aring_off = bring_off + AM_RING * AM_BSLOT;     // [4 waves][AM_RING][AM_ASLOT]
    static constexpr int bias_off = aring_off + 4 * AM_RING * AM_ASLOT;  // [2][256] offset terms of an item's outputs (int32 or double)
    static constexpr int total = bias_off + 2 * AM_TILE_M * 8;
};

// xp: plane tiles of the slice, [word tile][nk][PLANES][1024]; the slice covers coefficient tiles c0 .. c0+cw-1
// of all 2*l1 limb rows (n_tiles_n = 2*l1*cw word tiles); nk = n_kpad / 32, a multiple of AM_RING.
// FP_EPI: every active prime is below 2^50, so the planes are recombined in double precision (recombine_fp) and bias
// points to doubles [l1][n_tiles_m * 256], the offset term of every output reduced modulo each limb's prime; else the
// planes are recombined in 64-bit integers and bias points to int32 [n_tiles_m * 256], 128 * column sum of the weights.
template <int PLANES, bool FP_EPI>
__global__ __launch_bounds__(AM_THREADS) void k_accumulate_mfma(const char *xp, int c0, int cw, int n_kpad, const v4i *wfrag, const void *bias,
                                                                int m, AmPrimes pr, int N, int l1, u64 *out, int limb_stride_out,
                                                                int n_tiles_n, int n_tiles_m, int workers_per_xcd, int m_group) {
    HIP_DYNAMIC_SHARED(char, smem)
    typedef AmLayout<PLANES> LY;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), g = lane >> 5, nl = lane & 31;
    const int nk = n_kpad / AM_TILE_K;
    const u32 smem0 = lds_addr(smem);
    // the wave copies plane tiles pb0 and pb1 of every step (the last plane twice where 2*wave+1 runs past it)
    const int pb0 = 2 * wv < PLANES ? 2 * wv : PLANES - 1, pb1 = 2 * wv + 1 < PLANES ? 2 * wv + 1 : PLANES - 1;
    // wave-uniform LDS byte addresses of this wave's copy targets (slot 0)
    const u32 b_lds0 = (u32)__builtin_amdgcn_readfirstlane((int)(smem0 + LY::bring_off + pb0 * 1024));
    const u32 b_lds1 = (u32)__builtin_amdgcn_readfirstlane((int)(smem0 + LY::bring_off + pb1 * 1024));
    const u32 a_lds = (u32)__builtin_amdgcn_readfirstlane((int)(smem0 + LY::aring_off + wv * AM_RING * AM_ASLOT));
    const char *a_rd = smem + LY::aring_off + wv * AM_RING * AM_ASLOT + lane * 16;
    const char *b_rd = smem + LY::bring_off + lane * 16;
    const size_t ct_words_out = (size_t)2 * limb_stride_out * N;
    const int xcd = blockIdx.x & 7, worker = blockIdx.x >> 3;
    const int n_nt = (n_tiles_n + 7) / 8;  // word tiles of this XCD
    const int items = n_nt * n_tiles_m;
    const int per_group = n_nt * m_group, last_group = (n_tiles_m - 1) / m_group;

    // item index -> (output tile, word tile of the slice); false for the padding slots of the last group of 8 word tiles.
    // Items are ordered: group of m_group output tiles, word tile, output tile inside the group; the workers of an
    // XCD therefore share both plane tiles and weight fragments through its L2.
    auto decode = [&](int item, int &m_tile, int &nt_local) {
        const int mg = item / per_group < last_group ? item / per_group : last_group;
        const int j = item - mg * per_group;
        const int gsize = n_tiles_m - mg * m_group < m_group ? n_tiles_m - mg * m_group : m_group;
        m_tile = mg * m_group + j % gsize;
        nt_local = (j / gsize) * 8 + xcd;
        return nt_local < n_tiles_n;
    };
    auto next_valid = [&](int item) {
        int mt, nt;
        while (item < items && !decode(item, mt, nt)) item += workers_per_xcd;
        return item;
    };

    // The copies of all items of this workgroup form one stream of steps: the ring never drains between items.
    // pb/pa are the running per-lane source pointers of the stream.
    // pb/pa are wave-uniform (scalar registers, advanced by the scalar unit); a lane adds its own 16 * lane bytes.
    const char *pb[2], *pa;
    const u32 lane_off = (u32)lane * 16;
    auto seek = [&](int item) {
        int mt, nt;
        decode(item, mt, nt);
        const char *pbase = xp + (size_t)nt * nk * PLANES * 1024;
        pb[0] = pbase + pb0 * 1024;
        pb[1] = pbase + pb1 * 1024;
        pa = (const char *)(wfrag + ((size_t)mt * nk * 4 + wv) * 128);
    };
    // one of the wave's two plane tiles of the stream's next step -> ring slot
    auto issue_b = [&](int slot, int c) {
        dma_load16_s(pb[c], lane_off, (c ? b_lds1 : b_lds0) + (u32)slot * AM_BSLOT);
        pb[c] += PLANES * 1024;
    };
    // one of the wave's two weight fragments of the stream's next step -> ring slot
    auto issue_a = [&](int slot, int c) {
        dma_load16_s(pa + c * 1024, lane_off, a_lds + (u32)slot * AM_ASLOT + c * 1024);
        if (c == 1) pa += 8192;
    };

    // offset terms of an item's 256 outputs -> one of two LDS buffers (64 per wave); issued one item ahead
    constexpr int BIAS_BYTES = FP_EPI ? 8 : 4;
    const u32 bias_lds = (u32)__builtin_amdgcn_readfirstlane((int)(smem0 + LY::bias_off + wv * 64 * BIAS_BYTES));
    auto issue_bias = [&](int item, int buf) {
        int mt, nt;
        decode(item, mt, nt);
        if (FP_EPI) {
            // the wave's 64 doubles of the item's limb, as two copies of 4 bytes per lane (256 contiguous bytes each)
            const int pl = nt / cw, limb = pl - (pl / l1) * l1;
            const char *src = (const char *)((const double *)bias + (size_t)limb * n_tiles_m * AM_TILE_M + mt * AM_TILE_M + wv * 64) + lane * 4;
            dma_load4(src, bias_lds + (u32)buf * (AM_TILE_M * 8));
            dma_load4(src + 256, bias_lds + (u32)buf * (AM_TILE_M * 8) + 256);
        } else {
            dma_load4((const int32_t *)bias + mt * AM_TILE_M + wv * 64 + lane, bias_lds + (u32)buf * (AM_TILE_M * 4));
        }
    };

    int item = next_valid(worker);
    if (item >= items) return;
    issue_bias(item, 0);
    // Copies are issued in one fixed order, "iteration j issues B(j+8) then A(j+8) into slot j % 8" (j counts the
    // steps of the stream), from j = -8 on, so that waiting until at most 24 copies are outstanding always means:
    // everything of iteration j-6 has landed.
    seek(item);
#pragma unroll
    for (int t = 0; t < AM_RING; t++) {  // iterations -8 .. -1: steps 0..7 of the first item
        issue_b(t, 0);
        issue_b(t, 1);
        issue_a(t, 0);
        issue_a(t, 1);
    }
    wait_vmcnt<4 * (AM_DEPTH - 1)>();  // steps 0 and 1 have landed
    __syncthreads();
    // Fragments live in two register sets used alternately: step ks multiplies from set ks & 1 while the
    // fragments of step ks+1 are read into the other set.  (With one set, the LDS read that refills a
    // fragment's registers has to wait for the matrix instructions still reading them, and every later
    // instruction of the wave queues behind it.)  nk is even, so every item starts on set 0.
    v4i bf[2][PLANES], af[2][2];
#pragma unroll
    for (int p = 0; p < PLANES; p++) bf[0][p] = *(const v4i *)(b_rd + p * 1024);
    af[0][0] = *(const v4i *)a_rd;
    af[0][1] = *(const v4i *)(a_rd + 1024);
    __syncthreads();  // slot 0 has been read by every wave before step 0 refills it

    for (int it = 0; item < items; it++) {
        int m_tile, nt_local;
        decode(item, m_tile, nt_local);
        const int next = next_valid(item + workers_per_xcd);
        const int pl = nt_local / cw, poly = pl / l1, limb = pl - poly * l1;
        const size_t off_out = ((size_t)poly * limb_stride_out + limb) * N + (size_t)(c0 + nt_local - pl * cw) * AM_TILE_N;
        const int i0 = m_tile * AM_TILE_M + wv * 64;
        // offset terms of this item's outputs: copied one item ahead into two buffers used alternately (the
        // other one may still be read by a wave that has not finished the previous item's recombination)
        const char *bl = smem + LY::bias_off + (it & 1) * AM_TILE_M * BIAS_BYTES;

        v16i acc[PLANES][2];
#pragma unroll
        for (int p = 0; p < PLANES; p++)
#pragma unroll
            for (int mb = 0; mb < 2; mb++)
#pragma unroll
                for (int r = 0; r < 16; r++) acc[p][mb][r] = 0;

        // Step ks multiplies from registers filled during step ks-1; meanwhile it reads the fragments of step
        // ks+1 from slot (ks+1) % RING and issues the copies of the stream's step ks+8 into slot ks % RING (read
        // during step ks-1, before the barrier that ended it).  During the last 8 steps of an item the stream
        // has moved on to the first 8 steps of the next item (after the last item: of the same item again,
        // which nobody reads).  Scheduling fences keep the LDS reads and the copies spread between the matrix
        // instructions.
        for (int ks0 = 0; ks0 < nk; ks0 += AM_RING) {
            if (ks0 + AM_RING == nk) {
                seek(next < items ? next : item);
                if (next < items) issue_bias(next, (it + 1) & 1);
            }
#pragma unroll
            for (int s = 0; s < AM_RING; s++) {
                const int cur = s & 1, nxt = cur ^ 1;
                const char *brn = b_rd + ((s + 1) % AM_RING) * AM_BSLOT;
                const char *arn = a_rd + ((s + 1) % AM_RING) * AM_ASLOT;
                af[nxt][0] = *(const v4i *)arn;
                af[nxt][1] = *(const v4i *)(arn + 1024);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int p = 0; p < PLANES; p++) {
                    bf[nxt][p] = *(const v4i *)(brn + p * 1024);
                    __builtin_amdgcn_sched_barrier(0);
                    acc[p][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[cur][0], bf[cur][p], acc[p][0], 0, 0, 0);
                    acc[p][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[cur][1], bf[cur][p], acc[p][1], 0, 0, 0);
                    if (p == 0) issue_b(s, 0);
                    if (p == 1) issue_b(s, 1);
                    if (p == 2) issue_a(s, 0);
                    if (p == 3) issue_a(s, 1);
                    __builtin_amdgcn_sched_barrier(0);
                }
                // keep this step's fragments alive up to here, so that the register allocator cannot hand
                // their registers to the next step's fragments while matrix instructions still read them
#pragma unroll
                for (int p = 0; p < PLANES; p++) asm volatile("" ::"v"(bf[cur][p]));
                asm volatile("" ::"v"(af[cur][0]), "v"(af[cur][1]));
                // The stores of the previous item's recombination are younger than the copies this step needs
                // but older than the ones it issued; the first step of an item therefore waits for everything
                // except its own copies, which drains those stores whatever order stores and loads complete in.
                if (ks0 == 0 && s == 0) wait_vmcnt<4>();
                else wait_vmcnt<4 * (AM_DEPTH - 1)>();  // step ks+2 has landed
                __syncthreads();
            }
        }
        // here bf[0]/af[0] already hold step 0 of the next item

        // Recombine planes, add the offset term 128 * sum_v W'[v][i] * sum_p 256^p, reduce mod q, store.
        // Accumulator register r of a lane holds output row 8*(r/4) + 4*(lane/32) + r%4 of the 32x32
        // block, column lane%32.
        const u64 q = pr.q[limb];
        const double q_inv = pr.q_inv[limb], qd = (double)q;
        u64 ones = 0;
#pragma unroll
        for (int p = 0; p < PLANES; p++) ones |= (u64)1 << (8 * p);
        const bool whole = i0 + 64 <= m;  // all 64 outputs of this wave exist (wave-uniform): stores need no bounds check
#pragma unroll
        for (int mb = 0; mb < 2; mb++) {
#pragma unroll
            for (int c = 0; c < 4; c++) {
                const int ib = i0 + mb * 32 + 8 * c + 4 * g;  // rows ib .. ib+3
                u64 res[4];
                if (FP_EPI) {
                    const double *b4 = (const double *)bl + (ib - m_tile * AM_TILE_M);
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        int S[PLANES];
#pragma unroll
                        for (int p = 0; p < PLANES; p++) S[p] = acc[p][mb][4 * c + e];
                        res[e] = recombine_fp<PLANES>(S, b4[e], qd, q_inv);
                    }
                } else {
                    const v4i b4 = *(const v4i *)((const int *)bl + (ib - m_tile * AM_TILE_M));
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        int64_t t = (int64_t)((u64)(int64_t)b4[e] * ones);
#pragma unroll
                        for (int p = 0; p < PLANES; p++) t += (int64_t)((u64)(int64_t)acc[p][mb][4 * c + e] << (8 * p));
                        res[e] = reduce_signed(t, q, q_inv);
                    }
                }
                u64 *o = out + (size_t)ib * ct_words_out + off_out + nl;
                if (whole) {
#pragma unroll
                    for (int e = 0; e < 4; e++) o[(size_t)e * ct_words_out] = res[e];
                } else {
#pragma unroll
                    for (int e = 0; e < 4; e++)
                        if (ib + e < m) o[(size_t)e * ct_words_out] = res[e];
                }
            }
        }
        item = next;
    }
    wait_vmcnt<0>();  // no copy may still be in flight into LDS when the workgroup ends
}

template <int P, bool FP_EPI>
static void am_launch(ensi_ctx *ctx, unsigned grid, hipStream_t st, const u64 *xbase, u32 xstride, int n_v, int n_kpad, const v4i *wfrag,
                      const void *bias, int m, int l1, int limb_stride_in, u64 *out, int limb_stride_out, int n_tiles_m, int workers,
                      int m_group, char *xp, int slice_ctiles, const double *d_rescale) {
    bool &attr_set = ctx->am_attr_set[(P == 5 ? 0 : 1) + (FP_EPI ? 0 : 2)];
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void *)k_accumulate_mfma<P, FP_EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, AmLayout<P>::total);
        attr_set = true;
    }
    const int nk = n_kpad / AM_TILE_K, ctiles = ctx->N / AM_TILE_N;
    AmPrimes pr;
    for (int i = 0; i < ENSI_MAX_EXT; i++) {
        pr.q[i] = i < l1 ? ctx->primes[i] : 1;
        pr.q_inv[i] = 1.0 / (double)pr.q[i];
    }
    for (int c0 = 0; c0 < ctiles; c0 += slice_ctiles) {
        const int cw = std::min(slice_ctiles, ctiles - c0);
        {
            ScopedTimer t(ctx, d_rescale ? "rescale_byte_planes" : "byte_planes", st);
            if (d_rescale)
                hipLaunchKernelGGL(k_byte_planes_rescale<P>, dim3(cw, nk / AM_RS_STEPS, 2), dim3(AM_THREADS), 0, st, xbase, xstride, n_v, nk, ctx->N, l1,
                                   limb_stride_in, c0, cw, xp, ctx->d_pc, d_rescale);
            else
                hipLaunchKernelGGL(k_byte_planes<P>, dim3(cw, nk / 8, 2 * l1), dim3(AM_THREADS), 0, st, xbase, xstride, n_v, nk, ctx->N, l1,
                                   limb_stride_in, c0, cw, xp);
        }
        {
            ScopedTimer t(ctx, "accumulate_mfma", st);
            hipLaunchKernelGGL((k_accumulate_mfma<P, FP_EPI>), dim3(grid), dim3(AM_THREADS), AmLayout<P>::total, st, (const char *)xp, c0, cw, n_kpad, wfrag,
                               bias, m, pr, ctx->N, l1, out, limb_stride_out, 2 * l1 * cw, n_tiles_m, workers, m_group);
        }
    }
}

// Coefficient tiles per slice: all of them if their planes fit the budget.
static int am_slice_ctiles(int ctiles, int l1, int n_kpad, int planes) {
    const size_t per_ctile = (size_t)2 * l1 * (n_kpad / AM_TILE_K) * (planes <= 5 ? 5 : 7) * 1024;
    const size_t budget = (size_t)16 << 30;
    return (int)std::min<size_t>((size_t)ctiles, std::max<size_t>(budget / per_ctile, 1));
}

// d_rescale != nullptr: the operands are read at l1 + 1 limbs and the scalar-multiply + rescale step is applied while
// their planes are built (constants as for k_rescale_fp at l1 + 1 limbs); out is at l1 limbs.
int launch_accumulate_mfma(ensi_ctx *ctx, const u64 *xbase, size_t xstride, int n_v, int n_kpad, const int8_t *d_wt, const int32_t *d_bias,
                           const double *d_bias_fp, int planes, int m, int l1, int limb_stride_in, u64 *out, int limb_stride_out, const double *d_rescale,
                           hipStream_t st) {
    const int ctiles = ctx->N / AM_TILE_N;
    const int n_tiles_m = (m + AM_TILE_M - 1) / AM_TILE_M;
    int &n_cu = ctx->n_cu;
    if (!n_cu) {
        hipDeviceProp_t prop;
        n_cu = hipGetDeviceProperties(&prop, ctx->device) == hipSuccess ? prop.multiProcessorCount : 256;
        if (n_cu < 8) n_cu = 8;
    }
    const int workers = n_cu / 8;  // one persistent workgroup per CU; workgroup b runs on XCD b % 8
    const unsigned grid = 8u * (unsigned)workers;
    const v4i *wf = (const v4i *)d_wt;
    const int m_group = 8;  // 8 output tiles x 4 word tiles in flight per XCD
    const int P = planes <= 5 ? 5 : 7;
    const int slice_ctiles = am_slice_ctiles(ctiles, l1, n_kpad, P);
    const size_t xp_words = ((size_t)slice_ctiles * 2 * l1 * (n_kpad / AM_TILE_K) * P * 1024 + 7) / 8;
    if (ctx->ws_xp_words < xp_words) {
        if (ctx->ws_xp) (void)hipFree(ctx->ws_xp);
        ctx->ws_xp = nullptr;
        ctx->ws_xp_words = 0;
        if (hipMalloc((void **)&ctx->ws_xp, xp_words * 8) != hipSuccess) {
            ctx->err = "device allocation of the byte-plane workspace failed";
            return ENSI_E_NOMEM;
        }
        ctx->ws_xp_words = xp_words;
    }
    bool fp_epi = d_bias_fp != nullptr;  // the double-precision recombination is exact while every active prime is below 2^50
    for (int i = 0; i < l1; i++) fp_epi = fp_epi && ctx->primes[i] < ((u64)1 << 50);
#define AM_LAUNCH(PL, FP)                                                                                                              \
    am_launch<PL, FP>(ctx, grid, st, xbase, (u32)xstride, n_v, n_kpad, wf, (FP) ? (const void *)d_bias_fp : (const void *)d_bias, m, l1, limb_stride_in, out, limb_stride_out, n_tiles_m, \
                      workers, m_group, (char *)ctx->ws_xp, slice_ctiles, d_rescale)
    if (P == 5) {
        if (fp_epi) AM_LAUNCH(5, true);
        else AM_LAUNCH(5, false);
    } else {
        if (fp_epi) AM_LAUNCH(7, true);
        else AM_LAUNCH(7, false);
    }
#undef AM_LAUNCH
    return ENSI_OK;
}

// ---------------------------------------------------------------- sustained rate of the matrix instruction
// A register-only loop of V_MFMA_I32_32X32X32_I8, eight independent accumulator blocks per wave, one workgroup of four
// waves per CU like the contraction: what the matrix pipes deliver at the clock the chip holds under that load.  No
// memory is touched inside the loop; the operands come from `seed` words so that the compiler cannot fold the loop.
__global__ __launch_bounds__(AM_THREADS) void k_matrix_rate(const int *seed, int iters, int *sink) {
    v4i a, b;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        a[i] = seed[(threadIdx.x * 4 + i) & 1023];
        b[i] = seed[(threadIdx.x * 4 + i + 512) & 1023];
    }
    v16i d[8];
#pragma unroll
    for (int j = 0; j < 8; j++)
#pragma unroll
        for (int r = 0; r < 16; r++) d[j][r] = 0;
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int j = 0; j < 8; j++) d[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, d[j], 0, 0, 0);
    }
    int t = 0;
#pragma unroll
    for (int j = 0; j < 8; j++) t += d[j][j];
    if (t == 0x7fffffff) sink[0] = t;  // keeps the loop alive; never true for these operands in practice, harmless if it is
}

int launch_matrix_rate(ensi_ctx *ctx, double seconds, double *ops_per_second, hipStream_t st) {
    int &n_cu = ctx->n_cu;
    if (!n_cu) {
        hipDeviceProp_t prop;
        n_cu = hipGetDeviceProperties(&prop, ctx->device) == hipSuccess ? prop.multiProcessorCount : 256;
        if (n_cu < 8) n_cu = 8;
    }
    std::vector<int> h(1024);
    u64 x = 0x9E3779B97F4A7C15ull;
    for (int &v : h) {
        x = x * 6364136223846793005ull + 1442695040888963407ull;
        v = (int)(x >> 32);
    }
    int *d_seed = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e = hipMalloc((void **)&d_seed, (h.size() + 1) * sizeof(int));
    if (e == hipSuccess) e = hipMemcpy(d_seed, h.data(), h.size() * sizeof(int), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    float ms = 0;
    // about 32 pipe cycles per instruction at roughly 1.6 GHz; the measured time is what counts
    const int iters = (int)std::max(1000.0, seconds * 1.6e9 / (32.0 * 8.0));
    if (e == hipSuccess) {
        hipLaunchKernelGGL(k_matrix_rate, dim3(n_cu), dim3(AM_THREADS), 0, st, d_seed, 1000, d_seed + 1024);
        (void)hipEventRecord(e0, st);
        hipLaunchKernelGGL(k_matrix_rate, dim3(n_cu), dim3(AM_THREADS), 0, st, d_seed, iters, d_seed + 1024);
        (void)hipEventRecord(e1, st);
        e = hipEventSynchronize(e1);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (d_seed) (void)hipFree(d_seed);
    if (e != hipSuccess || !(ms > 0)) {
        ctx->err = "the matrix-rate probe failed";
        return ENSI_E_HIP;
    }
    const double n_inst = (double)n_cu * 4 * (double)iters * 8;
    *ops_per_second = n_inst * 2.0 * 32 * 32 * 32 / (ms * 1e-3);
    return ENSI_OK;
}
