// Internal declarations shared by the library's translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include <map>
#include <string>
#include <vector>

#include "../../include/ensi.h"
#include "modarith.h"

#define ENSI_MAX_EXT 32   // max limbs of an extended basis (L + K)
#define ENSI_MAX_ALPHA 4
#define ENSI_MAX_K 4

// Per-prime constants, device-resident as one array indexed by prime id
// (0..L-1 = q chain, L..L+K-1 = p chain).
struct PrimeConst {
    u64 q;
    u64 qneg_inv;   // -q^{-1} mod 2^64
    u64 r2;         // 2^128 mod q   (to Montgomery form: mont_mul(x, r2))
    u64 n_inv;      // N^{-1} mod q
    u64 n_inv_s;    // its Shoup companion
    u64 pad[3];     // [0] 1 if this prime's transform tables hold doubles (fp64 path), [1] bits of 1/q, [2] bits of n_inv/q
};

// Which prime each limb row of a kernel's operand uses.
struct LimbMap {
    int32_t n;                  // limbs per polynomial in this operand
    int32_t prime[ENSI_MAX_EXT];
};

// Constants of the ModUp of one level (limbs = l1): per digit, per target limb.
struct ModUpConst {
    int32_t l1, K, alpha, beta;
    int32_t n_src[8];                               // limbs in digit j
    // device arrays
    u64 *inv;      // [beta][alpha]      (Q_j/q_i)^{-1} mod q_i
    u64 *inv_s;    // [beta][alpha]      Shoup companion
    u64 *hat;      // [beta][l1+K][alpha] (Q_j/q_i) mod t, Montgomery form (0 rows for limbs inside the digit)
};
struct ModDownConst {
    int32_t l1, K;
    u64 *inv;      // [K]   (P/p_k)^{-1} mod p_k
    u64 *inv_s;    // [K]
    u64 *hat;      // [l1][K]  (P/p_k) mod q_i, Montgomery form
    u64 *pinv;     // [l1]  P^{-1} mod q_i
    u64 *pinv_s;   // [l1]
    u64 *negtab;   // [l1][K+1]  j * (P mod q_i) mod q_i: what j negative centred residues add to the conversion
};

// Constants of the fused N = 2^16 key switch at one level (limbs = l1); all pointers device memory.
struct Ks16Const {
    int32_t l1, K, L, alpha, beta;
    int32_t n_src[8];          // limbs in digit j
    const u64 *inv, *inv_s;    // [l1]               (Q_j/q_a)^{-1} mod q_a of the digit that holds limb a, and its Shoup companion
    const u64 *hat_mont;       // [beta][ext][alpha] (Q_j/q_a) mod t, Montgomery form
    const double *hat_fp;      // [beta][ext][alpha][2]  the same value and value/t as doubles (targets below 2^50 only)
    const double *pmod_fp;     // [l1][2]            P mod q_i and (P mod q_i)/q_i
    const u64 *down_p;         // [K][2]             N^{-1} (P/p_k)^{-1} mod p_k and its Shoup companion
    const double *down_p_fp;   // [K][2]             the same value and value/p_k (special primes below 2^50 only)
    const double *down_q;      // [l1][2 + 4K]       N^{-1} P^{-1} mod q_i, /q_i; per k: p_k^{-1}, /q_i, 2^30 p_k^{-1}, /q_i
};

// One product of a plaintext multiplication: source ciphertext ([2][limb_stride][N] words) and plaintext index.
struct PmTerm {
    const u64 *src;
    int32_t pt;
    int32_t slot;  // set by the library: which of its group's distinct sources this is (a source that enters several
                   // products is transformed once)
};
// q_l^{-1} mod q_i and that divided by q_i, for the rescale that ends the fused plaintext multiplication
struct PmRescale {
    double w[ENSI_MAX_EXT], wp[ENSI_MAX_EXT];
};
// One group of outputs of out_o = Rescale(sum_t src_t (x) pt_t): outputs [0, n_out) of this group own the terms
// [begin[o], begin[o+1]) with begin[0] = t_base; every array is device memory.
struct PmGroup {
    const PmTerm *terms;    // whole table
    const int32_t *begin;   // this group's slice of the offsets: n_out + 1 entries
    int t_base, n_terms, n_out;
    const int32_t *owner;   // this group's distinct sources: owner[slot] = a term (index into the table) that names it
    int n_src;
    int l1, limb_stride_in;
    const u64 *pt;          // d_mont or d_fp of the plaintext batch
    int pt_limbs;
    u64 *ws_a, *ws_b, *ws_last;
    u64 *out;               // first output ciphertext of the group
    size_t out_stride;      // words between output ciphertexts
    int limb_stride_out;
};

// One ciphertext-ciphertext product as the host describes it: the two operand ciphertexts.
struct MmTerm {
    const u64 *a, *b;
    int32_t stride_a = 0;  // limb stride of a where it differs from the call's (0: the call's)
    int32_t pad = 0;
};
// On the device a group of outputs names every distinct operand ciphertext once ([2][limb_stride][N] words each), so
// that an operand shared by several products is gathered and transformed once, and its products as index pairs.
struct MmOperand {
    const u64 *p;  // where the operand lies
    const u64 *t;  // its transformed polynomials, [2][l1][N]: a slot of the group's operand array, or p itself
    int32_t limb_stride;
    int32_t pre;   // p already holds the transform (prepared operands, limb stride l1): neither gathered nor transformed
};
struct MmPair {
    int32_t a, b;
};
// One group of outputs of out_o = Rescale(Relin(sum_t a_t (x) b_t)); same conventions as PmGroup.
struct MmGroup {
    const MmOperand *ops;  // the group's operands; the first n_ops are gathered and transformed, prepared ones follow
    const MmPair *pairs;   // [n_terms], term t of the batch at index t - t_base
    const int32_t *begin;
    int t_base, n_terms, n_ops, n_out;
    int l1;
    int limbs_out;  // limbs copied to the output: l1 - 1 after the rescale, l1 without it
    int grid_x, grid_y;  // > 0: output x * grid_y + y sums, over j, a_(j,x) (x) b_(j,y): every output has the same number of
                         // terms in the same order, and outputs of a row share their left, of a column their right operands
    u64 *ws_a;   // [n_ops][2][l1][N] operand polynomials (transformed in place)
    u64 *ws_d;   // [n_out][3][l1][N]   d0, d2, d1: (d0, d2) is laid out like a ciphertext for the key switch
    u64 *ws_e;   // [n_out][2][l1][N]   relinearised product
    u64 *out;
    size_t out_stride;
    int limb_stride_out;
};

// One rotation to perform: everything the fused kernels need, device-resident.
struct RotDesc {
    const u64 *c0;      // source polynomial c0: [limb_stride_in][N]
    const u64 *digits;  // raised digits, transform domain: [beta][l1+K][N]
    const u64 *key;     // key: [beta_full][2][L+K][N], transform domain, Montgomery form
    u64 *out;           // destination ciphertext: [2][limb_stride_out][N]
    u32 g;              // Galois element
    u32 g_inv;          // its inverse mod 2N
    u32 accumulate;     // fused N = 2^16 kernels only: add the result to what `out` holds instead of overwriting it
    u32 pad;
};

// Everything about one ternary_matmul that depends only on (W, s, d, m, placement).
struct MatmulPlan {
    u64 hash;
    std::vector<int8_t> w_copy;  // the weights the plan was built from (cache hits are confirmed byte by byte)
    int s, d, m, placement, c_tot, n_in, l1;
    int n_v, n_rot;
    std::vector<int> vid;        // [n_in][c_tot] -> operand index or -1
    int n_kpad, m_pad, planes;   // matrix-core layout (planes = 0: not built, use the plain-ALU kernel)
    u32 *d_masks = nullptr;      // [tiles32][n_v][2] (+1 bits, -1 bits)
    int8_t *d_wt = nullptr;      // [m_pad][n_kpad] weights, operand index fastest
    int32_t *d_bias = nullptr;   // [m_pad] 128 * column sum of the weights
    double *d_bias_fp = nullptr; // [l1][m_pad] that offset times sum_p 256^p, reduced modulo each limb's prime (all primes below 2^50), else null
};

struct KernelTimer {
    std::string name;
    double ms = 0;
    int64_t count = 0;
};

// One pinned host buffer of the ring that carries small host arrays (descriptors, term tables, constants) to the
// device: the copy is asynchronous, and the buffer is reused only after the event recorded behind its copy has fired.
struct StageSlot {
    void *host = nullptr;
    size_t cap = 0;
    hipEvent_t ev = nullptr;
    bool pending = false;
};
#define ENSI_STAGE_SLOTS 8

struct ensi_ctx {
    ensi_params prm;
    int log_n, N, L, K, alpha;
    double scale;
    int device;
    std::vector<u64> primes;        // L + K
    std::vector<u64> psi;           // chosen 2N-th roots
    PrimeConst *d_pc = nullptr;     // [L+K]
    u64 *d_tw = nullptr;            // [L+K][4][N]: fwd, fwd Shoup, inv, inv Shoup
    double *d_cos = nullptr;        // [2N] cos(pi e / N)
    u32 *d_rot_exp = nullptr;       // [N/2] 5^j mod 2N
    std::vector<u32> rot_exp;
    std::map<int, ModUpConst> modup;      // by l1
    std::map<int, ModDownConst> moddown;  // by l1
    bool ks16 = false;                    // N = 2^16 and every ciphertext prime below 2^50: fused key-switching kernels
    std::map<int, Ks16Const> ks16c;       // by l1
    u64 *ws_y = nullptr; size_t ws_y_words = 0;   // inner factors of the basis conversion (ModUp)
    u64 *ws_ysp = nullptr; size_t ws_ysp_words = 0;  // centred special-limb residues (ModDown)
    // scratch for key switching, grown on demand
    u64 *ws_digits = nullptr; size_t ws_digits_words = 0;
    u64 *ws_u = nullptr; size_t ws_u_words = 0;
    RotDesc *ws_desc = nullptr; size_t ws_desc_n = 0;
    u64 *ws_virt = nullptr; size_t ws_virt_words = 0;   // unpacked (rotated) operands of the matmul
    u64 *ws_plan = nullptr; size_t ws_plan_words = 0;   // operand pointer table, small constants
    u64 *ws_xp = nullptr; size_t ws_xp_words = 0;       // byte planes of the accumulate's operands (one slice of the words)
    u64 *ws_pa = nullptr; size_t ws_pa_words = 0;       // plaintext multiplication: transformed sources of a group of outputs
    u64 *ws_pb = nullptr; size_t ws_pb_words = 0;       //   sums of products of the group
    u64 *ws_pl = nullptr; size_t ws_pl_words = 0;       //   centred last limbs of the group
    u64 *ws_pt = nullptr; size_t ws_pt_words = 0;       //   term table and offsets
    u64 *ws_rot = nullptr; size_t ws_rot_words = 0;     // rotated copies of the inputs of Alg. 2
    u64 *ws_ma = nullptr; size_t ws_ma_words = 0;       // ciphertext products: operand polynomials of a group
    u64 *ws_md = nullptr; size_t ws_md_words = 0;       //   (d0, d2, d1) per output
    u64 *ws_me = nullptr; size_t ws_me_words = 0;       //   relinearised products
    u64 *ws_mt = nullptr; size_t ws_mt_words = 0;       //   term table and offsets
    u64 *ws_rep = nullptr; size_t ws_rep_words = 0;     // CCMM: replicated elements of B
    u64 *ws_rtmp = nullptr; size_t ws_rtmp_words = 0;   //   rotated copy during a rotate-and-add step
    std::vector<MatmulPlan *> plans;                    // cached per weight matrix (weights are static server-side)
    int accumulate_mode = 0;                            // 0 auto, 1 plain-ALU kernel, 2 matrix-core kernel where valid
    int pmult_mode = 0;                                 // 0 auto, 1 always the generic kernels
    // sampler state for NULL randomness
    u64 sampler_ctr = 0;
    void *static_scratch = nullptr;  // this device's copy of the statically linked workspace (api_static.hip)
    size_t static_scratch_bytes = 0;
    StageSlot stage[ENSI_STAGE_SLOTS];
    int stage_next = 0;
    int n_cu = 0;                // compute units of the context's device (0: not queried yet)
    bool am_attr_set[4] = {false, false, false, false};  // dynamic LDS limit of the matrix-core accumulate kernels raised
    // timers
    bool profiling = false;
    std::vector<KernelTimer> timers;
    std::vector<std::pair<int, std::pair<hipEvent_t, hipEvent_t>>> pending;
    std::string err;
};

// Weights of one Alg. 1 product prepared once (ensi_weights_prepare): the plan, owned by the handle.
struct ensi_wt {
    ensi_ctx *ctx;
    MatmulPlan *plan;
    int limbs;
};
struct ensi_sk {
    ensi_ctx *ctx;
    std::vector<int8_t> s;  // host copy
    u64 *d_s_hat;           // [L+K][N] transform domain, Montgomery form
};
struct ensi_pk {
    ensi_ctx *ctx;
    u64 *d_pk;  // [2][L][N] transform domain, Montgomery form
};
struct ensi_gk {
    ensi_ctx *ctx;
    std::map<u32, u64 *> keys;  // Galois element -> device [beta][2][L+K][N]
};
struct ensi_pt {
    ensi_ctx *ctx;
    int n, limbs;
    double scale;
    u64 *d;  // [n][limbs][N] coefficient form
    // multiplier forms, built on first use by a plaintext multiplication
    mutable u64 *d_mont = nullptr;  // transform domain, Montgomery form
    mutable u64 *d_fp = nullptr;    // transform domain, doubles in [0,q), register order of the row pass (N = 2^16)
};
struct ensi_ct {
    ensi_ctx *ctx;
    int n, limbs, limbs_alloc;
    double scale;
    u64 *d;
    bool owns;
    bool prepared = false;  // holds transform-domain data that only ensi_ccmm_av reads (ensi_diagonalise_weights)
};

#define ENSI_FAIL(ctx, code, ...)                              \
    do {                                                       \
        char _b[512];                                          \
        snprintf(_b, sizeof(_b), __VA_ARGS__);                 \
        if (ctx) (ctx)->err = _b;                              \
        return (code);                                         \
    } while (0)

#define ENSI_HIP(ctx, expr)                                                                              \
    do {                                                                                                 \
        hipError_t _e = (expr);                                                                          \
        if (_e != hipSuccess) ENSI_FAIL(ctx, ENSI_E_HIP, "%s failed: %s", #expr, hipGetErrorString(_e)); \
    } while (0)

// ---- timers ---------------------------------------------------------------
int timer_id(ensi_ctx *ctx, const char *name);
void timer_begin(ensi_ctx *ctx, int id, hipStream_t st);
void timer_end(ensi_ctx *ctx, hipStream_t st);

struct ScopedTimer {
    ensi_ctx *c;
    hipStream_t st;
    bool on;
    ScopedTimer(ensi_ctx *ctx, const char *name, hipStream_t s) : c(ctx), st(s), on(ctx->profiling) {
        if (on) timer_begin(c, timer_id(c, name), st);
    }
    ~ScopedTimer() {
        if (on) timer_end(c, st);
    }
};

// ---- launchers (defined in the .hip files) ---------------------------------
// Transform n_inst limb rows in place; row r uses prime map.prime[r % map.n].
void launch_ntt(ensi_ctx *ctx, u64 *data, int n_inst, const LimbMap &map, bool inverse, hipStream_t st);
void launch_ntt16(ensi_ctx *ctx, u64 *data, int n_inst, const LimbMap &map, bool inverse, hipStream_t st);  // N = 2^16 only
void launch_ntt16_gather(ensi_ctx *ctx, u64 *data, const MmOperand *ops, int n_ops, int l1, hipStream_t st);  // N = 2^16 only

// fused key switch for N = 2^16 (keyswitch16.hip)
void launch_ks16_key_format(ensi_ctx *ctx, u64 *key, int beta_full, hipStream_t st);
// raises n_ct ciphertexts: dig [n_ct][beta*ext + l1][N] receives the transformed digits of c1 and P*c0
void launch_ks16_raise(ensi_ctx *ctx, const Ks16Const &kc, const u64 *ct_base, size_t ct_stride_words, int limb_stride, int n_ct,
                       u64 *ybuf, u64 *dig, hipStream_t st);
// inner product + inverse transform + ModDown for n_rot descriptors (desc.digits = the ciphertext's block of dig)
// members > 1: the descriptors come in groups of `members` rotations of one ciphertext (same digits and destination);
// a group's inner products are added before one inverse transform and one ModDown
void launch_ks16_switch(ensi_ctx *ctx, const Ks16Const &kc, const RotDesc *d_desc, int n_rot, u64 *u, u64 *ysp, int limb_stride_out,
                        hipStream_t st, int members = 1);

void launch_modup(ensi_ctx *ctx, const ModUpConst &mc, const u64 *ct_base, size_t ct_stride_words, int limb_stride,
                  int n_ct, u64 *digits, hipStream_t st);
void launch_inner(ensi_ctx *ctx, const RotDesc *d_desc, int n_rot, int l1, int beta, u64 *u, hipStream_t st);
void launch_moddown(ensi_ctx *ctx, const ModDownConst &mc, const RotDesc *d_desc, int n_rot, int limb_stride_in,
                    int limb_stride_out, const u64 *u, hipStream_t st);
// operand v of the signed sums is the ciphertext at xbase + v*xstride words
void launch_accumulate(ensi_ctx *ctx, const u64 *xbase, size_t xstride, int n_v, const u32 *d_masks, int m, int l1,
                       int limb_stride_in, u64 *out, int limb_stride_out, hipStream_t st);
// d_fconsts != nullptr selects the fp64 kernel (all active primes below 2^50)
void launch_rescale(ensi_ctx *ctx, u64 *ct, int n_ct, int l1, int limb_stride, const u64 *d_consts, const double *d_fconsts,
                    hipStream_t st);
// planes: 5 or 7 byte planes contracted; weights d_wt in fragment order [m_pad/256][n_kpad/32][4][2][64][16], n_kpad a
// multiple of 256.  Grows ctx->ws_xp (byte planes of a slice of the operand words); returns an ENSI_E_* code.
// d_rescale != nullptr: operands are read at l1 + 1 limbs and multiplied/rescaled on the fly (fp64 constants [5][l1+1]).
int launch_accumulate_mfma(ensi_ctx *ctx, const u64 *xbase, size_t xstride, int n_v, int n_kpad, const int8_t *d_wt, const int32_t *d_bias,
                           const double *d_bias_fp,
                           int planes, int m, int l1, int limb_stride_in, u64 *out, int limb_stride_out, const double *d_rescale,
                           hipStream_t st);
// sustained int8 matrix-instruction rate over the whole chip, measured for about `seconds`
int launch_matrix_rate(ensi_ctx *ctx, double seconds, double *ops_per_second, hipStream_t st);

// plaintext multiplication (pmult.hip).  The generic pair works for every ring size and prime; the fused one needs
// N = 2^16 and ciphertext primes below 2^50.
void launch_pm_generic(ensi_ctx *ctx, const PmGroup &g, const u64 *d_consts, const double *d_fconsts, hipStream_t st);
void launch_pm16(ensi_ctx *ctx, const PmGroup &g, const PmRescale &rs, hipStream_t st);
void launch_pm16_pt_format(ensi_ctx *ctx, const u64 *ntt_form, int n_rows, u64 *out, hipStream_t st);

// ciphertext-ciphertext products (ccmm.hip)
void launch_mm_tensor(ensi_ctx *ctx, const MmGroup &g, hipStream_t st);
void launch_mm_add_d1(ensi_ctx *ctx, const MmGroup &g, hipStream_t st);
void launch_mm_scatter(ensi_ctx *ctx, const MmGroup &g, hipStream_t st);
// a += b on batches of n ciphertexts with l1 active limbs and their own limb strides
void launch_ct_add(ensi_ctx *ctx, u64 *a, int stride_a, const u64 *b, int stride_b, int l1, int n, hipStream_t st);

void launch_small_to_rns(ensi_ctx *ctx, const int8_t *d_in, int n_poly, const LimbMap &map, u64 *out, hipStream_t st);
void launch_i64_to_rns(ensi_ctx *ctx, const int64_t *d_in, int n_poly, const LimbMap &map, u64 *out, hipStream_t st);
void launch_uniform(ensi_ctx *ctx, u64 *out, const LimbMap &map, u64 seed, u64 stream_id, hipStream_t st);
// out = a (.) b_mont  (+ add) per limb row; rows cycle through map
void launch_mul_mont(ensi_ctx *ctx, u64 *out, const u64 *a, const u64 *b_mont, int n_rows, const LimbMap &map,
                     hipStream_t st);
void launch_add(ensi_ctx *ctx, u64 *out, const u64 *a, const u64 *b, int n_rows, const LimbMap &map, hipStream_t st);
void launch_to_mont(ensi_ctx *ctx, u64 *data, int n_rows, const LimbMap &map, hipStream_t st);
// stored key words (Montgomery form, or doubles on the limbs the fused N = 2^16 kernels read as such) -> ordinary residues
void launch_key_to_plain(ensi_ctx *ctx, u64 *data, int n_rows, const LimbMap &map, bool fp_format, hipStream_t st);
// *d_bad += number of words >= their prime
void launch_count_noncanonical(ensi_ctx *ctx, const u64 *data, int n_rows, const LimbMap &map, unsigned int *d_bad, hipStream_t st);
// d_sums[c] += wrap-around sum of the active limb words of ciphertext c
void launch_ct_checksum(ensi_ctx *ctx, const u64 *ct, int n, int l1, int limb_stride, u64 *d_sums, hipStream_t st);
// b = -a*s + e (+ factor[row] * sg), all transform domain; s_mont in Montgomery form; writes b in Montgomery form
void launch_key_assemble(ensi_ctx *ctx, u64 *b_out, const u64 *a, const u64 *s_mont, const u64 *e, const u64 *sg,
                         const u64 *d_factor, const LimbMap &map, hipStream_t st);
void launch_automorphism_coef(ensi_ctx *ctx, u64 *out, const u64 *in, const LimbMap &map, u32 g_inv, hipStream_t st);
// plaintext y of the batch holds its n_slots values in slots [slot0 + y*slot_step, ...+n_slots), zeros elsewhere
// (allocates its transform workspace, waits for the stream and frees it again; so does launch_decode)
hipError_t launch_encode(ensi_ctx *ctx, const double *d_slots, int n_pt, int n_slots, int slot0, int slot_step, double scale,
                         int64_t *d_coeffs, hipStream_t st);
void launch_crt_center(ensi_ctx *ctx, const u64 *m, int n_ct, int n_limbs_used, double *out, hipStream_t st);
void launch_center_i64(ensi_ctx *ctx, const u64 *m, size_t stride_words, int n, int64_t *out, hipStream_t st);
hipError_t launch_decode(ensi_ctx *ctx, const double *d_coeffs, int n_ct, int slot_begin, int n_slots, double inv_scale, double *d_out,
                         hipStream_t st);
