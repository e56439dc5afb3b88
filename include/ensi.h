/*
 * ensi.h -- C ABI of the MI355X (gfx950) library for CKKS-encrypted ternary
 * matrix multiplication: the multiplication-free plaintext-ciphertext product
 * of the ENSI paper (Alg. 1, PCMM) under column-wise SIMD packing, together
 * with the CKKS primitives it stands on (Preliminaries: KeyGen, Encryption,
 * Decryption, Addition, Rotation).
 *
 * Conventions
 *   - Every function returns 0 on success or a negative ENSI_E_* code; a
 *     message for the last failure on a context is kept by ensi_last_error().
 *     Nothing throws across this boundary.
 *   - "host" pointers are ordinary CPU memory borrowed for the duration of the
 *     call; "device" pointers are HIP device memory on the context's GPU.
 *   - Handles are opaque, owned by the caller, and released with the matching
 *     *_free.  A ciphertext handle is a BATCH of n ciphertexts stored
 *     contiguously on the device as u64 words [n][2][limbs_alloc][N]:
 *     polynomial-major, then RNS limb, then coefficient (unit stride),
 *     coefficient form, canonical residues in [0, q_i).  Only the first
 *     `limbs` (<= limbs_alloc) limbs of each polynomial are active.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work on it and return; results are ready after the stream
 *     is synchronised.  Calls that return host data synchronise themselves.
 *     A context serves ONE stream at a time: its workspaces are shared by all
 *     calls, so calls on one context must not overlap on different streams (use
 *     one context per concurrent stream).  Workspaces grow on demand (a device
 *     allocation inside the call the first time a larger size is needed).
 *   - Ring degree N = 2^log_n, n = N/2 slots.  Primes: q_0..q_{L-1} of q_bits
 *     bits and p_0..p_{K-1} of p_bits bits, the largest primes = 1 mod 2N
 *     below 2^bits, descending (P chain skips members of the Q chain).
 *   - Random material is either passed in (int8 host arrays: ternary
 *     polynomials, small error polynomials) or, where the pointer is NULL,
 *     drawn by the library: from the operating system's cryptographic generator
 *     when params.seed is 0 (the only setting fit for real keys), from a
 *     deterministic generator keyed by params.seed otherwise.  THE SEEDED PATH IS
 *     FOR REPRODUCIBLE TESTS AND BENCHMARKS ONLY: the seed is a public parameter,
 *     so a secret key drawn from it is predictable.  Uniform ring elements (the
 *     public halves of keys, which need no secrecy) come from
 *     a counter-based generator keyed by (seed, stream id, prime index):
 *       mix(z): z^=z>>30; z*=0xBF58476D1CE4E5B9; z^=z>>27; z*=0x94D049BB133111EB; z^=z>>31
 *       key = mix(mix(mix(seed)+stream)+prime_index)
 *       coefficient i = (mix(key+G*(2i+1))*2^64 + mix(key+G*(2i+2))) mod q,  G=0x9E3779B97F4A7C15
 *     with stream 1 for the public key and (2<<56)|(g<<8)|digit for the key of
 *     Galois element g.
 */
#ifndef ENSI_H
#define ENSI_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ENSI_OK 0
#define ENSI_E_BADARG -1 /* null pointer, value out of range, weight outside {-1,0,1} */
#define ENSI_E_NOKEY -2  /* a needed rotation step has no Galois key in the key set */
#define ENSI_E_LEVEL -3  /* operands at different levels, or no limb left to drop */
#define ENSI_E_SHAPE -4  /* batch sizes / layout do not fit together */
#define ENSI_E_NOMEM -5  /* device or host allocation failed */
#define ENSI_E_HIP -6    /* a HIP runtime call failed */

#define ENSI_PLACE_ZERO 0     /* every output column in slot block 0 */
#define ENSI_PLACE_DIAGONAL 1 /* output column i in slot block i mod c_tot */

typedef struct ensi_ctx ensi_ctx;
typedef struct ensi_sk ensi_sk;
typedef struct ensi_pk ensi_pk;
typedef struct ensi_gk ensi_gk;
typedef struct ensi_pt ensi_pt;
typedef struct ensi_ct ensi_ct;
typedef struct ensi_wt ensi_wt;

typedef struct ensi_params {
    int32_t log_n;     /* ring degree N = 2^log_n, 4 <= log_n <= 16 */
    int32_t q_bits;    /* bit size of the ciphertext primes (<= 60) */
    int32_t q_count;   /* L: number of ciphertext primes (<= 28) */
    int32_t p_bits;    /* bit size of the special primes (<= 61) */
    int32_t p_count;   /* K: number of special primes (1..4) */
    int32_t alpha;     /* limbs per key-switching digit (1..4) */
    int32_t log_scale; /* encoding scale Delta = 2^log_scale */
    uint64_t seed;     /* 0: NULL randomness is drawn from the operating system's cryptographic generator;
                          non-zero: from a deterministic generator keyed by this value (tests and benchmarks only) */
} ensi_params;

/* ---- context ----------------------------------------------------------- */
/* Finds the primes, builds transform tables and conversion constants and
 * uploads them to the current HIP device. */
int ensi_ctx_create(const ensi_params *params, ensi_ctx **out);
void ensi_ctx_free(ensi_ctx *ctx);
const char *ensi_last_error(const ensi_ctx *ctx); /* string owned by ctx; "" if none */
/* q: host[L], p: host[K] */
int ensi_get_primes(const ensi_ctx *ctx, uint64_t *q, uint64_t *p);

/* ---- keys (Preliminaries, KeyGen) -------------------------------------- */
/* s: host int8[N] ternary secret; e: host int8[N] error; either may be NULL
 * (library samples).  pk = (-a s + e, a) over Q_L, a = counter stream 1 of
 * seed_a. */
int ensi_keygen(ensi_ctx *ctx, const int8_t *s, const int8_t *e, uint64_t seed_a, ensi_sk **sk, ensi_pk **pk);
void ensi_sk_free(ensi_sk *sk);
void ensi_pk_free(ensi_pk *pk);
/* One hybrid key-switching key per rotation step (duplicates are merged).
 * e: host int8[n_steps][beta][N] errors (beta = ceil(L/alpha)) or NULL. For
 * step k the Galois element is g = 5^(k mod n) mod 2N, and for each digit j
 * (b_j, a_j) over Q_L*P with b_j = -a_j s + e_j + [P]_{q_i} phi_g(s) on the
 * limbs i of digit j only. */
int ensi_galois_keygen(ensi_ctx *ctx, const ensi_sk *sk, const int32_t *steps, int32_t n_steps, const int8_t *e,
                       uint64_t seed_a, ensi_gk **gk);
void ensi_gk_free(ensi_gk *gk);

/* ---- key import / export (System model: the client generates the keys, the server holds only the public and
 *      evaluation keys; Preliminaries, KeyGen) ---------------------------------------------------------------
 * Key material crosses the boundary in coefficient form as canonical residues in [0, prime): what a client
 * produced elsewhere (or another implementation of the same key definitions) can be loaded without the secret
 * key ever reaching this process.  Imports check every word and fail with ENSI_E_BADARG on a value that is not
 * below its prime.
 * sk: host int8[N], ternary coefficients.
 * pk: host u64[2][L][N] = (b, a) with b = -a s + e over Q_L.
 * A switching key (Galois key of one rotation step, or the evaluation key of Mult under step 0, i.e. the identity
 * element): host u64[beta][2][L+K][N], digit-major, per digit (b_j, a_j) over Q_L + P, beta = ceil(L/alpha).
 * ensi_gk_import adds the key of `step` to *gk (a NULL *gk is created; an existing key of that step is replaced).
 * ensi_gk_elements writes the Galois elements g = 5^step mod 2N of the keys a set holds (capacity cap) and returns
 * their number. */
int ensi_sk_import(ensi_ctx *ctx, const int8_t *s, ensi_sk **sk);
int ensi_sk_export(ensi_ctx *ctx, const ensi_sk *sk, int8_t *s);
int ensi_pk_import(ensi_ctx *ctx, const uint64_t *words, ensi_pk **pk);
int ensi_pk_export(ensi_ctx *ctx, const ensi_pk *pk, uint64_t *words);
int ensi_gk_import(ensi_ctx *ctx, ensi_gk **gk, int32_t step, const uint64_t *words);
int ensi_gk_export(ensi_ctx *ctx, const ensi_gk *gk, int32_t step, uint64_t *words);
int ensi_gk_elements(const ensi_gk *gk, int32_t *elements_out, int32_t cap);

/* ---- plaintexts (column-wise SIMD encoding, pi) ------------------------- */
/* slots: host double[n_pt][n_slots] real values, zero-padded to N/2 slots.
 * Slot j sits at the root exp(i pi 5^j / N); coefficients are
 * round-half-away((2 Delta/N) sum_j z_j cos(pi 5^j k / N)).  `limbs` = number
 * of active Q limbs (level + 1). */
int ensi_encode(ensi_ctx *ctx, const double *slots, int32_t n_pt, int32_t n_slots, int32_t limbs, ensi_pt **pt);
/* The same encoding at another scale (1 <= scale < 2^63 / max|slot|), e.g. the prime a following rescale
 * drops, so that multiplying by the plaintext and rescaling leaves a ciphertext's scale unchanged. */
int ensi_encode_at(ensi_ctx *ctx, const double *slots, int32_t n_pt, int32_t n_slots, int32_t limbs, double scale, ensi_pt **pt);
/* Sets the scale a plaintext batch is taken to be encoded at (imported coefficients start at the context's). */
int ensi_pt_set_scale(ensi_pt *pt, double scale);
/* coeffs: host int64[n_pt][N] signed integer coefficients (already encoded). */
int ensi_pt_import(ensi_ctx *ctx, const int64_t *coeffs, int32_t n_pt, int32_t limbs, ensi_pt **pt);
/* coeffs: host int64[n_pt][N], centred representative of limb 0 (exact only while |m| < q_0/2). */
int ensi_pt_export(ensi_ctx *ctx, const ensi_pt *pt, int64_t *coeffs);
void ensi_pt_free(ensi_pt *pt);

/* ---- ciphertexts -------------------------------------------------------- */
/* Allocates an (uninitialised) batch on the device. */
int ensi_ct_alloc(ensi_ctx *ctx, int32_t n, int32_t limbs, ensi_ct **ct);
/* Wraps caller-owned device memory of n*2*limbs*N u64 words (e.g. a PyTorch
 * int64 tensor); the caller keeps ownership and must keep it alive. */
int ensi_ct_wrap(ensi_ctx *ctx, void *device_words, int32_t n, int32_t limbs, double scale, ensi_ct **ct);
void ensi_ct_free(ensi_ct *ct);
int ensi_ct_info(const ensi_ct *ct, int32_t *n, int32_t *limbs, double *scale, void **device_words);
/* host u64[n][2][limbs][N], compact (active limbs only). */
int ensi_ct_export(ensi_ctx *ctx, const ensi_ct *ct, uint64_t *limbs_out);
int ensi_ct_import(ensi_ctx *ctx, const uint64_t *limbs_in, int32_t n, int32_t limbs, double scale, ensi_ct **ct);
/* sums: host u64[n]; sums[c] = the sum modulo 2^64 of all active limb words of ciphertext c (both polynomials).
 * A whole batch can be compared with a reference (or with another kernel's result) without downloading it, e.g.
 * the outputs of Alg. 1 at sizes where only sampled outputs can be recomputed.  Synchronises the stream. */
int ensi_ct_checksum(ensi_ctx *ctx, const ensi_ct *ct, uint64_t *sums, void *stream);

/* Enc_pk: ct_i = v_i pk + (m_i + e0_i, e1_i).  v, e0, e1: host int8[n_pt][N] or
 * NULL (all three given or all three NULL). */
int ensi_encrypt(ensi_ctx *ctx, const ensi_pk *pk, const ensi_pt *pt, const int8_t *v, const int8_t *e0,
                 const int8_t *e1, ensi_ct **ct);
/* Dec_sk then decode: slots_out host double[n][n_slots] = real parts of slots
 * [slot_begin, slot_begin+n_slots) of c0 + c1 s (CRT of limbs 0,1, centred,
 * divided by the ciphertext's scale). */
int ensi_decrypt(ensi_ctx *ctx, const ensi_sk *sk, const ensi_ct *ct, int32_t slot_begin, int32_t n_slots,
                 double *slots_out);

/* ---- Rot (Preliminaries, Rotation): out_i = Rot(in_i; steps[i]) --------- */
/* Cyclic left shift of the slot vector by steps[i] (negative = inverse
 * rotation), by the automorphism X -> X^g and hybrid key switching:
 * digit-decompose c1, ModUp each digit to Q_l + P (fast basis conversion, no
 * correction), automorphism, inner product with the key, ModDown (basis
 * conversion P -> Q_l on centred residues, so the division error is zero-mean),
 * add phi_g(c0).  steps: host int32[n].  in and out are batches of
 * equal n and limbs and must not overlap.  Level and scale are unchanged. */
int ensi_rotate(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *in, const int32_t *steps, ensi_ct *out, void *stream);

/* ---- Rot without allocation ---------------------------------------------- */
/* For callers that cannot allocate device memory while they run: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same result (word for word) and same errors as
 * ensi_rotate, but every intermediate (descriptors, raised digits, accumulators, conversion residues) lives in a
 * workspace that is linked into the library as a device array instead of being allocated: 96 MiB, held by every GPU
 * the library runs on from load time to the end of the process.  The call allocates and frees nothing (the
 * constants of every level, the pinned staging ring and the workspace's address are set up by ensi_ctx_create);
 * the per-kernel timers must be off.  Limits: at most 64 ciphertexts per call and
 *   n * (beta (l+K) + 3 l + 4 K) * 8 N  (+ n * l * 8 N on rings of 2^16 with ciphertext primes below 2^50)  bytes
 * <= 96 MiB, l = in.limbs, beta = ceil(l / alpha) -- one ciphertext of the 2^16 ring at 16 + 4 limbs (80 MiB), the
 * full 64 on the 2^12 ring at 3 + 1; anything larger fails with ENSI_E_SHAPE and a message that names the size.  All calls on one GPU share that
 * one workspace, whatever context or stream they use, and it keeps the previous call's contents: calls that
 * overlap in time on one GPU race (each call overwrites everything it later reads, so nothing needs clearing
 * between calls that do not overlap). */
int ensi_rotate_static(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *in, const int32_t *steps, ensi_ct *out, void *stream);

/* ---- Alg. 1 (PCMM): Y = X W on ciphertexts, additions/subtractions only - */
/* in : ceil(d/c_tot) packed ciphertexts, c_tot = (N/2)/s; ciphertext G holds
 *      activation column G*c_tot+b (s tokens) in slots [b*s,(b+1)*s).  c_tot=1
 *      is one column per ciphertext (the paper's own packing) and needs no key.
 * W  : host int8[d][m], row-major, values in {-1,0,+1}.
 * out: batch of m ciphertexts; out_i carries column i of Y in slot block p_i
 *      (placement); its other blocks are unspecified.  Same level/scale as in.
 * Packed inputs are first unpacked into column-aligned operands by rotations
 * (one ModUp per packed input, shared by all its rotations; gk must hold a key
 * for step rho*s for every needed rho), then every output is the signed sum of
 * its operands limb-wise mod q_i (zero weights skipped; an all-zero weight
 * column gives the all-zero ciphertext). */
int ensi_ternary_matmul(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *in, int32_t s, int32_t d, const int8_t *W,
                        int32_t m, int32_t placement, ensi_ct *out, void *stream);

/* Selects the kernel that forms the signed sums of Alg. 1: 0 = automatic (the
 * int8 matrix-core contraction over byte planes whenever N >= 32 and the exact
 * sum of the operands fits a signed 64-bit word, else the plain-ALU kernel), 1 = always the
 * plain-ALU kernel, 2 = same as 0.  Both give identical residues. */
int ensi_set_accumulate_mode(ensi_ctx *ctx, int32_t mode);

/* Diagnostics for the measurement of Alg. 1's contraction: runs a register-only
 * loop of the int8 matrix instruction the contraction is built from (one
 * workgroup of four waves per compute unit, no memory traffic) for about
 * `seconds` (0 < seconds <= 2) and returns the operations per second the chip
 * sustains at the clock it holds under that load -- the ceiling the contraction
 * can be compared with besides the data-sheet peak.  ops_per_second: host
 * pointer.  Returns after the probe has finished. */
int ensi_matrix_rate_probe(ensi_ctx *ctx, double seconds, double *ops_per_second, void *stream);

/* ---- scalar multiply + rescale (between two PCMM layers) ---------------- */
/* In place on the whole batch: c <- c * round(kappa q_l) mod q_i, then limb l
 * is dropped: c_i <- (c_i - [c_l]) q_l^{-1} mod q_i with [c_l] the centred
 * representative of limb l (division with rounding to nearest).  limbs decreases
 * by one (limbs_alloc is unchanged).  The encoded values are multiplied by
 * kappa (0 < |kappa| < 1); the scale absorbs only the rounding of the constant:
 * scale' = scale * round(kappa q_l) / (kappa q_l). */
int ensi_mul_scalar_rescale(ensi_ctx *ctx, ensi_ct *ct, double kappa, void *stream);

/* The step between two PCMM layers and the second layer (Alg. 1) as one call: the same result as
 * ensi_mul_scalar_rescale(in, kappa) followed by ensi_ternary_matmul(NULL, in, s = N/2, d = in->n, W, m,
 * ENSI_PLACE_ZERO, out), i.e. `in` holds one activation column per ciphertext (the paper's own packing, no
 * rotations) and out_i = sum_j W[j][i] * rescale(kappa * in_j).  W: host int8[in->n][m].  out: batch of m
 * ciphertexts with one limb less than `in`.  Where the matrix-core path applies (all active primes below
 * 2^50), the rescaled operands are formed while the accumulate reads them and never written to memory.
 * `in` is consumed: its handle takes the level and scale of the rescaled batch, its words are unspecified
 * afterwards (rescaled in place or left as they were). */
int ensi_rescale_ternary_matmul(ensi_ctx *ctx, ensi_ct *in, double kappa, const int8_t *W, int32_t m, ensi_ct *out, void *stream);

/* ---- Alg. 1 with the weights prepared once ------------------------------- */
/* The weights of a layer are fixed while activations change (System model: the server holds W in the clear), so
 * everything Alg. 1 derives from W alone -- which operands exist, the weight of each operand in each output in the
 * layout the kernels read, the validation of the values -- can be built once, outside the step.
 * ensi_weights_prepare does that for inputs at `limbs` limbs (W, s, d, m, placement as for ensi_ternary_matmul; W is
 * not referenced after the call); ensi_ternary_matmul_prepared and ensi_rescale_ternary_matmul_prepared then compute
 * exactly what ensi_ternary_matmul and ensi_rescale_ternary_matmul compute (for the latter the weights are prepared
 * with s = N/2, d = in.n, ENSI_PLACE_ZERO and limbs = in.limbs - 1).  The plain entry points keep a small cache of
 * plans instead, looked up by a hash of W and confirmed by comparing W byte by byte. */
int ensi_weights_prepare(ensi_ctx *ctx, const int8_t *W, int32_t s, int32_t d, int32_t m, int32_t placement, int32_t limbs, ensi_wt **wt);
void ensi_weights_free(ensi_wt *wt);
int ensi_ternary_matmul_prepared(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *in, const ensi_wt *wt, ensi_ct *out, void *stream);
int ensi_rescale_ternary_matmul_prepared(ensi_ctx *ctx, ensi_ct *in, double kappa, const ensi_wt *wt, ensi_ct *out, void *stream);

/* ---- PMult (Preliminaries, Multiplication) summed and rescaled once ------ */
/* out_o = Rescale( sum_{t in [begin[o], begin[o+1])} in[term_ct[t]] (x) pt[term_pt[t]] ),  o = 0..n_out-1.
 * A product multiplies both ciphertext polynomials by the plaintext polynomial in R_{Q_l}; the products of one
 * output are added at the product scale and limb l is dropped once: c_i <- (c_i - [c_l]) q_l^{-1} mod q_i with
 * [c_l] the centred representative.  begin: host int32[n_out+1], begin[0] = 0, non-decreasing; term_ct, term_pt:
 * host int32[begin[n_out]], indices into the batches `in` and `pt` (pt needs at least in's limbs; an output
 * without terms is the zero ciphertext).  out: batch of n_out ciphertexts with one limb less than `in`, must not
 * overlap `in`; its scale becomes in.scale * pt.scale / q_l.  The plaintext batch is transformed on its first
 * use and keeps that form until freed. */
int ensi_pmult_sum_rescale(ensi_ctx *ctx, const ensi_ct *in, const ensi_pt *pt, const int32_t *begin, const int32_t *term_ct,
                           const int32_t *term_pt, int32_t n_out, ensi_ct *out, void *stream);
/* Selects the kernels of the plaintext multiplication: 0 = automatic (the fused N = 2^16 kernels whenever the
 * ring is 2^16 and every ciphertext prime is below 2^50, else the generic ones), 1 = always the generic
 * kernels.  Both give identical residues. */
int ensi_set_pmult_mode(ensi_ctx *ctx, int32_t mode);

/* ---- merge of block-placed outputs into packed ciphertexts --------------- */
/* Not in the paper: with several activation columns per ciphertext (c_tot = (N/2)/s), Alg. 1 leaves output
 * column i in slot block i mod c_tot of its own ciphertext (ENSI_PLACE_DIAGONAL); masking each output to its
 * block and adding c_tot of them gives the packed form the next layer reads:
 *   out_G = Rescale( sum_{b < c_tot} in[G c_tot + b] (x) mask_b ),  G = 0..ceil(in.n / c_tot)-1,
 * mask_b = 1 on slots [b s, (b+1) s), 0 elsewhere.  ensi_block_masks encodes the c_tot masks at `limbs` limbs and
 * scale q_{limbs-1} (the prime the rescale drops: the ciphertext scale is unchanged). */
int ensi_block_masks(ensi_ctx *ctx, int32_t s, int32_t c_tot, int32_t limbs, ensi_pt **pt);
int ensi_merge(ensi_ctx *ctx, const ensi_ct *in, const ensi_pt *masks, int32_t c_tot, ensi_ct *out, void *stream);

/* ---- Alg. 2 (secure RoPE) ----------------------------------------------- */
/* out_i = in_i (x) cos + (Rot(in_i; 1) (x) neg + Rot(in_i; -1) (x) pos) (x) sin with neg = (-1,0,-1,0,...),
 * pos = (0,1,0,1,...): slot 2k becomes x_2k cos_2k - x_2k+1 sin_2k, slot 2k+1 becomes x_2k+1 cos_2k+1 +
 * x_2k sin_2k+1.  The 0/+-1 masks are applied to the sin vector in the clear, so the protocol costs the one
 * level the paper's operation table gives it: ensi_rope_plaintexts encodes cos, neg (.) sin and pos (.) sin
 * (host double[n_slots] each) at `limbs` limbs and scale q_{limbs-1}, and ensi_rope evaluates
 *   out_i = Rescale( in_i (x) pt_0 + Rot(in_i; 1) (x) pt_1 + Rot(in_i; -1) (x) pt_2 )
 * with one ModUp per input shared by its two rotations.  gk must hold keys for steps +1 and -1.  out: batch of
 * in.n ciphertexts with one limb less than `in`, must not overlap it. */
int ensi_rope_plaintexts(ensi_ctx *ctx, const double *cos_v, const double *sin_v, int32_t n_slots, int32_t limbs, ensi_pt **pt);
int ensi_rope(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *in, const ensi_pt *pt, ensi_ct *out, void *stream);

/* ---- Mult (Preliminaries, Multiplication) and the CCMM section ---------- */
/* Evaluation key (Preliminaries, KeyGen: evk): the hybrid key-switching key from s^2 to s, same digit structure as
 * a Galois key; e: host int8[beta][N] or NULL; the uniform parts are the streams (3 << 56) | j of seed_a.  The
 * returned key set holds only this key; free with ensi_gk_free. */
int ensi_relin_keygen(ensi_ctx *ctx, const ensi_sk *sk, const int8_t *e, uint64_t seed_a, ensi_gk **rk);
/* Level alignment: the handle's ciphertexts are read modulo Q_{limbs} from now on (limbs <= current limbs; the
 * scale and the words are unchanged). */
int ensi_ct_drop_limbs(ensi_ct *ct, int32_t limbs);
/* out_o = Rescale( Relin( sum_{t in [begin[o], begin[o+1])} a[term_a[t]] (x) b[term_b[t]] ) ),  o = 0..n_out-1.
 * A product is the tensor product (a0 b0, a0 b1 + a1 b0, a1 b1) in R_{Q_l}; the products of one output are added,
 * the third polynomial is switched from s^2 to s with the evaluation key (decompose, ModUp, inner product,
 * ModDown, as in ensi_rotate with the identity automorphism) and limb l is dropped once with rounding to nearest.
 * a, b: batches at the same number of limbs; begin/term_a/term_b as in ensi_pmult_sum_rescale; out: n_out
 * ciphertexts with one limb less, not overlapping a or b; out.scale = a.scale * b.scale / q_l. */
int ensi_mult_sum_relin_rescale(ensi_ctx *ctx, const ensi_gk *rk, const ensi_ct *a, const ensi_ct *b, const int32_t *begin,
                                const int32_t *term_a, const int32_t *term_b, int32_t n_out, ensi_ct *out, void *stream);
/* The rotate-and-add fill used by the element extraction below, t <- sum_{e < r_end / r_begin} Rot(t; sign e r_begin)
 * (r_end / r_begin a power of two): while two doublings remain they are taken as one step of radix four,
 * t <- t + Rot(t; r) + Rot(t; 2r) + Rot(t; 3r), whose three rotations share one ModUp of t; a last single doubling is
 * t <- t + Rot(t; r).  ensi_fill_steps writes the rotation steps this schedule uses (the Galois keys a caller has to
 * provide) to steps_out (capacity cap) and returns their number (or a negative ENSI_E_* code). */
int ensi_fill_steps(int32_t r_begin, int32_t r_end, int32_t sign, int32_t *steps_out, int32_t cap);
/* Element extraction of the CCMM section: out_o holds, in every slot, the value that slot k_o of in[src[o]] held:
 * one product with the one-hot mask masks[mask_idx[o]] (1 in slot k_o, else 0) and one rescale, then the fill
 * over all N/2 slots (the figure with the paper's own schedule is not part of its text; this schedule has the
 * logarithmic rotation count it states).  gk must hold keys for ensi_fill_steps(1, N/2, 1).  ensi_one_hot_masks encodes the masks of slots 0..count-1 at `limbs` limbs and scale
 * q_{limbs-1}.  src, mask_idx: host int32[n_out]; out: n_out ciphertexts with one limb less than `in`. */
int ensi_one_hot_masks(ensi_ctx *ctx, int32_t count, int32_t limbs, ensi_pt **pt);
int ensi_replicate(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *in, const int32_t *src, const ensi_pt *masks,
                   const int32_t *mask_idx, int32_t n_out, ensi_ct *out, void *stream);
/* C = A B on ciphertexts (CCMM section): A: d column ciphertexts (a_j = column j of A, tokens along the slots),
 * B: m column ciphertexts (b_i holds B[j][i] in slot j for j < d and ZERO in every other slot), both at the same
 * number of limbs l;  c_i = Rescale(Relin(sum_j a_j (x) b_i^(j))) with b_i^(j) = B[j][i] replicated into every
 * slot.  Element extraction in two stages, `period` a power of two with d <= period <= N/2: per column, the fill
 * with steps period, 2 period, ... makes it periodic (u[p] = b[p mod period], no level); per element, one product
 * with masks[j] (1 in the slots congruent to j modulo period) and one rescale, then the fill over a period.  (The figure with the paper's own
 * baby-step giant-step schedule is not part of its text; this one shares the giant steps among the elements of a
 * column.)  gk must hold keys for ensi_fill_steps(period, N/2, 1) and ensi_fill_steps(1, period, 1); masks: at least d plaintexts from
 * ensi_periodic_masks(period, count >= d, limbs = l); a_j is read at the level of the replicated elements.
 * out: m ciphertexts with l - 2 limbs. */
int ensi_periodic_masks(ensi_ctx *ctx, int32_t period, int32_t count, int32_t limbs, ensi_pt **pt);
int ensi_ccmm(ensi_ctx *ctx, const ensi_gk *rk, const ensi_gk *gk, const ensi_ct *A, const ensi_ct *B, const ensi_pt *masks,
              int32_t period, ensi_ct *out, void *stream);

/* The same product with several heads per ciphertext (the column-encoded by row-encoded form of the CCMM section,
 * e.g. Q K^T): ciphertext j of A holds column j of every A_h, head h in slot block h (s slots per block, s a power
 * of two); ciphertext j of B holds B_h[j][i] in slot h s + i (i.e. B^T column-encoded, as K is).  Output c holds,
 * in block h, column cols[c] of C_h = A_h B_h:  out_c = Rescale(Relin(sum_j a_j (x) b^(j, cols[c]))), where
 * b^(j, i) is slot i of every block of b_j copied into all s slots of its block: Rot(b_j; i) brings it to the block's
 * first slot (one ModUp per b_j serves all i), the block-start mask keeps it (one product, one rescale), and the
 * fill with negative steps copies it upwards through the block.  gk must hold keys for the steps cols[c] and for
 * ensi_fill_steps(1, s, -1); mask: one plaintext from ensi_block_start_mask(s, limbs = l).  A, B: d ciphertexts each at l
 * limbs; out: n_cols ciphertexts at l - 2 limbs. */
int ensi_block_start_mask(ensi_ctx *ctx, int32_t s, int32_t limbs, ensi_pt **pt);
int ensi_ccmm_blocks(ensi_ctx *ctx, const ensi_gk *rk, const ensi_gk *gk, const ensi_ct *A, const ensi_ct *B, int32_t s,
                     const int32_t *cols, int32_t n_cols, const ensi_pt *mask, ensi_ct *out, void *stream);

/* The block-wise product with the element extraction split into giant and baby steps (CCMM section: masks,
 * rotations and a shared part of the work per group of elements; the figure with the paper's own schedule is not in
 * its text), over term lists so that both attention products fit:
 *   out_o = Rescale(Relin(sum over t in [begin[o], begin[o+1]) of A[term_a[t]] (x) E(B[term_b[t]], term_slot[t]))),
 * where E(b, slot) is slot `slot` of every block of s slots of b copied into all s slots of its block.
 * Q K^T: terms of output o are (j, j, i_o) for all j; weights times V: terms of output i are (j, i, j) for all j.
 * With slot = g period + e:  giant step, once per (b, g): Rot(b; g period) brings the segment to the block's start,
 * the head mask keeps its `period` slots (one product, one rescale), the fill with steps -period, -2 period, ... repeats
 * it through the block; baby step, per element: Rot(.; e) brings the element to the start of every period, the mask of
 * the slots congruent to 0 modulo the period keeps it (one product, one rescale), the fill with steps -1, -2, ... copies it
 * through the period.  An element named by several terms of a group of outputs is formed once; the segments are formed
 * once for the whole call when it names at most 1024 of them (about 2 (l - 1) N words each), else once per group.
 * gk must hold keys for the steps g period and e in use and for ensi_fill_steps(period, s, -1) and
 * ensi_fill_steps(1, period, -1).  mask_head: ensi_block_head_mask(s, period, limbs = l); mask_start:
 * ensi_periodic_masks(period, 1, limbs = l - 1).  A, B at l limbs (l >= 4); out: n_out ciphertexts at l - 3 limbs.
 * begin: host int32[n_out + 1]; term_*: host int32[begin[n_out]].  An output's products are relinearised together,
 * so all its distinct elements are held at once (about 2 (l - 2) N words each); outputs are grouped up to 512 elements. */
int ensi_block_head_mask(ensi_ctx *ctx, int32_t s, int32_t period, int32_t limbs, ensi_pt **pt);
int ensi_ccmm_bsgs(ensi_ctx *ctx, const ensi_gk *rk, const ensi_gk *gk, const ensi_ct *A, const ensi_ct *B, int32_t s, int32_t period,
                   const int32_t *begin, const int32_t *term_a, const int32_t *term_b, const int32_t *term_slot, int32_t n_out,
                   const ensi_pt *mask_head, const ensi_pt *mask_start, ensi_ct *out, void *stream);

/* A whole segment of output columns of the block-wise product at once (the Q K^T form of ensi_ccmm_blocks: ciphertext
 * j of B holds B_h[j][i] in slot h s + i): out_c, c < period, holds in block h column g period + c of C_h = A_h B_h.
 * The replication of an element stops at the giant step of ensi_ccmm_bsgs: w_j = segment g of b_j repeated through
 * every block.  Rot(w_j; e) then holds, in slot x, element (x + e) mod period of the segment, so the diagonal
 * D_e = Rescale(Relin(sum_j a_j (x) Rot(w_j; e))) holds in slot x the entry of output column (x + e) mod period; in
 * the last e slots of a block, where that rotation reads the next block, D'_e built with Rot(w_j; e - period) holds
 * the same entries.  Baby and giant steps over the 2 period - 1 diagonals: a diagonal's rotation amount is e1 + t with
 * 0 <= e1 < baby and t a multiple of baby; w_j is rotated by e1 only, a_j by -t, and the relinearised sum of their
 * products by t, at the product's scale, before its rescale.  One plaintext product then sorts the diagonals into the
 * period columns: out_c = Rescale(sum_e R (.) D_e [+ T (.) D'_e]) with the masks of ensi_segment_masks.  Per segment and
 * ciphertext of B: one giant step of the extraction, one ModUp and baby - 1 rotations; per ciphertext of A one ModUp and
 * 2 period / baby - 1 rotations; no per-element fill.
 * gk: keys for the steps g period, ensi_fill_steps(period, s, -1), 1 .. baby - 1 and +-baby k, k = 1 .. period / baby.
 * mask_head: ensi_block_head_mask(s, period, limbs = l); masks: ensi_segment_masks(s, period, limbs = l - 2), 3 period
 * plaintexts: for r < period, index r = the slots of every block congruent to r modulo the period, index period + r
 * = those without the block's last period, index 2 period + r = those of the last period only.
 * A, B: d ciphertexts each at l limbs (l >= 4); out: period ciphertexts at l - 3 limbs.
 * The rotations of the columns of A do not depend on the segment: ensi_ccmm_left_giant_steps forms them once,
 * out[j nT + k] = Rot(a_j; -t_k) on the first l - 1 limbs for the nT = 2 period / baby giant steps t_k = -period,
 * -period + baby, ..., period - baby (baby = 1: the 2 period - 1 steps -(period - 1) .. period - 1; out allocated at exactly l - 1 limbs; prepare != 0 leaves it in the transform
 * domain, as for ensi_diagonalise_weights), and ensi_ccmm_segment takes that batch in place of A (it tells the two by
 * their level: l limbs = plain columns, l - 1 limbs = moved columns, d nT of them). */
int ensi_ccmm_left_giant_steps(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *A, int32_t period, int32_t baby, int32_t prepare, ensi_ct *out,
                               void *stream);
int ensi_segment_masks(ensi_ctx *ctx, int32_t s, int32_t period, int32_t limbs, ensi_pt **pt);
int ensi_ccmm_segment(ensi_ctx *ctx, const ensi_gk *rk, const ensi_gk *gk, const ensi_ct *A, const ensi_ct *B, int32_t s, int32_t period,
                      int32_t baby, int32_t g, const ensi_pt *mask_head, const ensi_pt *masks, ensi_ct *out, void *stream);

/* The other attention product, weights times V, without replicating single elements (CCMM section; A = the s x s
 * weights of every head column-encoded, ciphertext j = column j with head h in block h; V column-encoded alike):
 *   out_i = sum over the tokens j of the given segments of a_j (x) E(v_i, j)   (products relinearised and rescaled).
 * Per column v_i and segment g, w = that segment of v_i repeated through every block (the giant step of
 * ensi_ccmm_bsgs): slot x of Rot(w; e) holds V[g period + (x + e) mod period][i].  The weights are brought into the
 * matching arrangement once, for all columns of V: diagonal e < period of a segment holds in slot x the entry of column
 * (x + e) mod period, except in the block's last e slots, which diagonal period - 1 + e (e >= 1) holds, paired with
 * Rot(w; e - period); zero elsewhere.  Baby and giant steps over the 2 period - 1 diagonals: a diagonal's rotation
 * amount is e1 + t with 0 <= e1 < baby and t a multiple of baby; w is rotated by e1 only (one ModUp, baby - 1
 * rotations), the diagonal is rotated by -t when it is formed, the products of all diagonals and segments that share
 * t are added, relinearised and rescaled together, that sum is rotated by t, and out_i is the sum over t.
 * ensi_diagonalise_weights: A holds n_seg * period columns (whole segments, in order); out[k (2 period - 1) + q] is
 * diagonal q of segment k: plaintext products with ensi_segment_masks(s, period, limbs = l), summed and rescaled once,
 * then rotated by -t; out: n_seg (2 period - 1) ciphertexts allocated at exactly l - 1 limbs.  prepare != 0 leaves out in
 * the transform domain, where ensi_ccmm_av reads it in place for every column of V; such a batch is no ciphertext for
 * any other entry point (export and decrypt refuse it).  gk: keys for the giant steps t and -t: +-baby k, k = 1 ..
 * period / baby.
 * ensi_ccmm_av: Ad from above (same period and baby) for the segments g0 .. g0 + n_seg - 1, at l - 1 limbs; V: m
 * ciphertexts at l limbs (l >= 3); mask_head: ensi_block_head_mask(s, period, limbs = l); out: m ciphertexts at l - 2
 * limbs.  gk: keys for the steps (g0 + k) period, ensi_fill_steps(period, s, -1), 1 .. baby - 1 and the giant steps.
 * Two levels below V. */
int ensi_diagonalise_weights(ensi_ctx *ctx, const ensi_gk *gk, const ensi_ct *A, int32_t s, int32_t period, int32_t baby,
                             const ensi_pt *masks, int32_t prepare, ensi_ct *out, void *stream);
int ensi_ccmm_av(ensi_ctx *ctx, const ensi_gk *rk, const ensi_gk *gk, const ensi_ct *Ad, const ensi_ct *V, int32_t s, int32_t period,
                 int32_t baby, int32_t g0, const ensi_pt *mask_head, ensi_ct *out, void *stream);

/* ---- transform alone (parity and measurement of the NTT kernels) -------- */
/* data: device u64[n_limbs][N]; limb r uses prime index prime_idx[r] (host
 * int32[n_limbs]; 0..L-1 = q, L..L+K-1 = p).  In place.  Forward output order
 * is internal to the library; inverse(forward(x)) == x. */
int ensi_ntt(ensi_ctx *ctx, void *data, int32_t n_limbs, const int32_t *prime_idx, int32_t inverse, void *stream);

/* ---- per-kernel timers --------------------------------------------------- */
/* While enabled, every kernel launch is bracketed by HIP events on its
 * stream; ensi_profile_read synchronises and returns accumulated milliseconds
 * and launch counts per kernel class.  names_out: host buffer receiving
 * '\n'-separated class names; ms/count: host arrays of capacity cap. Returns
 * the number of classes. */
int ensi_profile_enable(ensi_ctx *ctx, int32_t on);
int ensi_profile_read(ensi_ctx *ctx, char *names_out, int32_t names_cap, double *ms, int64_t *count, int32_t cap);

#ifdef __cplusplus
}
#endif
#endif /* ENSI_H */
