"""Seeded synthetic inputs and the five workload shapes.

This module serves both the GPU library's tests/benchmark and the CPU oracle.
It holds none of the method's arithmetic: only shapes, parameter choices and
numpy random draws (weights, activations, and the small secret/error/mask
polynomials that key generation and encryption consume as inputs).

The draws stand in for BitNet b1.58 weights and transformer activations, which
the paper evaluates on but which are not available here: weights are iid
ternary with P(-1)=P(+1)=0.3, P(0)=0.4; activations are uniform [-1,1] or
N(0,1) clipped to [-4,4].
"""
from dataclasses import dataclass

import numpy as np

BASE_SEED = 250909424
ERROR_SIGMA = 3.2


@dataclass(frozen=True)
class Workload:
    name: str
    index: int
    log_n: int
    q_bits: int
    q_count: int
    p_bits: int
    p_count: int
    alpha: int
    log_scale: int
    tokens: int = 0  # s
    d_in: int = 0  # d
    d_out: int = 0  # m
    d_mid: int = 0  # FFN hidden width (two-layer workloads only)
    placement: str = "diagonal"
    act: str = "uniform"  # "uniform" [-1,1] or "normal" N(0,1) clipped to [-4,4]
    batch: int = 0  # key-switch microbench: number of ciphertexts
    kappa: float = 0.0  # scalar applied before the rescale between two layers
    op: str = "matmul"  # "matmul" (Alg. 1, the default), "rope" (Alg. 2), "merge" (block merge of placed outputs), "ccmm", "ccmm_blocks",
    #                     "ccmm_bsgs" (Q K^T form), "ccmm_bsgs_av" (weights times V form), "ccmm_segment" or "ccmm_av"
    period: int = 0  # baby-step range of the block-wise element extraction in giant and baby steps
    baby: int = 0  # segment forms: baby-step range over the diagonals of a segment

    @property
    def N(self):
        return 1 << self.log_n

    @property
    def n_slots(self):
        return self.N // 2

    @property
    def c_tot(self):
        return self.n_slots // self.tokens if self.tokens else 0

    def param_tuple(self):
        return (self.log_n, self.q_bits, self.q_count, self.p_bits, self.p_count, self.alpha, self.log_scale)


WORKLOADS = [
    Workload("tiny", 0, 12, 36, 3, 37, 1, 1, 30, tokens=32, d_in=64, d_out=64, placement="diagonal", act="uniform"),
    Workload("keyswitch", 1, 16, 50, 10, 60, 3, 3, 40, batch=64, act="uniform"),
    Workload("proj768", 2, 16, 50, 12, 60, 4, 4, 40, tokens=32, d_in=768, d_out=768, placement="diagonal", act="normal"),
    Workload("attn2560", 3, 16, 50, 16, 60, 4, 4, 40, tokens=128, d_in=2560, d_out=2560, placement="diagonal", act="normal"),
    Workload("ffn2560", 4, 16, 50, 16, 60, 4, 4, 40, tokens=128, d_in=2560, d_out=2560, d_mid=6912, placement="zero",
             act="normal", kappa=2.0 ** -5),
]
# One of the paper's own PCMM shapes (Table III, QKV projection): 2048 tokens, 1536 x 1536 -- 16 columns per
# ciphertext, 96 packed inputs, 15 rotation amounts.  Not one of the five benchmark configurations: a bench/test extra.
WORKLOADS.append(Workload("paper1536", 5, 16, 50, 16, 60, 4, 4, 40, tokens=2048, d_in=1536, d_out=1536, placement="diagonal", act="normal"))
# The paper's RoPE shape (Table III: 2048 x 96 per head, 16 heads): the 1536 query columns of 2048 tokens, 16 per
# ciphertext, i.e. 96 ciphertexts; and the merge of that projection's 1536 block-placed outputs into 96 packed
# ciphertexts.  Bench/test extras like paper1536.
WORKLOADS.append(Workload("rope1536", 6, 16, 50, 16, 60, 4, 4, 40, tokens=2048, d_in=1536, act="uniform", op="rope"))
WORKLOADS.append(Workload("merge1536", 7, 16, 50, 16, 60, 4, 4, 40, tokens=2048, d_in=1536, act="uniform", op="merge"))
# A slice of the paper's attention-score product (Table III: Q K^T per head, head width 96): A = d_in = 96 column
# ciphertexts, B = d_out = 8 columns of K^T, one head per ciphertext, tokens filling the slot axis.  The full
# product has 2048 such columns per head; a step of 8 keeps the benchmark to about a second.
WORKLOADS.append(Workload("ccmm96", 8, 16, 50, 16, 60, 4, 4, 40, tokens=32768, d_in=96, d_out=8, act="uniform", op="ccmm"))
# The paper's feed-forward shape (Table III: 2048 x 1536 -> 4096 -> 1536), run like ffn2560: 16 columns per input
# ciphertext, first layer placed in block 0, scalar-multiply + rescale, rotation-free second layer.
WORKLOADS.append(Workload("paperffn", 9, 16, 50, 16, 60, 4, 4, 40, tokens=2048, d_in=1536, d_out=1536, d_mid=4096, placement="zero",
                          act="normal", kappa=2.0 ** -5))
# The paper's attention-score product at its own packing (Table III: (2048 x 96) by (2048 x 96)^T, 16 heads): Q and K
# column-encoded with the 16 heads of a column in the 16 blocks of one ciphertext (96 ciphertexts each); a step
# computes d_out = 8 of the 2048 output columns for all heads at once.
WORKLOADS.append(Workload("ccmmqk", 10, 16, 50, 16, 60, 4, 4, 40, tokens=2048, d_in=96, d_out=8, act="uniform", op="ccmm_blocks"))
# The same product with the element extraction in giant and baby steps (period 16): a step computes the d_out = 16
# output columns of one segment (columns 16..31), whose giant steps are shared.  Three levels instead of two.
WORKLOADS.append(Workload("ccmmqkbsgs", 11, 16, 50, 16, 60, 4, 4, 40, tokens=2048, d_in=96, d_out=16, act="uniform", op="ccmm_bsgs", period=16))
# A whole segment of 64 output columns (64 .. 127) from its diagonals, in baby steps of 4 (no per-element fills).
WORKLOADS.append(Workload("ccmmqkseg", 14, 16, 50, 16, 60, 4, 4, 40, tokens=2048, d_in=96, d_out=64, act="uniform", op="ccmm_segment", period=64,
                          baby=4))
# A slice of the paper's other attention product (Table III: (2048 x 2048) by (2048 x 96), 16 heads): the attention
# weights column-encoded (column j = one ciphertext, 16 heads in its blocks), V column-encoded.  Output column i is
# sum_j a_j (x) E(v_i, j) over the 2048 tokens j; a step forms d_out = 1 output over the first d_in = 512 of them.
WORKLOADS.append(Workload("ccmmav", 12, 16, 50, 16, 60, 4, 4, 40, tokens=2048, d_in=512, d_out=1, act="uniform", op="ccmm_bsgs_av", period=16))
# The paper's QKV projection shape at its default ring (N' = 2^14: 8192 slots, 4 columns of 2048 tokens per
# ciphertext, 384 packed inputs, 3 rotation amounts) on a chain that fits that ring (6 x 50-bit + 2 x 60-bit primes).
# The fused N = 2^16 kernels do not apply: transforms, ModUp, inner product and ModDown run as separate kernels.
WORKLOADS.append(Workload("paper1536n14", 13, 14, 50, 6, 60, 2, 2, 40, tokens=2048, d_in=1536, d_out=1536, placement="diagonal", act="normal"))
# The same slice of weights times V from diagonalised weights (prepared once for all 96 columns of V, outside the step).
WORKLOADS.append(Workload("ccmmavseg", 15, 16, 50, 16, 60, 4, 4, 40, tokens=2048, d_in=512, d_out=1, act="uniform", op="ccmm_av", period=64,
                          baby=8))
# The ccmm96 shape (one head of 32768 tokens per ciphertext, inner width 96) through the weights-times-V entry point: the
# inner index is the slot index of B's columns, so A's 96 columns (padded to one segment of 128) are diagonalised once
# and every column of B costs one giant step of the extraction, 31 baby-step rotations and 255 products.
WORKLOADS.append(Workload("ccmm96av", 16, 16, 50, 16, 60, 4, 4, 40, tokens=32768, d_in=96, d_out=8, act="uniform", op="ccmm_av", period=128,
                          baby=32))
BY_NAME = {w.name: w for w in WORKLOADS}

# key-switch microbench: steps 2^0..2^14 plus the inverse rotation -1
KEYSWITCH_STEPS = [1 << i for i in range(15)] + [-1]


def rng_for(index, salt=0):
    return np.random.default_rng(BASE_SEED + index + 1000 * salt)


def ternary_weights(rng, d, m):
    """Row-major d x m int8 in {-1,0,+1}, P(-1)=P(+1)=0.3, P(0)=0.4."""
    u = rng.random((d, m))
    return (np.where(u < 0.3, -1, 0) + np.where(u >= 0.7, 1, 0)).astype(np.int8)


def activations(rng, tokens, d, kind):
    if kind == "uniform":
        return rng.uniform(-1.0, 1.0, size=(tokens, d))
    return np.clip(rng.standard_normal((tokens, d)), -4.0, 4.0)


def pack_columns(X, n_slots):
    """Column-wise SIMD packing with several columns per ciphertext: packed vector
    G holds column G*c_tot+b in slots [b*s,(b+1)*s).  Returns [n_ct][n_slots]."""
    s, d = X.shape
    c_tot = n_slots // s
    n_ct = -(-d // c_tot)
    out = np.zeros((n_ct, n_slots), dtype=np.float64)
    for j in range(d):
        G, b = divmod(j, c_tot)
        out[G, b * s:(b + 1) * s] = X[:, j]
    return out


def ternary_poly(rng, n):
    """Uniform ternary polynomial (secret key, encryption mask), int8[n]."""
    return rng.integers(-1, 2, size=n, dtype=np.int8)


def error_poly(rng, shape):
    """Rounded Gaussian, sigma 3.2, clipped at +-19 (about 6 sigma), int8."""
    e = np.rint(rng.normal(0.0, ERROR_SIGMA, size=shape))
    return np.clip(e, -19, 19).astype(np.int8)


# Synthetic residue words for tests that need far more ciphertext data than anything could
# encrypt: word w of operand v, a fixed 64-bit mix cut to `bits` bits (always a valid residue of a
# prime of more than `bits` bits).  Only +, *, ^, >>, & on 64-bit integers with wrap-around, written
# so that numpy uint64 arrays and torch int64 tensors give the same low bits (shifts are masked,
# so logical and arithmetic shifts agree).
_MIX1, _MIX2, _MIX3 = 0x1E3779B97F4A7C15, 0x3F58476D1CE4E5B9, 0x14D049BB133111EB


def synthetic_words(v, w, bits):
    """v, w: integer arrays/tensors (broadcast against each other) of one 64-bit integer type."""
    h = (v + 1) * _MIX1 + (w + 1) * _MIX2
    h = h ^ ((h >> 29) & ((1 << 35) - 1))
    h = h * _MIX3
    h = h ^ ((h >> 32) & ((1 << 32) - 1))
    return (h >> 11) & ((1 << bits) - 1)
