"""ctypes binding of libensi_hip.so: argument marshalling only.

Every function mirrors one entry point of include/ensi.h; all arithmetic runs
inside the library's HIP kernels.  There is no fallback: if the shared library
is missing or a call fails, an exception is raised.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libensi_hip.so")
_lib = None

PLACE_ZERO, PLACE_DIAGONAL = 0, 1
_PLACEMENTS = {"zero": PLACE_ZERO, "diagonal": PLACE_DIAGONAL}

EXPORTED = [
    "ensi_ctx_create", "ensi_ctx_free", "ensi_last_error", "ensi_get_primes", "ensi_keygen", "ensi_sk_free",
    "ensi_pk_free", "ensi_galois_keygen", "ensi_gk_free", "ensi_encode", "ensi_pt_import", "ensi_pt_export",
    "ensi_pt_free", "ensi_ct_alloc", "ensi_ct_wrap", "ensi_ct_free", "ensi_ct_info", "ensi_ct_export",
    "ensi_ct_import", "ensi_encrypt", "ensi_decrypt", "ensi_rotate", "ensi_ternary_matmul",
    "ensi_set_accumulate_mode", "ensi_mul_scalar_rescale", "ensi_rescale_ternary_matmul", "ensi_encode_at", "ensi_pt_set_scale",
    "ensi_pmult_sum_rescale", "ensi_set_pmult_mode", "ensi_block_masks", "ensi_merge", "ensi_rope_plaintexts", "ensi_rope", "ensi_relin_keygen",
    "ensi_ct_drop_limbs", "ensi_mult_sum_relin_rescale", "ensi_fill_steps", "ensi_one_hot_masks", "ensi_replicate", "ensi_periodic_masks", "ensi_ccmm", "ensi_block_start_mask", "ensi_ccmm_blocks", "ensi_block_head_mask", "ensi_ccmm_bsgs", "ensi_segment_masks", "ensi_ccmm_segment", "ensi_ccmm_left_giant_steps", "ensi_diagonalise_weights", "ensi_ccmm_av", "ensi_ntt", "ensi_profile_enable", "ensi_profile_read",
    "ensi_sk_import", "ensi_sk_export", "ensi_pk_import", "ensi_pk_export", "ensi_gk_import", "ensi_gk_export", "ensi_gk_elements",
    "ensi_ct_checksum", "ensi_weights_prepare", "ensi_weights_free", "ensi_ternary_matmul_prepared", "ensi_rescale_ternary_matmul_prepared",
    "ensi_rotate_static", "ensi_matrix_rate_probe",
]


class EnsiError(RuntimeError):
    pass


class _Params(ctypes.Structure):
    _fields_ = [("log_n", ctypes.c_int32), ("q_bits", ctypes.c_int32), ("q_count", ctypes.c_int32),
                ("p_bits", ctypes.c_int32), ("p_count", ctypes.c_int32), ("alpha", ctypes.c_int32),
                ("log_scale", ctypes.c_int32), ("seed", ctypes.c_uint64)]


def load():
    """Loads the built library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise EnsiError("libensi_hip.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        lib = ctypes.CDLL(LIB_PATH)
        lib.ensi_last_error.restype = ctypes.c_char_p
        for name in EXPORTED:
            getattr(lib, name)  # raises AttributeError on a missing symbol
        for name in EXPORTED:
            if name.endswith("_free") or name == "ensi_last_error":
                continue
            getattr(lib, name).restype = ctypes.c_int
        for name in ("ensi_ctx_free", "ensi_sk_free", "ensi_pk_free", "ensi_gk_free", "ensi_pt_free", "ensi_ct_free", "ensi_weights_free"):
            getattr(lib, name).restype = None
            getattr(lib, name).argtypes = [ctypes.c_void_p]
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i8(a, shape=None):
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.int8)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise EnsiError("expected int8 array of shape %s, got %s" % (shape, a.shape))
    return a


class Context:
    def __init__(self, log_n, q_bits, q_count, p_bits, p_count, alpha, log_scale, seed=1):
        self.lib = load()
        self.params = _Params(log_n, q_bits, q_count, p_bits, p_count, alpha, log_scale, seed)
        self.h = ctypes.c_void_p()
        rc = self.lib.ensi_ctx_create(ctypes.byref(self.params), ctypes.byref(self.h))
        if rc:
            raise EnsiError("ensi_ctx_create failed with code %d" % rc)
        self.N = 1 << log_n
        self.n_slots = self.N // 2
        self.L, self.K, self.alpha = q_count, p_count, alpha
        self.beta = -(-q_count // alpha)

    def _check(self, rc):
        if rc:
            raise EnsiError("code %d: %s" % (rc, self.lib.ensi_last_error(self.h).decode()))

    def close(self):
        if self.h:
            self.lib.ensi_ctx_free(self.h)
            self.h = ctypes.c_void_p()

    def primes(self):
        q = np.zeros(self.L, dtype=np.uint64)
        p = np.zeros(self.K, dtype=np.uint64)
        self._check(self.lib.ensi_get_primes(self.h, _ptr(q), _ptr(p)))
        return [int(x) for x in q], [int(x) for x in p]

    # ---- keys
    def keygen(self, s=None, e=None, seed_a=0):
        s, e = _i8(s, (self.N,)), _i8(e, (self.N,))
        sk, pk = ctypes.c_void_p(), ctypes.c_void_p()
        self._check(self.lib.ensi_keygen(self.h, _ptr(s), _ptr(e), ctypes.c_uint64(seed_a), ctypes.byref(sk), ctypes.byref(pk)))
        return _Handle(self, sk, "ensi_sk_free"), _Handle(self, pk, "ensi_pk_free")

    def galois_keygen(self, sk, steps, e=None, seed_a=0):
        steps = np.ascontiguousarray(steps, dtype=np.int32)
        e = _i8(e, (len(steps), self.beta, self.N))
        gk = ctypes.c_void_p()
        self._check(self.lib.ensi_galois_keygen(self.h, sk.h, _ptr(steps), len(steps), _ptr(e), ctypes.c_uint64(seed_a), ctypes.byref(gk)))
        return _Handle(self, gk, "ensi_gk_free")

    def relin_keygen(self, sk, e=None, seed_a=0):
        e = _i8(e, (self.beta, self.N))
        rk = ctypes.c_void_p()
        self._check(self.lib.ensi_relin_keygen(self.h, sk.h, _ptr(e), ctypes.c_uint64(seed_a), ctypes.byref(rk)))
        return _Handle(self, rk, "ensi_gk_free")

    def sk_import(self, s):
        s = _i8(s, (self.N,))
        sk = ctypes.c_void_p()
        self._check(self.lib.ensi_sk_import(self.h, _ptr(s), ctypes.byref(sk)))
        return _Handle(self, sk, "ensi_sk_free")

    def sk_export(self, sk):
        out = np.empty(self.N, dtype=np.int8)
        self._check(self.lib.ensi_sk_export(self.h, sk.h, _ptr(out)))
        return out

    def pk_import(self, words):
        a = np.ascontiguousarray(words, dtype=np.uint64)
        if a.shape != (2, self.L, self.N):
            raise EnsiError("expected uint64 [2][L][N]")
        pk = ctypes.c_void_p()
        self._check(self.lib.ensi_pk_import(self.h, _ptr(a), ctypes.byref(pk)))
        return _Handle(self, pk, "ensi_pk_free")

    def pk_export(self, pk):
        out = np.empty((2, self.L, self.N), dtype=np.uint64)
        self._check(self.lib.ensi_pk_export(self.h, pk.h, _ptr(out)))
        return out

    def gk_import(self, step, words, gk=None):
        """Adds the switching key of `step` (uint64 [beta][2][L+K][N]) to the key set gk (a new set if None)."""
        a = np.ascontiguousarray(words, dtype=np.uint64)
        if a.shape != (self.beta, 2, self.L + self.K, self.N):
            raise EnsiError("expected uint64 [beta][2][L+K][N]")
        h = ctypes.c_void_p(gk.h.value if gk is not None else None)
        self._check(self.lib.ensi_gk_import(self.h, ctypes.byref(h), int(step), _ptr(a)))
        if gk is None:
            gk = _Handle(self, h, "ensi_gk_free")
        return gk

    def gk_export(self, gk, step):
        out = np.empty((self.beta, 2, self.L + self.K, self.N), dtype=np.uint64)
        self._check(self.lib.ensi_gk_export(self.h, gk.h, int(step), _ptr(out)))
        return out

    def gk_elements(self, gk):
        n = self.lib.ensi_gk_elements(gk.h, None, 0)
        if n < 0:
            raise EnsiError("ensi_gk_elements failed with code %d" % n)
        out = np.zeros(max(n, 1), dtype=np.int32)
        self.lib.ensi_gk_elements(gk.h, _ptr(out), n)
        return [int(x) for x in out[:n]]

    # ---- plaintexts
    def encode(self, slots, limbs):
        slots = np.ascontiguousarray(np.atleast_2d(slots), dtype=np.float64)
        pt = ctypes.c_void_p()
        self._check(self.lib.ensi_encode(self.h, _ptr(slots), slots.shape[0], slots.shape[1], limbs, ctypes.byref(pt)))
        return _Handle(self, pt, "ensi_pt_free", n=slots.shape[0])

    def pt_import(self, coeffs, limbs):
        coeffs = np.ascontiguousarray(np.atleast_2d(coeffs), dtype=np.int64)
        if coeffs.shape[1] != self.N:
            raise EnsiError("coefficient arrays must have N entries")
        pt = ctypes.c_void_p()
        self._check(self.lib.ensi_pt_import(self.h, _ptr(coeffs), coeffs.shape[0], limbs, ctypes.byref(pt)))
        return _Handle(self, pt, "ensi_pt_free", n=coeffs.shape[0])

    def encode_at(self, slots, limbs, scale):
        slots = np.ascontiguousarray(np.atleast_2d(slots), dtype=np.float64)
        pt = ctypes.c_void_p()
        self._check(self.lib.ensi_encode_at(self.h, _ptr(slots), slots.shape[0], slots.shape[1], limbs, ctypes.c_double(scale), ctypes.byref(pt)))
        return _Handle(self, pt, "ensi_pt_free", n=slots.shape[0])

    def pt_set_scale(self, pt, scale):
        self._check(self.lib.ensi_pt_set_scale(pt.h, ctypes.c_double(scale)))
        return pt

    def pt_export(self, pt):
        out = np.empty((pt.n, self.N), dtype=np.int64)
        self._check(self.lib.ensi_pt_export(self.h, pt.h, _ptr(out)))
        return out

    # ---- ciphertexts
    def ct_alloc(self, n, limbs):
        ct = ctypes.c_void_p()
        self._check(self.lib.ensi_ct_alloc(self.h, n, limbs, ctypes.byref(ct)))
        return Ciphertexts(self, ct)

    def ct_wrap(self, device_ptr, n, limbs, scale):
        ct = ctypes.c_void_p()
        self._check(self.lib.ensi_ct_wrap(self.h, ctypes.c_void_p(int(device_ptr)), n, limbs, ctypes.c_double(scale), ctypes.byref(ct)))
        return Ciphertexts(self, ct)

    def ct_import(self, limbs_array, scale):
        a = np.ascontiguousarray(limbs_array, dtype=np.uint64)
        if a.ndim != 4 or a.shape[1] != 2 or a.shape[3] != self.N:
            raise EnsiError("expected uint64 [n][2][limbs][N]")
        ct = ctypes.c_void_p()
        self._check(self.lib.ensi_ct_import(self.h, _ptr(a), a.shape[0], a.shape[2], ctypes.c_double(scale), ctypes.byref(ct)))
        return Ciphertexts(self, ct)

    def encrypt(self, pk, pt, v=None, e0=None, e1=None):
        shape = (pt.n, self.N)
        v, e0, e1 = _i8(v, shape), _i8(e0, shape), _i8(e1, shape)
        ct = ctypes.c_void_p()
        self._check(self.lib.ensi_encrypt(self.h, pk.h, pt.h, _ptr(v), _ptr(e0), _ptr(e1), ctypes.byref(ct)))
        return Ciphertexts(self, ct)

    def decrypt(self, sk, ct, slot_begin=0, n_slots=None):
        slot_begin = int(slot_begin)
        n_slots = self.n_slots - slot_begin if n_slots is None else int(n_slots)
        out = np.empty((ct.n, n_slots), dtype=np.float64)
        self._check(self.lib.ensi_decrypt(self.h, sk.h, ct.h, slot_begin, n_slots, _ptr(out)))
        return out

    # ---- hot path
    def rotate(self, gk, ct_in, steps, ct_out=None, stream=0):
        steps = np.ascontiguousarray(steps, dtype=np.int32)
        if len(steps) != ct_in.n:
            raise EnsiError("one step per ciphertext")
        if ct_out is None:
            ct_out = self.ct_alloc(ct_in.n, ct_in.limbs)
        self._check(self.lib.ensi_rotate(self.h, gk.h, ct_in.h, _ptr(steps), ct_out.h, ctypes.c_void_p(stream)))
        return ct_out

    def rotate_static(self, gk, ct_in, steps, ct_out, stream=0):
        """ensi_rotate on the statically linked workspace: allocates nothing (the caller provides ct_out)."""
        steps = np.ascontiguousarray(steps, dtype=np.int32)
        if len(steps) != ct_in.n:
            raise EnsiError("one step per ciphertext")
        self._check(self.lib.ensi_rotate_static(self.h, gk.h, ct_in.h, _ptr(steps), ct_out.h, ctypes.c_void_p(stream)))
        return ct_out

    def ternary_matmul(self, gk, ct_in, s, d, W, placement="diagonal", ct_out=None, stream=0):
        W = np.ascontiguousarray(W, dtype=np.int8)
        if W.ndim != 2 or W.shape[0] != d:
            raise EnsiError("W must be int8 [d][m]")
        m = W.shape[1]
        if ct_out is None:
            ct_out = self.ct_alloc(m, ct_in.limbs)
        self._check(self.lib.ensi_ternary_matmul(self.h, gk.h if gk is not None else None, ct_in.h, s, d, _ptr(W), m,
                                                 _PLACEMENTS[placement], ct_out.h, ctypes.c_void_p(stream)))
        return ct_out

    def weights_prepare(self, W, s, d, placement, limbs):
        """Everything Alg. 1 derives from the weights alone, built once; `limbs`: the level of the inputs."""
        W = np.ascontiguousarray(W, dtype=np.int8)
        if W.ndim != 2 or W.shape[0] != d:
            raise EnsiError("W must be int8 [d][m]")
        wt = ctypes.c_void_p()
        self._check(self.lib.ensi_weights_prepare(self.h, _ptr(W), int(s), int(d), W.shape[1], _PLACEMENTS[placement], int(limbs), ctypes.byref(wt)))
        return _Handle(self, wt, "ensi_weights_free", n=W.shape[1])

    def ternary_matmul_prepared(self, gk, ct_in, wt, ct_out=None, stream=0):
        if ct_out is None:
            ct_out = self.ct_alloc(wt.n, ct_in.limbs)
        self._check(self.lib.ensi_ternary_matmul_prepared(self.h, gk.h if gk is not None else None, ct_in.h, wt.h, ct_out.h, ctypes.c_void_p(stream)))
        return ct_out

    def rescale_ternary_matmul_prepared(self, ct_in, kappa, wt, ct_out=None, stream=0):
        if ct_out is None:
            ct_out = self.ct_alloc(wt.n, ct_in.limbs - 1)
        self._check(self.lib.ensi_rescale_ternary_matmul_prepared(self.h, ct_in.h, ctypes.c_double(kappa), wt.h, ct_out.h, ctypes.c_void_p(stream)))
        return ct_out

    def set_accumulate_mode(self, mode):
        self._check(self.lib.ensi_set_accumulate_mode(self.h, int(mode)))

    def matrix_rate_probe(self, seconds=0.3, stream=0):
        """Sustained int8 matrix-instruction rate of the chip (operations per second), measured for about `seconds`."""
        rate = ctypes.c_double()
        self._check(self.lib.ensi_matrix_rate_probe(self.h, ctypes.c_double(seconds), ctypes.byref(rate), ctypes.c_void_p(stream)))
        return rate.value

    def mul_scalar_rescale(self, ct, kappa, stream=0):
        self._check(self.lib.ensi_mul_scalar_rescale(self.h, ct.h, ctypes.c_double(kappa), ctypes.c_void_p(stream)))
        return ct

    def rescale_ternary_matmul(self, ct_in, kappa, W, ct_out=None, stream=0):
        W = np.ascontiguousarray(W, dtype=np.int8)
        if W.ndim != 2 or W.shape[0] != ct_in.n:
            raise EnsiError("W must be int8 [n_in][m]")
        m = W.shape[1]
        if ct_out is None:
            ct_out = self.ct_alloc(m, ct_in.limbs - 1)
        self._check(self.lib.ensi_rescale_ternary_matmul(self.h, ct_in.h, ctypes.c_double(kappa), _ptr(W), m, ct_out.h, ctypes.c_void_p(stream)))
        return ct_out

    def pmult_sum_rescale(self, ct_in, pt, begin, term_ct, term_pt, ct_out=None, stream=0):
        begin = np.ascontiguousarray(begin, dtype=np.int32)
        term_ct = np.ascontiguousarray(term_ct, dtype=np.int32)
        term_pt = np.ascontiguousarray(term_pt, dtype=np.int32)
        n_out = len(begin) - 1
        if n_out < 1 or len(term_ct) != begin[-1] or len(term_pt) != begin[-1]:
            raise EnsiError("begin must hold n_out + 1 offsets and end at the number of terms")
        if ct_out is None:
            ct_out = self.ct_alloc(n_out, ct_in.limbs - 1)
        self._check(self.lib.ensi_pmult_sum_rescale(self.h, ct_in.h, pt.h, _ptr(begin), _ptr(term_ct), _ptr(term_pt), n_out, ct_out.h,
                                                    ctypes.c_void_p(stream)))
        return ct_out

    def set_pmult_mode(self, mode):
        self._check(self.lib.ensi_set_pmult_mode(self.h, int(mode)))

    def block_masks(self, s, c_tot, limbs):
        pt = ctypes.c_void_p()
        self._check(self.lib.ensi_block_masks(self.h, int(s), int(c_tot), int(limbs), ctypes.byref(pt)))
        return _Handle(self, pt, "ensi_pt_free", n=c_tot)

    def merge(self, ct_in, masks, c_tot, ct_out=None, stream=0):
        if ct_out is None:
            ct_out = self.ct_alloc(-(-ct_in.n // c_tot), ct_in.limbs - 1)
        self._check(self.lib.ensi_merge(self.h, ct_in.h, masks.h, int(c_tot), ct_out.h, ctypes.c_void_p(stream)))
        return ct_out

    def rope_plaintexts(self, cos, sin, limbs):
        cos = np.ascontiguousarray(cos, dtype=np.float64)
        sin = np.ascontiguousarray(sin, dtype=np.float64)
        if cos.ndim != 1 or cos.shape != sin.shape:
            raise EnsiError("cos and sin must be vectors of equal length")
        pt = ctypes.c_void_p()
        self._check(self.lib.ensi_rope_plaintexts(self.h, _ptr(cos), _ptr(sin), len(cos), int(limbs), ctypes.byref(pt)))
        return _Handle(self, pt, "ensi_pt_free", n=3)

    def rope(self, gk, ct_in, pt, ct_out=None, stream=0):
        if ct_out is None:
            ct_out = self.ct_alloc(ct_in.n, ct_in.limbs - 1)
        self._check(self.lib.ensi_rope(self.h, gk.h, ct_in.h, pt.h, ct_out.h, ctypes.c_void_p(stream)))
        return ct_out

    def ct_drop_limbs(self, ct, limbs):
        self._check(self.lib.ensi_ct_drop_limbs(ct.h, int(limbs)))
        return ct

    def mult_sum_relin_rescale(self, rk, ct_a, ct_b, begin, term_a, term_b, ct_out=None, stream=0):
        begin = np.ascontiguousarray(begin, dtype=np.int32)
        term_a = np.ascontiguousarray(term_a, dtype=np.int32)
        term_b = np.ascontiguousarray(term_b, dtype=np.int32)
        n_out = len(begin) - 1
        if n_out < 1 or len(term_a) != begin[-1] or len(term_b) != begin[-1]:
            raise EnsiError("begin must hold n_out + 1 offsets and end at the number of terms")
        if ct_out is None:
            ct_out = self.ct_alloc(n_out, ct_a.limbs - 1)
        self._check(self.lib.ensi_mult_sum_relin_rescale(self.h, rk.h, ct_a.h, ct_b.h, _ptr(begin), _ptr(term_a), _ptr(term_b), n_out,
                                                         ct_out.h, ctypes.c_void_p(stream)))
        return ct_out

    def fill_steps(self, r_begin, r_end, sign=1):
        out = np.zeros(128, dtype=np.int32)
        n = self.lib.ensi_fill_steps(int(r_begin), int(r_end), int(sign), _ptr(out), len(out))
        if n < 0 or n > len(out):
            raise EnsiError("ensi_fill_steps failed with code %d" % n)
        return [int(x) for x in out[:n]]

    def one_hot_masks(self, count, limbs):
        pt = ctypes.c_void_p()
        self._check(self.lib.ensi_one_hot_masks(self.h, int(count), int(limbs), ctypes.byref(pt)))
        return _Handle(self, pt, "ensi_pt_free", n=count)

    def replicate(self, gk, ct_in, src, masks, mask_idx, ct_out=None, stream=0):
        src = np.ascontiguousarray(src, dtype=np.int32)
        mask_idx = np.ascontiguousarray(mask_idx, dtype=np.int32)
        if len(src) != len(mask_idx) or len(src) < 1:
            raise EnsiError("one source and one mask index per output")
        if ct_out is None:
            ct_out = self.ct_alloc(len(src), ct_in.limbs - 1)
        self._check(self.lib.ensi_replicate(self.h, gk.h, ct_in.h, _ptr(src), masks.h, _ptr(mask_idx), len(src), ct_out.h,
                                            ctypes.c_void_p(stream)))
        return ct_out

    def periodic_masks(self, period, count, limbs):
        pt = ctypes.c_void_p()
        self._check(self.lib.ensi_periodic_masks(self.h, int(period), int(count), int(limbs), ctypes.byref(pt)))
        return _Handle(self, pt, "ensi_pt_free", n=count)

    def ccmm(self, rk, gk, ct_a, ct_b, masks, period, ct_out=None, stream=0):
        if ct_out is None:
            ct_out = self.ct_alloc(ct_b.n, ct_b.limbs - 2)
        self._check(self.lib.ensi_ccmm(self.h, rk.h, gk.h, ct_a.h, ct_b.h, masks.h, int(period), ct_out.h, ctypes.c_void_p(stream)))
        return ct_out

    def block_start_mask(self, s, limbs):
        pt = ctypes.c_void_p()
        self._check(self.lib.ensi_block_start_mask(self.h, int(s), int(limbs), ctypes.byref(pt)))
        return _Handle(self, pt, "ensi_pt_free", n=1)

    def ccmm_blocks(self, rk, gk, ct_a, ct_b, s, cols, mask, ct_out=None, stream=0):
        cols = np.ascontiguousarray(cols, dtype=np.int32)
        if ct_out is None:
            ct_out = self.ct_alloc(len(cols), ct_b.limbs - 2)
        self._check(self.lib.ensi_ccmm_blocks(self.h, rk.h, gk.h, ct_a.h, ct_b.h, int(s), _ptr(cols), len(cols), mask.h, ct_out.h,
                                              ctypes.c_void_p(stream)))
        return ct_out

    def block_head_mask(self, s, period, limbs):
        pt = ctypes.c_void_p()
        self._check(self.lib.ensi_block_head_mask(self.h, int(s), int(period), int(limbs), ctypes.byref(pt)))
        return _Handle(self, pt, "ensi_pt_free", n=1)

    def ccmm_bsgs(self, rk, gk, ct_a, ct_b, s, period, terms, mask_head, mask_start, ct_out=None, stream=0):
        """terms: per output a list of (index into ct_a, index into ct_b, slot)."""
        begin = np.zeros(len(terms) + 1, dtype=np.int32)
        begin[1:] = np.cumsum([len(t) for t in terms])
        flat = np.array([x for t in terms for x in t], dtype=np.int32).reshape(-1, 3)
        ta, tb, ts = (np.ascontiguousarray(flat[:, k]) for k in range(3))
        if ct_out is None:
            ct_out = self.ct_alloc(len(terms), ct_b.limbs - 3)
        self._check(self.lib.ensi_ccmm_bsgs(self.h, rk.h, gk.h, ct_a.h, ct_b.h, int(s), int(period), _ptr(begin), _ptr(ta), _ptr(tb),
                                            _ptr(ts), len(terms), mask_head.h, mask_start.h, ct_out.h, ctypes.c_void_p(stream)))
        return ct_out

    def segment_masks(self, s, period, limbs):
        pt = ctypes.c_void_p()
        self._check(self.lib.ensi_segment_masks(self.h, int(s), int(period), int(limbs), ctypes.byref(pt)))
        return _Handle(self, pt, "ensi_pt_free", n=3 * period)

    def ccmm_left_giant_steps(self, gk, ct_a, period, baby, ct_out=None, prepare=False, stream=0):
        if ct_out is None:
            n_giant = 2 * int(period) - 1 if int(baby) == 1 else 2 * int(period) // int(baby)
            ct_out = self.ct_alloc(ct_a.n * n_giant, ct_a.limbs - 1)
        self._check(self.lib.ensi_ccmm_left_giant_steps(self.h, gk.h, ct_a.h, int(period), int(baby), int(bool(prepare)), ct_out.h,
                                                        ctypes.c_void_p(stream)))
        return ct_out

    def ccmm_segment(self, rk, gk, ct_a, ct_b, s, period, baby, g, mask_head, masks, ct_out=None, stream=0):
        if ct_out is None:
            ct_out = self.ct_alloc(int(period), ct_b.limbs - 3)
        self._check(self.lib.ensi_ccmm_segment(self.h, rk.h, gk.h, ct_a.h, ct_b.h, int(s), int(period), int(baby), int(g), mask_head.h,
                                               masks.h, ct_out.h, ctypes.c_void_p(stream)))
        return ct_out

    def diagonalise_weights(self, gk, ct_a, s, period, baby, masks, ct_out=None, prepare=False, stream=0):
        if ct_out is None:
            ct_out = self.ct_alloc(ct_a.n // int(period) * (2 * int(period) - 1), ct_a.limbs - 1)
        self._check(self.lib.ensi_diagonalise_weights(self.h, gk.h, ct_a.h, int(s), int(period), int(baby), masks.h, int(bool(prepare)),
                                                      ct_out.h, ctypes.c_void_p(stream)))
        return ct_out

    def ccmm_av(self, rk, gk, ct_ad, ct_v, s, period, baby, g0, mask_head, ct_out=None, stream=0):
        if ct_out is None:
            ct_out = self.ct_alloc(ct_v.n, ct_v.limbs - 2)
        self._check(self.lib.ensi_ccmm_av(self.h, rk.h, gk.h, ct_ad.h, ct_v.h, int(s), int(period), int(baby), int(g0), mask_head.h,
                                          ct_out.h, ctypes.c_void_p(stream)))
        return ct_out

    def ntt(self, device_ptr, prime_idx, inverse=False, stream=0):
        prime_idx = np.ascontiguousarray(prime_idx, dtype=np.int32)
        self._check(self.lib.ensi_ntt(self.h, ctypes.c_void_p(int(device_ptr)), len(prime_idx), _ptr(prime_idx), int(inverse),
                                      ctypes.c_void_p(stream)))

    # ---- timers
    def profile_enable(self, on=True):
        self._check(self.lib.ensi_profile_enable(self.h, int(on)))

    def profile_read(self):
        cap = 64
        names = ctypes.create_string_buffer(4096)
        ms = np.zeros(cap, dtype=np.float64)
        cnt = np.zeros(cap, dtype=np.int64)
        n = self.lib.ensi_profile_read(self.h, names, 4096, _ptr(ms), _ptr(cnt), cap)
        if n < 0:
            self._check(n)
        nm = names.value.decode().split("\n")[:n]
        return {nm[i]: (float(ms[i]), int(cnt[i])) for i in range(n)}


class _Handle:
    def __init__(self, ctx, h, free_name, n=0):
        self.ctx, self.h, self._free, self.n = ctx, h, free_name, n

    def free(self):
        if self.h:
            getattr(self.ctx.lib, self._free)(self.h)
            self.h = ctypes.c_void_p()


class Ciphertexts(_Handle):
    """A batch of ciphertexts resident on the device."""

    def __init__(self, ctx, h):
        super().__init__(ctx, h, "ensi_ct_free")

    def _info(self):
        n, limbs, scale, ptr = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_double(), ctypes.c_void_p()
        self.ctx._check(self.ctx.lib.ensi_ct_info(self.h, ctypes.byref(n), ctypes.byref(limbs), ctypes.byref(scale), ctypes.byref(ptr)))
        return n.value, limbs.value, scale.value, ptr.value

    @property
    def n(self):
        return self._info()[0]

    @n.setter
    def n(self, _):
        pass

    @property
    def limbs(self):
        return self._info()[1]

    @property
    def scale(self):
        return self._info()[2]

    @property
    def device_ptr(self):
        return self._info()[3]

    def checksum(self, stream=0):
        """Wrap-around 64-bit sum of the active limb words of every ciphertext of the batch."""
        out = np.zeros(self._info()[0], dtype=np.uint64)
        self.ctx._check(self.ctx.lib.ensi_ct_checksum(self.ctx.h, self.h, _ptr(out), ctypes.c_void_p(stream)))
        return out

    def export(self):
        n, limbs, _, _ = self._info()
        out = np.empty((n, 2, limbs, self.ctx.N), dtype=np.uint64)
        self.ctx._check(self.ctx.lib.ensi_ct_export(self.ctx.h, self.h, _ptr(out)))
        return out
