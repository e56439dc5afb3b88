"""Plain CPU CKKS for the encrypted ternary matmul path -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package; the GPU library never does and shares no code with it.

What is computed, and from where:
  * column-wise SIMD encoding, Enc, Dec, Add, Rot: the paper's Preliminaries
    (Homomorphic Encryption and RNS-CKKS; SIMD Encoding; Rotation);
  * the multiplication-free plaintext-ciphertext product: Alg. 1 (PCMM) and the
    worked toy example before it, which fixes the index order Y = X W;
  * plaintext multiplication (Preliminaries, Multiplication) followed by one
    rescale, the secure RoPE protocol (Alg. 2) built on it, and the mask-and-add
    merge of block-placed outputs into densely packed ciphertexts (not in the
    paper: it closes the loop of the packed reading of Alg. 1);
  * ciphertext-ciphertext multiplication (Preliminaries, Multiplication: Mult)
    with relinearisation by the evaluation key and one rescale, and the
    ciphertext-ciphertext matrix product of the CCMM section built on it
    (element extraction by a one-hot mask and doubling rotate-and-add steps);
  * everything the paper leaves to its CKKS library (transform, hybrid key
    switching, rescale): the standard published definitions, in the order
    decompose -> ModUp -> automorphism -> key inner product -> ModDown.

Steps are taken one at a time, each a call into the plain C routines of
orc_kernels.c or a numpy expression; no fusion, no lazy reduction.
"""
import ctypes
import os

import numpy as np

from .params import Params

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

_u64p = ctypes.POINTER(ctypes.c_uint64)


def _lib():
    global _LIB
    if _LIB is None:
        path = os.path.join(_HERE, "liborc.so")
        if not os.path.exists(path):
            from .build import build
            build()
        _LIB = ctypes.CDLL(path)
        _LIB.orc_powmod.restype = ctypes.c_uint64
        _LIB.orc_powmod.argtypes = [ctypes.c_uint64] * 3
    return _LIB


def _p(a):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def _u64(x):
    return np.ascontiguousarray(np.array(x, dtype=np.uint64))


GK_STREAM_TAG = 2 << 56
RK_STREAM_TAG = 3 << 56
PK_STREAM = 1


class Ciphertext:
    """(c0, c1), each [l1][N] uint64 coefficient-form residues in [0, q_i)."""

    def __init__(self, c0, c1, scale):
        self.c0, self.c1, self.scale = c0, c1, scale

    @property
    def l1(self):
        return self.c0.shape[0]

    def limbs(self):
        return np.stack([self.c0, self.c1])


class Oracle:
    def __init__(self, params: Params):
        self.pr = params
        self.lib = _lib()
        pr = params
        self.N = pr.N
        self.n = pr.n_slots
        self.ext_primes_full = pr.q + pr.p
        # slot j <-> root exponent 5^j mod 2N
        e = np.empty(self.n, dtype=np.int64)
        x = 1
        for j in range(self.n):
            e[j] = x
            x = x * 5 % (2 * self.N)
        self.rot_exp = e

    # ------------------------------------------------------------------ ring
    def _primes_psi(self, primes):
        return _u64(primes), _u64([self.pr.psi[m] for m in primes])

    def ntt(self, a, primes, inverse=False):
        """a: [len(primes)][N] -> transformed copy (negacyclic, natural order)."""
        a = np.ascontiguousarray(a, dtype=np.uint64).copy()
        q, psi = self._primes_psi(primes)
        self.lib.orc_ntt(_p(a), len(primes), self.pr.log_n, _p(q), _p(psi), int(inverse))
        return a

    def polymul(self, a, b, primes):
        """Product in prod_i Z_{q_i}[X]/(X^N+1), limb-wise."""
        fa, fb = self.ntt(a, primes), self.ntt(b, primes)
        q = _u64(primes)
        c = np.empty_like(fa)
        self.lib.orc_pointwise_mul(_p(c), _p(fa), _p(fb), len(primes), self.N, _p(q))
        return self.ntt(c, primes, inverse=True)

    def polymul_naive(self, a, b, q):
        a = np.ascontiguousarray(a, dtype=np.uint64)
        b = np.ascontiguousarray(b, dtype=np.uint64)
        c = np.empty_like(a)
        self.lib.orc_negacyclic_naive(_p(c), _p(a), _p(b), len(a), ctypes.c_uint64(q))
        return c

    def add(self, a, b, primes):
        c = np.empty_like(a)
        self.lib.orc_add(_p(c), _p(np.ascontiguousarray(a)), _p(np.ascontiguousarray(b)), len(primes), self.N, _p(_u64(primes)))
        return c

    def sub(self, a, b, primes):
        c = np.empty_like(a)
        self.lib.orc_sub(_p(c), _p(np.ascontiguousarray(a)), _p(np.ascontiguousarray(b)), len(primes), self.N, _p(_u64(primes)))
        return c

    def mul_scalar(self, a, scalars, primes):
        c = np.empty_like(a)
        self.lib.orc_mul_scalar(_p(c), _p(np.ascontiguousarray(a)), _p(_u64(scalars)), len(primes), self.N, _p(_u64(primes)))
        return c

    def automorphism(self, a, g, primes):
        out = np.empty_like(a)
        self.lib.orc_automorphism(_p(out), _p(np.ascontiguousarray(a)), len(primes), self.N, ctypes.c_uint64(g), _p(_u64(primes)))
        return out

    def small_to_rns(self, v, primes):
        v = np.ascontiguousarray(v, dtype=np.int8)
        out = np.empty((len(primes), self.N), dtype=np.uint64)
        self.lib.orc_small_to_rns(_p(out), _p(v), len(primes), self.N, _p(_u64(primes)))
        return out

    def i64_to_rns(self, v, primes):
        v = np.ascontiguousarray(v, dtype=np.int64)
        out = np.empty((len(primes), self.N), dtype=np.uint64)
        self.lib.orc_i64_to_rns(_p(out), _p(v), len(primes), self.N, _p(_u64(primes)))
        return out

    def uniform(self, seed, stream, prime_ids, primes):
        out = np.empty((len(primes), self.N), dtype=np.uint64)
        for r, (pid, q) in enumerate(zip(prime_ids, primes)):
            self.lib.orc_uniform(_p(out[r]), self.N, ctypes.c_uint64(seed), ctypes.c_uint64(stream),
                                 ctypes.c_uint64(pid), ctypes.c_uint64(q))
        return out

    # -------------------------------------------------------------- encoding
    def encode_coeffs(self, z, scale=None):
        """pi: real slot vector (zero-padded to N/2) -> signed integer coefficients.
        m_k = round((2 Delta/N) Re sum_j z_j conj(zeta_j^k)), zeta_j = exp(i pi 5^j / N),
        rounding half away from zero.  Evaluated with one length-2N FFT.  Delta is the
        parameter set's scale unless another one is given."""
        N = self.N
        scale = self.pr.scale if scale is None else scale
        zz = np.zeros(self.n, dtype=np.float64)
        zz[: len(z)] = np.asarray(z, dtype=np.float64)
        A = np.zeros(2 * N, dtype=np.complex128)
        A[self.rot_exp] = zz
        A[2 * N - self.rot_exp] = zz  # conjugate positions (real input)
        m = np.fft.fft(A)[:N].real * (scale / N)
        return (np.sign(m) * np.floor(np.abs(m) + 0.5)).astype(np.int64)

    def encode_coeffs_direct(self, z):
        """Same map by the defining O(N * N/2) sum (small N only)."""
        N = self.N
        zz = np.zeros(self.n, dtype=np.float64)
        zz[: len(z)] = np.asarray(z, dtype=np.float64)
        k = np.arange(N, dtype=np.float64)[:, None]
        ang = np.pi * self.rot_exp[None, :].astype(np.float64) * k / N
        m = (2.0 * self.pr.scale / N) * (np.cos(ang) @ zz)
        return (np.sign(m) * np.floor(np.abs(m) + 0.5)).astype(np.int64)

    def decode_coeffs(self, m, scale=None):
        """z_j = m(zeta_j) / Delta for real-valued coefficient vector m (float64)."""
        N = self.N
        B = np.zeros(2 * N, dtype=np.complex128)
        B[:N] = m
        F = np.fft.ifft(B) * (2 * N)
        return F[self.rot_exp] / (scale if scale is not None else self.pr.scale)

    def encode(self, z, l1):
        return self.i64_to_rns(self.encode_coeffs(z), self.pr.q[:l1])

    # ------------------------------------------------------------------ keys
    def keygen(self, s, e, seed):
        """KeyGen (paper, Preliminaries).  s: ternary secret, e: rounded-Gaussian
        error, both int8[N] supplied by the caller; a is the counter-based uniform
        stream PK_STREAM.  pk = (-a s + e, a) over Q_L."""
        pr = self.pr
        sk = np.ascontiguousarray(s, dtype=np.int8)
        a = self.uniform(seed, PK_STREAM, range(pr.L), pr.q)
        s_rns = self.small_to_rns(sk, pr.q)
        e_rns = self.small_to_rns(e, pr.q)
        b = self.add(self.sub(np.zeros_like(a), self.polymul(a, s_rns, pr.q), pr.q), e_rns, pr.q)
        return sk, (b, a)

    def _switch_keygen(self, sk, target, e, seed, stream_base):
        """Hybrid key-switching key from the secret `target` ([L+K][N] residues, coefficient form) to s:
        for every digit j of the full chain, (b_j, a_j) over Q_L * P with b_j = -a_j s + e_j +
        [P]_{q_i} target on the limbs i of digit j only.  e: int8[beta][N]."""
        pr = self.pr
        ext = pr.q + pr.p
        ids = list(range(pr.L + pr.K))
        s_ext = self.small_to_rns(sk, ext)
        beta = pr.beta(pr.L)
        bs, as_ = [], []
        for j in range(beta):
            a = self.uniform(seed, stream_base | j, ids, ext)
            e_rns = self.small_to_rns(e[j], ext)
            b = self.add(self.sub(np.zeros_like(a), self.polymul(a, s_ext, ext), ext), e_rns, ext)
            factor = [(pr.P % ext[i]) if i in pr.digit_limbs(j, pr.L) else 0 for i in ids]
            b = self.add(b, self.mul_scalar(target, factor, ext), ext)
            bs.append(b)
            as_.append(a)
        return np.stack(bs), np.stack(as_)

    def galois_keygen(self, sk, step, e, seed):
        """Key for Rot(.; step): switches from phi_g(s) to s (g = 5^step); uniform streams
        GK_STREAM_TAG | g << 8 | j."""
        pr = self.pr
        g = pr.galois_element(step)
        ext = pr.q + pr.p
        s_g = self.automorphism(self.small_to_rns(sk, ext), g, ext)
        b, a = self._switch_keygen(sk, s_g, e, seed, GK_STREAM_TAG | (g << 8))
        return {"g": g, "step": step, "b": b, "a": a, "ntt": {}}

    def relin_keygen(self, sk, e, seed):
        """Evaluation key of Mult (paper, Preliminaries: KeyGen, evk): switches from s^2 to s;
        uniform streams RK_STREAM_TAG | j.  Used through the same inner product as a rotation
        key with the identity automorphism (g = 1)."""
        pr = self.pr
        ext = pr.q + pr.p
        s_ext = self.small_to_rns(sk, ext)
        b, a = self._switch_keygen(sk, self.polymul(s_ext, s_ext, ext), e, seed, RK_STREAM_TAG)
        return {"g": 1, "step": 0, "b": b, "a": a, "ntt": {}}

    # ------------------------------------------------------- encrypt/decrypt
    def encrypt(self, pt_rns, pk, v, e0, e1):
        """Enc_pk (paper, Preliminaries): ct = v pk + (m + e0, e1) at the level of pt."""
        l1 = pt_rns.shape[0]
        pr = self.pr
        q = pr.q[:l1]
        v_rns = self.small_to_rns(v, q)
        c0 = self.add(self.add(self.polymul(v_rns, pk[0][:l1], q), pt_rns, q), self.small_to_rns(e0, q), q)
        c1 = self.add(self.polymul(v_rns, pk[1][:l1], q), self.small_to_rns(e1, q), q)
        return Ciphertext(c0, c1, pr.scale)

    def decrypt_coeffs(self, ct, sk):
        """c0 + c1 s, CRT of limbs 0 and 1, centred; float64 coefficients."""
        pr = self.pr
        l1 = ct.l1
        use = min(l1, 2)
        q = pr.q[:use]
        s_rns = self.small_to_rns(sk, q)
        m = self.add(ct.c0[:use], self.polymul(np.ascontiguousarray(ct.c1[:use]), s_rns, q), q)
        out = np.empty(self.N, dtype=np.float64)
        if use == 2:
            self.lib.orc_crt2_center(_p(out), _p(np.ascontiguousarray(m[0])), _p(np.ascontiguousarray(m[1])),
                                     ctypes.c_uint64(q[0]), ctypes.c_uint64(q[1]), self.N)
        else:
            self.lib.orc_center1(_p(out), _p(np.ascontiguousarray(m[0])), ctypes.c_uint64(q[0]), self.N)
        return out

    def decrypt(self, ct, sk):
        """Dec_sk followed by decoding; returns the real parts of all N/2 slots."""
        return self.decode_coeffs(self.decrypt_coeffs(ct, sk), ct.scale).real

    # ---------------------------------------------------------- key switching
    def bconv(self, src, qs, inv, tgt, hat, centered=False):
        out = np.empty((len(tgt), self.N), dtype=np.uint64)
        self.lib.orc_bconv(_p(out), _p(np.ascontiguousarray(src)), len(qs), len(tgt), self.N, _p(_u64(qs)), _p(_u64(inv)),
                           _p(_u64(hat)), _p(_u64(tgt)), int(centered))
        return out

    def mod_up(self, c1):
        """Digit decomposition + ModUp: [l1][N] -> [beta][l1+K][N], coefficient form.
        Limbs inside a digit are copied; every other limb of Q_l and all of P gets
        the fast basis conversion of the digit (no overflow correction)."""
        pr = self.pr
        l1 = c1.shape[0]
        out = np.empty((pr.beta(l1), l1 + pr.K, self.N), dtype=np.uint64)
        for j in range(pr.beta(l1)):
            src, qs, inv, tgt_idx, tgt, hat = pr.modup_constants(j, l1)
            out[j, src] = c1[src]
            out[j, tgt_idx] = self.bconv(c1[src], qs, inv, tgt, hat)
        return out

    def mod_down(self, u, l1):
        """[l1+K][N] -> [l1][N]: (u - BConv_{P->Q}([u]_P)) * P^{-1} mod q_i.  The conversion takes
        the residues [u P_k^^-1]_{p_k} centred, so what is subtracted is [u]_P + v P with v
        symmetric around zero: the division error then has no constant component (an uncentred
        conversion leaves a mean of about (K-1)/2 per coefficient, which the decoding
        concentrates on the few slots whose roots are nearest 1)."""
        pr = self.pr
        inv, tgt, hat, p_inv = pr.moddown_constants(l1)
        r = self.bconv(u[l1:], pr.p, inv, tgt, hat, centered=True)
        return self.mul_scalar(self.sub(np.ascontiguousarray(u[:l1]), r, tgt), p_inv, tgt)

    def _key_at_level(self, gk, l1):
        pr = self.pr
        if l1 not in gk["ntt"]:
            sel = list(range(l1)) + list(range(pr.L, pr.L + pr.K))
            primes = [(pr.q + pr.p)[i] for i in sel]
            beta = pr.beta(l1)
            kb = np.stack([self.ntt(gk["b"][j][sel], primes) for j in range(beta)])
            ka = np.stack([self.ntt(gk["a"][j][sel], primes) for j in range(beta)])
            gk["ntt"] = {l1: (primes, kb, ka)}
        return gk["ntt"][l1]

    def _key_inner_product(self, digits, gk, l1):
        """Automorphism of every raised digit and the inner product with the key over the extended
        basis: (u0, u1), transform domain."""
        pr = self.pr
        g = gk["g"]
        primes, kb, ka = self._key_at_level(gk, l1)
        qv = _u64(primes)
        u0 = np.zeros((l1 + pr.K, self.N), dtype=np.uint64)
        u1 = np.zeros_like(u0)
        for j in range(digits.shape[0]):
            dg = self.ntt(self.automorphism(digits[j], g, primes), primes)
            self.lib.orc_pointwise_mac(_p(u0), _p(dg), _p(np.ascontiguousarray(kb[j])), len(primes), self.N, _p(qv))
            self.lib.orc_pointwise_mac(_p(u1), _p(dg), _p(np.ascontiguousarray(ka[j])), len(primes), self.N, _p(qv))
        return primes, u0, u1

    def rotate_from_digits(self, c0, digits, gk, scale):
        """Steps c-f of the rotation: automorphism of every raised digit and of c0,
        key inner product over the extended basis, ModDown, add phi_g(c0)."""
        return self.rotate_sum_from_digits(c0, digits, [gk], scale)

    def rotate_sum_from_digits(self, c0, digits, gks, scale):
        """sum_k Rot(.; step_k) of one ciphertext with one ModDown: the key inner products of all
        members are added over the extended basis before the inverse transform and the division by
        P (ModDown is linear up to its rounding, so this is a key switch of the sum with one
        rounding instead of one per member), then sum_k phi_{g_k}(c0) is added.  With one member it
        is the rotation itself."""
        l1 = c0.shape[0]
        u0 = u1 = None
        for gk in gks:
            primes, v0, v1 = self._key_inner_product(digits, gk, l1)
            u0 = v0 if u0 is None else self.add(u0, v0, primes)
            u1 = v1 if u1 is None else self.add(u1, v1, primes)
        u0 = self.ntt(u0, primes, inverse=True)
        u1 = self.ntt(u1, primes, inverse=True)
        q = self.pr.q[:l1]
        out0 = self.mod_down(u0, l1)
        for gk in gks:
            out0 = self.add(out0, self.automorphism(np.ascontiguousarray(c0), gk["g"], q), q)
        out1 = self.mod_down(u1, l1)
        return Ciphertext(out0, out1, scale)

    def rotate(self, ct, gk):
        """Rot(ct; k) for the step the key was generated for (paper, Rotation)."""
        return self.rotate_from_digits(ct.c0, self.mod_up(ct.c1), gk, ct.scale)

    # ------------------------------------------------------------------ PCMM
    @staticmethod
    def placement_block(i, c_tot, placement):
        return 0 if placement == "zero" else i % c_tot

    def plan(self, W, c_tot, placement):
        """For output i: list of (packed input G, rotation amount rho, sign) with
        virtual column j = G*c_tot + b needed at rho = (b - p_i) mod c_tot."""
        d, m = W.shape
        plan = []
        for i in range(m):
            p_i = self.placement_block(i, c_tot, placement)
            terms = []
            for j in range(d):
                w = int(W[j, i])
                if w:
                    terms.append((j // c_tot, (j % c_tot - p_i) % c_tot, w))
            plan.append(terms)
        return plan

    def accumulate(self, terms, l1, scale):
        """Alg. 1 for one output: y starts as the all-zero ciphertext; add the
        operand where the weight is +1, subtract where it is -1, skip zeros.
        terms: list of (Ciphertext, sign)."""
        q = _u64(self.pr.q[:l1])
        outs = []
        for poly in (0, 1):
            y = np.empty((l1, self.N), dtype=np.uint64)
            keep = [np.ascontiguousarray(t.c0 if poly == 0 else t.c1) for t, _ in terms]
            ptrs = (ctypes.c_void_p * max(1, len(keep)))(*[a.ctypes.data for a in keep])
            signs = np.array([sg for _, sg in terms], dtype=np.int8)
            self.lib.orc_signed_accumulate(_p(y), ptrs, _p(np.ascontiguousarray(signs)), len(keep), l1, self.N, _p(q))
            outs.append(y)
        return Ciphertext(outs[0], outs[1], scale)

    def ternary_matmul(self, cts, s, d, W, placement, gks):
        """Y = X W on ciphertexts (Alg. 1).  cts: packed inputs, ciphertext G
        holding column G*c_tot+b in slot block b; gks: {rho: key for step rho*s}.
        Unpacks by rotations into column-aligned operands, then add/sub only."""
        c_tot = self.n // s
        W = np.asarray(W)
        assert W.shape[0] == d and len(cts) == -(-d // c_tot)
        plan = self.plan(W, c_tot, placement)
        need = sorted({(G, rho) for terms in plan for (G, rho, _) in terms})
        digits = {}
        virt = {}
        for G, rho in need:
            if rho == 0:
                virt[(G, rho)] = cts[G]
                continue
            if G not in digits:
                digits[G] = self.mod_up(cts[G].c1)
            virt[(G, rho)] = self.rotate_from_digits(cts[G].c0, digits[G], gks[rho], cts[G].scale)
        l1, scale = cts[0].l1, cts[0].scale
        return [self.accumulate([(virt[(G, rho)], w) for (G, rho, w) in terms], l1, scale) for terms in plan]

    # --------------------------------------------------------------- rescale
    def mul_scalar_rescale(self, ct, kappa):
        """c <- c * round(kappa q_l) (negative constants as q_i - |.|), then drop limb l:
        c'_i = (c_i - [c_l]) q_l^{-1} mod q_i with [c_l] the centred representative of limb l in
        (-q_l/2, q_l/2] (division with rounding to nearest: zero-mean error).  The encoded
        values are multiplied by kappa; the scale only absorbs the rounding of the
        constant: scale' = scale * round(kappa q_l) / (kappa q_l)."""
        pr = self.pr
        l1 = ct.l1
        ql = pr.q[l1 - 1]
        k = int(np.sign(kappa) * np.floor(abs(kappa) * ql + 0.5))
        q = pr.q[:l1]
        const = [k % m for m in q]
        rest = q[: l1 - 1]
        ql_inv = [pow(ql, -1, m) for m in rest]
        out = []
        for c in (ct.c0, ct.c1):
            c = self.mul_scalar(np.ascontiguousarray(c), const, q)
            top = c[l1 - 1]
            neg = top > np.uint64(ql // 2)  # centred representative is top - ql
            last = np.stack([np.where(neg, (top % np.uint64(m) + np.uint64(m - ql % m)) % np.uint64(m), top % np.uint64(m)) for m in rest])
            out.append(self.mul_scalar(self.sub(np.ascontiguousarray(c[: l1 - 1]), last, rest), ql_inv, rest))
        return Ciphertext(out[0], out[1], ct.scale * k / (kappa * ql))

    # ---------------------------------------------- plaintext multiplication
    def rescale(self, ct):
        """Drops limb l: c'_i = (c_i - [c_l]) q_l^{-1} mod q_i, [c_l] the centred
        representative of limb l in (-q_l/2, q_l/2], i.e. the exact integer quotient
        round(c / q_l) of the centred coefficient; the scale is divided by q_l."""
        pr = self.pr
        l1 = ct.l1
        ql = pr.q[l1 - 1]
        rest = pr.q[: l1 - 1]
        ql_inv = [pow(ql, -1, m) for m in rest]
        out = []
        for c in (ct.c0, ct.c1):
            top = c[l1 - 1]
            neg = top > np.uint64(ql // 2)
            last = np.stack([np.where(neg, (top % np.uint64(m) + np.uint64(m - ql % m)) % np.uint64(m), top % np.uint64(m)) for m in rest])
            out.append(self.mul_scalar(self.sub(np.ascontiguousarray(c[: l1 - 1]), last, rest), ql_inv, rest))
        return Ciphertext(out[0], out[1], ct.scale / ql)

    def pmult(self, ct, pt, pt_scale):
        """PMult (Preliminaries, Multiplication): (c0 m, c1 m) in R_{Q_l}; pt is the
        plaintext polynomial m as [l1][N] residues; the scales multiply.  No rescale."""
        q = self.pr.q[: ct.l1]
        return Ciphertext(self.polymul(ct.c0, pt, q), self.polymul(ct.c1, pt, q), ct.scale * pt_scale)

    def add_ct(self, a, b):
        """Add (Preliminaries): component-wise sum; both at the same level and scale."""
        q = self.pr.q[: a.l1]
        return Ciphertext(self.add(a.c0, b.c0, q), self.add(a.c1, b.c1, q), a.scale)

    def pmult_sum_rescale(self, terms, pt_scale):
        """Rescale(sum_t ct_t [x] pt_t): the products are added at the product scale and the
        sum is rescaled once.  terms: list of (Ciphertext, pt residues [l1][N])."""
        acc = None
        for ct, pt in terms:
            prod = self.pmult(ct, pt, pt_scale)
            acc = prod if acc is None else self.add_ct(acc, prod)
        return self.rescale(acc)

    # -------------------------------------------------------- Alg. 2 (RoPE)
    @staticmethod
    def rope_masks(n):
        """neg = (-1, 0, -1, 0, ...), pos = (0, 1, 0, 1, ...) over n slots (Alg. 2, first step)."""
        j = np.arange(n)
        return np.where(j % 2 == 0, -1.0, 0.0), np.where(j % 2 == 1, 1.0, 0.0)

    def rope_plaintexts(self, cos, sin, l1):
        """The three plaintext polynomials Alg. 2 multiplies by, as integer coefficients
        [3][N] at scale q_l (the prime the rescale drops, so the ciphertext scale is
        unchanged): cos, neg (.) sin and pos (.) sin.  The 0/+-1 masks are applied to the
        sin vector in the clear: multiplying a ciphertext by a mask and then by sin would
        cost two levels, and the paper's operation table gives RoPE one level."""
        neg, pos = self.rope_masks(self.n)
        ql = float(self.pr.q[l1 - 1])
        c = np.zeros(self.n)
        s = np.zeros(self.n)
        c[: len(cos)] = cos
        s[: len(sin)] = sin
        return np.stack([self.encode_coeffs(v, ql) for v in (c, neg * s, pos * s)])

    def rope(self, q_ct, pts, gk_plus, gk_minus):
        """Alg. 2 on one ciphertext: r = Rot(q; 1) [x] neg, l = Rot(q; -1) [x] pos, t = r + l,
        y = q [x] cos + t [x] sin, with the masks folded into sin (rope_plaintexts) so that
        y = Rescale(q [x] cos + Rot(q; 1) [x] (neg sin) + Rot(q; -1) [x] (pos sin)).
        pts: integer coefficients [3][N] from rope_plaintexts; gk_plus / gk_minus: Galois keys
        of steps +1 and -1.  One ModUp serves both rotations."""
        l1 = q_ct.l1
        prm = self.pr.q[:l1]
        ql = float(prm[-1])
        rns = [self.i64_to_rns(p, prm) for p in pts]
        digits = self.mod_up(q_ct.c1)
        r = self.rotate_from_digits(q_ct.c0, digits, gk_plus, q_ct.scale)
        l = self.rotate_from_digits(q_ct.c0, digits, gk_minus, q_ct.scale)
        return self.pmult_sum_rescale([(q_ct, rns[0]), (r, rns[1]), (l, rns[2])], ql)

    # ------------------------------------------- merge of placed outputs
    def block_masks(self, s, c_tot, l1):
        """Integer coefficients [c_tot][N] of the slot masks 1 on block b = slots [b s, (b+1) s),
        0 elsewhere, at scale q_l."""
        ql = float(self.pr.q[l1 - 1])
        out = []
        for b in range(c_tot):
            z = np.zeros(self.n)
            z[b * s:(b + 1) * s] = 1.0
            out.append(self.encode_coeffs(z, ql))
        return np.stack(out)

    def merge(self, cts, masks, c_tot):
        """Packs outputs placed by block (output i carries its column in block i mod c_tot)
        into dense ciphertexts: packed_G = Rescale(sum_b y_{G c_tot + b} [x] mask_b).  masks:
        integer coefficients from block_masks.  A ragged last group simply has fewer terms."""
        l1 = cts[0].l1
        prm = self.pr.q[:l1]
        ql = float(prm[-1])
        rns = [self.i64_to_rns(m, prm) for m in masks]
        out = []
        for g0 in range(0, len(cts), c_tot):
            grp = cts[g0:g0 + c_tot]
            out.append(self.pmult_sum_rescale([(ct, rns[b]) for b, ct in enumerate(grp)], ql))
        return out

    # ------------------------------------- ciphertext-ciphertext multiplication
    def drop_limbs(self, ct, l1):
        """Level alignment: the same ciphertext modulo Q_{l1} (its last limbs are dropped, the
        scale is unchanged)."""
        return Ciphertext(np.ascontiguousarray(ct.c0[:l1]), np.ascontiguousarray(ct.c1[:l1]), ct.scale)

    def tensor_sum(self, pairs):
        """sum_t a_t (x) b_t before relinearisation: (d0, d1, d2) = (sum a0 b0, sum a0 b1 + a1 b0,
        sum a1 b1), which decrypts under (1, s, s^2)."""
        l1 = pairs[0][0].l1
        q = self.pr.q[:l1]
        d = [np.zeros((l1, self.N), dtype=np.uint64) for _ in range(3)]
        for a, b in pairs:
            d[0] = self.add(d[0], self.polymul(a.c0, b.c0, q), q)
            d[1] = self.add(d[1], self.add(self.polymul(a.c0, b.c1, q), self.polymul(a.c1, b.c0, q), q), q)
            d[2] = self.add(d[2], self.polymul(a.c1, b.c1, q), q)
        return d

    def relinearize(self, d, rk, scale):
        """(d0, d1, d2) -> (d0 + KS_0(d2), d1 + KS_1(d2)) with the evaluation key: the hybrid key
        switch of the rotation (decompose, ModUp, inner product, ModDown) with g = 1."""
        ks = self.rotate_from_digits(d[0], self.mod_up(d[2]), rk, scale)
        q = self.pr.q[: d[0].shape[0]]
        return Ciphertext(ks.c0, self.add(ks.c1, d[1], q), scale)

    def mult_sum_relin_rescale(self, pairs, rk):
        """Rescale(Relin(sum_t a_t (x) b_t)): Mult (paper, Preliminaries) on every pair, the
        products added before the one relinearisation and the one rescale."""
        a0, b0 = pairs[0]
        return self.rescale(self.relinearize(self.tensor_sum(pairs), rk, a0.scale * b0.scale))

    # ------------------------------------------------------------------ CCMM
    def one_hot_masks(self, ks, l1):
        """Integer coefficients [len(ks)][N] of the masks (0,..,0,1,0,..,0) with the 1 in slot k, at scale q_l."""
        ql = float(self.pr.q[l1 - 1])
        out = []
        for k in ks:
            z = np.zeros(self.n)
            z[k] = 1.0
            out.append(self.encode_coeffs(z, ql))
        return np.stack(out)

    @staticmethod
    def fill_steps(r_begin, r_end, sign=1):
        """Rotation steps of the rotate-and-add fill t <- sum_{e < r_end / r_begin} Rot(t; sign e r_begin)
        (r_end / r_begin a power of two), as a list of groups: while two doublings remain they are taken
        as one step of radix four, t <- t + Rot(t; r) + Rot(t; 2r) + Rot(t; 3r), whose three rotations
        share one ModUp of t and one ModDown (rotate_sum_from_digits); a last single doubling is
        t <- t + Rot(t; r)."""
        groups, r = [], r_begin
        while r < r_end:
            if 2 * r < r_end:
                groups.append([sign * r, sign * 2 * r, sign * 3 * r])
                r *= 4
            else:
                groups.append([sign * r])
                r *= 2
        return groups

    def fill(self, t, r_begin, r_end, gks, sign=1):
        """The fill of fill_steps on a ciphertext; gks: dict step -> Galois key."""
        for group in self.fill_steps(r_begin, r_end, sign):
            t = self.add_ct(t, self.rotate_sum_from_digits(t.c0, self.mod_up(t.c1), [gks[step] for step in group], t.scale))
        return t

    def replicate(self, ct, mask, gks):
        """The element-extraction step of the CCMM section: keep one slot (PMult by its mask, one
        rescale), then copy it into every slot by the rotate-and-add fill of fill_steps over all
        N/2 slots.  gks: dict step -> Galois key for the steps of fill_steps(1, N/2).  The figure with the paper's own
        schedule is not in the text; this rotate-and-add schedule reaches the logarithmic
        rotation count it states."""
        l1 = ct.l1
        ql = float(self.pr.q[l1 - 1])
        t = self.pmult_sum_rescale([(ct, self.i64_to_rns(mask, self.pr.q[:l1]))], ql)
        return self.fill(t, 1, self.n, gks)

    def periodic_masks(self, period, count, l1):
        """Integer coefficients [count][N] of the masks with a 1 in every slot congruent to j modulo
        `period` (j = 0..count-1), 0 elsewhere, at scale q_l."""
        ql = float(self.pr.q[l1 - 1])
        out = []
        for j in range(count):
            z = np.zeros(self.n)
            z[j::period] = 1.0
            out.append(self.encode_coeffs(z, ql))
        return np.stack(out)

    def spread_periods(self, ct, period, gks):
        """Giant steps of the element extraction, shared by all elements of a column: a ciphertext
        whose slots beyond the first `period` are zero becomes periodic, u[p] = ct[p mod period], by
        the fill of fill_steps(period, N/2).  No level is consumed."""
        return self.fill(ct, period, self.n, gks)

    def extract_from_periodic(self, u, mask, period, gks):
        """Baby steps, per element: keep the slots congruent to j modulo the period (PMult by the
        periodic mask, one rescale), then fill every window of `period` slots from its single
        non-zero entry by the fill of fill_steps(1, period)."""
        l1 = u.l1
        ql = float(self.pr.q[l1 - 1])
        t = self.pmult_sum_rescale([(u, self.i64_to_rns(mask, self.pr.q[:l1]))], ql)
        return self.fill(t, 1, period, gks)

    def ccmm(self, a_cts, b_cts, d, period, rk, gks):
        """C = A B on ciphertexts (CCMM section): A column-encoded (a_j = column j, tokens along the
        slots), b_i = column i of B with B[j, i] in slot j < d and zeros in every other slot;
        c_i = sum_j a_j (x) b_i^(j), where b_i^(j) is B[j, i] replicated into every slot.  Element
        extraction in two stages (period = a power of two >= d): log2(n/period) rotate-and-add steps
        per column make it periodic, then per element one mask product and log2(period) steps.  The
        figure with the paper's own baby-step giant-step schedule is not in its text; this one shares
        the giant steps among the d elements of a column and has the logarithmic rotation count per
        element the text states.  Costs two levels (mask, product)."""
        l1 = b_cts[0].l1
        masks = self.periodic_masks(period, d, l1)
        out = []
        for b in b_cts:
            u = self.spread_periods(b, period, gks)
            reps = [self.extract_from_periodic(u, masks[j], period, gks) for j in range(d)]
            out.append(self.mult_sum_relin_rescale([(self.drop_limbs(a_cts[j], l1 - 1), reps[j]) for j in range(d)], rk))
        return out

    # ------------------------------------------- CCMM with several heads per ciphertext
    def block_start_mask(self, s, l1):
        """Integer coefficients [N] of the mask with a 1 in the first slot of every block of s slots, at scale q_l."""
        z = np.zeros(self.n)
        z[::s] = 1.0
        return self.encode_coeffs(z, float(self.pr.q[l1 - 1]))

    def extract_blockwise(self, ct, i, s, mask0, gks):
        """Element extraction when a ciphertext packs one block of s slots per head: slot i of every
        block is copied into all s slots of its block.  Rot(.; i) brings it to the block's first
        slot, the block-start mask keeps it (PMult, one rescale), and log2(s) steps
        the fill of fill_steps(1, s, -1) copies it upwards through the block without touching the next one.
        gks: dict step -> Galois key, with the steps i and -2^k."""
        l1 = ct.l1
        ql = float(self.pr.q[l1 - 1])
        t = self.rotate(ct, gks[i]) if i else ct
        t = self.pmult_sum_rescale([(t, self.i64_to_rns(mask0, self.pr.q[:l1]))], ql)
        return self.fill(t, 1, s, gks, sign=-1)

    def ccmm_blocks(self, a_cts, b_cts, s, cols, rk, gks):
        """C_h = A_h B_h for all heads h at once (CCMM section, the column-encoded by row-encoded
        form): ciphertext j of A holds column j of every A_h (head h in slot block h, s tokens), and
        ciphertext j of B holds, in slot h s + i, the entry B_h[j, i] -- i.e. B^T column-encoded,
        as K is for Q K^T.  Output column i (one ciphertext, block h = column i of C_h) is
        sum_j a_j (x) b^(j,i) with b^(j,i) the block-wise replication of slot i of b_j.  cols: the
        output columns to compute.  Two levels (mask, product)."""
        l1 = b_cts[0].l1
        mask0 = self.block_start_mask(s, l1)
        out = []
        for i in cols:
            reps = [self.extract_blockwise(b, i, s, mask0, gks) for b in b_cts]
            out.append(self.mult_sum_relin_rescale([(self.drop_limbs(a, l1 - 1), r) for a, r in zip(a_cts, reps)], rk))
        return out

    # ------------- CCMM over heads, a whole segment of output columns at once (no baby-step fills)
    def segment_masks(self, s, period, l1):
        """Integer coefficients [3 period][N] of the masks that sort the diagonals of ccmm_segment into
        columns, at scale q_l: for r < period, R_r (index r) = 1 in the slots of every block whose offset
        is congruent to r modulo the period; R_r^- (index period + r) = R_r without the last period of
        the block; T_r (index 2 period + r) = R_r in the last period only."""
        ql = float(self.pr.q[l1 - 1])
        out = []
        for kind in range(3):
            for r in range(period):
                z = np.zeros(self.n)
                for b0 in range(0, self.n, s):
                    if kind != 2:
                        z[b0 + r:b0 + s - (period if kind == 1 else 0):period] = 1.0
                    else:
                        z[b0 + s - period + r] = 1.0
                out.append(self.encode_coeffs(z, ql))
        return np.stack(out)

    @staticmethod
    def segment_mask_terms(period, c):
        """Which diagonal feeds output column c of a segment through which mask: a list of
        (e, primed, mask index into segment_masks).  Slot x of diagonal D_e holds column
        (x + e) mod period, so column c takes the residue class r = (c - e) mod period of D_e; where
        that class meets the last e slots of a block (r >= period - e) those slots come from D'_e."""
        terms = []
        for e in range(period):
            r = (c - e) % period
            if e and r >= period - e:
                terms.append((e, False, period + r))
                terms.append((e, True, 2 * period + r))
            else:
                terms.append((e, False, r))
        return terms

    @staticmethod
    def diagonal_schedule(period, baby):
        """Baby steps and giant steps over the diagonals of a segment: diagonal q (q < period: rotation
        amount q; q >= period: amount q - 2 period + 1, the one used in the last slots of a block) has
        amount = e1 + t with 0 <= e1 < baby and t a multiple of baby; returns the list of (e1, t).
        The operand that is rotated per product only moves by e1; the other operand is pre-rotated by
        -t and the sum of all products with the same t is rotated by t afterwards."""
        out = []
        for q in range(2 * period - 1):
            amount = q if q < period else q - 2 * period + 1
            e1 = amount % baby
            out.append((e1, amount - e1))
        return out

    def ccmm_segment(self, a_cts, b_cts, s, period, baby, g, rk, gks):
        """CCMM section, several heads per ciphertext, the `period` output columns g period ..
        (g+1) period - 1 of C_h = A_h B_h at once (the Q K^T form: ciphertext j of B holds B_h[j, i] in
        slot h s + i).  The replication of an element stops at the giant step: w_j = the segment of b_j
        repeated through every block (spread_segment).  Then Rot(w_j; e) puts, in slot x, element
        (x + e) mod period of the segment, so D_e = sum_j a_j (x) Rot(w_j; e) holds in slot x the
        entry of output column (x + e) mod period: the period diagonals hold all entries of the
        period columns.  A rotation by e reads past the block's end in its last e slots; there
        D'_e, built with Rot(w_j; e - period), holds the same entries.  Baby and giant steps over the
        diagonals (diagonal_schedule, amount = e1 + t): w_j is rotated by e1 < baby only, a_j by -t,
        and the relinearised sum of their products by t, at the product's scale, before its rescale.
        One more plaintext product sorts the diagonals: column c = Rescale(sum_e mask (.) D_e [+ mask'
        (.) D'_e]) (segment_mask_terms).  Three levels (head mask, product, sorting masks)."""
        l1 = b_cts[0].l1
        mask_head = self.block_head_mask(s, period, l1)
        w = [self.spread_segment(b, g, s, period, mask_head, gks) for b in b_cts]
        a2 = [self.drop_limbs(a, l1 - 1) for a in a_cts]
        sched = self.diagonal_schedule(period, baby)
        w_rot = {0: w}
        a_rot = {0: a2}
        for e1, t in sched:
            if e1 not in w_rot:
                w_rot[e1] = [self.rotate(wj, gks[e1]) for wj in w]
            if t not in a_rot:
                a_rot[t] = [self.rotate(aj, gks[-t]) for aj in a2]
        d_all = []
        for e1, t in sched:
            pairs = list(zip(a_rot[t], w_rot[e1]))
            part = self.relinearize(self.tensor_sum(pairs), rk, pairs[0][0].scale * pairs[0][1].scale)
            if t:
                part = self.rotate(part, gks[t])
            d_all.append(self.rescale(part))
        diag, diag_p = d_all[:period], [None] + d_all[period:]
        masks = self.segment_masks(s, period, l1 - 2)
        q = self.pr.q[:l1 - 2]
        out = []
        for c in range(period):
            terms = [((diag_p if primed else diag)[e], self.i64_to_rns(masks[mi], q)) for e, primed, mi in self.segment_mask_terms(period, c)]
            out.append(self.pmult_sum_rescale(terms, float(self.pr.q[l1 - 3])))
        return out

    def diagonalise_weights(self, a_cts, s, period, baby, gks):
        """The left operand of ccmm_av in the arrangement its right operand's rotations need: a_cts
        = the `period` columns g period + c of A (column-encoded, one block of s slots per head);
        returns 2 period - 1 ciphertexts one level down.  Entry e < period: slot x holds column
        (x + e) mod period where x + e stays inside the block, 0 in the block's last e slots; entry
        period - 1 + e (e >= 1): the same column in those last e slots, 0 elsewhere (plaintext
        products with the masks of segment_masks, summed and rescaled once); each entry is then
        rotated by -t, its giant step of diagonal_schedule."""
        l1 = a_cts[0].l1
        masks = self.segment_masks(s, period, l1)
        q = self.pr.q[:l1]
        ql = float(self.pr.q[l1 - 1])
        lo, hi = [], []
        for e in range(period):
            tl, th = [], []
            for c in range(period):
                r = (c - e) % period
                if e and r >= period - e:
                    tl.append((a_cts[c], self.i64_to_rns(masks[period + r], q)))
                    th.append((a_cts[c], self.i64_to_rns(masks[2 * period + r], q)))
                else:
                    tl.append((a_cts[c], self.i64_to_rns(masks[r], q)))
            lo.append(self.pmult_sum_rescale(tl, ql))
            if e:
                hi.append(self.pmult_sum_rescale(th, ql))
        sched = self.diagonal_schedule(period, baby)
        return [self.rotate(ct, gks[-t]) if t else ct for ct, (_, t) in zip(lo + hi, sched)]

    def ccmm_av(self, ad_segs, v_cts, s, period, baby, g0, rk, gks):
        """CCMM section, several heads per ciphertext, the weights-times-V form: out_i = sum_j a_j (x)
        E(v_i, j) over the tokens j of the segments g0, g0 + 1, ... (ad_segs[k] = diagonalise_weights
        of the columns of segment g0 + k), without replicating single elements: with w = the
        segment of v_i repeated through every block (spread_segment), slot x of Rot(w; e) holds
        V[g period + (x + e) mod period, i], which is what diagonal e of the weights multiplies in
        that slot; the last e slots of a block take Rot(w; e - period) and diagonal period - 1 + e.
        Baby steps and giant steps over the diagonals (diagonal_schedule): w is only rotated by e1 <
        baby; the products whose diagonals share a giant step t are added and relinearised together,
        that sum is rotated by t at the product's scale (a key switch after the rescale would add its
        rounding to a ciphertext of scale Delta^2 / q_l, a thousand times less headroom), and out_i is
        the sum over t, rescaled once.  Two levels (masks on both operands, the product)."""
        l1 = v_cts[0].l1
        mask_head = self.block_head_mask(s, period, l1)
        sched = self.diagonal_schedule(period, baby)
        out = []
        for v in v_cts:
            groups = {}
            for k, ad in enumerate(ad_segs):
                w = self.spread_segment(v, g0 + k, s, period, mask_head, gks)
                rot = [w] + [self.rotate(w, gks[e1]) for e1 in range(1, baby)]
                for q, (e1, t) in enumerate(sched):
                    groups.setdefault(t, []).append((ad[q], rot[e1]))
            acc = None
            for t in sorted(groups):
                a0, b0 = groups[t][0]
                part = self.relinearize(self.tensor_sum(groups[t]), rk, a0.scale * b0.scale)
                if t:
                    part = self.rotate(part, gks[t])
                acc = part if acc is None else self.add_ct(acc, part)
            out.append(self.rescale(acc))
        return out

    # ------------------------- CCMM over heads, element extraction in baby steps and giant steps
    def block_head_mask(self, s, period, l1):
        """Integer coefficients [N] of the mask with a 1 in the first `period` slots of every block of s slots, at scale q_l."""
        z = np.zeros(self.n)
        for x in range(period):
            z[x::s] = 1.0
        return self.encode_coeffs(z, float(self.pr.q[l1 - 1]))

    def spread_segment(self, ct, g, s, period, mask_head, gks):
        """Giant step of the block-wise extraction, shared by the `period` elements of a segment:
        Rot(.; g period) brings slots [g period, (g+1) period) of every block to the block's start,
        the head mask keeps them (PMult, one rescale), and the fill of fill_steps(period, s, -1)
        repeats them upwards through the block: slot h s + x then holds slot h s + g period +
        (x mod period) of the input."""
        l1 = ct.l1
        t = self.rotate(ct, gks[g * period]) if g else ct
        t = self.pmult_sum_rescale([(t, self.i64_to_rns(mask_head, self.pr.q[:l1]))], float(self.pr.q[l1 - 1]))
        return self.fill(t, period, s, gks, sign=-1)

    def extract_from_segment(self, w, b, period, mask_start, gks):
        """Baby step, per element: Rot(.; b) brings element b of every period of the spread segment
        to the period's first slot, the mask of the slots congruent to 0 modulo the period keeps it
        (PMult, one rescale) and the fill of fill_steps(1, period, -1) copies it upwards through its
        period.  Nothing crosses a block boundary: every read stays below the block's end."""
        l1 = w.l1
        t = self.rotate(w, gks[b]) if b else w
        t = self.pmult_sum_rescale([(t, self.i64_to_rns(mask_start, self.pr.q[:l1]))], float(self.pr.q[l1 - 1]))
        return self.fill(t, 1, period, gks, sign=-1)

    def ccmm_bsgs(self, a_cts, b_cts, s, period, terms, rk, gks):
        """CCMM section, several heads per ciphertext (blocks of s slots), with the element
        extraction split into giant and baby steps: out_o = sum over (ia, ib, slot) in terms[o] of
        a_ia (x) E(b_ib, slot), where E copies slot `slot` of every block of b_ib into all s slots
        of its block, slot = g period + b.  Segments (ib, g) and elements (ib, slot) that several
        terms name are formed once.  Q K^T: terms[o] = [(j, j, i_o) for j]; weights times V:
        terms[i] = [(j, i, j) for j].  Three levels (two masks, the product)."""
        l1 = b_cts[0].l1
        mask_head = self.block_head_mask(s, period, l1)
        mask_start = self.periodic_masks(period, 1, l1 - 1)[0]
        segs, reps, out = {}, {}, []
        for tl in terms:
            pairs = []
            for ia, ib, slot in tl:
                g, b = divmod(slot, period)
                if (ib, g) not in segs:
                    segs[(ib, g)] = self.spread_segment(b_cts[ib], g, s, period, mask_head, gks)
                if (ib, slot) not in reps:
                    reps[(ib, slot)] = self.extract_from_segment(segs[(ib, g)], b, period, mask_start, gks)
                pairs.append((self.drop_limbs(a_cts[ia], l1 - 2), reps[(ib, slot)]))
            out.append(self.mult_sum_relin_rescale(pairs, rk))
        return out
