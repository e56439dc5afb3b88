"""Shared set-up for the parity tests: the same seeded randomness is handed to the
CPU oracle and to the GPU library, which then have to agree bit for bit."""
import numpy as np

import workloads as wl
from oracle import Oracle, Params
from oracle.ckks import Ciphertext


class Pair:
    """Oracle + library context on one parameter set, with one key pair."""

    def __init__(self, param_tuple, seed=7, key_seed=1234):
        from paper_2509_09424_amd import binding
        self.binding = binding
        self.pr = Params(*param_tuple)
        self.o = Oracle(self.pr)
        self.ctx = binding.Context(*param_tuple, seed=seed)
        self.rng = np.random.default_rng(seed)
        self.N, self.n = self.o.N, self.o.n
        self.key_seed = key_seed
        s, e = wl.ternary_poly(self.rng, self.N), wl.error_poly(self.rng, self.N)
        self.o_sk, self.o_pk = self.o.keygen(s, e, key_seed)
        self.g_sk, self.g_pk = self.ctx.keygen(s, e, key_seed)

    def close(self):
        self.ctx.close()

    def galois_keys(self, steps, seed=99):
        """Same error polynomials and uniform seed on both sides.  Returns (oracle dict by step, library key set)."""
        steps = list(steps)
        beta = self.pr.beta(self.pr.L)
        e = wl.error_poly(self.rng, (len(steps), beta, self.N))
        o_gks = {st: self.o.galois_keygen(self.o_sk, st, e[i], seed) for i, st in enumerate(steps)}
        g_gk = self.ctx.galois_keygen(self.g_sk, steps, e, seed) if steps else None
        return o_gks, g_gk

    def encrypt_both(self, slots, limbs):
        """slots: [n_ct][<=n] float.  Encodes with the ORACLE, imports the integer
        plaintext into the library, encrypts on both sides with the same randomness."""
        slots = np.atleast_2d(slots)
        n_ct = slots.shape[0]
        coeffs = np.stack([self.o.encode_coeffs(z) for z in slots])
        v = np.stack([wl.ternary_poly(self.rng, self.N) for _ in range(n_ct)])
        e0 = wl.error_poly(self.rng, (n_ct, self.N))
        e1 = wl.error_poly(self.rng, (n_ct, self.N))
        o_cts = [self.o.encrypt(self.o.i64_to_rns(coeffs[i], self.pr.q[:limbs]), self.o_pk, v[i], e0[i], e1[i]) for i in range(n_ct)]
        g_pt = self.ctx.pt_import(coeffs, limbs)
        g_ct = self.ctx.encrypt(self.g_pk, g_pt, v, e0, e1)
        g_pt.free()
        return o_cts, g_ct


def stack_cts(cts):
    return np.stack([c.limbs() for c in cts])


def to_oracle_cts(arr, scale):
    return [Ciphertext(np.ascontiguousarray(a[0]), np.ascontiguousarray(a[1]), scale) for a in arr]
