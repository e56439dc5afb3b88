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


def note(msg):
    """Progress line of a long test: straight to the terminal (past pytest's capture) and, when the environment
    names a file in ENSI_PROGRESS_LOG, appended to it."""
    import os
    import sys
    import time
    line = "[%s] %s\n" % (time.strftime("%H:%M:%S"), msg)
    try:
        os.write(sys.__stderr__.fileno() if sys.__stderr__ is not None else 2, line.encode())
    except OSError:
        pass
    path = os.environ.get("ENSI_PROGRESS_LOG")
    if path:
        try:
            with open(path, "a") as f:
                f.write(line)
        except OSError:
            pass


def oracle_columns(o, o_sk, o_cts, s, jobs, error_of_step, seed_a, block=32, tell=None):
    """Alg. 1 on the oracle for sampled output columns only, at sizes where the whole product does not fit the
    host.  jobs: list of (W, placement, cols) -- several products of the same packed inputs, so that the rotations,
    the expensive part, are computed once for all of them.  The rotation amounts are worked through in blocks: for a
    block, the oracle generates the block's Galois keys, rotates every packed input that needs them (one ModUp per
    input, kept), adds the block's operands into each sampled column with the oracle's own signed accumulate, and
    discards them.  Modular sums do not depend on the grouping, so the result is word for word what
    Oracle.ternary_matmul returns for these columns.  error_of_step(step) -> int8[beta][N], the error polynomials
    of that step's key.  Returns one {column: Ciphertext} per job."""
    c_tot = o.n // s
    L, scale = o_cts[0].l1, o_cts[0].scale
    terms = []
    for W, placement, cols in jobs:
        W = np.asarray(W)
        t = {}
        for i in cols:
            p_i = o.placement_block(i, c_tot, placement)
            t[i] = [(int(j) // c_tot, (int(j) % c_tot - p_i) % c_tot, int(W[j, i])) for j in np.nonzero(W[:, i])[0]]
        terms.append(t)
    need = sorted({(G, rho) for t in terms for tl in t.values() for (G, rho, _) in tl})
    rhos = sorted({rho for _, rho in need})
    digits = {}
    acc = [{i: None for i in t} for t in terms]
    for b0 in range(0, len(rhos), block):
        virt = {}
        for rho in rhos[b0:b0 + block]:
            Gs = [G for (G, r) in need if r == rho]
            if rho == 0:
                for G in Gs:
                    virt[(G, 0)] = o_cts[G]
                continue
            gk = o.galois_keygen(o_sk, rho * s, error_of_step(rho * s), seed_a)
            for G in Gs:
                if G not in digits:
                    digits[G] = o.mod_up(o_cts[G].c1)
                virt[(G, rho)] = o.rotate_from_digits(o_cts[G].c0, digits[G], gk, scale)
            del gk
        for t, a in zip(terms, acc):
            for i, tl_all in t.items():
                tl = [(virt[(G, rho)], w) for (G, rho, w) in tl_all if (G, rho) in virt]
                if tl:
                    part = o.accumulate(tl, L, scale)
                    a[i] = part if a[i] is None else o.add_ct(a[i], part)
        if tell:
            tell("oracle: rotation amounts %d..%d of %d done (%d operands in this block)" % (b0 + 1, min(b0 + block, len(rhos)), len(rhos), len(virt)))
    for a in acc:
        for i in a:
            if a[i] is None:
                a[i] = o.accumulate([], L, scale)
    return acc
