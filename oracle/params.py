"""CKKS parameter derivation for the CPU oracle -- TEST INFRASTRUCTURE ONLY.

Everything here is exact Python big-integer arithmetic.  The paper fixes only
the ring R_Q = Z_Q[X]/(X^N'+1) with Q a product of distinct primes
(Preliminaries, RNS-CKKS); prime selection and the constants of the basis
conversions are this build's reading, restated in the function docstrings.
The GPU library derives the same quantities with its own 64-bit code; the two
meet only through bit-exact comparison of results.
"""

_MR_BASES = (2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37)  # deterministic below 3.3e24


def is_prime(x: int) -> bool:
    if x < 2:
        return False
    for b in _MR_BASES:
        if x % b == 0:
            return x == b
    d, r = x - 1, 0
    while d % 2 == 0:
        d //= 2
        r += 1
    for b in _MR_BASES:
        y = pow(b, d, x)
        if y in (1, x - 1):
            continue
        for _ in range(r - 1):
            y = y * y % x
            if y == x - 1:
                break
        else:
            return False
    return True


def ntt_primes(bits: int, count: int, two_n: int, skip=()):
    """Largest `count` primes below 2^bits that are 1 mod 2N, scanning downward;
    the first found is index 0.  Values in `skip` are passed over (used when the
    Q and P chains have the same bit size)."""
    x = ((1 << bits) - 1) // two_n * two_n + 1
    if x >= (1 << bits):
        x -= two_n
    out = []
    while len(out) < count:
        if x < two_n:
            raise ValueError("ran out of candidates")
        if x not in skip and is_prime(x):
            out.append(x)
        x -= two_n
    return out


def primitive_2n_root(q: int, two_n: int) -> int:
    """Some primitive 2N-th root of unity mod q (which one is internal to the
    oracle: all comparisons are made on coefficient-form residues)."""
    for g in range(2, 1000):
        psi = pow(g, (q - 1) // two_n, q)
        if pow(psi, two_n // 2, q) == q - 1:
            return psi
    raise ValueError("no root found")


class Params:
    """One CKKS parameter set.

    q[0..L]   : ciphertext primes, Q_l = q_0...q_l (paper: Q = prod q_i)
    p[0..K-1] : special primes of hybrid key switching, P = prod p_k
    alpha     : limbs per key-switching digit; digit j = limbs [j*alpha, (j+1)*alpha) cut at the level
    scale     : 2^log_scale (the encoding scale Delta)
    """

    def __init__(self, log_n, q_bits, q_count, p_bits, p_count, alpha, log_scale, q=None, p=None):
        self.log_n = log_n
        self.N = 1 << log_n
        self.n_slots = self.N // 2
        # explicit chains (q, p) let tests run a larger ring's primes at a small N
        self.q = list(q) if q is not None else ntt_primes(q_bits, q_count, 2 * self.N)
        self.p = list(p) if p is not None else ntt_primes(p_bits, p_count, 2 * self.N, skip=set(self.q))
        self.alpha = alpha
        self.log_scale = log_scale
        self.scale = float(1 << log_scale)
        self.psi = {m: primitive_2n_root(m, 2 * self.N) for m in self.q + self.p}
        self.P = 1
        for m in self.p:
            self.P *= m

    @property
    def L(self):
        return len(self.q)

    @property
    def K(self):
        return len(self.p)

    def beta(self, l1):
        return -(-l1 // self.alpha)

    def digit_limbs(self, j, l1):
        return list(range(j * self.alpha, min((j + 1) * self.alpha, l1)))

    def galois_element(self, step):
        """Rot(c;k) shifts slots left by k (paper, Rotation); under the embedding
        used by encode (slot j at root exponent 5^j) that is X -> X^(5^k)."""
        return pow(5, step % self.n_slots, 2 * self.N)

    def modup_constants(self, j, l1):
        """Digit j at level l1-1: source limbs, (Q_j/q_i)^{-1} mod q_i, targets,
        and (Q_j/q_i) mod t for every target t in (Q_l minus digit) + P."""
        src = self.digit_limbs(j, l1)
        qs = [self.q[i] for i in src]
        Qj = 1
        for m in qs:
            Qj *= m
        inv = [pow(Qj // m, -1, m) for m in qs]
        tgt_idx = [i for i in range(l1) if i not in src] + [l1 + k for k in range(self.K)]
        tgt = [self.q[i] for i in range(l1) if i not in src] + list(self.p)
        hat = [[(Qj // m) % t for m in qs] for t in tgt]
        return src, qs, inv, tgt_idx, tgt, hat

    def moddown_constants(self, l1):
        inv = [pow(self.P // m, -1, m) for m in self.p]
        tgt = self.q[:l1]
        hat = [[(self.P // m) % t for m in self.p] for t in tgt]
        p_inv = [pow(self.P, -1, t) for t in tgt]
        return inv, tgt, hat, p_inv
