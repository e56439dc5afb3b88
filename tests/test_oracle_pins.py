"""Pins for the CPU oracle: each part is checked against something other than
itself -- the schoolbook product, Python big integers, closed forms, the
paper's printed toy example, float64 linear algebra."""
import math
import os

import numpy as np
import pytest

import workloads as wl
from oracle import Oracle, Params
from oracle.params import is_prime

HERE = os.path.dirname(os.path.abspath(__file__))


def crt(residues, moduli):
    M = 1
    for m in moduli:
        M *= m
    x = 0
    for r, m in zip(residues, moduli):
        Mi = M // m
        x += int(r) * Mi * pow(Mi, -1, m)
    return x % M, M


def small_params(wlcfg, log_n):
    """The workload's own primes (found for its full ring) run at a small ring."""
    full = Params(*wlcfg.param_tuple())
    return Params(log_n, 0, 0, 0, 0, wlcfg.alpha, wlcfg.log_scale, q=full.q, p=full.p)


@pytest.fixture(scope="module")
def all_small():
    return [small_params(w, 8) for w in wl.WORKLOADS]


# ------------------------------------------------------------------ primes
@pytest.mark.parametrize("w", wl.WORKLOADS, ids=lambda w: w.name)
def test_prime_chains(w):
    pr = Params(*w.param_tuple())
    assert len(pr.q) == w.q_count and len(pr.p) == w.p_count
    assert len(set(pr.q + pr.p)) == len(pr.q + pr.p)
    for m, bits in [(x, w.q_bits) for x in pr.q] + [(x, w.p_bits) for x in pr.p]:
        assert m.bit_length() == bits
        assert m % (2 * pr.N) == 1
        # Fermat + trial division, independent of the Miller-Rabin used to find them
        assert pow(2, m - 1, m) == 1 and pow(3, m - 1, m) == 1
        assert all(m % f for f in range(3, 2000, 2))
        assert pow(pr.psi[m], pr.N, m) == m - 1
    assert pr.q == sorted(pr.q, reverse=True)


def test_prime_chains_are_the_largest_primes_in_descending_order():
    """The chains must hold the LARGEST primes = 1 mod 2N below 2^bits, none skipped: every candidate from the top
    down to the last chain member is tested with an independent primality routine (sympy), and the primes among
    them must be the chain, in that order (a search that passed over a prime would fail here; the P chain has its
    own bit size in every workload, so it skips nothing)."""
    sympy = pytest.importorskip("sympy")
    seen = set()
    for w in wl.WORKLOADS:
        if w.param_tuple()[:5] in seen:
            continue
        seen.add(w.param_tuple()[:5])
        pr = Params(*w.param_tuple())
        two_n = 2 * pr.N
        for chain, bits in ((pr.q, w.q_bits), (pr.p, w.p_bits)):
            x = ((1 << bits) - 1) // two_n * two_n + 1
            assert x < (1 << bits) and x + two_n >= (1 << bits)  # the largest candidate below 2^bits
            found = []
            while x >= chain[-1]:
                if sympy.isprime(x):
                    found.append(x)
                x -= two_n
            assert found == chain, (w.name, bits)
        assert not set(pr.q) & set(pr.p)


def test_is_prime_small_table():
    known = [2, 3, 5, 7, 11, 13, 97, 65537, 2147483647, (1 << 61) - 1]
    comp = [1, 4, 561, 6601, 2147483649, (1 << 61) + 1, 3215031751]
    assert all(is_prime(x) for x in known) and not any(is_prime(x) for x in comp)


# --------------------------------------------------------------------- NTT
def test_ntt_is_the_defining_sum():
    pr = Params(4, 30, 2, 31, 1, 1, 20)
    o = Oracle(pr)
    rng = np.random.default_rng(0)
    for q in pr.q + pr.p:
        a = rng.integers(0, q, size=o.N, dtype=np.uint64)
        got = o.ntt(a[None, :], [q])[0]
        psi = pr.psi[q]
        for k in range(o.N):
            want = sum(int(a[i]) * pow(psi, (2 * k + 1) * i, q) for i in range(o.N)) % q
            assert int(got[k]) == want


def test_ntt_product_matches_schoolbook_on_every_prime(all_small):
    rng = np.random.default_rng(1)
    for pr in all_small:
        o = Oracle(pr)
        for q in pr.q + pr.p:
            a = rng.integers(0, q, size=o.N, dtype=np.uint64)
            b = rng.integers(0, q, size=o.N, dtype=np.uint64)
            got = o.polymul(a[None, :], b[None, :], [q])[0]
            assert np.array_equal(got, o.polymul_naive(a, b, q))


def test_schoolbook_against_python_ints():
    q, n = 1000003 * 0 + 998244353, 16
    pr = Params(4, 0, 0, 0, 0, 1, 20, q=[q], p=[])
    o = Oracle(pr)
    rng = np.random.default_rng(2)
    a = rng.integers(0, q, size=n, dtype=np.uint64)
    b = rng.integers(0, q, size=n, dtype=np.uint64)
    want = [0] * n
    for i in range(n):
        for j in range(n):
            k = i + j
            if k < n:
                want[k] += int(a[i]) * int(b[j])
            else:
                want[k - n] -= int(a[i]) * int(b[j])
    assert [int(x) for x in o.polymul_naive(a, b, q)] == [w % q for w in want]


def test_ntt_roundtrip_and_x_power(all_small):
    rng = np.random.default_rng(3)
    pr = all_small[3]
    o = Oracle(pr)
    primes = pr.q + pr.p
    a = np.stack([rng.integers(0, q, size=o.N, dtype=np.uint64) for q in primes])
    assert np.array_equal(o.ntt(o.ntt(a, primes), primes, inverse=True), a)
    # X^(N-1) * X = -1
    x1 = np.zeros((len(primes), o.N), dtype=np.uint64)
    xn = np.zeros_like(x1)
    x1[:, 1] = 1
    xn[:, o.N - 1] = 1
    prod = o.polymul(x1, xn, primes)
    want = np.zeros_like(x1)
    want[:, 0] = np.array([q - 1 for q in primes], dtype=np.uint64)
    assert np.array_equal(prod, want)


# ---------------------------------------------------------------- encoding
def test_encode_fft_matches_direct_sum_and_roundtrip():
    pr = Params(10, 36, 3, 37, 1, 1, 30)
    o = Oracle(pr)
    rng = np.random.default_rng(4)
    z = rng.uniform(-1, 1, o.n)
    m = o.encode_coeffs(z)
    assert np.abs(m - o.encode_coeffs_direct(z)).max() <= 1
    back = o.decode_coeffs(m.astype(np.float64))
    assert np.abs(back.real - z).max() < 2.0 ** -20
    assert np.abs(back.imag).max() < 2.0 ** -20


def test_encode_is_ring_homomorphism_and_rotation_direction():
    pr = Params(8, 50, 2, 60, 1, 1, 24)
    o = Oracle(pr)
    rng = np.random.default_rng(5)
    z1, z2 = rng.uniform(-1, 1, o.n), rng.uniform(-1, 1, o.n)
    q = pr.q
    m1, m2 = o.i64_to_rns(o.encode_coeffs(z1), q), o.i64_to_rns(o.encode_coeffs(z2), q)
    prod = o.polymul(m1, m2, q)
    ct = type("C", (), {})()
    from oracle.ckks import Ciphertext
    c = Ciphertext(prod, np.zeros_like(prod), pr.scale ** 2)
    coeffs = o.decrypt_coeffs(c, np.zeros(o.N, dtype=np.int8))
    got = o.decode_coeffs(coeffs, pr.scale ** 2).real
    assert np.abs(got - z1 * z2).max() < 1e-4
    # Rot(c;k)[i] = c[i+k]  (paper, Rotation): phi_{5^k} of the encoding decodes to the left shift
    for k in (1, 3, o.n - 1):
        g = pr.galois_element(k)
        rot = o.automorphism(m1, g, q)
        cr = Ciphertext(rot, np.zeros_like(rot), pr.scale)
        z = o.decode_coeffs(o.decrypt_coeffs(cr, np.zeros(o.N, dtype=np.int8))).real
        assert np.abs(z - np.roll(z1, -k)).max() < 1e-5
    assert pr.galois_element(-1) == pow(5, o.n - 1, 2 * o.N)


def test_crt_center_against_python_ints():
    pr = Params(4, 50, 2, 60, 1, 1, 20)
    o = Oracle(pr)
    from oracle.ckks import Ciphertext
    rng = np.random.default_rng(6)
    q0, q1 = pr.q
    vals = [int(v) for v in rng.integers(-(1 << 62), 1 << 62, size=o.N)]
    vals[0], vals[1], vals[2] = (q0 * q1) // 2, -((q0 * q1) // 2), 0
    c0 = np.array([[v % q0 for v in vals], [v % q1 for v in vals]], dtype=np.uint64)
    got = o.decrypt_coeffs(Ciphertext(c0, np.zeros_like(c0), 1.0), np.zeros(o.N, dtype=np.int8))
    assert np.array_equal(got, np.array([float(v) for v in vals]))


# ------------------------------------------------------ basis conversions
@pytest.mark.parametrize("widx", [0, 1, 3])
def test_modup_is_digit_plus_small_multiple_of_Qj(widx, all_small):
    pr = all_small[widx]
    o = Oracle(pr)
    rng = np.random.default_rng(7)
    for l1 in {pr.L, max(1, pr.L - 1)}:
        c1 = np.stack([rng.integers(0, q, size=o.N, dtype=np.uint64) for q in pr.q[:l1]])
        up = o.mod_up(c1)
        ext = pr.q[:l1] + pr.p
        assert up.shape == (pr.beta(l1), l1 + pr.K, o.N)
        for j in range(pr.beta(l1)):
            src = pr.digit_limbs(j, l1)
            qs = [pr.q[i] for i in src]
            for idx in range(0, o.N, 37):
                dval, Qj = crt([c1[i, idx] for i in src], qs)
                us = set()
                for t_i, t in enumerate(ext):
                    r = int(up[j, t_i, idx])
                    if t_i in src:
                        assert r == int(c1[t_i, idx])
                        continue
                    u = (r - dval) * pow(Qj, -1, t) % t
                    us.add(u)
                assert len(us) == 1 and 0 <= us.pop() < len(src)


@pytest.mark.parametrize("widx", [0, 1, 3])
def test_moddown_is_exact_division_up_to_small_symmetric_integer(widx, all_small):
    pr = all_small[widx]
    o = Oracle(pr)
    rng = np.random.default_rng(8)
    l1 = pr.L
    ext = pr.q[:l1] + pr.p
    u = np.stack([rng.integers(0, q, size=o.N, dtype=np.uint64) for q in ext])
    out = o.mod_down(u, l1)
    for idx in range(0, o.N, 29):
        full, _ = crt([u[i, idx] for i in range(len(ext))], ext)
        up, P = crt([u[l1 + k, idx] for k in range(pr.K)], pr.p)
        up = up - P if up > P // 2 else up  # centred representative of [u]_P
        exact = (full - up) // P
        assert (full - up) % P == 0
        # out = (u - [u]_P)/P - v ([u]_P centred) with one small integer v per coefficient, |v| <= K/2
        vs = {(exact - int(out[i, idx]) + pr.K) % pr.q[i] - pr.K for i in range(l1)}
        assert len(vs) == 1 and abs(vs.pop()) <= pr.K / 2


def test_rescale_is_exact_division(all_small):
    pr = all_small[4]
    o = Oracle(pr)
    from oracle.ckks import Ciphertext
    rng = np.random.default_rng(9)
    l1 = pr.L
    q = pr.q[:l1]
    c0 = np.stack([rng.integers(0, m, size=o.N, dtype=np.uint64) for m in q])
    c1 = np.stack([rng.integers(0, m, size=o.N, dtype=np.uint64) for m in q])
    kappa = -(2.0 ** -5)
    out = o.mul_scalar_rescale(Ciphertext(c0, c1, pr.scale), kappa)
    ql = q[-1]
    k = -int(math.floor(abs(kappa) * ql + 0.5))
    assert out.l1 == l1 - 1 and out.scale == pr.scale * k / (kappa * ql)
    for idx in range(0, o.N, 41):
        for src, dst in ((c0, out.c0), (c1, out.c1)):
            val, Q = crt([src[i, idx] for i in range(l1)], q)
            val = val * k % Q
            top = val % ql
            top = top - ql if top > ql // 2 else top  # centred: division with rounding to nearest
            exact = (val - top) // ql
            assert (val - top) % ql == 0 and abs(exact * ql - val) <= ql // 2
            assert [int(dst[i, idx]) for i in range(l1 - 1)] == [exact % m for m in q[:-1]]


# --------------------------------------------------------- whole key switch
def _keys(o, rng, seed=11):
    sk, pk = o.keygen(wl.ternary_poly(rng, o.N), wl.error_poly(rng, o.N), seed)
    return sk, pk


def _enc(o, rng, pk, z, l1):
    return o.encrypt(o.encode(z, l1), pk, wl.ternary_poly(rng, o.N), wl.error_poly(rng, o.N), wl.error_poly(rng, o.N))


def test_pure_rescale_is_exact_division(all_small):
    """Rescale without a constant: the centred integer coefficient divided by q_l, rounded to nearest."""
    pr = all_small[1]
    o = Oracle(pr)
    from oracle.ckks import Ciphertext
    rng = np.random.default_rng(19)
    l1 = pr.L - 1
    q = pr.q[:l1]
    c0 = np.stack([rng.integers(0, m, size=o.N, dtype=np.uint64) for m in q])
    c1 = np.stack([rng.integers(0, m, size=o.N, dtype=np.uint64) for m in q])
    c0[-1, :4] = [0, q[-1] // 2, q[-1] // 2 + 1, q[-1] - 1]  # both sides of the centring threshold
    out = o.rescale(Ciphertext(c0, c1, 3.0 * q[-1]))
    ql = q[-1]
    assert out.l1 == l1 - 1 and out.scale == 3.0
    for idx in list(range(4)) + list(range(4, o.N, 37)):
        for src, dst in ((c0, out.c0), (c1, out.c1)):
            val, Q = crt([src[i, idx] for i in range(l1)], q)
            val = val - Q if val > Q // 2 else val
            exact = (2 * val + ql) // (2 * ql)  # round to nearest (q_l odd: no ties)
            assert abs(exact * ql - val) <= ql // 2
            assert [int(dst[i, idx]) for i in range(l1 - 1)] == [exact % m for m in q[:-1]]


def test_pmult_against_schoolbook_and_slotwise_product():
    w = wl.WORKLOADS[1]
    pr = small_params(w, 6)
    o = Oracle(pr)
    rng = np.random.default_rng(23)
    sk, pk = _keys(o, rng)
    l1 = 4
    q = pr.q[:l1]
    ql = float(q[-1])
    z = rng.uniform(-1, 1, o.n)
    wv = rng.uniform(-2, 2, o.n)
    ct = _enc(o, rng, pk, z, l1)
    m = o.encode_coeffs(wv, ql)
    # the encoding at another scale decodes back at that scale
    assert np.abs(o.decode_coeffs(m.astype(np.float64), ql).real - wv).max() < 1e-9
    pt = o.i64_to_rns(m, q)
    prod = o.pmult(ct, pt, ql)
    assert prod.scale == ct.scale * ql and prod.l1 == l1
    # each component is the negacyclic product with the integer polynomial m (schoolbook, per prime)
    for comp_in, comp_out in ((ct.c0, prod.c0), (ct.c1, prod.c1)):
        for i, m_i in enumerate(q):
            assert np.array_equal(comp_out[i], o.polymul_naive(comp_in[i], pt[i], m_i))
    # and the slots multiply; the rescale brings the scale back and drops one limb
    out = o.pmult_sum_rescale([(ct, pt)], ql)
    assert out.l1 == l1 - 1 and abs(out.scale / ct.scale - 1) < 1e-12
    assert np.abs(o.decrypt(out, sk) - z * wv).max() < 1e-3
    # a sum of two products is rescaled once
    z2 = rng.uniform(-1, 1, o.n)
    w2 = rng.uniform(-2, 2, o.n)
    ct2 = _enc(o, rng, pk, z2, l1)
    pt2 = o.i64_to_rns(o.encode_coeffs(w2, ql), q)
    out2 = o.pmult_sum_rescale([(ct, pt), (ct2, pt2)], ql)
    assert np.abs(o.decrypt(out2, sk) - (z * wv + z2 * w2)).max() < 1e-3


def test_rope_against_the_rotary_formula():
    """Alg. 2 against the pairwise rotation of the positional-encoding equation written out on
    cleartext: (x_{2k}, x_{2k+1}) -> (x_{2k} cos - x_{2k+1} sin, x_{2k+1} cos + x_{2k} sin)."""
    w = wl.WORKLOADS[1]
    pr = small_params(w, 8)
    o = Oracle(pr)
    rng = np.random.default_rng(29)
    sk, pk = _keys(o, rng)
    l1 = pr.L
    x = rng.uniform(-1, 1, o.n)
    theta = rng.uniform(0, 2 * np.pi, o.n // 2)
    cos, sin = np.repeat(np.cos(theta), 2), np.repeat(np.sin(theta), 2)
    # slot-dependent values that are not pairwise equal would also be handled; make one pair unequal
    cos[0], cos[1], sin[0], sin[1] = 0.3, -0.7, 0.9, 0.2
    want = np.empty_like(x)
    want[0::2] = x[0::2] * cos[0::2] - x[1::2] * sin[0::2]
    want[1::2] = x[1::2] * cos[1::2] + x[0::2] * sin[1::2]
    ct = _enc(o, rng, pk, x, l1)
    beta = pr.beta(pr.L)
    gk_p = o.galois_keygen(sk, 1, wl.error_poly(rng, (beta, o.N)), 31)
    gk_m = o.galois_keygen(sk, -1, wl.error_poly(rng, (beta, o.N)), 31)
    pts = o.rope_plaintexts(cos, sin, l1)
    y = o.rope(ct, pts, gk_p, gk_m)
    assert y.l1 == l1 - 1 and abs(y.scale / ct.scale - 1) < 1e-12  # one level, scale kept
    assert np.abs(o.decrypt(y, sk) - want).max() < 1e-3
    neg, pos = Oracle.rope_masks(8)
    assert neg.tolist() == [-1, 0, -1, 0, -1, 0, -1, 0] and pos.tolist() == [0, 1, 0, 1, 0, 1, 0, 1]


def test_merge_packs_placed_outputs():
    w = wl.WORKLOADS[1]
    pr = small_params(w, 7)
    o = Oracle(pr)
    rng = np.random.default_rng(37)
    sk, pk = _keys(o, rng)
    l1 = 3
    s, c_tot = 8, 8  # n = 64 slots
    m = 19           # two full groups and a ragged one
    Y = rng.uniform(-1, 1, (m, s))
    cts = []
    for i in range(m):
        z = rng.uniform(-1, 1, o.n)  # other blocks hold unrelated values
        b = i % c_tot
        z[b * s:(b + 1) * s] = Y[i]
        cts.append(_enc(o, rng, pk, z, l1))
    masks = o.block_masks(s, c_tot, l1)
    packed = o.merge(cts, masks, c_tot)
    assert len(packed) == 3 and all(p.l1 == l1 - 1 for p in packed)
    for G, p in enumerate(packed):
        dec = o.decrypt(p, sk)
        for b in range(c_tot):
            i = G * c_tot + b
            want = Y[i] if i < m else np.zeros(s)
            assert np.abs(dec[b * s:(b + 1) * s] - want).max() < 1e-3


@pytest.mark.parametrize("widx,log_n", [(0, 10), (1, 10), (3, 10)])
def test_key_switch_noise_and_rotation(widx, log_n):
    w = wl.WORKLOADS[widx]
    pr = small_params(w, log_n)
    o = Oracle(pr)
    rng = np.random.default_rng(10 + widx)
    sk, pk = _keys(o, rng)
    z = rng.uniform(-1, 1, o.n)
    ct = _enc(o, rng, pk, z, pr.L)
    assert np.abs(o.decrypt(ct, sk) - z).max() < 1e-3
    for step in (1, 5, -1, o.n // 2):
        gk = o.galois_keygen(sk, step, wl.error_poly(rng, (pr.beta(pr.L), o.N)), 12)
        rot = o.rotate(ct, gk)
        assert rot.l1 == ct.l1 and rot.scale == ct.scale  # Rot consumes no level
        assert np.abs(o.decrypt(rot, sk) - np.roll(z, -step)).max() < 1e-3
        # (out0 + out1 s) - phi_g(c0 + c1 s) is a small polynomial
        q = pr.q[:2]
        s_rns = o.small_to_rns(sk, q)
        lhs = o.add(rot.c0[:2], o.polymul(np.ascontiguousarray(rot.c1[:2]), s_rns, q), q)
        inner = o.add(ct.c0[:2], o.polymul(np.ascontiguousarray(ct.c1[:2]), s_rns, q), q)
        diff = o.sub(lhs, o.automorphism(inner, gk["g"], q), q)
        from oracle.ckks import Ciphertext
        noise = o.decrypt_coeffs(Ciphertext(diff, np.zeros_like(diff), 1.0), np.zeros(o.N, dtype=np.int8))
        assert np.abs(noise).max() < pr.scale * 1e-3 / math.sqrt(o.N)


def test_sum_of_rotations_with_one_moddown():
    """Two rotations of one ciphertext switched together: the sum of the two slot shifts, and within a few
    units per coefficient of the two rotations done separately."""
    w = wl.WORKLOADS[1]
    pr = small_params(w, 9)
    o = Oracle(pr)
    rng = np.random.default_rng(21)
    sk, pk = _keys(o, rng)
    z = rng.uniform(-1, 1, o.n)
    ct = _enc(o, rng, pk, z, pr.L)
    beta = pr.beta(pr.L)
    gks = [o.galois_keygen(sk, st, wl.error_poly(rng, (beta, o.N)), 6) for st in (2, -5)]
    digits = o.mod_up(ct.c1)
    both = o.rotate_sum_from_digits(ct.c0, digits, gks, ct.scale)
    assert np.abs(o.decrypt(both, sk) - (np.roll(z, -2) + np.roll(z, 5))).max() < 1e-3
    one = o.rotate_sum_from_digits(ct.c0, digits, gks[:1], ct.scale)
    assert np.array_equal(one.limbs(), o.rotate(ct, gks[0]).limbs())
    sep = o.add_ct(o.rotate(ct, gks[0]), o.rotate(ct, gks[1]))
    q = np.array(pr.q[:pr.L], dtype=np.int64)[None, :, None]
    diff = (both.limbs().astype(np.int64) - sep.limbs().astype(np.int64)) % q
    diff = np.where(diff > q // 2, diff - q, diff)
    # the same up to the rounding of the division by P and the small multiples of P the fast basis conversion adds:
    # a small integer polynomial, identical on every limb
    assert 1 <= np.abs(diff).max() <= pr.K + 1
    assert all(np.array_equal(diff[:, 0], diff[:, i]) for i in range(1, pr.L))


def test_radix_four_fill_step_is_three_rotations_with_one_rounding():
    """The group of three of the rotate-and-add fill, t + Rot(t; r) + Rot(t; 2r) + Rot(t; 3r) with one ModDown for
    the three rotations: the same slots as the three rotations done and rounded separately, the difference a small
    integer polynomial that is identical on every limb; and the fill built from such steps against its plain
    definition sum_{e < 16} Rot(t; e) taken with fifteen separate rotations."""
    w = wl.WORKLOADS[1]
    pr = small_params(w, 9)
    o = Oracle(pr)
    rng = np.random.default_rng(23)
    sk, pk = _keys(o, rng)
    z = rng.uniform(-1, 1, o.n) / 16
    ct = _enc(o, rng, pk, z, pr.L)
    beta = pr.beta(pr.L)
    gks = {st: o.galois_keygen(sk, st, wl.error_poly(rng, (beta, o.N)), 6) for st in range(1, 16)}
    assert Oracle.fill_steps(1, 16) == [[1, 2, 3], [4, 8, 12]] and Oracle.fill_steps(1, 8) == [[1, 2, 3], [4]]
    assert Oracle.fill_steps(2, 16, -1) == [[-2, -4, -6], [-8]]
    r = 4
    group = [gks[r], gks[2 * r], gks[3 * r]]
    joint = o.rotate_sum_from_digits(ct.c0, o.mod_up(ct.c1), group, ct.scale)
    sep = o.add_ct(o.add_ct(o.rotate(ct, group[0]), o.rotate(ct, group[1])), o.rotate(ct, group[2]))
    want = np.roll(z, -r) + np.roll(z, -2 * r) + np.roll(z, -3 * r)
    assert np.abs(o.decrypt(joint, sk) - want).max() < 1e-3
    q = np.array(pr.q[:pr.L], dtype=np.int64)[None, :, None]
    diff = (joint.limbs().astype(np.int64) - sep.limbs().astype(np.int64)) % q
    diff = np.where(diff > q // 2, diff - q, diff)
    # one rounding of the division by P against three: each is at most (K + 1) / 2 in size
    assert 1 <= np.abs(diff).max() <= 2 * (pr.K + 1)
    assert all(np.array_equal(diff[:, 0], diff[:, i]) for i in range(1, pr.L))
    # the whole fill against the plain sum of all sixteen shifts
    filled = o.fill(ct, 1, 16, gks)
    plain = ct
    for e in range(1, 16):
        plain = o.add_ct(plain, o.rotate(ct, gks[e]))
    ref = sum(np.roll(z, -e) for e in range(16))
    assert np.abs(o.decrypt(filled, sk) - ref).max() < 1e-3 and np.abs(o.decrypt(plain, sk) - ref).max() < 1e-3
    assert np.abs(o.decrypt(filled, sk) - o.decrypt(plain, sk)).max() < 1e-4


def test_rotate_at_lower_level():
    w = wl.WORKLOADS[4]
    pr = small_params(w, 9)
    o = Oracle(pr)
    rng = np.random.default_rng(20)
    sk, pk = _keys(o, rng)
    z = rng.uniform(-1, 1, o.n)
    ct = _enc(o, rng, pk, z, pr.L - 3)  # 13 limbs: last digit is partial
    gk = o.galois_keygen(sk, 3, wl.error_poly(rng, (pr.beta(pr.L), o.N)), 5)
    rot = o.rotate(ct, gk)
    assert rot.l1 == pr.L - 3
    assert np.abs(o.decrypt(rot, sk) - np.roll(z, -3)).max() < 1e-3


# ------------------------------------------- ciphertext x ciphertext, CCMM
def test_relinearised_product_keeps_the_phase_and_multiplies_slots():
    w = wl.WORKLOADS[1]
    pr = small_params(w, 8)
    o = Oracle(pr)
    from oracle.ckks import Ciphertext
    rng = np.random.default_rng(61)
    sk, pk = _keys(o, rng)
    l1 = 5  # partial second digit (alpha = 3)
    za, zb, zc, zd = (rng.uniform(-1, 1, o.n) for _ in range(4))
    a, b, c, d = (_enc(o, rng, pk, z, l1) for z in (za, zb, zc, zd))
    rk = o.relin_keygen(sk, wl.error_poly(rng, (pr.beta(pr.L), o.N)), 17)
    # the evaluation key is a key-switching key for s^2: b_j + a_j s - P s^2 is small on the limbs of digit j
    ext = pr.q + pr.p
    s_ext = o.small_to_rns(sk, ext)
    s2 = o.polymul(s_ext, s_ext, ext)
    for j in range(pr.beta(pr.L)):
        lhs = o.add(rk["b"][j], o.polymul(rk["a"][j], s_ext, ext), ext)
        for i in range(len(ext)):
            want = (pr.P % ext[i]) if i in pr.digit_limbs(j, pr.L) else 0
            diff = (lhs[i].astype(object) - want * s2[i].astype(object)) % ext[i]
            diff = np.where(diff > ext[i] // 2, diff - ext[i], diff)
            assert np.abs(diff).max() <= 19, (j, i)
    # tensor product: decrypts under (1, s, s^2) to the product of the two phases (schoolbook check on limb 0)
    q = pr.q[:l1]
    dd = o.tensor_sum([(a, b)])
    s_q = o.small_to_rns(sk, q)
    pa = o.add(a.c0, o.polymul(a.c1, s_q, q), q)
    pb = o.add(b.c0, o.polymul(b.c1, s_q, q), q)
    s2q = o.polymul(s_q, s_q, q)
    phase = o.add(o.add(dd[0], o.polymul(dd[1], s_q, q), q), o.polymul(dd[2], s2q, q), q)
    assert np.array_equal(phase[0], o.polymul_naive(pa[0], pb[0], q[0]))
    # relinearisation changes the phase by a small polynomial only
    rl = o.relinearize(dd, rk, a.scale * b.scale)
    ph2 = o.add(rl.c0, o.polymul(rl.c1, s_q, q), q)
    diff = o.sub(ph2[:2], phase[:2], q[:2])
    noise = o.decrypt_coeffs(Ciphertext(diff, np.zeros_like(diff), 1.0), np.zeros(o.N, dtype=np.int8))
    assert np.abs(noise).max() < 2.0 ** 20  # against a product scale of 2^80
    # Mult: slots multiply, one level, scale Delta^2 / q_l; a sum of two products is rescaled once
    out = o.mult_sum_relin_rescale([(a, b)], rk)
    assert out.l1 == l1 - 1 and abs(out.scale / (pr.scale ** 2 / q[-1]) - 1) < 1e-12
    assert np.abs(o.decrypt(out, sk) - za * zb).max() < 1e-3
    out2 = o.mult_sum_relin_rescale([(a, b), (c, d)], rk)
    assert np.abs(o.decrypt(out2, sk) - (za * zb + zc * zd)).max() < 1e-3
    # dropping limbs keeps the message
    assert np.abs(o.decrypt(o.drop_limbs(a, 3), sk) - za).max() < 1e-3


def test_replicate_and_ccmm_against_numpy():
    """CCMM section: c_i = sum_j a_j (x) b_i^(j) equals the float64 product A B."""
    w = wl.WORKLOADS[1]
    pr = small_params(w, 5)  # 16 slots
    o = Oracle(pr)
    rng = np.random.default_rng(67)
    sk, pk = _keys(o, rng)
    l1 = 4
    s_tok, d, m = o.n, 3, 2
    A = rng.uniform(-1, 1, (s_tok, d))
    B = rng.uniform(-1, 1, (d, m))
    beta = pr.beta(pr.L)
    period = 4
    steps = {st for grp in Oracle.fill_steps(1, o.n) + Oracle.fill_steps(period, o.n) + Oracle.fill_steps(1, period) for st in grp}
    gks = {st: o.galois_keygen(sk, st, wl.error_poly(rng, (beta, o.N)), 71) for st in sorted(steps)}
    # the fill schedule: radix four while two doublings remain, the sum of all shifts in any case
    assert Oracle.fill_steps(1, 16) == [[1, 2, 3], [4, 8, 12]] and Oracle.fill_steps(2, 16, -1) == [[-2, -4, -6], [-8]]
    rk = o.relin_keygen(sk, wl.error_poly(rng, (beta, o.N)), 73)
    a_cts = [_enc(o, rng, pk, A[:, j], l1) for j in range(d)]
    b_cts = []
    for i in range(m):
        z = np.zeros(o.n)  # B[j, i] in slot j, zeros elsewhere
        z[:d] = B[:, i]
        b_cts.append(_enc(o, rng, pk, z, l1))
    # the fill is the sum of all shifts, whatever the radix of its steps
    zs = rng.uniform(-1, 1, o.n)
    filled = o.fill(_enc(o, rng, pk, zs, l1), 1, 8, gks)
    assert filled.l1 == l1 and np.abs(o.decrypt(filled, sk) - sum(np.roll(zs, -e) for e in range(8))).max() < 1e-3
    # the general extraction: any slot of any ciphertext into every slot
    zf = rng.uniform(-1, 1, o.n)
    rep = o.replicate(_enc(o, rng, pk, zf, l1), o.one_hot_masks([5], l1)[0], gks)
    assert rep.l1 == l1 - 1 and np.abs(o.decrypt(rep, sk) - zf[5]).max() < 1e-3
    # the two-stage extraction of the matrix product: giant steps make the column periodic, baby steps fill
    u = o.spread_periods(b_cts[0], period, gks)
    assert u.l1 == l1 and np.abs(o.decrypt(u, sk) - np.tile(np.concatenate([B[:, 0], [0.0]]), o.n // period)).max() < 1e-3
    one = o.extract_from_periodic(u, o.periodic_masks(period, d, l1)[1], period, gks)
    assert one.l1 == l1 - 1 and np.abs(o.decrypt(one, sk) - B[1, 0]).max() < 1e-3
    C = o.ccmm(a_cts, b_cts, d, period, rk, gks)
    assert len(C) == m and all(c.l1 == l1 - 2 for c in C)
    for i in range(m):
        assert np.abs(o.decrypt(C[i], sk) - (A @ B)[:, i]).max() < 1e-3


def test_blockwise_extraction_and_ccmm_over_heads():
    """Several heads per ciphertext: Q_h K_h^T for every head at once against numpy."""
    w = wl.WORKLOADS[1]
    pr = small_params(w, 6)  # 32 slots: 4 heads of 8 tokens
    o = Oracle(pr)
    rng = np.random.default_rng(79)
    sk, pk = _keys(o, rng)
    l1, s, heads, d = 4, 8, 4, 3
    Q = rng.uniform(-1, 1, (heads, s, d))
    K = rng.uniform(-1, 1, (heads, s, d))
    a_cts = [_enc(o, rng, pk, np.concatenate([Q[h][:, j] for h in range(heads)]), l1) for j in range(d)]
    b_cts = [_enc(o, rng, pk, np.concatenate([K[h][:, j] for h in range(heads)]), l1) for j in range(d)]
    beta = pr.beta(pr.L)
    cols = [0, 3, 7]
    steps = [c for c in cols if c] + [st for grp in Oracle.fill_steps(1, s, -1) for st in grp]
    gks = {st: o.galois_keygen(sk, st, wl.error_poly(rng, (beta, o.N)), 83) for st in steps}
    rk = o.relin_keygen(sk, wl.error_poly(rng, (beta, o.N)), 89)
    mask0 = o.block_start_mask(s, l1)
    rep = o.extract_blockwise(b_cts[1], 3, s, mask0, gks)
    want = np.concatenate([np.full(s, K[h][3, 1]) for h in range(heads)])
    assert rep.l1 == l1 - 1 and np.abs(o.decrypt(rep, sk) - want).max() < 1e-3
    C = o.ccmm_blocks(a_cts, b_cts, s, cols, rk, gks)
    assert len(C) == len(cols) and all(c.l1 == l1 - 2 for c in C)
    for c, i in zip(C, cols):
        ref = np.concatenate([(Q[h] @ K[h].T)[:, i] for h in range(heads)])
        assert np.abs(o.decrypt(c, sk) - ref).max() < 1e-3, i


def test_giant_and_baby_step_extraction_over_heads():
    """Block-wise extraction in giant and baby steps: the spread segment, one extracted element, and both
    attention products (Q K^T and weights times V) for every head at once against numpy."""
    w = wl.WORKLOADS[1]
    pr = small_params(w, 6)  # 32 slots: 2 heads of 16 tokens
    o = Oracle(pr)
    rng = np.random.default_rng(97)
    sk, pk = _keys(o, rng)
    l1, s, heads, d, period = 5, 16, 2, 3, 4
    Q = rng.uniform(-1, 1, (heads, s, d))
    K = rng.uniform(-1, 1, (heads, s, d))
    a_cts = [_enc(o, rng, pk, np.concatenate([Q[h][:, j] for h in range(heads)]), l1) for j in range(d)]
    b_cts = [_enc(o, rng, pk, np.concatenate([K[h][:, j] for h in range(heads)]), l1) for j in range(d)]
    beta = pr.beta(pr.L)
    cols = [0, 6, 15]
    steps = set(range(1, period)) | {g * period for g in range(1, s // period)}
    steps |= {st for grp in Oracle.fill_steps(period, s, -1) + Oracle.fill_steps(1, period, -1) for st in grp}
    gks = {st: o.galois_keygen(sk, st, wl.error_poly(rng, (beta, o.N)), 101) for st in sorted(steps)}
    rk = o.relin_keygen(sk, wl.error_poly(rng, (beta, o.N)), 103)
    # the head mask: ones in the first `period` slots of every block
    mh = o.block_head_mask(s, period, l1)
    z = o.decode_coeffs(mh.astype(np.float64), float(pr.q[l1 - 1]))
    assert np.abs(z - np.tile(np.concatenate([np.ones(period), np.zeros(s - period)]), heads)).max() < 1e-9
    # giant step: segment 1 of every block, repeated through the block
    seg = o.spread_segment(b_cts[2], 1, s, period, mh, gks)
    want = np.concatenate([np.tile(K[h][period:2 * period, 2], s // period) for h in range(heads)])
    assert seg.l1 == l1 - 1 and np.abs(o.decrypt(seg, sk) - want).max() < 1e-3
    # baby step: element 2 of that segment, i.e. slot 6 of every block, in all slots of its block
    one = o.extract_from_segment(seg, 2, period, o.periodic_masks(period, 1, l1 - 1)[0], gks)
    want = np.concatenate([np.full(s, K[h][6, 2]) for h in range(heads)])
    assert one.l1 == l1 - 2 and np.abs(o.decrypt(one, sk) - want).max() < 1e-3
    # Q K^T, columns 0, 6 (giant and baby step both non-trivial) and 15 (last slot of a block)
    C = o.ccmm_bsgs(a_cts, b_cts, s, period, [[(j, j, i) for j in range(d)] for i in cols], rk, gks)
    assert len(C) == len(cols) and all(c.l1 == l1 - 3 for c in C)
    for c, i in zip(C, cols):
        ref = np.concatenate([(Q[h] @ K[h].T)[:, i] for h in range(heads)])
        assert np.abs(o.decrypt(c, sk) - ref).max() < 1e-3, i
    # weights times V: a_j = column j of the s x s weights (j < s), v_i = column i of V; out_i = sum_j a_j (x) E(v_i, j)
    Wt = rng.uniform(-1, 1, (heads, s, s)) / 4
    V = rng.uniform(-1, 1, (heads, s, 2))
    w_cts = [_enc(o, rng, pk, np.concatenate([Wt[h][:, j] for h in range(heads)]), l1) for j in range(s)]
    v_cts = [_enc(o, rng, pk, np.concatenate([V[h][:, i] for h in range(heads)]), l1) for i in range(2)]
    O = o.ccmm_bsgs(w_cts, v_cts, s, period, [[(j, i, j) for j in range(s)] for i in range(2)], rk, gks)
    for i in range(2):
        ref = np.concatenate([(Wt[h] @ V[h])[:, i] for h in range(heads)])
        assert O[i].l1 == l1 - 3 and np.abs(o.decrypt(O[i], sk) - ref).max() < 1e-3, i


def test_segment_of_columns_from_diagonals():
    """The segment form of the block-wise CCMM: masks, the diagonal arrangement, and the columns against numpy."""
    w = wl.WORKLOADS[1]
    pr = small_params(w, 6)  # 32 slots: 2 heads of 16 tokens
    o = Oracle(pr)
    rng = np.random.default_rng(107)
    sk, pk = _keys(o, rng)
    l1, s, heads, d, period = 5, 16, 2, 3, 4
    Q = rng.uniform(-1, 1, (heads, s, d))
    K = rng.uniform(-1, 1, (heads, s, d))
    a_cts = [_enc(o, rng, pk, np.concatenate([Q[h][:, j] for h in range(heads)]), l1) for j in range(d)]
    b_cts = [_enc(o, rng, pk, np.concatenate([K[h][:, j] for h in range(heads)]), l1) for j in range(d)]
    beta = pr.beta(pr.L)
    steps = set(range(1, period)) | set(range(-period, 0)) | {period} | {g * period for g in range(1, s // period)}
    steps |= {st for grp in Oracle.fill_steps(period, s, -1) for st in grp}
    gks = {st: o.galois_keygen(sk, st, wl.error_poly(rng, (beta, o.N)), 109) for st in sorted(steps)}
    rk = o.relin_keygen(sk, wl.error_poly(rng, (beta, o.N)), 113)
    # the sorting masks partition the slots: for every e the masks of the terms of all columns cover each slot once
    masks = o.segment_masks(s, period, l1 - 2)
    dec = np.stack([o.decode_coeffs(m.astype(np.float64), float(pr.q[l1 - 3])) for m in masks])
    assert np.abs(dec - np.round(dec)).max() < 1e-9
    dec = np.round(dec)
    for r in range(period):
        assert np.array_equal(dec[r], dec[period + r] + dec[2 * period + r]) and dec[2 * period + r].sum() == heads
    assert np.array_equal(dec[:period].sum(axis=0), np.ones(o.n))
    S = np.stack([Q[h] @ K[h].T for h in range(heads)])  # [head][token][column]
    x = np.arange(s)
    for c in range(period):
        for e, primed, mi in Oracle.segment_mask_terms(period, c):
            sel = dec[mi][:s] > 0
            assert np.all((x[sel] + e) % period == c)               # the diagonal holds column c there
            assert np.all(x[sel] + e >= s if primed else x[sel] + e < s)  # and the rotation it was built with stays inside the block
    for g, baby in ((0, 4), (2, 2), (3, 1)):
        C = o.ccmm_segment(a_cts, b_cts, s, period, baby, g, rk, gks)
        assert len(C) == period and all(c.l1 == l1 - 3 for c in C)
        for c in range(period):
            ref = np.concatenate([S[h][:, g * period + c] for h in range(heads)])
            assert np.abs(o.decrypt(C[c], sk) - ref).max() < 1e-3, (g, c)


def test_weights_times_v_from_diagonalised_weights():
    """The weights-times-V form without single-element replication: the diagonalised weights, the schedule of baby
    and giant steps over the diagonals, and the product over segments against numpy."""
    w = wl.WORKLOADS[1]
    pr = small_params(w, 6)  # 32 slots: 2 heads of 16 tokens
    o = Oracle(pr)
    rng = np.random.default_rng(127)
    sk, pk = _keys(o, rng)
    l1, s, heads, period, m = 4, 16, 2, 4, 2
    Wt = rng.uniform(-1, 1, (heads, s, s)) / 4
    V = rng.uniform(-1, 1, (heads, s, m))
    a_cts = [_enc(o, rng, pk, np.concatenate([Wt[h][:, j] for h in range(heads)]), l1) for j in range(s)]
    v_cts = [_enc(o, rng, pk, np.concatenate([V[h][:, i] for h in range(heads)]), l1) for i in range(m)]
    beta = pr.beta(pr.L)
    steps = set(range(1, period)) | set(range(-period, 0)) | {period} | {g * period for g in range(1, s // period)}
    steps |= {st for grp in Oracle.fill_steps(period, s, -1) for st in grp}
    gks = {st: o.galois_keygen(sk, st, wl.error_poly(rng, (beta, o.N)), 131) for st in sorted(steps)}
    rk = o.relin_keygen(sk, wl.error_poly(rng, (beta, o.N)), 137)
    # every diagonal's rotation amount splits into a baby step below `baby` and a giant step that is a multiple of it
    assert Oracle.diagonal_schedule(4, 2) == [(0, 0), (1, 0), (0, 2), (1, 2), (1, -4), (0, -2), (1, -2)]
    assert Oracle.diagonal_schedule(4, 4) == [(0, 0), (1, 0), (2, 0), (3, 0), (1, -4), (2, -4), (3, -4)]
    # segment 2 of the weights, diagonalised: entry e holds column 2 period + (x + e) mod period in slot x, split at the
    # block's end, and is then shifted by its giant step
    g = 2
    x = np.arange(s)
    for baby in (2, 4):
        sched = Oracle.diagonal_schedule(period, baby)
        ad = o.diagonalise_weights(a_cts[g * period:(g + 1) * period], s, period, baby, gks)
        assert len(ad) == 2 * period - 1 and all(c.l1 == l1 - 1 for c in ad)
        for q, (e1, t) in enumerate(sched):
            e = q if q < period else q - period + 1
            keep = (x + e < s) if q < period else (x + e >= s)
            plain = np.concatenate([np.where(keep, Wt[h][x, g * period + (x + e) % period], 0.0) for h in range(heads)])
            assert np.abs(o.decrypt(ad[q], sk) - np.roll(plain, t)).max() < 1e-3, (baby, q)  # Rot(.; -t)[y] = plain[y - t]
    # the product over segments 1 and 2, then over all four, with both splits of the diagonals
    for g0, n_seg, baby in ((1, 2, 2), (0, 4, 4), (0, 4, 1)):
        ads = [o.diagonalise_weights(a_cts[(g0 + k) * period:(g0 + k + 1) * period], s, period, baby, gks) for k in range(n_seg)]
        O = o.ccmm_av(ads, v_cts, s, period, baby, g0, rk, gks)
        lo, hi = g0 * period, (g0 + n_seg) * period
        for i in range(m):
            ref = np.concatenate([Wt[h][:, lo:hi] @ V[h][lo:hi, i] for h in range(heads)])
            assert O[i].l1 == l1 - 2 and np.abs(o.decrypt(O[i], sk) - ref).max() < 1e-3, (g0, baby, i)


def _attention_inputs(seed):
    """Two heads of 16 tokens per ciphertext: Q, K (width 3), weights (16 x 16) and V (2 columns), encrypted
    column-wise at 5 limbs, with every Galois key the block-wise CCMM forms ask for at period 4."""
    w = wl.WORKLOADS[1]
    pr = small_params(w, 6)
    o = Oracle(pr)
    rng = np.random.default_rng(seed)
    sk, pk = _keys(o, rng)
    l1, s, heads, d, period, m = 5, 16, 2, 3, 4, 2
    Q = rng.uniform(-1, 1, (heads, s, d))
    K = rng.uniform(-1, 1, (heads, s, d))
    Wt = rng.uniform(-1, 1, (heads, s, s)) / 4
    V = rng.uniform(-1, 1, (heads, s, m))
    col = lambda M3, j: np.concatenate([M3[h][:, j] for h in range(heads)])  # noqa: E731
    cts = {"q": [_enc(o, rng, pk, col(Q, j), l1) for j in range(d)], "k": [_enc(o, rng, pk, col(K, j), l1) for j in range(d)],
           "w": [_enc(o, rng, pk, col(Wt, j), l1) for j in range(s)], "v": [_enc(o, rng, pk, col(V, i), l1) for i in range(m)]}
    beta = pr.beta(pr.L)
    steps = set(range(1, s)) | set(range(-period, 0))
    steps |= {st for grp in Oracle.fill_steps(1, s, -1) + Oracle.fill_steps(period, s, -1) for st in grp}
    gks = {st: o.galois_keygen(sk, st, wl.error_poly(rng, (beta, o.N)), 211) for st in sorted(steps)}
    rk = o.relin_keygen(sk, wl.error_poly(rng, (beta, o.N)), 223)
    return o, sk, cts, gks, rk, (Q, K, Wt, V), (l1, s, heads, d, period, m)


def test_segment_form_against_the_plain_definition_of_ccmm(monkeypatch):
    """The optimised Q K^T form (a segment of columns from its diagonals, baby and giant steps) anchored to the
    plain definition of the CCMM section, c_i = sum_j a_j (x) b_i^(j) with every element replicated on its own
    (extract_blockwise: rotate, one-slot mask, fill): same decrypted columns within 1e-3 on one seeded input, one
    level more (three against two).  The schedule of the segment form is this build's reading and was fixed
    together with the library's; this test is what ties it to the definition.  Two planted mistakes must fail it:
    a giant step taken with the wrong sign, and the diagonals of the block's last slots left out."""
    o, sk, cts, gks, rk, (Q, K, Wt, V), (l1, s, heads, d, period, m) = _attention_inputs(301)
    g = 2
    cols = list(range(g * period, (g + 1) * period))
    plain = o.ccmm_blocks(cts["q"], cts["k"], s, cols, rk, gks)
    assert all(c.l1 == l1 - 2 for c in plain)
    dec_plain = np.stack([o.decrypt(c, sk) for c in plain])
    ref = np.stack([np.concatenate([(Q[h] @ K[h].T)[:, i] for h in range(heads)]) for i in cols])
    assert np.abs(dec_plain - ref).max() < 1e-3

    def segment(baby):
        C = o.ccmm_segment(cts["q"], cts["k"], s, period, baby, g, rk, gks)
        assert len(C) == period and all(c.l1 == l1 - 3 for c in C)
        return np.stack([o.decrypt(c, sk) for c in C])

    for baby in (1, 2, 4):
        assert np.abs(segment(baby) - dec_plain).max() < 1e-3, baby
    good_schedule, good_terms = Oracle.diagonal_schedule, Oracle.segment_mask_terms
    monkeypatch.setattr(Oracle, "diagonal_schedule", staticmethod(lambda P, b: [(e1, -t) for e1, t in good_schedule(P, b)]))
    assert np.abs(segment(2) - dec_plain).max() > 1e-2  # mutation 1: giant steps with the wrong sign
    monkeypatch.setattr(Oracle, "diagonal_schedule", staticmethod(good_schedule))
    monkeypatch.setattr(Oracle, "segment_mask_terms", staticmethod(lambda P, c: [t for t in good_terms(P, c) if not t[1]]))
    assert np.abs(segment(2) - dec_plain).max() > 1e-2  # mutation 2: the last slots of a block never filled
    monkeypatch.setattr(Oracle, "segment_mask_terms", staticmethod(good_terms))
    assert np.abs(segment(2) - dec_plain).max() < 1e-3


def test_diagonalised_weights_form_against_the_plain_definition_of_ccmm(monkeypatch):
    """The optimised weights-times-V form anchored to the plain definition out_i = sum_j a_j (x) E(v_i, j), every
    element E(v_i, j) replicated on its own through its block: same decrypted columns within 1e-3, both two levels
    below the operands.  Planted mistakes that must fail: the diagonal arrangement shifted by one column, and the
    products of different giant steps added without their rotation."""
    o, sk, cts, gks, rk, (Q, K, Wt, V), (l1, s, heads, d, period, m) = _attention_inputs(307)
    mask0 = o.block_start_mask(s, l1)
    g0, n_seg = 1, 2
    toks = range(g0 * period, (g0 + n_seg) * period)
    plain = []
    for i in range(m):
        reps = [o.extract_blockwise(cts["v"][i], j, s, mask0, gks) for j in toks]
        plain.append(o.mult_sum_relin_rescale([(o.drop_limbs(cts["w"][j], l1 - 1), r) for j, r in zip(toks, reps)], rk))
    assert all(c.l1 == l1 - 2 for c in plain)
    dec_plain = np.stack([o.decrypt(c, sk) for c in plain])
    lo, hi = g0 * period, (g0 + n_seg) * period
    ref = np.stack([np.concatenate([Wt[h][:, lo:hi] @ V[h][lo:hi, i] for h in range(heads)]) for i in range(m)])
    assert np.abs(dec_plain - ref).max() < 1e-3

    def av(baby, shift=0):
        ads = [o.diagonalise_weights(cts["w"][(g0 + k) * period + shift:(g0 + k + 1) * period + shift], s, period, baby, gks)
               for k in range(n_seg)]
        O = o.ccmm_av(ads, cts["v"], s, period, baby, g0, rk, gks)
        assert len(O) == m and all(c.l1 == l1 - 2 for c in O)
        return np.stack([o.decrypt(c, sk) for c in O])

    for baby in (1, 2, 4):
        assert np.abs(av(baby) - dec_plain).max() < 1e-3, baby
    assert np.abs(av(2, shift=1) - dec_plain).max() > 1e-2  # mutation 1: weights columns off by one against V's rows
    good_rotate = Oracle.rotate
    calls = {"n": 0}

    def rotate_skipping_sums(self, ct, gk):
        # mutation 2: ccmm_av's rotations of the relinearised sums (the ones at the product's scale) are skipped
        if ct.scale > 2.0 ** 70:
            calls["n"] += 1
            return ct
        return good_rotate(self, ct, gk)
    ads = [o.diagonalise_weights(cts["w"][(g0 + k) * period:(g0 + k + 1) * period], s, period, 2, gks) for k in range(n_seg)]
    monkeypatch.setattr(Oracle, "rotate", rotate_skipping_sums)
    bad = np.stack([o.decrypt(c, sk) for c in o.ccmm_av(ads, cts["v"], s, period, 2, g0, rk, gks)])
    monkeypatch.setattr(Oracle, "rotate", good_rotate)
    assert calls["n"] > 0 and np.abs(bad - dec_plain).max() > 1e-2


# -------------------------------------------------------------------- PCMM
def _read_toy():
    W, Y = [], {}
    for line in open(os.path.join(HERE, "golden", "pcmm_toy.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "W":
            W.append([int(x) for x in t[1:]])
        else:
            Y[int(t[1])] = [(int(x[1:]), 1 if x[0] == "+" else -1) for x in t[2:]]
    return np.array(W, dtype=np.int8), Y


def test_pcmm_toy_example_from_paper():
    W, Y = _read_toy()
    pr = Params(4, 36, 3, 37, 1, 1, 30)
    o = Oracle(pr)
    rng = np.random.default_rng(21)
    sk, pk = _keys(o, rng)
    s, d = 4, 4  # the example's s=d=4; ring with 8 slots, one column per ciphertext pair below
    X = rng.uniform(-1, 1, (o.n, d))  # c_tot = 1: every ciphertext is one column (the paper's own packing)
    cts = [_enc(o, rng, pk, X[:, j], pr.L) for j in range(d)]
    out = o.ternary_matmul(cts, o.n, d, W, "zero", {})  # no Galois key needed
    assert len(out) == 2
    for i, terms in Y.items():
        for poly in ("c0", "c1"):
            for l, q in enumerate(pr.q):
                want = [0] * o.N
                for j, sg in terms:
                    for k in range(o.N):
                        want[k] += sg * int(getattr(cts[j], poly)[l, k])
                assert [int(v) for v in getattr(out[i], poly)[l]] == [v % q for v in want]
        assert out[i].l1 == pr.L and out[i].scale == pr.scale  # level and scale unchanged
    got = np.stack([o.decrypt(c, sk) for c in out], axis=1)
    assert np.abs(got - X @ W.astype(np.float64)).max() < 1e-3


def test_pcmm_identity_and_zero_column():
    pr = Params(6, 36, 3, 37, 1, 1, 30)
    o = Oracle(pr)
    rng = np.random.default_rng(22)
    sk, pk = _keys(o, rng)
    d = 3
    cts = [_enc(o, rng, pk, rng.uniform(-1, 1, o.n), pr.L) for _ in range(d)]
    W = np.eye(d, 4, dtype=np.int8)  # last output column is all zero
    out = o.ternary_matmul(cts, o.n, d, W, "zero", {})
    for j in range(d):
        assert np.array_equal(out[j].c0, cts[j].c0) and np.array_equal(out[j].c1, cts[j].c1)
    assert not out[3].c0.any() and not out[3].c1.any()  # transparent zero ciphertext


@pytest.mark.parametrize("placement", ["diagonal", "zero"])
def test_pcmm_tiny_workload_end_to_end(placement, tiny_oracle):
    w = wl.WORKLOADS[0]
    o = tiny_oracle
    pr = o.pr
    rng = wl.rng_for(w.index)
    W = wl.ternary_weights(rng, w.d_in, w.d_out)
    X = wl.activations(rng, w.tokens, w.d_in, w.act)
    sk, pk = _keys(o, rng)
    packed = wl.pack_columns(X, o.n)
    assert packed.shape[0] == 1
    cts = [_enc(o, rng, pk, packed[0], pr.L)]
    c_tot = w.c_tot
    plan = o.plan(W, c_tot, placement)
    rhos = sorted({rho for t in plan for (_, rho, _) in t if rho})
    assert len(rhos) <= c_tot - 1
    gks = {rho: o.galois_keygen(sk, rho * w.tokens, wl.error_poly(rng, (pr.beta(pr.L), o.N)), 33) for rho in rhos}
    out = o.ternary_matmul(cts, w.tokens, w.d_in, W, placement, gks)
    assert sum(len(t) for t in plan) == int(np.count_nonzero(W))  # one ciphertext add/sub per non-zero weight
    ref = X @ W.astype(np.float64)
    err = 0.0
    for i, c in enumerate(out):
        p_i = o.placement_block(i, c_tot, placement)
        z = o.decrypt(c, sk)[p_i * w.tokens:(p_i + 1) * w.tokens]
        err = max(err, np.abs(z - ref[:, i]).max())
        assert c.l1 == pr.L and c.scale == pr.scale
    # measured 3.6e-4 (diagonal) and 2.5e-4 (zero placement): with the centred ModDown no slot collects a
    # constant offset any more, so both placements meet the workload's bound
    assert err < 1e-3


def test_splitmix64_published_vectors():
    """The generator under the uniform sampler against its published outputs: the reference test vector for
    seed 1234567 (five decimal values, as printed with the reference implementation) and the first outputs for
    seed 0.  A wrong shift, multiplier, increment or a finaliser applied before the increment fails here."""
    import ctypes
    o = Oracle(Params(4, 50, 1, 60, 1, 1, 20))
    out = np.empty(5, dtype=np.uint64)
    o.lib.orc_splitmix64(out.ctypes.data_as(ctypes.c_void_p), 5, ctypes.c_uint64(1234567))
    assert [int(x) for x in out] == [6457827717110365317, 3203168211198807973, 9817491932198370423, 4593380528125082431,
                                     16408922859458223821]
    o.lib.orc_splitmix64(out.ctypes.data_as(ctypes.c_void_p), 5, ctypes.c_uint64(0))
    assert [int(x) for x in out] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F, 0xF88BB8A8724C81EC,
                                     0x1B39896A51A8749B]


def test_uniform_samples_are_pairs_of_generator_outputs_and_look_uniform():
    """Structure and distribution of the uniform ring elements.  (1) A sample is two consecutive outputs of the
    pinned generator read as one 128-bit number and reduced mod q, the generator started at the key of (seed,
    stream, prime index): regenerated here with the pinned routine and Python integers, for a modulus above 2^63
    (so that a reduction that dropped the high word, or took the words in the other order, shows).  The key
    derivation itself (three finalisers) is this build's own format and has no outside pin.  (2) Residues mod each
    prime of a chain: mean and a 64-bin chi-square against the uniform law; streams, prime indices and seeds that
    differ give unrelated sequences."""
    import ctypes
    M = (1 << 64) - 1
    pr = Params(10, 50, 2, 60, 2, 2, 20)
    o = Oracle(pr)

    def mix(z):
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9 & M
        z = (z ^ (z >> 27)) * 0x94D049BB133111EB & M
        return z ^ (z >> 31)

    big_q = (1 << 64) - 59
    n = 64
    got = [int(x) for x in o.uniform(99, 7, [3], [big_q])[0][:n]]
    key = mix((mix((mix(99) + 7) & M) + 3) & M)
    out = np.empty(2 * n, dtype=np.uint64)
    o.lib.orc_splitmix64(out.ctypes.data_as(ctypes.c_void_p), 2 * n, ctypes.c_uint64(key))
    assert got == [((int(out[2 * i]) << 64) | int(out[2 * i + 1])) % big_q for i in range(n)]
    N = o.N
    for pid, q in enumerate(pr.q + pr.p):
        x = np.concatenate([o.uniform(5, st, [pid], [q])[0] for st in range(16)]).astype(np.float64)  # 16384 samples
        assert x.max() < q
        assert abs(x.mean() / q - 0.5) < 4 * (1 / 12 ** 0.5) / len(x) ** 0.5  # 4 sigma of the mean of a uniform law
        counts = np.histogram(x, bins=64, range=(0, float(q)))[0]
        chi2 = ((counts - len(x) / 64) ** 2 / (len(x) / 64)).sum()
        assert chi2 < 63 + 5 * (2 * 63) ** 0.5, (pid, chi2)  # 5 sigma above the mean of chi-square with 63 degrees
    a = o.uniform(5, 1, [0], [pr.q[0]])[0]
    for other in (o.uniform(5, 2, [0], [pr.q[0]])[0], o.uniform(6, 1, [0], [pr.q[0]])[0], o.uniform(5, 1, [1], [pr.q[0]])[0]):
        assert np.count_nonzero(a == other) <= 1
        assert abs(np.corrcoef(a.astype(np.float64), other.astype(np.float64))[0, 1]) < 5 / N ** 0.5


def test_uniform_stream_follows_its_specification():
    """The sampler is this build's own format (no external pin): check the C
    routine against the written specification evaluated with Python integers."""
    M = (1 << 64) - 1

    def mix(z):
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9 & M
        z = (z ^ (z >> 27)) * 0x94D049BB133111EB & M
        return z ^ (z >> 31)

    # SplitMix64 (Steele, Lea, Flood 2014) first output for seed 0, as widely tabulated
    assert mix(0x9E3779B97F4A7C15) == 0xE220A8397B1DCDAF
    pr = Params(4, 50, 1, 60, 1, 1, 20)
    o = Oracle(pr)
    seed, stream, pid, q = 12345, (2 << 56) | (5 << 8) | 1, 3, pr.p[0]
    got = o.uniform(seed, stream, [pid], [q])[0]
    G = 0x9E3779B97F4A7C15
    key = mix((mix((mix(seed) + stream) & M) + pid) & M)
    want = [((mix((key + G * (2 * i + 1)) & M) << 64) | mix((key + G * (2 * i + 2)) & M)) % q for i in range(o.N)]
    assert [int(x) for x in got] == want


def test_streamed_columns_equal_the_whole_product(tiny_oracle):
    """The helper the full-size parity tests use (the oracle's Alg. 1 on sampled columns, streamed over blocks of
    rotation amounts, several products of one input at once) returns exactly the columns of Oracle.ternary_matmul."""
    from helpers import oracle_columns
    w = wl.WORKLOADS[0]
    o = tiny_oracle
    pr = o.pr
    rng = wl.rng_for(w.index, salt=3)
    W1 = wl.ternary_weights(rng, w.d_in, w.d_out)
    W2 = wl.ternary_weights(rng, w.d_in, 40)
    W2[:, 7] = 0
    X = wl.activations(rng, w.tokens, w.d_in, w.act)
    sk, pk = _keys(o, rng)
    cts = [_enc(o, rng, pk, wl.pack_columns(X, o.n)[0], pr.L)]
    s, c_tot = w.tokens, w.c_tot
    e = wl.error_poly(rng, (c_tot - 1, pr.beta(pr.L), o.N))
    gks = {rho: o.galois_keygen(sk, rho * s, e[rho - 1], 33) for rho in range(1, c_tot)}
    full1 = o.ternary_matmul(cts, s, w.d_in, W1, "diagonal", gks)
    full2 = o.ternary_matmul(cts, s, w.d_in, W2, "zero", gks)
    cols1, cols2 = [0, 5, 17, 63], [0, 7, 39]
    got1, got2 = oracle_columns(o, sk, cts, s, [(W1, "diagonal", cols1), (W2, "zero", cols2)], lambda st: e[st // s - 1], 33, block=5)
    for i in cols1:
        assert np.array_equal(got1[i].limbs(), full1[i].limbs()), i
    for i in cols2:
        assert np.array_equal(got2[i].limbs(), full2[i].limbs()), i
    assert not got2[7].limbs().any()
