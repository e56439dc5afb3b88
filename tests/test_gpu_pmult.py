"""GPU parity of the plaintext multiplication with one rescale, of the block merge built on it and of
the secure RoPE protocol (Alg. 2), through the C ABI.  Plaintext polynomials are encoded by the oracle
and imported as integers, so every output limb must equal the oracle's bit for bit; the library's own
plaintext encoders are checked through decryption."""
import numpy as np
import pytest

import workloads as wl
from helpers import Pair, stack_cts, to_oracle_cts
from oracle import Oracle

pytestmark = pytest.mark.gpu

SMALL4 = (10, 50, 6, 60, 4, 4, 40)
WIDE = (10, 55, 4, 60, 2, 2, 40)  # ciphertext primes above 2^50: integer rescale kernel
KEYSWITCH = wl.WORKLOADS[1].param_tuple()


@pytest.fixture(scope="module")
def full():
    p = Pair(KEYSWITCH)
    yield p
    p.close()


def random_cts(p, n_ct, l1, seed):
    """Uniform residues (parity is on RNS words; no key is involved)."""
    rng = np.random.default_rng(seed)
    q = p.pr.q[:l1]
    arr = np.stack([np.stack([np.stack([rng.integers(0, m, size=p.N, dtype=np.uint64) for m in q]) for _ in range(2)]) for _ in range(n_ct)])
    return arr, to_oracle_cts(arr, p.pr.scale), p.ctx.ct_import(arr, p.pr.scale)


def random_plaintexts(p, n_pt, l1, seed):
    """Integer polynomials of slot vectors in [-2, 2] encoded at scale q_l by the oracle; imported into the library."""
    rng = np.random.default_rng(seed)
    ql = float(p.pr.q[l1 - 1])
    coeffs = np.stack([p.o.encode_coeffs(rng.uniform(-2, 2, p.n), ql) for _ in range(n_pt)])
    g_pt = p.ctx.pt_set_scale(p.ctx.pt_import(coeffs, l1), ql)
    rns = [p.o.i64_to_rns(c, p.pr.q[:l1]) for c in coeffs]
    return rns, g_pt, ql


def check_terms(p, o_cts, g_ct, rns, g_pt, ql, begin, term_ct, term_pt, l1, what):
    out = p.ctx.pmult_sum_rescale(g_ct, g_pt, begin, term_ct, term_pt)
    got = out.export()
    assert out.limbs == l1 - 1 and abs(out.scale / p.pr.scale - 1) < 1e-12
    for o in range(len(begin) - 1):
        terms = [(o_cts[term_ct[t]], rns[term_pt[t]]) for t in range(begin[o], begin[o + 1])]
        want = p.o.pmult_sum_rescale(terms, ql).limbs() if terms else np.zeros((2, l1 - 1, p.N), dtype=np.uint64)
        assert np.array_equal(got[o], want), (what, o)
    out.free()


@pytest.mark.parametrize("params,l1", [(SMALL4, 6), (SMALL4, 3), (WIDE, 4)], ids=["six-limbs", "three-limbs", "wide-primes"])
def test_pmult_sum_rescale_small_ring(params, l1):
    """Generic kernels: ragged term lists, an output without terms, a ciphertext and a plaintext used twice."""
    p = Pair(params)
    _, o_cts, g_ct = random_cts(p, 5, l1, 41)
    rns, g_pt, ql = random_plaintexts(p, 3, l1, 42)
    begin = [0, 1, 1, 4, 6, 17]
    term_ct = [0, 1, 2, 3, 4, 4] + [i % 5 for i in range(11)]
    term_pt = [0, 1, 2, 0, 1, 2] + [i % 3 for i in range(11)]
    check_terms(p, o_cts, g_ct, rns, g_pt, ql, begin, term_ct, term_pt, l1, "generic")
    g_ct.free()
    g_pt.free()
    p.close()


def test_pmult_sum_rescale_full_ring_both_kernel_sets(full):
    """N = 2^16, primes below 2^50: the fused kernels (a 19-term output crosses two of the accumulator's
    reductions, one output has no term) and the generic kernels, each against the oracle."""
    p = full
    l1 = 3
    _, o_cts, g_ct = random_cts(p, 4, l1, 43)
    rns, g_pt, ql = random_plaintexts(p, 3, l1, 44)
    begin = [0, 19, 19, 20, 23]
    term_ct = [i % 4 for i in range(19)] + [3, 0, 1, 2]
    term_pt = [i % 3 for i in range(19)] + [2, 0, 1, 2]
    for mode, what in ((0, "fused"), (1, "generic")):
        p.ctx.set_pmult_mode(mode)
        check_terms(p, o_cts, g_ct, rns, g_pt, ql, begin, term_ct, term_pt, l1, what)
    p.ctx.set_pmult_mode(0)
    # operands and outputs whose limb stride is wider than their level (both went through a rescale)
    _, o4, g4 = random_cts(p, 2, 4, 48)
    p.ctx.mul_scalar_rescale(g4, 0.5)
    o3 = [p.o.mul_scalar_rescale(c, 0.5) for c in o4]
    dst = p.ctx.ct_alloc(2, 3)
    p.ctx.mul_scalar_rescale(dst, 0.5)  # contents are irrelevant: two limbs at a stride of three
    out = p.ctx.pmult_sum_rescale(g4, g_pt, [0, 1, 2], [0, 1], [1, 2], dst)
    want = [p.o.pmult_sum_rescale([(o3[i], rns[i + 1])], ql).limbs() for i in range(2)]
    assert out.limbs == 2 and np.array_equal(out.export(), np.stack(want))
    for h in (g4, dst, g_ct, g_pt):
        h.free()


def test_pmult_errors(full):
    p = full
    _, _, g_ct = random_cts(p, 2, 3, 45)
    _, g_pt, _ = random_plaintexts(p, 1, 3, 46)
    with pytest.raises(p.binding.EnsiError, match="code -1"):
        p.ctx.pmult_sum_rescale(g_ct, g_pt, [0, 1], [2], [0])  # ciphertext index outside the batch
    with pytest.raises(p.binding.EnsiError, match="code -1"):
        p.ctx.pmult_sum_rescale(g_ct, g_pt, [0, 1], [0], [1])  # plaintext index outside the batch
    bad = p.ctx.ct_alloc(1, 3)
    with pytest.raises(p.binding.EnsiError, match="code -3"):
        p.ctx.pmult_sum_rescale(g_ct, g_pt, [0, 1], [0], [0], bad)  # output not one level below
    low = p.ctx.ct_import(np.zeros((1, 2, 1, p.N), dtype=np.uint64), 1.0)
    with pytest.raises(p.binding.EnsiError, match="code -3"):
        p.ctx.pmult_sum_rescale(low, g_pt, [0, 1], [0], [0], bad)  # no limb left to drop
    # a call whose every output is empty: zero ciphertexts, nothing read
    none = p.ctx.pmult_sum_rescale(g_ct, g_pt, [0, 0, 0], [], [])
    assert none.n == 2 and none.limbs == 2 and not none.export().any()
    for h in (g_ct, g_pt, bad, low, none):
        h.free()


# ------------------------------------------------------------------ merge
def test_merge_small_ring_against_oracle_and_cleartext():
    p = Pair(SMALL4)
    l1, s, c_tot, m = 3, 64, 8, 19  # 512 slots, two full groups and a ragged one
    Y = p.rng.uniform(-1, 1, (m, s))
    z = p.rng.uniform(-1, 1, (m, p.n))
    for i in range(m):
        z[i, (i % c_tot) * s:(i % c_tot + 1) * s] = Y[i]
    o_cts, g_ct = p.encrypt_both(z, l1)
    masks = p.o.block_masks(s, c_tot, l1)
    ql = float(p.pr.q[l1 - 1])
    g_masks = p.ctx.pt_set_scale(p.ctx.pt_import(masks, l1), ql)
    out = p.ctx.merge(g_ct, g_masks, c_tot)
    want = p.o.merge(o_cts, masks, c_tot)
    assert out.n == 3 and out.limbs == l1 - 1
    assert np.array_equal(out.export(), stack_cts(want))
    # the library's own masks: the same packing after decryption
    lib_masks = p.ctx.block_masks(s, c_tot, l1)
    assert np.abs(p.ctx.pt_export(lib_masks) - masks).max() <= 64  # fp64 summation order at scale 2^50
    out2 = p.ctx.merge(g_ct, lib_masks, c_tot)
    dec = p.ctx.decrypt(p.g_sk, out2)
    for i in range(3 * c_tot):
        G, b = divmod(i, c_tot)
        want_blk = Y[i] if i < m else np.zeros(s)
        assert np.abs(dec[G, b * s:(b + 1) * s] - want_blk).max() < 1e-3, i
    for h in (g_ct, g_masks, lib_masks, out, out2):
        h.free()
    p.close()


def test_merge_full_ring(full):
    """Fused kernels; block structure of a packed projection (s = 4096 tokens, 8 blocks), 11 placed outputs."""
    p = full
    l1, s, c_tot, m = 3, 4096, 8, 11
    _, o_cts, g_ct = random_cts(p, m, l1, 47)
    masks = p.o.block_masks(s, c_tot, l1)
    g_masks = p.ctx.pt_set_scale(p.ctx.pt_import(masks, l1), float(p.pr.q[l1 - 1]))
    out = p.ctx.merge(g_ct, g_masks, c_tot)
    want = p.o.merge(o_cts, masks, c_tot)
    assert np.array_equal(out.export(), stack_cts(want))
    for h in (g_ct, g_masks, out):
        h.free()


# ------------------------------------------------------------------- RoPE
def rope_case(p, n_ct, l1, seed):
    rng = np.random.default_rng(seed)
    x = rng.uniform(-1, 1, (n_ct, p.n))
    theta = rng.uniform(0, 2 * np.pi, p.n // 2)
    cos, sin = np.repeat(np.cos(theta), 2), np.repeat(np.sin(theta), 2)
    want = np.empty_like(x)
    want[:, 0::2] = x[:, 0::2] * cos[0::2] - x[:, 1::2] * sin[0::2]
    want[:, 1::2] = x[:, 1::2] * cos[1::2] + x[:, 0::2] * sin[1::2]
    return x, cos, sin, want


@pytest.mark.parametrize("params,l1", [(SMALL4, 6), (SMALL4, 5), (WIDE, 4)], ids=["six-limbs", "partial-digit", "wide-primes"])
def test_rope_small_ring(params, l1):
    p = Pair(params)
    x, cos, sin, want = rope_case(p, 3, l1, 51)
    o_gks, g_gk = p.galois_keys([1, -1])
    o_cts, g_ct = p.encrypt_both(x, l1)
    pts = p.o.rope_plaintexts(cos, sin, l1)
    g_pt = p.ctx.pt_set_scale(p.ctx.pt_import(pts, l1), float(p.pr.q[l1 - 1]))
    out = p.ctx.rope(g_gk, g_ct, g_pt)
    ref = [p.o.rope(c, pts, o_gks[1], o_gks[-1]) for c in o_cts]
    assert out.limbs == l1 - 1 and abs(out.scale / ref[0].scale - 1) < 1e-12
    assert np.array_equal(out.export(), stack_cts(ref))
    assert np.abs(p.ctx.decrypt(p.g_sk, out) - want).max() < 1e-3
    # plaintexts encoded by the library
    lib_pt = p.ctx.rope_plaintexts(cos, sin, l1)
    out2 = p.ctx.rope(g_gk, g_ct, lib_pt)
    assert np.abs(p.ctx.decrypt(p.g_sk, out2) - want).max() < 1e-3
    for h in (g_ct, g_pt, lib_pt, out, out2, g_gk):
        h.free()
    p.close()


def test_rope_single_ciphertext_full_ring(full):
    """The smallest batch: one ciphertext, one group, at the top level of the parameter set."""
    p = full
    l1 = p.pr.L
    x, cos, sin, want = rope_case(p, 1, l1, 53)
    o_gks, g_gk = p.galois_keys([1, -1])
    o_cts, g_ct = p.encrypt_both(x, l1)
    pts = p.o.rope_plaintexts(cos, sin, l1)
    g_pt = p.ctx.pt_set_scale(p.ctx.pt_import(pts, l1), float(p.pr.q[l1 - 1]))
    out = p.ctx.rope(g_gk, g_ct, g_pt)
    assert np.array_equal(out.export()[0], p.o.rope(o_cts[0], pts, o_gks[1], o_gks[-1]).limbs())
    assert np.abs(p.ctx.decrypt(p.g_sk, out) - want).max() < 1e-3
    for h in (g_ct, g_pt, out, g_gk):
        h.free()


def test_rope_full_ring(full):
    """Fused key switch and fused multiplication at N = 2^16; 35 ciphertexts span two groups of the
    batched rotation, a sample of them is checked against the oracle, all of them after decryption."""
    p = full
    l1, n_ct = 3, 35
    x, cos, sin, want = rope_case(p, n_ct, l1, 52)
    o_gks, g_gk = p.galois_keys([1, -1])
    o_cts, g_ct = p.encrypt_both(x, l1)
    pts = p.o.rope_plaintexts(cos, sin, l1)
    g_pt = p.ctx.pt_set_scale(p.ctx.pt_import(pts, l1), float(p.pr.q[l1 - 1]))
    out = p.ctx.rope(g_gk, g_ct, g_pt)
    got = out.export()
    for i in (0, 1, 31, 32, 34):
        assert np.array_equal(got[i], p.o.rope(o_cts[i], pts, o_gks[1], o_gks[-1]).limbs()), i
    assert np.abs(p.ctx.decrypt(p.g_sk, out) - want).max() < 1e-3
    only_plus = p.ctx.galois_keygen(p.g_sk, [1], None, 5)
    with pytest.raises(p.binding.EnsiError, match="code -2"):
        p.ctx.rope(only_plus, g_ct, g_pt, out)
    for h in (g_ct, g_pt, out, g_gk, only_plus):
        h.free()
