"""Key material across the boundary (System model: the client generates the keys, the server holds only the
public and evaluation keys; Preliminaries, KeyGen).  Keys the library generates must equal the oracle's word for
word when both get the same randomness; keys the oracle generates must work when imported into a context that
never saw the secret key."""
import numpy as np
import pytest

import workloads as wl
from helpers import Pair, stack_cts

pytestmark = pytest.mark.gpu

TINY = wl.WORKLOADS[0].param_tuple()
SMALL3 = (10, 50, 5, 60, 3, 3, 40)
KEYSWITCH = wl.WORKLOADS[1].param_tuple()


def gk_words(gk):
    """Oracle key -> [beta][2][L+K][N]: per digit (b_j, a_j)."""
    return np.stack([np.stack([gk["b"][j], gk["a"][j]]) for j in range(gk["b"].shape[0])])


@pytest.mark.parametrize("params", [TINY, SMALL3, KEYSWITCH], ids=["tiny", "alpha3", "full-ring"])
def test_exported_keys_equal_the_oracles(params):
    p = Pair(params)
    try:
        assert np.array_equal(p.ctx.sk_export(p.g_sk), p.o_sk)
        assert np.array_equal(p.ctx.pk_export(p.g_pk), np.stack(p.o_pk))
        steps = [1, -1, 5]
        o_gks, g_gk = p.galois_keys(steps)
        for st in steps:
            assert np.array_equal(p.ctx.gk_export(g_gk, st), gk_words(o_gks[st])), "Galois key of step %d" % st
        assert sorted(p.ctx.gk_elements(g_gk)) == sorted(p.pr.galois_element(st) for st in steps)
        e = wl.error_poly(p.rng, (p.pr.beta(p.pr.L), p.N))
        o_rk = p.o.relin_keygen(p.o_sk, e, 17)
        g_rk = p.ctx.relin_keygen(p.g_sk, e, 17)
        assert np.array_equal(p.ctx.gk_export(g_rk, 0), gk_words(o_rk))
        with pytest.raises(p.binding.EnsiError):
            p.ctx.gk_export(g_gk, 7)  # no key for that step
        g_gk.free()
        g_rk.free()
    finally:
        p.close()


@pytest.mark.parametrize("params", [SMALL3, KEYSWITCH], ids=["alpha3", "full-ring"])
def test_server_context_with_imported_public_keys_only(params):
    """The oracle plays the client: it generates every key and encrypts; the library context imports the public key,
    Galois keys and the evaluation key (never the secret key) and computes; results equal the oracle's bit for bit."""
    from paper_2509_09424_amd import binding
    from oracle import Oracle, Params
    pr = Params(*params)
    o = Oracle(pr)
    rng = np.random.default_rng(41)
    sk, pk = o.keygen(wl.ternary_poly(rng, o.N), wl.error_poly(rng, o.N), 5)
    beta = pr.beta(pr.L)
    steps = [2, -3]
    o_gks = {st: o.galois_keygen(sk, st, wl.error_poly(rng, (beta, o.N)), 7) for st in steps}
    o_rk = o.relin_keygen(sk, wl.error_poly(rng, (beta, o.N)), 9)
    ctx = binding.Context(*params, seed=3)
    try:
        g_pk = ctx.pk_import(np.stack(pk))
        g_gk = None
        for st in steps:
            g_gk = ctx.gk_import(st, gk_words(o_gks[st]), g_gk)
        g_rk = ctx.gk_import(0, gk_words(o_rk))
        z = rng.uniform(-1, 1, (2, o.n))
        coeffs = np.stack([o.encode_coeffs(v) for v in z])
        v = np.stack([wl.ternary_poly(rng, o.N) for _ in range(2)])
        e0, e1 = wl.error_poly(rng, (2, o.N)), wl.error_poly(rng, (2, o.N))
        limbs = pr.L
        o_cts = [o.encrypt(o.i64_to_rns(coeffs[i], pr.q[:limbs]), pk, v[i], e0[i], e1[i]) for i in range(2)]
        g_pt = ctx.pt_import(coeffs, limbs)
        g_ct = ctx.encrypt(g_pk, g_pt, v, e0, e1)
        assert np.array_equal(g_ct.export(), stack_cts(o_cts))  # encryption under the imported public key
        out = ctx.rotate(g_gk, g_ct, steps)
        assert np.array_equal(out.export(), stack_cts([o.rotate(c, o_gks[st]) for c, st in zip(o_cts, steps)]))
        prod = ctx.mult_sum_relin_rescale(g_rk, g_ct, g_ct, [0, 1], [0], [1])
        assert np.array_equal(prod.export()[0], o.mult_sum_relin_rescale([(o_cts[0], o_cts[1])], o_rk).limbs())
        # round trip: what was imported comes back out unchanged, and a replaced key takes effect
        assert np.array_equal(ctx.gk_export(g_gk, 2), gk_words(o_gks[2]))
        assert np.array_equal(ctx.pk_export(g_pk), np.stack(pk))
        ctx.gk_import(2, gk_words(o_gks[-3]), g_gk)
        assert np.array_equal(ctx.gk_export(g_gk, 2), gk_words(o_gks[-3]))
        # a word that is not a residue below its prime is refused
        bad = gk_words(o_gks[2]).copy()
        bad[1, 0, 2, 5] = np.uint64(pr.q[2])
        with pytest.raises(binding.EnsiError):
            ctx.gk_import(2, bad, g_gk)
        bad_pk = np.stack(pk).copy()
        bad_pk[1, 0, 0] = np.uint64(2 ** 63)
        with pytest.raises(binding.EnsiError):
            ctx.pk_import(bad_pk)
        # the secret key imported on its own decrypts what the server computed
        g_sk = ctx.sk_import(sk)
        dec = ctx.decrypt(g_sk, out, 0, 64)
        for i, st in enumerate(steps):
            assert np.abs(dec[i] - np.roll(z[i], -st)[:64]).max() < 1e-3
        with pytest.raises(binding.EnsiError):
            ctx.sk_import(np.full(o.N, 2, dtype=np.int8))
        for h in (g_pk, g_gk, g_rk, g_pt, g_ct, out, prod, g_sk):
            h.free()
    finally:
        ctx.close()


def test_null_randomness_comes_from_the_operating_system_when_the_seed_is_zero():
    """seed = 0: secret keys of two key generations differ, are ternary with all three values present, and the key
    pair works; a non-zero seed reproduces the same keys run after run (test mode)."""
    from paper_2509_09424_amd import binding
    w = wl.WORKLOADS[0]
    ctx = binding.Context(*w.param_tuple(), seed=0)
    try:
        sk1, pk1 = ctx.keygen(None, None, 11)
        sk2, pk2 = ctx.keygen(None, None, 11)
        s1, s2 = ctx.sk_export(sk1), ctx.sk_export(sk2)
        assert set(np.unique(s1)) == {-1, 0, 1} and not np.array_equal(s1, s2)
        assert abs(np.mean(s1 == 0) - 1 / 3) < 0.05 and abs(s1.astype(np.float64).mean()) < 0.06
        z = np.random.default_rng(0).uniform(-1, 1, (1, ctx.n_slots))
        pt = ctx.encode(z, w.q_count)
        ct = ctx.encrypt(pk1, pt)
        ct2 = ctx.encrypt(pk1, pt)
        assert not np.array_equal(ct.export(), ct2.export())  # fresh encryption randomness each time
        assert np.abs(ctx.decrypt(sk1, ct) - z).max() < 1e-3
        pk_words = ctx.pk_export(pk1)
        for h in (sk1, pk1, sk2, pk2, pt, ct, ct2):
            h.free()
        assert pk_words.shape == (2, w.q_count, ctx.N)
    finally:
        ctx.close()
    keys = []
    for _ in range(2):
        ctx = binding.Context(*w.param_tuple(), seed=5)
        sk, pk = ctx.keygen(None, None, 11)
        keys.append(ctx.sk_export(sk))
        sk.free()
        pk.free()
        ctx.close()
    assert np.array_equal(keys[0], keys[1])


def test_checksum_is_the_wrapping_sum_of_the_active_words():
    p = Pair(SMALL3)
    try:
        z = p.rng.uniform(-1, 1, (3, p.n))
        _, g_ct = p.encrypt_both(z, p.pr.L)
        with np.errstate(over="ignore"):
            want = g_ct.export().reshape(3, -1).sum(axis=1, dtype=np.uint64)
        assert np.array_equal(g_ct.checksum(), want)
        p.ctx.ct_drop_limbs(g_ct, 2)  # only the active limbs count
        with np.errstate(over="ignore"):
            want = g_ct.export().reshape(3, -1).sum(axis=1, dtype=np.uint64)
        assert g_ct.export().shape[2] == 2 and np.array_equal(g_ct.checksum(), want)
        g_ct.free()
    finally:
        p.close()


def test_prepared_weights_give_the_same_product():
    """ensi_weights_prepare + the *_prepared entry points against the plain ones: identical words, with and without
    rotations, and for the fused rescale + second layer; a second matrix of the same shape is not confused with the
    first (the plan cache compares the weights themselves)."""
    p = Pair((10, 50, 6, 60, 4, 4, 40))
    try:
        rng = np.random.default_rng(3)
        s, d, m = p.n // 4, 7, 9
        W = wl.ternary_weights(rng, d, m)
        W2 = W.copy()
        W2[3, 4] = (W2[3, 4] + 2) % 3 - 1  # one weight changed
        X = rng.uniform(-1, 1, (s, d))
        o_cts, g_ct = p.encrypt_both(wl.pack_columns(X, p.n), p.pr.L)
        _, g_gk = p.galois_keys([r * s for r in range(1, 4)])
        for placement in ("diagonal", "zero"):
            plain = p.ctx.ternary_matmul(g_gk, g_ct, s, d, W, placement)
            other = p.ctx.ternary_matmul(g_gk, g_ct, s, d, W2, placement)
            wt = p.ctx.weights_prepare(W, s, d, placement, p.pr.L)
            prep = p.ctx.ternary_matmul_prepared(g_gk, g_ct, wt)
            assert np.array_equal(prep.export(), plain.export()) and not np.array_equal(other.export(), plain.export())
            again = p.ctx.ternary_matmul(g_gk, g_ct, s, d, W, placement)  # cache hit on the first matrix again
            assert np.array_equal(again.export(), plain.export())
            with pytest.raises(p.binding.EnsiError):
                low = p.ctx.ct_alloc(g_ct.n, p.pr.L - 1)
                p.ctx.ternary_matmul_prepared(g_gk, low, wt, p.ctx.ct_alloc(m, p.pr.L - 1))  # prepared for another level
            for h in (plain, other, prep, again, wt):
                h.free()
        # second layer: one column per ciphertext, fused with the scalar-multiply + rescale
        dd, mm = 5, 6
        Wd = wl.ternary_weights(rng, dd, mm)
        _, a = p.encrypt_both(rng.uniform(-1, 1, (dd, p.n)), p.pr.L)
        _, b = p.encrypt_both(np.zeros((1, p.n)), p.pr.L)
        words = a.export()
        a2 = p.ctx.ct_import(words, a.scale)
        want = p.ctx.rescale_ternary_matmul(a, 2.0 ** -3, Wd)
        wt = p.ctx.weights_prepare(Wd, p.n, dd, "zero", p.pr.L - 1)
        got = p.ctx.rescale_ternary_matmul_prepared(a2, 2.0 ** -3, wt)
        assert np.array_equal(got.export(), want.export()) and got.scale == want.scale
        for h in (a, a2, b, want, got, wt, g_ct, g_gk):
            h.free()
    finally:
        p.close()


def test_matrix_rate_probe_reports_a_rate_below_the_data_sheet_peak():
    from paper_2509_09424_amd import binding
    ctx = binding.Context(*TINY, seed=1)
    try:
        rate = ctx.matrix_rate_probe(0.05)
        assert 0.5e15 < rate < 5.2e15  # int8 dense peak of the chip is 5.0e15 operations per second
        with pytest.raises(binding.EnsiError):
            ctx.matrix_rate_probe(5.0)
    finally:
        ctx.close()
