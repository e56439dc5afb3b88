"""Alg. 1 with the workloads' own weights at full size, against the oracle on sampled output columns.

The BitNet-shaped workloads do not fit the host whole (40 GiB of unpacked operands), so the oracle computes a sample
of the output columns -- at least 32 per product, always columns 0 and m-1, the rest seeded -- streaming over blocks
of rotation amounts (helpers.oracle_columns), and every word of those output ciphertexts must match.  The library
also returns the wrap-around 64-bit sum of every output ciphertext; the oracle reproduces it for the sampled
columns, and the two accumulate kernels (matrix-core and plain ALU) must agree on it for ALL outputs.
"""
import numpy as np
import pytest

import workloads as wl
from helpers import Pair, note, oracle_columns

pytestmark = pytest.mark.gpu


def sampled_columns(m, seed, count=32):
    rng = np.random.default_rng(seed)
    cols = {0, m - 1}
    while len(cols) < count:
        cols.add(int(rng.integers(0, m)))
    return sorted(cols)


def word_sum(limbs):
    with np.errstate(over="ignore"):
        return limbs.reshape(-1).sum(dtype=np.uint64)


def library_product(p, g_gk, g_ct, s, d, W, placement, cols, tag):
    """The product on the library, all outputs: returns the words of the sampled columns, their decryptions, and
    the checksum of every output; the plain-ALU kernel must give the same checksums as the matrix-core kernel."""
    c_tot = p.n // s
    out = p.ctx.ternary_matmul(g_gk, g_ct, s, d, W, placement)
    sums = out.checksum()
    n_o, limbs_o, scale_o, base_o = out._info()
    ct_words = 2 * limbs_o * p.N
    words, dec = {}, {}
    for i in cols:
        one = p.ctx.ct_wrap(int(base_o) + 8 * ct_words * i, 1, limbs_o, scale_o)
        words[i] = one.export()[0]
        dec[i] = p.ctx.decrypt(p.g_sk, one, p.o.placement_block(i, c_tot, placement) * s, s)[0]
        one.free()
    p.ctx.set_accumulate_mode(1)
    p.ctx.ternary_matmul(g_gk, g_ct, s, d, W, placement, out)
    sums_alu = out.checksum()
    p.ctx.set_accumulate_mode(0)
    out.free()
    assert np.array_equal(sums_alu, sums), "%s: the two accumulate kernels disagree on %d outputs" % (tag, int((sums_alu != sums).sum()))
    note("%s: library product done, checksums of all %d outputs agree between the two accumulate kernels" % (tag, W.shape[1]))
    return words, dec, sums


def compare_columns(got, want, X, W, cols, tag):
    words, dec, sums = got
    ref = X @ W[:, cols].astype(np.float64)
    err = 0.0
    for k, i in enumerate(cols):
        assert np.array_equal(words[i], want[i].limbs()), "%s: output column %d differs from the oracle" % (tag, i)
        assert int(sums[i]) == int(word_sum(want[i].limbs())), "%s: checksum of column %d" % (tag, i)
        err = max(err, float(np.abs(dec[i] - ref[:, k]).max()))
    assert err < 1e-3, "%s: decrypted error %.3e" % (tag, err)
    note("%s: %d sampled columns bit-exact against the oracle (checksums too), decrypted max error %.2e" % (tag, len(cols), err))


def test_bitnet_shapes_own_weights_on_sampled_columns():
    """The two BitNet-2B-shaped products that unpack by rotations: the FFN up-projection (2560 -> 6912, every output
    in block 0, the first half of the FFN workload) and the attention projection (2560 -> 2560, diagonal placement),
    each with its workload's own seeded weights.  Both share one parameter set, one token count and one set of 255
    Galois keys, and -- so that the oracle's 2550 rotations are paid once -- one encrypted input, the FFN workload's
    activations: each product is checked on 32 sampled columns (0, m-1 and 30 seeded)."""
    ffn, attn = wl.BY_NAME["ffn2560"], wl.BY_NAME["attn2560"]
    assert ffn.param_tuple() == attn.param_tuple() and ffn.tokens == attn.tokens and ffn.d_in == attn.d_in
    p = Pair(ffn.param_tuple())
    try:
        rng = wl.rng_for(ffn.index)
        W_up = wl.ternary_weights(rng, ffn.d_in, ffn.d_mid)
        X = wl.activations(rng, ffn.tokens, ffn.d_in, ffn.act)
        W_attn = wl.ternary_weights(wl.rng_for(attn.index), attn.d_in, attn.d_out)
        s, d, c_tot = ffn.tokens, ffn.d_in, ffn.c_tot
        L, beta = p.pr.L, p.pr.beta(p.pr.L)
        o_cts, g_ct = p.encrypt_both(wl.pack_columns(X, p.n), L)
        steps = [r * s for r in range(1, c_tot)]
        e = wl.error_poly(p.rng, (len(steps), beta, p.N))
        g_gk = p.ctx.galois_keygen(p.g_sk, steps, e, 99)
        note("bitnet shapes: %d inputs encrypted, %d Galois keys generated" % (len(o_cts), len(steps)))
        cols_up = sampled_columns(ffn.d_mid, 2509)
        cols_at = sampled_columns(attn.d_out, 9424)
        got_up = library_product(p, g_gk, g_ct, s, d, W_up, "zero", cols_up, "ffn2560 up-projection")
        got_at = library_product(p, g_gk, g_ct, s, d, W_attn, "diagonal", cols_at, "attn2560")
        g_ct.free()
        g_gk.free()
        want_up, want_at = oracle_columns(p.o, p.o_sk, o_cts, s, [(W_up, "zero", cols_up), (W_attn, "diagonal", cols_at)],
                                          lambda st: e[st // s - 1], 99, tell=lambda t: note("bitnet shapes " + t))
        compare_columns(got_up, want_up, X, W_up, cols_up, "ffn2560 up-projection")
        compare_columns(got_at, want_at, X, W_attn, cols_at, "attn2560")
    finally:
        p.close()


def test_proj768_own_weights_on_sampled_columns():
    """The 768 x 768 projection (32 tokens, one packed input, diagonal placement, up to 1023 rotation amounts) with
    its own seeded weights and activations on 32 sampled columns."""
    w = wl.BY_NAME["proj768"]
    p = Pair(w.param_tuple())
    try:
        rng = wl.rng_for(w.index)
        W = wl.ternary_weights(rng, w.d_in, w.d_out)
        X = wl.activations(rng, w.tokens, w.d_in, w.act)
        s, d, c_tot = w.tokens, w.d_in, w.c_tot
        L, beta = p.pr.L, p.pr.beta(p.pr.L)
        o_cts, g_ct = p.encrypt_both(wl.pack_columns(X, p.n), L)
        steps = [r * s for r in range(1, c_tot)]
        e = wl.error_poly(p.rng, (len(steps), beta, p.N))
        g_gk = p.ctx.galois_keygen(p.g_sk, steps, e, 99)
        note("proj768: %d Galois keys generated" % len(steps))
        cols = sampled_columns(w.d_out, 768)
        got = library_product(p, g_gk, g_ct, s, d, W, "diagonal", cols, "proj768")
        g_ct.free()
        g_gk.free()
        (want,) = oracle_columns(p.o, p.o_sk, o_cts, s, [(W, "diagonal", cols)], lambda st: e[st // s - 1], 99, tell=lambda t: note("proj768 " + t))
        compare_columns(got, want, X, W, cols, "proj768")
    finally:
        p.close()
