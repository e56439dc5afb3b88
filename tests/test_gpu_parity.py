"""GPU parity: the HIP library against the CPU oracle, through the C ABI, on the
same seeded inputs.  Integer results (RNS limbs) must match bit for bit;
decrypted slots must lie within 1e-3 of the float64 product."""
import numpy as np
import pytest

import workloads as wl
from helpers import Pair, stack_cts, to_oracle_cts

pytestmark = pytest.mark.gpu

TINY = wl.WORKLOADS[0].param_tuple()
# a small ring with the BitNet-shaped workloads' chain structure (alpha=4, partial last digit at lower levels)
SMALL4 = (10, 50, 6, 60, 4, 4, 40)
SMALL3 = (10, 50, 5, 60, 3, 3, 40)  # alpha=3: digits 3+2


@pytest.fixture(scope="module")
def tiny():
    p = Pair(TINY)
    yield p
    p.close()


@pytest.fixture(scope="module")
def small4():
    p = Pair(SMALL4)
    yield p
    p.close()


def test_primes_match_oracle(tiny):
    q, p = tiny.ctx.primes()
    assert q == tiny.pr.q and p == tiny.pr.p


def test_ntt_roundtrip_and_evaluation_set(tiny):
    rng = np.random.default_rng(0)
    primes = tiny.pr.q + tiny.pr.p
    x = np.stack([rng.integers(0, m, size=tiny.N, dtype=np.uint64) for m in primes])
    # ship the rows to the device inside a ciphertext-shaped import (2 ciphertexts x 2 polys x 1 limb)
    ct = tiny.ctx.ct_import(x.reshape(2, 2, 1, tiny.N) % np.uint64(tiny.pr.q[0]), 1.0)
    x = ct.export().reshape(4, tiny.N)
    idx = [0, 0, 0, 0]
    tiny.ctx.ntt(ct.device_ptr, idx, inverse=False)
    fwd = ct.export().reshape(4, tiny.N)
    want = tiny.o.ntt(x, [tiny.pr.q[0]] * 4)
    # whichever primitive root a side picked, the transform is the set of evaluations at all odd powers
    assert np.array_equal(np.sort(fwd, axis=1), np.sort(want, axis=1))
    assert not np.array_equal(fwd, x)
    tiny.ctx.ntt(ct.device_ptr, idx, inverse=True)
    assert np.array_equal(ct.export().reshape(4, tiny.N), x)
    ct.free()


def test_encode_within_one_and_import_export(tiny):
    rng = np.random.default_rng(1)
    z = rng.uniform(-1, 1, (2, tiny.n))
    pt = tiny.ctx.encode(z, tiny.pr.L)
    got = tiny.ctx.pt_export(pt)
    want = np.stack([tiny.o.encode_coeffs(v) for v in z])
    assert np.abs(got - want).max() <= 1
    assert (got != want).mean() < 0.01
    pt2 = tiny.ctx.pt_import(want, tiny.pr.L)
    assert np.array_equal(tiny.ctx.pt_export(pt2), want)
    pt.free()
    pt2.free()


def test_encrypt_bit_exact_and_decrypt(tiny):
    rng = np.random.default_rng(2)
    z = rng.uniform(-1, 1, (3, tiny.n))
    o_cts, g_ct = tiny.encrypt_both(z, tiny.pr.L)
    assert np.array_equal(g_ct.export(), stack_cts(o_cts))
    got = tiny.ctx.decrypt(tiny.g_sk, g_ct)
    want = np.stack([tiny.o.decrypt(c, tiny.o_sk) for c in o_cts])
    assert np.abs(got - want).max() < 1e-7
    assert np.abs(got - z).max() < 1e-3
    part = tiny.ctx.decrypt(tiny.g_sk, g_ct, slot_begin=64, n_slots=32)
    assert np.abs(part - want[:, 64:96]).max() < 1e-7
    g_ct.free()


@pytest.mark.parametrize("params", [TINY, SMALL4, SMALL3], ids=["tiny", "alpha4", "alpha3"])
def test_rotate_bit_exact(params):
    p = Pair(params)
    try:
        steps = [1, -1, 5, p.n // 2, 3]
        o_gks, g_gk = p.galois_keys(sorted(set(steps)))
        z = p.rng.uniform(-1, 1, (len(steps), p.n))
        for limbs in sorted({p.pr.L, max(2, p.pr.L - 1), 2}, reverse=True):
            o_cts, g_ct = p.encrypt_both(z, limbs)
            out = p.ctx.rotate(g_gk, g_ct, steps)
            want = [p.o.rotate(c, o_gks[st]) for c, st in zip(o_cts, steps)]
            assert np.array_equal(out.export(), stack_cts(want)), "limbs=%d" % limbs
            dec = p.ctx.decrypt(p.g_sk, out)
            for i, st in enumerate(steps):
                assert np.abs(dec[i] - np.roll(z[i], -st)).max() < 1e-3
            assert out.limbs == limbs and out.scale == g_ct.scale
            out.free()
            g_ct.free()
        g_gk.free()
    finally:
        p.close()


@pytest.mark.parametrize("placement", ["diagonal", "zero"])
def test_tiny_workload_matmul_bit_exact(tiny, placement):
    w = wl.WORKLOADS[0]
    rng = wl.rng_for(w.index)
    W = wl.ternary_weights(rng, w.d_in, w.d_out)
    X = wl.activations(rng, w.tokens, w.d_in, w.act)
    packed = wl.pack_columns(X, tiny.n)
    o_cts, g_ct = tiny.encrypt_both(packed, tiny.pr.L)
    rhos = list(range(1, w.c_tot))
    o_by_step, g_gk = tiny.galois_keys([r * w.tokens for r in rhos])
    o_gks = {r: o_by_step[r * w.tokens] for r in rhos}
    want = tiny.o.ternary_matmul(o_cts, w.tokens, w.d_in, W, placement, o_gks)
    for mode in (1, 2):  # plain-ALU kernel, then the matrix-core kernel
        tiny.ctx.set_accumulate_mode(mode)
        out = tiny.ctx.ternary_matmul(g_gk, g_ct, w.tokens, w.d_in, W, placement)
        assert np.array_equal(out.export(), stack_cts(want)), "accumulate mode %d" % mode
        if mode == 1:
            out.free()
    tiny.ctx.set_accumulate_mode(0)
    assert out.limbs == tiny.pr.L and out.scale == g_ct.scale  # PCMM consumes no level
    ref = X @ W.astype(np.float64)
    err = 0.0
    dec = tiny.ctx.decrypt(tiny.g_sk, out)
    for i in range(w.d_out):
        p_i = 0 if placement == "zero" else i % w.c_tot
        err = max(err, np.abs(dec[i, p_i * w.tokens:(p_i + 1) * w.tokens] - ref[:, i]).max())
    assert err < 1e-3  # both placements (the oracle measures 3.6e-4 and 2.5e-4)
    out.free()
    g_ct.free()
    g_gk.free()


def test_matmul_paper_packing_needs_no_key(small4):
    """One column per ciphertext (c_tot = 1): the paper's own packing; pure add/sub."""
    p = small4
    d, m = 37, 70  # ragged against the 32-wide output tiles
    rng = np.random.default_rng(5)
    W = wl.ternary_weights(rng, d, m)
    W[:, 3] = 0  # an all-zero weight column gives the all-zero ciphertext
    X = rng.uniform(-1, 1, (p.n, d))
    for limbs in (p.pr.L, 3):
        o_cts, g_ct = p.encrypt_both(X.T, limbs)
        want = p.o.ternary_matmul(o_cts, p.n, d, W, "zero", {})
        for mode in (1, 2):
            p.ctx.set_accumulate_mode(mode)
            out = p.ctx.ternary_matmul(None, g_ct, p.n, d, W, "zero")
            got = out.export()
            assert np.array_equal(got, stack_cts(want)), "accumulate mode %d, limbs %d" % (mode, limbs)
            if mode == 1:
                out.free()
        p.ctx.set_accumulate_mode(0)
        assert not got[3].any()
        dec = p.ctx.decrypt(p.g_sk, out)
        assert np.abs(dec.T - X @ W.astype(np.float64)).max() < 1e-3
        out.free()
        g_ct.free()


def test_matmul_several_packed_inputs(small4):
    p = small4
    s, d, m = 64, 19, 13  # c_tot = 8: three packed inputs, the last one ragged
    rng = np.random.default_rng(6)
    W = wl.ternary_weights(rng, d, m)
    X = rng.uniform(-1, 1, (s, d))
    packed = wl.pack_columns(X, p.n)
    assert packed.shape[0] == 3
    o_cts, g_ct = p.encrypt_both(packed, p.pr.L)
    c_tot = p.n // s
    o_by_step, g_gk = p.galois_keys([r * s for r in range(1, c_tot)])
    o_gks = {r: o_by_step[r * s] for r in range(1, c_tot)}
    for placement in ("diagonal", "zero"):
        want = p.o.ternary_matmul(o_cts, s, d, W, placement, o_gks)
        for mode in (1, 2):
            p.ctx.set_accumulate_mode(mode)
            out = p.ctx.ternary_matmul(g_gk, g_ct, s, d, W, placement)
            assert np.array_equal(out.export(), stack_cts(want)), (placement, mode)
            if mode == 1:
                out.free()
        p.ctx.set_accumulate_mode(0)
        dec = p.ctx.decrypt(p.g_sk, out)
        ref = X @ W.astype(np.float64)
        for i in range(m):
            p_i = 0 if placement == "zero" else i % c_tot
            assert np.abs(dec[i, p_i * s:(p_i + 1) * s] - ref[:, i]).max() < 1e-3
        out.free()
    g_ct.free()
    g_gk.free()


def test_matmul_many_operands_and_wide_primes():
    """Long sums: 300 operands on 50-bit primes (matrix-core kernel, several k-steps, nine
    256-output tiles: one full group of eight plus a ragged one) and 40 operands on 60-bit primes (plain-ALU kernel with mid-loop reductions,
    the only valid one there)."""
    for params, d, m in (((8, 50, 3, 60, 1, 3, 40), 300, 2100), ((8, 60, 2, 61, 1, 2, 40), 40, 33)):
        p = Pair(params)
        try:
            rng = np.random.default_rng(8)
            W = wl.ternary_weights(rng, d, m)
            X = rng.uniform(-1, 1, (p.n, d)) * 0.05
            o_cts, g_ct = p.encrypt_both(X.T, p.pr.L)
            want = stack_cts(p.o.ternary_matmul(o_cts, p.n, d, W, "zero", {}))
            for mode in (1, 2):
                p.ctx.set_accumulate_mode(mode)
                out = p.ctx.ternary_matmul(None, g_ct, p.n, d, W, "zero")
                assert np.array_equal(out.export(), want), (params, mode)
                out.free()
            g_ct.free()
        finally:
            p.close()


def test_mul_scalar_rescale_bit_exact_and_two_layer(small4):
    p = small4
    rng = np.random.default_rng(7)
    z = rng.uniform(-1, 1, (2, p.n))
    for kappa in (2.0 ** -5, -0.3):
        o_cts, g_ct = p.encrypt_both(z, p.pr.L)
        want = [p.o.mul_scalar_rescale(c, kappa) for c in o_cts]
        p.ctx.mul_scalar_rescale(g_ct, kappa)
        assert g_ct.limbs == p.pr.L - 1
        assert np.array_equal(g_ct.export(), stack_cts(want))
        assert g_ct.scale == want[0].scale
        dec = p.ctx.decrypt(p.g_sk, g_ct)
        assert np.abs(dec - kappa * z).max() < 1e-3
        # a rotation after the rescale runs at the lower level on the strided storage
        o_gks, g_gk = p.galois_keys([2])
        rot = p.ctx.rotate(g_gk, g_ct, [2, 2])
        want_rot = [p.o.rotate(c, o_gks[2]) for c in want]
        assert np.array_equal(rot.export(), stack_cts(want_rot))
        rot.free()
        g_gk.free()
        g_ct.free()


def test_rescale_fused_into_second_layer_bit_exact(small4):
    """Scalar-multiply + rescale applied while the second layer's accumulate reads its operands
    (one call) against the oracle's two steps, on both accumulate paths and for a ragged operand count."""
    p = small4
    d, m = 37, 70
    rng = np.random.default_rng(9)
    W = wl.ternary_weights(rng, d, m)
    X = rng.uniform(-1, 1, (p.n, d))
    for limbs, kappa in ((p.pr.L, 2.0 ** -5), (3, -0.3)):
        o_cts, _ = p.encrypt_both(X.T, limbs)
        o_mid = [p.o.mul_scalar_rescale(c, kappa) for c in o_cts]
        want = stack_cts(p.o.ternary_matmul(o_mid, p.n, d, W, "zero", {}))
        for mode in (1, 2):
            g_ct = p.ctx.ct_import(stack_cts(o_cts), o_cts[0].scale)
            p.ctx.set_accumulate_mode(mode)
            out = p.ctx.rescale_ternary_matmul(g_ct, kappa, W)
            assert out.limbs == limbs - 1 and g_ct.limbs == limbs - 1
            assert np.array_equal(out.export(), want), "accumulate mode %d, limbs %d" % (mode, limbs)
            assert out.scale == o_mid[0].scale == g_ct.scale
            if mode == 2:
                dec = p.ctx.decrypt(p.g_sk, out)
                assert np.abs(dec.T - (kappa * X) @ W.astype(np.float64)).max() < 1e-3
            out.free()
            g_ct.free()
        p.ctx.set_accumulate_mode(0)
    E = p.binding.EnsiError
    one = p.ctx.ct_import(stack_cts(o_cts)[:, :, :1], 1.0)
    dst = p.ctx.ct_alloc(m, 1)
    with pytest.raises(E, match="code -3"):
        p.ctx.rescale_ternary_matmul(one, 0.5, W, dst)  # no limb left to drop
    dst.free()
    one.free()


def test_error_paths(tiny):
    E = tiny.binding.EnsiError
    z = np.zeros((1, tiny.n))
    _, g_ct = tiny.encrypt_both(z, tiny.pr.L)
    _, g_gk = tiny.galois_keys([1])
    with pytest.raises(E, match="code -2"):
        tiny.ctx.rotate(g_gk, g_ct, [2])  # no key for step 2
    W = np.zeros((64, 64), dtype=np.int8)
    W[0, 0] = 2
    with pytest.raises(E, match="code -1"):
        tiny.ctx.ternary_matmul(g_gk, g_ct, 32, 64, W)
    W[0, 0] = 1
    W[5, 0] = 1
    with pytest.raises(E, match="code -2"):
        tiny.ctx.ternary_matmul(None, g_ct, 32, 64, W, "zero")  # needs rotations, no key set
    with pytest.raises(E, match="code -4"):
        tiny.ctx.ternary_matmul(g_gk, g_ct, 32, 4000, np.zeros((4000, 2), dtype=np.int8))  # needs 2 packed inputs
    low = tiny.ctx.ct_alloc(1, 2)
    with pytest.raises(E, match="code -3"):
        tiny.ctx.rotate(g_gk, g_ct, [1], low)
    low.free()
    g_ct.free()
    g_gk.free()


# ---------------------------------------------------------------- full ring (N = 2^16)
KEYSWITCH = wl.WORKLOADS[1].param_tuple()  # 10 x 50-bit + 3 x 60-bit, alpha = 3


@pytest.fixture(scope="module")
def full():
    p = Pair(KEYSWITCH)
    yield p
    p.close()


def test_full_ring_ntt_roundtrip_and_evaluation_set(full):
    """The N = 2^16 transform (register radix-16 steps; fp64 arithmetic on the 50-bit primes,
    integer arithmetic on the 60-bit ones)."""
    rng = np.random.default_rng(10)
    L = full.pr.L
    primes = full.pr.q + full.pr.p
    idx = [0, L - 1, L, L + 2]  # two 50-bit primes, two 60-bit primes
    x = np.stack([rng.integers(0, full.pr.q[-1], size=full.N, dtype=np.uint64) for _ in idx])
    x[0, :4] = [0, 1, full.pr.q[0] - 1, full.pr.q[0] // 2]
    x[0] %= np.uint64(full.pr.q[0])
    ct = full.ctx.ct_import(x.reshape(2, 2, 1, full.N) % np.uint64(full.pr.q[0]), 1.0)
    x = ct.export().reshape(4, full.N)
    full.ctx.ntt(ct.device_ptr, idx, inverse=False)
    fwd = ct.export().reshape(4, full.N)
    want = full.o.ntt(x, [primes[i] for i in idx])
    assert np.array_equal(np.sort(fwd, axis=1), np.sort(want, axis=1))
    full.ctx.ntt(ct.device_ptr, idx, inverse=True)
    assert np.array_equal(ct.export().reshape(4, full.N), x)
    ct.free()


def test_full_ring_ntt_batch_with_ragged_groups(full):
    """A batch whose limbs cycle through three primes (two below 2^50, one above) and whose count leaves the last
    group of every prime incomplete: the row pass runs a tile for up to eight limbs of one prime per block."""
    import torch
    rng = np.random.default_rng(12)
    L = full.pr.L
    primes = full.pr.q + full.pr.p
    pattern = [1, L + 1, L - 1]
    n = 29  # 10, 10 and 9 limbs per prime: groups of 8 + 2, 8 + 2, 8 + 1
    idx = [pattern[r % 3] for r in range(n)]
    x = np.stack([rng.integers(0, primes[i], size=full.N, dtype=np.uint64) for i in idx])
    buf = torch.from_numpy(x.view(np.int64)).cuda()
    full.ctx.ntt(buf.data_ptr(), idx, inverse=False)
    torch.cuda.synchronize()
    fwd = buf.cpu().numpy().view(np.uint64)
    for r in (0, 1, 2, 23, 24, 26, 27, 28):  # first limbs, and the limbs of the incomplete groups
        want = full.o.ntt(x[r:r + 1], [primes[idx[r]]])[0]
        assert np.array_equal(np.sort(fwd[r]), np.sort(want)), r
    # limbs of one prime are transformed alike: same input -> same output, whatever its place in a group
    y = x.copy()
    y[27] = x[0]
    buf2 = torch.from_numpy(y.view(np.int64)).cuda()
    full.ctx.ntt(buf2.data_ptr(), idx, inverse=False)
    torch.cuda.synchronize()
    assert np.array_equal(buf2[27].cpu().numpy(), buf[0].cpu().numpy())
    full.ctx.ntt(buf.data_ptr(), idx, inverse=True)
    torch.cuda.synchronize()
    assert np.array_equal(buf.cpu().numpy().view(np.uint64), x)


def test_full_ring_rotate_bit_exact(full):
    p = full
    steps = [1, -1, 4096]
    o_gks, g_gk = p.galois_keys(sorted(set(steps)))
    z = p.rng.uniform(-1, 1, (len(steps), p.n))
    for limbs in (p.pr.L, 4):
        o_cts, g_ct = p.encrypt_both(z, limbs)
        assert np.array_equal(g_ct.export(), stack_cts(o_cts))
        out = p.ctx.rotate(g_gk, g_ct, steps)
        want = [p.o.rotate(c, o_gks[st]) for c, st in zip(o_cts, steps)]
        assert np.array_equal(out.export(), stack_cts(want)), "limbs=%d" % limbs
        dec = p.ctx.decrypt(p.g_sk, out, 0, 256)
        for i, st in enumerate(steps):
            assert np.abs(dec[i] - np.roll(z[i], -st)[:256]).max() < 1e-3
        out.free()
        g_ct.free()
    g_gk.free()


def test_full_ring_rotate_all_sixteen_galois_elements(full, capsys):
    """The key-switch microbenchmark's own step set at the full level: one ciphertext per Galois element (steps
    2^0 .. 2^14 and -1), every one bit-exact against the oracle and a left shift of the slots after decryption."""
    p = full
    steps = list(wl.KEYSWITCH_STEPS)
    assert len(steps) == 16 and len({p.pr.galois_element(st) for st in steps}) == 16
    o_gks, g_gk = p.galois_keys(steps)
    z = p.rng.uniform(-1, 1, (len(steps), p.n))
    o_cts, g_ct = p.encrypt_both(z, p.pr.L)
    out = p.ctx.rotate(g_gk, g_ct, steps)
    got = out.export()
    for i, st in enumerate(steps):
        assert np.array_equal(got[i], p.o.rotate(o_cts[i], o_gks[st]).limbs()), "step %d" % st
    dec = p.ctx.decrypt(p.g_sk, out)
    err = max(np.abs(dec[i] - np.roll(z[i], -st)).max() for i, st in enumerate(steps))
    assert err < 1e-3
    with capsys.disabled():
        print("\n[cfg 2, alpha = 3] 16 Galois elements bit-exact; decrypted max abs error %.3e" % err, flush=True)
    out.free()
    g_ct.free()
    g_gk.free()


def test_full_ring_rotate_literal_three_digits(capsys):
    """The literal reading of "dnum = 3" for the key-switch configuration: 10 ciphertext primes in three digits of
    4, 4 and 2 limbs (alpha = 4) against three special primes.  A digit is then larger than P, so the switching
    noise is far above the 1e-3 bound: parity (which does not depend on the noise) is gated, the decrypted error is
    only reported."""
    w = wl.WORKLOADS[1]
    p = Pair((w.log_n, w.q_bits, w.q_count, w.p_bits, w.p_count, 4, w.log_scale))
    try:
        assert p.pr.beta(p.pr.L) == 3
        steps = [1, -1, 1 << 7, 1 << 14]
        o_gks, g_gk = p.galois_keys(steps)
        z = p.rng.uniform(-1, 1, (len(steps), p.n))
        o_cts, g_ct = p.encrypt_both(z, p.pr.L)
        out = p.ctx.rotate(g_gk, g_ct, steps)
        got = out.export()
        for i, st in enumerate(steps):
            assert np.array_equal(got[i], p.o.rotate(o_cts[i], o_gks[st]).limbs()), "step %d" % st
        dec = p.ctx.decrypt(p.g_sk, out)
        err = max(np.abs(dec[i] - np.roll(z[i], -st)).max() for i, st in enumerate(steps))
        with capsys.disabled():
            print("\n[cfg 2, literal alpha = 4, beta = 3] bit-exact; decrypted max abs error %.3e (reported, not gated)" % err, flush=True)
        out.free()
        g_ct.free()
        g_gk.free()
    finally:
        p.close()


def test_full_ring_matmul_bit_exact(full):
    p = full
    s, d, m = p.n // 4, 6, 5  # c_tot = 4: two packed inputs, rotations by 1..3 blocks
    rng = np.random.default_rng(11)
    W = wl.ternary_weights(rng, d, m)
    W[0, 0], W[5, 4] = 1, -1
    X = np.clip(rng.standard_normal((s, d)), -4, 4)
    packed = wl.pack_columns(X, p.n)
    o_cts, g_ct = p.encrypt_both(packed, p.pr.L)
    o_by_step, g_gk = p.galois_keys([r * s for r in range(1, 4)])
    o_gks = {r: o_by_step[r * s] for r in range(1, 4)}
    want = stack_cts(p.o.ternary_matmul(o_cts, s, d, W, "diagonal", o_gks))
    for mode in (1, 2):
        p.ctx.set_accumulate_mode(mode)
        out = p.ctx.ternary_matmul(g_gk, g_ct, s, d, W, "diagonal")
        assert np.array_equal(out.export(), want), "accumulate mode %d" % mode
        if mode == 1:
            out.free()
    p.ctx.set_accumulate_mode(0)
    ref = X @ W.astype(np.float64)
    for i in range(m):
        one = p.ctx.decrypt(p.g_sk, out, (i % 4) * s, 512)
        assert np.abs(one[i] - ref[:512, i]).max() < 1e-3
    out.free()
    g_ct.free()
    g_gk.free()


@pytest.mark.parametrize("params,why", [
    ((16, 45, 4, 48, 2, 2, 36), "every prime below 2^50: the special limbs take the fp64 path of the fused kernels too"),
    ((16, 55, 3, 60, 1, 2, 40), "ciphertext primes above 2^50: the unfused integer kernels at N = 2^16"),
], ids=["all-fp", "wide-q"])
def test_full_ring_rotate_other_prime_sizes(params, why):
    p = Pair(params)
    steps = [3, -5]
    o_gks, g_gk = p.galois_keys(steps)
    z = p.rng.uniform(-1, 1, (len(steps), p.n))
    for limbs in (p.pr.L, 1):
        o_cts, g_ct = p.encrypt_both(z, limbs)
        out = p.ctx.rotate(g_gk, g_ct, steps)
        want = [p.o.rotate(c, o_gks[st]) for c, st in zip(o_cts, steps)]
        assert np.array_equal(out.export(), stack_cts(want)), (why, limbs)
        out.free()
        g_ct.free()
    g_gk.free()
    p.close()


def test_full_ring_rotate_batch_longer_than_one_group(full):
    """More ciphertexts than the library raises at once (groups of 64), at a low level to keep the oracle quick."""
    p = full
    n_ct = 67
    steps = [1 if i % 2 else -1 for i in range(n_ct)]
    o_gks, g_gk = p.galois_keys([1, -1])
    z = p.rng.uniform(-1, 1, (n_ct, p.n))
    o_cts, g_ct = p.encrypt_both(z, 2)
    out = p.ctx.rotate(g_gk, g_ct, steps)
    got = out.export()
    for i in (0, 1, 62, 63, 64, 65, 66):
        assert np.array_equal(got[i], p.o.rotate(o_cts[i], o_gks[steps[i]]).limbs()), i
    out.free()
    g_ct.free()
    g_gk.free()
