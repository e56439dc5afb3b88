"""GPU parity of ciphertext-ciphertext multiplication (Mult with one relinearisation and one rescale), of the
element replication and of the CCMM product built on them, through the C ABI: every output limb must equal the
oracle's bit for bit (same keys from the same seeded randomness, plaintext masks encoded by the oracle)."""
import numpy as np
import pytest

import workloads as wl
from helpers import Pair, stack_cts

pytestmark = pytest.mark.gpu

SMALL4 = (10, 50, 6, 60, 4, 4, 40)
WIDE = (10, 55, 4, 60, 2, 2, 40)      # ciphertext primes above 2^50: integer kernels throughout
TINY5 = (5, 50, 5, 60, 3, 3, 40)      # 16 slots: the whole CCMM against numpy in a blink
KEYSWITCH = wl.WORKLOADS[1].param_tuple()


def relin_keys(p, seed=77):
    e = wl.error_poly(p.rng, (p.pr.beta(p.pr.L), p.N))
    return p.o.relin_keygen(p.o_sk, e, seed), p.ctx.relin_keygen(p.g_sk, e, seed)


def mult_case(p, l1, n_ct=4):
    z = p.rng.uniform(-1, 1, (2 * n_ct, p.n))
    o_cts, g_ct = p.encrypt_both(z, l1)
    return z, o_cts, g_ct


@pytest.mark.parametrize("params,l1", [(SMALL4, 6), (SMALL4, 5), (WIDE, 4)], ids=["six-limbs", "partial-digit", "wide-primes"])
def test_mult_sum_relin_rescale_small_ring(params, l1):
    p = Pair(params)
    o_rk, g_rk = relin_keys(p)
    z, o_cts, g_ct = mult_case(p, l1)
    # output 0: one product; 1: nothing; 2: a sum of five products with repeated operands; 3: a square
    begin = [0, 1, 1, 6, 7]
    ta = [0, 1, 2, 3, 4, 5, 6]
    tb = [7, 6, 5, 4, 3, 1, 6]
    out = p.ctx.mult_sum_relin_rescale(g_rk, g_ct, g_ct, begin, ta, tb)
    got = out.export()
    assert out.limbs == l1 - 1 and abs(out.scale / (p.pr.scale ** 2 / p.pr.q[l1 - 1]) - 1) < 1e-12
    for o in range(4):
        pairs = [(o_cts[ta[t]], o_cts[tb[t]]) for t in range(begin[o], begin[o + 1])]
        if pairs:
            want = p.o.mult_sum_relin_rescale(pairs, o_rk).limbs()
            ref = sum(z[ta[t]] * z[tb[t]] for t in range(begin[o], begin[o + 1]))
            dec = p.ctx.decrypt(p.g_sk, out)[o]
            assert np.abs(dec - ref).max() < 1e-3, o
        else:
            want = np.zeros((2, l1 - 1, p.N), dtype=np.uint64)
        assert np.array_equal(got[o], want), o
    # without an evaluation key in the set
    _, g_gk = p.galois_keys([3])
    with pytest.raises(p.binding.EnsiError, match="code -2"):
        p.ctx.mult_sum_relin_rescale(g_gk, g_ct, g_ct, [0, 1], [0], [1], out)
    for h in (g_ct, out, g_rk, g_gk):
        h.free()
    p.close()


def test_mult_full_ring():
    """N = 2^16: the transform and key-switch kernels of the fused path carry the product; a low level keeps the
    oracle quick; operands whose limb stride is wider than their level."""
    p = Pair(KEYSWITCH)
    o_rk, g_rk = relin_keys(p)
    l1 = 4
    z, o_cts, g_ct = mult_case(p, l1, n_ct=2)
    p.ctx.ct_drop_limbs(g_ct, 3)
    o3 = [p.o.drop_limbs(c, 3) for c in o_cts]
    out = p.ctx.mult_sum_relin_rescale(g_rk, g_ct, g_ct, [0, 2, 3], [0, 1, 2], [3, 2, 2])
    want = [p.o.mult_sum_relin_rescale([(o3[0], o3[3]), (o3[1], o3[2])], o_rk), p.o.mult_sum_relin_rescale([(o3[2], o3[2])], o_rk)]
    assert out.limbs == 2 and np.array_equal(out.export(), stack_cts(want))
    dec = p.ctx.decrypt(p.g_sk, out)
    assert np.abs(dec[0] - (z[0] * z[3] + z[1] * z[2])).max() < 1e-3 and np.abs(dec[1] - z[2] ** 2).max() < 1e-3
    for h in (g_ct, out, g_rk):
        h.free()
    p.close()


def doubling_keys(p, period=None):
    """Keys for the steps of the library's fill schedule (the oracle follows its own and must find its keys here)."""
    steps = set(p.ctx.fill_steps(1, p.n))
    if period:
        steps |= set(p.ctx.fill_steps(period, p.n)) | set(p.ctx.fill_steps(1, period))
    return p.galois_keys(sorted(steps))


@pytest.mark.parametrize("params", [TINY5, SMALL4], ids=["16-slots", "512-slots"])
def test_replicate_against_oracle(params):
    p = Pair(params)
    l1 = p.pr.L
    o_gks, g_gk = doubling_keys(p)
    z = p.rng.uniform(-1, 1, (2, p.n))
    o_cts, g_ct = p.encrypt_both(z, l1)
    ks = [0, 3, p.n - 1]
    masks = p.o.one_hot_masks(ks, l1)
    g_masks = p.ctx.pt_set_scale(p.ctx.pt_import(masks, l1), float(p.pr.q[l1 - 1]))
    src, mi = [0, 1, 1, 0], [1, 0, 2, 2]
    out = p.ctx.replicate(g_gk, g_ct, src, g_masks, mi)
    want = [p.o.replicate(o_cts[src[o]], masks[mi[o]], o_gks) for o in range(4)]
    assert out.limbs == l1 - 1 and np.array_equal(out.export(), stack_cts(want))
    dec = p.ctx.decrypt(p.g_sk, out)
    for o in range(4):
        assert np.abs(dec[o] - z[src[o], ks[mi[o]]]).max() < 1e-3, o
    # the library's own one-hot masks decode to the same selection
    lib = p.ctx.one_hot_masks(4, l1)
    out2 = p.ctx.replicate(g_gk, g_ct, [1], lib, [3])
    assert np.abs(p.ctx.decrypt(p.g_sk, out2)[0] - z[1, 3]).max() < 1e-3
    for h in (g_ct, g_masks, lib, out, out2, g_gk):
        h.free()
    p.close()


@pytest.mark.parametrize("params,d,m,period", [(TINY5, 3, 2, 4), (SMALL4, 5, 3, 8), (SMALL4, 8, 2, 8)], ids=["16-slots", "512-slots", "d-equals-period"])
def test_ccmm_against_oracle_and_numpy(params, d, m, period):
    """CCMM section, C = A B, with the two-stage element extraction."""
    p = Pair(params)
    l1 = p.pr.L
    A = p.rng.uniform(-1, 1, (p.n, d))
    Bm = p.rng.uniform(-1, 1, (d, m))
    o_gks, g_gk = doubling_keys(p, period)
    o_rk, g_rk = relin_keys(p)
    zb = np.zeros((m, p.n))  # B[j, i] in slot j of ciphertext i, zeros elsewhere
    zb[:, :d] = Bm.T
    o_a, g_a = p.encrypt_both(A.T, l1)
    o_b, g_b = p.encrypt_both(zb, l1)
    masks = p.o.periodic_masks(period, d, l1)
    g_masks = p.ctx.pt_set_scale(p.ctx.pt_import(masks, l1), float(p.pr.q[l1 - 1]))
    out = p.ctx.ccmm(g_rk, g_gk, g_a, g_b, g_masks, period)
    want = p.o.ccmm(o_a, o_b, d, period, o_rk, o_gks)
    assert out.n == m and out.limbs == l1 - 2 and abs(out.scale / want[0].scale - 1) < 1e-12
    assert np.array_equal(out.export(), stack_cts(want))
    assert np.abs(p.ctx.decrypt(p.g_sk, out) - (A @ Bm).T).max() < 1e-3
    # the library's own masks
    lib = p.ctx.periodic_masks(period, d, l1)
    out2 = p.ctx.ccmm(g_rk, g_gk, g_a, g_b, lib, period)
    assert np.abs(p.ctx.decrypt(p.g_sk, out2) - (A @ Bm).T).max() < 1e-3
    with pytest.raises(p.binding.EnsiError, match="code -1"):
        p.ctx.ccmm(g_rk, g_gk, g_a, g_b, g_masks, 3, out)  # not a power of two
    for h in (g_a, g_b, g_masks, lib, out, out2, g_gk, g_rk):
        h.free()
    p.close()


def test_ccmm_full_ring_at_the_benchmark_parameters():
    """N = 2^16 with the 16 + 4 limb chain of the ccmm96 benchmark workload (fused key-switch and multiplication
    kernels), a narrow product (d = 4, one output column) so that the oracle's 13 giant steps, 8 baby steps and
    4 products take seconds.  Bit-exact against the oracle, and against numpy after decryption."""
    w = wl.BY_NAME["ccmm96"]
    p = Pair(w.param_tuple())
    l1, d, m, period = p.pr.L, 4, 1, 4
    A = p.rng.uniform(-1, 1, (p.n, d))
    Bm = p.rng.uniform(-1, 1, (d, m))
    o_gks, g_gk = doubling_keys(p, period)
    o_rk, g_rk = relin_keys(p)
    zb = np.zeros((m, p.n))
    zb[:, :d] = Bm.T
    o_a, g_a = p.encrypt_both(A.T, l1)
    o_b, g_b = p.encrypt_both(zb, l1)
    masks = p.o.periodic_masks(period, d, l1)
    g_masks = p.ctx.pt_set_scale(p.ctx.pt_import(masks, l1), float(p.pr.q[l1 - 1]))
    out = p.ctx.ccmm(g_rk, g_gk, g_a, g_b, g_masks, period)
    want = p.o.ccmm(o_a, o_b, d, period, o_rk, o_gks)
    assert out.limbs == l1 - 2 and np.array_equal(out.export(), stack_cts(want))
    assert np.abs(p.ctx.decrypt(p.g_sk, out) - (A @ Bm).T).max() < 1e-3
    for h in (g_a, g_b, g_masks, out, g_gk, g_rk):
        h.free()
    p.close()


def heads_case(p, l1, s, d, cols):
    heads = p.n // s
    Q = p.rng.uniform(-1, 1, (heads, s, d))
    K = p.rng.uniform(-1, 1, (heads, s, d))
    za = np.stack([np.concatenate([Q[h][:, j] for h in range(heads)]) for j in range(d)])
    zb = np.stack([np.concatenate([K[h][:, j] for h in range(heads)]) for j in range(d)])
    o_a, g_a = p.encrypt_both(za, l1)
    o_b, g_b = p.encrypt_both(zb, l1)
    steps = sorted(set(c for c in cols if c)) + p.ctx.fill_steps(1, s, -1)
    o_gks, g_gk = p.galois_keys(steps)
    ref = np.stack([np.concatenate([(Q[h] @ K[h].T)[:, i] for h in range(heads)]) for i in cols])
    return o_a, g_a, o_b, g_b, o_gks, g_gk, ref


@pytest.mark.parametrize("params,l1,s,d,cols", [(SMALL4, 6, 64, 5, [0, 1, 63]), (SMALL4, 4, 512, 3, [7]), (WIDE, 4, 128, 18, [5, 0])],
                         ids=["8-heads", "one-head", "wide-primes-two-groups"])
def test_ccmm_blocks_small_ring(params, l1, s, d, cols):
    """Several heads per ciphertext (Q K^T form): bit-exact against the oracle, numpy after decryption."""
    p = Pair(params)
    o_a, g_a, o_b, g_b, o_gks, g_gk, ref = heads_case(p, l1, s, d, cols)
    o_rk, g_rk = relin_keys(p)
    mask0 = p.o.block_start_mask(s, l1)
    g_mask = p.ctx.pt_set_scale(p.ctx.pt_import(mask0[None, :], l1), float(p.pr.q[l1 - 1]))
    out = p.ctx.ccmm_blocks(g_rk, g_gk, g_a, g_b, s, cols, g_mask)
    want = p.o.ccmm_blocks(o_a, o_b, s, cols, o_rk, o_gks)
    assert out.n == len(cols) and out.limbs == l1 - 2
    assert np.array_equal(out.export(), stack_cts(want))
    assert np.abs(p.ctx.decrypt(p.g_sk, out) - ref).max() < 1e-3
    lib = p.ctx.block_start_mask(s, l1)
    out2 = p.ctx.ccmm_blocks(g_rk, g_gk, g_a, g_b, s, cols, lib)
    assert np.abs(p.ctx.decrypt(p.g_sk, out2) - ref).max() < 1e-3
    with pytest.raises(p.binding.EnsiError, match="code -1"):
        p.ctx.ccmm_blocks(g_rk, g_gk, g_a, g_b, s, [s], g_mask, out2 if len(cols) == 1 else None)  # column outside the block
    for h in (g_a, g_b, g_mask, lib, out, out2, g_gk, g_rk):
        h.free()
    p.close()


def test_ccmm_blocks_full_ring():
    """N = 2^16 (fused kernels), 16 heads of 2048 tokens as in the paper's attention shape, a narrow inner
    dimension and a low level so that the oracle's 11 fill steps per element take seconds."""
    p = Pair(KEYSWITCH)
    l1, s, d, cols = 4, 2048, 2, [3, 0]
    o_a, g_a, o_b, g_b, o_gks, g_gk, ref = heads_case(p, l1, s, d, cols)
    o_rk, g_rk = relin_keys(p)
    mask0 = p.o.block_start_mask(s, l1)
    g_mask = p.ctx.pt_set_scale(p.ctx.pt_import(mask0[None, :], l1), float(p.pr.q[l1 - 1]))
    out = p.ctx.ccmm_blocks(g_rk, g_gk, g_a, g_b, s, cols, g_mask)
    want = p.o.ccmm_blocks(o_a, o_b, s, cols, o_rk, o_gks)
    assert np.array_equal(out.export(), stack_cts(want))
    assert np.abs(p.ctx.decrypt(p.g_sk, out) - ref).max() < 1e-3
    for h in (g_a, g_b, g_mask, out, g_gk, g_rk):
        h.free()
    p.close()


def test_ccmm_blocks_at_the_benchmark_parameters():
    """The 16 + 4 limb chain and the 16 x 2048 packing of the ccmmqk benchmark workload, with a narrow inner
    dimension (d = 2, one output column) so that the oracle's 22 fill steps at 15 limbs take seconds."""
    w = wl.BY_NAME["ccmmqk"]
    p = Pair(w.param_tuple())
    l1, s, d, cols = p.pr.L, w.tokens, 2, [5]
    o_a, g_a, o_b, g_b, o_gks, g_gk, ref = heads_case(p, l1, s, d, cols)
    o_rk, g_rk = relin_keys(p)
    mask0 = p.o.block_start_mask(s, l1)
    g_mask = p.ctx.pt_set_scale(p.ctx.pt_import(mask0[None, :], l1), float(p.pr.q[l1 - 1]))
    out = p.ctx.ccmm_blocks(g_rk, g_gk, g_a, g_b, s, cols, g_mask)
    want = p.o.ccmm_blocks(o_a, o_b, s, cols, o_rk, o_gks)
    assert out.limbs == l1 - 2 and np.array_equal(out.export(), stack_cts(want))
    assert np.abs(p.ctx.decrypt(p.g_sk, out) - ref).max() < 1e-3
    for h in (g_a, g_b, g_mask, out, g_gk, g_rk):
        h.free()
    p.close()


# ------------------------------------------------ extraction in giant and baby steps, term lists
def bsgs_keys(p, s, period, slots):
    steps = {sl % period for sl in slots} | {sl // period * period for sl in slots}
    steps |= set(p.ctx.fill_steps(period, s, -1)) | set(p.ctx.fill_steps(1, period, -1))
    return p.galois_keys(sorted(st for st in steps if st))


def bsgs_masks(p, s, period, l1):
    mh = p.ctx.pt_set_scale(p.ctx.pt_import(p.o.block_head_mask(s, period, l1)[None, :], l1), float(p.pr.q[l1 - 1]))
    ms = p.ctx.pt_set_scale(p.ctx.pt_import(p.o.periodic_masks(period, 1, l1 - 1), l1 - 1), float(p.pr.q[l1 - 2]))
    return mh, ms


@pytest.mark.parametrize("params,l1,s,period,d,cols", [(SMALL4, 6, 64, 8, 5, [0, 1, 9, 63, 15]), (SMALL4, 5, 512, 64, 3, [77]),
                                                       (WIDE, 4, 128, 16, 18, [5, 37])],
                         ids=["8-heads", "one-head", "wide-primes-two-groups"])
def test_ccmm_bsgs_qk_form_small_ring(params, l1, s, period, d, cols):
    """Q K^T over heads with the extraction in giant and baby steps: bit-exact against the oracle, numpy after
    decryption; the library's own masks give the same product within the bound."""
    p = Pair(params)
    heads = p.n // s
    Q = p.rng.uniform(-1, 1, (heads, s, d))
    K = p.rng.uniform(-1, 1, (heads, s, d))
    o_a, g_a = p.encrypt_both(np.stack([np.concatenate([Q[h][:, j] for h in range(heads)]) for j in range(d)]), l1)
    o_b, g_b = p.encrypt_both(np.stack([np.concatenate([K[h][:, j] for h in range(heads)]) for j in range(d)]), l1)
    o_gks, g_gk = bsgs_keys(p, s, period, cols)
    o_rk, g_rk = relin_keys(p)
    mh, ms = bsgs_masks(p, s, period, l1)
    terms = [[(j, j, i) for j in range(d)] for i in cols]
    out = p.ctx.ccmm_bsgs(g_rk, g_gk, g_a, g_b, s, period, terms, mh, ms)
    want = p.o.ccmm_bsgs(o_a, o_b, s, period, terms, o_rk, o_gks)
    assert out.n == len(cols) and out.limbs == l1 - 3
    assert np.array_equal(out.export(), stack_cts(want))
    ref = np.stack([np.concatenate([(Q[h] @ K[h].T)[:, i] for h in range(heads)]) for i in cols])
    assert np.abs(p.ctx.decrypt(p.g_sk, out) - ref).max() < 1e-3
    lh, ls = p.ctx.block_head_mask(s, period, l1), p.ctx.periodic_masks(period, 1, l1 - 1)
    out2 = p.ctx.ccmm_bsgs(g_rk, g_gk, g_a, g_b, s, period, terms, lh, ls)
    assert np.abs(p.ctx.decrypt(p.g_sk, out2) - ref).max() < 1e-3
    with pytest.raises(p.binding.EnsiError, match="code -1"):
        p.ctx.ccmm_bsgs(g_rk, g_gk, g_a, g_b, s, period, [[(0, 0, s)]], mh, ms)  # slot outside the block
    with pytest.raises(p.binding.EnsiError, match="code -3"):
        p.ctx.ccmm_bsgs(g_rk, g_gk, g_a, g_b, s, period, terms, ms, ms)  # head mask one level short
    _, g_few = p.galois_keys([1])
    with pytest.raises(p.binding.EnsiError, match="code -2"):
        p.ctx.ccmm_bsgs(g_rk, g_few, g_a, g_b, s, period, [[(0, 0, s - 1)]], mh, ms)  # no key for the giant step
    g_few.free()
    for h in (g_a, g_b, mh, ms, lh, ls, out, out2, g_gk, g_rk):
        h.free()
    p.close()


def test_ccmm_bsgs_weights_times_v_small_ring():
    """The other attention product: out_i = sum_j a_j (x) E(v_i, j) with the s columns of the weights in a and the
    columns of V in b; an output without terms, elements shared between outputs, more than 16 sources per stage."""
    p = Pair(SMALL4)
    l1, s, period, m = 5, 32, 4, 2
    heads = p.n // s
    Wt = p.rng.uniform(-1, 1, (heads, s, s)) / 4
    V = p.rng.uniform(-1, 1, (heads, s, m))
    o_a, g_a = p.encrypt_both(np.stack([np.concatenate([Wt[h][:, j] for h in range(heads)]) for j in range(s)]), l1)
    o_b, g_b = p.encrypt_both(np.stack([np.concatenate([V[h][:, i] for h in range(heads)]) for i in range(m)]), l1)
    o_gks, g_gk = bsgs_keys(p, s, period, range(s))
    o_rk, g_rk = relin_keys(p)
    mh, ms = bsgs_masks(p, s, period, l1)
    # outputs 0, 1: the product; 2: nothing; 3: a sum that reuses elements of output 0 with other columns of a
    terms = [[(j, i, j) for j in range(s)] for i in range(m)] + [[], [(1, 0, 0), (0, 0, 1), (5, 1, 31)]]
    out = p.ctx.ccmm_bsgs(g_rk, g_gk, g_a, g_b, s, period, terms, mh, ms)
    want = p.o.ccmm_bsgs(o_a, o_b, s, period, [t for t in terms if t], o_rk, o_gks)
    got = out.export()
    assert out.limbs == l1 - 3 and np.array_equal(got[[0, 1, 3]], stack_cts(want)) and not got[2].any()
    dec = p.ctx.decrypt(p.g_sk, out)
    for i in range(m):
        assert np.abs(dec[i] - np.concatenate([(Wt[h] @ V[h])[:, i] for h in range(heads)])).max() < 1e-3
    ref3 = np.concatenate([Wt[h][:, 1] * V[h][0, 0] + Wt[h][:, 0] * V[h][1, 0] + Wt[h][:, 5] * V[h][31, 1] for h in range(heads)])
    assert np.abs(dec[3] - ref3).max() < 1e-3
    for h in (g_a, g_b, mh, ms, out, g_gk, g_rk):
        h.free()
    p.close()


def test_ccmm_bsgs_full_ring():
    """N = 2^16 (fused kernels), 16 heads of 2048 tokens, period 16, a narrow inner dimension and a low level so
    that the oracle's fills take seconds; two columns of one segment and one of another."""
    p = Pair(KEYSWITCH)
    l1, s, period, d, cols = 5, 2048, 16, 2, [35, 32, 2047]
    heads = p.n // s
    Q = p.rng.uniform(-1, 1, (heads, s, d))
    K = p.rng.uniform(-1, 1, (heads, s, d))
    o_a, g_a = p.encrypt_both(np.stack([np.concatenate([Q[h][:, j] for h in range(heads)]) for j in range(d)]), l1)
    o_b, g_b = p.encrypt_both(np.stack([np.concatenate([K[h][:, j] for h in range(heads)]) for j in range(d)]), l1)
    o_gks, g_gk = bsgs_keys(p, s, period, cols)
    o_rk, g_rk = relin_keys(p)
    mh, ms = bsgs_masks(p, s, period, l1)
    terms = [[(j, j, i) for j in range(d)] for i in cols]
    out = p.ctx.ccmm_bsgs(g_rk, g_gk, g_a, g_b, s, period, terms, mh, ms)
    want = p.o.ccmm_bsgs(o_a, o_b, s, period, terms, o_rk, o_gks)
    assert out.limbs == l1 - 3 and np.array_equal(out.export(), stack_cts(want))
    ref = np.stack([np.concatenate([(Q[h] @ K[h].T)[:, i] for h in range(heads)]) for i in cols])
    assert np.abs(p.ctx.decrypt(p.g_sk, out) - ref).max() < 1e-3
    for h in (g_a, g_b, mh, ms, out, g_gk, g_rk):
        h.free()
    p.close()


def test_ccmm_bsgs_at_the_benchmark_parameters():
    """The 16 + 4 limb chain and the 16 x 2048 packing of the attention benchmark workloads, period 16, with a
    narrow inner dimension (two terms, one output) so that the oracle's fills at 13 to 15 limbs take seconds."""
    w = wl.BY_NAME["ccmmqk"]
    p = Pair(w.param_tuple())
    l1, s, period, d, cols = p.pr.L, w.tokens, 16, 2, [1029]
    heads = p.n // s
    Q = p.rng.uniform(-1, 1, (heads, s, d))
    K = p.rng.uniform(-1, 1, (heads, s, d))
    o_a, g_a = p.encrypt_both(np.stack([np.concatenate([Q[h][:, j] for h in range(heads)]) for j in range(d)]), l1)
    o_b, g_b = p.encrypt_both(np.stack([np.concatenate([K[h][:, j] for h in range(heads)]) for j in range(d)]), l1)
    o_gks, g_gk = bsgs_keys(p, s, period, cols)
    o_rk, g_rk = relin_keys(p)
    mh, ms = bsgs_masks(p, s, period, l1)
    terms = [[(j, j, i) for j in range(d)] for i in cols]
    out = p.ctx.ccmm_bsgs(g_rk, g_gk, g_a, g_b, s, period, terms, mh, ms)
    want = p.o.ccmm_bsgs(o_a, o_b, s, period, terms, o_rk, o_gks)
    assert out.limbs == l1 - 3 and np.array_equal(out.export(), stack_cts(want))
    ref = np.stack([np.concatenate([(Q[h] @ K[h].T)[:, i] for h in range(heads)]) for i in cols])
    assert np.abs(p.ctx.decrypt(p.g_sk, out) - ref).max() < 1e-3
    for h in (g_a, g_b, mh, ms, out, g_gk, g_rk):
        h.free()
    p.close()


def test_ccmm_bsgs_more_segments_than_are_kept_for_a_call():
    """Period 1 makes every slot its own segment: 40 ciphertexts of 32-slot blocks name 1280 segments, more than the
    library keeps for a whole call, so each group of outputs forms its own; outputs of 430, 430 and 420 elements
    give three groups."""
    p = Pair(SMALL4)
    l1, s, period, nb = 5, 32, 1, 40
    heads = p.n // s
    za = p.rng.uniform(-1, 1, (nb, p.n)) / 8
    zb = p.rng.uniform(-1, 1, (nb, p.n))
    o_a, g_a = p.encrypt_both(za, l1)
    o_b, g_b = p.encrypt_both(zb, l1)
    o_gks, g_gk = bsgs_keys(p, s, period, range(s))
    o_rk, g_rk = relin_keys(p)
    mh, ms = bsgs_masks(p, s, period, l1)
    pairs = [(b, sl) for b in range(nb) for sl in range(s)]
    terms = [[(b, b, sl) for b, sl in pairs[0:430]], [(b, b, sl) for b, sl in pairs[430:860]], [(b, b, sl) for b, sl in pairs[860:1280]]]
    out = p.ctx.ccmm_bsgs(g_rk, g_gk, g_a, g_b, s, period, terms, mh, ms)
    want = p.o.ccmm_bsgs(o_a, o_b, s, period, terms, o_rk, o_gks)
    assert np.array_equal(out.export(), stack_cts(want))
    dec = p.ctx.decrypt(p.g_sk, out)
    for o, tl in enumerate(terms):
        ref = sum(za[b] * np.repeat(zb[b].reshape(heads, s)[:, sl], s) for b, _, sl in tl)
        assert np.abs(dec[o] - ref).max() < 1e-3, o
    for h in (g_a, g_b, mh, ms, out, g_gk, g_rk):
        h.free()
    p.close()


def test_ccmm_forms_share_one_context():
    """The extraction forms, a batched rotation and a plain product run one after the other on one context at
    N = 2^16 (they share its workspaces, which grow and are reused): every result equals the oracle's, and the first
    call repeated at the end gives the same words again."""
    p = Pair(KEYSWITCH)
    l1, s, period, d, cols = 5, 2048, 16, 2, [35, 2047]
    heads = p.n // s
    Q = p.rng.uniform(-1, 1, (heads, s, d))
    K = p.rng.uniform(-1, 1, (heads, s, d))
    o_a, g_a = p.encrypt_both(np.stack([np.concatenate([Q[h][:, j] for h in range(heads)]) for j in range(d)]), l1)
    o_b, g_b = p.encrypt_both(np.stack([np.concatenate([K[h][:, j] for h in range(heads)]) for j in range(d)]), l1)
    steps = {sl % period for sl in cols} | {sl // period * period for sl in cols} | set(cols)
    steps |= set(p.ctx.fill_steps(period, s, -1)) | set(p.ctx.fill_steps(1, period, -1)) | set(p.ctx.fill_steps(1, s, -1))
    o_gks, g_gk = p.galois_keys(sorted(st for st in steps if st))
    o_rk, g_rk = relin_keys(p)
    mh, ms = bsgs_masks(p, s, period, l1)
    m0 = p.ctx.pt_set_scale(p.ctx.pt_import(p.o.block_start_mask(s, l1)[None, :], l1), float(p.pr.q[l1 - 1]))
    terms = [[(j, j, i) for j in range(d)] for i in cols]
    first = p.ctx.ccmm_bsgs(g_rk, g_gk, g_a, g_b, s, period, terms, mh, ms).export()
    assert np.array_equal(first, stack_cts(p.o.ccmm_bsgs(o_a, o_b, s, period, terms, o_rk, o_gks)))
    rot = p.ctx.rotate(g_gk, g_a, [cols[0], -1])
    assert np.array_equal(rot.export(), stack_cts([p.o.rotate(o_a[0], o_gks[cols[0]]), p.o.rotate(o_a[1], o_gks[-1])]))
    blocks = p.ctx.ccmm_blocks(g_rk, g_gk, g_a, g_b, s, cols, m0)
    assert np.array_equal(blocks.export(), stack_cts(p.o.ccmm_blocks(o_a, o_b, s, cols, o_rk, o_gks)))
    prod = p.ctx.mult_sum_relin_rescale(g_rk, g_a, g_b, [0, 2], [0, 1], [0, 1])
    assert np.array_equal(prod.export(), stack_cts([p.o.mult_sum_relin_rescale([(o_a[0], o_b[0]), (o_a[1], o_b[1])], o_rk)]))
    again = p.ctx.ccmm_bsgs(g_rk, g_gk, g_a, g_b, s, period, terms, mh, ms)
    assert np.array_equal(again.export(), first)
    for h in (g_a, g_b, mh, ms, m0, rot, blocks, prod, again, g_gk, g_rk):
        h.free()
    p.close()


# ------------------------------------------------ a whole segment of columns from its diagonals
def segment_case(p, l1, s, period, baby, d, g):
    heads = p.n // s
    Q = p.rng.uniform(-1, 1, (heads, s, d))
    K = p.rng.uniform(-1, 1, (heads, s, d))
    o_a, g_a = p.encrypt_both(np.stack([np.concatenate([Q[h][:, j] for h in range(heads)]) for j in range(d)]), l1)
    o_b, g_b = p.encrypt_both(np.stack([np.concatenate([K[h][:, j] for h in range(heads)]) for j in range(d)]), l1)
    giant = {k * baby for k in range(1, period // baby + 1)}
    steps = set(range(1, baby)) | giant | {-t for t in giant} | {g * period} | set(p.ctx.fill_steps(period, s, -1))
    o_gks, g_gk = p.galois_keys(sorted(st for st in steps if st))
    mh = p.ctx.pt_set_scale(p.ctx.pt_import(p.o.block_head_mask(s, period, l1)[None, :], l1), float(p.pr.q[l1 - 1]))
    ms = p.ctx.pt_set_scale(p.ctx.pt_import(p.o.segment_masks(s, period, l1 - 2), l1 - 2), float(p.pr.q[l1 - 3]))
    ref = np.stack([np.concatenate([(Q[h] @ K[h].T)[:, g * period + c] for h in range(heads)]) for c in range(period)])
    return o_a, g_a, o_b, g_b, o_gks, g_gk, mh, ms, ref


@pytest.mark.parametrize("params,l1,s,period,baby,d,g", [(SMALL4, 6, 64, 8, 2, 5, 3), (SMALL4, 5, 512, 4, 4, 3, 0), (SMALL4, 5, 16, 16, 4, 2, 0),
                                                         (SMALL4, 5, 64, 8, 1, 2, 7), (WIDE, 4, 128, 16, 4, 18, 7)],
                         ids=["8-heads", "one-head-first-segment-baby-steps-only", "segment-is-the-block", "giant-steps-only",
                              "wide-primes-two-groups"])
def test_ccmm_segment_small_ring(params, l1, s, period, baby, d, g):
    """A segment of output columns from its diagonals: bit-exact against the oracle, numpy after decryption; the
    library's own masks give the same product within the bound."""
    p = Pair(params)
    o_a, g_a, o_b, g_b, o_gks, g_gk, mh, ms, ref = segment_case(p, l1, s, period, baby, d, g)
    o_rk, g_rk = relin_keys(p)
    out = p.ctx.ccmm_segment(g_rk, g_gk, g_a, g_b, s, period, baby, g, mh, ms)
    want = p.o.ccmm_segment(o_a, o_b, s, period, baby, g, o_rk, o_gks)
    assert out.n == period and out.limbs == l1 - 3
    assert np.array_equal(out.export(), stack_cts(want))
    assert np.abs(p.ctx.decrypt(p.g_sk, out) - ref).max() < 1e-3
    # the columns of A moved by their giant steps once, outside the call (as ciphertexts, then left in the transform domain)
    for prepare in (False, True):
        ap = p.ctx.ccmm_left_giant_steps(g_gk, g_a, period, baby, prepare=prepare)
        assert ap.n == d * (2 * period - 1 if baby == 1 else 2 * period // baby) and ap.limbs == l1 - 1
        outp = p.ctx.ccmm_segment(g_rk, g_gk, ap, g_b, s, period, baby, g, mh, ms)
        assert np.array_equal(outp.export(), stack_cts(want)), prepare
        ap.free()
        outp.free()
    lh, ls = p.ctx.block_head_mask(s, period, l1), p.ctx.segment_masks(s, period, l1 - 2)
    out2 = p.ctx.ccmm_segment(g_rk, g_gk, g_a, g_b, s, period, baby, g, lh, ls)
    assert np.abs(p.ctx.decrypt(p.g_sk, out2) - ref).max() < 1e-3
    with pytest.raises(p.binding.EnsiError, match="code -1"):
        p.ctx.ccmm_segment(g_rk, g_gk, g_a, g_b, s, period, baby, s // period, mh, ms, out2)  # segment outside the block
    with pytest.raises(p.binding.EnsiError, match="code -3"):
        p.ctx.ccmm_segment(g_rk, g_gk, g_a, g_b, s, period, baby, g, ms, ms, out2)  # head mask two levels short
    for h in (g_a, g_b, mh, ms, lh, ls, out, out2, g_gk, g_rk):
        h.free()
    p.close()


@pytest.mark.parametrize("period,baby,g", [(4, 2, 511), (4, 1, 0), (8, 4, 255)], ids=["grid-4x2", "grid-7x1", "grid-4x4"])
def test_ccmm_segment_full_ring(period, baby, g):
    """N = 2^16 (fused kernels, the tiled multiply-add over the grid of giant and baby steps: one whole tile, a ragged
    one, several), 16 heads of 2048 tokens, a narrow inner dimension and a low level."""
    p = Pair(KEYSWITCH)
    l1, s, d = 5, 2048, 2
    o_a, g_a, o_b, g_b, o_gks, g_gk, mh, ms, ref = segment_case(p, l1, s, period, baby, d, g)
    o_rk, g_rk = relin_keys(p)
    out = p.ctx.ccmm_segment(g_rk, g_gk, g_a, g_b, s, period, baby, g, mh, ms)
    want = p.o.ccmm_segment(o_a, o_b, s, period, baby, g, o_rk, o_gks)
    assert out.limbs == l1 - 3 and np.array_equal(out.export(), stack_cts(want))
    assert np.abs(p.ctx.decrypt(p.g_sk, out) - ref).max() < 1e-3
    ap = p.ctx.ccmm_left_giant_steps(g_gk, g_a, period, baby, prepare=True)  # columns of A moved once, in the transform domain
    outp = p.ctx.ccmm_segment(g_rk, g_gk, ap, g_b, s, period, baby, g, mh, ms)
    assert np.array_equal(outp.export(), stack_cts(want))
    for h in (g_a, g_b, mh, ms, out, ap, outp, g_gk, g_rk):
        h.free()
    p.close()


def test_ccmm_segment_at_the_benchmark_parameters():
    """The 16 + 4 limb chain and the 16 x 2048 packing of the benchmark workload with a narrow inner dimension (d = 2),
    at period 16 in baby steps of 4 (the benchmark runs 32 and 8, whose 1536 sorting products take the oracle a minute)."""
    w = wl.BY_NAME["ccmmqk"]
    p = Pair(w.param_tuple())
    l1, s, period, baby, d, g = p.pr.L, w.tokens, 16, 4, 2, 64
    o_a, g_a, o_b, g_b, o_gks, g_gk, mh, ms, ref = segment_case(p, l1, s, period, baby, d, g)
    o_rk, g_rk = relin_keys(p)
    out = p.ctx.ccmm_segment(g_rk, g_gk, g_a, g_b, s, period, baby, g, mh, ms)
    want = p.o.ccmm_segment(o_a, o_b, s, period, baby, g, o_rk, o_gks)
    assert out.limbs == l1 - 3 and np.array_equal(out.export(), stack_cts(want))
    assert np.abs(p.ctx.decrypt(p.g_sk, out) - ref).max() < 1e-3
    for h in (g_a, g_b, mh, ms, out, g_gk, g_rk):
        h.free()
    p.close()


# ------------------------------------------------ weights times V from diagonalised weights
def av_case(p, l1, s, period, baby, g0, n_seg, m):
    heads = p.n // s
    lo, hi = g0 * period, (g0 + n_seg) * period
    Wt = p.rng.uniform(-1, 1, (heads, s, s)) / 8
    V = p.rng.uniform(-1, 1, (heads, s, m))
    o_a, g_a = p.encrypt_both(np.stack([np.concatenate([Wt[h][:, j] for h in range(heads)]) for j in range(lo, hi)]), l1)
    o_v, g_v = p.encrypt_both(np.stack([np.concatenate([V[h][:, i] for h in range(heads)]) for i in range(m)]), l1)
    giant = {k * baby for k in range(1, period // baby + 1)}
    steps = set(range(1, baby)) | giant | {-t for t in giant} | {(g0 + k) * period for k in range(n_seg)} | set(p.ctx.fill_steps(period, s, -1))
    o_gks, g_gk = p.galois_keys(sorted(st for st in steps if st))
    mh = p.ctx.pt_set_scale(p.ctx.pt_import(p.o.block_head_mask(s, period, l1)[None, :], l1), float(p.pr.q[l1 - 1]))
    ms = p.ctx.pt_set_scale(p.ctx.pt_import(p.o.segment_masks(s, period, l1), l1), float(p.pr.q[l1 - 1]))
    ref = np.stack([np.concatenate([Wt[h][:, lo:hi] @ V[h][lo:hi, i] for h in range(heads)]) for i in range(m)])
    return o_a, g_a, o_v, g_v, o_gks, g_gk, mh, ms, ref


@pytest.mark.parametrize("params,l1,s,period,baby,g0,n_seg,m", [(SMALL4, 5, 32, 4, 2, 0, 8, 2), (SMALL4, 4, 64, 8, 8, 2, 3, 3),
                                                                (SMALL4, 4, 64, 8, 1, 1, 2, 1), (WIDE, 4, 128, 16, 4, 5, 2, 1),
                                                                (SMALL4, 4, 512, 8, 2, 0, 1, 2)],
                         ids=["whole-block", "some-segments-baby-steps-only", "giant-steps-only", "wide-primes", "one-head-one-segment"])
def test_ccmm_av_small_ring(params, l1, s, period, baby, g0, n_seg, m):
    """Diagonalised weights and the weights-times-V product: bit-exact against the oracle, numpy after decryption;
    the library's own masks give the same product within the bound."""
    p = Pair(params)
    o_a, g_a, o_v, g_v, o_gks, g_gk, mh, ms, ref = av_case(p, l1, s, period, baby, g0, n_seg, m)
    o_rk, g_rk = relin_keys(p)
    ad = p.ctx.diagonalise_weights(g_gk, g_a, s, period, baby, ms)
    o_ad = [p.o.diagonalise_weights(o_a[k * period:(k + 1) * period], s, period, baby, o_gks) for k in range(n_seg)]
    assert ad.n == n_seg * (2 * period - 1) and ad.limbs == l1 - 1
    assert np.array_equal(ad.export(), stack_cts([c for seg in o_ad for c in seg]))
    out = p.ctx.ccmm_av(g_rk, g_gk, ad, g_v, s, period, baby, g0, mh)
    want = p.o.ccmm_av(o_ad, o_v, s, period, baby, g0, o_rk, o_gks)
    assert out.n == m and out.limbs == l1 - 2
    assert np.array_equal(out.export(), stack_cts(want))
    assert np.abs(p.ctx.decrypt(p.g_sk, out) - ref).max() < 1e-3
    # the weights left in the transform domain: the same words come out
    adp = p.ctx.diagonalise_weights(g_gk, g_a, s, period, baby, ms, prepare=True)
    outp = p.ctx.ccmm_av(g_rk, g_gk, adp, g_v, s, period, baby, g0, mh)
    assert np.array_equal(outp.export(), stack_cts(want))
    with pytest.raises(p.binding.EnsiError, match="code -1"):
        adp.export()
    with pytest.raises(p.binding.EnsiError, match="code -1"):
        p.ctx.mult_sum_relin_rescale(g_rk, adp, adp, [0, 1], [0], [0])  # prepared weights are no ciphertexts
    adp.free()
    outp.free()
    lh, ls = p.ctx.block_head_mask(s, period, l1), p.ctx.segment_masks(s, period, l1)
    ad2 = p.ctx.diagonalise_weights(g_gk, g_a, s, period, baby, ls)
    out2 = p.ctx.ccmm_av(g_rk, g_gk, ad2, g_v, s, period, baby, g0, lh)
    assert np.abs(p.ctx.decrypt(p.g_sk, out2) - ref).max() < 1e-3
    with pytest.raises(p.binding.EnsiError, match="code -1"):
        p.ctx.ccmm_av(g_rk, g_gk, ad, g_v, s, period, baby, s // period - n_seg + 1, mh, out2)  # last segment outside the block
    shallow = p.ctx.ct_alloc(m, l1 - 1)
    with pytest.raises(p.binding.EnsiError, match="code -3"):
        p.ctx.ccmm_av(g_rk, g_gk, ad, g_v, s, period, baby, g0, mh, shallow)  # output one level below V instead of two
    with pytest.raises(p.binding.EnsiError, match="code -4"):
        p.ctx.diagonalise_weights(g_gk, g_a, s, period, baby, ms, shallow)  # output batch of the wrong size
    for h in (g_a, g_v, mh, ms, lh, ls, ad, ad2, out, out2, shallow, g_gk, g_rk):
        h.free()
    p.close()


def test_ccmm_av_full_ring():
    """N = 2^16 (fused kernels), 16 heads of 2048 tokens, period 4 in baby steps of 2, two segments in the middle of the
    block, a low level."""
    p = Pair(KEYSWITCH)
    l1, s, period, baby, g0, n_seg, m = 4, 2048, 4, 2, 100, 2, 1
    o_a, g_a, o_v, g_v, o_gks, g_gk, mh, ms, ref = av_case(p, l1, s, period, baby, g0, n_seg, m)
    o_rk, g_rk = relin_keys(p)
    ad = p.ctx.diagonalise_weights(g_gk, g_a, s, period, baby, ms)
    o_ad = [p.o.diagonalise_weights(o_a[k * period:(k + 1) * period], s, period, baby, o_gks) for k in range(n_seg)]
    assert np.array_equal(ad.export(), stack_cts([c for seg in o_ad for c in seg]))
    out = p.ctx.ccmm_av(g_rk, g_gk, ad, g_v, s, period, baby, g0, mh)
    want = p.o.ccmm_av(o_ad, o_v, s, period, baby, g0, o_rk, o_gks)
    assert out.limbs == l1 - 2 and np.array_equal(out.export(), stack_cts(want))
    assert np.abs(p.ctx.decrypt(p.g_sk, out) - ref).max() < 1e-3
    adp = p.ctx.diagonalise_weights(g_gk, g_a, s, period, baby, ms, prepare=True)  # weights left in the transform domain
    outp = p.ctx.ccmm_av(g_rk, g_gk, adp, g_v, s, period, baby, g0, mh)
    assert np.array_equal(outp.export(), stack_cts(want))
    for h in (g_a, g_v, mh, ms, ad, adp, out, outp, g_gk, g_rk):
        h.free()
    p.close()


def test_ccmm_av_at_the_benchmark_parameters():
    """The 16 + 4 limb chain and the 16 x 2048 packing of the benchmark workload on one segment, at period 16 in baby
    steps of 4 (the benchmark runs 32 and 8, whose 3000 diagonalising products take the oracle a minute)."""
    w = wl.BY_NAME["ccmmqk"]
    p = Pair(w.param_tuple())
    l1, s, period, baby, g0, n_seg, m = p.pr.L, w.tokens, 16, 4, 127, 1, 1
    o_a, g_a, o_v, g_v, o_gks, g_gk, mh, ms, ref = av_case(p, l1, s, period, baby, g0, n_seg, m)
    o_rk, g_rk = relin_keys(p)
    ad = p.ctx.diagonalise_weights(g_gk, g_a, s, period, baby, ms)
    o_ad = [p.o.diagonalise_weights(o_a, s, period, baby, o_gks)]
    assert np.array_equal(ad.export(), stack_cts(o_ad[0]))
    out = p.ctx.ccmm_av(g_rk, g_gk, ad, g_v, s, period, baby, g0, mh)
    want = p.o.ccmm_av(o_ad, o_v, s, period, baby, g0, o_rk, o_gks)
    assert out.limbs == l1 - 2 and np.array_equal(out.export(), stack_cts(want))
    assert np.abs(p.ctx.decrypt(p.g_sk, out) - ref).max() < 1e-3
    adp = p.ctx.diagonalise_weights(g_gk, g_a, s, period, baby, ms, prepare=True)
    outp = p.ctx.ccmm_av(g_rk, g_gk, adp, g_v, s, period, baby, g0, mh)
    assert np.array_equal(outp.export(), stack_cts(want))
    for h in (g_a, g_v, mh, ms, ad, adp, out, outp, g_gk, g_rk):
        h.free()
    p.close()
