"""Parity at the full sizes of the BitNet-shaped workloads, in the launch configuration
the benchmark times.  The oracle cannot run these workloads whole, so it computes sampled
outputs:

  * scalar-multiply + rescale and the Alg. 1 signed sums are word-wise operations, so the
    oracle evaluates them on a sample of word positions of every operand (an Oracle built on
    the same primes with a short ring of sampled words) and the sampled output words must
    match bit for bit;
  * the unpack rotations are exposed through a weight matrix with a single +-1 per output
    column: that output then is one rotated input, which the oracle computes for a sample
    of outputs (one Galois key each);
  * with the workload's own weights the decrypted outputs must match the float64 product
    and the two accumulate kernels must agree.
"""
import numpy as np
import pytest

import workloads as wl
from helpers import Pair, stack_cts
from oracle import Oracle, Params
from oracle.ckks import Ciphertext

pytestmark = pytest.mark.gpu


def sample_positions(N):
    """192 words at each end and 128 around the middle of every limb row: 512 positions."""
    return np.concatenate([np.arange(0, 192), np.arange(N // 2 - 64, N // 2 + 64), np.arange(N - 192, N)])


@pytest.mark.parametrize("name", ["ffn2560", "paperffn"])
def test_ffn_rescale_and_down_projection_full_size(name):
    """FFN workloads, second half: the d_mid ciphertexts at 16 limbs (6912 for the BitNet shape, 4096 for the
    paper's) are multiplied by kappa and rescaled, then contracted with the d_mid x d_out ternary matrix (zero
    placement, one column per ciphertext).  Inputs are synthetic residue words (not encryptions: parity is on
    RNS words), generated identically by torch on the device and numpy on the host."""
    import torch
    from paper_2509_09424_amd import binding
    w = wl.BY_NAME[name]
    rng = wl.rng_for(w.index)
    wl.ternary_weights(rng, w.d_in, w.d_mid)  # same draw order as the benchmark
    wl.activations(rng, w.tokens, w.d_in, w.act)
    W2 = wl.ternary_weights(rng, w.d_mid, w.d_out)
    ctx = binding.Context(*w.param_tuple(), seed=3)
    N, L, d, m = w.N, w.q_count, w.d_mid, w.d_out
    words = 2 * L * N
    bits = w.q_bits - 1
    try:
        # device side: operand v, word index = position inside its [2][L][N] block
        mid_t = torch.empty((d, words), dtype=torch.int64, device="cuda")
        widx = torch.arange(words, dtype=torch.int64, device="cuda")[None, :]
        for v0 in range(0, d, 64):
            v = torch.arange(v0, min(v0 + 64, d), dtype=torch.int64, device="cuda")[:, None]
            mid_t[v0:v0 + v.shape[0]] = wl.synthetic_words(v, widx, bits)
        torch.cuda.synchronize()
        mid = ctx.ct_wrap(mid_t.data_ptr(), d, L, 2.0 ** w.log_scale)
        ctx.mul_scalar_rescale(mid, w.kappa)
        assert mid.limbs == L - 1
        out_t = torch.empty(m * 2 * (L - 1) * N, dtype=torch.int64, device="cuda")
        out = ctx.ct_wrap(out_t.data_ptr(), m, L - 1, 1.0)
        ctx.ternary_matmul(None, mid, w.n_slots, d, W2, "zero", out)
        torch.cuda.synchronize()
        assert out.limbs == L - 1 and out.n == m

        # oracle side: sampled words of every operand, 16 operands side by side per call
        pos = sample_positions(N)
        S = len(pos)
        per_call = 16
        qs, ps = ctx.primes()
        pr = Params(13, w.q_bits, L, w.p_bits, w.p_count, w.alpha, w.log_scale, q=qs, p=ps)
        o = Oracle(pr)
        assert o.N == S * per_call
        row = (np.arange(2 * L, dtype=np.uint64)[:, None] * np.uint64(N) + pos.astype(np.uint64)[None, :])  # [2L][S] word indices
        resc = np.empty((d, 2, L - 1, S), dtype=np.uint64)
        scale_out = None
        for v0 in range(0, d, per_call):
            vs = np.arange(v0, v0 + per_call, dtype=np.uint64)  # d is a multiple of 16
            with np.errstate(over="ignore"):
                x = wl.synthetic_words(vs[:, None, None], row[None, :, :], bits)  # [16][2L][S]
            x = x.reshape(per_call, 2, L, S).transpose(1, 2, 0, 3).reshape(2, L, per_call * S)
            r = o.mul_scalar_rescale(Ciphertext(np.ascontiguousarray(x[0]), np.ascontiguousarray(x[1]), 2.0 ** w.log_scale), w.kappa)
            scale_out = r.scale
            resc[v0:v0 + per_call] = r.limbs().reshape(2, L - 1, per_call, S).transpose(2, 0, 1, 3)
        assert d % per_call == 0
        assert abs(mid.scale / scale_out - 1) < 1e-12

        # the rescaled operands themselves (a sample of them, read back from the device buffer)
        mid_view = mid_t.view(d, 2, L, N)
        for v in (0, 1, d // 2 - 1, d - 1):
            got = mid_view[v, :, :L - 1, :].cpu().numpy().astype(np.uint64)[:, :, pos]
            assert np.array_equal(got, resc[v]), "rescaled operand %d" % v

        # sampled outputs of the contraction: first/last of a 256-output tile, first/last overall, a middle one
        o_s = Oracle(Params(9, w.q_bits, L, w.p_bits, w.p_count, w.alpha, w.log_scale, q=pr.q, p=pr.p))
        assert o_s.N == S
        n_o, limbs_o, scale_o, base_o = out._info()
        ct_words = 2 * limbs_o * N
        for i in (0, 255, 256, m // 2 - 1, m - 1):
            one = ctx.ct_wrap(int(base_o) + 8 * ct_words * i, 1, limbs_o, scale_o)
            got = one.export()[0][:, :, pos]
            one.free()
            nz = np.nonzero(W2[:, i])[0]
            terms = [(Ciphertext(resc[v, 0], resc[v, 1], 1.0), int(W2[v, i])) for v in nz]
            want = o_s.accumulate(terms, L - 1, 1.0).limbs()
            assert np.array_equal(got, want), "output %d" % i
        # the same two steps as one call (rescale applied while the accumulate reads its operands): every output
        # word must equal the two-step result
        out.free()
        mid.free()
        for v0 in range(0, d, 64):
            v = torch.arange(v0, min(v0 + 64, d), dtype=torch.int64, device="cuda")[:, None]
            mid_t[v0:v0 + v.shape[0]] = wl.synthetic_words(v, widx, bits)
        torch.cuda.synchronize()
        mid = ctx.ct_wrap(mid_t.data_ptr(), d, L, 2.0 ** w.log_scale)
        out2_t = torch.empty_like(out_t)
        out2 = ctx.ct_wrap(out2_t.data_ptr(), m, L - 1, 1.0)
        ctx.rescale_ternary_matmul(mid, w.kappa, W2, out2)
        torch.cuda.synchronize()
        assert mid.limbs == L - 1 and abs(out2.scale / scale_out - 1) < 1e-12
        assert torch.equal(out2_t, out_t), "fused rescale + matmul differs from the two-step result"
        out2.free()
        mid.free()
    finally:
        ctx.close()
        # hand the 180 GB of test tensors back to the device (the library allocates outside torch's pool)
        mid_t = out_t = out2_t = widx = None
        torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["proj768", "attn2560", "paper1536", "paper1536n14"])
def test_projection_full_size(name):
    """Projection workloads at full size -- the 768 x 768 projection (32 tokens, one packed input, 1023 Galois keys),
    the attention projection (128 tokens, 2560 x 2560, 10 packed inputs, 255 Galois keys) and the paper's QKV shape (2048 tokens, 1536 x 1536; 96 packed inputs and 15 keys at N = 2^16,
    384 packed inputs and 3 keys at the paper's default ring N = 2^14, where the unfused kernels run), diagonal
    placement: unpack rotations against the oracle on sampled outputs, then the workload's own weights."""
    w = wl.BY_NAME[name]
    p = Pair(w.param_tuple())
    try:
        rng = wl.rng_for(w.index)
        W = wl.ternary_weights(rng, w.d_in, w.d_out)
        X = wl.activations(rng, w.tokens, w.d_in, w.act)
        s, d, m, c_tot = w.tokens, w.d_in, w.d_out, w.c_tot
        L, beta = p.pr.L, p.pr.beta(p.pr.L)
        packed = wl.pack_columns(X, p.n)
        o_cts, g_ct = p.encrypt_both(packed, L)
        steps = [r * s for r in range(1, c_tot)]
        e = wl.error_poly(p.rng, (len(steps), beta, p.N))
        g_gk = p.ctx.galois_keygen(p.g_sk, steps, e, 99)

        # one +-1 per output column, every input column used once: output i is a rotated input
        src = (np.arange(m) * 7 + 3) % d
        sign = np.where(np.arange(m) % 3 == 0, -1, 1).astype(np.int8)
        Wsel = np.zeros((d, m), dtype=np.int8)
        Wsel[src, np.arange(m)] = sign
        out = p.ctx.ternary_matmul(g_gk, g_ct, s, d, Wsel, "diagonal")
        n_o, limbs_o, scale_o, base_o = out._info()
        ct_words = 2 * limbs_o * p.N
        q = np.array(p.pr.q[:L], dtype=np.uint64)[None, :, None]
        digits = {}
        for i in (0, 1, min(1000, m - 2), m - 1):
            G, b = int(src[i]) // c_tot, int(src[i]) % c_tot
            rho = (b - i % c_tot) % c_tot  # the input's block b has to land in block i % c_tot
            if rho:
                gk = p.o.galois_keygen(p.o_sk, rho * s, e[rho - 1], 99)
                if G not in digits:
                    digits[G] = p.o.mod_up(o_cts[G].c1)
                want = p.o.rotate_from_digits(o_cts[G].c0, digits[G], gk, o_cts[G].scale).limbs()
            else:
                want = o_cts[G].limbs()
            if sign[i] < 0:
                want = (q - want) % q
            one = p.ctx.ct_wrap(int(base_o) + 8 * ct_words * i, 1, limbs_o, scale_o)
            got = one.export()[0]
            one.free()
            assert np.array_equal(got, want), "output %d (input %d rotated by %d blocks)" % (i, G, rho)

        # the workload's own weights: decrypted sample against the float64 product, and the
        # matrix-core kernel against the plain-ALU kernel on the same sample
        sample = [i for i in (0, 1, 255, 256, 1279) if i < m - 1] + [m - 1]
        ref = X @ W.astype(np.float64)
        got = {}
        for mode in (2, 1):
            p.ctx.set_accumulate_mode(mode)
            p.ctx.ternary_matmul(g_gk, g_ct, s, d, W, "diagonal", out)
            for i in sample:
                one = p.ctx.ct_wrap(int(base_o) + 8 * ct_words * i, 1, limbs_o, scale_o)
                if mode == 2:
                    got[i] = one.export()[0]
                    dec = p.ctx.decrypt(p.g_sk, one, (i % c_tot) * s, s)[0]
                    assert np.abs(dec - ref[:, i]).max() < 1e-3, "output %d" % i
                else:
                    assert np.array_equal(one.export()[0], got[i]), "kernels disagree on output %d" % i
                one.free()
        p.ctx.set_accumulate_mode(0)
        out.free()
        g_ct.free()
        g_gk.free()
    finally:
        p.close()


def test_rope_full_size():
    """Alg. 2 at the shape the benchmark times (rope1536: 96 packed ciphertexts at 16 limbs, three groups of the
    batched rotation): a sample of the outputs against the oracle bit for bit, all of them after decryption."""
    w = wl.BY_NAME["rope1536"]
    p = Pair(w.param_tuple())
    try:
        L = p.pr.L
        n_ct = -(-w.d_in // w.c_tot)
        rng = wl.rng_for(w.index)
        x = rng.uniform(-1.0, 1.0, size=(n_ct, p.n))
        theta = rng.uniform(0.0, 2.0 * np.pi, p.n // 2)
        cos, sin = np.repeat(np.cos(theta), 2), np.repeat(np.sin(theta), 2)
        want = np.empty_like(x)
        want[:, 0::2] = x[:, 0::2] * cos[0::2] - x[:, 1::2] * sin[0::2]
        want[:, 1::2] = x[:, 1::2] * cos[1::2] + x[:, 0::2] * sin[1::2]
        o_gks, g_gk = p.galois_keys([1, -1])
        o_cts, g_ct = p.encrypt_both(x, L)
        pts = p.o.rope_plaintexts(cos, sin, L)
        g_pt = p.ctx.pt_set_scale(p.ctx.pt_import(pts, L), float(p.pr.q[L - 1]))
        out = p.ctx.rope(g_gk, g_ct, g_pt)
        assert out.n == n_ct and out.limbs == L - 1
        n_o, limbs_o, scale_o, base_o = out._info()
        ct_words = 2 * limbs_o * p.N
        for i in (0, 31, 32, n_ct - 1):
            one = p.ctx.ct_wrap(int(base_o) + 8 * ct_words * i, 1, limbs_o, scale_o)
            got = one.export()[0]
            one.free()
            assert np.array_equal(got, p.o.rope(o_cts[i], pts, o_gks[1], o_gks[-1]).limbs()), "ciphertext %d" % i
        assert np.abs(p.ctx.decrypt(p.g_sk, out) - want).max() < 1e-3
        for h in (g_ct, g_pt, out, g_gk):
            h.free()
    finally:
        p.close()


def test_merge_full_size():
    """The merge at the shape the benchmark times (merge1536: 1536 block-placed outputs at 16 limbs into 96 packed
    ciphertexts, three groups of 32 outputs).  Inputs are synthetic residue words generated identically on the
    device and on the host; a sample of packed outputs is compared with the oracle bit for bit."""
    import torch
    from paper_2509_09424_amd import binding
    w = wl.BY_NAME["merge1536"]
    ctx = binding.Context(*w.param_tuple(), seed=3)
    N, L, m, c_tot, s = w.N, w.q_count, w.d_in, w.c_tot, w.tokens
    words = 2 * L * N
    bits = w.q_bits - 1
    try:
        in_t = torch.empty((m, words), dtype=torch.int64, device="cuda")
        widx = torch.arange(words, dtype=torch.int64, device="cuda")[None, :]
        for v0 in range(0, m, 64):
            v = torch.arange(v0, min(v0 + 64, m), dtype=torch.int64, device="cuda")[:, None]
            in_t[v0:v0 + v.shape[0]] = wl.synthetic_words(v, widx, bits)
        torch.cuda.synchronize()
        qs, ps = ctx.primes()
        pr = Params(w.log_n, w.q_bits, L, w.p_bits, w.p_count, w.alpha, w.log_scale, q=qs, p=ps)
        o = Oracle(pr)
        masks = o.block_masks(s, c_tot, L)
        ql = float(qs[L - 1])
        g_masks = ctx.pt_set_scale(ctx.pt_import(masks, L), ql)
        src = ctx.ct_wrap(in_t.data_ptr(), m, L, 2.0 ** w.log_scale)
        out = ctx.merge(src, g_masks, c_tot)
        torch.cuda.synchronize()
        assert out.n == m // c_tot and out.limbs == L - 1 and abs(out.scale / 2.0 ** w.log_scale - 1) < 1e-12
        n_o, limbs_o, scale_o, base_o = out._info()
        ct_words = 2 * limbs_o * N
        rns = [o.i64_to_rns(mk, pr.q[:L]) for mk in masks]
        hidx = np.arange(words, dtype=np.uint64)
        for G in (0, 31, 32, m // c_tot - 1):
            terms = []
            for b in range(c_tot):
                with np.errstate(over="ignore"):
                    x = wl.synthetic_words(np.uint64(G * c_tot + b), hidx, bits).reshape(2, L, N)
                terms.append((Ciphertext(np.ascontiguousarray(x[0]), np.ascontiguousarray(x[1]), 1.0), rns[b]))
            want = o.pmult_sum_rescale(terms, ql).limbs()
            one = ctx.ct_wrap(int(base_o) + 8 * ct_words * G, 1, limbs_o, scale_o)
            got = one.export()[0]
            one.free()
            assert np.array_equal(got, want), "packed output %d" % G
        for h in (src, out, g_masks):
            h.free()
    finally:
        ctx.close()
        in_t = widx = None
        torch.cuda.empty_cache()
