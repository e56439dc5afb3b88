"""The allocation-free rotation (ensi_rotate_static) against ensi_rotate: the same words, on calls in a row that
share the statically linked workspace -- the second with a smaller input, so that what the first call left behind
must not leak into it -- and the stated size limit."""
import numpy as np
import pytest

import workloads as wl
from helpers import Pair

pytestmark = pytest.mark.gpu

SMALL3 = (10, 50, 5, 60, 3, 3, 40)
KEYSWITCH = wl.WORKLOADS[1].param_tuple()


def _both(p, g_gk, z, limbs, steps):
    _, g_ct = p.encrypt_both(z, limbs)
    want = p.ctx.rotate(g_gk, g_ct, steps)
    got = p.ctx.ct_alloc(g_ct.n, limbs)
    p.ctx.rotate_static(g_gk, g_ct, steps, got)
    a, b = got.export(), want.export()
    for h in (g_ct, want, got):
        h.free()
    return a, b


@pytest.mark.parametrize("params", [SMALL3, wl.WORKLOADS[0].param_tuple()], ids=["fused-free-ring", "tiny"])
def test_rotate_static_two_calls_in_a_row_small_rings(params):
    p = Pair(params)
    try:
        steps = [1, -1, 5, 3, -1, 1, 5]
        o_gks, g_gk = p.galois_keys(sorted(set(steps)))
        z = p.rng.uniform(-1, 1, (len(steps), p.n))
        a, b = _both(p, g_gk, z, p.pr.L, steps)  # first call: 7 ciphertexts at the top level
        assert np.array_equal(a, b)
        # and against the oracle itself, for one of them
        o_cts, g_ct = p.encrypt_both(z[:1], p.pr.L)
        got = p.ctx.ct_alloc(1, p.pr.L)
        p.ctx.rotate_static(g_gk, g_ct, steps[:1], got)
        assert np.array_equal(got.export()[0], p.o.rotate(o_cts[0], o_gks[steps[0]]).limbs())
        got.free()
        g_ct.free()
        a, b = _both(p, g_gk, z[:2], 2, [5, -1])  # second call: smaller batch, lower level, same workspace
        assert np.array_equal(a, b)
        a, b = _both(p, g_gk, z[:3], p.pr.L, [3, 3, 1])  # and a larger one again
        assert np.array_equal(a, b)
        g_gk.free()
    finally:
        p.close()


def test_rotate_static_full_ring_and_size_limit():
    p = Pair(KEYSWITCH)
    try:
        steps = [4096, -1]
        o_gks, g_gk = p.galois_keys(steps)
        z = p.rng.uniform(-1, 1, (2, p.n))
        a, b = _both(p, g_gk, z[:1], p.pr.L, steps[:1])  # one ciphertext at 10 + 3 limbs: 52 MiB of the 96
        assert np.array_equal(a, b)
        a, b = _both(p, g_gk, z, 4, steps)  # then two at 4 limbs
        assert np.array_equal(a, b)
        # two ciphertexts at the top level do not fit: refused with the size in the message, nothing launched
        _, g_ct = p.encrypt_both(z, p.pr.L)
        out = p.ctx.ct_alloc(2, p.pr.L)
        with pytest.raises(p.binding.EnsiError, match="static workspace holds"):
            p.ctx.rotate_static(g_gk, g_ct, steps, out)
        # the timers create events, which is an allocation: refused while they are on
        p.ctx.profile_enable(True)
        one = p.ctx.ct_wrap(g_ct.device_ptr, 1, p.pr.L, g_ct.scale)
        with pytest.raises(p.binding.EnsiError):
            p.ctx.rotate_static(g_gk, one, steps[:1], p.ctx.ct_wrap(out.device_ptr, 1, p.pr.L, 1.0))
        p.ctx.profile_enable(False)
        for h in (g_ct, out, g_gk):
            h.free()
    finally:
        p.close()
