#!/usr/bin/env python3
"""Benchmark of the encrypted ternary matmul hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input:
  * matmul workloads: unpack rotations (ModUp, NTT, key inner product, iNTT,
    ModDown) + Alg. 1 accumulate (+ scalar-multiply/rescale + second layer for
    the FFN workload), inputs and keys already resident in HBM;
  * the key-switch microbenchmark (always run as a second leg): 64 ciphertexts,
    each rotated by one of 16 Galois elements, reported as rotations/s.
One JSON line is printed.  `value` is ms/layer of the matmul workload;
`rotations` carries the rotations/s figure; `roofline` describes the dominant
kernel class of the timed step; `cpu_baseline` is the CPU oracle timed on a
bounded sample of the same workload on this host.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402

HBM_PEAK_GBS = 8000.0
INT8_MFMA_PEAK_TOPS = 5000.0  # dense int8 matrix-core peak, TOP/s
# plain integer ALU: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz 32-bit lane-ops/s; one 64-bit add = 2 of them
U64_ADD_PEAK = 256 * 4 * 16 * 2.4e9 / 2
NNZ_FRACTION = 0.6  # P(-1) + P(+1) of the synthetic ternary weights


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


class Runner:
    def __init__(self, w, seed=1, separate_rescale=False):
        from paper_2509_09424_amd import binding
        self.w = w
        self.separate_rescale = separate_rescale
        self.ctx = binding.Context(*w.param_tuple(), seed=seed)
        self.N, self.n = w.N, w.n_slots
        self.L, self.K, self.alpha = w.q_count, w.p_count, w.alpha
        self.beta = -(-self.L // self.alpha)
        self.sk, self.pk = self.ctx.keygen(None, None, 11)

    def sync(self):
        import torch
        torch.cuda.synchronize()

    def close(self):
        """Frees every device-side handle of this runner and its context (a later leg needs the memory)."""
        import torch
        torch.cuda.synchronize()
        for name, v in list(vars(self).items()):
            if name != "ctx" and hasattr(v, "free") and hasattr(v, "h"):
                v.free()
        self.buf = None
        self.ctx.close()
        torch.cuda.empty_cache()

    # ---- workload set-up (untimed): inputs and keys made resident on the device
    def setup(self):
        w = self.w
        rng = wl.rng_for(w.index)
        if w.name == "keyswitch":
            X = rng.uniform(-1.0, 1.0, size=(w.batch, self.n))
            pt = self.ctx.encode(X, self.L)
            self.ct_in = self.ctx.encrypt(self.pk, pt)
            pt.free()
            self.steps = [wl.KEYSWITCH_STEPS[b % 16] for b in range(w.batch)]
            self.gk = self.ctx.galois_keygen(self.sk, wl.KEYSWITCH_STEPS, None, 13)
            self.ct_out = self.ctx.ct_alloc(w.batch, self.L)
            self.X = X
            return
        if w.op == "rope":
            # Alg. 2 on the packed query ciphertexts: one angle per slot pair
            n_ct = -(-w.d_in // w.c_tot)
            self.X = rng.uniform(-1.0, 1.0, size=(n_ct, self.n))
            theta = rng.uniform(0.0, 2.0 * np.pi, self.n // 2)
            self.cos, self.sin = np.repeat(np.cos(theta), 2), np.repeat(np.sin(theta), 2)
            pt = self.ctx.encode(self.X, self.L)
            self.ct_in = self.ctx.encrypt(self.pk, pt)
            pt.free()
            self.gk = self.ctx.galois_keygen(self.sk, [1, -1], None, 13)
            self.pt = self.ctx.rope_plaintexts(self.cos, self.sin, self.L)
            self.ct_out = self.ctx.ct_alloc(n_ct, self.L - 1)
            return
        if w.op == "ccmm":
            # C = A B: A = d_in columns of `n` tokens, B = d_out columns with their d_in entries in the first slots
            d, m = w.d_in, w.d_out
            self.A = rng.uniform(-1.0, 1.0, size=(self.n, d))
            self.B = rng.uniform(-1.0, 1.0, size=(d, m))
            zb = np.zeros((m, self.n))
            zb[:, :d] = self.B.T
            pt = self.ctx.encode(np.ascontiguousarray(self.A.T), self.L)
            self.ct_a = self.ctx.encrypt(self.pk, pt)
            pt.free()
            pt = self.ctx.encode(zb, self.L)
            self.ct_in = self.ctx.encrypt(self.pk, pt)
            pt.free()
            self.period = 1 << (d - 1).bit_length()
            steps = sorted(set(self.ctx.fill_steps(self.period, self.n) + self.ctx.fill_steps(1, self.period)))
            self.gk = self.ctx.galois_keygen(self.sk, steps, None, 13)
            self.rk = self.ctx.relin_keygen(self.sk, None, 17)
            self.pt = self.ctx.periodic_masks(self.period, d, self.L)
            self.ct_out = self.ctx.ct_alloc(m, self.L - 2)
            return
        if w.op == "ccmm_blocks":
            # Q K^T for every head: ciphertext j holds column j of all heads (head h in block h)
            d, m, sl = w.d_in, w.d_out, w.tokens
            heads = self.n // sl
            self.Q = rng.uniform(-1.0, 1.0, size=(heads, sl, d))
            self.K = rng.uniform(-1.0, 1.0, size=(heads, sl, d))
            za = np.stack([np.concatenate([self.Q[h][:, j] for h in range(heads)]) for j in range(d)])
            zb = np.stack([np.concatenate([self.K[h][:, j] for h in range(heads)]) for j in range(d)])
            pt = self.ctx.encode(za, self.L)
            self.ct_a = self.ctx.encrypt(self.pk, pt)
            pt.free()
            pt = self.ctx.encode(zb, self.L)
            self.ct_in = self.ctx.encrypt(self.pk, pt)
            pt.free()
            self.cols = list(range(m))
            steps = [c for c in self.cols if c] + self.ctx.fill_steps(1, sl, -1)
            self.gk = self.ctx.galois_keygen(self.sk, steps, None, 13)
            self.rk = self.ctx.relin_keygen(self.sk, None, 17)
            self.pt = self.ctx.block_start_mask(sl, self.L)
            self.ct_out = self.ctx.ct_alloc(m, self.L - 2)
            return
        if w.op == "ccmm_av":
            # weights times V from diagonalised weights: d_in tokens = d_in / period segments, d_out columns of V
            import torch
            sl, P, m = w.tokens, w.period, w.d_out
            d = -(-w.d_in // P) * P  # whole segments: columns of A beyond d_in are zero, as are the entries of V they meet
            heads = self.n // sl
            self.Wt = rng.uniform(-1.0, 1.0, size=(heads, sl, d)) / 16
            self.Wt[:, :, w.d_in:] = 0.0
            self.V = rng.uniform(-1.0, 1.0, size=(heads, sl, m))
            self.V[:, w.d_in:, :] = 0.0
            za = np.stack([np.concatenate([self.Wt[h][:, j] for h in range(heads)]) for j in range(d)])
            zb = np.stack([np.concatenate([self.V[h][:, i] for h in range(heads)]) for i in range(m)])
            self.ref = np.stack([np.concatenate([self.Wt[h] @ self.V[h][:d, i] for h in range(heads)]) for i in range(m)])
            pt = self.ctx.encode(za, self.L)
            ct_a = self.ctx.encrypt(self.pk, pt)
            pt.free()
            pt = self.ctx.encode(zb, self.L)
            self.ct_in = self.ctx.encrypt(self.pk, pt)
            pt.free()
            self.baby = w.baby  # the column of V is rotated by the baby steps only; the weights carry the giant steps
            giant = {k * self.baby for k in range(1, P // self.baby + 1)}
            steps = set(range(1, self.baby)) | giant | {-t for t in giant} | {g * P for g in range(1, d // P)} | set(self.ctx.fill_steps(P, sl, -1))
            self.gk = self.ctx.galois_keygen(self.sk, sorted(steps), None, 13)
            self.rk = self.ctx.relin_keygen(self.sk, None, 17)
            self.pt = self.ctx.block_head_mask(sl, P, self.L)
            masks = self.ctx.segment_masks(sl, P, self.L)
            # the weights are rearranged once for all columns of V: outside the timed step, its time reported beside it
            self.ct_a = self.ctx.diagonalise_weights(self.gk, ct_a, sl, P, self.baby, masks, prepare=True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            self.ctx.diagonalise_weights(self.gk, ct_a, sl, P, self.baby, masks, self.ct_a, prepare=True)
            torch.cuda.synchronize()
            self.prepare_ms = (time.perf_counter() - t0) * 1e3
            log("diagonalised %d weight columns in %.1f ms (once for all columns of V)" % (d, self.prepare_ms))
            ct_a.free()
            masks.free()
            self.ct_out = self.ctx.ct_alloc(m, self.L - 2)
            return
        if w.op in ("ccmm_bsgs", "ccmm_bsgs_av", "ccmm_segment"):
            # both attention products for every head at once, element extraction in giant and baby steps
            sl, P = w.tokens, w.period
            heads = self.n // sl
            if w.op in ("ccmm_bsgs", "ccmm_segment"):
                # Q K^T: ciphertext j holds column j of all heads; a step forms the columns of segment 1
                d, m = w.d_in, w.d_out
                self.Q = rng.uniform(-1.0, 1.0, size=(heads, sl, d))
                self.K = rng.uniform(-1.0, 1.0, size=(heads, sl, d))
                za = np.stack([np.concatenate([self.Q[h][:, j] for h in range(heads)]) for j in range(d)])
                zb = np.stack([np.concatenate([self.K[h][:, j] for h in range(heads)]) for j in range(d)])
                self.cols = list(range(P, P + m))
                self.terms = [[(j, j, i) for j in range(d)] for i in self.cols]
                self.ref = np.stack([np.concatenate([(self.Q[h] @ self.K[h].T)[:, i] for h in range(heads)]) for i in self.cols])
            else:
                # weights times V: ciphertext j of A holds column j of the weights of all heads (d_in of them), B the
                # d_out columns of V; output i sums over the d_in tokens j
                d, m = w.d_in, w.d_out
                self.Wt = rng.uniform(-1.0, 1.0, size=(heads, sl, d)) / 16
                self.V = rng.uniform(-1.0, 1.0, size=(heads, sl, m))
                za = np.stack([np.concatenate([self.Wt[h][:, j] for h in range(heads)]) for j in range(d)])
                zb = np.stack([np.concatenate([self.V[h][:, i] for h in range(heads)]) for i in range(m)])
                self.terms = [[(j, i, j) for j in range(d)] for i in range(m)]
                self.ref = np.stack([np.concatenate([self.Wt[h] @ self.V[h][:d, i] for h in range(heads)]) for i in range(m)])
            pt = self.ctx.encode(za, self.L)
            self.ct_a = self.ctx.encrypt(self.pk, pt)
            pt.free()
            pt = self.ctx.encode(zb, self.L)
            self.ct_in = self.ctx.encrypt(self.pk, pt)
            pt.free()
            slots = sorted({t[2] for tl in self.terms for t in tl})
            steps = {x // P * P for x in slots} | set(self.ctx.fill_steps(P, sl, -1))
            if w.op == "ccmm_segment":
                # the whole segment 1 from its diagonals, in baby steps of the spread operands and giant steps of the columns of Q
                assert m == P
                self.baby = w.baby
                giant = {k * self.baby for k in range(1, P // self.baby + 1)}
                steps |= set(range(1, self.baby)) | giant | {-t for t in giant}
                self.pt2 = self.ctx.segment_masks(sl, P, self.L - 2)
            else:
                steps |= {x % P for x in slots} | set(self.ctx.fill_steps(1, P, -1))
                self.pt2 = self.ctx.periodic_masks(P, 1, self.L - 1)
            self.gk = self.ctx.galois_keygen(self.sk, sorted(x for x in steps if x), None, 13)
            self.rk = self.ctx.relin_keygen(self.sk, None, 17)
            self.pt = self.ctx.block_head_mask(sl, P, self.L)
            self.ct_out = self.ctx.ct_alloc(len(self.terms), self.L - 3)
            if w.op == "ccmm_segment":
                # the columns of Q moved by their giant steps once for all 64 segments: outside the timed step, time reported
                import torch
                plain = self.ct_a
                self.ct_a = self.ctx.ccmm_left_giant_steps(self.gk, plain, P, self.baby, prepare=True)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                self.ctx.ccmm_left_giant_steps(self.gk, plain, P, self.baby, self.ct_a, prepare=True)
                torch.cuda.synchronize()
                self.prepare_ms = (time.perf_counter() - t0) * 1e3
                log("moved %d columns of Q by their giant steps in %.1f ms (once for all segments)" % (d, self.prepare_ms))
                plain.free()
            return
        if w.op == "merge":
            # d_in block-placed outputs: one group of c_tot encrypted columns, repeated for every packed output
            import torch
            c_tot, s = w.c_tot, w.tokens
            self.Y = rng.uniform(-1.0, 1.0, size=(c_tot, s))
            z = rng.uniform(-1.0, 1.0, size=(c_tot, self.n))  # the other blocks hold unrelated values
            for b in range(c_tot):
                z[b, b * s:(b + 1) * s] = self.Y[b]
            pt = self.ctx.encode(z, self.L)
            grp = self.ctx.encrypt(self.pk, pt)
            pt.free()
            words = 2 * self.L * self.N
            self.buf = torch.empty((w.d_in, words), dtype=torch.int64, device="cuda")
            scale = grp.scale
            host = torch.from_numpy(grp.export().view(np.int64).reshape(c_tot, words)).cuda()
            for g0 in range(0, w.d_in, c_tot):
                self.buf[g0:g0 + c_tot] = host[: min(c_tot, w.d_in - g0)]
            torch.cuda.synchronize()
            grp.free()
            self.ct_in = self.ctx.ct_wrap(self.buf.data_ptr(), w.d_in, self.L, scale)
            self.pt = self.ctx.block_masks(s, c_tot, self.L)
            self.ct_out = self.ctx.ct_alloc(-(-w.d_in // c_tot), self.L - 1)
            return
        self.W = wl.ternary_weights(rng, w.d_in, w.d_mid or w.d_out)
        self.X = wl.activations(rng, w.tokens, w.d_in, w.act)
        if w.d_mid:
            self.W2 = wl.ternary_weights(rng, w.d_mid, w.d_out)
        packed = wl.pack_columns(self.X, self.n)
        pt = self.ctx.encode(packed, self.L)
        self.ct_in = self.ctx.encrypt(self.pk, pt)
        pt.free()
        c_tot = w.c_tot
        n_rho = min(c_tot, w.d_in)
        rot_steps = [r * w.tokens for r in range(1, c_tot)] if w.placement == "diagonal" else [r * w.tokens for r in range(1, n_rho)]
        t0 = time.time()
        self.gk = self.ctx.galois_keygen(self.sk, rot_steps, None, 13) if rot_steps else None
        log("generated %d Galois keys in %.1f s" % (len(rot_steps), time.time() - t0))
        self.ct_out = self.ctx.ct_alloc(w.d_mid or w.d_out, self.L)
        # everything Alg. 1 derives from the weights alone is built once, outside the step (the weights of a layer are static)
        self.wt = self.ctx.weights_prepare(self.W, w.tokens, w.d_in, w.placement, self.L)
        if w.d_mid:
            self.ct_out2 = self.ctx.ct_alloc(w.d_out, self.L - 1)
            self.wt2 = self.ctx.weights_prepare(self.W2, self.n, w.d_mid, "zero", self.L - 1)

    def step(self):
        w = self.w
        if w.name == "keyswitch":
            self.ctx.rotate(self.gk, self.ct_in, self.steps, self.ct_out)
            return
        if w.op == "rope":
            self.ctx.rope(self.gk, self.ct_in, self.pt, self.ct_out)
            return
        if w.op == "merge":
            self.ctx.merge(self.ct_in, self.pt, w.c_tot, self.ct_out)
            return
        if w.op == "ccmm":
            self.ctx.ccmm(self.rk, self.gk, self.ct_a, self.ct_in, self.pt, self.period, self.ct_out)
            return
        if w.op == "ccmm_blocks":
            self.ctx.ccmm_blocks(self.rk, self.gk, self.ct_a, self.ct_in, w.tokens, self.cols, self.pt, self.ct_out)
            return
        if w.op in ("ccmm_bsgs", "ccmm_bsgs_av"):
            self.ctx.ccmm_bsgs(self.rk, self.gk, self.ct_a, self.ct_in, w.tokens, w.period, self.terms, self.pt, self.pt2, self.ct_out)
            return
        if w.op == "ccmm_av":
            self.ctx.ccmm_av(self.rk, self.gk, self.ct_a, self.ct_in, w.tokens, w.period, self.baby, 0, self.pt, self.ct_out)
            return
        if w.op == "ccmm_segment":
            self.ctx.ccmm_segment(self.rk, self.gk, self.ct_a, self.ct_in, w.tokens, w.period, self.baby, 1, self.pt, self.pt2, self.ct_out)
            return
        self.ctx.ternary_matmul_prepared(self.gk, self.ct_in, self.wt, self.ct_out)
        if w.d_mid:
            # the rescale works in place and lowers the level: restore the handle's level by re-wrapping
            if getattr(self, "mid", None) is not None:
                self.mid.free()
            mid = self.ctx.ct_wrap(self.ct_out.device_ptr, w.d_mid, self.L, self.ct_in.scale)
            self.mid = mid
            if self.separate_rescale:
                self.ctx.mul_scalar_rescale(mid, w.kappa)
                self.ctx.ternary_matmul_prepared(None, mid, self.wt2, self.ct_out2)
            else:
                # scalar-multiply + rescale applied while the second layer reads its operands
                self.ctx.rescale_ternary_matmul_prepared(mid, w.kappa, self.wt2, self.ct_out2)

    def check(self):
        """Decrypts a few outputs and compares with the float64 product (sanity, untimed)."""
        w = self.w
        self.sync()
        if w.name == "keyswitch":
            dec = self.ctx.decrypt(self.sk, self.ct_out)
            err = max(np.abs(dec[b] - np.roll(self.X[b], -self.steps[b])).max() for b in range(w.batch))
            return float(err)
        if w.op == "rope":
            x, c, s_ = self.X, self.cos, self.sin
            ref = np.empty_like(x)
            ref[:, 0::2] = x[:, 0::2] * c[0::2] - x[:, 1::2] * s_[0::2]
            ref[:, 1::2] = x[:, 1::2] * c[1::2] + x[:, 0::2] * s_[1::2]
            return float(np.abs(self.ctx.decrypt(self.sk, self.ct_out) - ref).max())
        if w.op == "merge":
            dec = self.ctx.decrypt(self.sk, self.ct_out)
            return float(np.abs(dec - self.Y.reshape(1, -1)).max())
        if w.op == "ccmm":
            dec = self.ctx.decrypt(self.sk, self.ct_out)
            return float(np.abs(dec - (self.A @ self.B).T).max())
        if w.op == "ccmm_blocks":
            dec = self.ctx.decrypt(self.sk, self.ct_out)
            heads = self.n // w.tokens
            ref = np.stack([np.concatenate([(self.Q[h] @ self.K[h].T)[:, i] for h in range(heads)]) for i in self.cols])
            return float(np.abs(dec - ref).max())
        if w.op in ("ccmm_bsgs", "ccmm_bsgs_av", "ccmm_segment", "ccmm_av"):
            return float(np.abs(self.ctx.decrypt(self.sk, self.ct_out) - self.ref).max())
        ref = self.X @ self.W.astype(np.float64)
        out = self.ct_out
        if w.d_mid:
            ref = (ref * w.kappa) @ self.W2.astype(np.float64)
            out = self.ct_out2
        m = w.d_out
        err = 0.0
        # decrypt only a sample of output ciphertexts through wrapped single-ciphertext views
        sample = sorted(set([0, 1, m // 2, m - 1] + list(np.random.default_rng(0).integers(0, m, 12))))
        n, limbs, scale, base = out._info()
        alloc = self.L - 1 if w.d_mid else self.L
        words = 2 * alloc * self.N
        for i in sample:
            one = self.ctx.ct_wrap(int(base) + 8 * words * int(i), 1, limbs, scale)
            p_i = 0 if (w.placement == "zero" or w.d_mid) else i % w.c_tot
            dec = self.ctx.decrypt(self.sk, one, p_i * w.tokens, w.tokens)[0]
            err = max(err, float(np.abs(dec - ref[:, i]).max()))
            one.free()
        return err


def time_steps(runner, steps, warmup):
    import torch
    for _ in range(warmup):
        runner.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        runner.step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def kernel_profile(runner):
    """One extra, untimed step with the library's HIP-event timers on: per-class total ms and launches."""
    import torch
    torch.cuda.synchronize()
    runner.ctx.profile_read()
    runner.ctx.profile_enable(True)
    runner.step()
    torch.cuda.synchronize()
    prof = runner.ctx.profile_read()
    runner.ctx.profile_enable(False)
    return prof


def profile_facts(workload, kernel):
    """Figures that come from rocprofv3 counter runs rather than from this process, read from the tracked summary
    profiles/bench_<workload>_kernels_and_hbm_counters.txt: lines of the form
        @facts <kernel> key=value key=value ...
    (fetch_GiB_per_step, write_GiB_per_step, launches_per_step, mfma_busy, valu_util, sclk_GHz).  Returns {} when the
    summary or the line is missing, so a stale constant can never be reported."""
    path = os.path.join(ROOT, "profiles", "bench_%s_kernels_and_hbm_counters.txt" % workload)
    facts = {}
    try:
        for line in open(path):
            t = line.split()
            if len(t) >= 2 and t[0] == "@facts" and t[1] == kernel:
                for kv in t[2:]:
                    k, _, v = kv.partition("=")
                    facts[k] = float(v)
    except OSError:
        pass
    return facts


def fill_counts(r_begin, r_end):
    """(rotations, raises) of the library's rotate-and-add fill between two strides: steps of radix four (three
    rotations on one raise) while two doublings remain, then a single doubling."""
    rot = raises = 0
    r = r_begin
    while r < r_end:
        if 2 * r < r_end:
            rot, raises, r = rot + 3, raises + 1, r * 4
        else:
            rot, raises, r = rot + 1, raises + 1, r * 2
    return rot, raises


def roofline_for(w, prof):
    """Roofline entry of the dominant kernel class of the step (largest total time)."""
    N, L, K, alpha = w.N, w.q_count, w.p_count, w.alpha
    unit = 8.0 * N  # bytes of one limb
    # key-switch work as stages at one level each: (limbs, rotations, raises, switch-backs to the ciphertext basis --
    # grouped rotations share one --, keys streamed); plaintext multiplications as (limbs, products, outputs)
    ks, pm, mm = [], [], []  # mm: ciphertext products as (limbs, distinct operands transformed, outputs)
    if w.name == "keyswitch":
        ks.append((L, w.batch, w.batch, w.batch, w.batch))  # every rotation streams its key
    elif w.op == "rope":
        n_ct = -(-w.d_in // w.c_tot)
        ks.append((L, 2 * n_ct, n_ct, 2 * n_ct, 2 * -(-n_ct // 32)))  # inputs are rotated 32 at a time, a key is read once per group
        pm.append((L, 3 * n_ct, n_ct))
    elif w.op == "merge":
        pm.append((L, w.d_in, -(-w.d_in // w.c_tot)))
    elif w.op == "ccmm_blocks":
        # per element: one aligning rotation (the raise shared by all columns of a ciphertext of B), one mask product and
        # log2(s) fill steps one level down; per output one relinearisation
        n_el = w.d_in * w.d_out
        f_rot, f_raise = fill_counts(1, w.tokens)
        ks.append((L - 1, n_el * (1 + f_rot) + w.d_out, w.d_in + n_el * f_raise + w.d_out, n_el * (1 + f_raise) + w.d_out,
                   -(-w.d_in // 16) * w.d_out + f_rot * -(-n_el // 64) + 1))
        pm.append((L, n_el, n_el))
        mm.append((L - 1, w.d_in + n_el, w.d_out))
    elif w.op == "ccmm":
        # every element of B: one mask product and log2(period) rotate-and-add steps one level down (the log2(n/period)
        # steps per column at the top level and the relinearisations are few and counted with them)
        n_el = w.d_in * w.d_out
        period = 1 << (w.d_in - 1).bit_length()
        b_rot, b_raise = fill_counts(1, period)
        g_rot, g_raise = fill_counts(period, w.n_slots)
        n_raise = n_el * b_raise + w.d_out * g_raise + w.d_out
        ks.append((L - 1, n_el * b_rot + w.d_out * g_rot + w.d_out, n_raise, n_raise, b_rot * -(-n_el // 64) + g_rot + 1))
        pm.append((L, n_el, n_el))
        mm.append((L - 1, w.d_in + n_el, w.d_out))
    elif w.op in ("ccmm_bsgs", "ccmm_bsgs_av"):
        # giant steps per segment (aligning rotation at the top level, head mask, fill over the block one level down),
        # baby steps per element (aligning rotation there, period-start mask, fill over the period two levels down),
        # one relinearisation per output
        P = w.period
        if w.op == "ccmm_bsgs":
            n_el, n_seg, n_src = w.d_in * w.d_out, w.d_in * -(-w.d_out // P), w.d_in
        else:
            n_el, n_seg, n_src = w.d_in * w.d_out, -(-w.d_in // P) * w.d_out, w.d_out
        g_rot, g_raise = fill_counts(P, w.tokens)
        b_rot, b_raise = fill_counts(1, P)
        ks.append((L, n_seg, n_src, n_seg, -(-n_src // 16) * max(1, n_seg // max(n_src, 1))))
        ks.append((L - 1, n_seg * g_rot + n_el, n_seg * (g_raise + 1), n_seg * g_raise + n_el, g_rot * -(-n_seg // 64) + (P - 1) * -(-n_seg // 16)))
        ks.append((L - 2, n_el * b_rot + w.d_out, n_el * b_raise + w.d_out, n_el * b_raise + w.d_out, b_rot * -(-n_el // 64) + 1))
        pm.append((L, n_seg, n_seg))
        pm.append((L - 1, n_el, n_el))
        mm.append((L - 2, w.d_in + n_el, w.d_out))
    elif w.op == "ccmm_av":
        # per column of V and segment: one giant step (aligning rotation at the top level, head mask, fill over the block one
        # level down) and 2P-2 rotations of the spread operand on one raise; one relinearisation per output
        P, n_seg, m, baby = w.period, -(-w.d_in // w.period), w.d_out, w.baby
        g_rot, g_raise = fill_counts(P, w.tokens)
        n_sg, n_t = n_seg * m, 2 * P // baby  # spread operands; giant steps (sums per output)
        ks.append((L, n_sg, m, n_sg, n_seg))
        ks.append((L - 1, n_sg * (g_rot + baby - 1) + n_t * m, n_sg * (g_raise + 1) + n_t * m, n_sg * (g_raise + baby - 1) + n_t * m,
                   g_rot * -(-n_sg // 64) + (baby - 1) * -(-n_sg // 16) + 1))
        ks.append((L - 1, (n_t - 1) * m, (n_t - 1) * m, (n_t - 1) * m, (n_t - 1) * m))  # the sums rotated by their giant steps, before the rescale
        pm.append((L, n_sg, n_sg))
        mm.append((L - 1, n_sg * baby, n_t * m))  # the prepared weights are not transformed again
    elif w.op == "ccmm_segment":
        # per ciphertext of B: one giant step (aligning rotation at the top level, head mask, fill over the block one level
        # down) and 2P-2 rotations of the spread operand on one raise; 2P-1 relinearisations two levels down; the sorting
        # products of the 2P-1 diagonals into P columns
        P, dd, baby = w.period, w.d_in, w.baby
        g_rot, g_raise = fill_counts(P, w.tokens)
        n_diag, n_t = 2 * P - 1, 2 * P // baby
        ks.append((L, dd, dd, dd, -(-dd // 16)))
        # one level down: the fills, the baby steps of the spread operands and the giant steps of the columns of Q on one raise
        # each, the relinearisations, the giant steps of the sums that have one
        n_rs = n_diag - baby
        # (the columns of Q are moved by their giant steps and transformed once for all segments, outside the step)
        ks.append((L - 1, dd * (g_rot + baby - 1) + n_diag + n_rs, dd * (g_raise + 1) + n_diag + n_rs,
                   dd * (g_raise + baby - 1) + n_diag + n_rs, g_rot * -(-dd // 64) + (baby - 1) * -(-dd // 16) + 1 + n_rs))
        pm.append((L, dd, dd))
        pm.append((L - 2, P * P + P * (P - 1) // 2, P, n_diag))  # every diagonal enters many sorting products, transformed once
        mm.append((L - 1, dd * baby, n_diag))
    else:
        n_in = -(-w.d_in // w.c_tot)
        # the packed inputs (up to 16) are rotated together, so a key is read once per rotation amount
        ks.append((L, w.d_in - n_in, n_in, w.d_in - n_in, -(-n_in // 16) * (min(w.c_tot, w.d_in) - 1)))

    fused_ks = w.log_n == 16 and w.q_bits <= 50  # the key switch transforms inside its own kernels

    def ks_sum(f):
        return sum(f(l, -(-l // alpha), l + K, n_rot, n_raise, n_sw, n_key) for l, n_rot, n_raise, n_sw, n_key in ks)

    def pm_sum(f):
        # (limbs, products, outputs[, distinct sources: a source that enters several products is column-transformed once])
        return sum(f(e[0], e[1], e[2], e[3] if len(e) > 3 else e[1]) for e in pm)

    # HBM-bound classes: algorithmic limb-units per step (every operand read once, every result written once)
    hbm = {
        # fused path (N = 2^16, ciphertext primes below 2^50)
        "ks_pre": ks_sum(lambda l, b, e, rot, ra, sw, key: ra * 2 * l),
        "ks_modup_fcols": ks_sum(lambda l, b, e, rot, ra, sw, key: ra * (3 * l + b * e + l)),        # y, c1, c0 in; raised digits and P*c0 out
        "ks_frows": ks_sum(lambda l, b, e, rot, ra, sw, key: ra * 2 * (b * e + l)),
        # ciphertext limbs: digits, P*c0, key in; accumulators out
        "ks_inner_irows": ks_sum(lambda l, b, e, rot, ra, sw, key: rot * (b * l + l) + sw * 2 * l + key * 2 * b * l),
        # special limbs (integer arithmetic)
        "ks_inner_irows_wide": ks_sum(lambda l, b, e, rot, ra, sw, key: rot * b * K + sw * 2 * K + key * 2 * b * K),
        "ks_icols_special": ks_sum(lambda l, b, e, rot, ra, sw, key: sw * 4 * K),                    # special limbs in, split residues out
        "ks_icols_moddown": ks_sum(lambda l, b, e, rot, ra, sw, key: sw * (2 * l + 2 * K + 2 * l)),  # accumulators and residues in, ciphertext out
        # unfused path
        # library transforms: of the key switch on the unfused path; of the ciphertext products' operands (two passes, each
        # limb in and out) and of their three sums per output, back
        "ntt": (0 if fused_ks else ks_sum(lambda l, b, e, rot, ra, sw, key: 2 * (ra * b * e + rot * 2 * e)))
               + sum(4 * (ops * 2 * l + outs * 3 * l) for l, ops, outs in mm),
        "inner_product": ks_sum(lambda l, b, e, rot, ra, sw, key: rot * (b * e + 2 * e) + key * 2 * b * e),  # digits in, accumulators out; keys
        "modup": ks_sum(lambda l, b, e, rot, ra, sw, key: ra * (l + b * e)),
        "moddown": ks_sum(lambda l, b, e, rot, ra, sw, key: rot * (2 * e + 3 * l)),
        "mul_scalar_rescale": (w.d_mid or 0) * (2 * L + 2 * (L - 1)),
        # plane split: 8 bytes read + planes bytes written per operand word (units of 8 bytes per word: /N below)
        "byte_planes": (w.d_in * 2 * L + (0 if "rescale_byte_planes" in prof else (w.d_mid or 0) * 2 * (L - 1))) * (8 + 7) / 8.0,
        "rescale_byte_planes": (w.d_mid or 0) * (2 * L + 2 * (L - 1) * 7 / 8.0),
        # plaintext multiplication, summed and rescaled (the few plaintext limbs are not counted)
        "pm_fcols": pm_sum(lambda l, t, o, src: src * 4 * l),                    # source limbs in, column-transformed limbs out
        "pm_frows_mac_irows": pm_sum(lambda l, t, o, src: (t + o) * 2 * l),      # those in, one sum per output limb out
        "pm_icols_last": pm_sum(lambda l, t, o, src: o * 4),
        "pm_icols_rescale": pm_sum(lambda l, t, o, src: o * (2 * (l - 1) + 2 + 2 * (l - 1))),
    }
    members = {"ntt": ["ntt_fwd_cols", "ntt_fwd_rows", "ntt_inv_rows", "ntt_inv_cols"]}
    classes = list(hbm) + ["accumulate", "accumulate_mfma"]
    tot = {g: sum(prof.get(k, (0.0, 0))[0] for k in members.get(g, [g])) for g in classes}
    dom = max(tot, key=tot.get)
    ms = tot[dom]
    launches = sum(prof.get(k, (0.0, 0))[1] for k in members.get(dom, [dom]))
    if dom == "accumulate_mfma":
        # Alg. 1 on the matrix cores: one int8 multiply-add per (output, operand, limb word, byte plane); 7 planes at 50 bits
        planes = -(-w.q_bits // 8)
        planes = 5 if planes <= 5 else 7 if planes <= 7 else 8
        # (outputs x operands x limb words) of each layer; the second layer of the FFN workload runs one level down
        cells = w.d_in * (w.d_mid or w.d_out) * 2.0 * L * N + (w.d_mid * w.d_out * 2.0 * (L - 1) * N if w.d_mid else 0)
        ops = 2.0 * cells * planes              # dense: every weight, zero or not, is a multiply-add per byte plane
        own = 2.0 * NNZ_FRACTION * cells * planes  # the method's own work (Alg. 1 skips zero weights), in the same unit
        facts = profile_facts(w.name, dom)
        traffic = None
        if "fetch_GiB_per_step" in facts and "write_GiB_per_step" in facts:
            traffic = (facts["fetch_GiB_per_step"] + facts["write_GiB_per_step"]) * 2.0 ** 30 / max(launches, 1)
        tops = ops / (ms * 1e-3) / 1e12
        return dom, {"bound": "mfma", "achieved": tops, "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                     "frac": tops / INT8_MFMA_PEAK_TOPS, "frac_dense": tops / INT8_MFMA_PEAK_TOPS,
                     "frac_own_work": own / (ms * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS, "traffic": traffic, "kernel": dom,
                     "launch_ms": ms / max(launches, 1), "launches": launches, "ops_per_launch": ops / max(launches, 1),
                     "algorithmic_bytes_per_launch": ((w.d_in + (w.d_mid or w.d_out)) * 2 * L + ((w.d_mid + w.d_out) * 2 * (L - 1) if w.d_mid else 0)) * unit / max(launches, 1),
                     "mfma_busy": facts.get("mfma_busy"), "valu_util": facts.get("valu_util"), "sclk_GHz": facts.get("sclk_GHz")}
    if dom == "accumulate":
        # Alg. 1: one 64-bit add/sub per non-zero weight per limb word
        ops = NNZ_FRACTION * (w.d_in * (w.d_mid or w.d_out) * 2.0 * L * N + (w.d_mid * w.d_out * 2.0 * (L - 1) * N if w.d_mid else 0))
        return dom, {"bound": "alu", "achieved": ops / (ms * 1e-3) / 1e12, "peak": U64_ADD_PEAK / 1e12, "unit": "Tadd64/s",
                     "frac": ops / (ms * 1e-3) / U64_ADD_PEAK, "traffic": None, "kernel": dom,
                     "launch_ms": ms / max(launches, 1), "launches": launches}
    gbs = unit * hbm[dom] / (ms * 1e-3) / 1e9
    return dom, {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                 "traffic": None, "kernel": dom, "launch_ms": ms / max(launches, 1), "launches": launches}


def hbm_fractions(w, prof_all):
    """Algorithmic GB/s of every HBM-bound kernel class that ran in the step (for the key-switch target)."""
    out = {}
    for name in list(prof_all):
        one = {name: prof_all[name]}
        if name == "byte_planes" and "rescale_byte_planes" in prof_all:
            one["rescale_byte_planes"] = (0.0, 0)
        try:
            dom, roof = roofline_for(w, one)
        except ZeroDivisionError:
            continue
        if dom == name and roof["bound"] == "hbm" and roof["achieved"] > 0:
            out[name] = {"GB/s": round(roof["achieved"], 1), "frac": round(roof["frac"], 4)}
            # vector-ALU issue-slot utilisation and memory-side rate of the same kernel, from the tracked counter summary
            out[name].update({k: v for k, v in profile_facts("keyswitch", name).items() if k in ("valu_util", "memory_side_TBps")})
    return out


def cpu_baseline(w, budget_s=12.0):
    """The CPU oracle, as it stands, on a bounded sample of the workload (about `budget_s` seconds of CPU
    work): repeated ModUps, hoisted rotations and Alg. 1 ciphertext add/subs at the workload's
    parameters; extrapolated linearly to the step's counts."""
    from oracle import Oracle, Params
    t_setup = time.time()
    pr = Params(*w.param_tuple())
    o = Oracle(pr)
    rng = np.random.default_rng(5)
    sk, pk = o.keygen(wl.ternary_poly(rng, o.N), wl.error_poly(rng, o.N), 3)
    z = rng.uniform(-1, 1, o.n)
    ct = o.encrypt(o.encode(z, pr.L), pk, wl.ternary_poly(rng, o.N), wl.error_poly(rng, o.N), wl.error_poly(rng, o.N))
    step = w.tokens if (w.tokens and w.op == "matmul") else 1
    gk = o.galois_keygen(sk, step, wl.error_poly(rng, (pr.beta(pr.L), o.N)), 4)
    o._key_at_level(gk, pr.L)
    log("oracle set-up %.1f s" % (time.time() - t_setup))

    def repeat(fn, seconds):
        n, t0 = 0, time.perf_counter()
        while True:
            out = fn()
            n += 1
            dt = time.perf_counter() - t0
            if dt >= seconds:
                return out, dt / n, n

    cores = len(os.sched_getaffinity(0))
    if w.name == "keyswitch":
        digits, t_modup, n1 = repeat(lambda: o.mod_up(ct.c1), budget_s * 0.3)
        rot, t_rot, n2 = repeat(lambda: o.rotate_from_digits(ct.c0, digits, gk, ct.scale), budget_s * 0.7)
        per = t_modup + t_rot
        return {"value": 1.0 / per, "unit": "rotations/s", "cores": cores, "kind": "oracle",
                "sample": "%d ModUps (%.3f s each) + %d key switches (%.3f s each) at the workload's parameters" % (n1, t_modup, n2, t_rot)}
    if w.op == "rope":
        n_ct = -(-w.d_in // w.c_tot)
        gk_m = o.galois_keygen(sk, -1, wl.error_poly(rng, (pr.beta(pr.L), o.N)), 4)
        o._key_at_level(gk_m, pr.L)
        theta = rng.uniform(0, 2 * np.pi, o.n // 2)
        pts = o.rope_plaintexts(np.repeat(np.cos(theta), 2), np.repeat(np.sin(theta), 2), pr.L)
        _, t_one, n1 = repeat(lambda: o.rope(ct, pts, gk, gk_m), budget_s)
        return {"value": n_ct * t_one * 1e3, "unit": "ms/batch", "cores": cores, "kind": "oracle",
                "sample": "%d ciphertexts through Alg. 2 (%.3f s each), extrapolated linearly to %d" % (n1, t_one, n_ct)}
    if w.op in ("ccmm", "ccmm_blocks", "ccmm_bsgs", "ccmm_bsgs_av", "ccmm_segment", "ccmm_av"):
        n_el = n_pm = w.d_in * w.d_out
        if w.op == "ccmm":
            period = 1 << (w.d_in - 1).bit_length()
            n_rot = n_el * fill_counts(1, period)[0] + w.d_out * fill_counts(period, w.n_slots)[0]
        elif w.op == "ccmm_blocks":
            n_rot = n_el * (1 + fill_counts(1, w.tokens)[0])
        elif w.op == "ccmm_av":
            n_diag, n_sg = 2 * w.period - 1, -(-w.d_in // w.period) * w.d_out
            n_rot = n_sg * (1 + fill_counts(w.period, w.tokens)[0] + w.baby - 1) + (2 * w.period // w.baby - 1) * w.d_out
            n_el = n_sg * n_diag
            n_pm = n_sg
        elif w.op == "ccmm_segment":
            n_diag = 2 * w.period - 1
            n_rot = w.d_in * (1 + fill_counts(w.period, w.tokens)[0] + w.baby - 1) + n_diag - w.baby
            n_el = w.d_in * n_diag
            n_pm = w.d_in + w.period * w.period + w.period * (w.period - 1) // 2
        else:
            n_seg = w.d_in * -(-w.d_out // w.period) if w.op == "ccmm_bsgs" else -(-w.d_in // w.period) * w.d_out
            n_rot = n_seg * (1 + fill_counts(w.period, w.tokens)[0]) + n_el * (1 + fill_counts(1, w.period)[0])
            n_pm = n_el + n_seg
        _, t_rot, n1 = repeat(lambda: o.rotate(ct, gk), budget_s * 0.5)
        mask_rns = o.i64_to_rns(o.periodic_masks(16, 1, pr.L)[0], pr.q)
        _, t_pm, n2 = repeat(lambda: o.pmult(ct, mask_rns, float(pr.q[-1])), budget_s * 0.2)
        _, t_ts, n3 = repeat(lambda: o.tensor_sum([(ct, ct)]), budget_s * 0.3)
        return {"value": (n_rot * t_rot + n_pm * t_pm + n_el * t_ts) * 1e3, "unit": "ms/batch", "cores": cores, "kind": "oracle",
                "sample": "%d rotations (%.3f s each), %d plaintext products (%.3f s), %d tensor products (%.3f s) at the top level, "
                          "extrapolated linearly to %d rotations, %d plaintext and %d tensor products (additions, relinearisations "
                          "and rescales left out)" % (n1, t_rot, n2, t_pm, n3, t_ts, n_rot, n_pm, n_el)}
    if w.op == "merge":
        masks = o.block_masks(w.tokens, 2, pr.L)
        mask_rns = o.i64_to_rns(masks[0], pr.q)
        _, t_one, n1 = repeat(lambda: o.pmult(ct, mask_rns, float(pr.q[-1])), budget_s)
        return {"value": w.d_in * t_one * 1e3, "unit": "ms/batch", "cores": cores, "kind": "oracle",
                "sample": "%d plaintext multiplications (%.3f s each), extrapolated linearly to %d (additions and rescales left out)"
                          % (n1, t_one, w.d_in)}
    digits, t_modup, n1 = repeat(lambda: o.mod_up(ct.c1), budget_s * 0.15)
    rot, t_rot, n2 = repeat(lambda: o.rotate_from_digits(ct.c0, digits, gk, ct.scale), budget_s * 0.45)
    n_terms = 256
    terms = [(rot if k % 2 else ct, 1 if k % 3 else -1) for k in range(n_terms)]
    _, t_acc, n3 = repeat(lambda: o.accumulate(terms, pr.L, ct.scale), budget_s * 0.4)
    t_add = t_acc / n_terms
    c_tot = w.c_tot
    n_in = -(-w.d_in // c_tot)
    n_rot = w.d_in - n_in
    nnz = 0.6 * w.d_in * (w.d_mid or w.d_out) + (0.6 * w.d_mid * w.d_out if w.d_mid else 0)
    total = n_in * t_modup + n_rot * t_rot + nnz * t_add
    return {"value": total * 1e3, "unit": "ms/layer", "cores": cores, "kind": "oracle",
            "sample": "%d ModUps (%.3f s each) + %d hoisted rotations (%.3f s each) + %d ciphertext add/subs (%.5f s each), "
                      "extrapolated linearly to %d ModUps, %d rotations, %.3g add/subs" % (n1, t_modup, n2, t_rot, n3 * n_terms, t_add, n_in, n_rot, nnz)}


def stagewise_rotation_units(w):
    """Limb-units (8N bytes) one rotation moves when every stage of the textbook hybrid key switch goes
    through HBM exactly once: inverse transform of c1, ModUp, transform of the raised digits, key inner
    product, inverse transform of the special limbs, ModDown, transform back, combination with c0."""
    L, K = w.q_count, w.p_count
    beta = -(-L // w.alpha)
    ext = L + K
    E = beta * ext - L
    return 2 * L + (L + E) + 2 * E + (3 * beta * ext + 2 * ext) + 4 * K + (2 * K + 2 * L) + 4 * L + 7 * L


def ntt_leg(ctx, w, n_limbs=1024, reps=5):
    """Stand-alone transform throughput (row (a1) of the scope table): n_limbs limb rows of N words, forward then
    inverse, in place, timed by the library's per-kernel HIP events; once on 50-bit ciphertext primes (the fp64-assisted
    kernels) and once on the 60-bit special primes (integer kernels).  Algorithmic bytes: a transform reads and
    writes its limb once (2 limb-units); the two-pass implementation moves each limb twice (4 limb-units)."""
    import torch
    N = w.N
    buf = torch.randint(0, 1 << 49, (n_limbs, N), dtype=torch.int64, device="cuda")
    out = {}
    for tag, primes in (("q50", list(range(w.q_count))), ("p60", list(range(w.q_count, w.q_count + w.p_count)))):
        idx = [primes[r % len(primes)] for r in range(n_limbs - n_limbs % len(primes))]
        rows = len(idx)
        ctx.ntt(buf.data_ptr(), idx, inverse=False)
        ctx.ntt(buf.data_ptr(), idx, inverse=True)
        torch.cuda.synchronize()
        ctx.profile_read()
        ctx.profile_enable(True)
        for _ in range(reps):
            ctx.ntt(buf.data_ptr(), idx, inverse=False)
            ctx.ntt(buf.data_ptr(), idx, inverse=True)
        torch.cuda.synchronize()
        prof = ctx.profile_read()
        ctx.profile_enable(False)
        ms = sum(prof.get(k, (0.0, 0))[0] for k in ("ntt_fwd_cols", "ntt_fwd_rows", "ntt_inv_rows", "ntt_inv_cols")) / reps
        units = 2 * rows  # transforms per repetition (forward + inverse of every row)
        gbs2 = units * 2 * 8.0 * N / (ms * 1e-3) / 1e9
        out[tag] = {"limbs": rows, "ms_fwd_plus_inv": round(ms, 4), "transforms_per_s": units / (ms * 1e-3),
                    "GB/s_at_2_units": round(gbs2, 1), "frac_at_2_units": round(gbs2 / HBM_PEAK_GBS, 4),
                    "GB/s_at_4_units": round(2 * gbs2, 1), "frac_at_4_units": round(2 * gbs2 / HBM_PEAK_GBS, 4),
                    "kernels_ms": {k: round(v[0] / reps, 4) for k, v in sorted(prof.items()) if v[1]}}
    del buf
    return out


def run_leg(name, steps, warmup, separate_rescale=False, with_ntt=False):
    """One workload: set-up, timed steps, decrypted check, per-kernel profile.  Returns the leg's dictionary."""
    w = wl.BY_NAME[name]
    t0 = time.time()
    r = Runner(w, separate_rescale=separate_rescale)
    try:
        r.setup()
        log("%s: set-up done in %.1f s" % (name, time.time() - t0))
        ms = time_steps(r, steps, warmup)
        err = r.check()
        prof = kernel_profile(r)
        dom, roof = roofline_for(w, prof)
        if roof["bound"] == "mfma":
            # the data-sheet peak assumes 2.4 GHz; under matrix load the chip holds a lower clock.  A register-only loop of
            # the same matrix instruction, run right after the timed steps, gives the rate the pipes sustain on this
            # machine: the second ceiling the contraction is compared with.
            sustained = r.ctx.matrix_rate_probe(0.4) / 1e12
            roof["sustained_peak_measured"] = round(sustained, 1)
            roof["frac_of_sustained"] = round(roof["achieved"] / sustained, 4)
        log("%s: %.3f ms/step over %d steps, decrypted max abs error %.3e, dominant kernel %s" % (name, ms, steps, err, dom))
        leg = {"workload": name, "ms_per_step": ms, "steps": steps, "decrypt_max_abs_err": err, "roofline": roof,
               "kernels_ms_per_step": {k: {"ms": round(v[0], 4), "launches": v[1]} for k, v in sorted(prof.items())},
               "hbm_kernels": hbm_fractions(w, prof)}
        if hasattr(r, "prepare_ms"):
            leg["prepare_ms"] = r.prepare_ms
        if w.name == "keyswitch":
            rps = w.batch / (ms * 1e-3)
            gbs = rps * stagewise_rotation_units(w) * 8.0 * w.N / 1e9
            leg.update({"value": rps, "unit": "rotations/s", "ms_per_batch": ms,
                        "stagewise": {"units_per_rotation": stagewise_rotation_units(w), "GB/s": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}})
        if with_ntt:
            leg["ntt"] = ntt_leg(r.ctx, w)
        return leg
    finally:
        r.close()


def compact(leg):
    """What the extra legs contribute to the line: time, error, dominant kernel and its fraction."""
    roof = leg["roofline"]
    out = {"ms_per_step": round(leg["ms_per_step"], 3), "decrypt_max_abs_err": leg["decrypt_max_abs_err"], "dominant_kernel": roof["kernel"],
           "bound": roof["bound"], "frac": round(roof["frac"], 4), "kernels_ms_per_step": {k: v["ms"] for k, v in leg["kernels_ms_per_step"].items()}}
    if "frac_own_work" in roof:
        out["frac_own_work"] = round(roof["frac_own_work"], 4)
    if "prepare_ms" in leg:
        out["prepare_ms"] = round(leg["prepare_ms"], 1)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="ffn2560", choices=[w.name for w in wl.WORKLOADS])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-keyswitch-leg", action="store_true")
    ap.add_argument("--no-extra-legs", action="store_true",
                    help="skip the compact legs of the other BASELINE matmul configurations and of the NEXT-row workloads")
    ap.add_argument("--separate-rescale", action="store_true",
                    help="FFN workload: run scalar-multiply + rescale as its own in-place pass instead of inside the second layer")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB read + 1 GiB write elementwise kernel (calibrates profiler byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP library has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    torch.cuda.init()
    w = wl.BY_NAME[args.workload]
    log("workload %s on %s" % (w.name, torch.cuda.get_device_name(0)))
    main_leg = run_leg(w.name, args.steps, args.warmup, separate_rescale=args.separate_rescale, with_ntt=(w.name == "keyswitch"))
    ms = main_leg["ms_per_step"]
    line = {
        "metric": "encrypted ternary matmul ms/layer + key-switched rotations/sec at N=2^16",
        "value": ms, "unit": "ms/layer" if (w.name != "keyswitch" and w.op == "matmul") else "ms/batch",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": w.name, "log_n": w.log_n, "q_limbs": w.q_count, "p_limbs": w.p_count, "alpha": w.alpha,
                   "tokens": w.tokens, "d_in": w.d_in, "d_mid": w.d_mid, "d_out": w.d_out, "placement": w.placement},
        "decrypt_max_abs_err": main_leg["decrypt_max_abs_err"], "roofline": main_leg["roofline"],
        **({"prepare_ms": main_leg["prepare_ms"]} if "prepare_ms" in main_leg else {}),
        "kernels_ms_per_step": main_leg["kernels_ms_per_step"], "hbm_kernels": main_leg["hbm_kernels"],
    }
    if w.name == "keyswitch":
        line["rotations"] = {k: main_leg[k] for k in ("value", "unit", "stagewise")}
        line["rotations"]["workload"] = "keyswitch"
        line["ntt"] = main_leg["ntt"]
    if args.copy_probe:
        a = torch.zeros(1 << 27, dtype=torch.int64, device="cuda")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        torch.add(a, 1, out=b)
        torch.cuda.synchronize()
        del a, b
    if w.name != "keyswitch" and not args.no_keyswitch_leg:
        # BASELINE configs[1]: the rotations/s half of the metric, with the stand-alone transform beside it
        # (a batch takes under 4 ms: 20 timed batches, so that the first launch's latency does not show in the mean)
        k = run_leg("keyswitch", max(args.steps, 20), max(args.warmup, 2), with_ntt=True)
        line["rotations"] = {"value": k["value"], "unit": "rotations/s", "workload": "keyswitch", "ms_per_batch": k["ms_per_batch"],
                             "steps": k["steps"],
                             "stagewise": k["stagewise"], "decrypt_max_abs_err": k["decrypt_max_abs_err"], "roofline": k["roofline"],
                             "hbm_kernels": k["hbm_kernels"], "kernels_ms_per_step": k["kernels_ms_per_step"]}
        line["ntt"] = k["ntt"]
        log("key-switch leg: %.1f rotations/s" % k["value"])
    if w.name == "ffn2560" and not args.no_extra_legs:
        # the metric is ms/layer on the three BitNet-shaped configurations: the other two as compact legs, then the rows
        # beyond the hot path (Alg. 2, the merge, the two attention products).  A leg that fails is reported, not fatal.
        n_extra = min(args.steps, 5)
        for key, names in (("other_configs", ["attn2560", "proj768"]), ("next_rows", ["rope1536", "merge1536", "ccmmqkseg", "ccmmavseg"])):
            line[key] = {}
            for name in names:
                try:
                    line[key][name] = compact(run_leg(name, n_extra, 1))
                except Exception as e:  # noqa: BLE001
                    line[key][name] = {"error": "%s: %s" % (type(e).__name__, e)}
                    log("%s failed: %s" % (name, e))
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
