"""Harness shared by the GPU parity tests: runs Alg. 1 on the device library and on the CPU
oracle from the same seeded inputs and compares element by element.

The path is separable per element index (element i of the K replicas plus per-replica
scalars), so the oracle may run on any subset S of a row's indices and still be exact.
Small cases take S = every index.  Full-size cases keep full buffers on the device and a
compact copy of S on the host.  Gradients at S follow the closed loop on the oracle's side,
g_k = (x_k - c) + sigma N(0,1) from the oracle's own x_k, rounded to the gradient dtype, and
are uploaded into the device's G at S; elsewhere G is seeded device noise that depends on
nothing the device path computed.  No oracle input comes from the device path.
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2504_18454_amd import Palsgd, make_config, palsgd_layout
from paper_2504_18454_amd.workloads import from_bf16_bits, to_bf16_bits

RTOL, ATOL = 1e-5, 1e-7      # |gpu - ora| <= RTOL |ora| + ATOL per element after all steps


def sample_indices(numels, offsets, row, per_edge, n_random, seed):
    """Sorted unique row positions: first/last `per_edge` elements of every tensor, `n_random`
    random positions, and every padding element next to a sampled edge."""
    if per_edge is None:
        return np.arange(row, dtype=np.int64)
    rng = np.random.default_rng(seed)
    parts = [rng.integers(0, row, size=n_random, dtype=np.int64)]
    for o, n in zip(offsets, numels):
        e = min(per_edge, n)
        parts.append(np.arange(o, o + e, dtype=np.int64))
        end_pad = (o + n + 63) // 64 * 64
        parts.append(np.arange(o + n - e, end_pad, dtype=np.int64))
    return np.unique(np.concatenate(parts))


def compact_table(idx, numels, offsets):
    """Tensor table of the compact row that holds only the sampled positions."""
    lo = np.searchsorted(idx, np.asarray(offsets, dtype=np.int64), side="left")
    hi = np.searchsorted(idx, np.asarray(offsets, dtype=np.int64) + np.asarray(numels, dtype=np.int64), side="left")
    return lo.astype(np.uint64), (hi - lo).astype(np.uint64)


class Run:
    def __init__(self, K, numels, *, inner="adamw", grad_dtype="f32", p=0.1, H=16, alpha=1e-3, eta=16.0,
                 sigma=0.01, seed=0, wd_mult=None, per_edge=None, n_random=0, row_extra=0, device="cuda:0",
                 fill_noise=True, c_scale=1.0, moment_floor_by_gradient=False, **hyper):
        self.K, self.numels, self.inner, self.grad_dtype = K, list(numels), inner, grad_dtype
        self.p, self.H, self.alpha, self.eta, self.sigma, self.seed = p, H, alpha, eta, sigma, seed
        self.dev = torch.device(device)
        self.cfg = make_config(K, numels, inner=inner, grad_dtype=grad_dtype, p=p, H=H, seed=seed,
                               wd_mult=wd_mult, **hyper)
        self.row, self.offsets = palsgd_layout(self.cfg)
        self.stride = self.row + 64 * row_extra
        self.idx = sample_indices(self.numels, self.offsets, self.row, per_edge, n_random, seed + 1)
        self.full = per_edge is None
        self.fill_noise = fill_noise and not self.full
        # which sampled positions are tensor elements (not padding)
        self.real_s = np.zeros(self.idx.size, bool)
        for o, n in zip(self.offsets, self.numels):
            a, b = np.searchsorted(self.idx, [o, o + n])
            self.real_s[a:b] = True
        self.rng = np.random.default_rng(seed + 2)
        self.gen = torch.Generator(device=self.dev)
        self.gen.manual_seed(seed + 3)
        # seeded inputs: x0 on the device (padding zero), target c only where the oracle looks
        f = torch.float32
        x0 = torch.empty(self.row, dtype=f, device=self.dev)
        x0.normal_(0.0, 0.02, generator=self.gen)
        pad = torch.ones(self.row, dtype=torch.bool, device=self.dev)
        for o, n in zip(self.offsets, self.numels):
            pad[o:o + n] = False
        self.pad_idx = pad.nonzero().flatten()
        del pad
        x0.index_fill_(0, self.pad_idx, 0.0)
        self.idx_dev = torch.from_numpy(self.idx).to(self.dev)
        x0_s = x0[self.idx_dev].cpu().numpy()
        # quadratic target c ~ c_scale N(0,1): gradients are of order c_scale, which sets how much absolute
        # rounding error fp32 sums of them carry against the tolerance's 1e-7 floor
        self.c_s = np.where(self.real_s, np.float32(c_scale) * self.rng.standard_normal(self.idx.size, dtype=np.float32),
                            np.float32(0))
        # device buffers (caller-owned)
        KS = (K, self.stride)
        self.X = torch.empty(KS, dtype=f, device=self.dev)
        self.M = torch.empty(KS, dtype=f, device=self.dev)
        self.V = torch.empty(KS, dtype=f, device=self.dev) if inner == "adamw" else None
        gdt = torch.float32 if grad_dtype == "f32" else torch.bfloat16
        self.G = torch.zeros(KS, dtype=gdt, device=self.dev)
        self.XG = torch.empty(self.stride, dtype=f, device=self.dev)
        self.OM = torch.empty(self.stride, dtype=f, device=self.dev)
        self.OV = torch.empty(self.stride, dtype=f, device=self.dev) if hyper.get("outer_opt") == "adamw" else None
        if row_extra:                      # sentinel beyond the padded row: must never be touched
            for t_ in self.state_arrays():
                t_[..., self.row:] = 777.0
        self.lib = Palsgd(self.cfg, self.X, self.M, self.V, self.G, self.XG, self.OM, self.stride, x0=x0, OV=self.OV)
        torch.cuda.synchronize()
        # oracle over the compact row
        coff, cnum = compact_table(self.idx, self.numels, self.offsets)
        keep = cnum > 0
        wdm = None if wd_mult is None else np.asarray(wd_mult, np.float32)[keep]
        self.ora = oracle.OracleState(K, x0_s, coff[keep], cnum[keep], inner=inner, grad_dtype=grad_dtype, p=p, H=H,
                                      seed=seed, wd_mult=wdm, **hyper)
        self.t = 0
        # Optional reading of the tolerance's absolute floor for the SGD-momentum buffer (see compare()): a running
        # maximum, per worker and position, of |g_hat| (the scaled gradient InnerOPT was fed) and of the buffer itself.
        self.moment_floor_by_gradient = moment_floor_by_gradient
        self.gmax = np.zeros((K, self.idx.size), np.float64)

    def state_arrays(self):
        return tuple(t for t in (self.X, self.M, self.XG, self.OM, self.V, self.OV) if t is not None)

    # ------------------------------------------------------------------ one iteration
    def oracle_side_gradients(self):
        """Closed loop on the oracle's side at the sampled positions: sets the oracle's G and returns the same
        bits as a device tensor [K, len(idx)] in the gradient dtype."""
        g = (self.ora.X - self.c_s[None, :]) + np.float32(self.sigma) * self.rng.standard_normal(
            self.ora.X.shape, dtype=np.float32)
        g = np.where(self.real_s[None, :], g, np.float32(0)).astype(np.float32)
        if self.grad_dtype == "f32":
            self.ora.G[...] = g
            return torch.from_numpy(g).to(self.dev)
        bits = to_bf16_bits(g)
        self.ora.G[...] = bits
        return torch.from_numpy(bits.view(np.int16)).to(self.dev).view(torch.bfloat16)

    def make_gradients(self):
        """Oracle-side closed loop at the sampled positions; seeded noise elsewhere on the device."""
        K = self.K
        gd = self.oracle_side_gradients()
        if self.fill_noise:
            for k in range(K):
                row = self.G[k, :self.row]
                if self.grad_dtype == "f32":
                    row.normal_(0.0, 1.0, generator=self.gen)
                else:
                    tmp = torch.empty(self.row, dtype=torch.float32, device=self.dev)
                    tmp.normal_(0.0, 1.0, generator=self.gen)
                    row.copy_(tmp)
                    del tmp
                row.index_fill_(0, self.pad_idx, 0)
        for k in range(K):
            self.G[k].index_copy_(0, self.idx_dev, gd[k])

    def iterate(self, steps, *, fused=True, grad_scale=None, mask_fn=None, check_every=0, clip=None, diag_outer=False,
                fused_sync=False):
        for _ in range(steps):
            t = self.t
            self.make_gradients()
            mo = None if mask_fn is None else np.asarray(mask_fn(t), np.uint8)
            gs64 = None if grad_scale is None else np.asarray(grad_scale, np.float32).astype(np.float64)
            if clip is not None:
                # global-norm clipping: a reduction over the whole row, so only for full-coverage runs
                assert self.full
                norms_dev = torch.empty(self.K, dtype=torch.float32, device=self.dev)
                self.lib.palsgd_clip_grad_norm(clip, norms_dev)
                norms = self.ora.grad_norms()
                np.testing.assert_allclose(norms_dev.cpu().numpy(), norms, rtol=1e-5)
                scales = np.array([oracle.clip_scale(v, float(np.float32(clip))) for v in norms])
                gs64 = scales if gs64 is None else gs64 * scales
                self.last_scales = scales
            self.note_gradients(gs64)
            if diag_outer:                 # oracle: local update, a look at the state, then the outer step
                mask_o = self.ora.local_step(t, self.alpha, self.eta, grad_scale=gs64, mask_override=mo)
                synced = (t + 1) % self.H == 0
                if synced:
                    assert self.full
                    want_diag = self.ora.diagnostics()
                    ora_x, ora_xg = self.ora.X.astype(np.float64), self.ora.XG.astype(np.float64)
                    self.ora.outer_step()
            else:
                mask_o, synced = self.ora.iteration(t, self.alpha, self.eta, grad_scale=gs64, mask_override=mo)
            if mo is None:
                assert np.array_equal(self.lib.palsgd_draw(t), mask_o), f"draws differ at t={t}"
            if fused_sync and (t + 1) % self.H == 0:   # local update and outer step of a sync step in one launch
                assert synced
                self.lib.palsgd_step_sync(t, self.alpha, self.eta, grad_scale, mo)
                self.t += 1
                continue
            if fused:
                self.lib.palsgd_step(t, self.alpha, self.eta, grad_scale, mo)
            else:                          # the two branches as separate calls, mixing first
                self.lib.palsgd_pseudo_sync(t, self.alpha, self.eta, mo)
                self.lib.palsgd_inner_step(t, self.alpha, grad_scale, mo)
            if (t + 1) % self.H == 0:
                assert synced
                if diag_outer:
                    out = torch.empty(2, dtype=torch.float32, device=self.dev)
                    slack = self.diagnostics_slack(ora_x, ora_xg)       # from the device's state before the outer step
                    self.lib.palsgd_outer_step_diag(t, out)
                    self.assert_diagnostics(out.cpu().numpy(), want_diag, slack)
                    self.last_diag = want_diag
                else:
                    self.lib.palsgd_outer_step(t)
            self.t += 1
            if check_every and self.t % check_every == 0:
                self.compare()
        torch.cuda.synchronize()

    def ddp_iterate(self, steps, grad_scale=None, clip=None, shared=False):
        """DDP warm-up steps: every worker applies the update of the averaged gradient (clipped by the
        norm of that average when `clip` is given; a whole-row reduction, so full-coverage runs only).
        shared: through palsgd_ddp_step_shared, which leaves the rows of X to the end of the warm-up."""
        gs64 = None if grad_scale is None else np.asarray(grad_scale, np.float32).astype(np.float64)
        for _ in range(steps):
            self.make_gradients()
            gs_o = gs64
            if clip is not None:
                assert self.full
                norm_dev = torch.empty(1, dtype=torch.float32, device=self.dev)
                self.lib.palsgd_clip_mean_grad_norm(clip, grad_scale, norm_dev)
                norm = self.ora.mean_grad_norm(gs64)
                np.testing.assert_allclose(float(norm_dev), norm, rtol=1e-5)
                scale = oracle.clip_scale(norm, float(np.float32(clip)))
                gs_o = (np.ones(self.K) if gs64 is None else gs64) * scale
                self.last_scales = np.array([scale])
            self.note_gradients(gs_o, averaged=True)
            self.ora.ddp_step(self.alpha, grad_scale=gs_o)
            (self.lib.palsgd_ddp_step_shared if shared else self.lib.palsgd_ddp_step)(self.t, self.alpha, grad_scale)
            self.t += 1
        torch.cuda.synchronize()

    def note_gradients(self, gs64, averaged=False):
        """Running maximum, per worker and position, of |g_hat| (g_hat = scale * g as the oracle's InnerOPT is
        about to see it; in a DDP step every worker sees the average, bounded here by the largest worker's)."""
        if not self.moment_floor_by_gradient:
            return
        g = self.ora.G if self.grad_dtype == "f32" else from_bf16_bits(self.ora.G)
        g = np.abs(g.astype(np.float64))
        if gs64 is not None:
            g = g * np.abs(np.asarray(gs64, np.float64))[:, None]
        if averaged:
            g = np.broadcast_to(g.max(axis=0)[None, :], g.shape)
        np.maximum(self.gmax, g, out=self.gmax)
        np.maximum(self.gmax, np.abs(self.ora.M.astype(np.float64)), out=self.gmax)   # and of the moment itself

    def diagnostics_slack(self, ora_x, ora_xg):
        """How far the two sides' diagnostics may differ, given how far their states differ right now.

        Xi and |Delta|^2 are sums of squares of differences of nearby numbers, each side's taken from its own
        fp32 state.  With delta = the largest |device - oracle| over X and XG at this moment, every difference
        d = x_k - x moves by at most 2 delta, so sum d^2 moves by at most sum (4 delta |d| + 4 delta^2); the same
        holds for Delta = x - mean_k x_k.  Returns (slack of Xi, slack of |Delta|^2); the fp32 summation of the
        device adds 1e-5 relative on top (assert_diagnostics)."""
        assert self.full
        torch.cuda.synchronize()
        dx = np.abs(self.device_sample(self.X).astype(np.float64) - ora_x).max()
        dg = np.abs(self.device_sample(self.XG).astype(np.float64) - ora_xg).max()
        delta = max(dx, dg)
        d = np.abs(ora_x - ora_xg[None, :])
        big = np.abs(ora_xg - ora_x.mean(axis=0))
        xi_slack = (4 * delta * d.sum() + 4 * delta * delta * d.size) / self.K
        d2_slack = 4 * delta * big.sum() + 4 * delta * delta * big.size
        return xi_slack, d2_slack

    @staticmethod
    def assert_diagnostics(got, want, slack):
        for name, g, w, s_ in zip(("Xi", "|Delta|^2"), got, want, slack):
            assert abs(float(g) - w) <= s_ + 1e-5 * abs(w) + 1e-30, (name, float(g), w, s_)

    def compare_diagnostics(self):
        assert self.full
        out = torch.empty(2, dtype=torch.float32, device=self.dev)
        slack = self.diagnostics_slack(self.ora.X.astype(np.float64), self.ora.XG.astype(np.float64))
        self.lib.palsgd_diagnostics(out)
        got = out.cpu().numpy().astype(np.float64)
        self.assert_diagnostics(got, self.ora.diagnostics(), slack)
        return got

    # ------------------------------------------------------------------ comparison
    def device_sample(self, T):
        if T.dim() == 1:
            return T[self.idx_dev].cpu().numpy()
        return torch.stack([T[k][self.idx_dev] for k in range(T.shape[0])]).cpu().numpy()

    def compare(self, rtol=RTOL, atol=ATOL, check_state=True):
        torch.cuda.synchronize()
        if check_state:
            tau, n_outer = self.lib.palsgd_get_state()
            assert tau == [int(v) for v in self.ora.tau], (tau, self.ora.tau)
            assert n_outer == self.ora.n_outer
        worst = {}
        pairs = [("X", self.X, self.ora.X), ("M", self.M, self.ora.M), ("XG", self.XG, self.ora.XG),
                 ("OM", self.OM, self.ora.OM)]
        if self.V is not None:
            pairs.append(("V", self.V, self.ora.V))
        if self.OV is not None:
            pairs.append(("OV", self.OV, self.ora.OV))
        for name, dev_t, want in pairs:
            got = self.device_sample(dev_t)
            assert np.isfinite(got).all(), name
            err = np.abs(got.astype(np.float64) - want.astype(np.float64))
            bound = rtol * np.abs(want.astype(np.float64)) + atol
            if name == "M" and self.moment_floor_by_gradient and self.inner == "sgdm":
                # The SGD-momentum buffer is a signed running sum of about 1/(1-mu) = 10 scaled gradients, stored in
                # fp32 on both sides, each side rounding its own copy at every step: e_t = mu e_(t-1) + rho_t with
                # |rho_t| <= 2^-24 (2 |buf_t| + |d_t|), d_t the term added at step t.  Where the buffer has cancelled
                # to near zero it still carries that history, up to 2^-24 (2 max|buf| + max|d|) / (1 - mu) in the
                # worst case (1.8e-6 at unit size for mu = 0.9) and about 1e-7 of its largest value in practice,
                # whatever its present size.  The fixed 1e-7 floor holds while the buffer stays around one; runs
                # at the benchmark configurations' gradient scale with caller-side multipliers up to 2 (|g_hat| up to
                # 9, buffer up to 20) state the floor as 1e-7 times the largest |g_hat| and |buf| of the worker's
                # row over the run.  AdamW's first moment is an AVERAGE of the gradients and keeps the fixed floor
                # at that scale too (observed: at most a quarter of it).
                worst["M_fixed_floor"] = float((err / bound).max())
                np.maximum(self.gmax, np.abs(want.astype(np.float64)), out=self.gmax)
                bound = rtol * np.abs(want.astype(np.float64)) + atol * np.maximum(1.0, self.gmax.max(axis=1, keepdims=True))
            worst[name] = float((err / bound).max())
            bad = err > bound
            if bad.any():
                w_ = np.unravel_index(np.argmax(err / bound), err.shape)
                detail = f"worst at {w_}: device {got[w_]!r}, oracle {want[w_]!r}, bound {bound[w_]:.3g}"
                if name == "M" and self.moment_floor_by_gradient and self.inner == "sgdm":
                    detail += f", largest |g_hat|, |M| seen there {self.gmax[w_]:.3g}, in the row {self.gmax[w_[0]].max():.3g}"
                raise AssertionError(f"{name}: {int(bad.sum())} of {bad.size} elements outside tolerance at t={self.t}; "
                                     f"worst err/bound {worst[name]:.3g}; {detail}")
        if self.stride > self.row:
            for T in self.state_arrays():
                assert bool((T[..., self.row:] == 777.0).all()), "wrote beyond the padded row"
        # padding stays exactly zero on the device
        if self.pad_idx.numel():
            assert not bool(self.X.index_select(1, self.pad_idx).any()), "padding of X became non-zero"
            assert not bool(self.XG.index_select(0, self.pad_idx).any()), "padding of XG became non-zero"
        return worst

    def close(self):
        self.lib.palsgd_destroy()


def periodic_counts(numels, offsets, B):
    """count[j] = how many tensor elements (not padding) of a padded row sit at positions i with i mod B == j."""
    count = np.zeros(B, np.int64)
    for o, n in zip(offsets, numels):
        full, rest = divmod(int(n), B)
        count += full
        a = int(o) % B
        if a + rest <= B:
            count[a:a + rest] += 1
        else:
            count[a:] += 1
            count[:a + rest - B] += 1
    return count


class PeriodicRun:
    """A full-size run in which EVERY element is checked, not a sample.

    All inputs repeat along a row with period B (x0, the quadratic's target, the gradient noise), and the
    weight decay is uniform, so position i of a row must follow the oracle's trajectory of position i mod B:
    the update is element-wise.  The oracle runs on one period (K rows of B elements); the device runs the
    full-size buffers in the launch configuration of the benchmark; the comparison covers all K * row
    elements of X, M, V and all of XG, OM, to the same tolerance as everywhere else.  Padding between
    tensors holds zeros in x0 and in the gradients and must still be exactly zero at the end.
    The gradients are closed-loop on the oracle's side: g = (x_k - c) + sigma * noise from the oracle's x_k.
    """

    def __init__(self, K, numels, *, B=1 << 16, inner="adamw", grad_dtype="f32", p=0.1, H=16, alpha=1e-3, eta=16.0,
                 sigma=0.01, seed=0, device="cuda:0", **hyper):
        self.K, self.B, self.grad_dtype = K, B, grad_dtype
        self.p, self.H, self.alpha, self.eta, self.sigma = p, H, alpha, eta, sigma
        self.dev = torch.device(device)
        self.cfg = make_config(K, numels, inner=inner, grad_dtype=grad_dtype, p=p, H=H, seed=seed, **hyper)
        self.row, offsets = palsgd_layout(self.cfg)
        self.count = periodic_counts(numels, offsets, B).astype(np.float64)
        self.reps, self.tail = divmod(self.row, B)
        self.rng = np.random.default_rng(seed + 2)
        x0_b = (np.float32(0.02) * self.rng.standard_normal(B, dtype=np.float32)).astype(np.float32)
        self.c_b = self.rng.standard_normal(B, dtype=np.float32)
        pad = torch.ones(self.row, dtype=torch.bool, device=self.dev)
        for o, n in zip(offsets, numels):
            pad[o:o + n] = False
        self.pad_idx = pad.nonzero().flatten()
        del pad
        f = torch.float32
        x0 = torch.empty(self.row, dtype=f, device=self.dev)
        self.tile_into(x0, torch.from_numpy(x0_b).to(self.dev))
        KS = (K, self.row)
        self.X = torch.empty(KS, dtype=f, device=self.dev)
        self.M = torch.empty(KS, dtype=f, device=self.dev)
        self.V = torch.empty(KS, dtype=f, device=self.dev) if inner == "adamw" else None
        self.G = torch.zeros(KS, dtype=f if grad_dtype == "f32" else torch.bfloat16, device=self.dev)
        self.XG = torch.empty(self.row, dtype=f, device=self.dev)
        self.OM = torch.empty(self.row, dtype=f, device=self.dev)
        self.lib = Palsgd(self.cfg, self.X, self.M, self.V, self.G, self.XG, self.OM, self.row, x0=x0)
        torch.cuda.synchronize()
        del x0
        self.ora = oracle.OracleState(K, x0_b, [0], [B], inner=inner, grad_dtype=grad_dtype, p=p, H=H, seed=seed, **hyper)
        self.t = 0

    def tile_into(self, dst_row, block):
        """dst_row[i] = block[i mod B] over the padded row, zero on the padding between tensors."""
        n = self.reps * self.B
        if self.reps:
            dst_row[:n].view(self.reps, self.B).copy_(block.unsqueeze(0).expand(self.reps, self.B))
        if self.tail:
            dst_row[n:self.row].copy_(block[:self.tail])
        if self.pad_idx.numel():
            dst_row.index_fill_(0, self.pad_idx, 0)

    def make_gradients(self):
        g = (self.ora.X - self.c_b[None, :]) + np.float32(self.sigma) * self.rng.standard_normal(
            self.ora.X.shape, dtype=np.float32)
        g = g.astype(np.float32)
        if self.grad_dtype == "f32":
            self.ora.G[...] = g
            gd = torch.from_numpy(g).to(self.dev)
        else:
            bits = to_bf16_bits(g)
            self.ora.G[...] = bits
            gd = torch.from_numpy(bits.view(np.int16)).to(self.dev).view(torch.bfloat16)
        for k in range(self.K):
            self.tile_into(self.G[k], gd[k])

    def block_gradients(self):
        g = self.ora.G if self.grad_dtype == "f32" else from_bf16_bits(self.ora.G)
        return g.astype(np.float64)

    def row_norms(self):
        """L2 norm of every worker's full-size gradient row, from one period: position i holds the block's
        value at i mod B on tensor elements and zero on padding, so the sum of squares is sum_j count[j] g[j]^2."""
        return np.sqrt((self.block_gradients() ** 2 * self.count[None, :]).sum(axis=1))

    def mean_row_norm(self):
        """The same for the full-size row of the averaged gradient (1/K) sum_k g_k."""
        return float(np.sqrt((self.block_gradients().mean(axis=0) ** 2 * self.count).sum()))

    def ddp_iterate(self, steps, *, clip=None, shared=False):
        """DDP warm-up steps at full size, optionally clipped by the norm of the averaged gradient."""
        for _ in range(steps):
            self.make_gradients()
            gs = None
            if clip is not None:
                norm_dev = torch.empty(1, dtype=torch.float32, device=self.dev)
                self.lib.palsgd_clip_mean_grad_norm(clip, None, norm_dev)
                norm = self.mean_row_norm()
                np.testing.assert_allclose(float(norm_dev), norm, rtol=1e-5)
                self.last_scales = np.array([oracle.clip_scale(norm, float(np.float32(clip)))])
                gs = np.ones(self.K) * self.last_scales[0]
            self.ora.ddp_step(self.alpha, grad_scale=gs)
            (self.lib.palsgd_ddp_step_shared if shared else self.lib.palsgd_ddp_step)(self.t, self.alpha)
            self.t += 1
        torch.cuda.synchronize()

    def iterate(self, steps, *, fused_sync=False, clip=None):
        for _ in range(steps):
            t = self.t
            self.make_gradients()
            gs = None
            if clip is not None:                       # per-worker clipping by the global norm of the worker's gradient
                norms_dev = torch.empty(self.K, dtype=torch.float32, device=self.dev)
                self.lib.palsgd_clip_grad_norm(clip, norms_dev)
                norms = self.row_norms()
                np.testing.assert_allclose(norms_dev.cpu().numpy(), norms, rtol=1e-5)
                gs = self.last_scales = np.array([oracle.clip_scale(v, float(np.float32(clip))) for v in norms])
            mask_o, synced = self.ora.iteration(t, self.alpha, self.eta, grad_scale=gs)
            assert np.array_equal(self.lib.palsgd_draw(t), mask_o), f"draws differ at t={t}"
            assert synced == ((t + 1) % self.H == 0)
            if synced and fused_sync:
                self.lib.palsgd_step_sync(t, self.alpha, self.eta)
            else:
                self.lib.palsgd_step(t, self.alpha, self.eta)
                if synced:
                    self.lib.palsgd_outer_step(t)
            self.t += 1
        torch.cuda.synchronize()

    def compare(self, rtol=RTOL, atol=ATOL, chunk=1 << 26):
        """Every element of every state array against the oracle's value for its position mod B."""
        tau, n_outer = self.lib.palsgd_get_state()
        assert tau == [int(v) for v in self.ora.tau] and n_outer == self.ora.n_outer
        rows = [("XG", self.XG, self.ora.XG), ("OM", self.OM, self.ora.OM)]
        for k in range(self.K):
            rows += [(f"X[{k}]", self.X[k], self.ora.X[k]), (f"M[{k}]", self.M[k], self.ora.M[k])]
            if self.V is not None:
                rows.append((f"V[{k}]", self.V[k], self.ora.V[k]))
        want_row = torch.empty(self.row, dtype=torch.float32, device=self.dev)
        worst, checked = 0.0, 0
        for name, got, want in rows:
            self.tile_into(want_row, torch.from_numpy(np.ascontiguousarray(want)).to(self.dev))
            for a in range(0, self.row, chunk):
                w = want_row[a:a + chunk].double()
                gdev = got[a:a + chunk]
                assert bool(torch.isfinite(gdev).all()), name
                ratio = (gdev.double() - w).abs() / (rtol * w.abs() + atol)
                r = float(ratio.max())
                assert r <= 1.0, f"{name}: {int((ratio > 1).sum())} elements outside tolerance in [{a}, {a + chunk}), worst {r:.3g}"
                worst = max(worst, r)
                checked += gdev.numel()
            if self.pad_idx.numel():
                assert not bool(got.index_select(0, self.pad_idx).any()), f"{name}: padding became non-zero"
        return worst, checked

    def close(self):
        self.lib.palsgd_destroy()
