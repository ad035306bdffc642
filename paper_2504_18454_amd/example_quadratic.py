"""Worked example: PALSGD on a noisy quadratic, driven through the library the way a training loop would.

K workers minimise f(x) = 0.5 |x - c|^2 from noisy gradients g_k = (x_k - c) + sigma N(0,1):
a DDP warm-up (Sec. 4.3), then Alg. 1 with AdamW inside, Nesterov outside, gradient clipping,
and the consensus distance of App. A.3 reported at every synchronisation.  Everything that
touches the model runs in the library's kernels; PyTorch only allocates and draws the noise.

    python -m paper_2504_18454_amd.example_quadratic
"""
from __future__ import annotations

import torch

from . import Palsgd, make_config, palsgd_layout


def run(K=8, numels=(50000, 1000, 64), warmup=20, steps=200, H=10, p=0.1, alpha=0.02, eta=1.0, sigma=0.1,
        clip=50.0, seed=0, device="cuda:0", verbose=True):
    dev = torch.device(device)
    cfg = make_config(K, list(numels), inner="adamw", grad_dtype="f32", p=p, H=H, weight_decay=0.0,
                      outer_lr=0.7, outer_momentum=0.5, outer_nesterov=True, seed=seed)
    row, offs = palsgd_layout(cfg)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    real = torch.zeros(row, dtype=torch.bool, device=dev)
    for o, n in zip(offs, numels):
        real[o:o + n] = True
    f = torch.float32
    c = torch.randn(row, dtype=f, device=dev, generator=gen) * real
    x0 = torch.zeros(row, dtype=f, device=dev)
    X, M, V, G = (torch.empty((K, row), dtype=f, device=dev) for _ in range(4))
    XG, OM = (torch.empty(row, dtype=f, device=dev) for _ in range(2))
    opt = Palsgd(cfg, X, M, V, G, XG, OM, row, x0=x0)
    diag = torch.zeros(2, dtype=f, device=dev)
    history = []

    def gradients(model):
        torch.sub(model, c, out=G) if model.dim() == 2 else G.copy_((model - c).expand_as(G))
        G.add_(torch.randn(G.shape, dtype=f, device=dev, generator=gen), alpha=sigma)
        G.mul_(real)

    for t in range(warmup):                       # DDP warm-up: every worker applies the averaged gradient
        gradients(XG)                             # one common model during the warm-up: XG (the rows of X follow later)
        opt.palsgd_clip_mean_grad_norm(clip)      # DDP clips the averaged gradient
        opt.palsgd_ddp_step_shared(t, alpha)
    for t in range(steps):                        # PALSGD phase, t counted from 0 again
        if t == 0:
            opt.palsgd_ddp_finish()               # every worker gets its model row and InnerOPT state
        gradients(X)
        opt.palsgd_clip_grad_norm(clip)
        opt.palsgd_step(t, alpha, eta)
        if (t + 1) % H == 0:
            opt.palsgd_outer_step_diag(t, diag)
            err = float((XG - c).norm() / c.norm())
            xi, d2 = diag.tolist()
            history.append((t + 1, err, xi, d2))
            if verbose:
                print(f"t={t + 1:4d}  |x - c|/|c| = {err:.4f}   consensus distance before the sync = {xi:.4e}   |Delta|^2 = {d2:.4e}")
    opt.palsgd_diagnostics(diag)
    after = diag.tolist()
    opt.palsgd_destroy()
    return history, after


if __name__ == "__main__":
    run()
