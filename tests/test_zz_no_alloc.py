"""palsgd_clip_grad_norm_noalloc, the entry point for callers that cannot allocate: through the C ABI, against
palsgd_clip_grad_norm on the same seeded inputs.  Both run the same kernels in the same order (only the memory
that holds the partial sums differs), so norms, scales and the step that consumes the scales agree bit for
bit; and both agree with the CPU checker to the tolerance of the other clipping tests."""
import ctypes as C

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import oracle  # noqa: E402
from paper_2504_18454_amd import Palsgd, PalsgdError, make_config, palsgd_layout  # noqa: E402
from paper_2504_18454_amd.workloads import from_bf16_bits  # noqa: E402


def _case(K, numels, grad_dtype, seed, max_norm):
    """One context pair over identical seeded buffers: clipping + gradient step through each entry point."""
    dev = torch.device("cuda:0")
    f = torch.float32
    outs = []
    for entry in ("palsgd_clip_grad_norm", "palsgd_clip_grad_norm_noalloc"):
        cfg = make_config(K, numels, grad_dtype=grad_dtype, p=0.0, H=4, seed=seed)
        row, offs = palsgd_layout(cfg)
        gen = torch.Generator(device=dev)
        gen.manual_seed(seed)
        real = torch.zeros(row, dtype=torch.bool, device=dev)
        for o, n in zip(offs, numels):
            real[o:o + n] = True
        x0 = torch.empty(row, dtype=f, device=dev).normal_(0.0, 0.02, generator=gen) * real
        X, M, V = (torch.empty((K, row), dtype=f, device=dev) for _ in range(3))
        XG, OM = (torch.empty(row, dtype=f, device=dev) for _ in range(2))
        G = torch.empty((K, row), dtype=f if grad_dtype == "f32" else torch.bfloat16, device=dev)
        for k in range(K):
            G[k].copy_(torch.empty(row, dtype=f, device=dev).normal_(0.0, 0.5 + 0.25 * k, generator=gen) * real)
        lib = Palsgd(cfg, X, M, V, G, XG, OM, row, x0=x0)
        norms = torch.full((K,), -1.0, dtype=f, device=dev)
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        getattr(lib, entry)(max_norm, norms)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before, "the call changed the amount of free device memory"
        lib.palsgd_step(0, 1e-3, 16.0, [1.0 + 0.5 * k for k in range(K)])      # consumes the scales
        torch.cuda.synchronize()
        outs.append(dict(norms=norms.cpu().numpy(), X=X.clone(), M=M.clone(), V=V.clone(), G=G, row=row, offs=offs,
                         tau=lib.palsgd_get_state()[0]))
        lib.palsgd_destroy()
    a, b = outs
    assert np.array_equal(a["norms"], b["norms"]) and (b["norms"] > 0).all()
    for name in ("X", "M", "V"):
        assert torch.equal(a[name], b[name]), name
    assert a["tau"] == b["tau"] == [1] * K
    # and against the CPU checker: norms, then the clipped step
    g = b["G"].cpu()
    g = g.numpy() if grad_dtype == "f32" else g.view(torch.int16).numpy().view(np.uint16)
    want = np.array([oracle.grad_norm(np.ascontiguousarray(g[k])) for k in range(K)])
    np.testing.assert_allclose(b["norms"], want, rtol=1e-5)
    assert (want > max_norm).any()                                              # the threshold was active
    x0h = (x0.cpu().numpy()).astype(np.float32)
    st = oracle.OracleState(K, x0h, b["offs"], numels, grad_dtype=grad_dtype, p=0.0, H=4, seed=seed)
    st.G[...] = g
    scales = np.array([oracle.clip_scale(v, float(np.float32(max_norm))) for v in want])
    st.local_step(0, 1e-3, 16.0, grad_scale=scales * np.array([1.0 + 0.5 * k for k in range(K)], np.float32).astype(np.float64))
    for name, got, ref in (("X", b["X"], st.X), ("M", b["M"], st.M), ("V", b["V"], st.V)):
        got = got.cpu().numpy().astype(np.float64)
        err = np.abs(got - ref.astype(np.float64))
        assert (err <= 1e-5 * np.abs(ref) + 1e-7).all(), (name, float(err.max()))


def test_noalloc_entry_equals_the_allocating_one_twice_in_a_row():
    # two calls in a row on one GPU, the second with a smaller input: what the first left in the static
    # array must not leak into the second
    _case(K=5, numels=[70000, 64, 1, 5000, 333, 2048, 17], grad_dtype="bf16", seed=91, max_norm=20.0)
    _case(K=2, numels=[700, 64, 3], grad_dtype="f32", seed=92, max_norm=2.0)


def test_noalloc_entry_rejects_what_the_static_array_cannot_hold():
    from paper_2504_18454_amd.binding import Buffers, lib
    cfg = make_config(64, [1 << 30])                     # 64 * 2^30 / 4096 = 2^24 partial sums > 2^22
    fake = 4096                                          # aligned, never dereferenced: the call fails before any launch
    b = Buffers(X=fake, M=fake, V=fake, G=fake, XG=fake, OM=fake, row_stride=1 << 30)
    ctx = C.c_void_p()
    assert lib().palsgd_init(C.byref(cfg), C.byref(b), None, None, C.byref(ctx)) == 0
    assert lib().palsgd_clip_grad_norm_noalloc(ctx, 1.0, None, None) == 1
    text = lib().palsgd_last_error(ctx).decode()
    assert "16777216" in text and "4194304" in text
    lib().palsgd_destroy(ctx)
