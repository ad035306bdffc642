"""GPU parity of the device-resident schedule (graph-capturable mode): draws, step counts and bias corrections
computed on the device must reproduce Alg. 1 exactly as the host-driven calls and the oracle do."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

RAGGED = [5000, 64, 1, 70000, 333, 2048, 17]


def _run(**kw):
    from parity import Run
    return Run(**kw)


@pytest.mark.parametrize("inner,grad_dtype,K,p", [("adamw", "f32", 5, 0.3), ("adamw", "bf16", 8, 0.05),
                                                 ("sgdm", "f32", 64, 0.25), ("adamw", "f32", 1, 0.5),
                                                 ("adamw", "bf16", 3, 0.0)])
def test_device_schedule_matches_oracle_and_hands_back_to_host(inner, grad_dtype, K, p):
    r = _run(K=K, numels=RAGGED, inner=inner, grad_dtype=grad_dtype, p=p, H=3, seed=50 + K, sigma=0.05,
             wd_mult=[1, 0, 1, 1, 0.5, 1, 0])
    r.iterate(2)                                          # host-driven first: the hand-over carries the step counts
    ae = torch.tensor([r.alpha, r.eta], dtype=torch.float32, device="cuda:0")
    r.lib.palsgd_capturable_begin(r.t)
    for _ in range(11):
        t = r.t
        r.make_gradients()
        _, synced = r.ora.iteration(t, r.alpha, r.eta)
        r.lib.palsgd_step_capturable(ae)
        if synced:
            r.lib.palsgd_outer_step(t)
        r.t += 1
    r.compare(check_state=False)
    assert r.lib.palsgd_capturable_end() == r.t
    r.compare()                                           # step counts read back from the device equal the oracle's
    r.iterate(4)                                          # and the host-driven path continues from them
    r.compare()
    r.close()


def test_host_driven_calls_are_refused_while_device_resident():
    from paper_2504_18454_amd import PalsgdError
    r = _run(K=2, numels=[256], p=0.2, H=4, seed=60)
    ae = torch.tensor([1e-3, 16.0], dtype=torch.float32, device="cuda:0")
    with pytest.raises(PalsgdError) as e:
        r.lib.palsgd_step_capturable(ae)
    assert e.value.status == 4
    r.lib.palsgd_capturable_begin(0)
    with pytest.raises(PalsgdError) as e:                 # a second begin would overwrite the device's step counts
        r.lib.palsgd_capturable_begin(5)
    assert e.value.status == 4
    for call in (lambda: r.lib.palsgd_step(0, 1e-3, 16.0), lambda: r.lib.palsgd_inner_step(0, 1e-3),
                 lambda: r.lib.palsgd_pseudo_sync(0, 1e-3, 16.0), lambda: r.lib.palsgd_ddp_step(0, 1e-3),
                 lambda: r.lib.palsgd_get_state(), lambda: r.lib.palsgd_set_state([0, 0], 0)):
        with pytest.raises(PalsgdError) as e:
            call()
        assert e.value.status == 4
    assert r.lib.palsgd_capturable_end() == 0
    r.lib.palsgd_step(0, 1e-3, 16.0)
    r.close()


@pytest.mark.parametrize("grad_dtype,clip,unit_scale", [("f32", None, False), ("bf16", None, False), ("f32", 20.0, False),
                                                        ("bf16", 20.0, False), ("f32", 50.0, True), ("bf16", 50.0, True)])
def test_replayed_graph_of_a_window_follows_alg1(grad_dtype, clip, unit_scale):
    """One captured window [H x (load gradients, (clip), local update), outer step with diagnostics] replayed for
    consecutive windows: t, the draws and the step counts advance on the device, alpha changes between replays
    through the device array, the clipping scales are recomputed on the device by every replay, and every
    replay is compared with the oracle.  The clipping and diagnostics calls inside the capture are the first of
    their kind on this context: nothing allocates after palsgd_init."""
    import oracle
    H, K = 3, 4
    r = _run(K=K, numels=RAGGED, grad_dtype=grad_dtype, p=0.3, H=H, seed=61, wd_mult=[1, 0, 1, 1, 0.5, 1, 0],
             **(dict(sigma=0.5, c_scale=1.0, moment_floor_by_gradient=True) if unit_scale
                else dict(sigma=0.1, c_scale=0.25) if clip else dict(sigma=0.05)))
    stage = torch.zeros((H,) + tuple(r.G.shape), dtype=r.G.dtype, device="cuda:0")
    ae = torch.tensor([r.alpha, r.eta], dtype=torch.float32, device="cuda:0")
    diag = torch.zeros(2, dtype=torch.float32, device="cuda:0")
    r.lib.palsgd_capturable_begin(0)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(g, stream=s):
        for i in range(H):
            r.G.copy_(stage[i])
            if clip:
                r.lib.palsgd_clip_grad_norm(clip)
            r.lib.palsgd_step_capturable(ae)
        r.lib.palsgd_outer_step_diag(0, diag)
    torch.cuda.synchronize()
    clipped = False
    for w in range(5):
        alpha = float(np.float32(r.alpha * (1.0 + 0.25 * w)))          # a learning-rate schedule across windows
        for i in range(H):
            gd = r.oracle_side_gradients()
            stage[i, :, :r.row].copy_(gd)
            scales = None
            if clip:
                scales = np.array([oracle.clip_scale(v, float(np.float32(clip))) for v in r.ora.grad_norms()])
                clipped = clipped or bool((scales < 1).any())
            r.note_gradients(scales)
            r.ora.local_step(r.t, alpha, r.eta, grad_scale=scales)
            synced = (r.t + 1) % H == 0
            if synced:                                                 # the captured outer step reports these
                want_diag = r.ora.diagnostics()
                r.ora.outer_step()
            r.t += 1
        assert synced
        ae.copy_(torch.tensor([alpha, r.eta], dtype=torch.float32))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        r.compare(check_state=False)
        np.testing.assert_allclose(diag.cpu().numpy(), want_diag, rtol=2e-3, atol=1e-12)
        junk = torch.randn(1 << 18, device="cuda:0").sum().item()     # eager work between replays
    assert r.lib.palsgd_capturable_end() == r.t
    tau, _ = r.lib.palsgd_get_state()
    assert tau == [int(v) for v in r.ora.tau]
    assert clipped == bool(clip)                                       # the threshold did bite
    r.close()


def test_config_gptneo125m_k8_device_schedule_sampled():
    """The benchmark configuration through the device-resident schedule: K=8, GPT-Neo-125M shapes, bf16 gradients,
    p=0.05, H=64, 130 steps (two outer steps), full-size buffers, oracle on sampled positions."""
    from paper_2504_18454_amd.workloads import workload
    w = workload("gptneo125m_k8")
    r = _run(K=w.K, numels=w.numels, inner=w.inner, grad_dtype=w.grad_dtype, p=w.p, H=w.H, alpha=w.alpha, eta=w.eta,
             sigma=w.sigma, seed=w.seed, per_edge=256, n_random=1 << 16)
    ae = torch.tensor([r.alpha, r.eta], dtype=torch.float32, device="cuda:0")
    r.lib.palsgd_capturable_begin(0)
    for _ in range(130):
        t = r.t
        r.make_gradients()
        _, synced = r.ora.iteration(t, r.alpha, r.eta)
        r.lib.palsgd_step_capturable(ae)
        if synced:
            r.lib.palsgd_outer_step(t)
        r.t += 1
    assert r.lib.palsgd_capturable_end() == 130
    print("worst err/bound", r.compare())
    r.close()
