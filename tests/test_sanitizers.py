"""The CPU checker, and the host half of the HIP library, under AddressSanitizer and UndefinedBehaviorSanitizer.

tests/oracle_sanitized.c includes oracle/palsgd_oracle.c and drives every routine on tiny models with
exact-size, strided buffers; it is built here with gcc -fsanitize=address,undefined and run as a child
process.  It must finish without a sanitizer report, and its check sums must equal those of the same cases
computed through the ordinary (unsanitized, -O2) library the other tests use."""
import os
import subprocess

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OFFS, NUMEL, WDM, N = [0, 8, 16, 24], [1, 3, 5, 17], [1.0, 0.0, 0.5, 1.0], 41


def _pattern(t, K):
    i = np.arange(N)
    real = np.zeros(N, bool)
    for o, n in zip(OFFS, NUMEL):
        real[o:o + n] = True
    g = np.stack([(((t * 31 + k * 17 + i * 7) % 13) - 6.0) * 0.125 for k in range(K)]).astype(np.float32)
    return np.where(real[None, :], g, np.float32(0)), real


def _weighted(a, w0):
    return float((a.astype(np.float64) * (w0 + np.arange(a.size))).sum())


def _case(inner, g_dtype, K, H):
    """The same case as one iteration of the loops in tests/oracle_sanitized.c, through the Python wrapper."""
    _, real = _pattern(0, K)
    x0 = np.where(real, np.float32(0.01) * (np.arange(N) + 1).astype(np.float32), np.float32(0)).astype(np.float32)
    st = oracle.OracleState(K, x0, OFFS, NUMEL, inner="adamw" if inner == 0 else "sgdm",
                            grad_dtype="f32" if g_dtype == 0 else "bf16", p=0.4, H=H, outer_lr=0.7, outer_momentum=0.9,
                            outer_nesterov=K != 2, inner_nesterov=H == 2, seed=11 + K, wd_mult=WDM)
    gs = np.array([1.0, 0.5, 2.0])[:K]

    def load(t):
        g, _ = _pattern(t, K)
        st.G[...] = g if g_dtype == 0 else (g.view(np.uint32) >> 16).astype(np.uint16)

    for t in range(2):
        load(t)
        c = oracle.clip_scale(st.mean_grad_norm(gs), 0.5)
        st.ddp_step(1e-3, grad_scale=gs * c)
    syncs, norms, diag = 0, 0.0, (0.0, 0.0)
    for t in range(2, 14):
        load(t)
        nk = st.grad_norms()
        norms += float(nk.sum())
        w = gs * np.array([oracle.clip_scale(v, 1.0) for v in nk])
        st.local_step(t, 1e-3, 16.0, grad_scale=w)
        if (t + 1) % H == 0:
            diag = st.diagnostics()
            st.outer_step()
            syncs += 1
    cx = sum(_weighted(st.X[k], 1.0 + 0.5 * k) for k in range(K))
    cm = sum(_weighted(st.M[k], 1.0 + 0.5 * k) for k in range(K))
    cv = sum(_weighted(st.V[k], 1.0 + 0.5 * k) for k in range(K))
    tau = [int(v) for v in st.tau]
    return [inner, g_dtype, K, H, syncs, tau[0], tau[1 if K > 1 else 0], tau[K - 1], cx, cm, cv,
            _weighted(st.XG, 1.0), _weighted(st.OM, 1.0), diag[0], diag[1], norms]


def test_checker_is_clean_under_address_and_ub_sanitizers(tmp_path):
    exe = tmp_path / "oracle_sanitized"
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-ffp-contract=off", "-o", str(exe), os.path.join(ROOT, "tests", "oracle_sanitized.c"), "-lm"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "sanitize" in built.stderr and "cannot find" in built.stderr:
        pytest.skip("the host compiler has no sanitizer runtime")
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stderr[-3000:]
    assert "Sanitizer" not in run.stderr and "runtime error" not in run.stderr, run.stderr[-3000:]
    lines = [ln.split() for ln in run.stdout.strip().split("\n")]
    cases = [ln for ln in lines if ln[0] not in ("k", "d")]
    assert len(cases) == 2 * 2 * 3 * 3
    oracle.set_threads(1)
    for ln in cases:
        inner, g_dtype, K, H = (int(v) for v in ln[:4])
        want = _case(inner, g_dtype, K, H)
        assert [int(v) for v in ln[:8]] == want[:8], ln
        np.testing.assert_allclose([float(v) for v in ln[8:]], want[8:], rtol=1e-12, atol=1e-300, err_msg=" ".join(ln[:4]))
    # draws with extreme counters, as the library's draw test takes them
    draws = [ln for ln in lines if ln[0] == "d"]
    for t, ln in enumerate(draws):
        assert int(ln[1]) == oracle.u24(2 ** 64 - 1, t << 60, 63, 64) and int(ln[2]) == oracle.draw(7, t, 2, 3, 0.999999)


def test_library_host_code_is_clean_under_address_and_ub_sanitizers(tmp_path):
    """The host half of the HIP library (layout, argument checks, per-step planning, draws, scalar state) in a
    build whose host code carries both sanitizers, driven by tests/host_sanitized.cpp through the C ABI.  The
    device code is compiled as usual and never runs: the program needs no GPU."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    exe = tmp_path / "host_sanitized"
    host_only = "-Xarch_host -fsanitize=address -Xarch_host -fsanitize=undefined".split()   # never the device code
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17"] + host_only + [
           "-fno-omit-frame-pointer", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-x", "hip", os.path.join(ROOT, "paper_2504_18454_amd", "csrc", "palsgd.hip"),
           os.path.join(ROOT, "tests", "host_sanitized.cpp"), "-o", str(exe)]
    built = subprocess.run(cmd, capture_output=True, text=True, cwd=str(tmp_path))
    assert built.returncode == 0, built.stderr[-3000:]
    # the HIP runtime keeps process-lifetime allocations: leak checking is for the checker's test above
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, (run.stdout[-500:], run.stderr[-3000:])
    assert "host ok" in run.stdout
    assert "Sanitizer" not in run.stderr and "runtime error" not in run.stderr, run.stderr[-3000:]
