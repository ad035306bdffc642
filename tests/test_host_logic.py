"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares,
and its host logic (layout, argument validation, branch draws, scalar state) behaves as
include/palsgd.h says.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2504_18454_amd import binding
from paper_2504_18454_amd.binding import Buffers, lib, make_config, palsgd_layout
from paper_2504_18454_amd.workloads import WORKLOADS, flat_layout, workload

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "palsgd.h")
FAKE = 4096  # a 16-byte aligned non-NULL address; never dereferenced on the host


def _declared():
    text = open(HEADER).read()
    return sorted(set(re.findall(r"\b(palsgd_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert set(binding.EXPORTS) == set(names)
    for n in names:
        assert hasattr(lib(), n), n


def test_layout_pads_tensors_to_64_rows_to_256_and_matches_generator_layout():
    for name in WORKLOADS:
        w = workload(name)
        P, offs = palsgd_layout(make_config(w.K, w.numels))
        goffs, grow = flat_layout(w.numels)
        assert (P, offs) == (grow, goffs)
        assert all(o % 64 == 0 for o in offs) and P % 256 == 0 and P >= w.P
    assert palsgd_layout(make_config(1, [1])) == (256, [0])
    assert palsgd_layout(make_config(1, [64, 65, 1])) == (256, [0, 64, 192])
    assert palsgd_layout(make_config(1, [250, 7])) == (512, [0, 256])


def _init(cfg, **over):
    b = dict(X=FAKE, M=FAKE, V=FAKE, G=FAKE, XG=FAKE, OM=FAKE)
    b["row_stride"] = over["row_stride"] if "row_stride" in over else palsgd_layout(cfg)[0]
    b.update(over)
    out = C.c_void_p()
    st = lib().palsgd_init(C.byref(cfg), C.byref(Buffers(**b)), None, None, C.byref(out))
    return st, out


def test_init_rejects_bad_arguments_without_touching_the_device():
    bad = [
        dict(cfg=dict(K=0)), dict(cfg=dict(K=65)), dict(cfg=dict(H=0)), dict(cfg=dict(p=1.0)), dict(cfg=dict(p=-0.1)),
        dict(cfg=dict(beta1=1.0)), dict(cfg=dict(beta2=-0.1)), dict(cfg=dict(eps=float("nan"))), dict(cfg=dict(eps=0.0)),
        dict(cfg=dict(outer_opt="adamw", outer_eps=0.0), buf=dict(OV=FAKE)),
        dict(cfg=dict(inner="sgdm", momentum=1.0)), dict(cfg=dict(outer_momentum=1.5)),
        dict(cfg=dict(outer_lr=float("inf"))), dict(cfg=dict(weight_decay=-1.0)),
        dict(cfg=dict(wd_mult=[1.0, float("nan")])),
        dict(cfg=dict(outer_opt="adamw")),                       # no OV buffer
        dict(cfg=dict(outer_opt="adamw", outer_beta2=1.0), buf=dict(OV=FAKE)), dict(cfg=dict(outer_opt=7)),
        dict(buf=dict(X=None)), dict(buf=dict(V=None)), dict(buf=dict(G=FAKE + 4)), dict(buf=dict(row_stride=192)),
        dict(buf=dict(row_stride=256 + 32)),
    ]
    for case in bad:
        kw = dict(K=4)
        kw.update(case.get("cfg", {}))
        K = kw.pop("K")
        cfg = make_config(K, [100, 7], **kw)
        st, out = _init(cfg, **case.get("buf", {}))
        assert st == binding.PALSGD_EINVAL, case
        assert not out.value
        assert b"palsgd_init" in lib().palsgd_last_error(None)
    # a row longer than the launch grids can cover
    cfg = make_config(2, [2 ** 33 + 1])
    st, out = _init(cfg)
    assert st == binding.PALSGD_EINVAL and not out.value and b"2^33" in lib().palsgd_last_error(None)
    # a stated parameter count that is not the sum of the tensor sizes
    cfg = make_config(2, [100, 7])
    cfg.P = 108
    st, out = _init(cfg, row_stride=256)
    assert st == binding.PALSGD_EINVAL and not out.value and b"107" in lib().palsgd_last_error(None)
    with pytest.raises(binding.PalsgdError, match="107"):
        palsgd_layout(cfg)
    cfg.P = 0                                               # not stated: accepted
    st, out = _init(cfg)
    assert st == binding.PALSGD_OK
    lib().palsgd_destroy(out)
    # empty model and zero-sized tensor
    for numels in ([], [5, 0]):
        cfg = make_config(2, numels)
        P = C.c_uint64()
        assert lib().palsgd_layout(C.byref(cfg), C.byref(P), None) == binding.PALSGD_EINVAL
    st, out = _init(make_config(2, [10], outer_opt="adamw"), OV=FAKE)
    assert st == binding.PALSGD_OK
    lib().palsgd_destroy(out)
    # SGD-momentum needs no V
    st, out = _init(make_config(2, [10], inner="sgdm"), V=None)
    assert st == binding.PALSGD_OK
    lib().palsgd_destroy(out)


def test_binding_refuses_tensors_the_kernels_could_not_index():
    import torch
    from paper_2504_18454_amd import Palsgd
    cfg = make_config(2, [100])                             # P_padded = 256
    host = torch.zeros(2, 256)
    with pytest.raises(ValueError, match="CUDA tensor"):    # host memory where device memory is expected
        Palsgd(cfg, host, host, host, host, host[0], host[0], 256)


def test_draws_equal_oracle_bit_for_bit(oracle_mod):
    for K, p, seed in ((4, 0.1, 0), (8, 0.05, 1), (16, 0.02, 3), (64, 0.25, 2 ** 63 + 5), (1, 0.5, 9), (3, 0.0, 4)):
        st, ctx = _init(make_config(K, [128], p=p, seed=seed))
        assert st == 0
        mask = np.zeros(K, np.uint8)
        for t in list(range(300)) + [2 ** 40 + 7, 2 ** 62]:
            assert lib().palsgd_draw(ctx, t, mask.ctypes.data_as(C.POINTER(C.c_uint8))) == 0
            want = [oracle_mod.draw(seed, t, k, K, p) for k in range(K)]
            assert list(mask) == want, (K, p, seed, t)
        lib().palsgd_destroy(ctx)


def test_state_roundtrip_and_step_argument_errors():
    st, ctx = _init(make_config(3, [128], p=0.0))
    assert st == 0
    tau = (C.c_uint64 * 3)(5, 6, 7)
    assert lib().palsgd_set_state(ctx, tau, 9) == 0
    got = (C.c_uint64 * 3)()
    n = C.c_uint64()
    assert lib().palsgd_get_state(ctx, got, C.byref(n)) == 0
    assert list(got) == [5, 6, 7] and n.value == 9
    # argument errors are reported before anything is launched
    assert lib().palsgd_step(ctx, 0, float("nan"), 1.0, None, None, None) == binding.PALSGD_EINVAL
    assert lib().palsgd_step(ctx, 0, -1.0, 1.0, None, None, None) == binding.PALSGD_EINVAL
    assert lib().palsgd_pseudo_sync(ctx, 0, 1e-3, float("inf"), None, None) == binding.PALSGD_EINVAL
    force_mix = (C.c_uint8 * 3)(0, 1, 0)
    assert lib().palsgd_step(ctx, 0, 1e-3, 16.0, None, force_mix, None) == binding.PALSGD_EINVAL   # p == 0
    assert b"p == 0" in lib().palsgd_last_error(ctx)
    gs = (C.c_float * 3)(1.0, float("nan"), 1.0)
    assert lib().palsgd_inner_step(ctx, 0, 1e-3, gs, (C.c_uint8 * 3)(1, 0, 1), None) == binding.PALSGD_EINVAL
    assert lib().palsgd_set_tuning(ctx, 2, 0, 0) == binding.PALSGD_EINVAL
    assert lib().palsgd_set_tuning(ctx, 0, 33, 0) == binding.PALSGD_EINVAL
    assert lib().palsgd_set_tuning(ctx, 0, 0, 4) == binding.PALSGD_EINVAL
    assert lib().palsgd_set_tuning(ctx, 12, 4, 2) == 0
    assert lib().palsgd_get_state(ctx, got, C.byref(n)) == 0 and list(got) == [5, 6, 7]    # state untouched
    # nothing to do is not an error and launches nothing: every worker mixes, inner_step skips all
    assert lib().palsgd_inner_step(ctx, 0, 1e-3, None, (C.c_uint8 * 3)(1, 1, 1), None) == 0
    lib().palsgd_destroy(ctx)
    for fn, args in ((lib().palsgd_step, (None, 0, 1e-3, 1.0, None, None, None)),
                     (lib().palsgd_outer_step, (None, 0, None)), (lib().palsgd_draw, (None, 0, None))):
        assert fn(*args) == binding.PALSGD_EINVAL
    lib().palsgd_destroy(None)


def test_norm_of_a_periodic_row_from_one_period(oracle_mod):
    """The every-element GPU tests take the norm of a full-size row whose content repeats with period B from
    one period: sum_j count[j] g[j]^2.  Here the same row is written out and handed to the checker's norm."""
    from parity import periodic_counts
    numels, B = [1000, 64, 3, 777, 130], 256
    offs, row = flat_layout(numels)
    count = periodic_counts(numels, offs, B)
    rng = np.random.default_rng(5)
    block = rng.standard_normal(B).astype(np.float32)
    full = np.zeros(row, np.float32)
    for o, n in zip(offs, numels):
        idx = np.arange(o, o + n)
        full[idx] = block[idx % B]
    assert count.sum() == sum(numels)
    want = oracle_mod.grad_norm(full)
    got = float(np.sqrt((block.astype(np.float64) ** 2 * count).sum()))
    assert got == pytest.approx(want, rel=1e-12)


def test_context_made_without_a_gpu_refuses_every_launch():
    """With no GPU visible palsgd_init still hands out a context (for the draws and the scalar state above),
    but nothing that would launch a kernel goes through: there is no CPU path."""
    import torch
    if torch.cuda.device_count() > 0:
        pytest.skip("a GPU is visible: the context is a real one")
    st, ctx = _init(make_config(3, [128], p=0.5))
    assert st == 0
    calls = [(lib().palsgd_step, (ctx, 0, 1e-3, 16.0, None, None, None)),
             (lib().palsgd_inner_step, (ctx, 0, 1e-3, None, None, None)),
             (lib().palsgd_pseudo_sync, (ctx, 0, 1e-3, 16.0, (C.c_uint8 * 3)(1, 1, 1), None)),
             (lib().palsgd_step_sync, (ctx, 0, 1e-3, 16.0, None, None, None)),
             (lib().palsgd_outer_step, (ctx, 0, None)), (lib().palsgd_outer_step_diag, (ctx, 0, FAKE, None)),
             (lib().palsgd_ddp_step, (ctx, 0, 1e-3, None, None)), (lib().palsgd_ddp_step_shared, (ctx, 0, 1e-3, None, None)),
             (lib().palsgd_ddp_finish, (ctx, None)), (lib().palsgd_clip_grad_norm, (ctx, 1.0, None, None)),
             (lib().palsgd_clip_mean_grad_norm, (ctx, 1.0, None, None, None)), (lib().palsgd_diagnostics, (ctx, FAKE, None)),
             (lib().palsgd_capturable_begin, (ctx, 0, None))]
    for fn, args in calls:
        assert fn(*args) == binding.PALSGD_EHIP, fn.__name__
        assert b"no GPU" in lib().palsgd_last_error(ctx)
    got, n = (C.c_uint64 * 3)(), C.c_uint64()
    assert lib().palsgd_get_state(ctx, got, C.byref(n)) == 0 and list(got) == [0, 0, 0] and n.value == 0   # nothing advanced
    lib().palsgd_destroy(ctx)
    # an initial model cannot be copied anywhere either
    cfg = make_config(3, [128])
    out = C.c_void_p()
    b = Buffers(X=FAKE, M=FAKE, V=FAKE, G=FAKE, XG=FAKE, OM=FAKE, row_stride=256)
    assert lib().palsgd_init(C.byref(cfg), C.byref(b), FAKE, None, C.byref(out)) == binding.PALSGD_EHIP and not out.value


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libpalsgd.so")
    with pytest.raises(ImportError):
        binding.lib()


def test_binding_structs_match_the_header_layout(tmp_path):
    """The ctypes mirrors of palsgd_config / palsgd_buffers have the header's size and field offsets
    (checked by compiling the header with the host C compiler)."""
    import subprocess
    fields_cfg = [f[0] for f in binding.Config._fields_]
    fields_buf = [f[0] for f in binding.Buffers._fields_]
    src = tmp_path / "layout.c"
    lines = ['#include <stdio.h>', '#include <stddef.h>', f'#include "{HEADER}"', 'int main(void){',
             'printf("%zu\\n", sizeof(palsgd_config));']
    lines += [f'printf("%zu\\n", offsetof(palsgd_config, {f}));' for f in fields_cfg]
    lines += ['printf("%zu\\n", sizeof(palsgd_buffers));']
    lines += [f'printf("%zu\\n", offsetof(palsgd_buffers, {f}));' for f in fields_buf]
    lines += ['printf("%d %d %d %d %d\\n", PALSGD_OK, PALSGD_EINVAL, PALSGD_ENOMEM, PALSGD_EHIP, PALSGD_ESTATE);',
              'printf("%u\\n", PALSGD_MAX_K);', 'return 0;}']
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-std=c11", "-Wall", "-Werror", "-o", str(exe), str(src)])
    out = subprocess.check_output([str(exe)], text=True).split("\n")
    want = [C.sizeof(binding.Config)] + [getattr(binding.Config, f).offset for f in fields_cfg]
    want += [C.sizeof(binding.Buffers)] + [getattr(binding.Buffers, f).offset for f in fields_buf]
    got = [int(v) for v in out[:len(want)]]
    assert got == want
    assert out[len(want)].split() == ["0", "1", "2", "3", "4"]
    assert (binding.PALSGD_OK, binding.PALSGD_EINVAL, binding.PALSGD_ENOMEM, binding.PALSGD_EHIP, binding.PALSGD_ESTATE) == (0, 1, 2, 3, 4)
    assert int(out[len(want) + 1]) == binding.MAX_K


def test_plain_c_program_is_built_and_fails_cleanly_without_a_gpu():
    """tests/c_abi_parity links against the library and the HIP runtime; without a device it stops at its
    first allocation with an error message (with a GPU it runs to completion, see the GPU tests)."""
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi_parity")
    if not os.path.exists(exe):
        pytest.skip("tests/c_abi_parity has not been built (python -c 'import __graft_entry__ as g; g.build()')")
    out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert out.returncode in (0, 2), (out.returncode, out.stderr)
    assert ("HIP error" in out.stderr) if out.returncode == 2 else ("PASS" in out.stdout)


def test_input_generators_import_nothing_of_the_device_path():
    """The seeded input generators serve the device path's tests and the CPU checker's alike; importing them
    alone must not bring in the binding (or the checker)."""
    import subprocess
    import sys
    code = ("import sys; import paper_2504_18454_amd.workloads as w; "
            "assert 'paper_2504_18454_amd.binding' not in sys.modules and 'oracle' not in sys.modules and 'ctypes' not in "
            "[m for m in sys.modules if m == 'paper_2504_18454_amd.binding']; print(len(w.WORKLOADS))")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, cwd=root)
    assert out.returncode == 0 and out.stdout.strip() == "6", out.stderr
