"""ctypes binding of libpalsgd.so: argument marshalling only.

Every step of the update path runs in the HIP kernels behind the C ABI of
include/palsgd.h; this module converts Python values to C arguments and turns
status codes into exceptions.  PyTorch appears only as the allocator of device
memory and the source of the HIP stream handle.  There is no fallback: if the
shared library is missing, importing the library handle raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "csrc", "libpalsgd.so")

PALSGD_OK, PALSGD_EINVAL, PALSGD_ENOMEM, PALSGD_EHIP, PALSGD_ESTATE = range(5)
INNER = {"adamw": 0, "sgdm": 1}
GRAD = {"f32": 0, "bf16": 1}
OUTER = {"sgd": 0, "adamw": 1}
MAX_K = 64

EXPORTS = ("palsgd_layout", "palsgd_init", "palsgd_draw", "palsgd_inner_step", "palsgd_pseudo_sync",
           "palsgd_step", "palsgd_outer_step", "palsgd_get_state", "palsgd_set_state",
           "palsgd_last_error", "palsgd_destroy", "palsgd_set_tuning", "palsgd_ddp_step",
           "palsgd_clip_grad_norm", "palsgd_diagnostics", "palsgd_outer_step_diag", "palsgd_capturable_begin",
           "palsgd_step_capturable", "palsgd_capturable_end", "palsgd_ddp_finish", "palsgd_clip_mean_grad_norm", "palsgd_step_sync",
           "palsgd_ddp_step_shared", "palsgd_set_outer_lr", "palsgd_clip_grad_norm_noalloc")


class PalsgdError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"palsgd status {status}: {text}")
        self.status = status


class Config(C.Structure):
    _fields_ = [("K", C.c_uint32), ("n_tensors", C.c_uint32), ("P", C.c_uint64),
                ("tensor_numel", C.POINTER(C.c_uint64)), ("tensor_wd_mult", C.POINTER(C.c_float)),
                ("inner", C.c_int32), ("grad_dtype", C.c_int32),
                ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("momentum", C.c_float), ("inner_nesterov", C.c_int32),
                ("p", C.c_double), ("H", C.c_uint32),
                ("outer_lr", C.c_float), ("outer_momentum", C.c_float), ("outer_nesterov", C.c_int32),
                ("seed", C.c_uint64), ("outer_opt", C.c_int32),
                ("outer_beta1", C.c_float), ("outer_beta2", C.c_float), ("outer_eps", C.c_float),
                ("outer_weight_decay", C.c_float)]


class Buffers(C.Structure):
    _fields_ = [("X", C.c_void_p), ("M", C.c_void_p), ("V", C.c_void_p), ("G", C.c_void_p),
                ("XG", C.c_void_p), ("OM", C.c_void_p), ("row_stride", C.c_uint64), ("OV", C.c_void_p)]


_lib = None


def lib() -> C.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2504_18454_amd.build` "
                              "(hipcc, gfx950); the PALSGD update path has no other implementation")
        L = C.CDLL(LIB_PATH)
        vp, u64, u32, f, st = C.c_void_p, C.c_uint64, C.c_uint32, C.c_float, C.c_int
        L.palsgd_layout.restype = st
        L.palsgd_layout.argtypes = [C.POINTER(Config), C.POINTER(u64), C.POINTER(u64)]
        L.palsgd_init.restype = st
        L.palsgd_init.argtypes = [C.POINTER(Config), C.POINTER(Buffers), vp, vp, C.POINTER(vp)]
        L.palsgd_draw.restype = st
        L.palsgd_draw.argtypes = [vp, u64, C.POINTER(C.c_uint8)]
        L.palsgd_inner_step.restype = st
        L.palsgd_inner_step.argtypes = [vp, u64, f, C.POINTER(f), C.POINTER(C.c_uint8), vp]
        L.palsgd_pseudo_sync.restype = st
        L.palsgd_pseudo_sync.argtypes = [vp, u64, f, f, C.POINTER(C.c_uint8), vp]
        L.palsgd_step.restype = st
        L.palsgd_step.argtypes = [vp, u64, f, f, C.POINTER(f), C.POINTER(C.c_uint8), vp]
        L.palsgd_step_sync.restype = st
        L.palsgd_step_sync.argtypes = [vp, u64, f, f, C.POINTER(f), C.POINTER(C.c_uint8), vp]
        L.palsgd_outer_step.restype = st
        L.palsgd_outer_step.argtypes = [vp, u64, vp]
        L.palsgd_ddp_step.restype = st
        L.palsgd_ddp_step.argtypes = [vp, u64, f, C.POINTER(f), vp]
        L.palsgd_ddp_step_shared.restype = st
        L.palsgd_ddp_step_shared.argtypes = [vp, u64, f, C.POINTER(f), vp]
        L.palsgd_ddp_finish.restype = st
        L.palsgd_ddp_finish.argtypes = [vp, vp]
        L.palsgd_clip_grad_norm.restype = st
        L.palsgd_clip_grad_norm.argtypes = [vp, f, vp, vp]
        L.palsgd_clip_grad_norm_noalloc.restype = st
        L.palsgd_clip_grad_norm_noalloc.argtypes = [vp, f, vp, vp]
        L.palsgd_clip_mean_grad_norm.restype = st
        L.palsgd_clip_mean_grad_norm.argtypes = [vp, f, C.POINTER(f), vp, vp]
        L.palsgd_diagnostics.restype = st
        L.palsgd_diagnostics.argtypes = [vp, vp, vp]
        L.palsgd_capturable_begin.restype = st
        L.palsgd_capturable_begin.argtypes = [vp, u64, vp]
        L.palsgd_step_capturable.restype = st
        L.palsgd_step_capturable.argtypes = [vp, vp, vp]
        L.palsgd_capturable_end.restype = st
        L.palsgd_capturable_end.argtypes = [vp, C.POINTER(u64), vp]
        L.palsgd_outer_step_diag.restype = st
        L.palsgd_outer_step_diag.argtypes = [vp, u64, vp, vp]
        L.palsgd_get_state.restype = st
        L.palsgd_get_state.argtypes = [vp, C.POINTER(u64), C.POINTER(u64)]
        L.palsgd_set_state.restype = st
        L.palsgd_set_state.argtypes = [vp, C.POINTER(u64), u64]
        L.palsgd_last_error.restype = C.c_char_p
        L.palsgd_last_error.argtypes = [vp]
        L.palsgd_destroy.restype = None
        L.palsgd_destroy.argtypes = [vp]
        L.palsgd_set_outer_lr.restype = st
        L.palsgd_set_outer_lr.argtypes = [vp, f]
        L.palsgd_set_tuning.restype = st
        L.palsgd_set_tuning.argtypes = [vp, u32, u32, u32]
        _lib = L
    return _lib


def make_config(K: int, tensor_numel: Sequence[int], *, inner: str = "adamw", grad_dtype: str = "f32",
                beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8, weight_decay: float = 0.01,
                momentum: float = 0.9, p: float = 0.1, H: int = 16, outer_lr: float = 0.2,
                outer_momentum: float = 0.9, outer_nesterov: bool = True, seed: int = 0,
                wd_mult: Optional[Sequence[float]] = None, inner_nesterov: bool = False,
                outer_opt: str = "sgd", outer_beta1: float = 0.9, outer_beta2: float = 0.999,
                outer_eps: float = 1e-8, outer_weight_decay: float = 0.0) -> Config:
    cfg = Config()
    n = len(tensor_numel)
    numel = (C.c_uint64 * max(n, 1))(*[int(v) for v in tensor_numel])
    cfg._keep = [numel]                              # keep the host arrays alive with the struct
    cfg.K, cfg.n_tensors = int(K), n
    cfg.P = sum(int(v) for v in tensor_numel)        # stated, so that the library checks it against the tensor list
    cfg.tensor_numel = C.cast(numel, C.POINTER(C.c_uint64))
    if wd_mult is not None:
        wm = (C.c_float * max(n, 1))(*[float(v) for v in wd_mult])
        cfg._keep.append(wm)
        cfg.tensor_wd_mult = C.cast(wm, C.POINTER(C.c_float))
    cfg.inner = INNER[inner] if isinstance(inner, str) else int(inner)
    cfg.grad_dtype = GRAD[grad_dtype] if isinstance(grad_dtype, str) else int(grad_dtype)
    cfg.beta1, cfg.beta2, cfg.eps = beta1, beta2, eps
    cfg.weight_decay, cfg.momentum = weight_decay, momentum
    cfg.inner_nesterov = int(bool(inner_nesterov))
    cfg.p, cfg.H = float(p), int(H)
    cfg.outer_lr, cfg.outer_momentum, cfg.outer_nesterov = outer_lr, outer_momentum, int(bool(outer_nesterov))
    cfg.seed = int(seed) & (2 ** 64 - 1)
    cfg.outer_opt = OUTER[outer_opt] if isinstance(outer_opt, str) else int(outer_opt)
    cfg.outer_beta1, cfg.outer_beta2, cfg.outer_eps = outer_beta1, outer_beta2, outer_eps
    cfg.outer_weight_decay = outer_weight_decay
    return cfg


def _check(status: int, ctx) -> None:
    if status != PALSGD_OK:
        text = lib().palsgd_last_error(ctx)
        raise PalsgdError(status, text.decode() if text else "")


def palsgd_layout(cfg: Config):
    """-> (P_padded, [tensor offsets])"""
    P = C.c_uint64(0)
    offs = (C.c_uint64 * max(cfg.n_tensors, 1))()
    _check(lib().palsgd_layout(C.byref(cfg), C.byref(P), offs), None)
    return int(P.value), [int(offs[j]) for j in range(cfg.n_tensors)]


def _u8(mask, n):
    """Host array of n bytes for the C side (which reads exactly n), or NULL."""
    if mask is None:
        return None, None
    a = np.ascontiguousarray(mask, dtype=np.uint8)
    if a.shape != (n,):
        raise ValueError(f"expected {n} entries (one per worker), got shape {a.shape}")
    return a, a.ctypes.data_as(C.POINTER(C.c_uint8))


def _f32(v, n):
    """Host array of n floats for the C side (which reads exactly n), or NULL."""
    if v is None:
        return None, None
    a = np.ascontiguousarray(v, dtype=np.float32)
    if a.shape != (n,):
        raise ValueError(f"expected {n} entries (one per worker), got shape {a.shape}")
    return a, a.ctypes.data_as(C.POINTER(C.c_float))


def _dev_f32(t, n, what):
    """Device address of a float32 array with room for n values: a torch CUDA tensor (checked) or a raw address."""
    if t is None or isinstance(t, int):
        return t
    import torch
    if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() >= n):
        raise ValueError(f"{what}: expected a contiguous float32 CUDA tensor of at least {n} elements")
    return t.data_ptr()


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


class Palsgd:
    """A context over caller-owned device buffers; one method per C entry point.

    X, M, V, G, XG, OM (and OV with OuterOPT = AdamW) are torch CUDA tensors (V may be None
    for SGD-momentum) or raw device addresses; they must outlive the context.
    """

    def __init__(self, cfg: Config, X, M, V, G, XG, OM, row_stride: int, x0=None, stream=None, OV=None):
        ptr = lambda t: None if t is None else (t if isinstance(t, int) else t.data_ptr())
        self._tensors = (X, M, V, G, XG, OM, OV, x0)      # keep references
        self.cfg = cfg
        self.K = int(cfg.K)
        self._check_tensors(cfg, X, M, V, G, XG, OM, OV, x0, int(row_stride))
        buf = Buffers(ptr(X), ptr(M), ptr(V), ptr(G), ptr(XG), ptr(OM), int(row_stride), ptr(OV))
        out = C.c_void_p()
        st = lib().palsgd_init(C.byref(cfg), C.byref(buf), ptr(x0), _stream_handle(stream), C.byref(out))
        _check(st, None)
        self._ctx = out

    @staticmethod
    def _check_tensors(cfg, X, M, V, G, XG, OM, OV, x0, row_stride):
        """Sizes and dtypes of the buffers that are torch tensors (raw addresses cannot be checked): the kernels
        index K rows of row_stride elements and trust the caller's allocation."""
        import torch
        P_padded, _ = palsgd_layout(cfg)
        K = int(cfg.K)
        rows = (K - 1) * row_stride + P_padded if row_stride >= P_padded else 0   # init rejects a short stride itself
        gdt = torch.float32 if cfg.grad_dtype == GRAD["f32"] else torch.bfloat16
        for name, t, need, dt in (("X", X, rows, torch.float32), ("M", M, rows, torch.float32), ("V", V, rows, torch.float32),
                                  ("G", G, rows, gdt), ("XG", XG, P_padded, torch.float32),
                                  ("OM", OM, P_padded, torch.float32), ("OV", OV, P_padded, torch.float32),
                                  ("x0", x0, P_padded, torch.float32)):
            if t is None or isinstance(t, int):
                continue
            if not (t.is_cuda and t.is_contiguous() and t.dtype == dt and t.numel() >= need):
                raise ValueError(f"{name}: expected a contiguous {dt} CUDA tensor of at least {need} elements, got "
                                 f"{t.dtype} {tuple(t.shape)} on {t.device}")

    # -- the C entry points, same names ------------------------------------------------
    def palsgd_draw(self, t: int) -> np.ndarray:
        mask = np.zeros(self.K, np.uint8)
        _check(lib().palsgd_draw(self._ctx, int(t), mask.ctypes.data_as(C.POINTER(C.c_uint8))), self._ctx)
        return mask

    def palsgd_inner_step(self, t, alpha_t, grad_scale=None, mask_override=None, stream=None):
        gs, gsp = _f32(grad_scale, self.K)
        mo, mop = _u8(mask_override, self.K)
        _check(lib().palsgd_inner_step(self._ctx, int(t), alpha_t, gsp, mop, _stream_handle(stream)), self._ctx)

    def palsgd_pseudo_sync(self, t, alpha_t, eta_t, mask_override=None, stream=None):
        mo, mop = _u8(mask_override, self.K)
        _check(lib().palsgd_pseudo_sync(self._ctx, int(t), alpha_t, eta_t, mop, _stream_handle(stream)), self._ctx)

    def palsgd_step(self, t, alpha_t, eta_t, grad_scale=None, mask_override=None, stream=None):
        gs, gsp = _f32(grad_scale, self.K)
        mo, mop = _u8(mask_override, self.K)
        _check(lib().palsgd_step(self._ctx, int(t), alpha_t, eta_t, gsp, mop, _stream_handle(stream)), self._ctx)

    def palsgd_step_sync(self, t, alpha_t, eta_t, grad_scale=None, mask_override=None, stream=None):
        gs, gsp = _f32(grad_scale, self.K)
        mo, mop = _u8(mask_override, self.K)
        _check(lib().palsgd_step_sync(self._ctx, int(t), alpha_t, eta_t, gsp, mop, _stream_handle(stream)), self._ctx)

    def palsgd_outer_step(self, t, stream=None):
        _check(lib().palsgd_outer_step(self._ctx, int(t), _stream_handle(stream)), self._ctx)

    def palsgd_ddp_step(self, t, alpha_t, grad_scale=None, stream=None):
        gs, gsp = _f32(grad_scale, self.K)
        _check(lib().palsgd_ddp_step(self._ctx, int(t), alpha_t, gsp, _stream_handle(stream)), self._ctx)

    def palsgd_ddp_step_shared(self, t, alpha_t, grad_scale=None, stream=None):
        gs, gsp = _f32(grad_scale, self.K)
        _check(lib().palsgd_ddp_step_shared(self._ctx, int(t), alpha_t, gsp, _stream_handle(stream)), self._ctx)

    def palsgd_ddp_finish(self, stream=None):
        _check(lib().palsgd_ddp_finish(self._ctx, _stream_handle(stream)), self._ctx)

    def palsgd_clip_grad_norm(self, max_norm, norms_out=None, stream=None):
        """norms_out: torch CUDA float32 tensor of K elements (or a device address), or None."""
        ptr = _dev_f32(norms_out, self.K, "norms_out")
        _check(lib().palsgd_clip_grad_norm(self._ctx, max_norm, ptr, _stream_handle(stream)), self._ctx)

    def palsgd_clip_grad_norm_noalloc(self, max_norm, norms_out=None, stream=None):
        """As palsgd_clip_grad_norm, through the library's static scratch (no allocation anywhere)."""
        ptr = _dev_f32(norms_out, self.K, "norms_out")
        _check(lib().palsgd_clip_grad_norm_noalloc(self._ctx, max_norm, ptr, _stream_handle(stream)), self._ctx)

    def palsgd_clip_mean_grad_norm(self, max_norm, grad_scale=None, norm_out=None, stream=None):
        """norm_out: torch CUDA float32 tensor of 1 element (or a device address), or None."""
        gs, gsp = _f32(grad_scale, self.K)
        ptr = _dev_f32(norm_out, 1, "norm_out")
        _check(lib().palsgd_clip_mean_grad_norm(self._ctx, max_norm, gsp, ptr, _stream_handle(stream)), self._ctx)

    def palsgd_diagnostics(self, out, stream=None):
        """out: torch CUDA float32 tensor of 2 elements (or a device address): Xi, |Delta|^2."""
        ptr = _dev_f32(out, 2, "out")
        _check(lib().palsgd_diagnostics(self._ctx, ptr, _stream_handle(stream)), self._ctx)

    def palsgd_outer_step_diag(self, t, out, stream=None):
        """Outer step + diagnostics taken just before it; out as in palsgd_diagnostics."""
        ptr = _dev_f32(out, 2, "out")
        _check(lib().palsgd_outer_step_diag(self._ctx, int(t), ptr, _stream_handle(stream)), self._ctx)

    def palsgd_capturable_begin(self, t0, stream=None):
        _check(lib().palsgd_capturable_begin(self._ctx, int(t0), _stream_handle(stream)), self._ctx)

    def palsgd_step_capturable(self, alpha_eta, stream=None):
        """alpha_eta: torch CUDA float32 tensor {alpha_t, eta_t} (or a device address)."""
        ptr = _dev_f32(alpha_eta, 2, "alpha_eta")
        _check(lib().palsgd_step_capturable(self._ctx, ptr, _stream_handle(stream)), self._ctx)

    def palsgd_capturable_end(self, stream=None) -> int:
        t = C.c_uint64(0)
        _check(lib().palsgd_capturable_end(self._ctx, C.byref(t), _stream_handle(stream)), self._ctx)
        return int(t.value)

    def palsgd_get_state(self):
        tau = (C.c_uint64 * self.K)()
        n_outer = C.c_uint64(0)
        _check(lib().palsgd_get_state(self._ctx, tau, C.byref(n_outer)), self._ctx)
        return [int(v) for v in tau], int(n_outer.value)

    def palsgd_set_state(self, tau, n_outer):
        if len(tau) != self.K:
            raise ValueError(f"expected {self.K} step counts (one per worker), got {len(tau)}")
        arr = (C.c_uint64 * self.K)(*[int(v) for v in tau])
        _check(lib().palsgd_set_state(self._ctx, arr, int(n_outer)), self._ctx)

    def palsgd_set_outer_lr(self, outer_lr):
        _check(lib().palsgd_set_outer_lr(self._ctx, outer_lr), self._ctx)

    def palsgd_set_tuning(self, step_waves_per_cu=0, outer_waves_per_cu=0, outer_variant=0):
        _check(lib().palsgd_set_tuning(self._ctx, int(step_waves_per_cu), int(outer_waves_per_cu),
                                       int(outer_variant)), self._ctx)

    def palsgd_destroy(self):
        if self._ctx is not None and self._ctx.value:
            lib().palsgd_destroy(self._ctx)
        self._ctx = None

    def __del__(self):
        try:
            self.palsgd_destroy()
        except Exception:
            pass
