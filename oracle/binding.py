"""ctypes binding of oracle/palsgd_oracle.c (argument marshalling only).

TEST INFRASTRUCTURE: see the header of palsgd_oracle.c.  All arrays are
C-contiguous numpy arrays that the C code updates in place.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        _lib.ora_u24.restype = C.c_uint32
        _lib.ora_u24.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32]
        _lib.ora_draw.restype = C.c_int
        _lib.ora_draw.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32, C.c_double]
        _lib.ora_set_threads.argtypes = [C.c_int]
        _lib.ora_get_threads.restype = C.c_int
        _lib.ora_mix.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_double]
        _lib.ora_adamw.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                   C.c_uint64, C.c_double, C.c_double, C.c_double, C.c_double,
                                   C.c_double, C.c_uint64, C.c_double]
        _lib.ora_sgdm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_uint64,
                                  C.c_double, C.c_double, C.c_double, C.c_double, C.c_int]
        _lib.ora_outer.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32, C.c_void_p, C.c_void_p,
                                   C.c_uint64, C.c_double, C.c_double, C.c_int]
        _lib.ora_outer_adamw.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_uint64, C.c_double, C.c_double, C.c_double, C.c_double, C.c_double,
                                         C.c_uint64]
        _lib.ora_local_step.argtypes = [C.c_void_p, C.c_uint64, C.c_double, C.c_double,
                                        C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.ora_outer_step.argtypes = [C.c_void_p]
        _lib.ora_ddp_step.argtypes = [C.c_void_p, C.c_double, C.c_void_p]
        _lib.ora_grad_norm.restype = C.c_double
        _lib.ora_grad_norm.argtypes = [C.c_void_p, C.c_int, C.c_uint64]
        _lib.ora_mean_grad_norm.restype = C.c_double
        _lib.ora_mean_grad_norm.argtypes = [C.c_void_p, C.c_int, C.c_uint64, C.c_uint32, C.c_uint64, C.c_void_p]
        _lib.ora_clip_scale.restype = C.c_double
        _lib.ora_clip_scale.argtypes = [C.c_double, C.c_double]
        _lib.ora_diagnostics.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32, C.c_void_p, C.c_uint64, C.c_void_p]
        _lib.ora_iteration.restype = C.c_int
        _lib.ora_iteration.argtypes = [C.c_void_p, C.c_uint64, C.c_double, C.c_double,
                                       C.c_void_p, C.c_void_p, C.c_void_p]
    return _lib


def set_threads(n: int) -> None:
    _load().ora_set_threads(int(n))


def get_threads() -> int:
    return int(_load().ora_get_threads())


def u24(seed: int, t: int, k: int, K: int) -> int:
    return int(_load().ora_u24(seed & (2**64 - 1), t, k, K))


def draw(seed: int, t: int, k: int, K: int, p: float) -> int:
    return int(_load().ora_draw(seed & (2**64 - 1), t, k, K, float(p)))


def _ptr(a, dtype):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags.c_contiguous, (a.dtype, dtype)
    return a.ctypes.data_as(C.c_void_p)


def _gptr(g):
    """Gradient array -> (pointer, dtype code).  float32 = fp32; uint16 = bf16 bit patterns."""
    if g.dtype == np.float32:
        return _ptr(g, np.float32), 0
    if g.dtype == np.uint16:
        return _ptr(g, np.uint16), 1
    raise TypeError("gradients must be float32 or uint16 (bf16 bits)")


def mix(x, xg, beta):
    _load().ora_mix(_ptr(x, np.float32), _ptr(xg, np.float32), x.size, float(beta))


def adamw(x, m, v, g, lr, beta1, beta2, eps, wd, tau, grad_scale=1.0):
    gp, gd = _gptr(g)
    _load().ora_adamw(_ptr(x, np.float32), _ptr(m, np.float32), _ptr(v, np.float32), gp, gd,
                      x.size, float(lr), float(beta1), float(beta2), float(eps), float(wd),
                      int(tau), float(grad_scale))


def sgdm(x, buf, g, lr, momentum, wd, grad_scale=1.0, nesterov=False):
    gp, gd = _gptr(g)
    _load().ora_sgdm(_ptr(x, np.float32), _ptr(buf, np.float32), gp, gd, x.size, float(lr),
                     float(momentum), float(wd), float(grad_scale), int(bool(nesterov)))


def outer(X, xg, om, lr_o, mu_o, nesterov):
    """X: [K, row] float32, updated in place together with xg, om ([row])."""
    K, row = X.shape
    _load().ora_outer(_ptr(X, np.float32), row, K, _ptr(xg, np.float32), _ptr(om, np.float32),
                      xg.size, float(lr_o), float(mu_o), int(bool(nesterov)))


def outer_adamw(X, xg, om, ov, lr_o, beta1, beta2, eps, wd, step):
    """Outer step with OuterOPT = AdamW; `step` counts outer steps from 1.  X, xg, om, ov updated in place."""
    K, row = X.shape
    _load().ora_outer_adamw(_ptr(X, np.float32), row, K, _ptr(xg, np.float32), _ptr(om, np.float32),
                            _ptr(ov, np.float32), xg.size, float(lr_o), float(beta1), float(beta2), float(eps),
                            float(wd), int(step))


def grad_norm(g):
    gp, gd = _gptr(g)
    return float(_load().ora_grad_norm(gp, gd, g.size))


def mean_grad_norm(G, grad_scale=None):
    """Norm of (1/K) sum_k grad_scale_k G[k] for G [K, row]."""
    gp, gd = _gptr(G)
    K, row = G.shape
    gs = None if grad_scale is None else np.ascontiguousarray(grad_scale, dtype=np.float64)
    gsp = None if gs is None else gs.ctypes.data_as(C.c_void_p)
    return float(_load().ora_mean_grad_norm(gp, gd, row, K, row, gsp))


def clip_scale(norm, max_norm):
    return float(_load().ora_clip_scale(float(norm), float(max_norm)))


def diagnostics(X, xg):
    """-> (Xi, |Delta|^2) for X [K, row] and xg [n <= row]."""
    K, row = X.shape
    out = np.zeros(2, np.float64)
    _load().ora_diagnostics(_ptr(X, np.float32), row, K, _ptr(xg, np.float32), xg.size,
                            out.ctypes.data_as(C.c_void_p))
    return float(out[0]), float(out[1])


class _CState(C.Structure):
    _fields_ = [
        ("K", C.c_uint32), ("n", C.c_uint64), ("row_stride", C.c_uint64),
        ("n_tensors", C.c_uint32), ("tensor_offset", C.c_void_p), ("tensor_numel", C.c_void_p),
        ("tensor_wd_mult", C.c_void_p),
        ("inner", C.c_int), ("g_dtype", C.c_int),
        ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
        ("weight_decay", C.c_double), ("momentum", C.c_double), ("inner_nesterov", C.c_int),
        ("p", C.c_double),
        ("H", C.c_uint32), ("outer_lr", C.c_double), ("outer_momentum", C.c_double),
        ("outer_nesterov", C.c_int), ("seed", C.c_uint64),
        ("X", C.c_void_p), ("M", C.c_void_p), ("V", C.c_void_p), ("G", C.c_void_p),
        ("XG", C.c_void_p), ("OM", C.c_void_p), ("tau", C.c_void_p), ("n_outer", C.c_uint64),
        ("outer_opt", C.c_int), ("outer_beta1", C.c_double), ("outer_beta2", C.c_double),
        ("outer_eps", C.c_double), ("outer_weight_decay", C.c_double), ("OV", C.c_void_p),
    ]


class OracleState:
    """K replicas of Alg. 1 in host memory.

    x0: [row] float32 initial model (every worker starts from it, Alg. 1).
    tensor_offset / tensor_numel: the tensors tiling a row; wd_mult optional.
    Hyper-parameters that the device path holds as fp32 must be passed here already
    rounded to fp32 (as Python floats) so that both sides see the same numbers.
    """

    def __init__(self, K, x0, tensor_offset, tensor_numel, *, inner="adamw", grad_dtype="f32",
                 beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, momentum=0.9, p=0.1, H=16,
                 outer_lr=0.2, outer_momentum=0.9, outer_nesterov=True, seed=0, wd_mult=None,
                 inner_nesterov=False, outer_opt="sgd", outer_beta1=0.9, outer_beta2=0.999, outer_eps=1e-8,
                 outer_weight_decay=0.0):
        self.lib = _load()
        x0 = np.ascontiguousarray(x0, dtype=np.float32)
        row = x0.size
        self.K, self.row = int(K), row
        self.inner = inner
        self.X = np.tile(x0, (K, 1))                       # x_k^(0) <- x^(0)
        self.XG = x0.copy()
        self.M = np.zeros((K, row), np.float32)
        self.V = np.zeros((K, row), np.float32)
        self.OM = np.zeros(row, np.float32)
        self.tau = np.zeros(K, np.uint64)
        self.gdtype = np.float32 if grad_dtype == "f32" else np.uint16
        self.G = np.zeros((K, row), self.gdtype)
        self._off = np.ascontiguousarray(tensor_offset, dtype=np.uint64)
        self._num = np.ascontiguousarray(tensor_numel, dtype=np.uint64)
        self._wdm = None if wd_mult is None else np.ascontiguousarray(wd_mult, dtype=np.float32)
        f32 = lambda v: float(np.float32(v))
        s = _CState()
        s.K, s.n, s.row_stride = K, row, row
        s.n_tensors = len(self._off)
        s.tensor_offset = self._off.ctypes.data
        s.tensor_numel = self._num.ctypes.data
        s.tensor_wd_mult = None if self._wdm is None else self._wdm.ctypes.data
        s.inner = 0 if inner == "adamw" else 1
        s.g_dtype = 0 if grad_dtype == "f32" else 1
        s.beta1, s.beta2, s.eps = f32(beta1), f32(beta2), f32(eps)
        s.weight_decay, s.momentum = f32(weight_decay), f32(momentum)
        s.inner_nesterov = int(bool(inner_nesterov))
        s.p, s.H = float(p), int(H)
        s.outer_lr, s.outer_momentum = f32(outer_lr), f32(outer_momentum)
        s.outer_nesterov = int(bool(outer_nesterov))
        s.seed = seed & (2**64 - 1)
        s.X, s.M, s.V = self.X.ctypes.data, self.M.ctypes.data, self.V.ctypes.data
        s.G, s.XG, s.OM = self.G.ctypes.data, self.XG.ctypes.data, self.OM.ctypes.data
        s.tau = self.tau.ctypes.data
        s.n_outer = 0
        self.OV = np.zeros(row, np.float32)
        s.outer_opt = 0 if outer_opt == "sgd" else 1
        s.outer_beta1, s.outer_beta2, s.outer_eps = f32(outer_beta1), f32(outer_beta2), f32(outer_eps)
        s.outer_weight_decay = f32(outer_weight_decay)
        s.OV = self.OV.ctypes.data
        self.s = s

    def set_outer_lr(self, outer_lr):
        """OuterOPT learning rate of the outer steps that follow (a schedule on it, App. B)."""
        self.s.outer_lr = float(np.float32(outer_lr))

    @property
    def n_outer(self):
        return int(self.s.n_outer)

    def _opt(self, a, dtype):
        if a is None:
            return None, None
        arr = np.ascontiguousarray(a, dtype=dtype)
        return arr, arr.ctypes.data_as(C.c_void_p)

    def local_step(self, t, alpha_t, eta_t, grad_scale=None, mask_override=None):
        gs, gsp = self._opt(grad_scale, np.float64)
        mo, mop = self._opt(mask_override, np.uint8)
        mask = np.zeros(self.K, np.uint8)
        self.lib.ora_local_step(C.byref(self.s), int(t), float(np.float32(alpha_t)),
                                float(np.float32(eta_t)), gsp, mop, mask.ctypes.data_as(C.c_void_p))
        return mask

    def outer_step(self):
        self.lib.ora_outer_step(C.byref(self.s))

    def ddp_step(self, alpha_t, grad_scale=None):
        gs, gsp = self._opt(grad_scale, np.float64)
        self.lib.ora_ddp_step(C.byref(self.s), float(np.float32(alpha_t)), gsp)

    def mean_grad_norm(self, grad_scale=None):
        return mean_grad_norm(self.G, grad_scale)

    def grad_norms(self):
        return np.array([grad_norm(self.G[k]) for k in range(self.K)])

    def diagnostics(self):
        return diagnostics(self.X, self.XG)

    def iteration(self, t, alpha_t, eta_t, grad_scale=None, mask_override=None):
        gs, gsp = self._opt(grad_scale, np.float64)
        mo, mop = self._opt(mask_override, np.uint8)
        mask = np.zeros(self.K, np.uint8)
        synced = self.lib.ora_iteration(C.byref(self.s), int(t), float(np.float32(alpha_t)),
                                        float(np.float32(eta_t)), gsp, mop,
                                        mask.ctypes.data_as(C.c_void_p))
        return mask, bool(synced)
