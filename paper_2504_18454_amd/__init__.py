"""PALSGD parameter-update path for AMD MI355X: HIP kernels behind a C ABI.

`binding` is the thin ctypes layer over csrc/libpalsgd.so; `workloads` holds the
seeded synthetic inputs; `build` compiles the library with hipcc for gfx950.
"""
from . import binding, workloads  # noqa: F401
from .binding import Palsgd, PalsgdError, make_config, palsgd_layout  # noqa: F401
