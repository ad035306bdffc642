"""CPU oracle of the PALSGD update path: TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import
this package.  The product path (paper_2504_18454_amd) never does.
"""
from .binding import (OracleState, adamw, clip_scale, diagnostics, draw, get_threads, grad_norm, mean_grad_norm, mix,
                      outer, outer_adamw, set_threads, sgdm, u24)

__all__ = ["OracleState", "adamw", "clip_scale", "diagnostics", "draw", "grad_norm", "mean_grad_norm", "get_threads", "mix", "outer",
           "outer_adamw", "set_threads", "sgdm", "u24"]
