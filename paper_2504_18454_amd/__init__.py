"""PALSGD parameter-update path for AMD MI355X: HIP kernels behind a C ABI.

`binding` is the thin ctypes layer over csrc/libpalsgd.so; `workloads` holds the
seeded synthetic inputs; `build` compiles the library with hipcc for gfx950.

The binding is imported on first use of one of its names, so that importing
`paper_2504_18454_amd.workloads` alone (the seeded input generators, which the
CPU checker's tests use as well) brings in nothing of the device path.
"""
_BINDING_NAMES = ("Palsgd", "PalsgdError", "make_config", "palsgd_layout")


def __getattr__(name):
    import importlib
    if name in _BINDING_NAMES or name == "binding":
        binding = importlib.import_module(".binding", __name__)
        return binding if name == "binding" else getattr(binding, name)
    if name in ("workloads", "build"):
        return importlib.import_module("." + name, __name__)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")


__all__ = list(_BINDING_NAMES) + ["binding", "workloads"]
