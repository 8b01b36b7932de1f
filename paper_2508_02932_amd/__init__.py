"""MI355X-native packed multi-LoRA linear layer (forward and backward).

``paper_2508_02932_amd.plora``     - thin ctypes binding of the C-ABI library (HIP kernels, gfx950)
``paper_2508_02932_amd.workloads`` - seeded synthetic inputs (no layer arithmetic)

The binding is imported on first use so that the input generators can be used without the
compiled library.
"""
import importlib

__all__ = ["plora", "workloads"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
