"""Capsule-convolution forward pass for AMD MI355X (gfx950).

The compute lives in the HIP library under ``csrc/`` behind a C ABI (``include/capscaps.h``);
``capscaps`` is the thin ctypes binding; ``workloads`` holds the seeded synthetic inputs.
The binding is imported lazily so that ``workloads`` can be used without the built library.
"""

__all__ = ["capscaps", "workloads"]


def __getattr__(name):
    if name in __all__:
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
