"""MI355X-native decoder-layer kernels (gfx950 HIP) behind the C ABI of include/tessera.h.

This package is a thin ctypes binding: argument marshalling only.  Every step of
the layer runs in the hand-written HIP kernels of libtessera.so; there is no CPU
or PyTorch fallback, and `binding` fails loudly when the library has not been
built (python -m paper_2604_10180_amd.build).

The binding is loaded on first use, so that `paper_2604_10180_amd.build` can be
imported (and run) before the library exists.
"""


def __getattr__(name):
    if name.startswith("__") or name in ("binding", "build"):
        raise AttributeError(name)          # submodules are imported by the import system itself
    import importlib
    return getattr(importlib.import_module(".binding", __name__), name)
