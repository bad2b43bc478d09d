"""MI355X-native online query phase of the Product Quantization Tree (arXiv 1702.05911).

  csrc/      HIP kernels for gfx950 and the C ABI (include/pqt.h) -> libpqt.so
  binding    ctypes binding with the C ABI's names (needs the built library and a GPU)
  builder    codebook and line-table training on a sample; drives the library's streaming builder
  buildlib   compiles libpqt.so with hipcc

The binding is imported on first use so that the builder and the build step work on a
machine without the compiled library; using the query path without it raises ImportError.
"""
import importlib

_BINDING_NAMES = ("Index", "Builder", "PqtError", "last_error")


def __getattr__(name):
    if name in _BINDING_NAMES or name == "binding" or name.startswith("pqt_"):   # the C ABI's names
        mod = importlib.import_module(".binding", __name__)
        return mod if name == "binding" else getattr(mod, name)
    if name in ("builder", "buildlib"):
        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
