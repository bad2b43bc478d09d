"""MI355X-native online query phase of the Product Quantization Tree (arXiv 1702.05911).

  csrc/      HIP kernels for gfx950 and the C ABI (include/pqt.h) -> libpqt.so
  binding    ctypes binding with the C ABI's names (needs the built library and a GPU)
  builder    offline index builder (codebooks, inverted lists, line codes) -> index file
  buildlib   compiles libpqt.so with hipcc

The binding is imported on first use so that the builder and the build step work on a
machine without the compiled library; using the query path without it raises ImportError.
"""
import importlib

_BINDING_NAMES = (
    "Index", "PqtError", "pqt_index_load", "pqt_index_free", "pqt_index_info", "pqt_set_budget",
    "pqt_query_batch", "pqt_query_batch_debug", "pqt_set_profiling", "pqt_stage_times", "pqt_last_error",
)


def __getattr__(name):
    if name in _BINDING_NAMES or name == "binding":
        mod = importlib.import_module(".binding", __name__)
        return mod if name == "binding" else getattr(mod, name)
    if name in ("builder", "buildlib"):
        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
