"""Thin Python binding of the PQT C ABI (include/pqt.h): argument marshalling only.

Every step of the query path runs inside libpqt.so's HIP kernels.  PyTorch is used for
device memory (tensors own the query/result buffers) and for the stream handle; there is
no CPU fallback -- if the library is missing, importing this module raises.
"""
import ctypes
import os

import torch  # noqa: F401  (loads the HIP runtime the library binds to)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpqt.so")

PQT_OK = 0
PQT_EINVAL, PQT_EIO, PQT_EFORMAT, PQT_ENOMEM, PQT_EHIP, PQT_EUNSUPPORTED = -1, -2, -3, -4, -5, -6

EXPORTS = (
    "pqt_index_load", "pqt_index_from_arrays", "pqt_index_save", "pqt_index_export", "pqt_train", "pqt_builder_create", "pqt_builder_add",
    "pqt_builder_finish", "pqt_builder_free", "pqt_index_free", "pqt_index_info", "pqt_set_budget", "pqt_query_batch",
    "pqt_query_batch_debug", "pqt_query_batch_noalloc", "pqt_noalloc_workspace_bytes", "pqt_set_bin_order",
    "pqt_index_set_vectors", "pqt_query_batch_exact", "pqt_brute_force", "pqt_measure_peaks", "pqt_set_profiling",
    "pqt_stage_times", "pqt_last_error",
)


class PqtError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"pqt error {code}: {message}")
        self.code = code


class _Info(ctypes.Structure):
    _fields_ = [("N", ctypes.c_uint64), ("H", ctypes.c_uint64),
                ("D", ctypes.c_uint32), ("P", ctypes.c_uint32), ("k1", ctypes.c_uint32),
                ("k2", ctypes.c_uint32), ("M", ctypes.c_uint32), ("T", ctypes.c_uint32),
                ("C", ctypes.c_uint32), ("device", ctypes.c_int32),
                ("bytes_index", ctypes.c_uint64), ("bytes_workspace", ctypes.c_uint64),
                ("code_format", ctypes.c_uint32), ("code_bytes", ctypes.c_uint32)]


_TAP_FIELDS = ("a", "sel", "L_d", "L_id", "n_tuples", "tuples", "tuple_keys", "n_slots", "slots",
               "n_cand", "cand_ids", "scores", "lut")


class _Arrays(ctypes.Structure):
    _fields_ = [("N", ctypes.c_uint64), ("H", ctypes.c_uint64)] + \
               [(n, ctypes.c_uint32) for n in ("D", "P", "k1", "k2", "M", "T", "C")] + \
               [(n, ctypes.c_void_p) for n in ("C1", "C2", "tbl_i", "tbl_j", "tbl_lambda", "cc",
                                               "offsets", "ids", "codes")] + \
               [("code_format", ctypes.c_uint32)]


class _TrainParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in ("D", "P", "k1", "k2", "M", "iters")] + \
               [("n", ctypes.c_uint64), ("n_table", ctypes.c_uint64)]


PQT_HOST, PQT_DEVICE = 0, 1
PQT_CODES_TABLE, PQT_CODES_PAIR_LAMBDA = 0, 1
PQT_ORDER_SUMMED_DISTANCE, PQT_ORDER_STATIC_SLOPES = 0, 1


class _Taps(ctypes.Structure):
    _fields_ = [(name, ctypes.c_void_p) for name in _TAP_FIELDS]


def load_library(path=LIB_PATH):
    if not os.path.exists(path):
        raise ImportError(f"{path} not found: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = ctypes.CDLL(path)
    vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    lib.pqt_index_load.argtypes = [ctypes.c_char_p, ci, ctypes.POINTER(vp)]
    lib.pqt_index_load.restype = ci
    lib.pqt_index_from_arrays.argtypes = [ctypes.POINTER(_Arrays), ci, ci, ctypes.POINTER(vp)]
    lib.pqt_index_from_arrays.restype = ci
    lib.pqt_index_export.argtypes = [vp, ctypes.POINTER(_Arrays), ci]
    lib.pqt_index_export.restype = ci
    lib.pqt_index_save.argtypes = [vp, ctypes.c_char_p]
    lib.pqt_index_save.restype = ci
    lib.pqt_train.argtypes = [ctypes.POINTER(_TrainParams), vp, ci, vp, vp, vp, vp, vp, vp, vp]
    lib.pqt_train.restype = ci
    lib.pqt_builder_create.argtypes = [ctypes.POINTER(_Arrays), ci, ctypes.POINTER(vp)]
    lib.pqt_builder_create.restype = ci
    lib.pqt_builder_add.argtypes = [vp, vp, i64, vp]
    lib.pqt_builder_add.restype = ci
    lib.pqt_builder_finish.argtypes = [vp, ctypes.POINTER(vp)]
    lib.pqt_builder_finish.restype = ci
    lib.pqt_builder_free.argtypes = [vp]
    lib.pqt_builder_free.restype = None
    lib.pqt_index_free.argtypes = [vp]
    lib.pqt_index_free.restype = None
    lib.pqt_index_info.argtypes = [vp, ctypes.POINTER(_Info)]
    lib.pqt_index_info.restype = ci
    lib.pqt_set_budget.argtypes = [vp, ctypes.c_uint32, ctypes.c_uint32]
    lib.pqt_set_budget.restype = ci
    lib.pqt_set_bin_order.argtypes = [vp, ci]
    lib.pqt_set_bin_order.restype = ci
    lib.pqt_query_batch.argtypes = [vp, vp, i64, ci, ci, vp, vp, vp]
    lib.pqt_query_batch.restype = ci
    lib.pqt_query_batch_debug.argtypes = [vp, vp, i64, ci, ci, vp, vp, vp, ctypes.POINTER(_Taps)]
    lib.pqt_query_batch_debug.restype = ci
    lib.pqt_query_batch_noalloc.argtypes = [vp, vp, i64, ci, ci, vp, vp, vp]
    lib.pqt_query_batch_noalloc.restype = ci
    lib.pqt_noalloc_workspace_bytes.argtypes = []
    lib.pqt_noalloc_workspace_bytes.restype = ctypes.c_size_t
    lib.pqt_index_set_vectors.argtypes = [vp, vp, ci, ci]
    lib.pqt_index_set_vectors.restype = ci
    lib.pqt_query_batch_exact.argtypes = [vp, vp, i64, ci, ci, ci, vp, vp, vp]
    lib.pqt_query_batch_exact.restype = ci
    lib.pqt_brute_force.argtypes = [vp, vp, i64, ci, vp, vp, vp]
    lib.pqt_brute_force.restype = ci
    lib.pqt_measure_peaks.argtypes = [ci, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.pqt_measure_peaks.restype = ci
    lib.pqt_set_profiling.argtypes = [vp, ci]
    lib.pqt_set_profiling.restype = ci
    lib.pqt_stage_times.argtypes = [vp, ctypes.POINTER(ctypes.c_float * 4), ctypes.POINTER(ci)]
    lib.pqt_stage_times.restype = ci
    lib.pqt_last_error.argtypes = []
    lib.pqt_last_error.restype = ctypes.c_char_p
    return lib


_lib = load_library()


def _check(rc):
    if rc != PQT_OK:
        raise PqtError(rc, _lib.pqt_last_error().decode("utf-8", "replace"))


def _stream_handle(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


class Index:
    """Handle of an index resident on one GPU (pqt_index_load / pqt_index_free)."""

    def __init__(self, path=None, device=0, arrays=None, handle=None):
        self._h = ctypes.c_void_p()
        if handle is not None:
            self._h = handle                       # an index the library already made (pqt_builder_finish)
        elif arrays is None:
            _check(_lib.pqt_index_load(os.fsencode(path), int(device), ctypes.byref(self._h)))
        else:
            self._from_arrays(arrays, int(device))
        self.device = torch.device("cuda", int(device))
        self._D = self.info()["D"]

    def _from_arrays(self, a, device):
        """pqt_index_from_arrays.  `a`: mapping with the header fields, the small arrays as NumPy
        arrays, and offsets / ids / codes either all NumPy arrays (host) or all CUDA tensors on
        `device` (int32 or int64 values below 2**32 are narrowed to the ABI's uint32 here)."""
        import numpy as np
        keep = _small_arrays(a)
        on_device = torch.is_tensor(a["offsets"])
        big = []
        for n, width in (("offsets", 4), ("ids", 4), ("codes", 1)):
            t = a[n]
            if on_device:
                if not (torch.is_tensor(t) and t.is_cuda and t.device.index == device):
                    raise ValueError(f"{n}: offsets, ids and codes must all be tensors on cuda:{device}")
                if width == 4 and t.dtype != torch.int32:
                    t = t.to(torch.int32)          # wraps: the low 32 bits are the uint32 the ABI reads
                t = t.contiguous()
                big.append((t, t.data_ptr()))
            else:
                t = np.ascontiguousarray(t, dtype=np.uint32 if width == 4 else np.uint8)
                big.append((t, t.ctypes.data))
        if on_device:
            torch.cuda.synchronize(device)
        ca = _Arrays(N=int(a["N"]), H=int(a["H"]), D=int(a["D"]), P=int(a["P"]), k1=int(a["k1"]), k2=int(a["k2"]),
                     M=int(a["M"]), T=int(a["T"]), C=int(a["C"]),
                     C1=keep[0].ctypes.data, C2=keep[1].ctypes.data, tbl_i=keep[2].ctypes.data,
                     tbl_j=keep[3].ctypes.data, tbl_lambda=keep[4].ctypes.data, cc=keep[5].ctypes.data,
                     offsets=big[0][1], ids=big[1][1], codes=big[2][1], code_format=int(a.get("code_format", 0)))
        _check(_lib.pqt_index_from_arrays(ctypes.byref(ca), PQT_DEVICE if on_device else PQT_HOST, device,
                                          ctypes.byref(self._h)))

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            _lib.pqt_index_free(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        if _lib is not None:               # module globals are cleared while the interpreter shuts down
            self.close()

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def export(self, names=("offsets",)):
        """pqt_index_export of the large arrays named (offsets, ids, codes) into new CUDA tensors
        (int32 views of the uint32 data for offsets and ids)."""
        inf = self.info()
        shapes = {"offsets": ((inf["H"] + 1,), torch.int32), "ids": ((inf["N"],), torch.int32),
                  "codes": ((inf["N"], inf["code_bytes"]), torch.uint8)}
        bufs = {n: torch.empty(shapes[n][0], dtype=shapes[n][1], device=self.device) for n in names}
        ca = _Arrays(**{n: bufs[n].data_ptr() for n in names})
        _check(_lib.pqt_index_export(self._h, ctypes.byref(ca), PQT_DEVICE))
        return bufs

    def save(self, path):
        _check(_lib.pqt_index_save(self._h, os.fsencode(path)))

    def info(self):
        out = _Info()
        _check(_lib.pqt_index_info(self._h, ctypes.byref(out)))
        return {name: getattr(out, name) for name, _ in _Info._fields_}

    def set_budget(self, T, C):
        _check(_lib.pqt_set_budget(self._h, int(T), int(C)))

    def set_bin_order(self, order):
        _check(_lib.pqt_set_bin_order(self._h, int(order)))

    def _buffers(self, queries, k):
        if queries.dtype != torch.float32 or not queries.is_cuda or not queries.is_contiguous() or queries.dim() != 2:
            raise ValueError("queries must be a contiguous 2-D float32 CUDA tensor")
        nq = queries.shape[0]
        out_ids = torch.empty((nq, k), dtype=torch.int64, device=queries.device)
        out_dists = torch.empty((nq, k), dtype=torch.float32, device=queries.device)
        return nq, out_ids, out_dists

    def query_batch(self, queries, k, w, out_ids=None, out_dists=None, stream=None):
        """pqt_query_batch.  queries: (nq, D) float32 CUDA tensor.  Returns (ids int64, dists float32)."""
        if queries.dim() == 2 and queries.shape[1] != self._D:
            raise ValueError(f"queries have dimension {queries.shape[1]}, index has D={self._D}")
        nq, ids_, dists_ = self._buffers(queries, k)
        out_ids = ids_ if out_ids is None else out_ids
        out_dists = dists_ if out_dists is None else out_dists
        _check(_lib.pqt_query_batch(self._h, queries.data_ptr(), nq, int(k), int(w), out_ids.data_ptr(),
                                    out_dists.data_ptr(), _stream_handle(stream)))
        return out_ids, out_dists

    def query_batch_noalloc(self, queries, k, w, out_ids, out_dists, stream=None):
        """pqt_query_batch_noalloc: the caller brings the result tensors, nothing is allocated."""
        if queries.dim() != 2 or queries.shape[1] != self._D or queries.dtype != torch.float32 or \
                not queries.is_cuda or not queries.is_contiguous():
            raise ValueError(f"queries must be a contiguous (nq, {self._D}) float32 CUDA tensor")
        nq = queries.shape[0]
        for t, dt in ((out_ids, torch.int64), (out_dists, torch.float32)):
            if t.dtype != dt or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != (nq, int(k)):
                raise ValueError(f"results go to contiguous ({nq}, {k}) int64 / float32 CUDA tensors")
        _check(_lib.pqt_query_batch_noalloc(self._h, queries.data_ptr(), nq, int(k), int(w), out_ids.data_ptr(),
                                            out_dists.data_ptr(), _stream_handle(stream)))
        return out_ids, out_dists

    def query_batch_debug(self, queries, k, w, taps=_TAP_FIELDS, stream=None):
        """pqt_query_batch_debug.  Returns (ids, dists, dict of tap tensors)."""
        inf = self.info()
        if queries.dim() == 2 and queries.shape[1] != inf["D"]:
            raise ValueError(f"queries have dimension {queries.shape[1]}, index has D={inf['D']}")
        nq, out_ids, out_dists = self._buffers(queries, k)
        P, M, k1, T, C, R = inf["P"], inf["M"], inf["k1"], inf["T"], inf["C"], w * inf["k2"]
        dev = queries.device
        shapes = {
            "a": ((nq, M, k1), torch.float32), "sel": ((nq, P, w), torch.int32),
            "L_d": ((nq, P, R), torch.float32), "L_id": ((nq, P, R), torch.int32),
            "n_tuples": ((nq,), torch.int32), "tuples": ((nq, T, 4), torch.int16),
            "tuple_keys": ((nq, T), torch.float32), "n_slots": ((nq,), torch.int32),
            "slots": ((nq, T), torch.int64), "n_cand": ((nq,), torch.int32),
            "cand_ids": ((nq, C), torch.int64), "scores": ((nq, C), torch.float32),
            "lut": ((nq, M, 256), torch.float32),
        }
        bufs = {name: torch.zeros(shapes[name][0], dtype=shapes[name][1], device=dev) for name in taps}
        ct = _Taps(**{name: bufs[name].data_ptr() for name in taps})
        _check(_lib.pqt_query_batch_debug(self._h, queries.data_ptr(), nq, int(k), int(w), out_ids.data_ptr(),
                                          out_dists.data_ptr(), _stream_handle(stream), ctypes.byref(ct)))
        return out_ids, out_dists, bufs

    def set_vectors(self, vectors):
        """pqt_index_set_vectors.  vectors: (N, D) float32 or uint8; a NumPy array is copied to the GPU,
        a CUDA tensor is used in place (this object keeps a reference to it); None detaches."""
        import numpy as np
        if vectors is None:
            _check(_lib.pqt_index_set_vectors(self._h, None, 0, PQT_HOST))
            self._vectors = None
            return
        on_device = torch.is_tensor(vectors)
        if on_device:
            if not (vectors.is_cuda and vectors.is_contiguous() and vectors.dtype in (torch.float32, torch.uint8)):
                raise ValueError("vectors must be a contiguous float32 or uint8 CUDA tensor")
            elem, ptr = vectors.element_size(), vectors.data_ptr()
            torch.cuda.synchronize(vectors.device)
        else:
            if vectors.dtype not in (np.float32, np.uint8):
                raise ValueError("vectors must be float32 or uint8")
            vectors = np.ascontiguousarray(vectors)
            elem, ptr = vectors.dtype.itemsize, vectors.ctypes.data
        inf = self.info()
        if tuple(vectors.shape) != (inf["N"], inf["D"]):
            raise ValueError(f"vectors have shape {tuple(vectors.shape)}, index has N={inf['N']} D={inf['D']}")
        _check(_lib.pqt_index_set_vectors(self._h, ptr, elem, PQT_DEVICE if on_device else PQT_HOST))
        self._vectors = vectors if on_device else None

    def query_batch_exact(self, queries, k_short, k, w, out_ids=None, out_dists=None, stream=None):
        """pqt_query_batch_exact.  Returns (ids int64, exact squared distances float32)."""
        nq, ids_, dists_ = self._buffers(queries, k)
        out_ids = ids_ if out_ids is None else out_ids
        out_dists = dists_ if out_dists is None else out_dists
        _check(_lib.pqt_query_batch_exact(self._h, queries.data_ptr(), nq, int(k_short), int(k), int(w),
                                          out_ids.data_ptr(), out_dists.data_ptr(), _stream_handle(stream)))
        return out_ids, out_dists

    def brute_force(self, queries, k, out_ids=None, out_dists=None, stream=None):
        """pqt_brute_force.  Returns (ids int64, exact squared distances float32)."""
        nq, ids_, dists_ = self._buffers(queries, k)
        out_ids = ids_ if out_ids is None else out_ids
        out_dists = dists_ if out_dists is None else out_dists
        _check(_lib.pqt_brute_force(self._h, queries.data_ptr(), nq, int(k), out_ids.data_ptr(),
                                    out_dists.data_ptr(), _stream_handle(stream)))
        return out_ids, out_dists

    def set_profiling(self, enabled):
        _check(_lib.pqt_set_profiling(self._h, 1 if enabled else 0))

    def stage_times(self):
        """(ms per stage summed over the calls since the last read, number of calls)."""
        ms = (ctypes.c_float * 4)()
        calls = ctypes.c_int()
        _check(_lib.pqt_stage_times(self._h, ctypes.byref(ms), ctypes.byref(calls)))
        return [float(v) for v in ms], int(calls.value)


def _small_arrays(a):
    """The small host arrays in the ABI's order.  The line table may be missing for (pair, lambda)
    codes, which do not use it; zeros stand in."""
    import numpy as np
    small = {"C1": np.float32, "C2": np.float32, "tbl_i": np.uint8, "tbl_j": np.uint8,
             "tbl_lam": np.float32, "cc": np.float32}
    out = []
    for n, dt in small.items():
        v = a.get(n)
        if v is None and n.startswith("tbl_") and int(a.get("code_format", 0)) == PQT_CODES_PAIR_LAMBDA:
            v = np.zeros((int(a["M"]), 256), dtype=dt)
        out.append(np.ascontiguousarray(v, dtype=dt))
    return out


class Builder:
    """pqt_builder_create / add / finish / free: streams database vectors (CUDA tensors) into an index."""

    def __init__(self, params, device=0):
        keep = _small_arrays(params)
        ca = _Arrays(N=int(params["N"]), H=int(params["H"]), D=int(params["D"]), P=int(params["P"]),
                     k1=int(params["k1"]), k2=int(params["k2"]), M=int(params["M"]), T=int(params["T"]),
                     C=int(params["C"]), C1=keep[0].ctypes.data, C2=keep[1].ctypes.data,
                     tbl_i=keep[2].ctypes.data, tbl_j=keep[3].ctypes.data, tbl_lambda=keep[4].ctypes.data,
                     cc=keep[5].ctypes.data, offsets=None, ids=None, codes=None,
                     code_format=int(params.get("code_format", 0)))
        self._h = ctypes.c_void_p()
        self._device = int(device)
        self._D = int(params["D"])
        _check(_lib.pqt_builder_create(ctypes.byref(ca), self._device, ctypes.byref(self._h)))

    def add(self, vectors, stream=None):
        if vectors.dtype != torch.float32 or not vectors.is_cuda or not vectors.is_contiguous() or \
                vectors.dim() != 2 or vectors.shape[1] != self._D:
            raise ValueError(f"vectors must be a contiguous (n, {self._D}) float32 CUDA tensor")
        _check(_lib.pqt_builder_add(self._h, vectors.data_ptr(), vectors.shape[0], _stream_handle(stream)))

    def finish(self):
        h = ctypes.c_void_p()
        _check(_lib.pqt_builder_finish(self._h, ctypes.byref(h)))
        return Index(device=self._device, handle=h)

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            _lib.pqt_builder_free(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        if _lib is not None:
            self.close()


def pqt_measure_peaks(device=0):
    """(HBM read GB/s, fp32 MFMA TFLOP/s) measured on the device."""
    bw, fl = ctypes.c_double(), ctypes.c_double()
    _check(_lib.pqt_measure_peaks(int(device), ctypes.byref(bw), ctypes.byref(fl)))
    return bw.value, fl.value


def last_error():
    return _lib.pqt_last_error().decode("utf-8", "replace")


# ---- the C ABI's names, one to one ---------------------------------------------------------------
def pqt_index_load(path, device=0):
    return Index(path, device)


def pqt_index_from_arrays(arrays, device=0):
    return Index(device=device, arrays=arrays)


def pqt_index_export(index, names=("offsets",)):
    return index.export(names)


def pqt_index_save(index, path):
    index.save(path)


def pqt_train(vectors, *, P, k1, k2, M, iters=20, n_table=None, stream=None):
    """pqt_train.  vectors: contiguous (n, D) float32 CUDA tensor.  Returns the trained arrays as NumPy
    arrays named as the index arrays: C1, C2, tbl_i, tbl_j, tbl_lam, cc."""
    import numpy as np
    if vectors.dtype != torch.float32 or not vectors.is_cuda or not vectors.is_contiguous() or vectors.dim() != 2:
        raise ValueError("vectors must be a contiguous 2-D float32 CUDA tensor")
    n, D = vectors.shape
    n_table = n if n_table is None else min(int(n_table), n)
    out = dict(C1=np.zeros((P, k1, D // P), np.float32), C2=np.zeros((P, k1, k2, D // P), np.float32),
               tbl_i=np.zeros((M, 256), np.uint8), tbl_j=np.zeros((M, 256), np.uint8),
               tbl_lam=np.zeros((M, 256), np.float32), cc=np.zeros((M, k1, k1), np.float32))
    tp = _TrainParams(D=int(D), P=int(P), k1=int(k1), k2=int(k2), M=int(M), iters=int(iters), n=int(n), n_table=int(n_table))
    _check(_lib.pqt_train(ctypes.byref(tp), vectors.data_ptr(), vectors.device.index or 0, out["C1"].ctypes.data,
                          out["C2"].ctypes.data, out["tbl_i"].ctypes.data, out["tbl_j"].ctypes.data,
                          out["tbl_lam"].ctypes.data, out["cc"].ctypes.data, _stream_handle(stream)))
    return out


def pqt_builder_create(params, device=0):
    return Builder(params, device)


def pqt_builder_add(builder, vectors, stream=None):
    builder.add(vectors, stream)


def pqt_builder_finish(builder):
    return builder.finish()


def pqt_builder_free(builder):
    builder.close()


def pqt_index_free(index):
    index.close()


def pqt_index_info(index):
    return index.info()


def pqt_set_budget(index, T_bins, C_candidates):
    index.set_budget(T_bins, C_candidates)


def pqt_set_bin_order(index, order):
    index.set_bin_order(order)


def pqt_query_batch(index, queries, k, w, out_ids=None, out_dists=None, stream=None):
    return index.query_batch(queries, k, w, out_ids, out_dists, stream)


def pqt_query_batch_noalloc(index, queries, k, w, out_ids, out_dists, stream=None):
    return index.query_batch_noalloc(queries, k, w, out_ids, out_dists, stream)


def pqt_noalloc_workspace_bytes():
    return int(_lib.pqt_noalloc_workspace_bytes())


def pqt_query_batch_debug(index, queries, k, w, taps=_TAP_FIELDS, stream=None):
    return index.query_batch_debug(queries, k, w, taps, stream)


def pqt_index_set_vectors(index, vectors):
    index.set_vectors(vectors)


def pqt_query_batch_exact(index, queries, k_short, k, w, out_ids=None, out_dists=None, stream=None):
    return index.query_batch_exact(queries, k_short, k, w, out_ids, out_dists, stream)


def pqt_brute_force(index, queries, k, out_ids=None, out_dists=None, stream=None):
    return index.brute_force(queries, k, out_ids, out_dists, stream)


def pqt_set_profiling(index, enabled):
    index.set_profiling(enabled)


def pqt_stage_times(index):
    return index.stage_times()


def pqt_last_error():
    return last_error()
