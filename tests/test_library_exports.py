"""The C-ABI library loads and exports every symbol include/pqt.h declares (no compute calls)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "pqt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pqt_[a-z_]+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = _declared_symbols()
    for must in ("pqt_index_load", "pqt_index_free", "pqt_index_info", "pqt_set_budget", "pqt_query_batch",
                 "pqt_query_batch_debug", "pqt_last_error"):
        assert must in names


def test_library_exports_every_declared_symbol():
    import torch  # noqa: F401  the HIP runtime the library links against ships with torch
    path = os.path.join(ROOT, "paper_1702_05911_amd", "libpqt.so")
    if not os.path.exists(path):
        from paper_1702_05911_amd import buildlib
        buildlib.build_library()
    lib = ctypes.CDLL(path)
    for name in _declared_symbols():
        assert hasattr(lib, name), name
    lib.pqt_last_error.restype = ctypes.c_char_p
    assert lib.pqt_last_error() == b""


def test_binding_uses_the_same_names():
    import paper_1702_05911_amd.binding as b
    for name in _declared_symbols():
        assert hasattr(b, name), name
    # host-side argument checks that need no GPU
    rc = b._lib.pqt_index_info(None, None)
    assert rc == b.PQT_EINVAL and b"null" in b._lib.pqt_last_error()
    h = ctypes.c_void_p()
    rc = b._lib.pqt_index_load(b"/nonexistent/file.pqt", 0, ctypes.byref(h))
    assert rc == b.PQT_EIO


def test_product_builder_output_satisfies_the_oracle_definitions(tiny, tmp_path):
    """The package's fp32 builder is separate code; its index must be a valid PQT index by the
    oracle's definitions: bins partition X, every id sits in slot m(x), codes are nearest code points."""
    import numpy as np
    from oracle import pqt_build as B, pqt_index_io as IO
    from paper_1702_05911_amd import builder
    cfg, X, Y, _ = tiny
    path = str(tmp_path / "prod.pqt")
    builder.build_index(path, X, P=cfg.P, k1=cfg.k1, k2=cfg.k2, M=cfg.M, T=cfg.T, C=cfg.C, device="cpu")
    ix = IO.read_index(path)
    off = ix.offsets.astype(np.int64)
    assert off[0] == 0 and off[-1] == cfg.N and np.all(np.diff(off) >= 0)
    assert np.array_equal(np.sort(ix.ids), np.arange(cfg.N))
    np.testing.assert_allclose(ix.cc, B.pair_table(ix.C1, ix.M), rtol=1e-6)
    mism = 0
    for t in range(0, cfg.N, 41):
        slot = int(np.searchsorted(off, t, side="right")) - 1
        x = X[ix.ids[t]]
        mism += slot != B.bin_slot(x, ix.C1, ix.C2, ix.H)
        mism += not np.array_equal(ix.codes[t], B.encode_vector(x, ix.C1, ix.M, ix.tbl_i, ix.tbl_j, ix.tbl_lam))
    assert mism <= 2          # fp32 vs fp64 near-ties only
