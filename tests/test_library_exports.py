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


def test_offline_driver_holds_no_arithmetic():
    """The package's offline driver only marshals arguments: training, binning and encoding are the
    library's (pqt_train, pqt_builder_*)."""
    import inspect
    from paper_1702_05911_amd import builder
    src = inspect.getsource(builder)
    for banned in ("torch.cdist", ".argmin(", ".min(", "@", "bincount", "index_add", "cumsum", "torch.sort", "numpy"):
        assert banned not in src, banned


def test_slot_of_a_bin_by_reciprocal_multiplication():
    """The kernels take a bin number modulo H (Sec. 4: bins are hashed into the pointer array) without a
    division: r = bin - floor(bin * floor(2^64 / H) / 2^64) * H, then one conditional subtraction.  The same
    integer arithmetic in Python must give bin % H for every H >= 2 and every 64-bit bin number, the
    extreme ones included (the quotient estimate is the quotient or one less)."""
    import random
    rng = random.Random(7)
    mask = (1 << 64) - 1
    hs = [2, 3, 5, 997, 65537, 10_000_019, (1 << 31) - 1, (1 << 32) - 1, 1 << 20, (1 << 32) - 5]
    hs += [rng.randrange(2, 1 << 32) for _ in range(200)]
    for H in hs:
        H_inv = (1 << 64) // H
        bins = [0, 1, H - 1, H, H + 1, mask, mask - 1, (mask // H) * H, (mask // H) * H - 1, 1 << 36, (1 << 36) - 1]
        bins += [rng.randrange(0, 1 << 64) for _ in range(200)] + [rng.randrange(0, 1 << 36) for _ in range(200)]
        for b in bins:
            q = (b * H_inv) >> 64
            r = (b - q * H) & mask
            assert r < 2 * H, (H, b)
            if r >= H:
                r -= H
            assert r == b % H, (H, b)
