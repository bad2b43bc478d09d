"""The library's host-only code (index-file reader, array validation, fixed traversal-order tables) built
for the CPU with the address and undefined-behaviour sanitizers, and run on valid, truncated and corrupted
index files, on out-of-range sizes, and against the oracle's tables.  No GPU."""
import os
import struct
import subprocess

import numpy as np
import pytest

from oracle import pqt_index_io as IO
from oracle import pqt_query as Q

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, EINVAL, EIO, EFORMAT, ENOMEM, EHIP, EUNSUPPORTED = 0, -1, -2, -3, -4, -5, -6


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("host") / "sanitizer_driver")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-static-libasan", "-static-libubsan", "-ffp-contract=off",
           os.path.join(ROOT, "tests", "host", "sanitizer_driver.cpp"),
           os.path.join(ROOT, "paper_1702_05911_amd", "csrc", "pqt_host.cpp"), "-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr

    def run(*args):
        env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0",
                   UBSAN_OPTIONS="print_stacktrace=1")
        r = subprocess.run([exe] + [str(a) for a in args], capture_output=True, text=True, env=env, timeout=120)
        assert r.returncode == 0 and "Sanitizer" not in r.stderr and "runtime error" not in r.stderr, \
            f"{args}: exit {r.returncode}\n{r.stderr[-2000:]}"
        return r.stdout
    return run


def _rc(out):
    return int(out.split()[1])


def test_valid_files_load(driver, tiny, tiny_pair, tmp_path):
    for name, ix in (("tiny", tiny[3]), ("pair", tiny_pair[3])):
        path = str(tmp_path / f"{name}.pqt")
        IO.write_index(path, ix)
        out = driver("load", path)
        assert _rc(out) == OK
        assert int(out.split()[2]) == int(np.count_nonzero(np.diff(ix.offsets.astype(np.int64))))     # slots that hold a vector


def test_truncated_files_are_format_errors(driver, tiny, tmp_path):
    ix = tiny[3]
    path = str(tmp_path / "tiny.pqt")
    IO.write_index(path, ix)
    blob = open(path, "rb").read()
    cut = str(tmp_path / "cut.pqt")
    # every section boundary (multiples of 256 around the section starts), one byte either side, and a few odd places
    places = {0, 1, 8, 63, 64, 255, 256, 257, len(blob) - 1, len(blob) - 100, len(blob) // 2}
    pos = 256
    dp = ix.D // ix.P
    for nbytes in (ix.P * ix.k1 * dp * 4, ix.P * ix.k1 * ix.k2 * dp * 4, ix.M * 256, ix.M * 256, ix.M * 1024,
                   ix.M * ix.k1 * ix.k1 * 4, (ix.H + 1) * 4, ix.N * 4):
        pos = (pos + 255) // 256 * 256 + nbytes
        places |= {pos - 1, pos, pos + 1, (pos + 255) // 256 * 256}
    for n in sorted(p for p in places if 0 <= p < len(blob)):
        with open(cut, "wb") as f:
            f.write(blob[:n])
        assert _rc(driver("load", cut)) == EFORMAT, n
    assert _rc(driver("load", str(tmp_path / "missing.pqt"))) == EIO


def _patched(blob, offset, fmt, value):
    b = bytearray(blob)
    struct.pack_into(fmt, b, offset, value)
    return bytes(b)


def test_corrupted_headers_and_arrays(driver, tiny, tmp_path):
    ix = tiny[3]
    path = str(tmp_path / "tiny.pqt")
    IO.write_index(path, ix)
    blob = open(path, "rb").read()
    bad = str(tmp_path / "bad.pqt")
    cases = [
        (b"NOTANIDX" + blob[8:], EFORMAT),
        (_patched(blob, 8, "<I", 2), EFORMAT),                       # version
        (_patched(blob, 12, "<I", 0), EFORMAT),                      # D = 0
        (_patched(blob, 12, "<I", ix.D + 1), EFORMAT),               # D not a multiple of P and M
        (_patched(blob, 16, "<I", 3), EFORMAT),                      # P = 3 does not divide D = 32
        (_patched(blob, 20, "<I", 0xFFFFFFFF), EUNSUPPORTED),        # k1 beyond the limit
        (_patched(blob, 24, "<I", 5000), EUNSUPPORTED),              # k2 beyond the limit
        (_patched(blob, 28, "<I", 0), EFORMAT),                      # M = 0
        (_patched(blob, 32, "<Q", 2 ** 40), EUNSUPPORTED),           # N beyond 32 bits: nothing is allocated
        (_patched(blob, 32, "<Q", ix.N + 1), EFORMAT),               # N larger than the file holds
        (_patched(blob, 40, "<Q", ix.H + 1), EFORMAT),               # H above the number of bins
        (_patched(blob, 40, "<Q", 0), EFORMAT),
        (_patched(blob, 48, "<I", 0), EFORMAT),                      # T = 0
        (_patched(blob, 52, "<I", 1 << 20), EFORMAT),                # C beyond the limit
        (_patched(blob, 56, "<I", 64), EFORMAT),                     # offset_bits
        (_patched(blob, 60, "<I", 7), EFORMAT),                      # code_format
    ]
    for n, (data, want) in enumerate(cases):
        with open(bad, "wb") as f:
            f.write(data)
        out = driver("load", bad)
        assert _rc(out) == want, (n, out)
    # arrays: pointer array not monotone / not spanning the ids, table entry naming a centroid >= k1
    for mutate, want in ((lambda b: b.offsets.__setitem__(5, b.offsets[-1] + 7), EFORMAT),
                         (lambda b: b.offsets.__setitem__(-1, b.offsets[-1] - 1), EFORMAT),
                         (lambda b: b.offsets.__setitem__(0, 1), EFORMAT),
                         (lambda b: b.tbl_j.__setitem__((1, 17), ix.k1), EFORMAT)):
        broken = IO.read_index(path)
        broken.offsets, broken.tbl_j = broken.offsets.copy(), broken.tbl_j.copy()
        mutate(broken)
        IO.write_index(bad, broken)
        assert _rc(driver("load", bad)) == want


def test_pair_code_bytes_are_checked(driver, tiny_pair, tmp_path):
    ix = tiny_pair[3]
    path = str(tmp_path / "pair.pqt")
    IO.write_index(path, ix)
    broken = IO.read_index(path)
    broken.codes = broken.codes.copy()
    broken.codes[17, 2] = ix.k1 * (ix.k1 - 1) // 2                 # one past the last pair
    IO.write_index(path, broken)
    assert _rc(driver("load", path)) == EFORMAT


def test_size_limits(driver):
    ok = dict(D=128, P=2, k1=16, k2=8, M=8, N=1000, H=16384, T=1024, C=4096, fmt=0)

    def rc(**kw):
        v = dict(ok, **kw)
        return driver("sizes", *[v[n] for n in ("D", "P", "k1", "k2", "M", "N", "H", "T", "C", "fmt")]).split()[1:3]
    assert rc() == ["0", "plain"]
    assert rc(H=9973) == ["0", "hashed"]
    assert rc(P=4, H=10_000_019) == ["0", "hashed"]
    assert rc(P=4, k1=256, k2=1024, M=4)[0] == str(EUNSUPPORTED)    # (k1 k2)^4 = 2^72 bins
    assert rc(P=4, k1=256, k2=256, M=4, H=10 ** 9)[0] == str(EUNSUPPORTED)   # (2^16)^4 = 2^64: one too many for 64-bit bin numbers
    assert rc(P=4, k1=256, k2=128, M=4, H=10 ** 9) == ["0", "hashed"]       # 2^60 bins, hashed to 10^9 slots
    assert rc(k1=257)[0] == str(EUNSUPPORTED)
    assert rc(D=8200, M=8, P=2)[0] == str(EUNSUPPORTED)
    assert rc(M=3)[0] == str(EFORMAT)                              # M not a multiple of P
    assert rc(T=8193)[0] == str(EFORMAT)
    assert rc(fmt=1, k1=24)[0] == str(EUNSUPPORTED)                # 276 centroid pairs do not fit a byte
    assert rc(fmt=1, k1=23)[0] == "0"
    assert rc(fmt=1, k1=1, H=64)[0] == str(EUNSUPPORTED)            # no pair of centroids at all


def test_static_order_tables_equal_the_oracles(driver):
    """The ten fixed orders and the nine slope thresholds the library uploads are bit-identical to the oracle's."""
    for R, T in ((1, 1), (4, 16), (7, 30), (16, 100), (32, 1024), (64, 700), (128, 1024), (1024, 8192)):
        lines = driver("static", R, T).strip().split("\n")
        Tn = int(lines[0].split()[1])
        assert Tn == min(T, R * R)
        thr = np.array([float.fromhex(v) for v in lines[1].split()], dtype=np.float32)
        assert np.array_equal(thr, Q.slope_thresholds(np.float32))
        for i, s in enumerate(Q.slopes()):
            got = [tuple(int(v) for v in pair.split(",")) for pair in lines[2 + i].split()]
            if R <= 128:
                assert got == [tuple(t) for t in Q.static_order(R, T, s).tolist()], (R, T, i)
            assert len(got) == Tn and len(set(got)) == Tn


def test_region_size_counts_the_hyperbolic_region(driver):
    for nA, nB, Tn in ((8, 8, 64), (64, 64, 1024), (128, 16, 300), (5, 1000, 37), (1024, 1024, 8192)):
        want = sum(1 for a in range(min(nA, Tn)) for b in range(min(nB, Tn // (a + 1))))
        assert int(driver("region", nA, nB, Tn).split()[1]) == want
