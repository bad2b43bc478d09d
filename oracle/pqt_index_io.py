"""Oracle-side reader/writer of the PQT index file.

TEST INFRASTRUCTURE.  The file layout is an interface shared with the HIP
library (which has its own C++ reader) and with the package's builder (its own
writer); only the layout is common, no code.

Layout (little endian).  256-byte header:
   0  char[8]  "PQTIDX1\\0"
   8  u32 version (=1)   12 u32 D   16 u32 P   20 u32 k1   24 u32 k2   28 u32 M
  32  u64 N              40 u64 H   48 u32 T   52 u32 C    56 u32 offset_bits (=32)
  60  u32 code_format (0: one byte per sub-part, 1: two)   64..255 zero
then nine sections, each starting at the next multiple of 256 bytes:
  C1      f32 [P][k1][D/P]
  C2      f32 [P][k1][k2][D/P]
  tbl_i   u8  [M][256]
  tbl_j   u8  [M][256]
  tbl_lam f32 [M][256]
  cc      f32 [M][k1][k1]
  offsets u32 [H+1]
  ids     u32 [N]
  codes   u8  [N][M]   ([N][2M] for code_format 1)
"""
import struct

import numpy as np

from .pqt_query import PQTIndex

MAGIC = b"PQTIDX1\0"
ALIGN = 256


def _sections(D, P, k1, k2, M, N, H, code_format=0):
    dp = D // P
    return [
        ("C1", np.float32, (P, k1, dp)),
        ("C2", np.float32, (P, k1, k2, dp)),
        ("tbl_i", np.uint8, (M, 256)),
        ("tbl_j", np.uint8, (M, 256)),
        ("tbl_lam", np.float32, (M, 256)),
        ("cc", np.float32, (M, k1, k1)),
        ("offsets", np.uint32, (H + 1,)),
        ("ids", np.uint32, (N,)),
        ("codes", np.uint8, (N, M * (2 if code_format == 1 else 1))),
    ]


def write_index(path, ix: PQTIndex):
    hdr = bytearray(ALIGN)
    hdr[0:8] = MAGIC
    struct.pack_into("<6I", hdr, 8, 1, ix.D, ix.P, ix.k1, ix.k2, ix.M)
    struct.pack_into("<2Q", hdr, 32, ix.N, ix.H)
    struct.pack_into("<4I", hdr, 48, ix.T, ix.C, 32, ix.code_format)
    with open(path, "wb") as f:
        f.write(hdr)
        for name, dt, shape in _sections(ix.D, ix.P, ix.k1, ix.k2, ix.M, ix.N, ix.H, ix.code_format):
            arr = np.ascontiguousarray(getattr(ix, name), dtype=dt)
            assert arr.shape == shape, (name, arr.shape, shape)
            pad = (-f.tell()) % ALIGN
            f.write(b"\0" * pad)
            f.write(arr.tobytes())


def read_index(path) -> PQTIndex:
    with open(path, "rb") as f:
        hdr = f.read(ALIGN)
        if len(hdr) != ALIGN or hdr[0:8] != MAGIC:
            raise ValueError("not a PQT index file")
        ver, D, P, k1, k2, M = struct.unpack_from("<6I", hdr, 8)
        N, H = struct.unpack_from("<2Q", hdr, 32)
        T, C, obits, fmt = struct.unpack_from("<4I", hdr, 48)
        if ver != 1 or obits != 32 or fmt > 1:
            raise ValueError("unsupported PQT index version")
        fields = {}
        for name, dt, shape in _sections(D, P, k1, k2, M, N, H, fmt):
            f.seek((-f.tell()) % ALIGN, 1)
            cnt = int(np.prod(shape))
            arr = np.fromfile(f, dtype=dt, count=cnt)
            if arr.shape[0] != cnt:
                raise ValueError("truncated PQT index file")
            fields[name] = arr.reshape(shape)
    return PQTIndex(D=D, P=P, k1=k1, k2=k2, M=M, N=N, H=H, T=T, C=C, code_format=fmt, **fields)
