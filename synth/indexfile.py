"""Writer for the on-disk IVF-PQ index consumed by `rago_index_load` (little-endian).

Layout: 64-byte header {magic "RAGOIVPQ", u32 version=1, u32 metric (0 = inner product),
u32 d, u32 m, u32 ksub, u32 nlist, u64 n, zero padding} followed, back to back, by
centroids f32[nlist][d], codebooks f32[m][ksub][d/m], list_offsets i64[nlist+1],
codes u8[n][m] (list-major, one row per vector; u8[n][m/2] when ksub = 16: two 4-bit codes per byte, the
even sub-quantiser in the low nibble) and ids i64[n] (list-major).
"""
import struct

import numpy as np

MAGIC = b"RAGOIVPQ"
HEADER_BYTES = 64


def write_index(path, index, metric: int = 0) -> None:
    c = index["centroids"].detach().cpu().numpy().astype("<f4", copy=False)
    cb = index["codebooks"].detach().cpu().numpy().astype("<f4", copy=False)
    off = index["list_offsets"].detach().cpu().numpy().astype("<i8", copy=False)
    codes = index["codes"].detach().cpu().numpy().astype("u1", copy=False)
    ids = index["ids"].detach().cpu().numpy().astype("<i8", copy=False)
    nlist, d = c.shape
    m, ksub, _ = cb.shape
    n = codes.shape[0]
    hdr = MAGIC + struct.pack("<IIIIIIQ", 1, metric, d, m, ksub, nlist, n)
    hdr += b"\0" * (HEADER_BYTES - len(hdr))
    with open(path, "wb") as f:
        f.write(hdr)
        for a in (c, cb, off, codes, ids):
            f.write(np.ascontiguousarray(a).tobytes())
