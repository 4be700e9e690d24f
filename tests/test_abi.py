"""CPU-only: the C-ABI library loads and exports every symbol include/rago.h declares; host-side
argument checking works without a GPU."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2503_14649_amd", "librago.so")


def _lib():
    if not os.path.exists(LIB):
        import sys
        sys.path.insert(0, ROOT)
        from paper_2503_14649_amd.build import build
        build()
    return ctypes.CDLL(LIB)


def test_every_declared_symbol_is_exported():
    hdr = open(os.path.join(ROOT, "include", "rago.h")).read()
    names = set(re.findall(r"\b(rago_[a-z_0-9]+)\s*\(", hdr))
    names = {n for n in names if not n.startswith("rago_index_arrays") and n != "rago_status"}
    assert {"rago_index_load", "rago_ivfpq_search", "rago_flat_search", "rago_index_wrap"} <= names
    lib = _lib()
    for n in sorted(names):
        assert hasattr(lib, n), n


def test_host_side_argument_errors():
    lib = _lib()
    lib.rago_last_error.restype = ctypes.c_char_p
    h = ctypes.c_void_p()
    assert lib.rago_index_load(None, 0, ctypes.byref(h)) == -1
    assert lib.rago_index_load(b"/nonexistent/index.bin", 0, ctypes.byref(h)) == -2
    assert b"cannot open" in lib.rago_last_error()
    assert lib.rago_index_free(None) == 0
    assert lib.rago_ivfpq_search(None, None, ctypes.c_int64(1), 1, 1, None, None, None, None) == -1
    assert lib.rago_flat_search(None, None, 1, ctypes.c_int64(10), 16, 768, 500, None, None, 0, None) == -6


def test_bad_index_files(tmp_path):
    lib = _lib()
    lib.rago_last_error.restype = ctypes.c_char_p
    h = ctypes.c_void_p()
    p = tmp_path / "short.bin"
    p.write_bytes(b"RAGOIVPQ" + b"\0" * 10)
    assert lib.rago_index_load(str(p).encode(), 0, ctypes.byref(h)) == -3
    p = tmp_path / "magic.bin"
    p.write_bytes(b"NOTANIDX" + b"\0" * 56)
    assert lib.rago_index_load(str(p).encode(), 0, ctypes.byref(h)) == -3
    import struct
    hdr = b"RAGOIVPQ" + struct.pack("<IIIIIIQ", 1, 0, 32, 16, 256, 4, 100)
    p = tmp_path / "trunc.bin"
    p.write_bytes(hdr + b"\0" * (64 - len(hdr)) + b"\0" * 1000)           # far shorter than the header says
    assert lib.rago_index_load(str(p).encode(), 0, ctypes.byref(h)) == -3
    assert b"truncated" in lib.rago_last_error()
    hdr = b"RAGOIVPQ" + struct.pack("<IIIIIIQ", 1, 0, 32, 16, 128, 4, 100)  # ksub != 256
    p = tmp_path / "ksub.bin"
    p.write_bytes(hdr + b"\0" * (64 - len(hdr)))
    assert lib.rago_index_load(str(p).encode(), 0, ctypes.byref(h)) == -6
