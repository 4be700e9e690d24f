"""Thin ctypes binding of librago.so: argument marshalling only.

Function names mirror the C ABI declared in include/rago.h.  PyTorch is used for device memory
(`torch.empty(..., device="cuda")`, `.data_ptr()`) and for the current HIP stream; every step of
the search runs inside the library's kernels.  There is no CPU fallback: importing this module
without a built library raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librago.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                      "(or paper_2503_14649_amd/build.py) first; there is no fallback path")
_lib = ctypes.CDLL(LIB_PATH)

_vp, _i64, _i32, _int = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int


class _Arrays(ctypes.Structure):
    _fields_ = [("d", _i32), ("m", _i32), ("nlist", _i32), ("metric", _i32), ("n", _i64), ("ksub", _i32), ("reserved", _i32),
                ("centroids", _vp), ("codebooks", _vp),
                ("list_offsets", _vp), ("codes", _vp), ("ids", _vp)]


class IndexDesc(ctypes.Structure):
    _fields_ = [("d", _i32), ("m", _i32), ("ksub", _i32), ("nlist", _i32), ("n", _i64), ("metric", _i32),
                ("device", _i32), ("max_list_len", _i64), ("code_bytes_resident", _i64)]


_lib.rago_last_error.restype = ctypes.c_char_p
_lib.rago_index_load.argtypes = [ctypes.c_char_p, _int, ctypes.POINTER(_vp)]
_lib.rago_index_wrap.argtypes = [ctypes.POINTER(_Arrays), _int, _int, ctypes.POINTER(_vp)]
_lib.rago_index_free.argtypes = [_vp]
_lib.rago_index_reserve.argtypes = [_vp, _i64, _i32, _i32]
_lib.rago_debug_force_scan_kernel.argtypes = [_int]
_lib.rago_debug_allocations.restype = _i64
_lib.rago_index_info.argtypes = [_vp, ctypes.POINTER(IndexDesc)]
_lib.rago_ivfpq_search.argtypes = [_vp, _vp, _i64, _i32, _i32, _vp, _vp, _vp, _vp]
_lib.rago_flat_search.argtypes = [_vp, _vp, _i32, _i64, _i32, _i32, _i32, _vp, _vp, _int, _vp]
_lib.rago_flat_search_f16.argtypes = _lib.rago_flat_search.argtypes
_lib.rago_flat_search_static.argtypes = [_vp, _vp, _i32, _i64, _i32, _i32, _i32, _i32, _vp, _vp, _int, _vp]
_lib.rago_index_set_upper_level.argtypes = [_vp, _i32, _vp, _vp, _vp, _int]
_lib.rago_index_set_upper_probe.argtypes = [_vp, _i32]
_lib.rago_debug_select_tree.argtypes = [_vp, _vp, _i64, _i32, _vp, _vp, _vp]
_lib.rago_debug_coarse.argtypes = [_vp, _vp, _i64, _vp, _vp]
_lib.rago_debug_select.argtypes = [_vp, _vp, _vp, _i64, _i32, _vp, _vp]
_lib.rago_debug_build_lut.argtypes = [_vp, _vp, _vp, _i64, _i32, _vp, _vp, _vp, _vp, _vp]
_lib.rago_debug_scan.argtypes = [_vp, _vp, _vp, _vp, _i64, _i32, _i32, _vp, _vp, _vp]
_lib.rago_debug_counters.argtypes = [_vp, _vp, _vp]
_lib.rago_debug_copy.argtypes = [_vp, _vp, _i64, _vp]
_lib.rago_debug_read_stream.argtypes = [_vp, _i64, _vp, _vp]
_lib.rago_debug_flat_profile.argtypes = [_int, _int]
_lib.rago_debug_flat_stage_ms.argtypes = [_int, _vp, _vp]
_lib.rago_debug_profile.argtypes = [_vp, _int]
_lib.rago_debug_stage_ms.argtypes = [_vp, _vp, _vp]


class RagoError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"rago error {code}: {msg}")
        self.code = code


def _chk(rc):
    if rc != 0:
        raise RagoError(rc, _lib.rago_last_error().decode())


def rago_last_error() -> str:
    return _lib.rago_last_error().decode()


def _stream(dev):
    return _vp(torch.cuda.current_stream(dev).cuda_stream)


def _ptr(t):
    return None if t is None else _vp(t.data_ptr())


def rago_index_load(path: str, device: int = 0):
    h = _vp()
    _chk(_lib.rago_index_load(os.fsencode(path), device, ctypes.byref(h)))
    return h


METRICS = {"ip": 0, "l2": 1}


def rago_index_wrap(index: dict, device: int = 0, metric="ip"):
    """index: tensors centroids [nlist][d] f32, codebooks [m][ksub][dsub] f32 (ksub 256, or 16 for 4-bit codes),
    list_offsets [nlist+1] i64, codes [n][m] u8 ([n][m/2] with ksub 16), ids [n] i64; all on the CPU or all on cuda:`device`.
    metric: "ip" (inner product) or "l2" (similarity = minus the squared Euclidean distance)."""
    c = index["centroids"].contiguous().float()
    cb = index["codebooks"].contiguous().float()
    off = index["list_offsets"].contiguous().to(torch.int64)
    codes = index["codes"].contiguous()
    ids = index["ids"].contiguous().to(torch.int64)
    assert codes.dtype == torch.uint8
    on_dev = c.is_cuda
    assert all(t.is_cuda == on_dev for t in (cb, off, codes, ids)), "all arrays must live on the same side"
    a = _Arrays(c.shape[1], cb.shape[0], c.shape[0], METRICS[metric] if isinstance(metric, str) else int(metric), codes.shape[0],
                cb.shape[1], 0, _ptr(c), _ptr(cb), _ptr(off), _ptr(codes), _ptr(ids))
    h = _vp()
    if on_dev:
        torch.cuda.synchronize(device)
    _chk(_lib.rago_index_wrap(ctypes.byref(a), int(on_dev), device, ctypes.byref(h)))
    return h


def rago_index_set_upper_level(h, upper: dict | None):
    """upper: tensors super_centroids [nsuper][d] f32, super_offsets [nsuper+1] i64, super_lists [nlist] i32, all on the
    CPU or all on the GPU; None removes the level."""
    if upper is None:
        _chk(_lib.rago_index_set_upper_level(h, 0, None, None, None, 0))
        return
    sc = upper["super_centroids"].contiguous().float()
    off = upper["super_offsets"].contiguous().to(torch.int64)
    sl = upper["super_lists"].contiguous().to(torch.int32)
    on_dev = sc.is_cuda
    assert off.is_cuda == on_dev and sl.is_cuda == on_dev, "all arrays must live on the same side"
    if on_dev:
        torch.cuda.synchronize(sc.device)
    _chk(_lib.rago_index_set_upper_level(h, sc.shape[0], _ptr(sc), _ptr(off), _ptr(sl), int(on_dev)))


def rago_index_set_upper_probe(h, nsp: int):
    _chk(_lib.rago_index_set_upper_probe(h, nsp))


def rago_index_free(h):
    _chk(_lib.rago_index_free(h))


def rago_index_info(h) -> IndexDesc:
    d = IndexDesc()
    _chk(_lib.rago_index_info(h, ctypes.byref(d)))
    return d


def rago_ivfpq_search(h, queries: torch.Tensor, nprobe: int, k: int, want_iscores: bool = True, out=None):
    """queries: cuda fp32 [nq][d].  Returns (ids i64 [nq][k], scores f32 [nq][k], iscores i32 [nq][k] or None)."""
    assert queries.is_cuda and queries.dtype == torch.float32 and queries.is_contiguous()
    nq, dev = queries.shape[0], queries.device
    if out is None:
        ids = torch.empty(nq, k, dtype=torch.int64, device=dev)
        scores = torch.empty(nq, k, dtype=torch.float32, device=dev)
        isc = torch.empty(nq, k, dtype=torch.int32, device=dev) if want_iscores else None
    else:
        ids, scores, isc = out
    _chk(_lib.rago_ivfpq_search(h, _ptr(queries), nq, nprobe, k, _ptr(ids), _ptr(scores), _ptr(isc), _stream(dev)))
    return ids, scores, isc


def rago_flat_search_f16(corpus: torch.Tensor, queries: torch.Tensor, k: int, out=None):
    """corpus fp16 [R][n][d], queries fp16 [R][nqr][d] on the GPU -> (ids i64 [R][nqr][k], scores f32)."""
    return _flat(_lib.rago_flat_search_f16, torch.float16, corpus, queries, k, out)


def rago_flat_search(corpus: torch.Tensor, queries: torch.Tensor, k: int, out=None):
    """corpus bf16 [R][n][d], queries bf16 [R][nqr][d] on the GPU -> (ids i64 [R][nqr][k], scores f32)."""
    return _flat(_lib.rago_flat_search, torch.bfloat16, corpus, queries, k, out)


def rago_flat_search_static(corpus: torch.Tensor, queries: torch.Tensor, k: int, out):
    """The flat search that allocates nothing: corpus / queries bf16 or fp16 (both alike), `out` = (ids i64
    [R][nqr][k], scores f32 [R][nqr][k]) preallocated by the caller."""
    assert corpus.is_cuda and queries.is_cuda and corpus.dtype == queries.dtype
    assert corpus.dtype in (torch.bfloat16, torch.float16) and corpus.is_contiguous() and queries.is_contiguous()
    R, n, d = corpus.shape
    nqr, dev = queries.shape[1], corpus.device
    ids, scores = out
    assert ids.shape == (R, nqr, k) and scores.shape == (R, nqr, k) and ids.dtype == torch.int64 and scores.dtype == torch.float32
    _chk(_lib.rago_flat_search_static(_ptr(corpus), _ptr(queries), R, n, nqr, d, k, int(corpus.dtype == torch.float16),
                                      _ptr(ids), _ptr(scores), dev.index or 0, _stream(dev)))
    return ids, scores


def _flat(fn, dtype, corpus, queries, k, out):
    assert corpus.is_cuda and queries.is_cuda and corpus.dtype == dtype and queries.dtype == dtype
    assert corpus.is_contiguous() and queries.is_contiguous()
    R, n, d = corpus.shape
    nqr, dev = queries.shape[1], corpus.device
    if out is None:
        ids = torch.empty(R, nqr, k, dtype=torch.int64, device=dev)
        scores = torch.empty(R, nqr, k, dtype=torch.float32, device=dev)
    else:
        ids, scores = out
    _chk(fn(_ptr(corpus), _ptr(queries), R, n, nqr, d, k, _ptr(ids), _ptr(scores), dev.index or 0, _stream(dev)))
    return ids, scores


def rago_debug_coarse(h, queries):
    info = rago_index_info(h)
    S = torch.empty(queries.shape[0], info.nlist, dtype=torch.float32, device=queries.device)
    _chk(_lib.rago_debug_coarse(h, _ptr(queries), queries.shape[0], _ptr(S), _stream(queries.device)))
    return S


def rago_debug_select_tree(h, queries, nprobe, nsp):
    """Probes through the upper level (nsp = the value given to rago_index_set_upper_probe): (probes, kept groups)."""
    queries = queries.contiguous()
    dev = queries.device
    nq = queries.shape[0]
    probes = torch.empty(nq, nprobe, dtype=torch.int32, device=dev)
    groups = torch.empty(nq, nsp, dtype=torch.int32, device=dev)
    _chk(_lib.rago_debug_select_tree(h, _ptr(queries), nq, nprobe, _ptr(probes), _ptr(groups), _stream(dev)))
    return probes, groups


def rago_debug_select(h, queries, S, nprobe):
    probes = torch.empty(S.shape[0], nprobe, dtype=torch.int32, device=S.device)
    _chk(_lib.rago_debug_select(h, _ptr(queries), _ptr(S), S.shape[0], nprobe, _ptr(probes), _stream(S.device)))
    return probes


def rago_debug_build_lut(h, queries, probes, want_f32=True):
    info = rago_index_info(h)
    nq, nprobe = probes.shape
    dev = queries.device
    mb = info.m // 2 if info.ksub == 16 else info.m          # code bytes per vector = tables per (query, list) pair
    L = torch.empty(nq, nprobe, mb, 256, dtype=torch.float32, device=dev) if want_f32 else None
    L8 = torch.empty(nq, nprobe, mb, 256, dtype=torch.uint8, device=dev)
    B = torch.empty(nq, nprobe, dtype=torch.int32, device=dev)
    delta = torch.empty(nq, dtype=torch.float32, device=dev)
    _chk(_lib.rago_debug_build_lut(h, _ptr(queries), _ptr(probes), nq, nprobe, _ptr(L), _ptr(L8), _ptr(B), _ptr(delta),
                                   _stream(dev)))
    return L, L8, B, delta


def rago_debug_scan(h, probes, LUT8, B, k):
    nq, nprobe = probes.shape
    dev = probes.device
    ids = torch.empty(nq, k, dtype=torch.int64, device=dev)
    isc = torch.empty(nq, k, dtype=torch.int32, device=dev)
    _chk(_lib.rago_debug_scan(h, _ptr(probes), _ptr(LUT8), _ptr(B), nq, nprobe, k, _ptr(ids), _ptr(isc), _stream(dev)))
    return ids, isc


def rago_debug_counters(h, device=0):
    out = (ctypes.c_int64 * 8)()
    _chk(_lib.rago_debug_counters(h, out, _stream(torch.device("cuda", device))))
    return list(out)


def rago_debug_copy(src: torch.Tensor, dst: torch.Tensor):
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _chk(_lib.rago_debug_copy(_ptr(src), _ptr(dst), nbytes, _stream(src.device)))


def rago_index_reserve(h, max_nq: int, max_nprobe: int, max_k: int):
    _chk(_lib.rago_index_reserve(h, max_nq, max_nprobe, max_k))


SCAN_KERNELS = {"auto": 0, "wide": 1, "narrow": 2, "wave": 3}


def rago_debug_force_scan_kernel(which):
    _chk(_lib.rago_debug_force_scan_kernel(SCAN_KERNELS[which] if isinstance(which, str) else int(which)))


def rago_debug_allocations() -> int:
    return int(_lib.rago_debug_allocations())


def rago_debug_read_stream(src: torch.Tensor, sink: torch.Tensor):
    """sink: uint32/int32 tensor of >= 4096 words on src's device."""
    assert sink.numel() >= 4096 and sink.element_size() == 4
    _chk(_lib.rago_debug_read_stream(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream(src.device)))


def rago_debug_flat_profile(device: int, enable: bool):
    _chk(_lib.rago_debug_flat_profile(device, int(enable)))


def rago_debug_flat_stage_ms(device: int):
    out = (ctypes.c_float * 2)()
    n = ctypes.c_int32()
    _chk(_lib.rago_debug_flat_stage_ms(device, out, ctypes.byref(n)))
    return {"scan": out[0], "merge": out[1]}, n.value


STAGES = ("coarse", "select", "lut", "scan_setup", "scan", "merge", "total")


def rago_debug_profile(h, enable: bool):
    _chk(_lib.rago_debug_profile(h, int(enable)))


def rago_debug_stage_ms(h):
    out = (ctypes.c_float * 8)()
    n = ctypes.c_int32()
    _chk(_lib.rago_debug_stage_ms(h, out, ctypes.byref(n)))
    return {name: float(out[i]) for i, name in enumerate(STAGES)}, int(n.value)


class Index:
    """Owning handle with the search calls as methods."""

    def __init__(self, handle, device=0):
        self.h, self.device = handle, device

    @classmethod
    def load(cls, path, device=0):
        return cls(rago_index_load(path, device), device)

    @classmethod
    def wrap(cls, index: dict, device=0, metric="ip"):
        return cls(rago_index_wrap(index, device, metric), device)

    def info(self):
        return rago_index_info(self.h)

    def search(self, queries, nprobe, k, **kw):
        return rago_ivfpq_search(self.h, queries, nprobe, k, **kw)

    def counters(self):
        return rago_debug_counters(self.h, self.device)

    def close(self):
        if self.h is not None:
            rago_index_free(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
