"""ctypes wrapper around the plain-C oracle (numpy arrays in, numpy arrays out).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the CPU-baseline leg of
the benchmark; never by the library or its Python binding.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rago_oracle.c")
_LIB = os.path.join(_HERE, "librago_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fused multiply-add, OpenMP over queries)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _arr(a, dt):
    return np.ascontiguousarray(np.asarray(a), dtype=dt)


def _chk(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


I64 = ctypes.c_int64


def num_threads() -> int:
    return int(_load().oracle_num_threads())


METRICS = {"ip": 0, "l2": 1}


def coarse(Q, C, metric="ip"):
    Q, C = _arr(Q, np.float32), _arr(C, np.float32)
    S = np.empty((Q.shape[0], C.shape[0]), np.float32)
    fn = _load().oracle_coarse_l2 if METRICS[metric] else _load().oracle_coarse
    _chk(fn(_p(Q), _p(C), I64(Q.shape[0]), I64(C.shape[0]), I64(Q.shape[1]), _p(S)), "coarse")
    return S


def select(S, nprobe):
    S = _arr(S, np.float32)
    probes = np.empty((S.shape[0], nprobe), np.int32)
    _chk(_load().oracle_select(_p(S), I64(S.shape[0]), I64(S.shape[1]), I64(nprobe), _p(probes)), "select")
    return probes


def select_tree(Q, upper, C, nsp, nprobe, metric="ip"):
    """Probes through an upper level: `upper` = dict(super_centroids [nsuper][d], super_offsets [nsuper+1],
    super_lists [nlist]); returns (probes [nq][nprobe], kept groups [nq][nsp])."""
    Q, C = _arr(Q, np.float32), _arr(C, np.float32)
    SC = _arr(upper["super_centroids"], np.float32)
    soff, sl = _arr(upper["super_offsets"], np.int64), _arr(upper["super_lists"], np.int32)
    nq, d = Q.shape
    probes, sup = np.empty((nq, nprobe), np.int32), np.empty((nq, nsp), np.int32)
    _chk(_load().oracle_select_tree(_p(Q), _p(SC), _p(soff), _p(sl), _p(C), I64(nq), I64(SC.shape[0]), I64(C.shape[0]), I64(d),
                                    I64(nsp), I64(nprobe), ctypes.c_int(METRICS[metric]), _p(probes), _p(sup)), "select_tree")
    return probes, sup


def lut_f32(Q, C, CB, probes, metric="ip"):
    Q, C, CB, probes = _arr(Q, np.float32), _arr(C, np.float32), _arr(CB, np.float32), _arr(probes, np.int32)
    nq, d = Q.shape
    m = CB.shape[0]
    L = np.empty((nq, probes.shape[1], m, 256), np.float32)
    fn = _load().oracle_lut_f32_l2 if METRICS[metric] else _load().oracle_lut_f32
    _chk(fn(_p(Q), _p(C), _p(CB), _p(probes), I64(nq), I64(probes.shape[1]), I64(d), I64(m), _p(L)), "lut_f32")
    return L


def quantise(L):
    L = _arr(L, np.float32)
    nq, nprobe, m, _ = L.shape
    LUT8 = np.empty(L.shape, np.uint8)
    B = np.empty((nq, nprobe), np.int32)
    delta = np.empty(nq, np.float32)
    _chk(_load().oracle_quantise(_p(L), I64(nq), I64(nprobe), I64(m), _p(LUT8), _p(B), _p(delta)), "quantise")
    return LUT8, B, delta


def scan_topk(probes, LUT8, B, delta, list_offsets, codes, ids, k):
    probes, LUT8, B = _arr(probes, np.int32), _arr(LUT8, np.uint8), _arr(B, np.int32)
    delta = None if delta is None else _arr(delta, np.float32)
    off, codes, ids = _arr(list_offsets, np.int64), _arr(codes, np.uint8), _arr(ids, np.int64)
    nq, nprobe = probes.shape
    m = codes.shape[1]
    oi, osc, ois = np.empty((nq, k), np.int64), np.empty((nq, k), np.float32), np.empty((nq, k), np.int32)
    _chk(_load().oracle_scan_topk(_p(probes), _p(LUT8), _p(B), _p(delta), _p(off), _p(codes), _p(ids), I64(nq),
                                  I64(nprobe), I64(m), I64(k), _p(oi), _p(ois), _p(osc)), "scan_topk")
    return oi, ois, osc


def adc_f32_topk(probes, L, list_offsets, codes, ids, k):
    probes, L = _arr(probes, np.int32), _arr(L, np.float32)
    off, codes, ids = _arr(list_offsets, np.int64), _arr(codes, np.uint8), _arr(ids, np.int64)
    nq, nprobe = probes.shape
    oi, osc = np.empty((nq, k), np.int64), np.empty((nq, k), np.float32)
    _chk(_load().oracle_adc_f32_topk(_p(probes), _p(L), _p(off), _p(codes), _p(ids), I64(nq), I64(nprobe),
                                     I64(codes.shape[1]), I64(k), _p(oi), _p(osc)), "adc_f32_topk")
    return oi, osc


def expand_pq4(codebooks16):
    """Codebooks of a 4-bit PQ index [m][16][dsub] -> the 256-word codebooks of its code bytes [m/2][256][2*dsub]."""
    cb = _arr(codebooks16, np.float32)
    m, ks, dsub = cb.shape
    assert ks == 16
    out = np.empty((m // 2, 256, 2 * dsub), np.float32)
    _chk(_load().oracle_expand_pq4(_p(cb), I64(m), I64(dsub), _p(out)), "expand_pq4")
    return out


def ivfpq_search(Q, index, nprobe, k, metric="ip"):
    """index: dict with numpy arrays centroids, codebooks, list_offsets, codes, ids.
    metric "ip" = inner product, "l2" = minus squared Euclidean distance."""
    Q = _arr(Q, np.float32)
    C, CB = _arr(index["centroids"], np.float32), _arr(index["codebooks"], np.float32)
    if CB.shape[1] == 16:              # 4-bit PQ: search on the codebooks of its code bytes
        CB = expand_pq4(CB)
    off, codes, ids = _arr(index["list_offsets"], np.int64), _arr(index["codes"], np.uint8), _arr(index["ids"], np.int64)
    nq, d = Q.shape
    oi, osc, ois = np.empty((nq, k), np.int64), np.empty((nq, k), np.float32), np.empty((nq, k), np.int32)
    probes, delta = np.empty((nq, nprobe), np.int32), np.empty(nq, np.float32)
    _chk(_load().oracle_ivfpq_search(_p(Q), I64(nq), I64(d), _p(C), I64(C.shape[0]), _p(CB), I64(CB.shape[0]),
                                     _p(off), _p(codes), _p(ids), I64(nprobe), I64(k), ctypes.c_int(METRICS[metric]),
                                     _p(oi), _p(osc), _p(ois), _p(probes), _p(delta)), "ivfpq_search")
    return dict(ids=oi, scores=osc, iscores=ois, probes=probes, delta=delta)


def flat_search(corpus_bits, query_bits, k, fmt="bf16"):
    """corpus_bits uint16 [R][n][d], query_bits uint16 [R][nq][d]: raw bit patterns of bf16 (default) or IEEE
    binary16 (`fmt="f16"`) numbers."""
    X, Qb = _arr(corpus_bits, np.uint16), _arr(query_bits, np.uint16)
    R, n, d = X.shape
    nqr = Qb.shape[1]
    oi, osc = np.empty((R, nqr, k), np.int64), np.empty((R, nqr, k), np.float32)
    fn = {"bf16": _load().oracle_flat_search, "f16": _load().oracle_flat_search_f16}[fmt]
    _chk(fn(_p(X), _p(Qb), I64(R), I64(n), I64(nqr), I64(d), I64(k), _p(oi), _p(osc)), "flat_search")
    return oi, osc
