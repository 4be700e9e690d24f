"""Optional HIP helper of the input generator (PQ encoding at billion-vector scale)."""
import ctypes
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csrc", "encode.hip")
_LIB = os.path.join(_HERE, "libsynth_encode.so")
_lib = None


def build() -> str:
    subprocess.check_call(["hipcc", "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
                           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                           "-Wno-unused-command-line-argument", "-o", _LIB, _SRC])
    return _LIB


def available() -> bool:
    return os.path.exists(_LIB)


def pq_encode(x, centroids, lists, codebooks, out):
    """x [n][d] f32, lists [n] i64, out [n][m] u8: all CUDA tensors."""
    global _lib
    import torch
    if _lib is None:
        _lib = ctypes.CDLL(_LIB)
        _lib.synth_pq_encode.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                                                  ctypes.c_void_p, ctypes.c_void_p]
    n, d = x.shape
    m = codebooks.shape[0]
    assert x.is_contiguous() and out.is_contiguous() and centroids.is_contiguous() and codebooks.is_contiguous()
    rc = _lib.synth_pq_encode(x.data_ptr(), centroids.data_ptr(), lists.data_ptr(), codebooks.data_ptr(), n, d, m,
                              out.data_ptr(), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    if rc != 0:
        raise RuntimeError(f"synth_pq_encode failed: {rc}")
