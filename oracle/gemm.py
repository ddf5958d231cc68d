"""Python face of the GEMM oracle (gemm_oracle.c) plus numpy decoders and the error metric.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

`gemm_fp64` is the definition D[i][j] = sum_k A[i][k] B[k][j] in fp64 over the
stored (already rounded) fp16 / bf16 / e4m3 inputs (Sec. 1, Sec. 3.1 of the
paper).  `gemm_numpy` is the library special case (decode, then a float64
matmul) that pins it.
"""
import ctypes
import os
import subprocess

import numpy as np

F16, BF16, E4M3 = 0, 1, 2
_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gemm_oracle.c")
_SO = os.path.join(_HERE, "libgemm_oracle.so")
_lib = None


def build(force=False):
    """Compile gemm_oracle.c with gcc + OpenMP next to its source."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
                               "-o", _SO, _SRC, "-lm"])
    return _SO


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_gemm.restype = ctypes.c_int
        lib.oracle_gemm.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                    ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                    ctypes.c_void_p, ctypes.c_int64, ctypes.c_int]
        lib.oracle_decode.restype = ctypes.c_double
        lib.oracle_decode.argtypes = [ctypes.c_uint32, ctypes.c_int]
        lib.oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads():
    """OpenMP threads the C oracle will use."""
    return _load().oracle_threads()


def _storage(a, dtype):
    want = np.uint8 if dtype == E4M3 else np.uint16
    a = np.ascontiguousarray(a)
    if a.dtype != want:
        raise TypeError("oracle inputs are raw bit patterns: %s expected, got %s" % (want, a.dtype))
    return a


def gemm_fp64(A_bits, B_bits, dtype, rows=None, order=1):
    """A_bits (M x K) and B_bits (K x N) hold storage bit patterns (uint16, or uint8 for
    e4m3).  Returns float64 D (M x N), or only the listed rows of it."""
    A_bits, B_bits = _storage(A_bits, dtype), _storage(B_bits, dtype)
    M, K = A_bits.shape
    K2, N = B_bits.shape
    if K != K2:
        raise ValueError("inner dimensions differ")
    if rows is None:
        rows_arr, n_rows, rows_ptr = None, M, None
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int64)
        n_rows, rows_ptr = len(rows_arr), rows_arr.ctypes.data
    D = np.empty((n_rows, N), dtype=np.float64)
    rc = _load().oracle_gemm(A_bits.ctypes.data, B_bits.ctypes.data, D.ctypes.data,
                             M, N, K, dtype, rows_ptr, n_rows, order)
    if rc != 0:
        raise ValueError("oracle_gemm rejected its arguments")
    return D


def decode_c(bits, dtype):
    """The C decoder, element by element (for pinning it)."""
    lib = _load()
    flat = np.asarray(bits).ravel()
    return np.array([lib.oracle_decode(int(b), dtype) for b in flat]).reshape(np.shape(bits))


def decode_numpy(bits, dtype):
    """Decode storage bit patterns to float64 with numpy only (independent of the C decoder)."""
    bits = np.asarray(bits)
    if dtype == F16:
        return bits.astype(np.uint16).view(np.float16).astype(np.float64)
    if dtype == BF16:
        return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    if dtype == E4M3:
        b = bits.astype(np.int64)
        sign = np.where(b & 0x80, -1.0, 1.0)
        e = (b >> 3) & 0xF
        f = b & 7
        sub = f / 8.0 * 2.0 ** -6
        nor = (1.0 + f / 8.0) * np.exp2((e - 7).astype(np.float64))
        v = np.where(e == 0, sub, nor)
        v = np.where((e == 15) & (f == 7), np.nan, v)
        return sign * v
    raise ValueError("unknown dtype")


def gemm_numpy(A_bits, B_bits, dtype):
    """Library special case: decode, then numpy's float64 matmul."""
    return decode_numpy(A_bits, dtype) @ decode_numpy(B_bits, dtype)


def rel_error(d, ref):
    """Max over elements of |d - ref| / max(|ref|, rms(ref)): element-wise relative error with
    an rms floor, so that entries that cancel to nearly zero do not dominate."""
    d = np.asarray(d, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    den = np.maximum(np.abs(ref), rms if rms > 0 else 1.0)
    return float(np.max(np.abs(d - ref) / den)) if ref.size else 0.0
