"""numpy-facing wrapper of the CPU oracle (oracle/rwkvq_oracle.c).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's CPU
baseline may import this; the GPU library never does, and this module imports
nothing from the GPU package.  All arithmetic lives in the C file; this wrapper
only marshals numpy arrays and widens fp16 / bf16 bit patterns of the
activations to float32 (exact).

The C file is compiled with gcc on first use (or when the source is newer than
the shared object).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from ctypes import c_int, c_int64, c_void_p

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rwkvq_oracle.c")
_SO = os.path.join(_HERE, "librwkvq_oracle.so")
CFLAGS = ["-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC", "-std=c11",
          "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    stale = (not os.path.exists(_SO)) or os.path.getmtime(_SO) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _SO + f".tmp{os.getpid()}"
        subprocess.run(["gcc", *CFLAGS, "-o", tmp, _SRC], check=True)
        os.replace(tmp, _SO)
    return _SO


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.rwkvq_oracle_half_to_float.restype = ctypes.c_float
        L.rwkvq_oracle_half_to_float.argtypes = [ctypes.c_uint16]
        L.rwkvq_oracle_bf16_to_float.restype = ctypes.c_float
        L.rwkvq_oracle_bf16_to_float.argtypes = [ctypes.c_uint16]
        L.rwkvq_oracle_float_to_half.restype = ctypes.c_uint16
        L.rwkvq_oracle_float_to_half.argtypes = [ctypes.c_float]
        L.rwkvq_oracle_float_to_bf16.restype = ctypes.c_uint16
        L.rwkvq_oracle_float_to_bf16.argtypes = [ctypes.c_float]
        L.rwkvq_oracle_field.restype = ctypes.c_uint32
        L.rwkvq_oracle_field.argtypes = [c_void_p, c_int, c_int64]
        L.rwkvq_oracle_unpack.restype = None
        L.rwkvq_oracle_unpack.argtypes = [c_void_p, c_int64, c_int64, c_int, c_int64, c_void_p]
        L.rwkvq_oracle_round.restype = None
        L.rwkvq_oracle_round.argtypes = [c_void_p, c_int64, c_int]
        L.rwkvq_oracle_sq_dequant.restype = None
        L.rwkvq_oracle_sq_dequant.argtypes = [c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int,
                                              c_int, c_void_p]
        L.rwkvq_oracle_vq_dequant.restype = None
        L.rwkvq_oracle_vq_dequant.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int, c_int,
                                              c_int, c_int, c_void_p]
        L.rwkvq_oracle_gemm.restype = None
        L.rwkvq_oracle_gemm.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int64, c_int, c_void_p]
        L.rwkvq_oracle_sq_linear.restype = None
        L.rwkvq_oracle_sq_linear.argtypes = [c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int,
                                             c_int, c_void_p, c_int64, c_int, c_int, c_void_p]
        L.rwkvq_oracle_vq_linear.restype = None
        L.rwkvq_oracle_vq_linear.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int, c_int, c_int,
                                             c_int, c_void_p, c_int64, c_int, c_int, c_void_p]
        L.rwkvq_oracle_threads.restype = c_int
        L.rwkvq_oracle_threads.argtypes = []
        _lib = L
    return _lib


_ROUND = {None: 0, "none": 0, "f32": 0, "f16": 1, "bf16": 2}
_ACC = {"f32": 0, "f64": 1}


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data_as(c_void_p)


def threads() -> int:
    return int(lib().rwkvq_oracle_threads())


def widen(bits: np.ndarray, dtype: str) -> np.ndarray:
    """fp16 / bf16 bit patterns (uint16) -> float32, exact."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float32)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << 16).view(np.float32)
    raise ValueError(dtype)


def unpack(words: np.ndarray, width: int, fields_per_row: int) -> np.ndarray:
    """[rows, words_per_row] uint32 bit strings -> [rows, fields_per_row] uint16 fields."""
    words, pw = _c(words, np.uint32)
    rows, wpr = words.shape
    assert fields_per_row * width <= wpr * 32
    out = np.empty((rows, fields_per_row), dtype=np.uint16)
    lib().rwkvq_oracle_unpack(pw, rows, wpr, width, fields_per_row, out.ctypes.data_as(c_void_p))
    return out


def round_weights(w: np.ndarray, to: str) -> np.ndarray:
    """Nearest-even rounding of float32 values to fp16 / bf16, returned as float32."""
    out = np.array(w, dtype=np.float32, order="C", copy=True)
    lib().rwkvq_oracle_round(out.ctypes.data_as(c_void_p), out.size, _ROUND[to])
    return out


def sq_dequant(codes, scales, zeros, K: int, bits: int = 3, group: int = 128) -> np.ndarray:
    codes, pc = _c(codes, np.uint32)
    scales, ps = _c(scales, np.uint16)
    zeros, pz = _c(zeros, np.uint16)
    N = codes.shape[0]
    assert codes.shape == (N, K * bits // 32) and scales.shape == (N, K // group) == zeros.shape
    w = np.empty((N, K), dtype=np.float32)
    lib().rwkvq_oracle_sq_dequant(pc, ps, pz, N, K, bits, group, w.ctypes.data_as(c_void_p))
    return w


def vq_dequant(indices, codebooks, K: int, kbits: int, vdim: int = 2, block_rows: int = 256,
               block_cols: int = 256) -> np.ndarray:
    indices, pi = _c(indices, np.uint32)
    codebooks, pcb = _c(codebooks, np.uint16)
    N = indices.shape[0]
    assert indices.shape == (N, (K // vdim) * kbits // 32)
    assert codebooks.shape == (N // block_rows, K // block_cols, 1 << kbits, vdim)
    w = np.empty((N, K), dtype=np.float32)
    lib().rwkvq_oracle_vq_dequant(pi, pcb, N, K, vdim, kbits, block_rows, block_cols,
                                  w.ctypes.data_as(c_void_p))
    return w


def gemm(w: np.ndarray, x: np.ndarray, acc: str = "f32") -> np.ndarray:
    """y[m, n] = sum_k w[n, k] x[m, k] (k ascending) in float32 or float64; returned as float64."""
    w, pw = _c(w, np.float32)
    x, px = _c(x, np.float32)
    N, K = w.shape
    M = x.shape[0]
    assert x.shape == (M, K)
    y = np.empty((M, N), dtype=np.float64)
    lib().rwkvq_oracle_gemm(pw, px, M, N, K, _ACC[acc], y.ctypes.data_as(c_void_p))
    return y


def linear(mat, x: np.ndarray, acc: str = "f32", weight_round=None) -> np.ndarray:
    """y = x Deq(W)^T for a matrix record with fields kind, N, K, kbits, codes, scales, zeros,
    codebooks (canonical layout); x is float32 [M, K].  Returned as float64 [M, N]."""
    x, px = _c(x, np.float32)
    M = x.shape[0]
    assert x.shape == (M, mat.K)
    y = np.empty((M, mat.N), dtype=np.float64)
    py = y.ctypes.data_as(c_void_p)
    codes, pc = _c(mat.codes, np.uint32)
    if mat.kind == "sq":
        scales, ps = _c(mat.scales, np.uint16)
        zeros, pz = _c(mat.zeros, np.uint16)
        lib().rwkvq_oracle_sq_linear(pc, ps, pz, mat.N, mat.K, 3, 128, px, M, _ROUND[weight_round],
                                     _ACC[acc], py)
    elif mat.kind == "vq":
        cb, pcb = _c(mat.codebooks, np.uint16)
        lib().rwkvq_oracle_vq_linear(pc, pcb, mat.N, mat.K, 2, mat.kbits, 256, 256, px, M,
                                     _ROUND[weight_round], _ACC[acc], py)
    else:
        raise ValueError(mat.kind)
    return y


def dequant(mat) -> np.ndarray:
    if mat.kind == "sq":
        return sq_dequant(mat.codes, mat.scales, mat.zeros, mat.K)
    return vq_dequant(mat.codes, mat.codebooks, mat.K, mat.kbits)


def narrow(y: np.ndarray, dtype: str) -> np.ndarray:
    """float32 values -> fp16 / bf16 bit patterns with the oracle's own nearest-even routines."""
    L = lib()
    f = {"f16": L.rwkvq_oracle_float_to_half, "bf16": L.rwkvq_oracle_float_to_bf16}[dtype]
    flat = np.ascontiguousarray(y, dtype=np.float32).ravel()
    return np.array([f(float(v)) for v in flat], dtype=np.uint16).reshape(np.shape(y))
