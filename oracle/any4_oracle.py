"""ctypes front end of the CPU oracle (oracle/any4_oracle.c).  TEST INFRASTRUCTURE ONLY:
imported by tests/, by the smoke check and by the benchmark's cpu_baseline leg, never
by the product package.  Arguments and results are numpy arrays on the host."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "any4_oracle.c")
# ANY4_ORACLE_SANITIZE=1 selects a second build of the same source with AddressSanitizer and
# UndefinedBehaviorSanitizer (tests/test_oracle_sanitized.py runs the pins against it)
_SANITIZE = os.environ.get("ANY4_ORACLE_SANITIZE", "") == "1"
_LIB = os.path.join(_HERE, "libany4_oracle_san.so" if _SANITIZE else "libany4_oracle.so")
GROUP = 128


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fused contraction of a*b+c expressions, so the
    two-step check inside the dequantiser really rounds twice)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
               "-fno-omit-frame-pointer"] if _SANITIZE else ["-O2"]
        subprocess.check_call(["gcc", *opt, "-std=c11", "-fPIC", "-shared", "-fopenmp",
                               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, p = ctypes.c_int64, ctypes.c_void_p
        lib.any4o_row_words.restype = i64
        lib.any4o_row_words.argtypes = [i64, ctypes.c_int]
        lib.any4o_code.restype = ctypes.c_uint32
        lib.any4o_code.argtypes = [p, i64, ctypes.c_int]
        lib.any4o_pack.restype = ctypes.c_int
        lib.any4o_pack.argtypes = [p, i64, i64, ctypes.c_int, p]
        lib.any4o_repack_words.restype = i64
        lib.any4o_repack_words.argtypes = [i64, i64, ctypes.c_int]
        lib.any4o_repack.restype = ctypes.c_int
        lib.any4o_repack.argtypes = [p, i64, i64, ctypes.c_int, p]
        lib.any4o_dequant.restype = i64
        lib.any4o_dequant.argtypes = [p, p, p, p, i64, i64, ctypes.c_int, p]
        lib.any4o_gemm.restype = ctypes.c_int
        lib.any4o_gemm.argtypes = [p, p, p, p, p, i64, i64, i64, ctypes.c_int, p, ctypes.c_int]
        lib.any4o_dequant_g.restype = i64
        lib.any4o_dequant_g.argtypes = [p, p, p, p, i64, i64, ctypes.c_int, i64, p]
        lib.any4o_gemm_g.restype = ctypes.c_int
        lib.any4o_gemm_g.argtypes = [p, p, p, p, p, i64, i64, i64, ctypes.c_int, i64, p, ctypes.c_int]
        lib.any4o_dequant_gd.restype = i64
        lib.any4o_dequant_gd.argtypes = [p, p, p, p, i64, i64, ctypes.c_int, i64, ctypes.c_int, p]
        lib.any4o_gemm_gd.restype = ctypes.c_int
        lib.any4o_gemm_gd.argtypes = [p, p, p, p, p, i64, i64, i64, ctypes.c_int, i64, ctypes.c_int, p, ctypes.c_int]
        lib.any4o_f16_bits_to_float.restype = ctypes.c_float
        lib.any4o_f16_bits_to_float.argtypes = [ctypes.c_uint16]
        lib.any4o_rms.restype = ctypes.c_double
        lib.any4o_rms.argtypes = [p, i64]
        lib.any4o_bits_per_weight.restype = ctypes.c_double
        lib.any4o_bits_per_weight.argtypes = [i64, ctypes.c_int]
        _lib = lib
    return _lib


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def row_words(K: int, bits: int) -> int:
    return int(_load().any4o_row_words(K, bits))


def pack(codes_u8: np.ndarray, bits: int) -> np.ndarray:
    """uint8 [N,K] (one code per byte) -> uint32 [N, K*bits/32]."""
    N, K = codes_u8.shape
    src, psrc = _c(codes_u8, np.uint8)
    out = np.empty((N, K * bits // 32), dtype=np.uint32)
    rc = _load().any4o_pack(psrc, N, K, bits, out.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError(f"any4o_pack failed with {rc}")
    return out


def repack(packed: np.ndarray, K: int, bits: int) -> np.ndarray:
    """uint32 [N, K*bits/32] -> the tile-major layout, uint32 [ceil(N/16)*16 * K*bits/32]."""
    N = packed.shape[0]
    a, pa = _c(packed, np.uint32)
    words = int(_load().any4o_repack_words(N, K, bits))
    if words < 0:
        raise ValueError("any4o_repack_words: bad arguments")
    out = np.empty(words, dtype=np.uint32)
    if _load().any4o_repack(pa, N, K, bits, out.ctypes.data_as(ctypes.c_void_p)) != 0:
        raise ValueError("any4o_repack: bad arguments")
    return out


def code(row_words_arr: np.ndarray, k: int, bits: int) -> int:
    r, pr = _c(row_words_arr, np.uint32)
    return int(_load().any4o_code(pr, k, bits))


def unpack(packed: np.ndarray, K: int, bits: int) -> np.ndarray:
    """Inverse of pack, element by element through any4o_code."""
    N = packed.shape[0]
    out = np.empty((N, K), dtype=np.uint8)
    for n in range(N):
        row = np.ascontiguousarray(packed[n], dtype=np.uint32)
        pr = row.ctypes.data_as(ctypes.c_void_p)
        for k in range(K):
            out[n, k] = _load().any4o_code(pr, k, bits)
    return out


def f16_bits_to_float(h: int) -> float:
    return float(_load().any4o_f16_bits_to_float(int(h)))


def dequant(packed, lut, scale, offset, K: int, bits: int, return_differ: bool = False, group: int = GROUP,
            f16: bool = False):
    """fp32 [N,K] dequantised weights; optionally also the count of elements whose
    fused and two-step roundings differ (expected 0 for bf16 storage).  scale / offset are
    [N, K / group]; f16: the 16-bit inputs are fp16 bit patterns instead of bf16."""
    N = packed.shape[0]
    a, pa = _c(packed, np.uint32)
    b, pb = _c(lut, np.uint16)
    c, pc = _c(scale, np.uint16)
    d, pd = _c(offset, np.uint16)
    w = np.empty((N, K), dtype=np.float32)
    if c.shape != (N, K // group) or d.shape != (N, K // group):
        raise ValueError("scale / offset must be [N, K / group]")
    differ = _load().any4o_dequant_gd(pa, pb, pc, pd, N, K, bits, group, 1 if f16 else 0, w.ctypes.data_as(ctypes.c_void_p))
    if differ < 0:
        raise ValueError("any4o_dequant: bad arguments")
    return (w, int(differ)) if return_differ else w


def gemm(x, packed, lut, scale, offset, K: int, bits: int, threads: int = 1, group: int = GROUP,
         f16: bool = False) -> np.ndarray:
    """fp64 [M,N] = x[M,K] . dequant(...)[N,K]^T, sequential in k.  scale / offset are [N, K / group];
    f16: the 16-bit inputs are fp16 bit patterns instead of bf16."""
    N = packed.shape[0]
    M = x.shape[0]
    xx, px = _c(x, np.uint16)
    a, pa = _c(packed, np.uint32)
    b, pb = _c(lut, np.uint16)
    c, pc = _c(scale, np.uint16)
    d, pd = _c(offset, np.uint16)
    y = np.empty((M, N), dtype=np.float64)
    if c.shape != (N, K // group) or d.shape != (N, K // group):
        raise ValueError("scale / offset must be [N, K / group]")
    rc = _load().any4o_gemm_gd(px, pa, pb, pc, pd, M, N, K, bits, group, 1 if f16 else 0,
                               y.ctypes.data_as(ctypes.c_void_p), threads)
    if rc != 0:
        raise ValueError("any4o_gemm: bad arguments")
    return y


def rms(y: np.ndarray) -> float:
    yy, py = _c(y, np.float64)
    return float(_load().any4o_rms(py, yy.size))


def bits_per_weight(K: int, bits: int) -> float:
    return float(_load().any4o_bits_per_weight(K, bits))


def gemm_tolerance(y64: np.ndarray, rms_value: float | None = None) -> np.ndarray:
    """Elementwise acceptance bound for a bf16 GEMM result against y64:
    1e-2 * rms(y64) plus half a bf16 ulp of the exact value (output rounding)."""
    r = rms(y64) if rms_value is None else rms_value
    return 1e-2 * r + np.abs(y64) * 2.0 ** -8
