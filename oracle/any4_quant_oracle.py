"""ctypes front end of the CPU oracle of the quantiser (oracle/any4_quant_oracle.c).
TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg, never by the product package.  Arguments and results are numpy arrays."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "any4_quant_oracle.c")
# ANY4_ORACLE_SANITIZE=1 selects a second build of the same source with AddressSanitizer and
# UndefinedBehaviorSanitizer (tests/test_oracle_sanitized.py runs the pins against it)
_SANITIZE = os.environ.get("ANY4_ORACLE_SANITIZE", "") == "1"
_LIB = os.path.join(_HERE, "libany4_quant_oracle_san.so" if _SANITIZE else "libany4_quant_oracle.so")
GROUP = 128


def build(force: bool = False) -> str:
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
        i64, p, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        lib.any4qo_scale_row.restype = ci
        lib.any4qo_scale_row.argtypes = [p, p, i64, ci, ci, p, p, p, p]
        lib.any4qo_init.restype = ci
        lib.any4qo_init.argtypes = [p, p, i64, ci, p, p]
        lib.any4qo_assign.restype = i64
        lib.any4qo_assign.argtypes = [p, i64, p, ci, p]
        lib.any4qo_update.restype = None
        lib.any4qo_update.argtypes = [p, p, p, i64, p, ci]
        lib.any4qo_objective.restype = ctypes.c_double
        lib.any4qo_objective.argtypes = [p, p, p, i64, p]
        lib.any4qo_lloyd.restype = ci
        lib.any4qo_lloyd.argtypes = [p, p, i64, ci, ci, p, p]
        lib.any4qo_emit.restype = None
        lib.any4qo_emit.argtypes = [p, ci, p, i64, p]
        lib.any4qo_quantize.restype = ci
        lib.any4qo_quantize.argtypes = [p, p, p, i64, i64, ci, ci, ci, p, p, p, p, p, ci]
        _lib = lib
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def scale_row(w, act, bits: int, symmetric: bool = False):
    """One row: (scale bf16 bits [G], offset bf16 bits [G], scaled weights fp32 [K], sample weights fp32 [K])."""
    w = _f32(w)
    K = w.shape[0]
    a = None if act is None else _f32(act)
    scale = np.empty(K // GROUP, dtype=np.uint16)
    offset = np.empty(K // GROUP, dtype=np.uint16)
    ws = np.empty(K, dtype=np.float32)
    s = np.empty(K, dtype=np.float32)
    rc = _load().any4qo_scale_row(_p(w), None if a is None else _p(a), K, bits, int(symmetric),
                                  _p(scale), _p(offset), _p(ws), _p(s))
    if rc != 0:
        raise ValueError("any4qo_scale_row: bad arguments")
    return scale, offset, ws, s


def init(ws, s, L: int, u):
    """Weighted k-means++ centres (fp64 [L]) from the draws u (fp32 [L], each in [0, 1))."""
    ws, s, u = _f32(ws), _f32(s), _f32(u)
    c = np.empty(L, dtype=np.float64)
    if _load().any4qo_init(_p(ws), _p(s), ws.shape[0], L, _p(u), _p(c)) != 0:
        raise MemoryError
    return c


def assign(ws, c, codes=None):
    """E-step.  Returns (codes uint8 [K], number of codes that changed)."""
    ws = _f32(ws)
    c = np.ascontiguousarray(c, dtype=np.float64)
    codes = np.full(ws.shape[0], 0xFF, dtype=np.uint8) if codes is None else np.ascontiguousarray(codes, dtype=np.uint8).copy()
    changed = _load().any4qo_assign(_p(ws), ws.shape[0], _p(c), c.shape[0], _p(codes))
    return codes, int(changed)


def update(ws, s, codes, c):
    """M-step.  Returns the new centres (fp64 [L])."""
    ws, s = _f32(ws), _f32(s)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    c = np.ascontiguousarray(c, dtype=np.float64).copy()
    _load().any4qo_update(_p(ws), _p(s), _p(codes), ws.shape[0], _p(c), c.shape[0])
    return c


def objective(ws, s, codes, c) -> float:
    ws, s = _f32(ws), _f32(s)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    c = np.ascontiguousarray(c, dtype=np.float64)
    return float(_load().any4qo_objective(_p(ws), _p(s), _p(codes), ws.shape[0], _p(c)))


def lloyd(ws, s, c0, iters: int):
    """Returns (centres fp64 [L], codes uint8 [K], M-steps done)."""
    ws, s = _f32(ws), _f32(s)
    c = np.ascontiguousarray(c0, dtype=np.float64).copy()
    codes = np.empty(ws.shape[0], dtype=np.uint8)
    done = _load().any4qo_lloyd(_p(ws), _p(s), ws.shape[0], c.shape[0], iters, _p(c), _p(codes))
    return c, codes, int(done)


def emit(c, codes):
    """Sorted bf16 table (uint16 [L]) and renumbered codes."""
    c = np.ascontiguousarray(c, dtype=np.float64)
    codes = np.ascontiguousarray(codes, dtype=np.uint8).copy()
    lut = np.empty(c.shape[0], dtype=np.uint16)
    _load().any4qo_emit(_p(c), c.shape[0], _p(codes), codes.shape[0], _p(lut))
    return lut, codes


def quantize(w, act, u, bits: int, symmetric: bool = False, iters: int = 20, threads: int = 1):
    """w fp32 [N,K]; act fp32 [K] or None; u fp32 [N, 2^bits].  Returns a dict with
    codes_u8 [N,K], lut / scale / offset (bf16 bit patterns) and msteps int32 [N]."""
    w = _f32(w)
    N, K = w.shape
    L = 1 << bits
    a = None if act is None else _f32(act)
    u = _f32(u)
    assert u.shape == (N, L)
    codes = np.empty((N, K), dtype=np.uint8)
    lut = np.empty((N, L), dtype=np.uint16)
    scale = np.empty((N, K // GROUP), dtype=np.uint16)
    offset = np.empty((N, K // GROUP), dtype=np.uint16)
    msteps = np.empty(N, dtype=np.int32)
    rc = _load().any4qo_quantize(_p(w), None if a is None else _p(a), _p(u), N, K, bits, int(symmetric), iters,
                                 _p(codes), _p(lut), _p(scale), _p(offset), _p(msteps), threads)
    if rc != 0:
        raise ValueError(f"any4qo_quantize failed with {rc}")
    return {"codes_u8": codes, "lut": lut, "scale": scale, "offset": offset, "msteps": msteps}
