"""Thin Python binding of libany4's C ABI (include/any4.h).

Argument marshalling only: every function takes torch tensors that already live in device
memory, checks dtype / shape / contiguity (every array the kernels index is compared with the
shape (N, K, bits, group) implies), and passes raw pointers plus the current HIP stream
to the library.  No arithmetic of the method happens here, and there is no fallback: if the
shared library is missing or a call is made with host tensors, this module raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libany4.so")
GROUP = 128

EXPORTS = ("any4_pack", "any4_dequant", "any4_gemm", "any4_gemm_workspace_bytes", "any4_repack", "any4_repack_bytes", "any4_gemm_repacked", "any4_dequant_grouped", "any4_gemm_grouped", "any4_dequant_f16", "any4_gemm_f16",
           "any4_quantize", "any4_quantize_with_gap", "any4_quantize_max_k", "any4_gemm_noalloc", "any4_dequant_single_table", "any4_gemm_single_table", "any4_strerror", "any4_version")


class Any4Error(RuntimeError):
    pass


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libany4.so from the package directory (build it with
    `python -m paper_2507_04610_amd.build`); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise Any4Error(f"{LIB_PATH} is missing: run `python -m paper_2507_04610_amd.build` first")
    lib = ctypes.CDLL(LIB_PATH)
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    lib.any4_pack.restype = ci
    lib.any4_pack.argtypes = [vp, i64, i64, ci, vp, vp]
    lib.any4_dequant.restype = ci
    lib.any4_dequant.argtypes = [vp, vp, vp, vp, i64, i64, ci, vp, vp]
    lib.any4_gemm.restype = ci
    lib.any4_gemm.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, ci, vp, vp, ctypes.c_size_t, vp]
    lib.any4_gemm_workspace_bytes.restype = ctypes.c_size_t
    lib.any4_gemm_workspace_bytes.argtypes = [i64, i64, i64, ci]
    lib.any4_dequant_grouped.restype = ci
    lib.any4_dequant_grouped.argtypes = [vp, vp, vp, vp, i64, i64, ci, ci, vp, vp]
    lib.any4_dequant_f16.restype = ci
    lib.any4_dequant_f16.argtypes = [vp, vp, vp, vp, i64, i64, ci, vp, vp]
    lib.any4_gemm_f16.restype = ci
    lib.any4_gemm_f16.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, ci, vp, vp, ctypes.c_size_t, vp]
    lib.any4_gemm_grouped.restype = ci
    lib.any4_gemm_grouped.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, ci, ci, vp, vp, ctypes.c_size_t, vp]
    lib.any4_gemm_repacked.restype = ci
    lib.any4_gemm_repacked.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, ci, vp, vp, ctypes.c_size_t, vp]
    lib.any4_dequant_single_table.restype = ci
    lib.any4_dequant_single_table.argtypes = [vp, vp, vp, vp, i64, i64, ci, vp, vp]
    lib.any4_gemm_single_table.restype = ci
    lib.any4_gemm_single_table.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, ci, vp, vp, ctypes.c_size_t, vp]
    lib.any4_gemm_noalloc.restype = ci
    lib.any4_gemm_noalloc.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, ci, vp, vp]
    lib.any4_repack.restype = ci
    lib.any4_repack.argtypes = [vp, i64, i64, ci, vp, vp]
    lib.any4_repack_bytes.restype = ctypes.c_size_t
    lib.any4_repack_bytes.argtypes = [i64, i64, ci]
    lib.any4_quantize.restype = ci
    lib.any4_quantize.argtypes = [vp, vp, vp, i64, i64, ci, ci, ci, vp, vp, vp, vp, vp, vp]
    lib.any4_quantize_with_gap.restype = ci
    lib.any4_quantize_with_gap.argtypes = [vp, vp, vp, i64, i64, ci, ci, ci, ctypes.c_double, vp, vp, vp, vp, vp, vp]
    lib.any4_quantize_max_k.restype = i64
    lib.any4_quantize_max_k.argtypes = []
    lib.any4_strerror.restype = ctypes.c_char_p
    lib.any4_strerror.argtypes = [ci]
    lib.any4_version.restype = ci
    lib.any4_version.argtypes = []
    _lib = lib
    return lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise Any4Error(f"{what} failed: {load_library().any4_strerror(rc).decode()} ({rc})")


def _dev(t: torch.Tensor, dtype, name: str) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise Any4Error(f"{name} must be a tensor in device memory")
    if t.dtype != dtype:
        raise Any4Error(f"{name} must have dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise Any4Error(f"{name} must be contiguous")
    return t.data_ptr()


def _shape(t: torch.Tensor, want, name: str) -> None:
    if tuple(t.shape) != tuple(want):
        raise Any4Error(f"{name} must have shape {tuple(want)}, got {tuple(t.shape)}")


def _check_quant_shapes(codes, lut, scale, offset, N, K, bits, group, repacked=False, single_table=False) -> None:
    """the kernels index these arrays from (N, K, bits, group) alone: a wrong shape would make them read
    out of bounds on the device, so it is refused here"""
    if bits not in (4, 3, 2):
        raise Any4Error(f"bits must be 4, 3 or 2, got {bits}")
    if K < 1 or K % GROUP or group < 1 or K % group:
        raise Any4Error(f"K = {K} must be a positive multiple of 128 and of the group size {group}")
    if repacked:
        need = (N + 15) // 16 * 16 * row_words(K, bits)
        if codes.numel() != need:
            raise Any4Error(f"rcodes must hold {need} words (any4_repack_bytes), got {codes.numel()}")
    else:
        _shape(codes, (N, row_words(K, bits)), "codes")
    if lut is not None and not (single_table and tuple(lut.shape) == (1, 1 << bits)):
        _shape(lut, (N, 1 << bits), "lut")
    _shape(scale, (N, K // group), "scale")
    _shape(offset, (N, K // group), "offset")


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def row_words(K: int, bits: int) -> int:
    return K * bits // 32


def any4_version() -> int:
    return int(load_library().any4_version())


def any4_strerror(code: int) -> str:
    return load_library().any4_strerror(code).decode()


def any4_gemm_workspace_bytes(M: int, N: int, K: int, bits: int = 4) -> int:
    return int(load_library().any4_gemm_workspace_bytes(M, N, K, bits))


def any4_pack(codes_u8: torch.Tensor, bits: int = 4, out: torch.Tensor | None = None) -> torch.Tensor:
    """uint8 [N,K] codes (one per byte) -> packed words, int32 tensor [N, K*bits/32]
    (torch has no usable uint32; the bit patterns are what matters)."""
    lib = load_library()
    N, K = codes_u8.shape
    src = _dev(codes_u8, torch.uint8, "codes_u8")
    if out is None:
        out = torch.empty((N, max(K * bits // 32, 0)), dtype=torch.int32, device=codes_u8.device)
    _shape(out, (N, max(K * bits // 32, 0)), "out")
    dst = _dev(out, torch.int32, "out")
    _check(lib.any4_pack(src, N, K, bits, dst, _stream()), "any4_pack")
    return out


def any4_dequant(codes: torch.Tensor, lut: torch.Tensor | None, scale: torch.Tensor, offset: torch.Tensor,
                 K: int, bits: int = 4, out: torch.Tensor | None = None, group: int = GROUP) -> torch.Tensor:
    """fp32 [N,K] dequantised weights (lut None with bits 4: the int4 grid, value = code - 8; lut of
    shape [1, 2^bits]: one table for the whole matrix);
    scale / offset are [N, K / group] (any4_dequant_grouped when group is not 128).
    lut / scale / offset are bf16, or all fp16 (any4_dequant_f16: groups of 128, a table)."""
    lib = load_library()
    N = codes.shape[0]
    pc = _dev(codes, torch.int32, "codes")
    dt = scale.dtype if isinstance(scale, torch.Tensor) and scale.dtype == torch.float16 else torch.bfloat16
    single = lut is not None and N != 1 and tuple(lut.shape) == (1, 1 << bits)
    _check_quant_shapes(codes, lut, scale, offset, N, K, bits, group, single_table=single)
    pl = _dev(lut, dt, "lut") if lut is not None else None
    ps = _dev(scale, dt, "scale")
    po = _dev(offset, dt, "offset")
    if out is None:
        out = torch.empty((N, K), dtype=torch.float32, device=codes.device)
    _shape(out, (N, K), "out")
    pw = _dev(out, torch.float32, "out")
    if single:
        if dt == torch.float16 or group != GROUP:
            raise Any4Error("one table for the whole matrix comes with bf16 and groups of 128")
        _check(lib.any4_dequant_single_table(pc, pl, ps, po, N, K, bits, pw, _stream()), "any4_dequant_single_table")
    elif dt == torch.float16:
        if group != GROUP:
            raise Any4Error("fp16 inputs come with groups of 128")
        _check(lib.any4_dequant_f16(pc, pl, ps, po, N, K, bits, pw, _stream()), "any4_dequant_f16")
    elif group == GROUP:
        _check(lib.any4_dequant(pc, pl, ps, po, N, K, bits, pw, _stream()), "any4_dequant")
    else:
        _check(lib.any4_dequant_grouped(pc, pl, ps, po, N, K, bits, group, pw, _stream()), "any4_dequant_grouped")
    return out


def _gemm(entry: str, x, codes, N, lut, scale, offset, bits, out, workspace, group=None):
    lib = load_library()
    M, K = x.shape
    dt = x.dtype if isinstance(x, torch.Tensor) and x.dtype == torch.float16 else torch.bfloat16
    if dt == torch.float16:
        if entry != "any4_gemm":
            raise Any4Error("fp16 inputs come with groups of 128 and the plain code layout")
        entry = "any4_gemm_f16"
    px = _dev(x, dt, "x")
    pc = _dev(codes, torch.int32, "codes")
    # a table of ONE row for a matrix of several: the single-table formats (any4_gemm_single_table)
    single = lut is not None and N != 1 and tuple(lut.shape) == (1, 1 << bits)
    if single:
        if entry != "any4_gemm":
            raise Any4Error("one table for the whole matrix comes with bf16, groups of 128 and the plain code layout")
        entry = "any4_gemm_single_table"
    _check_quant_shapes(codes, lut, scale, offset, N, K, bits, GROUP if group is None else group,
                        repacked=entry == "any4_gemm_repacked", single_table=single)
    pl = _dev(lut, dt, "lut") if lut is not None else None
    ps = _dev(scale, dt, "scale")
    po = _dev(offset, dt, "offset")
    if out is None:
        out = torch.empty((M, N), dtype=dt, device=x.device)
    _shape(out, (M, N), "out")
    py = _dev(out, dt, "out")
    need = int(lib.any4_gemm_workspace_bytes(M, N, K, bits))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    pw = workspace.data_ptr() if workspace is not None else None
    wbytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    if group is None:
        _check(getattr(lib, entry)(px, pc, pl, ps, po, M, N, K, bits, py, pw, wbytes, _stream()), entry)
    else:
        _check(getattr(lib, entry)(px, pc, pl, ps, po, M, N, K, bits, group, py, pw, wbytes, _stream()), entry)
    return out


def any4_gemm(x: torch.Tensor, codes: torch.Tensor, lut: torch.Tensor | None, scale: torch.Tensor,
              offset: torch.Tensor, bits: int = 4, out: torch.Tensor | None = None,
              workspace: torch.Tensor | None = None, group: int = GROUP) -> torch.Tensor:
    """bf16 [M,N] = x[M,K] . dequant(codes, lut, scale, offset)[N,K]^T
    (lut None with bits 4: the int4 grid, value = code - 8, run without a table; lut of shape
    [1, 2^bits]: one table for the whole matrix, any4_gemm_single_table);
    scale / offset are [N, K / group] (any4_gemm_grouped when group is not 128).
    With x, lut, scale, offset all fp16 the result is fp16 (any4_gemm_f16: groups of 128, a table)."""
    if group == GROUP:
        return _gemm("any4_gemm", x, codes, codes.shape[0], lut, scale, offset, bits, out, workspace)
    return _gemm("any4_gemm_grouped", x, codes, codes.shape[0], lut, scale, offset, bits, out, workspace, group)


NOALLOC_SCRATCH_BYTES = 48 << 20


def any4_gemm_noalloc(x: torch.Tensor, codes: torch.Tensor, lut: torch.Tensor | None, scale: torch.Tensor,
                      offset: torch.Tensor, bits: int = 4, out: torch.Tensor | None = None) -> torch.Tensor:
    """any4_gemm without a workspace: the library's own fixed scratch array serves (see include/any4.h;
    calls on one GPU must not overlap in time).  `out` should be passed by callers that must not allocate."""
    lib = load_library()
    M, K = x.shape
    N = codes.shape[0]
    px = _dev(x, torch.bfloat16, "x")
    pc = _dev(codes, torch.int32, "codes")
    _check_quant_shapes(codes, lut, scale, offset, N, K, bits, GROUP)
    pl = _dev(lut, torch.bfloat16, "lut") if lut is not None else None
    ps = _dev(scale, torch.bfloat16, "scale")
    po = _dev(offset, torch.bfloat16, "offset")
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    _shape(out, (M, N), "out")
    py = _dev(out, torch.bfloat16, "out")
    _check(lib.any4_gemm_noalloc(px, pc, pl, ps, po, M, N, K, bits, py, _stream()), "any4_gemm_noalloc")
    return out


def any4_repack_bytes(N: int, K: int, bits: int = 4) -> int:
    return int(load_library().any4_repack_bytes(N, K, bits))


def any4_repack(codes: torch.Tensor, bits: int = 4) -> torch.Tensor:
    """int32 [N, K*bits/32] packed codes -> the tile-major layout any4_gemm_repacked reads
    (int32, flat, any4_repack_bytes(N, K, bits) bytes)."""
    lib = load_library()
    N, W = codes.shape
    K = W * 32 // bits
    pc = _dev(codes, torch.int32, "codes")
    nbytes = int(lib.any4_repack_bytes(N, K, bits))
    if nbytes == 0:
        raise Any4Error("any4_repack: bad shape or bits")
    out = torch.empty(nbytes // 4, dtype=torch.int32, device=codes.device)
    _check(lib.any4_repack(pc, N, K, bits, out.data_ptr(), _stream()), "any4_repack")
    return out


def any4_gemm_repacked(x: torch.Tensor, rcodes: torch.Tensor, lut: torch.Tensor, scale: torch.Tensor,
                       offset: torch.Tensor, bits: int = 4, out: torch.Tensor | None = None,
                       workspace: torch.Tensor | None = None) -> torch.Tensor:
    """any4_gemm on codes re-arranged by any4_repack; N is taken from scale."""
    return _gemm("any4_gemm_repacked", x, rcodes, scale.shape[0], lut, scale, offset, bits, out, workspace)


def any4_quantize_max_k() -> int:
    return int(load_library().any4_quantize_max_k())


def any4_quantize(w: torch.Tensor, act: torch.Tensor | None, u: torch.Tensor, bits: int = 4,
                  symmetric: bool = False, iters: int = 20, centre_gap: float | None = None):
    """fp32 [N,K] weights, fp32 [K] mean |activation| per channel (or None), fp32 [N, 2^bits]
    uniform draws -> dict with codes_u8 uint8 [N,K], lut bf16 [N,2^bits], scale / offset bf16
    [N,K/128] and msteps int32 [N].  Everything stays in device memory.  centre_gap: None calls
    any4_quantize, a number calls any4_quantize_with_gap."""
    lib = load_library()
    N, K = w.shape
    L = 1 << bits
    pw = _dev(w, torch.float32, "w")
    pa = _dev(act, torch.float32, "act") if act is not None else None
    if tuple(u.shape) != (N, L):
        raise Any4Error(f"u must have shape ({N}, {L})")
    pu = _dev(u, torch.float32, "u")
    dev = w.device
    codes = torch.empty((N, K), dtype=torch.uint8, device=dev)
    lut = torch.empty((N, L), dtype=torch.bfloat16, device=dev)
    scale = torch.empty((N, max(K // GROUP, 0)), dtype=torch.bfloat16, device=dev)
    offset = torch.empty((N, max(K // GROUP, 0)), dtype=torch.bfloat16, device=dev)
    msteps = torch.empty((N,), dtype=torch.int32, device=dev)
    if centre_gap is None:
        _check(lib.any4_quantize(pw, pa, pu, N, K, bits, int(symmetric), iters, codes.data_ptr(), lut.data_ptr(),
                                 scale.data_ptr(), offset.data_ptr(), msteps.data_ptr(), _stream()), "any4_quantize")
    else:
        _check(lib.any4_quantize_with_gap(pw, pa, pu, N, K, bits, int(symmetric), iters, float(centre_gap),
                                          codes.data_ptr(), lut.data_ptr(), scale.data_ptr(), offset.data_ptr(),
                                          msteps.data_ptr(), _stream()), "any4_quantize_with_gap")
    return {"codes_u8": codes, "lut": lut, "scale": scale, "offset": offset, "msteps": msteps}
