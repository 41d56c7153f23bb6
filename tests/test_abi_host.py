"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "any4.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2507_04610_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2507_04610_amd import build
        build.build_library(verbose=False)
    return binding.load_library()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(any4_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"any4_pack", "any4_dequant", "any4_gemm", "any4_gemm_workspace_bytes",
            "any4_strerror", "any4_version"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_binding_lists_the_same_entry_points():
    from paper_2507_04610_amd import binding
    assert sorted(binding.EXPORTS) == declared_symbols()


def test_version_and_error_strings(lib):
    assert lib.any4_version() >= 100
    seen = set()
    for code in range(0, -7, -1):
        s = lib.any4_strerror(code).decode()
        assert s and s not in seen
        seen.add(s)
    assert b"unknown" in lib.any4_strerror(-99)


def test_bad_arguments_are_rejected_before_any_launch(lib):
    A = 0x1000          # fake, 16-byte aligned, never dereferenced: validation fails first
    # NULL pointers
    assert lib.any4_pack(None, 4, 128, 4, A, None) == -1
    assert lib.any4_dequant(A, A, None, A, 4, 128, 4, A, None) == -1
    # a NULL table selects the 4-bit integer grid and is an error for any other width
    assert lib.any4_dequant(A, None, A, A, 4, 128, 3, A, None) == -1
    assert lib.any4_gemm(A, A, None, A, A, 1, 4, 128, 2, A, None, 0, None) == -1
    assert lib.any4_gemm(A, A, A, A, A, 1, 4, 128, 4, None, None, 0, None) == -1
    assert lib.any4_repack(None, 4, 128, 4, A, None) == -1
    assert lib.any4_gemm_repacked(A, A, None, A, A, 1, 4, 128, 4, A, None, 0, None) == -1     # needs a table
    assert lib.any4_gemm_single_table(A, A, None, A, A, 1, 4, 128, 4, A, None, 0, None) == -1 # needs its one table
    assert lib.any4_dequant_single_table(A, None, A, A, 4, 128, 4, A, None) == -1
    # shapes
    assert lib.any4_repack(A, 4, 100, 4, A, None) == -2
    assert lib.any4_repack(A, 4, 128, 5, A, None) == -3
    assert lib.any4_repack(A, 4, 128, 4, A + 4, None) == -4
    assert lib.any4_pack(A, 0, 128, 4, A, None) == -2
    assert lib.any4_pack(A, 4, 100, 4, A, None) == -2
    assert lib.any4_dequant(A, A, A, A, 4, 0, 4, A, None) == -2
    assert lib.any4_gemm(A, A, A, A, A, 0, 4, 128, 4, A, None, 0, None) == -2
    assert lib.any4_gemm(A, A, A, A, A, 1, 4, 192, 4, A, None, 0, None) == -2
    # group sizes: 64, 128, 256, 512, 1024 and a divisor of K
    for group in (32, 96, 192, 2048, 0):
        assert lib.any4_gemm_grouped(A, A, A, A, A, 1, 4, 2048, 4, group, A, None, 0, None) == -2
        assert lib.any4_dequant_grouped(A, A, A, A, 4, 2048, 4, group, A, None) == -2
    assert lib.any4_gemm_grouped(A, A, A, A, A, 1, 4, 640, 4, 256, A, None, 0, None) == -2
    # bits
    for bits in (0, 1, 5, 8, -4):
        assert lib.any4_pack(A, 4, 128, bits, A, None) == -3
        assert lib.any4_gemm(A, A, A, A, A, 1, 4, 128, bits, A, None, 0, None) == -3
    # alignment
    assert lib.any4_pack(A + 4, 4, 128, 4, A, None) == -4
    assert lib.any4_dequant(A, A + 2, A, A, 4, 128, 4, A, None) == -4
    assert lib.any4_gemm(A, A, A, A, A, 1, 4, 128, 4, A + 8, None, 0, None) == -4


def test_noalloc_entry_point_checks_arguments_and_its_limit(lib):
    """any4_gemm_noalloc: the same refusals as any4_gemm, plus ANY4_ERR_WORKSPACE for a problem whose
    scratch exceeds the library's fixed array - all before anything touches the device"""
    from paper_2507_04610_amd import binding
    A = 0x1000
    assert lib.any4_gemm_noalloc(A, A, A, A, A, 0, 4, 128, 4, A, None) == -2
    assert lib.any4_gemm_noalloc(A, A, A, A, A, 1, 4, 192, 4, A, None) == -2
    assert lib.any4_gemm_noalloc(A, A, A, A, A, 1, 4, 128, 5, A, None) == -3
    assert lib.any4_gemm_noalloc(None, A, A, A, A, 1, 4, 128, 4, A, None) == -1
    assert lib.any4_gemm_noalloc(A, A, None, A, A, 1, 4, 128, 3, A, None) == -1
    assert lib.any4_gemm_noalloc(A, A, A, A, A + 2, 1, 4, 128, 4, A, None) == -4
    M, N, K = 16, 500000, 8192
    assert lib.any4_gemm_workspace_bytes(M, N, K, 4) > binding.NOALLOC_SCRATCH_BYTES
    assert lib.any4_gemm_noalloc(A, A, A, A, A, M, N, K, 4, A, None) == -5
    header = open(HEADER).read()
    assert re.search(r"#define ANY4_NOALLOC_SCRATCH_BYTES \((\d+)u << 20\)", header)
    assert int(re.search(r"#define ANY4_NOALLOC_SCRATCH_BYTES \((\d+)u << 20\)", header).group(1)) << 20 == binding.NOALLOC_SCRATCH_BYTES


def test_quantiser_entry_points_check_arguments(lib):
    A = 0x1000
    kmax = lib.any4_quantize_max_k()
    assert kmax >= 14336 and kmax % 128 == 0
    gap = lib.any4_quantize_with_gap
    assert lib.any4_quantize(None, None, A, 1, 128, 4, 0, 1, A, A, A, A, None, None) == -1
    assert lib.any4_quantize(A, None, A, 1, 128, 4, 0, 1, A, None, A, A, None, None) == -1
    assert lib.any4_quantize(A, None, A, 1, 100, 4, 0, 1, A, A, A, A, None, None) == -2
    assert lib.any4_quantize(A, None, A, 1, kmax + 128, 4, 0, 1, A, A, A, A, None, None) == -2
    assert lib.any4_quantize(A, None, A, 1, 128, 4, 0, -1, A, A, A, A, None, None) == -2
    assert lib.any4_quantize(A, None, A, 1, 128, 5, 0, 1, A, A, A, A, None, None) == -3
    assert lib.any4_quantize(A, A + 4, A, 1, 128, 4, 0, 1, A, A, A, A, None, None) == -4
    assert gap(A, None, A, 1, 128, 4, 0, 1, float("nan"), A, A, A, A, None, None) == -2
    assert gap(None, None, A, 1, 128, 4, 0, 1, 0.0, A, A, A, A, None, None) == -1
    assert gap(A, None, A, 1, 128, 4, 0, 1, -1.0, A + 8, A, A, A, None, None) == -4


def test_repack_size(lib):
    # whole tiles of 16 rows; invalid arguments need nothing
    assert lib.any4_repack_bytes(16, 128, 4) == 16 * 64
    assert lib.any4_repack_bytes(17, 256, 3) == 32 * 96
    assert lib.any4_repack_bytes(1, 128, 2) == 16 * 32
    assert lib.any4_repack_bytes(4, 100, 4) == 0 and lib.any4_repack_bytes(4, 128, 7) == 0


def test_workspace_contract(lib):
    # invalid problems need no workspace
    assert lib.any4_gemm_workspace_bytes(1, 4, 100, 4) == 0
    assert lib.any4_gemm_workspace_bytes(0, 4, 128, 4) == 0
    assert lib.any4_gemm_workspace_bytes(1, 4, 128, 7) == 0
    # a short row-count with a long K is split along K and needs fp32 partials of >= 2 slices
    M, N, K = 4, 64, 16384
    need = lib.any4_gemm_workspace_bytes(M, N, K, 4)
    assert need >= 2 * M * N * 4 and need % 16 == 0
    A = 0x1000
    assert lib.any4_gemm(A, A, A, A, A, M, N, K, 4, A, None, 0, None) == -5
    assert lib.any4_gemm(A, A, A, A, A, M, N, K, 4, A, A, need - 1, None) == -5
    # the matrix-core path keeps per-group sums of x: far smaller than x itself
    assert 0 < lib.any4_gemm_workspace_bytes(2048, 4096, 4096, 4) <= 2048 * 4096 * 2 // 32
