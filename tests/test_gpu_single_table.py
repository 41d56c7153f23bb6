"""Formats with ONE table for the whole matrix (the paper's nf4 / af4 comparisons: section 2.4.1, last
paragraph; section 5, "Speed Comparisons"): any4_gemm_single_table / any4_dequant_single_table against the
oracle run on the table written out N times, and bit for bit against the per-row entry points fed
the same N repeated rows.  Every kernel that can serve the call: the streaming kernel (K = 4096 and
K slabs), the whole-K kernel for M <= 4, 16 rows a launch, the matrix-core kernel (whole tiles and K
slices), the wavefront-per-row kernel for very long K."""
import numpy as np
import pytest

from paper_2507_04610_amd import inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def any4():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the parity tests must run on the GPU box")
    import paper_2507_04610_amd as lib
    lib.load_library()
    return lib


def dev_bf16(a_u16):
    return torch.from_numpy(np.ascontiguousarray(a_u16).view(np.int16)).cuda().view(torch.bfloat16)


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("M,N,K", [(1, 333, 4096), (1, 64, 128), (3, 17, 384), (8, 700, 640), (16, 100, 4480),
                                   (1, 200, 8192), (2, 333, 14336), (4, 100, 8192), (1, 115, 28672), (5, 48, 14336),
                                   (37, 100, 4096), (300, 384, 4096), (129, 130, 640), (2048, 200, 1024),
                                   (2, 5, 262272)])
def test_gemm_single_table(any4, oracle, bits, M, N, K):
    cs = inputs.make_case(M, N, K, bits, seed=inputs.case_seed(96, bits, (M + N) % 10))
    one = cs.lut[N // 2:N // 2 + 1].copy()                   # any row of the generated tables
    repeated = np.ascontiguousarray(np.repeat(one, N, axis=0))
    packed = oracle.pack(cs.codes_u8, bits)
    y64 = oracle.gemm(cs.x, packed, repeated, cs.scale, cs.offset, K, bits, threads=16)
    codes = torch.from_numpy(packed.view(np.int32)).cuda()
    x, sc, of = dev_bf16(cs.x), dev_bf16(cs.scale), dev_bf16(cs.offset)
    y = any4.any4_gemm(x, codes, dev_bf16(one), sc, of, bits)                 # [1, 2^bits]: the single-table entry point
    y_rows = any4.any4_gemm(x, codes, dev_bf16(repeated), sc, of, bits)        # [N, 2^bits]: a table per row
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y_rows.view(torch.int16)), "differs from the per-row path on repeated rows"
    got = y.float().cpu().numpy().astype(np.float64)
    tol = 1e-2 * oracle.rms(y64) + np.abs(y64) * 2.0 ** -8
    err = np.abs(got - y64)
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    assert np.all(err <= tol), ((M, N, K, bits), worst, float(err[worst]), float(tol[worst]))


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("N,K", [(5, 384), (257, 1152), (33, 14336)])
def test_dequant_single_table_bit_exact(any4, oracle, bits, N, K):
    cs = inputs.make_case(1, N, K, bits, seed=inputs.case_seed(97, bits, N % 7))
    one = cs.lut[:1].copy()
    packed = oracle.pack(cs.codes_u8, bits)
    w_ref = oracle.dequant(packed, np.ascontiguousarray(np.repeat(one, N, axis=0)), cs.scale, cs.offset, K, bits)
    w = any4.any4_dequant(torch.from_numpy(packed.view(np.int32)).cuda(), dev_bf16(one), dev_bf16(cs.scale),
                          dev_bf16(cs.offset), K, bits)
    torch.cuda.synchronize()
    assert np.array_equal(w.cpu().numpy().view(np.uint32), w_ref.view(np.uint32))


def test_single_table_needs_bf16_groups_of_128_and_the_plain_layout(any4):
    cs = inputs.make_case(1, 32, 1024, 4, 3)
    codes = any4.any4_pack(torch.from_numpy(cs.codes_u8).cuda(), 4)
    one = dev_bf16(cs.lut[:1])
    with pytest.raises(any4.Any4Error):
        any4.any4_gemm(dev_bf16(cs.x), codes, one, dev_bf16(cs.scale[:, ::2]), dev_bf16(cs.offset[:, ::2]), 4, group=256)
    with pytest.raises(any4.Any4Error):
        any4.any4_gemm_repacked(dev_bf16(cs.x), any4.any4_repack(codes, 4), one, dev_bf16(cs.scale), dev_bf16(cs.offset), 4)
