"""The kernel for one to four rows of x that walks the whole K axis inside one block (packed
activation operands, no K slabs): every shape class it distinguishes, against the oracle.
K = 128 * G with G a multiple of 8 and K >= 8192 goes to it: 2 .. 8 units per wavefront (odd and even:
the ring of code registers then does / does not depend on the tile's parity), wavefronts with fewer
groups than the others or none, one tile, fewer tiles than blocks, a few more tiles than blocks,
ragged last tile, all three code widths, both code layouts.  Bar as in test_gpu_parity.py."""
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


def run(any4, oracle, M, N, K, bits, seed):
    cs = inputs.make_case(M, N, K, bits, seed)
    # offsets of the size of the scaled table values and activations with a mean: the offset term counts
    rng = np.random.default_rng(seed + 5)
    cs.offset = inputs.f32_to_bf16_bits(rng.standard_normal(cs.offset.shape, dtype=np.float32) * np.float32(0.0125))
    cs.x = inputs.f32_to_bf16_bits(rng.standard_normal(cs.x.shape, dtype=np.float32) + np.float32(0.5))
    packed = oracle.pack(cs.codes_u8, bits)
    y64 = oracle.gemm(cs.x, packed, cs.lut, cs.scale, cs.offset, K, bits, threads=16)
    codes = torch.from_numpy(packed.view(np.int32)).cuda()
    args = (dev_bf16(cs.lut), dev_bf16(cs.scale), dev_bf16(cs.offset), bits)
    y = any4.any4_gemm(dev_bf16(cs.x), codes, *args)
    y_re = any4.any4_gemm_repacked(dev_bf16(cs.x), any4.any4_repack(codes, bits), *args)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y_re.view(torch.int16)), "re-laid-out codes"
    got = y.float().cpu().numpy().astype(np.float64)
    tol = 1e-2 * oracle.rms(y64) + np.abs(y64) * 2.0 ** -8
    err = np.abs(got - y64)
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    assert np.all(err <= tol), ((M, N, K, bits), "worst", worst, float(err[worst]), float(tol[worst]))


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("G", (64, 72, 96, 104, 112, 128, 160, 200, 224, 256))
def test_one_row_every_unit_count(any4, oracle, bits, G):
    """M = 1: 2 .. 8 units per wavefront; G = 72, 104, 112, 200: the last wavefronts own fewer groups or none"""
    run(any4, oracle, 1, 333, 128 * G, bits, seed=inputs.case_seed(71, bits, G % 10))


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("M,G", [(2, 64), (2, 72), (2, 96), (2, 112), (2, 128), (3, 64), (4, 64), (4, 40), (3, 48), (2, 40)])
def test_two_to_four_rows(any4, oracle, bits, M, G):
    """operand rows shared by 8 (M = 2) or 4 (M = 3, 4) groups"""
    run(any4, oracle, M, 200, 128 * G, bits, seed=inputs.case_seed(72, bits, M + G % 7))


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("M,N,G", [(1, 1, 64), (1, 15, 64), (2, 16, 64), (1, 17, 112), (4, 31, 64), (1, 4100, 64),
                                   (2, 8200, 64), (1, 8209, 72), (1, 9000, 112), (3, 12345, 64)])
def test_tile_counts(any4, oracle, bits, M, N, G):
    """one tile, a ragged only tile, fewer tiles than blocks, one or two tiles a block, three and more
    (the ring of small inputs goes round), a ragged last tile at the end of a long range"""
    run(any4, oracle, M, N, 128 * G, bits, seed=inputs.case_seed(73, bits, (M + N + G) % 10))
