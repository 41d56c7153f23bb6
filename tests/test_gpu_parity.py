"""Parity of the HIP path against the CPU oracle, through the C ABI, on a real MI355X.

Bars: packed words and dequantised fp32 weights bit-exact; GEMM outputs within
1e-2 * rms(y_fp64) + 2^-8 * |y_fp64| (half a bf16 ulp of output rounding) elementwise.
Small shapes are compared element by element, and so are the full benchmark shapes for M <= 16
(all M x N outputs); at M = 2048 one output column of every 128-wide block plus the first and last
block are compared over all rows of x, with rms taken over the compared block.
"""
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
    lib.load_library()                      # raises if libany4.so is missing
    return lib


def dev_bf16(a_u16):
    return torch.from_numpy(np.ascontiguousarray(a_u16).view(np.int16)).cuda().view(torch.bfloat16)


def dev_codes(packed_u32):
    return torch.from_numpy(np.ascontiguousarray(packed_u32).view(np.int32)).cuda()


def host_u32(t):
    return t.cpu().numpy().view(np.uint32)


def host_bf16_as_f64(t):
    return inputs.bf16_bits_to_f32(t.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)


def check_gemm(y_dev, y64, rms, what):
    y = host_bf16_as_f64(y_dev)
    tol = 1e-2 * rms + np.abs(y64) * 2.0 ** -8
    err = np.abs(y - y64)
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    assert np.all(err <= tol), (what, "worst", worst, float(err[worst]), float(tol[worst]), "rms", rms)
    return float((err / (1e-2 * rms)).max())


# ------------------------------------------------------------------------------ pack
@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("N,K", [(1, 128), (5, 384), (257, 1152), (64, 4096)])
def test_pack_bit_exact(any4, oracle, bits, N, K):
    rng = np.random.default_rng(100 + bits + N)
    codes = rng.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
    got = host_u32(any4.any4_pack(torch.from_numpy(codes).cuda(), bits))
    assert np.array_equal(got, oracle.pack(codes, bits))


def test_pack_masks_high_bits(any4, oracle):
    rng = np.random.default_rng(5)
    codes = rng.integers(0, 256, size=(3, 256), dtype=np.uint8)
    for bits in (4, 3, 2):
        got = host_u32(any4.any4_pack(torch.from_numpy(codes).cuda(), bits))
        assert np.array_equal(got, oracle.pack(codes & ((1 << bits) - 1), bits))


# ------------------------------------------------------------------------------ dequant
@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("N,K", [(1, 128), (3, 384), (130, 640), (257, 4224), (16, 14336)])
def test_dequant_bit_exact(any4, oracle, bits, N, K):
    cs = inputs.make_case(1, N, K, bits, seed=inputs.case_seed(2, N % 7, bits))
    packed = oracle.pack(cs.codes_u8, bits)
    w_ref = oracle.dequant(packed, cs.lut, cs.scale, cs.offset, K, bits)
    w = any4.any4_dequant(dev_codes(packed), dev_bf16(cs.lut), dev_bf16(cs.scale), dev_bf16(cs.offset), K, bits)
    assert np.array_equal(w.cpu().numpy().view(np.uint32), w_ref.view(np.uint32))


def test_dequant_special_values(any4, oracle):
    """Unsorted table with +-0, sub-normal, tiny and huge entries; zero offsets in half the rows."""
    N, K, bits = 8, 512, 4
    cs = inputs.make_case(1, N, K, bits, seed=9)
    specials = np.array([0x0000, 0x8000, 0x0001, 0x8001, 0x007F, 0x0080, 0x7F7F, 0xFF7F,
                         0x3F80, 0xBF80, 0x0100, 0x4000, 0x3400, 0xB400, 0x2000, 0x5000], np.uint16)
    lut = np.stack([np.roll(specials, n) for n in range(N)])
    offset = cs.offset.copy()
    offset[::2] = 0
    packed = oracle.pack(cs.codes_u8, bits)
    w_ref = oracle.dequant(packed, lut, cs.scale, offset, K, bits)
    w = any4.any4_dequant(dev_codes(packed), dev_bf16(lut), dev_bf16(cs.scale), dev_bf16(offset), K, bits)
    assert np.array_equal(w.cpu().numpy().view(np.uint32), w_ref.view(np.uint32))


# ------------------------------------------------------------------------------ gemm, element by element
def run_gemm_case(any4, oracle, M, N, K, bits, seed, mutate=None):
    cs = inputs.make_case(M, N, K, bits, seed)
    if mutate:
        mutate(cs)
    packed = oracle.pack(cs.codes_u8, bits)
    y64 = oracle.gemm(cs.x, packed, cs.lut, cs.scale, cs.offset, K, bits, threads=8)
    codes_dev = any4.any4_pack(torch.from_numpy(cs.codes_u8).cuda(), bits)
    assert np.array_equal(host_u32(codes_dev), packed)
    y = any4.any4_gemm(dev_bf16(cs.x), codes_dev, dev_bf16(cs.lut), dev_bf16(cs.scale), dev_bf16(cs.offset), bits)
    torch.cuda.synchronize()
    assert y.shape == (M, N) and y.dtype == torch.bfloat16
    return check_gemm(y, y64, oracle.rms(y64), (M, N, K, bits))


def test_gemm_config1(any4, oracle):
    """M=1, N=256, K=512, seed 0."""
    run_gemm_case(any4, oracle, 1, 256, 512, 4, seed=0)


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("M", (1, 2, 3, 5, 8, 13, 16))
def test_gemm_decode_small(any4, oracle, bits, M):
    # ragged N (not a multiple of any tile), K spanning several steps with a short tail
    run_gemm_case(any4, oracle, M, 333, 4224, bits, seed=inputs.case_seed(3, bits, M))


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("M,N,K", [(1, 1, 128), (4, 7, 128), (16, 64, 16384), (2, 40, 28672), (1, 2049, 256)])
def test_gemm_decode_edges(any4, oracle, bits, M, N, K):
    run_gemm_case(any4, oracle, M, N, K, bits, seed=inputs.case_seed(4, bits, M))


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("M,N,K", [(17, 128, 128), (100, 200, 256), (256, 384, 1024), (129, 130, 640), (300, 64, 2048)])
def test_gemm_prefill_small(any4, oracle, bits, M, N, K):
    run_gemm_case(any4, oracle, M, N, K, bits, seed=inputs.case_seed(5, bits, M % 10))


@pytest.mark.parametrize("bits", (4, 3, 2))
def test_gemm_decode_very_long_k(any4, oracle, bits):
    """K so long that the streaming kernel's slab count exceeds its limit: the wavefront-per-row
    kernel with a second-stage reduction takes over."""
    run_gemm_case(any4, oracle, 2, 5, 262272, bits, seed=inputs.case_seed(6, bits))


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("M,N,K", [(1, 16, 128), (3, 17, 384), (16, 100, 4480), (7, 4100, 512), (5, 48, 14336),
                                   (16, 33, 8192), (2, 700, 640)])
def test_gemm_decode_slabs_and_ragged_groups(any4, oracle, bits, M, N, K):
    """Streaming kernel: group counts that are / are not multiples of 4 (shared small inputs on and
    off), wavefronts without groups, several slabs, ragged last tile, more tiles than blocks."""
    run_gemm_case(any4, oracle, M, N, K, bits, seed=inputs.case_seed(7, bits, M))


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("M,N,K", [(1, 40, 8192), (2, 100, 14336), (1, 115, 28672), (2, 5000, 8192),
                                   (1, 16, 5120), (2, 33, 28672), (1, 48, 12288)])
def test_gemm_decode_long_k_few_rows(any4, oracle, bits, M, N, K):
    """One or two activation rows (fetched once per wavefront and re-distributed through LDS) and K
    beyond one slab: 2 to 7 slabs combined through the workspace, several tiles per block, ragged
    last tile."""
    run_gemm_case(any4, oracle, M, N, K, bits, seed=inputs.case_seed(9, bits, M))


def test_gemm_zero_offset_and_unsorted_table(any4, oracle):
    def mutate(cs):
        cs.offset[:] = 0                                   # symmetric scaling: beta = 0
        rng = np.random.default_rng(1)
        for n in range(cs.N):
            cs.lut[n] = cs.lut[n][rng.permutation(cs.lut.shape[1])]
    for M in (1, 16, 64):
        run_gemm_case(any4, oracle, M, 192, 1024, 4, seed=77, mutate=mutate)


@pytest.mark.parametrize("M", (1, 16, 64))
def test_gemm_other_4bit_formats_through_the_table(any4, oracle, M):
    """The paper's other 4-bit formats are tables too (section 4.2, last paragraph): one table shared
    by all rows (nf4-style) and the uniform integer grid -8 .. 7 (int4) run through the same path."""
    def shared_table(cs):
        cs.lut[:] = cs.lut[0]
    def int4_grid(cs):
        cs.lut[:] = inputs.f32_to_bf16_bits(np.arange(-8, 8, dtype=np.float32))
    for mutate in (shared_table, int4_grid):
        run_gemm_case(any4, oracle, M, 200, 2048, 4, seed=31, mutate=mutate)


@pytest.mark.parametrize("M,N,K", [(1, 333, 4224), (1, 64, 128), (3, 17, 384), (8, 700, 640), (16, 100, 4480),
                                   (2, 48, 14336), (16, 33, 8192), (40, 200, 1024), (300, 130, 640),
                                   (129, 260, 4224), (600, 140, 8192), (257, 1100, 384)])
def test_gemm_int4_grid_without_table(any4, oracle, M, N, K):
    """lut = NULL with 4-bit codes: the uniform integer grid (value = code - 8).  The oracle runs the
    same problem with that grid written out as every row's table; the device runs it table-free at
    every M (codes OR-ed into the mantissa of 128.0, the surplus taken off through the group sums of x),
    and the dequantised weights agree bit for bit."""
    cs = inputs.make_case(M, N, K, 4, seed=inputs.case_seed(11, 4, M % 10))
    cs.lut[:] = inputs.f32_to_bf16_bits(np.arange(-8, 8, dtype=np.float32))
    packed = oracle.pack(cs.codes_u8, 4)
    y64 = oracle.gemm(cs.x, packed, cs.lut, cs.scale, cs.offset, K, 4, threads=8)
    codes_dev = any4.any4_pack(torch.from_numpy(cs.codes_u8).cuda(), 4)
    y = any4.any4_gemm(dev_bf16(cs.x), codes_dev, None, dev_bf16(cs.scale), dev_bf16(cs.offset), 4)
    torch.cuda.synchronize()
    check_gemm(y, y64, oracle.rms(y64), ("int4", M, N, K))
    w = any4.any4_dequant(codes_dev, None, dev_bf16(cs.scale), dev_bf16(cs.offset), K, 4)
    assert np.array_equal(host_u32(w), oracle.dequant(packed, cs.lut, cs.scale, cs.offset, K, 4).view(np.uint32))


def test_no_table_needs_four_bits(any4):
    from paper_2507_04610_amd import binding
    cs = inputs.make_case(1, 16, 128, 3, seed=1)
    codes_dev = any4.any4_pack(torch.from_numpy(cs.codes_u8).cuda(), 3)
    with pytest.raises(binding.Any4Error):
        any4.any4_gemm(dev_bf16(cs.x), codes_dev, None, dev_bf16(cs.scale), dev_bf16(cs.offset), 3)


def test_gemm_is_reproducible(any4, oracle):
    cs = inputs.make_case(4, 64, 16384, 4, seed=12)
    codes = any4.any4_pack(torch.from_numpy(cs.codes_u8).cuda(), 4)
    args = (dev_bf16(cs.x), codes, dev_bf16(cs.lut), dev_bf16(cs.scale), dev_bf16(cs.offset), 4)
    assert any4.any4_gemm_workspace_bytes(4, 64, 16384, 4) > 0     # the split-K route
    a = any4.any4_gemm(*args).view(torch.int16).cpu()
    for _ in range(3):
        assert torch.equal(a, any4.any4_gemm(*args).view(torch.int16).cpu())


def test_gemm_with_k_slices_on_the_matrix_cores_is_reproducible_and_graph_safe(any4, oracle):
    """A problem of few tiles: the matrix-core kernel cuts them along K and the last slice to arrive
    adds the partial sums in slice order, so the result does not depend on which block was last; the
    arrival counters are left clean, so the same workspace serves replays of a captured launch."""
    M, N, K = 300, 384, 4096
    cs = inputs.make_case(M, N, K, 4, seed=21)
    packed = oracle.pack(cs.codes_u8, 4)
    codes = dev_codes(packed)
    x, lut, sc, of = dev_bf16(cs.x), dev_bf16(cs.lut), dev_bf16(cs.scale), dev_bf16(cs.offset)
    need = any4.any4_gemm_workspace_bytes(M, N, K, 4)
    assert need > 6 * 256 * 128 * 4                                  # partial tiles of several slices
    ws = torch.empty(need, dtype=torch.uint8, device="cuda").fill_(0xA5)       # no initialisation expected
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    a = any4.any4_gemm(x, codes, lut, sc, of, 4, out=y, workspace=ws).view(torch.int16).cpu().clone()
    y64 = oracle.gemm(cs.x, packed, cs.lut, cs.scale, cs.offset, K, 4, threads=8)
    check_gemm(y, y64, oracle.rms(y64), ("k slices", M, N, K))
    for _ in range(3):
        y.zero_()
        any4.any4_gemm(x, codes, lut, sc, of, 4, out=y, workspace=ws)
        assert torch.equal(a, y.view(torch.int16).cpu())
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        any4.any4_gemm(x, codes, lut, sc, of, 4, out=y, workspace=ws)          # warm-up on the capture stream
        with torch.cuda.graph(g, stream=side):
            any4.any4_gemm(x, codes, lut, sc, of, 4, out=y, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(3):
        y.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(a, y.view(torch.int16).cpu())


def test_gemm_rejects_small_workspace_and_leaves_output_alone(any4):
    cs = inputs.make_case(4, 64, 16384, 4, seed=12)
    codes = any4.any4_pack(torch.from_numpy(cs.codes_u8).cuda(), 4)
    y = torch.full((4, 64), 7.0, dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(any4.Any4Error):
        any4.any4_gemm(dev_bf16(cs.x), codes, dev_bf16(cs.lut), dev_bf16(cs.scale), dev_bf16(cs.offset), 4,
                       out=y, workspace=ws)
    torch.cuda.synchronize()
    assert torch.all(y == 7.0)


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("M,N,K", [(17, 64, 4096), (32, 256, 4096), (37, 100, 14336), (64, 512, 2048),
                                   (128, 96, 8192)])
def test_gemm_few_dozen_rows(any4, oracle, bits, M, N, K):
    """M just above 16: served by the streaming kernel, 16 rows of x per launch (ragged last launch,
    K slabs that share one workspace from launch to launch), or by the matrix-core kernel - whichever
    the library picks, the result must be the same GEMM."""
    run_gemm_case(any4, oracle, M, N, K, bits, seed=inputs.case_seed(6, bits, M))


# ------------------------------------------------------------------------------ other group sizes
def coarse(cs, group):
    """one scale / offset per `group` weights, taken from the generated 128-wide ones"""
    r = group // 128
    return np.ascontiguousarray(cs.scale[:, ::r]), np.ascontiguousarray(cs.offset[:, ::r])


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("group", (256, 512, 1024))
@pytest.mark.parametrize("N,K", [(5, 1024), (130, 2048), (17, 14336)])
def test_dequant_grouped_bit_exact(any4, oracle, bits, group, N, K):
    if K % group:
        pytest.skip("the group must divide K")
    cs = inputs.make_case(1, N, K, bits, seed=inputs.case_seed(7, bits, group))
    sc, of = coarse(cs, group)
    packed = oracle.pack(cs.codes_u8, bits)
    w_ref = oracle.dequant(packed, cs.lut, sc, of, K, bits, group=group)
    w = any4.any4_dequant(dev_codes(packed), dev_bf16(cs.lut), dev_bf16(sc), dev_bf16(of), K, bits, group=group)
    torch.cuda.synchronize()
    assert np.array_equal(w.cpu().numpy().view(np.uint32), w_ref.view(np.uint32))


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("group", (256, 512, 1024))
@pytest.mark.parametrize("M,N,K", [(1, 40, 1024), (5, 333, 4096), (16, 100, 2048), (2, 64, 14336), (1, 2049, 1024),
                                   (32, 256, 4096), (100, 200, 1024), (300, 130, 2048)])
def test_gemm_grouped(any4, oracle, bits, group, M, N, K):
    """Small M (streaming kernel, every wavefront reads the scales of its own chunks), a few dozen
    rows (the same kernel, 16 rows per launch) and large M (matrix cores, K slices included)."""
    if K % group:
        pytest.skip("the group must divide K")
    cs = inputs.make_case(M, N, K, bits, seed=inputs.case_seed(8, bits, group + M))
    sc, of = coarse(cs, group)
    packed = oracle.pack(cs.codes_u8, bits)
    y64 = oracle.gemm(cs.x, packed, cs.lut, sc, of, K, bits, threads=8, group=group)
    y = any4.any4_gemm(dev_bf16(cs.x), dev_codes(packed), dev_bf16(cs.lut), dev_bf16(sc), dev_bf16(of), bits, group=group)
    torch.cuda.synchronize()
    check_gemm(y, y64, oracle.rms(y64), ("group", group, M, N, K, bits))


def fine(M, N, K, bits, seed):
    """a case with scales / offsets per 64 weights: two independent draws interleaved along K, so
    that the two halves of every chunk of 128 carry unrelated values"""
    a, b = inputs.make_case(M, N, K, bits, seed), inputs.make_case(1, N, K, bits, seed + 1000)
    sc = np.ascontiguousarray(np.stack([a.scale, b.scale], axis=2).reshape(N, -1))
    of = np.ascontiguousarray(np.stack([a.offset, b.offset], axis=2).reshape(N, -1))
    return a, sc, of


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("N,K", [(5, 128), (130, 2048), (17, 14336), (33, 640)])
def test_dequant_groups_of_64_bit_exact(any4, oracle, bits, N, K):
    cs, sc, of = fine(1, N, K, bits, inputs.case_seed(17, bits, N))
    packed = oracle.pack(cs.codes_u8, bits)
    w_ref = oracle.dequant(packed, cs.lut, sc, of, K, bits, group=64)
    w = any4.any4_dequant(dev_codes(packed), dev_bf16(cs.lut), dev_bf16(sc), dev_bf16(of), K, bits, group=64)
    torch.cuda.synchronize()
    assert np.array_equal(w.cpu().numpy().view(np.uint32), w_ref.view(np.uint32))


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("M,N,K", [(1, 16, 128), (1, 40, 1024), (2, 333, 4224), (3, 17, 384), (5, 333, 4096), (8, 700, 640),
                                   (9, 100, 2048), (16, 100, 4480), (2, 64, 14336), (7, 40, 28672), (1, 2049, 1024),
                                   (17, 128, 128), (32, 256, 4096), (100, 200, 1024), (129, 130, 640), (300, 130, 2048),
                                   (260, 300, 8192)])
def test_gemm_groups_of_64(any4, oracle, bits, M, N, K):
    """Small M: the streaming kernel tells the halves of a chunk of 128 apart on the activation side,
    8 rows a launch (one launch, two, one or several K slabs, ragged N).  Larger M: the matrix-core
    kernel folds a scale in after every K step, whole tiles and K slices."""
    cs, sc, of = fine(M, N, K, bits, inputs.case_seed(18, bits, M + N))
    packed = oracle.pack(cs.codes_u8, bits)
    y64 = oracle.gemm(cs.x, packed, cs.lut, sc, of, K, bits, threads=8, group=64)
    y = any4.any4_gemm(dev_bf16(cs.x), dev_codes(packed), dev_bf16(cs.lut), dev_bf16(sc), dev_bf16(of), bits, group=64)
    torch.cuda.synchronize()
    check_gemm(y, y64, oracle.rms(y64), ("group 64", M, N, K, bits))


def test_gemm_groups_of_64_with_doubled_scales_is_the_group_128_result(any4):
    """every scale twice = groups of 128: the same sums, so the same bf16 output up to the order of
    the fp32 additions (compared within one bf16 unit, most of them equal)"""
    for M, N, K in ((4, 64, 2048), (64, 256, 1024)):
        t = inputs.make_case_device(M, N, K, 4, seed=5, device=torch.device("cuda:0"))
        codes = any4.any4_pack(t["codes_u8"], 4)
        y128 = any4.any4_gemm(t["x"], codes, t["lut"], t["scale"], t["offset"], 4)
        sc, of = t["scale"].repeat_interleave(2, dim=1).contiguous(), t["offset"].repeat_interleave(2, dim=1).contiguous()
        y64 = any4.any4_gemm(t["x"], codes, t["lut"], sc, of, 4, group=64)
        torch.cuda.synchronize()
        a, b = y128.float(), y64.float()
        assert torch.all((a - b).abs() <= 2.0 ** -7 * torch.maximum(a.abs(), b.abs()) + 1e-3)
        assert (y128.view(torch.int16) == y64.view(torch.int16)).float().mean() > 0.9


def test_groups_of_64_need_a_table_and_the_plain_layout(any4):
    cs, sc, of = fine(1, 16, 256, 4, 3)
    codes = any4.any4_pack(torch.from_numpy(cs.codes_u8).cuda(), 4)
    with pytest.raises(any4.Any4Error):
        any4.any4_gemm(dev_bf16(cs.x), codes, None, dev_bf16(sc), dev_bf16(of), 4, group=64)


def test_grouped_rejects_other_group_sizes(any4):
    cs = inputs.make_case(1, 16, 1024, 4, 3)
    codes = any4.any4_pack(torch.from_numpy(cs.codes_u8).cuda(), 4)
    for bad in (32, 96, 192, 2048, 0, -128):
        with pytest.raises(any4.Any4Error):
            any4.any4_gemm(dev_bf16(cs.x), codes, dev_bf16(cs.lut), dev_bf16(cs.scale), dev_bf16(cs.offset), 4, group=bad)
    cs = inputs.make_case(1, 16, 640, 4, 3)                 # 640 is not a multiple of 256
    codes = any4.any4_pack(torch.from_numpy(cs.codes_u8).cuda(), 4)
    with pytest.raises(any4.Any4Error):
        any4.any4_dequant(codes, dev_bf16(cs.lut), dev_bf16(cs.scale), dev_bf16(cs.offset), 640, 4, group=256)


# ------------------------------------------------------------------------------ fp16 storage
def dev_f16(a_u16):
    return torch.from_numpy(np.ascontiguousarray(a_u16).view(np.int16)).cuda().view(torch.float16)


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("N,K", [(1, 128), (130, 640), (17, 14336)])
def test_dequant_f16_bit_exact(any4, oracle, bits, N, K):
    cs = inputs.make_case(1, N, K, bits, seed=inputs.case_seed(21, bits, N % 7), f16=True)
    packed = oracle.pack(cs.codes_u8, bits)
    w_ref = oracle.dequant(packed, cs.lut, cs.scale, cs.offset, K, bits, f16=True)
    w = any4.any4_dequant(dev_codes(packed), dev_f16(cs.lut), dev_f16(cs.scale), dev_f16(cs.offset), K, bits)
    torch.cuda.synchronize()
    assert np.array_equal(w.cpu().numpy().view(np.uint32), w_ref.view(np.uint32))


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("M,N,K", [(1, 16, 128), (1, 333, 4224), (2, 40, 28672), (3, 17, 384), (5, 48, 14336), (8, 700, 640),
                                   (16, 100, 4480), (1, 2049, 256), (17, 128, 128), (40, 512, 4096), (100, 200, 256),
                                   (129, 130, 640), (300, 64, 2048), (260, 300, 8192)])
def test_gemm_f16(any4, oracle, bits, M, N, K):
    """fp16 activations, table, scales, offsets and output (the f16 matrix instructions): small M
    with one and several K slabs, shared small inputs on and off, a few dozen rows, large M with
    whole tiles and K slices.  Bar: 1e-2 * rms + half an fp16 unit of output rounding (2^-11 |y|)."""
    cs = inputs.make_case(M, N, K, bits, seed=inputs.case_seed(22, bits, M + N), f16=True)
    packed = oracle.pack(cs.codes_u8, bits)
    y64 = oracle.gemm(cs.x, packed, cs.lut, cs.scale, cs.offset, K, bits, threads=8, f16=True)
    y = any4.any4_gemm(dev_f16(cs.x), dev_codes(packed), dev_f16(cs.lut), dev_f16(cs.scale), dev_f16(cs.offset), bits)
    torch.cuda.synchronize()
    assert y.dtype == torch.float16 and y.shape == (M, N)
    got = y.cpu().numpy().astype(np.float64)
    rms = oracle.rms(y64)
    tol = 1e-2 * rms + np.abs(y64) * 2.0 ** -11
    err = np.abs(got - y64)
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    assert np.all(err <= tol), ("f16", M, N, K, bits, worst, float(err[worst]), float(tol[worst]), rms)


def test_f16_needs_a_table_groups_of_128_and_one_dtype(any4):
    cs = inputs.make_case(1, 16, 256, 4, 3, f16=True)
    codes = any4.any4_pack(torch.from_numpy(cs.codes_u8).cuda(), 4)
    x, lut, sc, of = dev_f16(cs.x), dev_f16(cs.lut), dev_f16(cs.scale), dev_f16(cs.offset)
    with pytest.raises(any4.Any4Error):
        any4.any4_gemm(x, codes, None, sc, of, 4)
    with pytest.raises(any4.Any4Error):
        any4.any4_gemm(x, codes, lut, sc[:, ::2].contiguous(), of[:, ::2].contiguous(), 4, group=256)
    with pytest.raises(any4.Any4Error):
        any4.any4_gemm(x, codes, lut.view(torch.bfloat16), sc, of, 4)             # mixed types
    with pytest.raises(any4.Any4Error):
        any4.any4_gemm_repacked(x, any4.any4_repack(codes, 4), lut, sc, of, 4)


# ------------------------------------------------------------------------------ tile-major re-layout
@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("N,K", [(16, 128), (21, 256), (1, 128), (257, 1152), (64, 4096), (5, 14336)])
def test_repack_bit_exact(any4, oracle, bits, N, K):
    codes = np.random.default_rng(N * 7 + bits).integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
    packed = oracle.pack(codes, bits)
    r = any4.any4_repack(dev_codes(packed), bits)
    torch.cuda.synchronize()
    assert r.numel() * 4 == any4.any4_repack_bytes(N, K, bits)
    assert np.array_equal(host_u32(r), oracle.repack(packed, K, bits))


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("M,N,K", [(1, 16, 128), (1, 333, 4224), (3, 17, 384), (8, 700, 640), (16, 100, 4480),
                                   (2, 40, 28672), (5, 4100, 512), (1, 2049, 256), (2, 100, 14336),
                                   (17, 128, 128), (100, 200, 256), (300, 64, 2048), (129, 130, 640)])
def test_gemm_repacked_equals_plain_layout(any4, oracle, bits, M, N, K):
    """Same kernels, same arithmetic, other addresses: the result is that of any4_gemm bit for bit,
    and within the GEMM tolerance of the oracle (which knows only the plain layout)."""
    cs = inputs.make_case(M, N, K, bits, inputs.case_seed(9, bits, M))
    packed = oracle.pack(cs.codes_u8, bits)
    y64 = oracle.gemm(cs.x, packed, cs.lut, cs.scale, cs.offset, K, bits, threads=8)
    codes_dev = dev_codes(packed)
    rcodes = any4.any4_repack(codes_dev, bits)
    args = (dev_bf16(cs.lut), dev_bf16(cs.scale), dev_bf16(cs.offset), bits)
    y_plain = any4.any4_gemm(dev_bf16(cs.x), codes_dev, *args)
    y_re = any4.any4_gemm_repacked(dev_bf16(cs.x), rcodes, *args)
    torch.cuda.synchronize()
    assert torch.equal(y_plain.view(torch.int16), y_re.view(torch.int16))
    check_gemm(y_re, y64, oracle.rms(y64), ("repacked", M, N, K, bits))


def test_gemm_repacked_needs_a_table(any4):
    cs = inputs.make_case(1, 16, 128, 4, 3)
    rcodes = any4.any4_repack(any4.any4_pack(torch.from_numpy(cs.codes_u8).cuda(), 4), 4)
    with pytest.raises(any4.Any4Error):
        any4.any4_gemm_repacked(dev_bf16(cs.x), rcodes, None, dev_bf16(cs.scale), dev_bf16(cs.offset), 4)


# ------------------------------------------------------------------------------ full benchmark shapes
# Every output is compared with the oracle where the oracle can compute it in seconds (M <= 16: all
# M x N elements); at M = 2048 all rows of one column in every 128-wide block of output columns
# (one per n-block of the matrix-core kernel) plus the whole first and last block of 128 columns.
# Packed words and re-laid-out words are compared over the whole matrix; dequantised weights over
# the whole matrix for the 8B linears and over the first 16 and last 4096 rows (the last tile
# included) of a full-size launch for the 70B ones.
ORACLE_THREADS = 16
DEQUANT_WHOLE_LIMIT = 28672 * 4096


def prefill_columns(N, rng):
    blocks = (N + 127) // 128
    one_per_block = [min(N - 1, b * 128 + int(rng.integers(0, 128))) for b in range(blocks)]
    return np.unique(np.concatenate([np.arange(0, min(128, N)), np.arange(max(0, N - 128), N), one_per_block]))


def gemm_tolerance_check(got, y64, rms, half_ulp, what):
    tol = 1e-2 * rms + np.abs(y64) * half_ulp
    err = np.abs(got - y64)
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    assert np.all(err <= tol), (what, "worst", worst, float(err[worst]), float(tol[worst]), "rms", rms)


def full_shape_check(any4, oracle, shape_name, N, K, bits, Ms, seed, group=128, f16=False, relayout=True):
    Mmax = max(Ms)
    cs = inputs.make_case(Mmax, N, K, bits, seed, f16=f16)
    if group == 64:
        other = inputs.make_case(1, N, K, bits, seed + 1000)
        sc = np.ascontiguousarray(np.stack([cs.scale, other.scale], axis=2).reshape(N, -1))
        of = np.ascontiguousarray(np.stack([cs.offset, other.offset], axis=2).reshape(N, -1))
    else:
        sc, of = np.ascontiguousarray(cs.scale[:, ::group // 128]), np.ascontiguousarray(cs.offset[:, ::group // 128])
    dev16 = dev_f16 if f16 else dev_bf16
    half_ulp = 2.0 ** -11 if f16 else 2.0 ** -8
    packed = oracle.pack(cs.codes_u8, bits)
    codes_dev = any4.any4_pack(torch.from_numpy(cs.codes_u8).cuda(), bits)
    assert np.array_equal(host_u32(codes_dev), packed), (shape_name, "packed words")
    lut, scale, offset = dev16(cs.lut), dev16(sc), dev16(of)
    rcodes = None
    if relayout:
        rcodes = any4.any4_repack(codes_dev, bits)
        assert np.array_equal(host_u32(rcodes), oracle.repack(packed, K, bits)), (shape_name, "re-laid-out words")
    # dequantised weights, bit for bit, from ONE launch on the whole matrix
    w = any4.any4_dequant(codes_dev, lut, scale, offset, K, bits, group=group)
    torch.cuda.synchronize()
    bands = [(0, N)] if N * K <= DEQUANT_WHOLE_LIMIT else [(0, 16), (N - 4096, N)]
    for r0, r1 in bands:
        w_ref = oracle.dequant(packed[r0:r1], cs.lut[r0:r1], sc[r0:r1], of[r0:r1], K, bits, group=group, f16=f16)
        assert np.array_equal(w[r0:r1].cpu().numpy().view(np.uint32), w_ref.view(np.uint32)), (shape_name, "dequant", r0, r1)
        del w_ref
    del w
    torch.cuda.empty_cache()
    rng = np.random.default_rng(seed + 1)
    for M in Ms:
        x = cs.x[:M]
        y = any4.any4_gemm(dev16(x), codes_dev, lut, scale, offset, bits, group=group)
        torch.cuda.synchronize()
        if rcodes is not None:
            y_re = any4.any4_gemm_repacked(dev16(x), rcodes, lut, scale, offset, bits)
            torch.cuda.synchronize()
            assert torch.equal(y.view(torch.int16), y_re.view(torch.int16)), (shape_name, M, "re-laid-out codes")
        if M <= 16:
            cols = None
            y64 = oracle.gemm(x, packed, cs.lut, sc, of, K, bits, threads=ORACLE_THREADS, group=group, f16=f16)
            got = y.float().cpu().numpy().astype(np.float64)
        else:
            cols = prefill_columns(N, rng)
            y64 = oracle.gemm(x, packed[cols], cs.lut[cols], sc[cols], of[cols], K, bits, threads=ORACLE_THREADS,
                              group=group, f16=f16)
            got = y[:, torch.from_numpy(cols).cuda()].float().cpu().numpy().astype(np.float64)
        assert got.shape == y64.shape
        gemm_tolerance_check(got, y64, oracle.rms(y64), half_ulp, (shape_name, M, N, K, bits, group, f16))


@pytest.mark.parametrize("name", list(inputs.LLAMA3_8B_SHAPES))
def test_llama3_8b_decode_and_prefill_shapes(any4, oracle, name):
    """Configs 2 and 4: M = 1, 8 (decode, every output) and M = 2048 (prefill, every n-block) on the 8B linears."""
    N, K = inputs.LLAMA3_8B_SHAPES[name]
    i = list(inputs.LLAMA3_8B_SHAPES).index(name)
    full_shape_check(any4, oracle, name, N, K, 4, (1, 8, 2048), seed=inputs.case_seed(20, i))


@pytest.mark.parametrize("variant", ("group64", "group1024", "f16"))
@pytest.mark.parametrize("name", list(inputs.LLAMA3_8B_SHAPES))
def test_llama3_8b_shapes_other_groups_and_fp16(any4, oracle, name, variant):
    """The full 8B linears at M = 1, 8 and 2048 with groups of 64 / 1024 weights and with fp16 storage."""
    N, K = inputs.LLAMA3_8B_SHAPES[name]
    i = list(inputs.LLAMA3_8B_SHAPES).index(name)
    group = {"group64": 64, "group1024": 1024, "f16": 128}[variant]
    if K % group:
        pytest.skip("the group must divide K")
    full_shape_check(any4, oracle, name, N, K, 4, (1, 8, 2048), seed=inputs.case_seed(60, i, len(variant)),
                     group=group, f16=variant == "f16", relayout=False)


@pytest.mark.parametrize("name", list(inputs.LLAMA3_70B_SHAPES))
def test_llama3_70b_batch_sweep(any4, oracle, name):
    """Config 3: M in {1, 2, 4, 8, 16} on the 70B linears, every output."""
    N, K = inputs.LLAMA3_70B_SHAPES[name]
    i = list(inputs.LLAMA3_70B_SHAPES).index(name)
    full_shape_check(any4, oracle, name, N, K, 4, (1, 2, 4, 8, 16), seed=inputs.case_seed(30, i))


@pytest.mark.parametrize("bits", (3, 2))
@pytest.mark.parametrize("name", list(inputs.LLAMA3_70B_SHAPES))
def test_llama3_70b_any3_any2(any4, oracle, name, bits):
    """Config 5: 3- and 2-bit variants at M = 1 and 16 on the 70B linears, every output."""
    N, K = inputs.LLAMA3_70B_SHAPES[name]
    i = list(inputs.LLAMA3_70B_SHAPES).index(name)
    full_shape_check(any4, oracle, name, N, K, bits, (1, 16), seed=inputs.case_seed(50 + bits, i))
