"""GPU parity on inputs that load the offset term of  y = sum_g scale_g * P_g + offset_g * X_g
(section 2.5.2: dequant = alpha * w_Q + beta; X_g = the sum of the group's activations).

The benchmark recipe draws zero-mean activations and offsets a tenth of the scaled table values, so
there the offset term is a small part of y.  Here: activations with mean 1 and a few channels 30
times larger (the outlier channels of language-model activations), offsets as large as the scaled
table values, an all-zero table (y is the offset term alone: its closed form is checked as well),
the table-free int4 path (whose 136 * scale * X_g surplus cancels against the same group sums), and
fp16 storage with group sums of the activations close to the largest finite fp16 number.
Bar: that of every GEMM test, 1e-2 * rms + half a unit of output rounding."""
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


def dev16(a_u16, f16=False):
    t = torch.from_numpy(np.ascontiguousarray(a_u16).view(np.int16)).cuda()
    return t.view(torch.float16 if f16 else torch.bfloat16)


def shifted_activations(cs, seed, mean=1.0, outliers=30.0, f16=False):
    """x ~ N(mean, 1), every 61st channel `outliers` times larger"""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((cs.M, cs.K), dtype=np.float32) + np.float32(mean)
    x[:, ::61] *= np.float32(outliers)
    cs.x = (inputs.f32_to_f16_bits if f16 else inputs.f32_to_bf16_bits)(x)


def check(any4, oracle, cs, lut_for_device="table", f16=False, what=None):
    bits, K = cs.bits, cs.K
    packed = oracle.pack(cs.codes_u8, bits)
    y64 = oracle.gemm(cs.x, packed, cs.lut, cs.scale, cs.offset, K, bits, threads=16, f16=f16)
    codes = torch.from_numpy(packed.view(np.int32)).cuda()
    lut = dev16(cs.lut, f16) if lut_for_device == "table" else None
    y = any4.any4_gemm(dev16(cs.x, f16), codes, lut, dev16(cs.scale, f16), dev16(cs.offset, f16), bits)
    torch.cuda.synchronize()
    got = y.float().cpu().numpy().astype(np.float64)
    rms = oracle.rms(y64)
    tol = 1e-2 * rms + np.abs(y64) * (2.0 ** -11 if f16 else 2.0 ** -8)
    err = np.abs(got - y64)
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    assert np.all(err <= tol), (what, "worst", worst, float(err[worst]), float(tol[worst]), "rms", rms)
    if lut_for_device == "table" and not f16:            # the re-laid-out route reads the same offsets
        y_re = any4.any4_gemm_repacked(dev16(cs.x), any4.any4_repack(codes, bits), lut, dev16(cs.scale), dev16(cs.offset), bits)
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), y_re.view(torch.int16)), what
    return y64, got


# one or two rows (fetched once, re-distributed through LDS), more rows, K slabs, ragged N, the
# matrix-core kernel with whole tiles and with K slices
SHAPES = [(1, 333, 4224), (2, 40, 28672), (5, 700, 640), (16, 100, 8192), (1, 4100, 4096), (64, 200, 2048), (300, 384, 4096)]


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_nonzero_mean_activations_with_outlier_channels(any4, oracle, bits, M, N, K):
    cs = inputs.make_case(M, N, K, bits, seed=inputs.case_seed(81, bits, M))
    shifted_activations(cs, seed=M + N)
    check(any4, oracle, cs, what=("mean-1 x", M, N, K, bits))


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_offsets_as_large_as_the_scaled_table(any4, oracle, bits, M, N, K):
    cs = inputs.make_case(M, N, K, bits, seed=inputs.case_seed(82, bits, M))
    rng = np.random.default_rng(N + K)
    cs.offset = inputs.f32_to_bf16_bits(rng.standard_normal(cs.offset.shape, dtype=np.float32) * np.float32(0.0125))
    shifted_activations(cs, seed=M + N + 1)
    check(any4, oracle, cs, what=("large offsets", M, N, K, bits))


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_zero_table_is_the_offset_term_alone(any4, oracle, bits, M, N, K):
    """LUT = 0: y[m][n] = sum_g offset[n][g] * X[m][g] (section 2.5.2 with w_Q = 0).  Checked against the
    oracle on the same inputs and against the closed form computed from the inputs directly."""
    cs = inputs.make_case(M, N, K, bits, seed=inputs.case_seed(83, bits, M))
    cs.lut[:] = 0
    shifted_activations(cs, seed=M + N + 2, outliers=1.0)
    y64, got = check(any4, oracle, cs, what=("zero table", M, N, K, bits))
    X = inputs.bf16_bits_to_f32(cs.x).astype(np.float64).reshape(M, K // 128, 128).sum(axis=2)      # [M, G]
    closed = X @ inputs.bf16_bits_to_f32(cs.offset).astype(np.float64).T
    assert np.allclose(y64, closed, rtol=1e-9, atol=1e-9 * np.abs(closed).max())
    assert np.all(np.abs(got - closed) <= 1e-2 * oracle.rms(closed) + np.abs(closed) * 2.0 ** -8)


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_int4_without_table_on_nonzero_mean_activations(any4, oracle, M, N, K):
    """lut = NULL: the table-free kernel turns code c into 128 + c and takes 136 * scale * X_g off again;
    with mean-1 activations that surplus is ~50 times the result it hides."""
    cs = inputs.make_case(M, N, K, 4, seed=inputs.case_seed(84, 4, M))
    cs.lut[:] = inputs.f32_to_bf16_bits(np.arange(-8, 8, dtype=np.float32))
    shifted_activations(cs, seed=M + N + 3)
    check(any4, oracle, cs, lut_for_device=None, what=("int4, mean-1 x", M, N, K))


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("M,N,K", [(1, 333, 4224), (2, 40, 8192), (16, 100, 2048), (64, 200, 2048), (300, 130, 1024)])
def test_gemm_f16_group_sums_near_the_fp16_limit(any4, oracle, bits, M, N, K):
    """fp16 storage: the sums of 128 consecutive activations pass through fp16 pairs and must stay
    below 65504 (stated in the header).  Activations ~ N(460, 20): group sums of about 58900, up to
    ~60000, i.e. 90 % of the limit."""
    cs = inputs.make_case(M, N, K, bits, seed=inputs.case_seed(85, bits, M), f16=True)
    rng = np.random.default_rng(M + K)
    x = (rng.standard_normal((M, K), dtype=np.float32) * np.float32(20.0) + np.float32(460.0))
    cs.x = inputs.f32_to_f16_bits(x)
    sums = inputs.f16_bits_to_f32(cs.x).astype(np.float64).reshape(M, K // 128, 128).sum(axis=2)
    assert 5.5e4 < np.abs(sums).max() < 65504.0
    check(any4, oracle, cs, f16=True, what=("f16 near the limit", M, N, K, bits))
