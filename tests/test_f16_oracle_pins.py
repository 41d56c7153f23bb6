"""Pins of the oracle's fp16 storage mode (any4o_*_gd with f16 != 0).  The paper names bfloat16 and
float16 as the types of the table entries (section 2.4.1); the arithmetic after the widening to
fp32 is the same for both."""
import numpy as np
import pytest

from paper_2507_04610_amd import inputs


def test_widening_of_all_65536_patterns_against_numpy(oracle):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.f16_bits_to_float(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))      # signed zeros and subnormals included


def test_a_few_patterns_from_the_format_definition(oracle):
    for pattern, value in ((0x3C00, 1.0), (0xC000, -2.0), (0x7BFF, 65504.0), (0x0400, 2.0 ** -14), (0x0001, 2.0 ** -24),
                           (0x3555, 0.333251953125), (0x8000, -0.0), (0x7C00, float("inf"))):
        assert oracle.f16_bits_to_float(pattern) == value


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("group", (64, 128, 256))
def test_gemm_reduces_to_a_library_matmul(oracle, bits, group):
    M, N, K = 3, 9, 512
    cs = inputs.make_case(M, N, K, bits, seed=31 + bits, f16=True)
    rng = np.random.default_rng(5)
    sc = inputs.f32_to_f16_bits(rng.uniform(0.005, 0.02, size=(N, K // group)).astype(np.float32))
    of = inputs.f32_to_f16_bits((rng.standard_normal((N, K // group)) * 0.002).astype(np.float32))
    packed = oracle.pack(cs.codes_u8, bits)
    w = oracle.dequant(packed, cs.lut, sc, of, K, bits, group=group, f16=True)
    y = oracle.gemm(cs.x, packed, cs.lut, sc, of, K, bits, group=group, f16=True)
    # the weights from the definition, in numpy: table entry * scale + offset, rounded once to fp32
    lut = cs.lut.view(np.float16).astype(np.float64)
    v = np.take_along_axis(lut, cs.codes_u8.astype(np.int64), axis=1)
    s = np.repeat(sc.view(np.float16).astype(np.float64), group, axis=1)
    o = np.repeat(of.view(np.float16).astype(np.float64), group, axis=1)
    assert np.array_equal(w, (v * s + o).astype(np.float32))
    x = cs.x.view(np.float16).astype(np.float64)
    want = x @ w.astype(np.float64).T
    assert np.allclose(y, want, rtol=0, atol=1e-12 * np.abs(want).max() * K)


def test_the_same_bits_mean_different_numbers_in_the_two_modes(oracle):
    """0x3C00 is 1.0 as fp16 and 0.0078125 as bf16: a mode mix-up cannot pass"""
    N, K, bits = 2, 128, 4
    codes = np.zeros((N, K), dtype=np.uint8)
    lut = np.full((N, 16), 0x3C00, dtype=np.uint16)
    one_h, one_b = np.full((N, 1), 0x3C00, np.uint16), np.full((N, 1), 0x3F80, np.uint16)
    zero = np.zeros((N, 1), np.uint16)
    packed = oracle.pack(codes, bits)
    assert np.all(oracle.dequant(packed, lut, one_h, zero, K, bits, f16=True) == 1.0)
    assert np.all(oracle.dequant(packed, lut, one_b, zero, K, bits, f16=False) == 0.0078125)
