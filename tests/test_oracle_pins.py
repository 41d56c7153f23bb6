"""Pins for the CPU oracle: everything here is checked against something other than
the oracle itself - exact rational arithmetic on tiny inputs, closed forms, invariants,
special cases that reduce to textbook/library routines, and the storage figures the
paper prints.  CPU only."""
from fractions import Fraction
import os

import numpy as np
import pytest

from paper_2507_04610_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
BITS = (4, 3, 2)


# ----------------------------------------------------------------------------- helpers
def bf16_fraction(bits16: int) -> Fraction:
    """Exact value of a finite bf16 bit pattern, from the IEEE field definition."""
    sign = -1 if bits16 >> 15 else 1
    e = (bits16 >> 7) & 0xFF
    m = bits16 & 0x7F
    assert e != 0xFF
    if e == 0:
        return sign * Fraction(m, 1 << 7) * Fraction(1, 1 << 126)
    return sign * (1 + Fraction(m, 1 << 7)) * (Fraction(2) ** (e - 127))


def fraction_to_f32(v: Fraction) -> np.float32:
    """Round an exact rational to fp32, round-to-nearest-even, no double rounding."""
    if v == 0:
        return np.float32(0.0)
    a = abs(v)
    e = 0
    while Fraction(2) ** (e + 1) <= a:
        e += 1
    while Fraction(2) ** e > a:
        e -= 1
    e = max(e, -126)
    quantum = Fraction(2) ** (e - 23)
    q = a / quantum
    n = q.numerator // q.denominator
    rem = q - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and n % 2 == 1):
        n += 1
    r = n * quantum
    out = np.float32(float(r))            # r is representable: conversion is exact
    assert Fraction(float(out)) == r
    return -out if v < 0 else out


def bigint_pack(codes_row, bits):
    """Definition of the storage format as one little-endian bit stream per row."""
    big = 0
    for k, c in enumerate(codes_row):
        big |= int(c) << (bits * k)
    nwords = len(codes_row) * bits // 32
    return [(big >> (32 * i)) & 0xFFFFFFFF for i in range(nwords)]


def bigint_code(words, k, bits):
    big = 0
    for i, w in enumerate(words):
        big |= int(w) << (32 * i)
    return (big >> (bits * k)) & ((1 << bits) - 1)


def tiny_case(bits, N=3, K=256, M=2, seed=7):
    return inputs.make_case(M, N, K, bits, seed)


# ----------------------------------------------------------------------------- P7 packing
def test_pack_literal_words(oracle):
    # 4-bit, low nibble first: codes 1..8 -> 0x87654321 by inspection
    c = np.zeros((1, 128), np.uint8)
    c[0, :8] = [1, 2, 3, 4, 5, 6, 7, 8]
    assert oracle.pack(c, 4)[0, 0] == 0x87654321
    # 2-bit, 16 per word: 0,1,2,3 repeated -> every byte is 0b11_10_01_00 = 0xE4
    c = np.zeros((1, 128), np.uint8)
    c[0, :16] = [0, 1, 2, 3] * 4
    assert oracle.pack(c, 2)[0, 0] == 0xE4E4E4E4
    # 3-bit stream: code 10 sits in bits 30..32 and straddles words 0 and 1.
    # codes: k=10 -> 0b101 (5), k=11 -> 0b111, everything else 0
    #   word0 bit30 = 1, bit31 = 0 ; word1 bit0 = 1 ; k=11 occupies word1 bits 1..3
    c = np.zeros((1, 128), np.uint8)
    c[0, 10] = 5
    c[0, 11] = 7
    p = oracle.pack(c, 3)
    assert p.shape == (1, 12)
    assert p[0, 0] == 0x40000000 and p[0, 1] == 0b1111 and not p[0, 2:].any()
    # k=21 sits in bits 63..65: straddles words 1 and 2
    c = np.zeros((1, 128), np.uint8)
    c[0, 21] = 0b011
    p = oracle.pack(c, 3)
    assert p[0, 1] == 0x80000000 and p[0, 2] == 0x1 and p[0, 0] == 0


@pytest.mark.parametrize("bits", BITS)
def test_pack_matches_bitstream_definition_and_round_trips(oracle, bits):
    rng = np.random.default_rng(11 + bits)
    codes = rng.integers(0, 1 << bits, size=(5, 384), dtype=np.uint8)
    packed = oracle.pack(codes, bits)
    assert packed.shape == (5, 384 * bits // 32) and packed.dtype == np.uint32
    for n in range(5):
        assert [int(v) for v in packed[n]] == bigint_pack(codes[n], bits)
        for k in (0, 1, 7, 8, 10, 15, 16, 21, 31, 32, 42, 127, 128, 383):
            assert oracle.code(packed[n], k, bits) == bigint_code(packed[n], k, bits) == codes[n, k]
    assert np.array_equal(oracle.unpack(packed, 384, bits), codes)


def test_pack_rejects_out_of_range_codes(oracle):
    c = np.zeros((1, 128), np.uint8)
    c[0, 5] = 8
    with pytest.raises(ValueError):
        oracle.pack(c, 3)


# ----------------------------------------------------------------------------- P1 brute force
@pytest.mark.parametrize("bits", BITS)
def test_exact_rational_brute_force(oracle, bits):
    cs = tiny_case(bits)
    packed = oracle.pack(cs.codes_u8, bits)
    w = oracle.dequant(packed, cs.lut, cs.scale, cs.offset, cs.K, bits)
    y = oracle.gemm(cs.x, packed, cs.lut, cs.scale, cs.offset, cs.K, bits)
    for n in range(cs.N):
        words = [int(v) for v in packed[n]]
        wrow = []
        for k in range(cs.K):
            c = bigint_code(words, k, bits)
            g = k // 128
            exact = (bf16_fraction(int(cs.lut[n, c])) * bf16_fraction(int(cs.scale[n, g]))
                     + bf16_fraction(int(cs.offset[n, g])))
            w32 = fraction_to_f32(exact)
            assert w32.view(np.uint32) == w[n, k].view(np.uint32), (n, k)
            wrow.append(Fraction(float(w32)))
        for m in range(cs.M):
            terms = [wrow[k] * bf16_fraction(int(cs.x[m, k])) for k in range(cs.K)]
            exact_y = sum(terms)
            mag = sum(abs(t) for t in terms)
            assert abs(Fraction(float(y[m, n])) - exact_y) <= mag * Fraction(cs.K, 2 ** 52), (m, n)


# ----------------------------------------------------------------------------- P2 int4 special case
@pytest.mark.parametrize("lo", (-8, 0))
def test_integer_table_reproduces_grouped_int4(oracle, lo):
    """A table holding the 16 consecutive integers starting at `lo` turns the format into
    ordinary group-wise int4: w = (q + lo) * s + o with q the unsigned code.  All operands
    and the sum fit in fp64 exactly, so fp64 arithmetic followed by one cast to fp32 is the
    correctly rounded result."""
    cs = inputs.make_case(2, 6, 512, 4, seed=3)
    ints = np.arange(16, dtype=np.float32) + lo
    lut = np.tile(inputs.f32_to_bf16_bits(ints), (cs.N, 1))
    assert np.array_equal(inputs.bf16_bits_to_f32(lut[0]), ints)
    packed = oracle.pack(cs.codes_u8, 4)
    w = oracle.dequant(packed, lut, cs.scale, cs.offset, cs.K, 4)
    s = np.repeat(inputs.bf16_bits_to_f32(cs.scale).astype(np.float64), 128, axis=1)
    o = np.repeat(inputs.bf16_bits_to_f32(cs.offset).astype(np.float64), 128, axis=1)
    expect = ((cs.codes_u8.astype(np.float64) + lo) * s + o).astype(np.float32)
    assert np.array_equal(w.view(np.uint32), expect.view(np.uint32))


# ----------------------------------------------------------------------------- P3 permutation
@pytest.mark.parametrize("bits", BITS)
def test_code_table_permutation_invariance(oracle, bits):
    cs = inputs.make_case(3, 8, 384, bits, seed=5)
    L = 1 << bits
    rng = np.random.default_rng(99)
    codes2 = np.empty_like(cs.codes_u8)
    lut2 = np.empty_like(cs.lut)
    for n in range(cs.N):
        pi = rng.permutation(L).astype(np.uint8)
        codes2[n] = pi[cs.codes_u8[n]]
        lut2[n, pi] = cs.lut[n]
    assert not np.array_equal(np.sort(lut2, axis=1), lut2)     # tables are no longer sorted
    p1, p2 = oracle.pack(cs.codes_u8, bits), oracle.pack(codes2, bits)
    w1 = oracle.dequant(p1, cs.lut, cs.scale, cs.offset, cs.K, bits)
    w2 = oracle.dequant(p2, lut2, cs.scale, cs.offset, cs.K, bits)
    assert np.array_equal(w1.view(np.uint32), w2.view(np.uint32))
    y1 = oracle.gemm(cs.x, p1, cs.lut, cs.scale, cs.offset, cs.K, bits)
    y2 = oracle.gemm(cs.x, p2, lut2, cs.scale, cs.offset, cs.K, bits)
    assert np.array_equal(y1, y2)


# ----------------------------------------------------------------------------- P4 one table per matrix
def test_shared_table_matches_vectorised_gather(oracle):
    """One table for the whole matrix (the nf4/af4 mode of section 2.4.1) is the per-row
    format with identical rows; numpy's gather + broadcast gives the same weights."""
    cs = inputs.make_case(1, 7, 256, 4, seed=8)
    lut = np.tile(cs.lut[:1], (cs.N, 1))
    packed = oracle.pack(cs.codes_u8, 4)
    w = oracle.dequant(packed, lut, cs.scale, cs.offset, cs.K, 4)
    v = inputs.bf16_bits_to_f32(cs.lut[0]).astype(np.float64)[cs.codes_u8]
    s = np.repeat(inputs.bf16_bits_to_f32(cs.scale).astype(np.float64), 128, axis=1)
    o = np.repeat(inputs.bf16_bits_to_f32(cs.offset).astype(np.float64), 128, axis=1)
    assert np.array_equal(w, (v * s + o).astype(np.float32))


# ----------------------------------------------------------------------------- P5 closed forms
def _ones_bf16(shape):
    return np.full(shape, 0x3F80, np.uint16)


@pytest.mark.parametrize("bits", BITS)
def test_one_hot_table_gives_masked_sums(oracle, bits):
    cs = inputs.make_case(2, 4, 384, bits, seed=21)
    packed = oracle.pack(cs.codes_u8, bits)
    xf = inputs.bf16_bits_to_f32(cs.x).astype(np.float64)
    for c in range(1 << bits):
        lut = np.zeros_like(cs.lut)
        lut[:, c] = 0x3F80
        y = oracle.gemm(cs.x, packed, lut, _ones_bf16(cs.scale.shape), np.zeros_like(cs.offset), cs.K, bits)
        for n in range(cs.N):
            expect = (xf * (cs.codes_u8[n] == c)).sum(axis=1)
            assert np.allclose(y[:, n], expect, rtol=0, atol=1e-12 * np.abs(xf).sum())


def test_constant_codes_and_zero_table(oracle):
    cs = inputs.make_case(3, 5, 512, 4, seed=22)
    xf = inputs.bf16_bits_to_f32(cs.x).astype(np.float64)
    xg = xf.reshape(cs.M, -1, 128).sum(axis=2)                       # [M, G]
    s = inputs.bf16_bits_to_f32(cs.scale).astype(np.float64)
    o = inputs.bf16_bits_to_f32(cs.offset).astype(np.float64)
    lutf = inputs.bf16_bits_to_f32(cs.lut).astype(np.float64)
    atol = 1e-12 * np.abs(xf).sum()
    # all codes equal c: y[m,n] = sum_g fl32(LUT[n][c] s_g + o_g) * sum_{k in g} x[m,k]
    codes = np.full_like(cs.codes_u8, 11)
    y = oracle.gemm(cs.x, oracle.pack(codes, 4), cs.lut, cs.scale, cs.offset, cs.K, 4)
    wg = (lutf[:, 11:12] * s + o).astype(np.float32).astype(np.float64)   # [N, G]
    assert np.allclose(y, xg @ wg.T, rtol=0, atol=atol)
    # zero table: only the offsets survive
    y = oracle.gemm(cs.x, oracle.pack(cs.codes_u8, 4), np.zeros_like(cs.lut), cs.scale, cs.offset, cs.K, 4)
    assert np.allclose(y, xg @ o.T, rtol=0, atol=atol)
    # zero offsets (the symmetric-scaling case): y is linear in the scale
    y0 = oracle.gemm(cs.x, oracle.pack(cs.codes_u8, 4), cs.lut, cs.scale, np.zeros_like(cs.offset), cs.K, 4)
    v = np.take_along_axis(lutf, cs.codes_u8.astype(np.int64), axis=1)     # [N, K]
    w0 = (v * np.repeat(s, 128, axis=1)).astype(np.float32).astype(np.float64)
    assert np.allclose(y0, xf @ w0.T, rtol=0, atol=atol)


@pytest.mark.parametrize("bits", BITS)
def test_unit_vector_activations_read_back_weights(oracle, bits):
    """x[m] = e_{k_m} makes y[m, n] = w[n, k_m] exactly; distinct k_m per m with M != N also
    catches a transposed output or operand."""
    cs = inputs.make_case(4, 6, 384, bits, seed=23)
    ks = [0, 127, 128, 383]
    x = np.zeros((4, cs.K), np.uint16)
    for m, k in enumerate(ks):
        x[m, k] = 0x3F80
    packed = oracle.pack(cs.codes_u8, bits)
    w = oracle.dequant(packed, cs.lut, cs.scale, cs.offset, cs.K, bits)
    y = oracle.gemm(x, packed, cs.lut, cs.scale, cs.offset, cs.K, bits)
    assert y.shape == (4, 6)
    for m, k in enumerate(ks):
        assert np.array_equal(y[m], w[:, k].astype(np.float64))
    # two-hot: exact sum of two weights
    x2 = np.zeros((1, cs.K), np.uint16)
    x2[0, 5] = 0x3F80
    x2[0, 300] = 0xBF80                                          # -1
    y2 = oracle.gemm(x2, packed, cs.lut, cs.scale, cs.offset, cs.K, bits)
    assert np.array_equal(y2[0], w[:, 5].astype(np.float64) - w[:, 300].astype(np.float64))


def test_group_index_is_k_div_128(oracle):
    """Table == 1, offset == 0, scale[n][g] = 2^(g-n): a unit activation at k returns the scale of
    group k // 128 of that row (the group bounds are g*128 <= k < (g+1)*128)."""
    N, K = 3, 640
    G = K // 128
    codes = np.zeros((N, K), np.uint8)
    lut = _ones_bf16((N, 16))
    sc = np.array([[2.0 ** (g - n) for g in range(G)] for n in range(N)], np.float32)
    scale = inputs.f32_to_bf16_bits(sc)
    packed = oracle.pack(codes, 4)
    for k in (0, 1, 127, 128, 129, 255, 256, 511, 512, 639):
        x = np.zeros((1, K), np.uint16)
        x[0, k] = 0x3F80
        y = oracle.gemm(x, packed, lut, scale, np.zeros_like(scale), K, 4)
        assert np.array_equal(y[0], sc[:, k // 128].astype(np.float64)), k


def test_sign_symmetry(oracle):
    cs = inputs.make_case(2, 5, 256, 4, seed=24)
    packed = oracle.pack(cs.codes_u8, 4)
    y = oracle.gemm(cs.x, packed, cs.lut, cs.scale, cs.offset, cs.K, 4)
    yn = oracle.gemm(cs.x, packed, cs.lut ^ 0x8000, cs.scale, cs.offset ^ 0x8000, cs.K, 4)
    assert np.array_equal(y, -yn)
    yx = oracle.gemm(cs.x ^ 0x8000, packed, cs.lut, cs.scale, cs.offset, cs.K, 4)
    assert np.array_equal(y, -yx)


# ----------------------------------------------------------------------------- P6 library matmul
@pytest.mark.parametrize("bits", BITS)
def test_reduces_to_library_fp64_matmul(oracle, bits):
    cs = inputs.make_case(5, 37, 1024, bits, seed=31)
    packed = oracle.pack(cs.codes_u8, bits)
    w = oracle.dequant(packed, cs.lut, cs.scale, cs.offset, cs.K, bits)
    y = oracle.gemm(cs.x, packed, cs.lut, cs.scale, cs.offset, cs.K, bits)
    xf = inputs.bf16_bits_to_f32(cs.x).astype(np.float64)
    ref = xf @ w.astype(np.float64).T
    bound = (np.abs(xf) @ np.abs(w.astype(np.float64)).T) * (cs.K * 2.0 ** -52)
    assert np.all(np.abs(y - ref) <= bound)
    assert np.isclose(oracle.rms(y), np.sqrt(np.mean(ref ** 2)), rtol=1e-12)
    # threads only distribute rows: identical bits
    y4 = oracle.gemm(cs.x, packed, cs.lut, cs.scale, cs.offset, cs.K, bits, threads=4)
    assert np.array_equal(y, y4)


# ----------------------------------------------------------------------------- P8 storage arithmetic
def _golden_bits():
    vals = {}
    with open(os.path.join(GOLDEN, "bits_per_weight.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                vals[k] = float(v)
    return vals


def test_bits_per_weight_matches_paper(oracle):
    g = _golden_bits()
    K = int(g["K"])
    assert oracle.bits_per_weight(K, 4) == g["any4_bits_per_weight"] == 4.3125
    cs = inputs.make_case(1, 4, K, 4, seed=1)
    packed = oracle.pack(cs.codes_u8, 4)
    nw = cs.N * K
    assert cs.lut.nbytes * 8 / nw == g["lut_overhead_bits"]
    assert (cs.scale.nbytes + cs.offset.nbytes) * 8 / nw == g["group_overhead_bits"]
    total = (packed.nbytes + cs.lut.nbytes + cs.scale.nbytes + cs.offset.nbytes) * 8 / nw
    assert total == g["any4_bits_per_weight"]
    assert (packed.nbytes + cs.scale.nbytes + cs.offset.nbytes) * 8 / nw == g["int4_grouped_bits_per_weight"]
    # 3- and 2-bit analogues (derived, not printed in the paper): 8- and 4-entry tables
    assert oracle.bits_per_weight(K, 3) == 3 + 8 * 16 / K + 0.25
    assert oracle.bits_per_weight(K, 2) == 2 + 4 * 16 / K + 0.25


# ----------------------------------------------------------------------------- P9 fused == two-step
@pytest.mark.parametrize("bits", BITS)
def test_fused_and_two_step_roundings_coincide(oracle, bits):
    cs = inputs.make_case(1, 256, 512, bits, seed=0)
    packed = oracle.pack(cs.codes_u8, bits)
    _, differ = oracle.dequant(packed, cs.lut, cs.scale, cs.offset, cs.K, bits, return_differ=True)
    assert differ == 0


def test_generator_matches_recipe():
    cs = inputs.make_case(1, 256, 512, 4, seed=0)
    assert cs.codes_u8.shape == (256, 512) and cs.codes_u8.max() == 15 and cs.codes_u8.min() == 0
    lut = inputs.bf16_bits_to_f32(cs.lut)
    assert np.all(np.diff(lut, axis=1) >= 0)
    s = inputs.bf16_bits_to_f32(cs.scale)
    assert s.shape == (256, 4) and s.min() >= 0.00499 and s.max() <= 0.0201
    o = inputs.bf16_bits_to_f32(cs.offset)
    assert abs(float(o.std()) - 0.002) < 4e-4
    again = inputs.make_case(1, 256, 512, 4, seed=0)
    assert np.array_equal(cs.codes_u8, again.codes_u8) and np.array_equal(cs.x, again.x)
    # bf16 storage conversion is round-to-nearest-even
    assert inputs.f32_to_bf16_bits(np.array([1.0, 1.00390625, 1.01171875], np.float32)).tolist() == \
        [0x3F80, 0x3F80, 0x3F82]
