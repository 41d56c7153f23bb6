"""Parity of the HIP quantiser against its CPU oracle, through the C ABI, on a real MI355X.

Bar: codes, tables, scales, offsets and the number of centre updates bit-exact.  Both sides
take every decision (nearest centre, drawn sample) in fp64 on the same fp32 inputs; the only
arithmetic that may differ is the association of fp64 sums (partial sums per thread), which can
change a decision only when a value lies within ~1e-13 (relative) of a decision boundary.
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
    lib.load_library()
    return lib


@pytest.fixture(scope="module")
def qoracle():
    from oracle import any4_quant_oracle
    any4_quant_oracle.build()
    return any4_quant_oracle


def bits16(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def run_and_compare(any4, qoracle, w, act, u, bits, symmetric, iters, what, centre_gap=None, by_value=()):
    """Bit-exact comparison of everything the quantiser returns.  Rows listed in `by_value` are rows with
    fewer distinct values than centres whose values are not short binary fractions: the weighted mean of
    equal numbers is that number or a neighbour depending on how the fp64 sum is associated, and with it
    whether the weights then move on to an equal centre.  Those rows are compared by the table value every
    weight ends up with (plus scales and offsets), not by code numbering and update count."""
    ref = qoracle.quantize(w, act, u, bits, symmetric=symmetric, iters=iters, threads=8)
    got = any4.any4_quantize(torch.from_numpy(w).cuda(), None if act is None else torch.from_numpy(act).cuda(),
                             torch.from_numpy(u).cuda(), bits, symmetric=symmetric, iters=iters, centre_gap=centre_gap)
    torch.cuda.synchronize()
    exact = np.array([i not in by_value for i in range(w.shape[0])])
    assert np.array_equal(bits16(got["scale"]), ref["scale"]), (what, "scale")
    assert np.array_equal(bits16(got["offset"]), ref["offset"]), (what, "offset")
    assert np.array_equal(got["msteps"].cpu().numpy()[exact], ref["msteps"][exact]), (what, "msteps")
    lut = bits16(got["lut"])
    assert np.array_equal(lut[exact], ref["lut"][exact]), (what, "lut")
    codes = got["codes_u8"].cpu().numpy()
    bad = np.argwhere(codes[exact] != ref["codes_u8"][exact])
    assert bad.size == 0, (what, "codes", bad[:5].tolist(), len(bad))
    assert int(codes.max()) < (1 << bits)
    rec_got = np.take_along_axis(lut, codes.astype(np.int64), axis=1)
    rec_ref = np.take_along_axis(ref["lut"], ref["codes_u8"].astype(np.int64), axis=1)
    assert np.array_equal(rec_got, rec_ref), (what, "table value per weight")
    return got, ref


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("N,K", [(3, 128), (5, 384), (17, 1152), (64, 4096)])
def test_quantize_matches_oracle(any4, qoracle, bits, N, K):
    qc = inputs.make_quant_case(N, K, bits, seed=40 + bits)
    run_and_compare(any4, qoracle, qc.w, qc.act, qc.u, bits, False, 25, (bits, N, K))


# the three ways through the kernels: every row by the per-weight method; rows sorted once (what any4_quantize
# does up to K = 16384); sorted rows that all hand over to the per-weight method in their first pass
METHODS = {"per_weight": -1.0, "sorted": 2.0 ** -40, "hand_over": 1e300}


@pytest.mark.parametrize("method", sorted(METHODS))
@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("N,K", [(5, 384), (33, 4096), (6, 8192), (5, 12288), (4, 16384)])
def test_quantize_methods_match_oracle(any4, qoracle, bits, N, K, method):
    qc = inputs.make_quant_case(N, K, bits, seed=140 + bits + K % 7)
    run_and_compare(any4, qoracle, qc.w, qc.act, qc.u, bits, False, 30, (method, bits, N, K), centre_gap=METHODS[method])


@pytest.mark.parametrize("method", sorted(METHODS))
def test_quantize_methods_symmetric_caps_and_degenerate_rows(any4, qoracle, method):
    gap = METHODS[method]
    qc = inputs.make_quant_case(7, 1024, 4, seed=17)
    run_and_compare(any4, qoracle, qc.w, qc.act, qc.u, 4, True, 25, (method, "symmetric"), centre_gap=gap)
    for iters in (0, 1, 2, 300):
        run_and_compare(any4, qoracle, qc.w, None, qc.u, 4, False, iters, (method, "iters", iters), centre_gap=gap)
    w = qc.w.copy()
    w[0, 128:256] = 0.25
    w[1, :] = -0.5
    w[2, :] = np.tile(np.array([-1.0, -0.25, 0.5, 0.875], np.float32), 256)
    w[3, :] = 0.0
    w[4, ::2] = -w[4, 1::2]                                 # pairs of equal magnitude: ties between centres
    act = qc.act.copy()
    act[::3] = 0.0
    # no sampling mass at all: every centre is drawn by index and no centre ever moves
    run_and_compare(any4, qoracle, qc.w, np.zeros_like(qc.act), qc.u, 4, False, 5, (method, "zero activations"), centre_gap=gap)
    for bits in (4, 3, 2):
        u = qc.u[:, :1 << bits].copy()
        # row 1 (constant) scales to exactly 0 without an offset-free scale; row 2 to four values that are no
        # short binary fractions
        run_and_compare(any4, qoracle, w, act, u, bits, False, 20, (method, "degenerate", bits), centre_gap=gap, by_value=(2,))
        run_and_compare(any4, qoracle, w, act, u, bits, True, 20, (method, "degenerate, symmetric", bits), centre_gap=gap,
                        by_value=(1, 2))


@pytest.mark.parametrize("bits", (4, 3, 2))
def test_quantize_symmetric_and_unit_activations(any4, qoracle, bits):
    qc = inputs.make_quant_case(9, 1024, bits, seed=7)
    run_and_compare(any4, qoracle, qc.w, qc.act, qc.u, bits, True, 25, ("symmetric", bits))
    run_and_compare(any4, qoracle, qc.w, None, qc.u, bits, False, 25, ("act=None", bits))


@pytest.mark.parametrize("iters", (0, 1, 3, 200))
def test_quantize_iteration_caps(any4, qoracle, iters):
    qc = inputs.make_quant_case(6, 768, 4, seed=3)
    got, ref = run_and_compare(any4, qoracle, qc.w, qc.act, qc.u, 4, False, iters, ("iters", iters))
    assert ref["msteps"].max() <= iters


def test_quantize_many_rows_and_repeatability(any4, qoracle):
    """More rows than the chip holds blocks at once (several rounds of blocks per compute unit), every row
    against the oracle, and two runs of the same call bit-equal in everything they return."""
    qc = inputs.make_quant_case(3000, 4096, 4, seed=99)
    got, ref = run_and_compare(any4, qoracle, qc.w, qc.act, qc.u, 4, False, 20, "3000 rows")
    again = any4.any4_quantize(torch.from_numpy(qc.w).cuda(), torch.from_numpy(qc.act).cuda(), torch.from_numpy(qc.u).cuda(),
                               4, iters=20)
    torch.cuda.synchronize()
    for k in ("codes_u8", "msteps"):
        assert torch.equal(got[k], again[k]), k
    for k in ("lut", "scale", "offset"):
        assert torch.equal(got[k].view(torch.int16), again[k].view(torch.int16)), k


def test_quantize_long_rows(any4, qoracle):
    """The Llama-3 down projections' K, and the largest K the library accepts."""
    for K in (14336, any4.any4_quantize_max_k()):
        qc = inputs.make_quant_case(4, K, 4, seed=K)
        run_and_compare(any4, qoracle, qc.w, qc.act, qc.u, 4, False, 15, ("K", K))


def test_quantize_degenerate_rows(any4, qoracle):
    """Constant groups (alpha falls back to 1), a constant row (no sampling mass after the first
    centre), a row with fewer distinct values than centres, channels with zero activation."""
    qc = inputs.make_quant_case(6, 512, 4, seed=12)
    w = qc.w.copy()
    w[0, 128:256] = 0.25                                   # one constant group
    w[1, :] = -0.5                                         # constant row
    w[2, :] = np.tile(np.array([-1.0, -0.25, 0.5, 0.875], np.float32), 128)   # 4 distinct values
    act = qc.act.copy()
    act[::3] = 0.0
    got, ref = run_and_compare(any4, qoracle, w, act, qc.u, 4, False, 20, "degenerate", by_value=(2,))
    lut = inputs.bf16_bits_to_f32(ref["lut"])
    sc = inputs.bf16_bits_to_f32(ref["scale"]).repeat(128, axis=1)
    of = inputs.bf16_bits_to_f32(ref["offset"]).repeat(128, axis=1)
    rec = np.take_along_axis(lut, ref["codes_u8"].astype(np.int64), axis=1) * sc + of
    assert np.array_equal(rec[1], w[1]) and np.array_equal(rec[2], w[2])


def test_quantize_feeds_the_gemm(any4, qoracle, oracle):
    """quantize -> pack -> GEMM on the device against the oracle chain on the host, and the
    quantised product stays close to the full-precision one."""
    N, K, M, bits = 96, 1024, 4, 4
    qc = inputs.make_quant_case(N, K, bits, seed=5)
    got, ref = run_and_compare(any4, qoracle, qc.w, qc.act, qc.u, bits, False, 25, "chain")
    rng = np.random.default_rng(9)
    x = inputs.f32_to_bf16_bits((rng.standard_normal((M, K)) * qc.act[None, :]).astype(np.float32))
    xd = torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    packed = any4.any4_pack(got["codes_u8"], bits)
    y = any4.any4_gemm(xd, packed, got["lut"], got["scale"], got["offset"], bits)
    y64 = oracle.gemm(x, oracle.pack(ref["codes_u8"], bits), ref["lut"], ref["scale"], ref["offset"], K, bits)
    yf = inputs.bf16_bits_to_f32(bits16(y)).astype(np.float64)
    tol = 1e-2 * oracle.rms(y64) + np.abs(y64) * 2.0 ** -8
    assert np.all(np.abs(yf - y64) <= tol)
    exact = inputs.bf16_bits_to_f32(x).astype(np.float64) @ qc.w.astype(np.float64).T
    assert np.linalg.norm(y64 - exact) / np.linalg.norm(exact) < 0.2


def test_quantize_rejects_bad_arguments(any4):
    from paper_2507_04610_amd import binding
    lib = any4.load_library()
    kmax = any4.any4_quantize_max_k()
    w = torch.zeros((1, kmax + 128), dtype=torch.float32, device="cuda")
    u = torch.zeros((1, 16), dtype=torch.float32, device="cuda")
    with pytest.raises(binding.Any4Error):
        any4.any4_quantize(w, None, u, 4)
    with pytest.raises(binding.Any4Error):
        any4.any4_quantize(w[:, :256].contiguous(), None, u, 5)
    out = torch.zeros(64, dtype=torch.uint8, device="cuda")
    assert lib.any4_quantize(None, None, u.data_ptr(), 1, 128, 4, 0, 1, out.data_ptr(), out.data_ptr(),
                             out.data_ptr(), out.data_ptr(), None, None) == -1
    assert lib.any4_quantize(w.data_ptr(), None, u.data_ptr(), 1, 128, 4, 0, -1, out.data_ptr(), out.data_ptr(),
                             out.data_ptr(), out.data_ptr(), None, None) == -2
