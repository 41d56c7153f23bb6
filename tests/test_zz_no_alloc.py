"""any4_gemm_noalloc (the entry point for callers that cannot allocate device memory) against
any4_gemm, through the C ABI: same problem, same bits in y.  Every pair of calls runs back to back
on the library's one scratch array per GPU, the second on a smaller problem, so that whatever the
first left behind (partial sums, counters) lies under the second's scratch."""
import ctypes

import numpy as np
import pytest

from paper_2507_04610_amd import inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def lib():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    from paper_2507_04610_amd import binding
    return binding.load_library()


def dev_bf16(a_u16):
    return torch.from_numpy(np.ascontiguousarray(a_u16).view(np.int16)).cuda().view(torch.bfloat16)


def problem(oracle, M, N, K, bits, seed):
    cs = inputs.make_case(M, N, K, bits, seed)
    packed = oracle.pack(cs.codes_u8, bits)
    t = {"M": M, "N": N, "K": K, "bits": bits, "cs": cs, "packed": packed,
         "x": dev_bf16(cs.x), "codes": torch.from_numpy(packed.view(np.int32)).cuda(), "lut": dev_bf16(cs.lut),
         "scale": dev_bf16(cs.scale), "offset": dev_bf16(cs.offset)}
    return t


def call_workspace(lib, t):
    """the existing entry point, with a workspace of the caller's"""
    need = lib.any4_gemm_workspace_bytes(t["M"], t["N"], t["K"], t["bits"])
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    y = torch.full((t["M"], t["N"]), 3.0, dtype=torch.bfloat16, device="cuda")
    rc = lib.any4_gemm(t["x"].data_ptr(), t["codes"].data_ptr(), t["lut"].data_ptr(), t["scale"].data_ptr(),
                       t["offset"].data_ptr(), t["M"], t["N"], t["K"], t["bits"], y.data_ptr(), ws.data_ptr(), need,
                       torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    torch.cuda.synchronize()
    return y, need


def call_noalloc(lib, t):
    y = torch.full((t["M"], t["N"]), 5.0, dtype=torch.bfloat16, device="cuda")
    rc = lib.any4_gemm_noalloc(t["x"].data_ptr(), t["codes"].data_ptr(), t["lut"].data_ptr(), t["scale"].data_ptr(),
                               t["offset"].data_ptr(), t["M"], t["N"], t["K"], t["bits"], y.data_ptr(),
                               torch.cuda.current_stream().cuda_stream)
    assert rc == 0, rc
    return y


PAIRS = [
    # K slabs of the streaming kernel (counters + fp32 partial sums), then a smaller problem of the same kind
    ((4, 64, 16384, 4), (2, 40, 8192, 4)),
    # K slices of the matrix-core kernel (group sums, counters, partial tiles), then a small one without slices
    ((300, 384, 4096, 4), (100, 200, 256, 4)),
    # no scratch at all after one that used it; 3- and 2-bit codes
    ((16, 100, 28672, 3), (1, 256, 512, 2)),
    # a few dozen rows: the streaming kernel 16 rows a launch, sharing the counters from launch to launch
    ((37, 100, 14336, 4), (17, 64, 4096, 4)),
]


@pytest.mark.parametrize("first,second", PAIRS)
def test_noalloc_equals_gemm_on_two_calls_in_a_row(lib, oracle, first, second):
    a, b = problem(oracle, *first, seed=71), problem(oracle, *second, seed=72)
    ref_a, need_a = call_workspace(lib, a)
    ref_b, need_b = call_workspace(lib, b)
    assert need_a > need_b or need_b == 0
    # two calls in a row on the stream, no synchronisation and no allocation in between
    ya = call_noalloc(lib, a)
    yb = call_noalloc(lib, b)
    torch.cuda.synchronize()
    assert torch.equal(ya.view(torch.int16), ref_a.view(torch.int16)), ("first call", first)
    assert torch.equal(yb.view(torch.int16), ref_b.view(torch.int16)), ("second call", second)
    # and against the oracle, to the GEMM bar
    for t, y in ((a, ya), (b, yb)):
        cs = t["cs"]
        y64 = oracle.gemm(cs.x, t["packed"], cs.lut, cs.scale, cs.offset, t["K"], t["bits"], threads=8)
        got = inputs.bf16_bits_to_f32(y.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
        tol = 1e-2 * oracle.rms(y64) + np.abs(y64) * 2.0 ** -8
        assert np.all(np.abs(got - y64) <= tol)
    # once more in the other order: the larger problem over what the smaller one left
    yb2 = call_noalloc(lib, b)
    ya2 = call_noalloc(lib, a)
    torch.cuda.synchronize()
    assert torch.equal(ya2.view(torch.int16), ref_a.view(torch.int16))
    assert torch.equal(yb2.view(torch.int16), ref_b.view(torch.int16))


def test_noalloc_rejects_what_its_scratch_cannot_hold(lib):
    from paper_2507_04610_amd import binding
    M, N, K = 16, 500000, 8192
    assert lib.any4_gemm_workspace_bytes(M, N, K, 4) > binding.NOALLOC_SCRATCH_BYTES
    y = torch.full((16,), 7.0, dtype=torch.bfloat16, device="cuda")
    A = y.data_ptr()          # never dereferenced: the size check comes first
    assert lib.any4_gemm_noalloc(A, A, A, A, A, M, N, K, 4, A, None) == -5
    torch.cuda.synchronize()
    assert torch.all(y == 7.0)
