"""The in-kernel combination of K slabs / K slices: whatever the workspace held before the call
(never-used memory, another call's partial sums, counters left by a call with another slab
count), the result is the same bits every time and within the GEMM bar of the oracle.  The hand-over
between blocks uses agent-scope atomics and tagged arrival counters; a lost or early hand-over
would show as a run-to-run difference, so every case is repeated many times and the loop stops at
the first difference."""
import numpy as np
import pytest

from paper_2507_04610_amd import inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

TAG = 0x00A4C0DE5EED17          # the library's counter tag (csrc/any4_splitk.h): (tag << 8 | arrivals)
REPEATS = 40


@pytest.fixture(scope="module")
def any4():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    import paper_2507_04610_amd as lib
    lib.load_library()
    return lib


def dev_bf16(a_u16):
    return torch.from_numpy(np.ascontiguousarray(a_u16).view(np.int16)).cuda().view(torch.bfloat16)


def fills(need, rng):
    """workspace contents before a call"""
    words = need // 8
    yield "zeros", torch.zeros(need, dtype=torch.uint8, device="cuda")
    yield "0xA5", torch.full((need,), 0xA5, dtype=torch.uint8, device="cuda")
    yield "random", torch.from_numpy(rng.integers(0, 256, need, dtype=np.uint8)).cuda()
    for stale in (64, 255):
        # every word a tagged counter with `stale` arrivals: more than any slab count of these problems
        # has (so it cannot be this call's own), as a call with another work split could leave behind
        w = torch.full((words,), (TAG << 8) | stale, dtype=torch.int64, device="cuda")
        yield f"tagged, {stale} arrivals", torch.cat([w.view(torch.uint8), torch.zeros(need - words * 8, dtype=torch.uint8, device="cuda")])


@pytest.mark.parametrize("M,N,K,bits", [(4, 64, 16384, 4), (1, 115, 28672, 4), (16, 333, 14336, 3), (2, 5000, 8192, 2),
                                        (300, 384, 4096, 4), (256, 130, 14336, 4)])
def test_result_does_not_depend_on_what_the_workspace_held(any4, oracle, M, N, K, bits):
    cs = inputs.make_case(M, N, K, bits, seed=inputs.case_seed(95, bits, M % 10))
    packed = oracle.pack(cs.codes_u8, bits)
    y64 = oracle.gemm(cs.x, packed, cs.lut, cs.scale, cs.offset, K, bits, threads=16)
    tol = 1e-2 * oracle.rms(y64) + np.abs(y64) * 2.0 ** -8
    need = any4.any4_gemm_workspace_bytes(M, N, K, bits)
    assert need > 0, "these problems are cut along K"
    x, codes = dev_bf16(cs.x), torch.from_numpy(packed.view(np.int32)).cuda()
    lut, sc, of = dev_bf16(cs.lut), dev_bf16(cs.scale), dev_bf16(cs.offset)
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    rng = np.random.default_rng(M + N)
    first = None
    for name, ws in fills(need, rng):
        for rep in range(REPEATS):
            y.fill_(9.0)
            # the same workspace again and again: after the first call it holds that call's leftovers
            any4.any4_gemm(x, codes, lut, sc, of, bits, out=y, workspace=ws)
            torch.cuda.synchronize()
            got = y.view(torch.int16).cpu()
            if first is None:
                first = got.clone()
                g64 = y.float().cpu().numpy().astype(np.float64)
                assert np.all(np.abs(g64 - y64) <= tol), (M, N, K, bits, "out of tolerance")
            assert torch.equal(first, got), (M, N, K, bits, name, "repeat", rep, "differs from the first result")
