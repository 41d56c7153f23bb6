"""Out-of-bounds detection on the GPU: every buffer of a call (outputs, workspace and the read-only
inputs) sits inside a larger allocation filled with a sentinel byte, with guard bands on both sides.
After the call every guard byte must still be the sentinel and every input byte unchanged.  One or
more cases per kernel variant: streaming kernel (plain / re-laid-out / table-free / groups above and
below 128 / fp16; one slab and several; ragged last tile), matrix-core kernel (whole tiles and K
slices), the wavefront-per-row kernel for very long K, pack, repack, dequant, quantiser and the
entry point that brings its own scratch."""
import numpy as np
import pytest

from paper_2507_04610_amd import inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

GUARD = 8192          # bytes on either side (a multiple of 16: the payload stays 16-byte aligned)
SENTINEL = 0xA5


@pytest.fixture(scope="module")
def any4():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    import paper_2507_04610_amd as lib
    lib.load_library()
    return lib


class Guarded:
    """a device tensor embedded in a sentinel-filled allocation"""

    def __init__(self, host=None, nbytes=None, dtype=None, shape=None, fill=None):
        if host is not None:
            host = np.ascontiguousarray(host)
            nbytes = host.nbytes
        self.nbytes = nbytes
        self.raw = torch.full((GUARD + nbytes + GUARD,), SENTINEL, dtype=torch.uint8, device="cuda")
        self.payload = self.raw[GUARD:GUARD + nbytes]
        if host is not None:
            self.payload.copy_(torch.from_numpy(host.view(np.uint8).reshape(-1)).cuda())
            self.before = self.payload.clone()
        else:
            self.before = None
            if fill is not None:
                self.payload.fill_(fill)
        self.dtype, self.shape = dtype, shape

    def tensor(self):
        return self.payload.view(self.dtype).view(*self.shape)

    def assert_intact(self, what):
        torch.cuda.synchronize()
        assert bool((self.raw[:GUARD] == SENTINEL).all()), (what, "bytes before the buffer were written")
        assert bool((self.raw[GUARD + self.nbytes:] == SENTINEL).all()), (what, "bytes after the buffer were written")
        if self.before is not None:
            assert torch.equal(self.payload, self.before), (what, "a read-only input was modified")


def guarded_case(oracle, M, N, K, bits, seed, group=128, f16=False):
    cs = inputs.make_case(M, N, K, bits, seed, f16=f16)
    dt = torch.float16 if f16 else torch.bfloat16
    if group == 64:
        sc, of = np.repeat(cs.scale, 2, axis=1), np.repeat(cs.offset, 2, axis=1)
    else:
        sc, of = np.ascontiguousarray(cs.scale[:, ::group // 128]), np.ascontiguousarray(cs.offset[:, ::group // 128])
    packed = oracle.pack(cs.codes_u8, bits)
    g = {
        "x": Guarded(cs.x, dtype=dt, shape=(M, K)),
        "codes": Guarded(packed, dtype=torch.int32, shape=packed.shape),
        "lut": Guarded(cs.lut, dtype=dt, shape=cs.lut.shape),
        "scale": Guarded(sc, dtype=dt, shape=sc.shape),
        "offset": Guarded(of, dtype=dt, shape=of.shape),
        "y": Guarded(nbytes=M * N * 2, dtype=dt, shape=(M, N), fill=0x11),
    }
    return cs, packed, sc, of, g


def all_intact(g, what):
    for name, buf in g.items():
        buf.assert_intact((what, name))


GEMM_CASES = [
    # (M, N, K, bits, variant)
    (1, 333, 4224, 4, "plain"), (1, 4099, 4096, 4, "plain"), (2, 40, 28672, 4, "plain"), (16, 100, 8192, 3, "plain"),
    (5, 70, 640, 2, "plain"), (3, 17, 384, 4, "plain"), (1, 256, 512, 4, "plain"),
    (1, 333, 4224, 4, "repacked"), (16, 49, 8192, 2, "repacked"), (2, 100, 14336, 3, "repacked"),
    (1, 333, 4224, 4, "no_table"), (16, 33, 8192, 4, "no_table"),
    (1, 333, 4096, 4, "group256"), (8, 100, 2048, 3, "group1024"),
    (1, 333, 4224, 4, "group64"), (13, 100, 4480, 2, "group64"),
    (1, 333, 4224, 4, "f16"), (16, 100, 4480, 3, "f16"),
    (37, 100, 14336, 4, "plain"),                   # a few dozen rows: 16 per launch
    (300, 384, 4096, 4, "plain"), (129, 130, 640, 3, "plain"), (2048, 200, 1024, 2, "plain"),   # matrix cores
    (300, 384, 4096, 4, "repacked"), (260, 300, 2048, 4, "group64"), (100, 200, 256, 4, "f16"), (40, 200, 1024, 4, "no_table"),
    (2, 5, 262272, 4, "plain"),                     # the wavefront-per-row kernel
]


@pytest.mark.parametrize("M,N,K,bits,variant", GEMM_CASES)
def test_gemm_writes_only_y_and_its_workspace(any4, oracle, M, N, K, bits, variant):
    group = {"group64": 64, "group256": 256, "group1024": 1024}.get(variant, 128)
    f16 = variant == "f16"
    cs, packed, sc, of, g = guarded_case(oracle, M, N, K, bits, seed=inputs.case_seed(91, bits, M % 10), group=group, f16=f16)
    need = any4.any4_gemm_workspace_bytes(M, N, K, bits)
    ws = Guarded(nbytes=max(need, 16), dtype=torch.uint8, shape=(max(need, 16),), fill=0x3C)
    g["ws"] = ws
    lut = None if variant == "no_table" else g["lut"].tensor()
    if variant == "repacked":
        r = any4.any4_repack(g["codes"].tensor(), bits)
        torch.cuda.synchronize()
        g["rcodes"] = Guarded(r.cpu().numpy(), dtype=torch.int32, shape=(r.numel(),))
        y = any4.any4_gemm_repacked(g["x"].tensor(), g["rcodes"].tensor(), lut, g["scale"].tensor(), g["offset"].tensor(), bits,
                                    out=g["y"].tensor(), workspace=ws.tensor())
    else:
        y = any4.any4_gemm(g["x"].tensor(), g["codes"].tensor(), lut, g["scale"].tensor(), g["offset"].tensor(), bits,
                           out=g["y"].tensor(), workspace=ws.tensor(), group=group)
    all_intact(g, (variant, M, N, K, bits))
    # and the result is the GEMM (the guard test is no substitute for parity, but a kernel that wrote
    # nothing at all would pass the guards)
    lut_host = cs.lut if variant != "no_table" else np.broadcast_to(
        inputs.f32_to_bf16_bits(np.arange(-8, 8, dtype=np.float32)), cs.lut.shape)
    y64 = oracle.gemm(cs.x, packed, lut_host, sc, of, K, bits, threads=16, group=group, f16=f16)
    got = y.float().cpu().numpy().astype(np.float64)
    tol = 1e-2 * oracle.rms(y64) + np.abs(y64) * (2.0 ** -11 if f16 else 2.0 ** -8)
    assert np.all(np.abs(got - y64) <= tol)


@pytest.mark.parametrize("M,N,K,bits", [(4, 64, 16384, 4), (300, 384, 4096, 3), (1, 100, 512, 2)])
def test_gemm_noalloc_writes_only_y(any4, oracle, M, N, K, bits):
    cs, packed, sc, of, g = guarded_case(oracle, M, N, K, bits, seed=92)
    any4.any4_gemm_noalloc(g["x"].tensor(), g["codes"].tensor(), g["lut"].tensor(), g["scale"].tensor(),
                           g["offset"].tensor(), bits, out=g["y"].tensor())
    all_intact(g, ("noalloc", M, N, K, bits))


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("N,K", [(5, 384), (257, 1152), (33, 14336)])
def test_pack_repack_dequant_write_only_their_outputs(any4, oracle, bits, N, K):
    cs = inputs.make_case(1, N, K, bits, seed=inputs.case_seed(93, bits, N % 7))
    W = K * bits // 32
    src = Guarded(cs.codes_u8, dtype=torch.uint8, shape=(N, K))
    out = Guarded(nbytes=N * W * 4, dtype=torch.int32, shape=(N, W), fill=0x11)
    any4.any4_pack(src.tensor(), bits, out=out.tensor())
    src.assert_intact("pack input")
    out.assert_intact("pack output")
    packed = oracle.pack(cs.codes_u8, bits)
    assert np.array_equal(out.tensor().cpu().numpy().view(np.uint32), packed)
    # repack: the binding allocates the output itself, so call the C ABI with a guarded buffer
    from paper_2507_04610_amd import binding
    lib = binding.load_library()
    rbytes = any4.any4_repack_bytes(N, K, bits)
    rout = Guarded(nbytes=rbytes, dtype=torch.int32, shape=(rbytes // 4,), fill=0x11)
    codes = Guarded(packed, dtype=torch.int32, shape=(N, W))
    assert lib.any4_repack(codes.tensor().data_ptr(), N, K, bits, rout.tensor().data_ptr(),
                           torch.cuda.current_stream().cuda_stream) == 0
    codes.assert_intact("repack input")
    rout.assert_intact("repack output")
    assert np.array_equal(rout.tensor().cpu().numpy().view(np.uint32), oracle.repack(packed, K, bits))
    # dequant
    lut, sc, of = (Guarded(a, dtype=torch.bfloat16, shape=a.shape) for a in (cs.lut, cs.scale, cs.offset))
    w = Guarded(nbytes=N * K * 4, dtype=torch.float32, shape=(N, K), fill=0x11)
    any4.any4_dequant(codes.tensor(), lut.tensor(), sc.tensor(), of.tensor(), K, bits, out=w.tensor())
    for name, b in (("codes", codes), ("lut", lut), ("scale", sc), ("offset", of), ("w", w)):
        b.assert_intact(("dequant", name))
    assert np.array_equal(w.tensor().cpu().numpy().view(np.uint32),
                          oracle.dequant(packed, cs.lut, cs.scale, cs.offset, K, bits).view(np.uint32))


@pytest.mark.parametrize("bits", (4, 3, 2))
def test_quantiser_writes_only_its_outputs(any4, bits):
    from paper_2507_04610_amd import binding
    lib = binding.load_library()
    N, K, L = 21, 1152, 1 << bits
    qc = inputs.make_quant_case(N, K, bits, seed=94)
    w, act, u = (Guarded(a, dtype=torch.float32, shape=a.shape) for a in (qc.w, qc.act, qc.u))
    codes = Guarded(nbytes=N * K, dtype=torch.uint8, shape=(N, K), fill=0x11)
    lut = Guarded(nbytes=N * L * 2, dtype=torch.bfloat16, shape=(N, L), fill=0x11)
    sc = Guarded(nbytes=N * (K // 128) * 2, dtype=torch.bfloat16, shape=(N, K // 128), fill=0x11)
    of = Guarded(nbytes=N * (K // 128) * 2, dtype=torch.bfloat16, shape=(N, K // 128), fill=0x11)
    ms = Guarded(nbytes=(N * 4 + 15) // 16 * 16, dtype=torch.int32, shape=((N * 4 + 15) // 16 * 4,), fill=0x11)
    rc = lib.any4_quantize(w.tensor().data_ptr(), act.tensor().data_ptr(), u.tensor().data_ptr(), N, K, bits, 0, 20,
                           codes.tensor().data_ptr(), lut.tensor().data_ptr(), sc.tensor().data_ptr(),
                           of.tensor().data_ptr(), ms.tensor().data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    for name, b in (("w", w), ("act", act), ("u", u), ("codes", codes), ("lut", lut), ("scale", sc), ("offset", of), ("msteps", ms)):
        b.assert_intact(("quantize", name))
    assert int(codes.tensor().max()) < L
    assert bool((ms.tensor()[N:] == 0x11111111).all()), "msteps past N were written"
