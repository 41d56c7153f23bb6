"""A seeded sweep over random (variant, bits, M, N, K): every entry point of the GEMM family against
the oracle on shapes nobody picked by hand (group counts that are / are not multiples of 4, ragged
N, every M regime).  Bar as in test_gpu_parity.py."""
import numpy as np
import pytest

from paper_2507_04610_amd import inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def dev16(a, f16):
    t = torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()
    return t.view(torch.float16 if f16 else torch.bfloat16)


@pytest.mark.parametrize("sweep_seed", (1, 2, 3))
def test_random_shapes_and_variants(oracle, sweep_seed):
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the parity tests must run on the GPU box")
    import paper_2507_04610_amd as any4
    any4.load_library()
    rng = np.random.default_rng(sweep_seed)
    for it in range(120):
        bits = int(rng.choice([4, 3, 2]))
        G = int(rng.choice([1, 2, 3, 4, 5, 8, 12, 16, 24, 32, 33, 40, 64, 100, 112]))
        K = 128 * G
        M = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 12, 16, 17, 31, 64, 100, 129, 257, 300]))
        N = int(rng.choice([1, 5, 15, 16, 17, 31, 33, 64, 100, 129, 255, 300, 513]))
        if M * N * K > 3e8:
            M = 8
        variant = str(rng.choice(["plain", "plain", "repack", "int4", "g64", "g256", "g512", "g1024", "f16"]))
        if variant == "int4" and bits != 4:
            variant = "plain"
        group = {"g64": 64, "g256": 256, "g512": 512, "g1024": 1024}.get(variant, 128)
        if K % group:
            variant, group = "plain", 128
        f16 = variant == "f16"
        seed = int(rng.integers(1 << 30))
        cs = inputs.make_case(M, N, K, bits, seed, f16=f16)
        lut = cs.lut
        if variant == "int4":                                # the table the table-free path stands for
            lut = np.tile(inputs.f32_to_bf16_bits(np.arange(-8, 8, dtype=np.float32)), (N, 1))
        if group == 64:
            other = inputs.make_case(1, N, K, bits, seed + 7)
            sc = np.ascontiguousarray(np.stack([cs.scale, other.scale], axis=2).reshape(N, -1))
            of = np.ascontiguousarray(np.stack([cs.offset, other.offset], axis=2).reshape(N, -1))
        else:
            r = max(group // 128, 1)
            sc, of = np.ascontiguousarray(cs.scale[:, ::r]), np.ascontiguousarray(cs.offset[:, ::r])
        packed = oracle.pack(cs.codes_u8, bits)
        y64 = oracle.gemm(cs.x, packed, lut, sc, of, K, bits, threads=8, group=group, f16=f16)
        codes = torch.from_numpy(packed.view(np.int32)).cuda()
        x_d, sc_d, of_d = dev16(cs.x, f16), dev16(sc, f16), dev16(of, f16)
        what = (sweep_seed, it, variant, bits, M, N, K, seed)
        print(what, flush=True)                              # names the case should the device fault
        if variant == "repack":
            y = any4.any4_gemm_repacked(x_d, any4.any4_repack(codes, bits), dev16(lut, f16), sc_d, of_d, bits)
        elif variant == "int4":
            y = any4.any4_gemm(x_d, codes, None, sc_d, of_d, bits)
        else:
            y = any4.any4_gemm(x_d, codes, dev16(lut, f16), sc_d, of_d, bits, group=group)
        torch.cuda.synchronize()
        got = y.float().cpu().numpy().astype(np.float64)
        tol = 1e-2 * oracle.rms(y64) + np.abs(y64) * (2.0 ** -11 if f16 else 2.0 ** -8)
        err = np.abs(got - y64)
        assert np.all(err <= tol), (what, float((err - tol).max()))


def test_random_dequant_pack_repack(oracle):
    """bit-exact legs on random shapes: pack, re-layout, dequant with every group size and both
    16-bit types"""
    import paper_2507_04610_amd as any4
    any4.load_library()
    rng = np.random.default_rng(9)
    for it in range(60):
        bits = int(rng.choice([4, 3, 2]))
        K = 128 * int(rng.choice([1, 2, 3, 5, 8, 16, 33, 112]))
        N = int(rng.choice([1, 7, 16, 17, 130, 257]))
        group = int(rng.choice([64, 128, 256, 512, 1024]))
        f16 = bool(rng.integers(2)) and group == 128
        if K % group:
            group = 128
        seed = int(rng.integers(1 << 30))
        cs = inputs.make_case(1, N, K, bits, seed, f16=f16)
        store = inputs.f32_to_f16_bits if f16 else inputs.f32_to_bf16_bits
        sc = store(rng.uniform(0.005, 0.02, size=(N, K // group)).astype(np.float32))
        of = store((rng.standard_normal((N, K // group)) * 0.002).astype(np.float32))
        print((it, bits, N, K, group, f16, seed), flush=True)
        packed = oracle.pack(cs.codes_u8, bits)
        codes = any4.any4_pack(torch.from_numpy(cs.codes_u8).cuda(), bits)
        assert np.array_equal(codes.cpu().numpy().view(np.uint32), packed)
        assert np.array_equal(any4.any4_repack(codes, bits).cpu().numpy().view(np.uint32), oracle.repack(packed, K, bits))
        w = any4.any4_dequant(codes, dev16(cs.lut, f16), dev16(sc, f16), dev16(of, f16), K, bits, group=group)
        torch.cuda.synchronize()
        w_ref = oracle.dequant(packed, cs.lut, sc, of, K, bits, group=group, f16=f16)
        assert np.array_equal(w.cpu().numpy().view(np.uint32), w_ref.view(np.uint32))
