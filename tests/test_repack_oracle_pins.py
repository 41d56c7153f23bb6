"""Pins of the oracle's tile-major re-layout (oracle/any4_oracle.c: any4o_repack) against things
other than itself: a word-level transpose written with numpy, single codes read back out of the
re-laid-out buffer with Python integer arithmetic, the zero padding of a ragged last tile, and
the multiset of words.  The layout follows the paper's offline re-arrangement of the weights into
the operand order of the matrix instruction (section 4.2, second paragraph), for a 64-lane
wavefront whose lane (n, q) owns row n of a 16-row tile and quarter q of a 128-code group."""
import numpy as np
import pytest

from paper_2507_04610_amd import inputs


def random_codes(N, K, bits, seed):
    return np.random.default_rng(seed).integers(0, 1 << bits, size=(N, K), dtype=np.uint8)


@pytest.mark.parametrize("bits", (4, 3, 2))
@pytest.mark.parametrize("N,K", [(16, 128), (32, 384), (48, 1024)])
def test_repack_is_a_transpose_of_quarter_pieces(oracle, bits, N, K):
    """A quarter of a group (32 codes) is exactly `bits` words in both layouts, so for N a multiple
    of 16 the re-layout is the axis permutation (t, n, g, q) -> (t, g, q, n) of those pieces."""
    packed = oracle.pack(random_codes(N, K, bits, 1), bits)
    G = K // 128
    want = packed.reshape(N // 16, 16, G, 4, bits).transpose(0, 2, 3, 1, 4).reshape(-1)
    assert np.array_equal(oracle.repack(packed, K, bits), want)


@pytest.mark.parametrize("bits", (4, 3, 2))
def test_single_codes_read_back(oracle, bits):
    """Code (r, k) sits at bit ((t G + g) 64 + 16 q + n) 32 bits + (k % 32) bits of the buffer."""
    N, K = 37, 640
    codes = random_codes(N, K, bits, 2)
    out = oracle.repack(oracle.pack(codes, bits), K, bits)
    big = int.from_bytes(out.tobytes(), "little")
    G = K // 128
    rng = np.random.default_rng(3)
    for _ in range(400):
        r, k = int(rng.integers(N)), int(rng.integers(K))
        t, n, g, q, e = r // 16, r % 16, k // 128, (k % 128) // 32, k % 32
        pos = (((t * G + g) * 64 + 16 * q + n) * 32 + e) * bits
        assert (big >> pos) & ((1 << bits) - 1) == codes[r, k], (r, k)


@pytest.mark.parametrize("bits", (4, 3, 2))
def test_ragged_last_tile_is_zero_padded(oracle, bits):
    N, K = 21, 256
    codes = random_codes(N, K, bits, 4) | 1                  # no zero code anywhere
    out = oracle.repack(oracle.pack(codes, bits), K, bits)
    assert out.size == 32 * K * bits // 32
    padded = np.zeros((32, K), np.uint8)
    padded[:N] = codes
    assert np.array_equal(out, oracle.repack(oracle.pack(padded, bits), K, bits))
    pieces = out.reshape(2, K // 128, 4, 16, bits)
    assert not pieces[1, :, :, 5:, :].any() and pieces[1, :, :, :5, :].all(axis=-1).any()


def test_words_are_only_moved(oracle):
    N, K, bits = 64, 512, 4
    packed = oracle.pack(random_codes(N, K, bits, 5), bits)
    out = oracle.repack(packed, K, bits)
    assert np.array_equal(np.sort(out), np.sort(packed.reshape(-1)))


def test_repack_rejects_bad_arguments(oracle):
    with pytest.raises(ValueError):
        oracle.repack(np.zeros((4, 3), np.uint32), 100, 4)
    with pytest.raises(ValueError):
        oracle.repack(np.zeros((4, 16), np.uint32), 128, 5)
