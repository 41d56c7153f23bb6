"""Pins for the CPU oracle of the quantiser: every check compares it with something other
than itself - the closed forms of the scaling equations, exact rational arithmetic,
scikit-learn's weighted Lloyd iterations, hand-computed k-means++ draws, sampling
frequencies, fixed-point conditions, and the global optimum by dynamic programming.
CPU only."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import any4_quant_oracle as qo
from paper_2507_04610_amd import inputs

from test_oracle_pins import bf16_fraction, fraction_to_f32

BITS = (4, 3, 2)


def bf16_rne(v32: np.float32) -> int:
    """fp32 -> bf16 bit pattern, round-to-nearest-even, from the field definition."""
    u = int(np.float32(v32).view(np.uint32))
    low = u & 0xFFFF
    up = u >> 16
    if low > 0x8000 or (low == 0x8000 and (up & 1)):
        up += 1
    return up & 0xFFFF


# ------------------------------------------------------------------ section 2.5.1: scaling
@pytest.mark.parametrize("bits", BITS)
def test_asymmetric_scaling_closed_form(bits):
    """alpha = (max - min) / (Qmax - Qmin), beta = min, w_S = (w - beta) / alpha, with values
    chosen so that nothing rounds: w_S must come out as the integers 0 .. 2^bits - 1 pattern."""
    q = (1 << bits) - 1
    alpha = 0.125
    beta = -1.0
    levels = np.arange(128) % (q + 1)
    w = (beta + alpha * levels).astype(np.float32)          # exact in fp32
    w2 = (0.5 + 0.25 * levels[::-1]).astype(np.float32)     # second group: alpha 0.25, beta 0.5
    scale, offset, ws, s = qo.scale_row(np.concatenate([w, w2]), None, bits)
    assert [float(bf16_fraction(int(v))) for v in scale] == [0.125, 0.25]
    assert [float(bf16_fraction(int(v))) for v in offset] == [-1.0, 0.5]
    assert np.array_equal(ws[:128], levels.astype(np.float32))
    assert np.array_equal(ws[128:], levels[::-1].astype(np.float32))
    assert np.array_equal(s[:128], np.full(128, 0.125, np.float32))      # E|x| = 1: s = alpha
    assert np.array_equal(s[128:], np.full(128, 0.25, np.float32))


@pytest.mark.parametrize("bits", BITS)
def test_symmetric_scaling_closed_form(bits):
    """alpha = max|w| / Qmax, beta = 0 with Qmax = 2^(bits-1) - 1."""
    qmax = (1 << (bits - 1)) - 1
    w = np.zeros(128, np.float32)
    w[5] = -0.25 * qmax
    w[9] = 0.125
    act = np.full(128, 3.0, np.float32)
    scale, offset, ws, s = qo.scale_row(w, act, bits, symmetric=True)
    assert float(bf16_fraction(int(scale[0]))) == 0.25 and int(offset[0]) == 0
    assert ws[5] == -qmax and ws[9] == 0.5 and ws[0] == 0.0
    assert np.array_equal(s, np.full(128, 0.75, np.float32))             # alpha * E|x|


def test_scaling_random_group_exact_rational():
    """A random group, every rounding step re-derived with exact rationals: fp32 (max - min),
    fp32 division by 15, bf16 rounding of alpha and beta, fp32 (w - beta), fp32 division."""
    rng = np.random.default_rng(3)
    w = (rng.standard_normal(128) * 0.02).astype(np.float32)
    act = (0.1 + rng.random(128)).astype(np.float32)
    scale, offset, ws, s = qo.scale_row(w, act, 4)
    mx, mn = Fraction(float(w.max())), Fraction(float(w.min()))
    alpha32 = fraction_to_f32(Fraction(float(fraction_to_f32(mx - mn))) / 15)
    a_bits, b_bits = bf16_rne(alpha32), bf16_rne(np.float32(w.min()))
    assert int(scale[0]) == a_bits and int(offset[0]) == b_bits
    a, b = bf16_fraction(a_bits), bf16_fraction(b_bits)
    for j in range(128):
        d = Fraction(float(fraction_to_f32(Fraction(float(w[j])) - b)))
        assert ws[j] == fraction_to_f32(d / a)
        assert s[j] == fraction_to_f32(a * Fraction(float(act[j])))


def test_constant_group_takes_unit_scale():
    w = np.full(128, 0.375, np.float32)
    scale, offset, ws, s = qo.scale_row(w, None, 4)
    assert float(bf16_fraction(int(scale[0]))) == 1.0 and float(bf16_fraction(int(offset[0]))) == 0.375
    assert np.all(ws == 0.0)


# ------------------------------------------------------------------ k-means++ initialisation
def test_kmeanspp_hand_computed_draws():
    """ws = [0, 1, 3, 6], s = [1, 2, 1, 4].
    centre 0: mass = s, running sums 1, 3, 4, 8; u = 0.3 -> 2.4 -> first index above is 1 (value 1).
    centre 1: squared distances to {1}: 1, 0, 4, 25; mass 1, 0, 4, 100; total 105;
              u = 0.04 -> 4.2; running sums 1, 1, 5 -> index 2 (value 3).
    centre 2: distances to {1, 3}: 1, 0, 0, 9; mass 1, 0, 0, 36; total 37; u = 0.5 -> 18.5 -> index 3 (value 6).
    centre 3: distances 1, 0, 0, 0; only index 0 has mass -> value 0 whatever u is."""
    ws = np.array([0, 1, 3, 6], np.float32)
    s = np.array([1, 2, 1, 4], np.float32)
    c = qo.init(ws, s, 4, np.array([0.3, 0.04, 0.5, 0.99], np.float32))
    assert c.tolist() == [1.0, 3.0, 6.0, 0.0]
    # the first draw alone: thresholds at 1/8, 3/8, 4/8 of the total mass
    for u0, want in ((0.0, 0.0), (0.12, 0.0), (0.13, 1.0), (0.37, 1.0), (0.38, 3.0), (0.49, 3.0), (0.51, 6.0), (0.999, 6.0)):
        assert qo.init(ws, s, 1, np.array([u0], np.float32))[0] == want


def test_kmeanspp_sampling_frequencies():
    """Over many uniform draws the first centre is picked with probability s_j / sum(s) and the
    second, given the first, with probability s_j d_j^2 / sum(s d^2) (D^2 weighting)."""
    rng = np.random.default_rng(11)
    ws = np.array([0.0, 0.5, 2.0, 2.5, 7.0, 9.0], np.float32)
    s = np.array([1.0, 3.0, 0.5, 2.0, 1.5, 1.0], np.float32)
    n = 20000
    first = np.array([qo.init(ws, s, 1, np.array([u], np.float32))[0] for u in rng.random(n, dtype=np.float32)])
    p = s / s.sum()
    for v, pv in zip(ws, p):
        f = np.mean(first == v)
        assert abs(f - pv) < 4 * np.sqrt(pv * (1 - pv) / n)
    u0 = np.float32(0.2)                                   # 0.2 * 9 = 1.8 -> index 1 (value 0.5)
    assert qo.init(ws, s, 1, np.array([u0], np.float32))[0] == 0.5
    second = np.array([qo.init(ws, s, 2, np.array([u0, u], np.float32))[1] for u in rng.random(n, dtype=np.float32)])
    m = s * (ws - 0.5) ** 2
    p2 = m / m.sum()
    for v, pv in zip(ws, p2):
        f = np.mean(second == v)
        assert abs(f - pv) < 4 * np.sqrt(pv * (1 - pv) / n) + 1e-9


def test_kmeanspp_zero_mass_fallback():
    """All samples equal: after the first centre nothing has mass; the draw indexes the row directly."""
    ws = np.full(8, 2.0, np.float32)
    s = np.ones(8, np.float32)
    assert qo.init(ws, s, 4, np.array([0.1, 0.5, 0.9, 0.0], np.float32)).tolist() == [2.0] * 4


# ------------------------------------------------------------------ Lloyd iterations (section 3.2)
def _row(seed, K=512, bits=4):
    qc = inputs.make_quant_case(1, K, bits, seed=seed)
    scale, offset, ws, s = qo.scale_row(qc.w[0], qc.act, bits)
    return qc, ws, s


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("seed", (1, 2, 3))
def test_lloyd_matches_scikit_learn(bits, seed):
    """Weighted Lloyd iterations from the same starting centres, run to a fixed point, against
    scikit-learn's KMeans (the library the paper's appendix names)."""
    from sklearn.cluster import KMeans
    L = 1 << bits
    qc, ws, s = _row(seed, 512, bits)
    c0 = qo.init(ws, s, L, qc.u[0])
    c, codes, done = qo.lloyd(ws, s, c0, 300)
    assert done < 300
    assert len(np.unique(codes)) == L, "pick another seed: scikit-learn relocates empty clusters"
    km = KMeans(n_clusters=L, init=c0.reshape(-1, 1), n_init=1, max_iter=300, tol=0.0, algorithm="lloyd")
    km.fit(ws.astype(np.float64).reshape(-1, 1), sample_weight=s.astype(np.float64))
    assert np.array_equal(km.labels_, codes)
    assert np.allclose(km.cluster_centers_[:, 0], c, rtol=1e-9, atol=1e-12)
    assert np.isclose(km.inertia_, qo.objective(ws, s, codes, c), rtol=1e-9)


@pytest.mark.parametrize("bits", BITS)
def test_steps_against_numpy_definitions(bits):
    """E-step = argmin of the squared difference (first minimum), M-step = Eq. (B) weighted mean,
    each re-computed with numpy from the definition."""
    L = 1 << bits
    qc, ws, s = _row(5, 384, bits)
    c = qo.init(ws, s, L, qc.u[0])
    for _ in range(4):
        codes, _ = qo.assign(ws, c)
        d = (ws.astype(np.float64)[:, None] - c[None, :]) ** 2
        assert np.array_equal(codes, np.argmin(d, axis=1))
        c_new = qo.update(ws, s, codes, c)
        for q in range(L):
            sel = codes == q
            if sel.any():
                want = np.sum(s[sel].astype(np.float64) * ws[sel]) / np.sum(s[sel].astype(np.float64))
                assert np.isclose(c_new[q], want, rtol=1e-12, atol=0)
            else:
                assert c_new[q] == c[q]
        c = c_new


@pytest.mark.parametrize("bits", BITS)
def test_objective_never_increases_and_fixed_point(bits):
    L = 1 << bits
    qc, ws, s = _row(7, 1024, bits)
    c = qo.init(ws, s, L, qc.u[0])
    codes, _ = qo.assign(ws, c)
    prev = qo.objective(ws, s, codes, c)
    # the objective re-computed from its definition
    assert np.isclose(prev, np.sum(s.astype(np.float64) * (ws.astype(np.float64) - c[codes]) ** 2), rtol=1e-12)
    for _ in range(200):
        c = qo.update(ws, s, codes, c)
        e1 = qo.objective(ws, s, codes, c)
        assert e1 <= prev * (1 + 1e-12)
        codes, changed = qo.assign(ws, c, codes)
        e2 = qo.objective(ws, s, codes, c)
        assert e2 <= e1 * (1 + 1e-12)
        prev = e2
        if changed == 0:
            break
    assert changed == 0
    c_end, codes_end, _ = qo.lloyd(ws, s, qo.init(ws, s, L, qc.u[0]), 300)
    assert np.array_equal(codes_end, codes) and np.array_equal(c_end, c)


def test_weight_scale_invariance_and_unit_weights():
    """Multiplying all sample weights by a constant changes nothing; with constant weights the
    centres are plain means (ordinary k-means)."""
    qc, ws, s = _row(9, 512, 4)
    c0 = qo.init(ws, s, 16, qc.u[0])
    c1, k1, _ = qo.lloyd(ws, s, c0, 100)
    c2, k2, _ = qo.lloyd(ws, (4 * s).astype(np.float32), c0, 100)
    assert np.array_equal(k1, k2) and np.allclose(c1, c2, rtol=1e-12)
    ones = np.ones_like(s)
    c3, k3, _ = qo.lloyd(ws, ones, c0, 100)
    for q in range(16):
        if (k3 == q).any():
            assert np.isclose(c3[q], ws[k3 == q].astype(np.float64).mean(), rtol=1e-12)


def weighted_kmeans_1d_optimum(x, wgt, k):
    """Global optimum of weighted 1-D k-means by dynamic programming over the sorted samples
    (clusters of an optimal solution are contiguous in sorted order)."""
    o = np.argsort(x, kind="stable")
    x, wgt = x[o].astype(np.float64), wgt[o].astype(np.float64)
    n = len(x)
    p0 = np.concatenate([[0], np.cumsum(wgt)])
    p1 = np.concatenate([[0], np.cumsum(wgt * x)])
    p2 = np.concatenate([[0], np.cumsum(wgt * x * x)])

    def cost(i, j):                                       # samples i .. j-1
        sw = p0[j] - p0[i]
        if sw <= 0:
            return 0.0
        sx = p1[j] - p1[i]
        return max(p2[j] - p2[i] - sx * sx / sw, 0.0)

    best = np.full((k + 1, n + 1), np.inf)
    best[0, 0] = 0.0
    for q in range(1, k + 1):
        for j in range(q, n + 1):
            best[q, j] = min(best[q - 1, i] + cost(i, j) for i in range(q - 1, j))
    return best[k, n]


@pytest.mark.parametrize("seed", (1, 2, 3, 4))
def test_lloyd_result_against_global_optimum(seed):
    """Lloyd's fixed point can never beat the dynamic-programming optimum, and with k-means++
    starts on a heavy-tailed row it stays close to it."""
    qc, ws, s = _row(seed, 128, 2)
    c, codes, _ = qo.lloyd(ws, s, qo.init(ws, s, 4, qc.u[0]), 300)
    got = qo.objective(ws, s, codes, c)
    opt = weighted_kmeans_1d_optimum(ws, s, 4)
    assert got >= opt * (1 - 1e-9)
    assert got <= 2.0 * opt


# ------------------------------------------------------------------ emission and the whole pipeline
def test_emit_sorts_and_renumbers():
    c = np.array([3.0, -1.0, 2.0, -1.0])
    codes = np.array([0, 1, 2, 3, 3, 0], np.uint8)
    lut, new = qo.emit(c, codes)
    assert [float(bf16_fraction(int(v))) for v in lut] == [-1.0, -1.0, 2.0, 3.0]
    assert new.tolist() == [3, 0, 2, 1, 1, 3]             # equal centres keep their order


@pytest.mark.parametrize("bits", BITS)
def test_row_with_few_distinct_values_is_reproduced(bits):
    """At most 2^bits distinct scaled values per row: the table holds exactly those values, the
    error is zero and alpha * table[code] + beta gives back every weight."""
    L = 1 << bits
    rng = np.random.default_rng(5)
    levels = np.sort(rng.choice(np.arange(0, 8 * (L - 1) + 1), size=L - 2, replace=False)).astype(np.float64) / 8
    levels = np.concatenate([[0.0], levels, [float(L - 1)]])[:L]        # includes 0 and 2^bits - 1: alpha stays 0.125
    levels = np.unique(np.concatenate([levels, [0.0, float(L - 1)]]))
    K = 256
    idx = rng.integers(0, len(levels), size=K)
    idx[:len(levels)] = np.arange(len(levels))
    idx[128:128 + len(levels)] = np.arange(len(levels))
    w = (-1.0 + 0.125 * levels[idx]).astype(np.float32)
    u = rng.random((1, L), dtype=np.float32)
    r = qo.quantize(w[None, :], None, u, bits, iters=50)
    lut = inputs.bf16_bits_to_f32(r["lut"][0])
    assert set(np.unique(lut).tolist()) == set(levels.tolist())
    sc = inputs.bf16_bits_to_f32(r["scale"][0]).repeat(128)
    of = inputs.bf16_bits_to_f32(r["offset"][0]).repeat(128)
    assert np.array_equal(lut[r["codes_u8"][0]] * sc + of, w)


@pytest.mark.parametrize("bits", BITS)
def test_quantize_is_the_composition_of_its_steps_and_beats_the_uniform_grid(bits):
    L = 1 << bits
    qc = inputs.make_quant_case(6, 512, bits, seed=21)
    r = qo.quantize(qc.w, qc.act, qc.u, bits, iters=25, threads=2)
    for n in range(qc.N):
        scale, offset, ws, s = qo.scale_row(qc.w[n], qc.act, bits)
        c, codes, done = qo.lloyd(ws, s, qo.init(ws, s, L, qc.u[n]), 25)
        lut, codes = qo.emit(c, codes)
        assert np.array_equal(r["scale"][n], scale) and np.array_equal(r["offset"][n], offset)
        assert np.array_equal(r["lut"][n], lut) and np.array_equal(r["codes_u8"][n], codes)
        assert r["msteps"][n] == done
        assert np.all(np.diff(inputs.bf16_bits_to_f32(lut)) >= 0)
        # weighted error of the learned table vs rounding to the integer grid 0 .. 2^bits - 1
        # (section 2.5.2 with the uniform format), both measured on the scaled row
        grid = np.clip(np.rint(ws), 0, L - 1)
        e_grid = np.sum(s.astype(np.float64) * (ws - grid) ** 2)
        e_any = qo.objective(ws, s, codes, np.sort(c))
        assert e_any < e_grid
