"""Pins of the CPU oracle against facts that do not come from the oracle itself:
brute force, closed forms, the quantizer's error bound, invariances, numpy
library routines and exact rational arithmetic.  The paper prints no worked
numerical example for this path (its per-layer SQNR / MSE curves are figures),
so no printed value is available as a fixture."""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import reference as orc

A, S, C = orc.ASYM_TENSOR, orc.SYM_TENSOR, orc.SYM_CHANNEL


# ----------------------------------------------------------------------------
# min / max (Sec. 2.1 Eq. 1-2)
# ----------------------------------------------------------------------------
def test_minmax_bruteforce_permutations():
    vals = [-1.5, -1.5, 0.0, -0.0, 2.25, 7.0]
    for r in range(1, 6):
        for combo in itertools.permutations(vals, r):
            mn, mx = orc.minmax(np.array(combo, np.float32))
            assert mn == min(combo) and mx == max(combo)
            # -0.0 is reported as +0.0
            assert not (mn == 0 and math.copysign(1.0, float(mn)) < 0)
            assert not (mx == 0 and math.copysign(1.0, float(mx)) < 0)
            i, j = orc.argminmax(np.array(combo, np.float32))
            assert combo[i] == min(combo) and combo[j] == max(combo)
            assert i == min(k for k, v in enumerate(combo) if v == min(combo))
            assert j == min(k for k, v in enumerate(combo) if v == max(combo))


def test_minmax_numpy_and_nan():
    rng = np.random.default_rng(1)
    x = rng.standard_normal(100_003).astype(np.float32)
    mn, mx = orc.minmax(x)
    assert mn == x.min() and mx == x.max()
    i, j = orc.argminmax(x)
    assert i == int(np.argmin(x)) and j == int(np.argmax(x))
    y = x.copy()
    y[::7] = np.nan                       # NaNs are ignored
    mn, mx = orc.minmax(y)
    assert mn == np.nanmin(y) and mx == np.nanmax(y)
    mn, mx = orc.minmax(np.array([3.5], np.float32))
    assert mn == 3.5 and mx == 3.5


# ----------------------------------------------------------------------------
# scale / zero-point closed forms (Eq. 2 with N = 256; Sec. 4 Eq. 4 with b = 8)
# ----------------------------------------------------------------------------
def test_params_closed_forms():
    # x in {-8, ..., 7.9375} step 2^-4: hi - lo = 15.9375, step 0.0625 exactly, zp = 0
    sc, inv, zp = orc.params(-8.0, 7.9375, A)
    assert sc == np.float32(0.0625) and inv == np.float32(16.0) and zp == 0
    # ReLU6 range [0, 6]
    sc, inv, zp = orc.params(0.0, 6.0, A)
    assert sc == np.float32(6.0) / np.float32(255.0)
    assert inv == np.float32(1.0) / sc and zp == -128
    # all-negative tensor: range widened to contain 0 -> zero maps to the top code
    sc, inv, zp = orc.params(-3.0, -1.0, A)
    assert sc == np.float32(3.0) / np.float32(255.0) and zp == 127
    # all-positive tensor: lo = 0
    sc, inv, zp = orc.params(2.0, 5.0, A)
    assert sc == np.float32(5.0) / np.float32(255.0) and zp == -128
    # symmetric: absmax 127 -> unit step
    for scheme in (S, C):
        sc, inv, zp = orc.params(-127.0, 3.0, scheme)
        assert sc == 1.0 and inv == 1.0 and zp == 0
        sc, inv, zp = orc.params(-1.0, 63.5, scheme)
        assert sc == 0.5 and inv == 2.0 and zp == 0
    # degenerate: all zeros, or a sub-normal step
    for scheme in (A, S):
        assert orc.params(0.0, 0.0, scheme) == (1.0, 1.0, 0)
        assert orc.params(0.0, 1e-40, scheme) == (1.0, 1.0, 0)


def test_zero_is_exact_and_zp_in_range():
    rng = np.random.default_rng(2)
    for _ in range(200):
        lo, hi = sorted(rng.standard_normal(2) * 10.0 ** rng.integers(-3, 4))
        sc, inv, zp = orc.params(lo, hi, A)
        assert -128 <= zp <= 127
        q = orc.quantize(np.zeros(1, np.float32), inv, zp)
        assert q[0] == zp
        assert orc.dequantize(q, sc, zp)[0] == 0.0


# ----------------------------------------------------------------------------
# int8 codes (Eq. 1 / Eq. 5) and dequantization (Eq. 3)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("zp,scale", [(0, 0.0625), (-128, 0.5), (-3, 2.0 ** -10), (100, 4.0)])
def test_int8_grid_gives_zero_error(zp, scale):
    k = np.arange(-128, 128, dtype=np.int32)
    x = ((k - zp).astype(np.float32) * np.float32(scale)).astype(np.float32)
    cal = orc.calibrate(x, A)
    # the calibrated step is the grid's own step (255 * 2^k / 255), so the grid is reproduced
    assert cal.scale[0] == np.float32(scale) and cal.zp[0] == zp
    fq = orc.fakequant(x, cal, A, keep_xhat=True)
    assert np.array_equal(fq.codes.astype(np.int32), k)
    assert np.array_equal(fq.xhat, x)
    m = orc.tensor_metrics(x, cal, fq)
    assert m.mse == 0.0 and m.sqnr_db == math.inf


def test_idempotence_and_power_of_two_invariance():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(50_000) * 0.7).astype(np.float32)
    cal = orc.calibrate(x, A)
    fq = orc.fakequant(x, cal, A, keep_xhat=True)
    # quantizing the dequantized tensor with the same parameters is the identity
    fq2 = orc.fakequant(fq.xhat, cal, A, keep_xhat=True)
    assert np.array_equal(fq2.codes, fq.codes) and fq2.sum_e2[0] == 0.0
    base = orc.tensor_metrics(x, cal, fq)
    for k in (-7, 5):
        y = (x * np.float32(2.0 ** k)).astype(np.float32)
        cy = orc.calibrate(y, A)
        fy = orc.fakequant(y, cy, A)
        assert cy.zp[0] == cal.zp[0] and cy.scale[0] == cal.scale[0] * np.float32(2.0 ** k)
        assert np.array_equal(fy.codes, fq.codes)
        my = orc.tensor_metrics(y, cy, fy)
        assert my.mse == pytest.approx(base.mse * 4.0 ** k, rel=1e-12)
        assert my.sqnr_db == pytest.approx(base.sqnr_db, abs=1e-9)


@pytest.mark.parametrize("scheme", [A, S])
def test_codes_are_nearest_grid_point_exact_arithmetic(scheme):
    """Against the definition in exact rationals: the code is the grid point
    nearest to x (ties aside), clamped to int8."""
    rng = np.random.default_rng(4)
    x = (rng.standard_normal(3000) * 1.3).astype(np.float32)
    cal = orc.calibrate(x, scheme)
    q = orc.fakequant(x, cal, scheme).codes.astype(int)
    sc, zp = Fraction(float(cal.scale[0])), int(cal.zp[0])
    n_edge = 0
    for xi, qi in zip(x.tolist(), q.tolist()):
        t = Fraction(xi) / sc + zp                 # exact position on the code axis
        near = max(-128, min(127, math.floor(t + Fraction(1, 2))))
        frac = abs((t - math.floor(t)) - Fraction(1, 2))
        if frac < Fraction(1, 10_000):              # fp32 multiply may tip a near-tie
            n_edge += 1
            assert abs(qi - near) <= 1
        else:
            assert qi == near
    assert n_edge < 20
    assert q.min() >= -128 and q.max() <= 127
    if scheme == A:
        assert q.min() == -128 and q.max() == 127   # the full range is used


def test_round_half_to_even_and_clamp():
    # step 1, zp 0: ties go to the even code; out-of-range values saturate
    x = np.array([0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5, 127.5, 1e6, -128.5, -129.5, -1e30],
                 np.float32)
    q = orc.quantize(x, 1.0, 0)
    assert q.tolist() == [0, 2, 2, 0, -2, -2, 126, 127, 127, -128, -128, -128]
    # zero-point is added after rounding: rne(0.5) + 1 = 1, not rne(1.5) = 2
    assert orc.quantize(np.array([0.5], np.float32), 1.0, 1).tolist() == [1]
    xh = orc.dequantize(np.array([-128, 0, 5, 127], np.int8), 0.25, 5)
    assert xh.tolist() == [-33.25, -1.25, 0.0, 30.5]


# ----------------------------------------------------------------------------
# MSE (Eq. 7): error bound of the method, numpy, cross-check
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("scheme", [A, S])
def test_error_bound_and_uniform_noise_model(scheme):
    rng = np.random.default_rng(5)
    x = (rng.standard_normal(400_000) * 2.0).astype(np.float32)
    cal = orc.calibrate(x, scheme)
    fq = orc.fakequant(x, cal, scheme, keep_xhat=True)
    sc = float(cal.scale[0])
    err = np.abs(x.astype(np.float64) - fq.xhat.astype(np.float64))
    assert err.max() <= sc * (1.0 + 1e-6)            # range ends (rounded zero-point)
    inner = (fq.codes > -128) & (fq.codes < 127)
    assert err[inner].max() <= sc * 0.5 * (1.0 + 1e-5)
    m = orc.tensor_metrics(x, cal, fq)
    assert m.mse <= sc * sc / 4.0
    assert m.mse == pytest.approx(sc * sc / 12.0, rel=0.02)
    # numpy float64 library routine
    ref = np.mean((x.astype(np.float64) - fq.xhat.astype(np.float64)) ** 2)
    assert m.mse == pytest.approx(ref, rel=1e-12)
    # pair metrics on (x, dequantized x) equal the quantizer's own error sums
    p = orc.pair_metrics(x, fq.xhat)
    assert p.sum_d2 == fq.sum_e2[0] and p.sum_ref2 == fq.sum_x2[0]
    assert p.mse == m.mse and p.sqnr_db == m.sqnr_db


def test_pair_metrics_numpy_and_asymmetry():
    rng = np.random.default_rng(6)
    a = rng.standard_normal(10_001).astype(np.float32)
    b = (a + 0.01 * rng.standard_normal(10_001)).astype(np.float32)
    p = orc.pair_metrics(a, b)
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    assert p.sum_ref2 == pytest.approx(np.sum(a64 * a64), rel=1e-13)
    assert p.sum_d2 == pytest.approx(np.sum((a64 - b64) ** 2), rel=1e-13)
    assert p.sqnr_db == pytest.approx(10 * np.log10(np.sum(a64 * a64) / np.sum((a64 - b64) ** 2)), abs=1e-10)
    # the signal is the first argument: swapping changes the signal energy only
    p2 = orc.pair_metrics(b, a)
    assert p2.sum_d2 == pytest.approx(p.sum_d2, rel=1e-13)
    assert p2.sum_ref2 == pytest.approx(np.sum(b64 * b64), rel=1e-13)
    # a constant offset c gives MSE = c^2 exactly
    c = orc.pair_metrics(a, a + np.float32(0.5))
    assert c.mse == pytest.approx(0.25, rel=1e-6)


# ----------------------------------------------------------------------------
# SQNR closed forms (Eq. 6)
# ----------------------------------------------------------------------------
def _sqnr(x, scheme=A):
    cal = orc.calibrate(x, scheme)
    fq = orc.fakequant(x, cal, scheme)
    return orc.tensor_metrics(x, cal, fq).sqnr_db, cal


def test_sqnr_uniform_closed_form():
    rng = np.random.default_rng(7)
    x = rng.uniform(-1.0, 1.0, 2_000_000).astype(np.float32)
    s, _ = _sqnr(x)
    # P_s = 1/3, P_n = (2/255)^2 / 12  ->  20 log10(255) = 48.13 dB
    assert s == pytest.approx(20 * math.log10(255.0), abs=0.05)


def test_sqnr_sine_closed_form():
    t = np.arange(4_000_000, dtype=np.float64)
    x = np.sin(t * 0.001234567).astype(np.float32)
    s, _ = _sqnr(x)
    # full-scale sine: 1.76 dB above the uniform input (6.02 * 8 + 1.76 neighbourhood)
    assert s == pytest.approx(20 * math.log10(255.0) + 10 * math.log10(1.5), abs=0.25)


@pytest.mark.parametrize("sigma", [0.5, 1.3, 2.0])
def test_sqnr_relu_gaussian_formula(sigma):
    rng = np.random.default_rng(8)
    x = np.maximum(rng.standard_normal(2_000_000) * sigma, 0).astype(np.float32)
    s, cal = _sqnr(x)
    mx = float(cal.max[0])
    # P_s = sigma^2 / 2, P_n = (max/255)^2 / 12 on the non-zero half (zeros are exact)
    expect = 10 * math.log10((sigma ** 2 / 2) / (0.5 * (mx / 255) ** 2 / 12))
    assert s == pytest.approx(expect, abs=0.05)


def test_sqnr_edge_values():
    assert orc.sqnr_db(1.0, 0.0) == math.inf
    assert orc.sqnr_db(0.0, 0.0) == math.inf
    assert orc.sqnr_db(0.0, 1.0) == -math.inf
    assert orc.sqnr_db(100.0, 1.0) == pytest.approx(20.0, abs=1e-12)
    assert orc.mse(6.0, 4) == 1.5


# ----------------------------------------------------------------------------
# tensor statistics vs numpy
# ----------------------------------------------------------------------------
def test_statistics_numpy():
    rng = np.random.default_rng(9)
    x = (rng.standard_normal(123_457) * 3 + 0.7).astype(np.float32)
    sx, sx2 = orc.moments(x)
    x64 = x.astype(np.float64)
    assert sx == pytest.approx(x64.sum(), rel=1e-12)
    assert sx2 == pytest.approx((x64 * x64).sum(), rel=1e-12)
    assert orc.variance(x) == pytest.approx(x64.var(), rel=1e-12)
    cal = orc.calibrate(x, A)
    m = orc.tensor_metrics(x, cal, orc.fakequant(x, cal, A))
    assert m.mean == pytest.approx(x64.mean(), rel=1e-12)
    assert m.var == pytest.approx(x64.var(), rel=1e-12)
    assert m.absmax == np.abs(x).max() and m.min == x.min() and m.max == x.max()


# ----------------------------------------------------------------------------
# per-output-channel scheme: each channel is an independent per-tensor problem
# ----------------------------------------------------------------------------
def test_per_channel_equals_per_row_problems():
    rng = np.random.default_rng(10)
    w = (rng.laplace(0, 0.05, (12, 27))).astype(np.float32)
    w[3] *= 20
    w[5] = 0.0                                       # a dead channel is degenerate
    cal = orc.calibrate(w, C, 12)
    fq = orc.fakequant(w, cal, C, 12)
    for c in range(12):
        rc = orc.calibrate(w[c], S)
        rf = orc.fakequant(w[c], rc, S)
        assert cal.scale[c] == rc.scale[0] and cal.zp[c] == 0
        assert cal.min[c] == w[c].min() and cal.max[c] == w[c].max()
        assert np.array_equal(fq.codes.reshape(12, 27)[c], rf.codes)
        assert fq.sum_e2[c] == rf.sum_e2[0]
    assert cal.scale[5] == 1.0 and fq.sum_e2[5] == 0.0
    m = orc.tensor_metrics(w, cal, fq)
    assert m.mse == pytest.approx(fq.sum_e2.sum() / w.size, rel=1e-13)
    # per-channel steps never lose to the single per-tensor step on outlier channels
    ct = orc.calibrate(w, S)
    mt = orc.tensor_metrics(w, ct, orc.fakequant(w, ct, S))
    assert m.mse < mt.mse
    with pytest.raises(ValueError):
        orc.calibrate(w, C, 5)


# ----------------------------------------------------------------------------
# SQNR delta (Sec. 6.4 Eq. 16)
# ----------------------------------------------------------------------------
def test_sqnr_delta_hand_worked():
    s = [40.0, 37.0, 43.0, 43.0, 20.0]
    assert orc.sqnr_deltas(s) == [0.0, -3.0, 6.0, 0.0, -23.0]
    assert np.allclose(orc.sqnr_deltas(s)[1:], np.diff(s))
    # real graph positions: the difference is divided by the distance
    assert orc.sqnr_deltas(s, [0, 2, 5, 6, 16]) == [0.0, -1.5, 2.0, 0.0, -2.3]
    # infinite SQNR is clamped before differencing
    assert orc.sqnr_deltas([math.inf, 50.0, -math.inf], cap_db=200.0) == [0.0, -150.0, -250.0]
    with pytest.raises(ValueError):
        orc.sqnr_deltas(s, [0, 1, 1, 2, 3])


# ----------------------------------------------------------------------------
# Algorithm 2 (RankLayersBySensitivity)
# ----------------------------------------------------------------------------
def test_rank_equals_stable_argsort_without_outliers():
    rng = np.random.default_rng(11)
    for _ in range(50):
        n = int(rng.integers(1, 40))
        w = rng.uniform(20, 50, n).round(0)           # rounded -> ties occur
        a = rng.uniform(20, 50, n).round(0)
        flat = np.ones(n)
        order, G = orc.rank_layers(w, a, flat, flat)
        dw = np.concatenate([[0.0], np.diff(w)])
        da = np.concatenate([[0.0], np.diff(a)])
        g = 0.6 * dw + 0.4 * da
        assert np.allclose(G, g, rtol=0, atol=1e-12)
        assert order == list(np.argsort(np.asarray(G), kind="stable"))


def test_rank_hand_worked_outliers():
    w = [40.0, 38.0, 45.0, 30.0, 31.0, 50.0]
    a = [30.0, 30.0, 30.0, 30.0, 30.0, 30.0]
    # weight deltas: 0 -2 7 -15 1 19 ; score = 0.6 * delta
    flat = [1.0] * 6
    order, G = orc.rank_layers(w, a, flat, flat)
    assert order == [3, 1, 0, 4, 2, 5]
    assert G == pytest.approx([0.0, -1.2, 4.2, -9.0, 0.6, 11.4])
    # one activation-MSE outlier (layer 5: 100 > 5 * mean 17.5): moved to the front
    m1 = [1.0, 1.0, 1.0, 1.0, 1.0, 100.0]
    assert orc.rank_layers(w, a, flat, m1)[0] == [5, 3, 1, 0, 4, 2]
    # exactly 5x the mean is not an outlier (strict inequality): mean 2, m = 10
    m_eq = [10.0, 0.0, 0.5, 0.5, 0.5, 0.5]
    assert orc.rank_layers(w, a, flat, m_eq)[0] == [3, 1, 0, 4, 2, 5]
    # two outliers among 12 layers: the larger MSE comes first
    w12 = [40.0 - i for i in range(12)]
    a12 = [30.0] * 12
    m2 = [1.0] * 12
    m2[4], m2[9] = 60.0, 90.0                         # mean 13.33, threshold 66.7 -> only 9
    assert orc.rank_layers(w12, a12, m2, m2)[0][:1] == [9]
    m2[4], m2[9] = 200.0, 300.0                       # mean 42.5, threshold 212.5 -> only 9
    assert orc.rank_layers(w12, a12, m2, m2)[0][0] == 9
    m3 = [1.0] * 30
    m3[7], m3[20] = 50.0, 80.0                        # mean 5.27, threshold 26.3 -> both
    order = orc.rank_layers([40.0] * 30, [30.0] * 30, m3, m3)[0]
    assert order[:2] == [20, 7] and order[2:] == [i for i in range(30) if i not in (7, 20)]
    # outlier that is already first stays first; equal outliers: lower index first
    m4 = [1.0] * 30
    m4[3] = m4[11] = 70.0
    order = orc.rank_layers([40.0] * 30, [30.0] * 30, m4, m4)[0]
    assert order[:3] == [3, 11, 0]


def test_rank_mse_sources_and_gains():
    w = [40.0, 30.0, 35.0, 20.0]
    a = [40.0, 45.0, 25.0, 44.0]
    wm = [1.0] * 20
    am = [1.0] * 20
    w20 = w + [20.0] * 16
    a20 = a + [44.0] * 16
    wm[2] = 100.0
    am[1] = 100.0
    cfg = orc.RankConfig
    assert orc.rank_layers(w20, a20, wm, am, cfg=cfg(mse_source=0))[0][0] == 1
    assert orc.rank_layers(w20, a20, wm, am, cfg=cfg(mse_source=1))[0][0] == 2
    o2 = orc.rank_layers(w20, a20, wm, am, cfg=cfg(mse_source=2))[0]
    assert set(o2[:2]) == {1, 2} and o2[:2] == [1, 2]      # equal ratios: lower index first
    # activation gain 0 reproduces a weight-delta-only list
    o = orc.rank_layers(w, a, [1.0] * 4, [1.0] * 4, cfg=cfg(alpha_w=1.0, alpha_a=0.0))[0]
    assert o == [3, 1, 0, 2]                                # deltas 0 -10 5 -15
    o = orc.rank_layers(w, a, [1.0] * 4, [1.0] * 4, cfg=cfg(alpha_w=0.0, alpha_a=1.0))[0]
    assert o == [2, 0, 1, 3]                                # deltas 0 5 -20 19
    with pytest.raises(ValueError):
        orc.rank_layers(w, a, [1.0] * 4, [1.0, math.nan, 1.0, 1.0])


def test_rank_bruteforce_properties():
    rng = np.random.default_rng(12)
    for _ in range(200):
        n = int(rng.integers(1, 60))
        w = rng.uniform(10, 60, n)
        a = rng.uniform(10, 60, n)
        m = rng.lognormal(0, 2.0, n)                  # heavy tail -> outliers happen
        order, G = orc.rank_layers(w, a, m, m)
        assert sorted(order) == list(range(n))        # a permutation
        out = [i for i in range(n) if m[i] > 5 * (math.fsum(m) / n)]
        k = len(out)
        assert set(order[:k]) == set(out)             # outliers form the prefix ...
        assert all(m[order[i]] >= m[order[i + 1]] for i in range(k - 1))   # ... by descending MSE
        rest = order[k:]
        assert all((G[rest[i]], rest[i]) <= (G[rest[i + 1]], rest[i + 1]) for i in range(len(rest) - 1))


# ----------------------------------------------------------------------------
# Sec. 7: baselines and the BOPs reduction rate (Eq. 17)
# ----------------------------------------------------------------------------
def test_bops_closed_forms():
    macs = [118_013_952, 115_605_504, 231_211_008, 512_000]
    # everything int8: 1 - 8/32 = 75 %; everything fp32: 0 %
    assert orc.bops_reduction_pct(macs, [False] * 4) == pytest.approx(75.0, abs=1e-12)
    assert orc.bops_reduction_pct(macs, [True] * 4) == pytest.approx(0.0, abs=1e-12)
    # hand-worked: MACs 1, 1, 2 with the last layer in fp32: 1 - (8 + 8 + 64) / 128 = 37.5 %
    assert orc.bops_reduction_pct([1, 1, 2], [False, False, True]) == pytest.approx(37.5, abs=1e-12)
    # the rate depends on MAC shares only
    assert orc.bops_reduction_pct([3, 3, 6], [False, False, True]) == pytest.approx(37.5, abs=1e-12)


def test_bops_select_hand_worked_and_bruteforce():
    macs = [1.0, 1.0, 2.0, 4.0]                    # shares 12.5 / 12.5 / 25 / 50 %
    order = [2, 0, 3, 1]
    # keeping layer 2 costs 0.75 * 25 = 18.75 points, layer 0 a further 9.375, layer 3 37.5
    assert orc.bops_select(order, macs, 75.0) == ([False] * 4, 0, pytest.approx(75.0))
    keep, k, pct = orc.bops_select(order, macs, 56.25)
    assert (keep, k) == ([False, False, True, False], 1) and pct == pytest.approx(56.25)
    keep, k, pct = orc.bops_select(order, macs, 50.0)
    assert (keep, k) == ([False, False, True, False], 1)      # 46.875 would be below 50
    keep, k, pct = orc.bops_select(order, macs, 46.0)
    assert (keep, k) == ([True, False, True, False], 2) and pct == pytest.approx(46.875)
    keep, k, pct = orc.bops_select(order, macs, 0.0)
    assert k == 4 and pct == pytest.approx(0.0, abs=1e-12)
    # brute force: the kept set is the longest prefix of the list that meets the target
    rng = np.random.default_rng(13)
    for _ in range(200):
        n = int(rng.integers(1, 30))
        m = rng.integers(1, 1000, n).astype(float)
        o = list(rng.permutation(n))
        tgt = float(rng.uniform(-5, 80))
        keep, k, pct = orc.bops_select(o, m, tgt)
        best = 0
        for j in range(n + 1):
            flags = [i in o[:j] for i in range(n)]
            if orc.bops_reduction_pct(m, flags) >= tgt:
                best = j
            else:
                break
        assert k == best and keep == [i in o[:k] for i in range(n)]
        assert pct >= tgt or k == 0
    with pytest.raises(ValueError):
        orc.bops_select([0, 0, 1], [1.0, 1.0, 1.0], 50.0)
    with pytest.raises(ValueError):
        orc.bops_select([0, 1], [0.0, 0.0], 50.0)


def test_config_text_literal():
    """Sec. 4 step 5: the per-layer bit-width table.  The paper prints no format; the one this
    build states (a header line, then index, name and 32 or 8 per layer, in layer order) is
    written out here by hand, so a swapped bit-width, a changed header or a lost line shows."""
    want = ("layer,name,bits\n"
            "0,conv1,8\n"
            "1,layer1.0.conv1,32\n"
            "2,layer1.0.conv2,8\n"
            "3,fc,32\n")
    assert orc.config_text([False, True, False, True], ["conv1", "layer1.0.conv1", "layer1.0.conv2", "fc"]) == want
    assert orc.config_text([1, 0]) == "layer,name,bits\n0,layer0,32\n1,layer1,8\n"
    assert orc.config_text([]) == "layer,name,bits\n"
    for bad in ("a,b", "a\nb", "a\rb"):
        with pytest.raises(ValueError):
            orc.config_text([True], [bad])


def test_baseline_orders():
    w = [40.0, 38.0, 45.0, 30.0, 38.0]
    assert orc.baseline_order(orc.INORDER, n=5) == [4, 3, 2, 1, 0]
    assert orc.baseline_order(orc.WEIGHT_SQNR_ORDER, w) == [3, 1, 4, 0, 2]
    assert orc.baseline_order(orc.WEIGHT_SQNR_ORDER, w) == list(np.argsort(w, kind="stable"))
    # weight gain 1, activation gain 0 on raw SQNR is not the delta list: the two differ
    assert orc.rank_layers(w, None, [1.0] * 5, None, cfg=orc.RankConfig(1.0, 0.0, mse_source=1))[0] != \
        orc.baseline_order(orc.WEIGHT_SQNR_ORDER, w)


def test_layer_macs_of_the_shape_tables():
    from paper_2501_07161_amd import synth
    # published per-image MAC totals: ResNet-18 1.81 G, ResNet-50 (v1, stride on the first 1x1) 3.86 G,
    # VGG-16 15.47 G, MobileNetV2 0.30 G
    for fn, want in ((synth.resnet18_layers, 1.814e9), (synth.resnet50_layers, 3.86e9),
                     (synth.vgg16_layers, 15.47e9), (synth.mobilenetv2_layers, 0.300e9)):
        assert sum(synth.layer_macs(fn())) == pytest.approx(want, rel=0.02)


# ----------------------------------------------------------------------------
# cosine similarity (Sec. 6.1 Eq. 8)
# ----------------------------------------------------------------------------
def test_cosine_similarity_pins():
    rng = np.random.default_rng(14)
    a = rng.standard_normal(20_001).astype(np.float32)
    b = (a + 0.3 * rng.standard_normal(20_001)).astype(np.float32)
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    want = float(a64 @ b64 / (np.linalg.norm(a64) * np.linalg.norm(b64)))     # library routines
    assert orc.cosine_similarity(a, b) == pytest.approx(want, abs=1e-13)
    assert orc.cosine_similarity(a, a) == pytest.approx(1.0, abs=1e-15)
    assert orc.cosine_similarity(a, -a) == pytest.approx(-1.0, abs=1e-15)
    assert orc.cosine_similarity(a, b) == pytest.approx(orc.cosine_similarity(b, a), abs=1e-15)
    # direction only: positive rescaling changes nothing, a power of two exactly nothing
    assert orc.cosine_similarity(a, b * np.float32(4.0)) == orc.cosine_similarity(a, b)
    assert orc.cosine_similarity(a * np.float32(3.0), b) == pytest.approx(want, abs=1e-7)
    # orthogonal and 45-degree vectors
    assert orc.cosine_similarity([1.0, 0.0, 0.0], [0.0, 2.0, 0.0]) == 0.0
    assert orc.cosine_similarity([1.0, 0.0], [1.0, 1.0]) == pytest.approx(math.sqrt(0.5), abs=1e-15)
    assert orc.cosine_similarity([3.0, 4.0], [4.0, 3.0]) == pytest.approx(24.0 / 25.0, abs=1e-15)
    # zero vectors (reading): both zero -> 1, one zero -> 0
    assert orc.cosine_similarity([0.0, 0.0], [0.0, 0.0]) == 1.0
    assert orc.cosine_similarity([0.0, 0.0], [1.0, 0.0]) == 0.0
    # a quantized tensor stays within a hair of its original: 1 - cos ~ MSE / (2 * mean x^2)
    x = (rng.standard_normal(200_000) * 0.7).astype(np.float32)
    cal = orc.calibrate(x, A)
    fq = orc.fakequant(x, cal, A, keep_xhat=True)
    m = orc.tensor_metrics(x, cal, fq)
    c = orc.cosine_similarity(x, fq.xhat)
    assert 1.0 - c == pytest.approx(m.mse / (2.0 * fq.sum_x2[0] / x.size), rel=0.05)


# ----------------------------------------------------------------------------
# calibration histograms (Sec. 5) and KL divergence (Sec. 6.1 Eq. 9)
# ----------------------------------------------------------------------------
def test_histogram_pins():
    rng = np.random.default_rng(15)
    # bin midpoints of a power-of-two grid: every element is far from an edge -> equal to numpy exactly
    nb = 256
    mids = ((np.arange(nb) + 0.5) / nb * 8.0 - 4.0).astype(np.float32)
    x = rng.choice(mids, 50_000).astype(np.float32)
    h = orc.histogram(x, -4.0, 4.0, nb)
    assert np.array_equal(h, np.histogram(x, bins=nb, range=(-4.0, 4.0))[0].astype(np.uint64))
    # one element per bin, both range ends included (the maximum lands in the last bin)
    assert orc.histogram(np.concatenate([mids, [-4.0, 4.0]]), -4.0, 4.0, nb).tolist() == \
        [2] + [1] * (nb - 2) + [2]
    # random data: total preserved, numpy agrees except for elements within rounding of an edge
    y = (rng.standard_normal(300_000) * 1.7).astype(np.float32)
    lo, hi = float(y.min()), float(y.max())
    for nbins in (7, 2048, 4096):
        h = orc.histogram(y, lo, hi, nbins)
        ref = np.histogram(y.astype(np.float64), bins=nbins, range=(lo, hi))[0]
        assert int(h.sum()) == y.size
        assert np.abs(np.cumsum(h.astype(np.int64)) - np.cumsum(ref)).max() <= 3
    # brute force on a tiny case with out-of-range values and a degenerate range
    z = np.array([-5.0, -1.0, -0.5, 0.0, 0.24, 0.25, 0.99, 1.0, 7.0], np.float32)
    assert orc.histogram(z, -1.0, 1.0, 8).tolist() == [2, 0, 1, 0, 2, 1, 0, 3]
    assert orc.histogram(z, 2.0, 2.0, 4).tolist() == [9, 0, 0, 0]


def test_kl_divergence_pins():
    from scipy.special import rel_entr
    rng = np.random.default_rng(16)
    p = rng.integers(1, 1000, 64)
    q = rng.integers(1, 1000, 64)
    want = float(rel_entr(p / p.sum(), q / q.sum()).sum())        # library routine
    assert orc.kl_divergence(p, q) == pytest.approx(want, rel=1e-12)
    assert orc.kl_divergence(p, p) == 0.0
    assert orc.kl_divergence(p, 3 * p) == pytest.approx(0.0, abs=1e-15)     # counts are normalised
    assert orc.kl_divergence(p, q) > 0 and orc.kl_divergence(q, p) > 0     # Gibbs
    assert orc.kl_divergence(p, q) != pytest.approx(orc.kl_divergence(q, p), rel=1e-3)   # not symmetric
    # two-bin closed form: P = (1/2, 1/2), Q = (1/4, 3/4)
    assert orc.kl_divergence([2, 2], [1, 3]) == pytest.approx(0.5 * math.log(2) + 0.5 * math.log(2 / 3), rel=1e-14)
    # empty P bins contribute nothing; an empty Q bin under a non-empty P bin gives +inf
    assert orc.kl_divergence([0, 4], [1, 3]) == pytest.approx(math.log(4 / 3), rel=1e-14)
    assert orc.kl_divergence([1, 3], [0, 4]) == math.inf
    # additive smoothing: (c + eps) / (n + eps * bins)
    assert orc.kl_divergence([1, 3], [0, 4], eps=1.0) == pytest.approx(
        (2 / 6) * math.log((2 / 6) / (1 / 6)) + (4 / 6) * math.log((4 / 6) / (5 / 6)), rel=1e-14)
    with pytest.raises(ValueError):
        orc.kl_divergence([1, 2], [1, 2, 3])


# ----------------------------------------------------------------------------
# conv + BN folding (Sec. 6.3 Eq. 10-12) and fusion-aware regrouping (Sec. 6.5)
# ----------------------------------------------------------------------------
def test_bn_fold_pins():
    rng = np.random.default_rng(17)
    w = rng.standard_normal((6, 3, 3, 3)).astype(np.float32)
    gamma = rng.uniform(0.5, 1.5, 6).astype(np.float32)
    var = rng.uniform(0.1, 4.0, 6).astype(np.float32)
    mean = rng.standard_normal(6).astype(np.float32)
    beta = rng.standard_normal(6).astype(np.float32)
    bias = rng.standard_normal(6).astype(np.float32)
    a, c = orc.bn_fold(w, gamma, var, mean, beta, bias)
    # the folded layer computes the same output as conv followed by BN (Eq. 10 vs Eq. 11)
    x = rng.standard_normal(27)
    for ch in range(6):
        conv = float(w[ch].reshape(-1).astype(np.float64) @ x) + float(bias[ch])
        bn = float(gamma[ch]) * (conv - float(mean[ch])) / math.sqrt(float(var[ch])) + float(beta[ch])
        fused = float(a[ch].reshape(-1).astype(np.float64) @ x) + float(c[ch])
        assert fused == pytest.approx(bn, rel=2e-6, abs=2e-6)
    # closed forms: gamma 2, var 4 -> factor exactly 1; gamma 1, var 0.25 -> factor 2
    one = np.ones(3, np.float32)
    a, c = orc.bn_fold(w[:3], 2 * one, 4 * one, 0 * one, 0 * one)
    assert np.array_equal(a, w[:3]) and np.array_equal(c, 0 * one)
    a, c = orc.bn_fold(w[:3], one, 0.25 * one, one, 3 * one, bias=2 * one)
    assert np.array_equal(a, 2 * w[:3]) and c.tolist() == [5.0, 5.0, 5.0]      # 2 * (2 - 1) + 3


def test_regroup_for_fusion():
    order = [4, 1, 5, 0, 3, 2]
    # singleton groups: nothing moves
    assert orc.regroup_for_fusion(order, [0, 1, 2, 3, 4, 5]) == order
    # layers 0 and 1 fuse, 2 and 3 fuse: a block sits where its most sensitive member was
    assert orc.regroup_for_fusion(order, [7, 7, 8, 8, 9, 10]) == [4, 1, 0, 5, 3, 2]
    assert orc.regroup_for_fusion(order, [0, 0, 0, 0, 0, 0]) == order
    rng = np.random.default_rng(18)
    for _ in range(200):
        n = int(rng.integers(1, 40))
        o = list(rng.permutation(n))
        g = list(rng.integers(0, max(1, n // 2), n))
        out = orc.regroup_for_fusion(o, g)
        assert sorted(out) == list(range(n))
        firsts = []
        for l in o:
            if g[l] not in firsts:
                firsts.append(g[l])
        blocks = []
        for l in out:                                   # groups are contiguous, in first-seen order
            if not blocks or blocks[-1] != g[l]:
                blocks.append(g[l])
        assert blocks == firsts
        for gid in firsts:                              # list order kept inside a block
            assert [l for l in out if g[l] == gid] == [l for l in o if g[l] == gid]
    with pytest.raises(ValueError):
        orc.regroup_for_fusion([0, 0], [1, 1])
