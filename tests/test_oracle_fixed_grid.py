"""Pins of the oracle's paper-literal quantiser Q_{delta,b} (Sec. 2.1, Eq. (1)-(2), Lemma 1)
and of the epoch commit (last step of Alg. 2 / Alg. 3).  CPU only."""
import math
from fractions import Fraction

import numpy as np
import pytest


def outcomes(oracle, v, delta, b):
    return np.array([oracle.fixed_round(v, delta, b, r) for r in range(65536)])


@pytest.mark.parametrize("v,delta,b", [(0.3, 0.25, 4), (-0.3, 0.25, 4), (0.07, 0.01, 8), (-0.0712, 0.01, 8),
                                       (0.9, 1.0, 2), (-1.2, 1.0, 2), (3.3e-4, 1e-5, 8), (-100.7, 1.0, 16),
                                       (0.999999, 1.0, 4), (-1e-9, 1.0, 4)])
def test_eq2_probabilities_exhaustive(oracle, v, delta, b):
    """Inside the range Eq. (2) gives floor with probability (delta*ceil(v/delta) - v)/delta and
    ceil with the rest.  Negative values round toward the same two neighbours (floor is toward
    minus infinity)."""
    k = outcomes(oracle, v, delta, b)
    a = np.float32(v) / np.float32(delta)                  # the oracle forms v/delta in fp32
    lo, hi = math.floor(float(a)), math.floor(float(a)) + 1
    assert set(np.unique(k)) <= {lo, hi}
    # frac(a) = fl(a - floor(a)) is formed in fp32 as well: exact for a >= 0, and for a tiny
    # negative a it rounds up to 1, i.e. "always ceil", 2^-16-close to the exact probability
    T = math.floor(Fraction(float(np.float32(a) - np.float32(lo))) * 65536)
    assert int((k == hi).sum()) == T
    exact = Fraction(float(np.float32(v))) / Fraction(float(np.float32(delta)))
    p_paper = exact - math.floor(exact)                     # (v - delta*floor(v/delta))/delta
    assert abs(Fraction(T, 65536) - p_paper) <= Fraction(1, 65536) + abs(exact) * Fraction(1, 2 ** 23)
    # E[Q(v)] = v inside the range (the cross term in the proof of Lemma 1 vanishes)
    mean = float(k.mean()) * float(np.float32(delta))
    assert abs(mean - v) <= delta * 2.0 ** -16 + abs(v) * 2.0 ** -22


@pytest.mark.parametrize("b", [2, 4, 8, 16])
def test_eq2_clamp_cases(oracle, b):
    delta = 0.5
    top, bottom = 2 ** (b - 1) - 1, -2 ** (b - 1)
    for r in (0, 1, 40000, 65535):
        assert oracle.fixed_round(delta * top, delta, b, r) == top           # the boundary itself
        assert oracle.fixed_round(delta * top + 0.01, delta, b, r) == top
        assert oracle.fixed_round(1e30, delta, b, r) == top
        assert oracle.fixed_round(delta * bottom, delta, b, r) == bottom
        assert oracle.fixed_round(delta * bottom - 0.01, delta, b, r) == bottom
        assert oracle.fixed_round(-1e30, delta, b, r) == bottom
    # just inside the top cell both neighbours occur, never anything above the top
    k = outcomes(oracle, delta * (top - 0.5), delta, b)
    assert set(np.unique(k)) == {top - 1, top}
    k = outcomes(oracle, delta * (bottom + 0.25), delta, b)
    assert set(np.unique(k)) == {bottom, bottom + 1} and int((k == bottom + 1).sum()) == 16384
    # on-grid values never move
    for kk in (bottom, -1, 0, 1, top):
        assert set(outcomes(oracle, delta * kk, delta, b)[::257]) == {kk}


def test_lemma1_both_halves(oracle):
    """Lemma 1: for v on the grid, E(Q(v') - v)^2 <= (v' - v)^2 + delta^2/4; outside the range
    the clamp only moves v' toward the grid: (Q(v') - v)^2 <= (v' - v)^2 for every draw."""
    delta, b = 0.125, 4
    grid = [delta * k for k in range(-8, 8)]
    for vp in (0.3, -0.71, 0.01, 0.8124, -0.99):                       # inside [-1, 0.875]
        k = outcomes(oracle, vp, delta, b).astype(np.float64) * delta
        a = delta * math.ceil(vp / delta)
        var_closed = (a - vp) * (vp - a + delta)                        # proof of Lemma 1
        assert abs(float(((k - vp) ** 2).mean()) - var_closed) <= delta * delta * 2.0 ** -14
        assert var_closed <= delta * delta / 4 + 1e-15
        for v in grid:
            lhs = float(((k - v) ** 2).mean())
            # Lemma 1, with the slack of the variate's 2^-16 resolution in the cross term
            assert lhs <= (vp - v) ** 2 + delta * delta / 4 + 2 * abs(vp - v) * delta * 2.0 ** -16 + 1e-12
            # the cross term vanishes up to the 2^-16 resolution of the variate
            assert abs(lhs - ((vp - v) ** 2 + var_closed)) <= 2 * abs(vp - v) * delta * 2.0 ** -16 + delta * delta * 2.0 ** -14
    for vp in (0.9, 5.0, -1.01, -40.0):                                 # outside the range
        k = outcomes(oracle, vp, delta, b)[::97].astype(np.float64) * delta
        assert len(set(k)) == 1                                         # deterministic clamp
        for v in grid:
            assert (k[0] - v) ** 2 <= (vp - v) ** 2 + 1e-15
        assert k[0] != vp                                               # and therefore biased there


def test_code_words_by_hand(oracle):
    """Two's-complement fields, coordinate i at bit i*b: written out by hand for on-grid inputs
    (on the grid there is no randomness)."""
    delta = 2.0 ** -7
    ks = [-8, -1, 0, 7, 3, -3, 1, -2]
    x = np.array(ks, np.float32) * delta
    assert list(oracle.quantize_fixed(x, delta, 4, 1, 2, 3)) == [0xE1D370F8]
    x = np.array([-128, -1, 127, 5, 1], np.float32) * delta
    assert list(oracle.quantize_fixed(x, delta, 8, 1, 2, 3)) == [0x057FFF80, 0x00000001]
    x = np.array([-2, -1, 0, 1, 1, 1], np.float32) * delta
    assert list(oracle.quantize_fixed(x, delta, 2, 1, 2, 3)) == [0b01_01_01_00_11_10]
    x = np.array([-32768, 32767, -2], np.float32) * delta
    assert list(oracle.quantize_fixed(x, delta, 16, 1, 2, 3)) == [0x7FFF8000, 0x0000FFFE]
    # values far outside land on the end codes
    x = np.array([1e9, -1e9], np.float32)
    assert list(oracle.quantize_fixed(x, delta, 8, 1, 2, 3)) == [0x807F]


@pytest.mark.parametrize("b", [2, 4, 8, 16])
def test_vector_call_keys_variates_on_the_coordinate(oracle, b):
    rng = np.random.default_rng(b)
    d = 203
    delta = 3e-4
    x = (rng.standard_normal(d) * 1e-3).astype(np.float32)
    c = (rng.standard_normal(d) * 1e-3).astype(np.float32)
    codes = oracle.quantize_fixed(x, delta, b, 77, 5, 9, center=c)
    assert codes.size == (d * b + 31) // 32
    v = (x - c).astype(np.float32)
    z, u, zs = oracle.dequantize_fixed_update(codes, d, delta, b, w_snap=c, zsum=np.ones(d, np.float32))
    for i in range(d):
        k = oracle.fixed_round(v[i], delta, b, oracle.uniform16(77, 5, 9, i))
        assert z[i] == np.float32(k) * np.float32(delta)
    assert np.array_equal(u, (c + z).astype(np.float32))
    assert np.array_equal(zs, (np.ones(d, np.float32) + z).astype(np.float32))
    used = (d * b) % 32
    if used:
        assert codes[-1] >> used == 0
    # inside the range the reconstruction error is below one grid step
    inside = np.abs(v) < delta * (2 ** (b - 1) - 1)
    assert np.all(np.abs(z[inside] - v[inside]) <= delta * (1 + 1e-5))


def test_fixed_grid_unbiased_monte_carlo(oracle):
    delta, b = 1e-3, 8
    v = np.array([0.01234, -0.0567, 0.0001, -0.00049, 0.1, 0.0, 0.0999, -0.1277], np.float32)
    n = 20000
    acc = np.zeros(8)
    for seed in range(n):
        z, _, _ = oracle.dequantize_fixed_update(oracle.quantize_fixed(v, delta, b, seed, 0, 0), 8, delta, b)
        acc += z
    assert np.all(np.abs(acc / n - v) <= 5 * delta / (2 * math.sqrt(n)) + delta * 2.0 ** -15)


def test_epoch_commit_and_mean_identity(oracle):
    """w_{t+1} = (1/K_t) sum_{k=0}^{K_t-1} u_{t,k}  (Alg. 2)  ==  w_t + (1/K_t) sum_k z_{t,k}  (Alg. 3),
    with z_{t,0} = 0: the sum runs over the iterates before each step, so the last z is not in it."""
    rng = np.random.default_rng(4)
    d, Kt = 257, 5
    w = rng.standard_normal(d).astype(np.float32)
    zs = [np.zeros(d, np.float32)] + [(rng.standard_normal(d) * 1e-2).astype(np.float32) for _ in range(Kt)]
    zsum = np.zeros(d, np.float32)
    us = []
    for k in range(Kt):                          # iterate k contributes z_{t,k} (z_{t,0} = 0), then steps to z_{t,k+1}
        u_k, zsum = oracle.apply_update(w, zs[k], zsum)
        us.append(u_k.astype(np.float64))
    w_next, z_reset = oracle.epoch_commit(w, zsum, Kt)
    assert not z_reset.any()
    assert np.array_equal(w_next, (w + (zsum / np.float32(Kt)).astype(np.float32)).astype(np.float32))
    alg2 = np.mean(us, axis=0)
    assert np.allclose(w_next, alg2, rtol=0, atol=2.0 ** -21)
    assert not np.allclose(w_next, w + np.mean(zs[1:], axis=0), rtol=0, atol=1e-5)   # shifting the window matters
    # K_t = 1: the epoch returns w_t itself, as Alg. 2 says (the only iterate averaged is u_{t,0} = w_t)
    w1, _ = oracle.epoch_commit(w, np.zeros(d, np.float32), 1)
    assert np.array_equal(w1, w)
