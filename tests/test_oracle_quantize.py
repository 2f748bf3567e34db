"""Pins for the oracle's quantizer and range rule (CPU only).

Nothing here re-types the oracle's formula: the checks are hand-worked values
(tests/golden), exact rational arithmetic with fractions.Fraction, grid
invariants, exhaustive enumeration and closed forms.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden", "qmf_rounding_cases.txt")


def _cases():
    out = []
    with open(GOLD) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if not line:
                continue
            n, m, f, v, away, even = line.split()
            out.append((int(n), int(m), int(f), float(v), int(away), int(even)))
    return out


def test_golden_file_has_cases():
    assert len(_cases()) >= 45


@pytest.mark.parametrize("n,m,f,v,away,even", _cases())
def test_hand_worked_cases(oracle, n, m, f, v, away, even):
    code, _, _ = oracle.quantize(np.array([v], np.float32), n, m, f, oracle.ROUND_AWAY)
    assert code[0] == away
    code, _, _ = oracle.quantize(np.array([v], np.float32), n, m, f, oracle.ROUND_EVEN)
    assert code[0] == even


def _exact_round(x32, f, n, mode):
    """Round the exact rational x * 2^f with Python integers (no floating point)."""
    t = Fraction(float(x32)) * (Fraction(2) ** f)
    fl = t.numerator // t.denominator
    frac = t - fl
    if frac > Fraction(1, 2):
        r = fl + 1
    elif frac < Fraction(1, 2):
        r = fl
    elif mode == "away":
        r = fl + 1 if t > 0 else fl
    else:
        r = fl if fl % 2 == 0 else fl + 1
    return max(-(1 << (n - 1)), min((1 << (n - 1)) - 1, r))


@pytest.mark.parametrize("n,m", [(16, 8), (16, 1), (16, 4), (16, 16), (8, 1), (8, 3), (12, 5), (2, 1), (3, 2)])
def test_against_exact_rational_arithmetic(oracle, n, m):
    f = n - m
    rng = np.random.default_rng(100 * n + m)
    span = 2.0 ** (m - 1)
    x = np.concatenate([
        rng.standard_normal(300).astype(np.float32) * np.float32(span / 2),
        rng.uniform(-1.2 * span, 1.2 * span, 300).astype(np.float32),
        # exact ties and near-ties around random grid points
        ((rng.integers(-(1 << (n - 1)) - 3, (1 << (n - 1)) + 3, 300) + 0.5) * 2.0 ** -f).astype(np.float32),
        np.array([0.0, -0.0, 1e-30, -1e-30, 1e30, -1e30, np.inf, -np.inf], np.float32),
    ])
    for mode, name in ((oracle.ROUND_AWAY, "away"), (oracle.ROUND_EVEN, "even")):
        code, _, _ = oracle.quantize(x, n, m, f, mode)
        for xi, ci in zip(x, code):
            if math.isinf(float(xi)):
                want = (1 << (n - 1)) - 1 if xi > 0 else -(1 << (n - 1))
            else:
                want = _exact_round(xi, f, n, name)
            assert ci == want, (float(xi), n, m, f, name)


def test_nan_maps_to_zero(oracle):
    code, z, s = oracle.quantize(np.array([np.nan, 1.0], np.float32), 16, 8, 8)
    assert list(code) == [0, 256] and z == 1 and s == 0


@pytest.mark.parametrize("n,m", [(16, 8), (16, 1), (8, 2), (5, 3)])
def test_grid_invariants(oracle, n, m):
    """Dequantized codes are multiples of 2^-f inside [-2^(m-1), 2^(m-1)-2^-f]; the
    error is at most half a step when nothing saturates; the map is monotone and idempotent."""
    f = n - m
    rng = np.random.default_rng(n * 31 + m)
    x = np.sort((rng.standard_normal(20000) * 2.0 ** (m - 1) * 0.7).astype(np.float32))
    for mode in (oracle.ROUND_AWAY, oracle.ROUND_EVEN):
        code, zeros, sats = oracle.quantize(x, n, m, f, mode)
        deq = code.astype(np.float64) * 2.0 ** -f
        assert deq.min() >= -(2.0 ** (m - 1)) and deq.max() <= 2.0 ** (m - 1) - 2.0 ** -f
        assert np.all(code == np.round(deq * 2.0 ** f))            # integer multiples of the step
        assert np.all(np.diff(code) >= 0)                           # monotone
        inside = (x.astype(np.float64) >= -(2.0 ** (m - 1)) - 2.0 ** -(f + 1)) & \
                 (x.astype(np.float64) < 2.0 ** (m - 1) - 2.0 ** -(f + 1))
        assert np.all(np.abs(deq[inside] - x[inside].astype(np.float64)) <= 2.0 ** -(f + 1))
        again, _, _ = oracle.quantize(deq.astype(np.float32), n, m, f, mode)
        assert np.array_equal(again, code)                          # idempotent
        assert zeros == int(np.count_nonzero(code == 0))
        clipped = (x.astype(np.float64) * 2.0 ** f >= 2.0 ** (n - 1) - 0.5) | \
                  (x.astype(np.float64) * 2.0 ** f < -(2.0 ** (n - 1)) - 0.5)
        # a tie exactly at the lower clip edge rounds to the edge under 'even'; none is drawn here
        assert sats == int(np.count_nonzero(clipped))


def test_exhaustive_grid_and_midpoints_q8_8(oracle):
    """Every grid point of Q8.8 maps to itself; every midpoint goes to the neighbour the mode names."""
    q = np.arange(-32768, 32768, dtype=np.int64)
    grid = (q * 2.0 ** -8).astype(np.float32)
    for mode in (oracle.ROUND_AWAY, oracle.ROUND_EVEN):
        code, _, _ = oracle.quantize(grid, 16, 8, 8, mode)
        assert np.array_equal(code, q)
    mid = ((q[:-1] + 0.5) * 2.0 ** -8).astype(np.float32)          # between q and q+1, exact in float32
    away, _, _ = oracle.quantize(mid, 16, 8, 8, oracle.ROUND_AWAY)
    assert np.array_equal(away, np.where(q[:-1] >= 0, q[:-1] + 1, q[:-1]))
    even, _, _ = oracle.quantize(mid, 16, 8, 8, oracle.ROUND_EVEN)
    assert np.array_equal(even, np.where(q[:-1] % 2 == 0, q[:-1], q[:-1] + 1))


def test_rejects_bad_formats(oracle):
    x = np.zeros(4, np.float32)
    for n, m, f in [(16, 8, 7), (16, 0, 16), (17, 1, 16), (1, 1, 0), (8, 9, -1)]:
        with pytest.raises(ValueError):
            oracle.quantize(x, n, m, f)


# ------------------------------------------------------------ stochastic rounding

def test_stochastic_two_point_support_and_threshold(oracle):
    """Sec. 2.4: the result is one of the two neighbouring grid points, the upper one exactly
    when the uniform draw is below the fractional part."""
    rng = np.random.default_rng(5)
    x = (rng.standard_normal(5000) * 3).astype(np.float32)
    u = rng.random(5000)
    code, _, _ = oracle.quantize_stochastic(x, u, 16, 8, 8)
    t = x.astype(np.float64) * 256.0
    fl = np.floor(t)
    assert np.all((code == fl) | (code == fl + 1))
    assert np.array_equal(code == fl + 1, (u < (t - fl)))
    # grid points never move, whatever the draw
    g = (np.arange(-500, 500) / 256.0).astype(np.float32)
    for uu in (0.0, 0.5, 0.999999):
        c, _, _ = oracle.quantize_stochastic(g, np.full(g.shape, uu), 16, 8, 8)
        assert np.array_equal(c, np.arange(-500, 500))


def test_stochastic_expectation(oracle):
    """Correct expectation: averaging over many draws recovers the input to ~1/sqrt(draws) of a step."""
    rng = np.random.default_rng(6)
    x = np.float32(0.7 / 256 + 3.0)            # fractional part 0.7 of a Q8.8 step
    draws = 200000
    code, _, _ = oracle.quantize_stochastic(np.full(draws, x, np.float32), rng.random(draws), 16, 8, 8)
    mean = code.mean() / 256.0
    assert abs(mean - float(x)) < 4 * math.sqrt(0.21 / draws) / 256.0
    # saturation still applies
    c, _, s = oracle.quantize_stochastic(np.array([500.0, -500.0], np.float32), np.array([0.3, 0.3]), 16, 8, 8)
    assert list(c) == [32767, -32768] and s == 2


# ------------------------------------------------------------------------ range

def _closed_form_m(maxabs, n):
    """threshold 0: m = 1 if max|v| < 1, else floor(log2 max|v|) + 2, capped at n."""
    if maxabs < 1.0:
        return 1
    return min(n, math.frexp(maxabs)[1] + 1)   # frexp exponent e: 2^(e-1) <= maxabs < 2^e


@pytest.mark.parametrize("maxabs,want", [
    (0.0, 1), (0.3, 1), (0.999999, 1), (1.0, 2), (1.5, 2), (1.9999, 2), (2.0, 3), (3.99, 3),
    (4.0, 4), (100.0, 8), (127.99, 8), (128.0, 9), (16383.0, 15), (16384.0, 16), (1e9, 16),
])
def test_range_threshold_zero_special_cases(oracle, maxabs, want):
    """max just below 2^k needs m = k+1, max exactly 2^k needs m = k+2 (Sec. 2.3: the integer
    part is checked against the largest number present)."""
    v = np.array([0.1, -maxabs, 0.0, maxabs / 2], np.float32)
    m, _ = oracle.range_float(v, 16, 0.0)
    assert m == want == _closed_form_m(float(np.float32(maxabs)), 16)
    m2, _ = oracle.range_float(-v, 16, 0.0)
    assert m2 == want


def test_range_brute_force_with_threshold(oracle):
    rng = np.random.default_rng(11)
    for trial in range(40):
        n = int(rng.integers(2, 17))
        v = (rng.standard_normal(int(rng.integers(1, 400))) * float(rng.choice([0.05, 1.0, 30.0, 5000.0]))).astype(np.float32)
        thr = float(rng.choice([0.0, 0.01, 0.1, 0.5]))
        m, lost = oracle.range_float(v, n, thr)
        # brute force with Python numbers, from the words of Sec. 2.3: shrink the integer part
        # while the share of values that no longer fit stays within the threshold
        want = n
        for mm in range(n, 0, -1):
            cnt = sum(1 for t in v if abs(float(t)) >= 2.0 ** (mm - 1))
            assert lost[mm] == cnt
            if cnt <= thr * len(v):
                want = mm
            else:
                break
        assert m == want
        assert np.all(np.diff(lost[1:].astype(np.int64)) <= 0)   # fewer lost with more integer bits


def test_range_gaussian_weights_need_at_most_two_integer_bits(oracle):
    """Sec. 3.1: for weights two integer bits (sign included) are usually enough."""
    import lp_inputs

    for w in lp_inputs.vgg16_conv_weights(seed=2, layers=["conv1_1", "conv1_2", "conv3_1"]):
        m, _ = oracle.range_float(w, 16, 0.0)
        assert m <= 2


def test_range_acc_matches_float_rule_on_exact_values(oracle):
    """Accumulators acc * 2^-f_acc with |acc| < 2^24 are exact float32 values, so the integer rule
    must agree with the float rule on them; with ReLU negatives never count."""
    rng = np.random.default_rng(12)
    for f_acc in (0, 7, 20):
        acc = rng.integers(-(1 << 23), 1 << 23, 2000)
        v = (acc.astype(np.float64) * 2.0 ** -f_acc).astype(np.float32)
        for thr in (0.0, 0.05):
            m_i, lost_i = oracle.range_acc(acc, f_acc, False, 16, thr)
            m_f, lost_f = oracle.range_float(v, 16, thr)
            assert m_i == m_f and np.array_equal(lost_i, lost_f)
            m_r, lost_r = oracle.range_acc(acc, f_acc, True, 16, thr)
            m_p, lost_p = oracle.range_float(np.maximum(v, 0), 16, thr)
            assert m_r == m_p and np.array_equal(lost_r, lost_p)
    # wide accumulators: 2^45 with 30 fraction bits is 2^15 -> needs m = 17 > n -> capped at n
    m, lost = oracle.range_acc(np.array([1 << 45, -(1 << 44)]), 30, False, 16, 0.0)
    assert m == 16 and lost[16] == 1
    m, _ = oracle.range_acc(np.array([(1 << 44) - 1]), 30, True, 16, 0.0)
    assert m == 15
