"""Pins for the oracle's conv / fc / act / maxpool (CPU only).

The integer results are checked against independent evaluations: float64
library routines on the dequantized values (exact, every partial sum is below
2^53), integer matmul, Python big-integer / Fraction arithmetic, identities
and closed forms.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as F


def _codes(rng, shape, n=16, zero_frac=0.0):
    c = rng.integers(-(1 << (n - 1)), 1 << (n - 1), shape)
    if zero_frac:
        c[rng.random(shape) < zero_frac] = 0
    return c.astype(np.int32)


@pytest.mark.parametrize("N,Cin,H,W,Cout,R,S,stride,pad", [
    (1, 1, 5, 5, 1, 3, 3, 1, 1),
    (2, 3, 7, 6, 4, 3, 3, 1, 1),
    (1, 5, 9, 8, 3, 3, 3, 1, 0),
    (2, 4, 10, 11, 5, 5, 5, 1, 2),
    (1, 2, 12, 12, 3, 7, 7, 1, 3),
    (2, 6, 8, 8, 7, 1, 1, 1, 0),
    (1, 3, 11, 9, 2, 3, 3, 2, 1),
    (1, 2, 9, 9, 2, 3, 5, 2, 2),
])
def test_conv_equals_float64_library_conv_on_real_values(oracle, N, Cin, H, W, Cout, R, S, stride, pad):
    """acc * 2^-(fx+fw) must equal the float64 convolution of the dequantized tensors exactly."""
    rng = np.random.default_rng(N * 1000 + Cin * 100 + R)
    fx, fw = 8, 15
    x, w = _codes(rng, (N, Cin, H, W), zero_frac=0.3), _codes(rng, (Cout, Cin, R, S))
    acc = oracle.conv(x, w, stride=stride, pad=pad)
    real = F.conv2d(torch.from_numpy(x.astype(np.float64) * 2.0 ** -fx),
                    torch.from_numpy(w.astype(np.float64) * 2.0 ** -fw), stride=stride, padding=pad).numpy()
    assert acc.shape == real.shape
    assert np.array_equal(acc.astype(np.float64), real * 2.0 ** (fx + fw))


def test_conv_brute_force_python_integers(oracle):
    """Tiny case recomputed with Python's unbounded integers, index by index."""
    rng = np.random.default_rng(3)
    N, Cin, H, W, Cout = 1, 2, 4, 5, 2
    x, w = _codes(rng, (N, Cin, H, W)), _codes(rng, (Cout, Cin, 3, 3))
    acc = oracle.conv(x, w, pad=1)
    for co in range(Cout):
        for y in range(H):
            for xx in range(W):
                tot = 0
                for ci in range(Cin):
                    for r in range(3):
                        for s in range(3):
                            iy, ix = y + r - 1, xx + s - 1
                            if 0 <= iy < H and 0 <= ix < W:
                                tot += int(x[0, ci, iy, ix]) * int(w[co, ci, r, s])
                assert int(acc[0, co, y, xx]) == tot


def test_conv_delta_kernel_and_shift(oracle):
    """A kernel with a single 1 copies (centre tap) or shifts (corner tap) the input; the
    border that a shift exposes is the zero padding."""
    rng = np.random.default_rng(4)
    x = _codes(rng, (1, 1, 6, 7))
    w = np.zeros((1, 1, 3, 3), np.int32)
    w[0, 0, 1, 1] = 5
    assert np.array_equal(oracle.conv(x, w)[0, 0], 5 * x[0, 0].astype(np.int64))
    w[:] = 0
    w[0, 0, 0, 0] = 1            # out[y,x] = in[y-1,x-1]
    out = oracle.conv(x, w)[0, 0]
    assert np.array_equal(out[1:, 1:], x[0, 0, :-1, :-1]) and not out[0].any() and not out[:, 0].any()
    w[:] = 0
    w[0, 0, 2, 1] = 1            # out[y,x] = in[y+1,x]
    out = oracle.conv(x, w)[0, 0]
    assert np.array_equal(out[:-1], x[0, 0, 1:]) and not out[-1].any()


def test_conv_1x1_is_integer_matmul_and_full_kernel_is_fc(oracle):
    rng = np.random.default_rng(5)
    x, w = _codes(rng, (2, 9, 4, 5)), _codes(rng, (6, 9, 1, 1))
    acc = oracle.conv(x, w, pad=0)
    want = np.einsum("nchw,oc->nohw", x.astype(np.int64), w[:, :, 0, 0].astype(np.int64))
    assert np.array_equal(acc, want)
    # kernel as large as the image, no padding: one output per (n, co) = a dot product = FC
    x, w = _codes(rng, (3, 4, 5, 6)), _codes(rng, (7, 4, 5, 6))
    acc = oracle.conv(x, w, pad=0)
    fc = oracle.fc(x.reshape(3, -1), w.reshape(7, -1))
    assert acc.shape == (3, 7, 1, 1) and np.array_equal(acc[:, :, 0, 0], fc)
    assert np.array_equal(fc, x.reshape(3, -1).astype(np.int64) @ w.reshape(7, -1).astype(np.int64).T)


def test_conv_linear_in_weights_and_bias_alignment(oracle):
    rng = np.random.default_rng(6)
    x = _codes(rng, (1, 3, 6, 6))
    w1, w2 = _codes(rng, (4, 3, 3, 3), n=15), _codes(rng, (4, 3, 3, 3), n=15)
    assert np.array_equal(oracle.conv(x, w1 + w2), oracle.conv(x, w1) + oracle.conv(x, w2))
    bias = _codes(rng, (4,))
    fx, fw, fb = 8, 15, 12
    with_b = oracle.conv(x, w1, bias=bias, f_acc=fx + fw, fb=fb)
    plain = oracle.conv(x, w1)
    # bias * 2^-fb expressed with fx+fw fraction bits
    assert np.array_equal(with_b - plain, np.broadcast_to((bias.astype(np.int64) << (fx + fw - fb))[None, :, None, None], plain.shape))
    with pytest.raises(ValueError):
        oracle.conv(x, w1, bias=bias, f_acc=10, fb=12)     # bias finer than the accumulator


def test_fc_bias_alignment_per_output_column(oracle):
    """LPInnerProduct with the quantized bias blob (Sec. 2.1): bias[o] joins column o of the
    accumulator as bias * 2^(f_acc - fb); checked against an int64 library matmul, with M != Nout
    and distinct bias entries so that a row/column mix-up cannot pass."""
    rng = np.random.default_rng(16)
    M, K, Nout = 5, 37, 9
    x, w = _codes(rng, (M, K)), _codes(rng, (Nout, K))
    bias = (np.arange(Nout, dtype=np.int32) - 4) * 1000 + 7          # all different, both signs
    fx, fw, fb = 9, 15, 11
    got = oracle.fc(x, w, bias=bias, f_acc=fx + fw, fb=fb)
    want = x.astype(np.int64) @ w.astype(np.int64).T + (bias.astype(np.int64) << (fx + fw - fb))[None, :]
    assert got.shape == (M, Nout) and np.array_equal(got, want)
    # fb == f_acc: the bias is added as it is
    assert np.array_equal(oracle.fc(x, w, bias=bias, f_acc=fb, fb=fb) - oracle.fc(x, w),
                          np.broadcast_to(bias.astype(np.int64)[None, :], (M, Nout)))
    # threads only spread the outer loop
    assert np.array_equal(oracle.fc(x, w, bias=bias, f_acc=fx + fw, fb=fb, threads=3), want)
    with pytest.raises(ValueError):
        oracle.fc(x, w, bias=bias, f_acc=10, fb=12)                  # bias finer than the accumulator


def test_extreme_values_need_the_int64_width(oracle):
    """All codes at -32768 over K = 25088: 25088 * 2^30, far beyond int32 and exact in int64."""
    K = 25088
    x = np.full((2, K), -32768, np.int32)
    w = np.full((3, K), -32768, np.int32)
    acc = oracle.fc(x, w)
    assert np.all(acc == K * (1 << 30))
    w[1] = 32767
    assert oracle.fc(x, w)[0, 1] == -32768 * 32767 * K
    # conv with K = 9*512
    xc = np.full((1, 512, 3, 3), 32767, np.int32)
    wc = np.full((1, 512, 3, 3), -32768, np.int32)
    acc = oracle.conv(xc, wc)
    assert acc[0, 0, 1, 1] == 9 * 512 * 32767 * -32768 and acc[0, 0, 0, 0] == 4 * 512 * 32767 * -32768


def test_conv_sampled_and_threads_agree_with_full(oracle):
    rng = np.random.default_rng(7)
    x, w = _codes(rng, (2, 5, 9, 7)), _codes(rng, (6, 5, 3, 3))
    bias = _codes(rng, (6,))
    full = oracle.conv(x, w, bias=bias, f_acc=20, fb=15)
    assert np.array_equal(full, oracle.conv(x, w, bias=bias, f_acc=20, fb=15, threads=4))
    idx = rng.integers(0, full.size, 50)
    assert np.array_equal(oracle.conv_sampled(x, w, idx, bias=bias, f_acc=20, fb=15), full.reshape(-1)[idx])
    with pytest.raises(ValueError):
        oracle.conv_sampled(x, w, np.array([full.size]))


# -------------------------------------------------------------------------- act

def _exact_round(v, s, relu, mode):
    """Round v / 2^s with Fractions (s may be negative); no clipping."""
    if relu and v < 0:
        v = 0
    t = Fraction(v) / (Fraction(2) ** s) if s >= 0 else Fraction(v) * (2 ** -s)
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
    return r


def _exact_act(v, s, n, relu, mode):
    return max(-(1 << (n - 1)), min((1 << (n - 1)) - 1, _exact_round(v, s, relu, mode)))


@pytest.mark.parametrize("s", [1, 2, 8, 15, 23, 30, 0, -3])
@pytest.mark.parametrize("relu", [True, False])
def test_act_against_exact_rational_arithmetic(oracle, s, relu):
    rng = np.random.default_rng(50 + s)
    n, fo = 16, 8
    f_acc = fo + s
    span = 1 << (15 + max(s, 0))
    acc = np.concatenate([
        rng.integers(-2 * span, 2 * span, 400),
        # ties and their neighbours
        (rng.integers(-40000, 40000, 300) * 2 + 1) * (1 << max(s - 1, 0)) + rng.integers(-1, 2, 300),
        np.array([0, 1, -1, span, -span, span - 1, -span - 1, (1 << 61), -(1 << 61)]),
    ]).astype(np.int64)
    for mode, name in ((oracle.ROUND_AWAY, "away"), (oracle.ROUND_EVEN, "even")):
        code, zeros, sats = oracle.act(acc, f_acc, n, n - fo, fo, relu, mode, with_sat=True)
        want = [_exact_act(int(v), s, n, relu, name) for v in acc]
        assert list(code) == want
        assert zeros == want.count(0)
        # clipped = the exactly rounded value lies outside the n-bit code range (Sec. 2.3: the
        # values a format loses); the sample holds values beyond both ends
        unclipped = [_exact_round(int(v), s, relu, name) for v in acc]
        want_sats = sum(1 for r in unclipped if r < -(1 << (n - 1)) or r > (1 << (n - 1)) - 1)
        assert sats == want_sats and want_sats > (0 if relu else 2)


def test_act_closed_form_zero_count(oracle):
    """With ReLU and s > 0 the output is 0 exactly when acc < 2^(s-1) (away) or acc <= 2^(s-1)
    (even); without ReLU (away) when |acc| < 2^(s-1)."""
    rng = np.random.default_rng(60)
    s, fo = 12, 8
    acc = rng.integers(-(1 << 14), 1 << 14, 100000).astype(np.int64)
    acc[:10] = [1 << 11, (1 << 11) - 1, (1 << 11) + 1, -(1 << 11), 0, -1, 1, 3 << 11, -(3 << 11), 5 << 11]
    _, z = oracle.act(acc, fo + s, 16, 8, fo, True, oracle.ROUND_AWAY)
    assert z == int(np.count_nonzero(acc < (1 << 11)))
    _, z = oracle.act(acc, fo + s, 16, 8, fo, True, oracle.ROUND_EVEN)
    assert z == int(np.count_nonzero(acc <= (1 << 11)))
    _, z = oracle.act(acc, fo + s, 16, 8, fo, False, oracle.ROUND_AWAY)
    assert z == int(np.count_nonzero(np.abs(acc) < (1 << 11)))


def test_act_hand_cases(oracle):
    # Q8.8 output from an accumulator with 23 fraction bits (Q8.8 x Q1.15): s = 15
    acc = np.array([1 << 15, (1 << 14), (1 << 14) - 1, 3 << 14, -(1 << 14), -(3 << 14), (32767 << 15) + (1 << 14),
                    -(32768 << 15) - (1 << 14) - 1, 5 << 14], np.int64)
    away, _ = oracle.act(acc, 23, 16, 8, 8, False, oracle.ROUND_AWAY)
    assert list(away) == [1, 1, 0, 2, -1, -2, 32767, -32768, 3]
    even, _ = oracle.act(acc, 23, 16, 8, 8, False, oracle.ROUND_EVEN)
    assert list(even) == [1, 0, 0, 2, 0, -2, 32767, -32768, 2]
    relu, z = oracle.act(acc, 23, 16, 8, 8, True, oracle.ROUND_AWAY)
    assert list(relu) == [1, 1, 0, 2, 0, 0, 32767, 0, 3] and z == 4
    # s <= 0: exact left shift, saturating
    up, _ = oracle.act(np.array([3, -3, 5000, -5000, 4095, -4096]), 5, 16, 8, 8, False, oracle.ROUND_AWAY)
    assert list(up) == [24, -24, 32767, -32768, 32760, -32768]


def test_act_commutes_with_relu_and_matches_quantize(oracle):
    """Quantize-then-ReLU (the order of Sec. 2.1) equals ReLU-then-quantize, and act() on an
    accumulator equals quantize() of the real number it stands for when that is a float32."""
    rng = np.random.default_rng(61)
    acc = rng.integers(-(1 << 23), 1 << 23, 5000).astype(np.int64)
    for mode in (oracle.ROUND_AWAY, oracle.ROUND_EVEN):
        relu_first, _ = oracle.act(acc, 14, 16, 6, 10, True, mode)
        quant_first, _ = oracle.act(acc, 14, 16, 6, 10, False, mode)
        assert np.array_equal(relu_first, np.maximum(quant_first, 0))
        real = (acc.astype(np.float64) * 2.0 ** -14).astype(np.float32)    # exact: |acc| < 2^24
        q, _, _ = oracle.quantize(real, 16, 6, 10, mode)
        assert np.array_equal(quant_first, q)


# ------------------------------------------------------- stochastic rounding in LPAct

@pytest.mark.parametrize("s", [1, 5, 12, 31, 40, 62])
def test_act_stochastic_against_exact_rationals(oracle, s):
    """Sec. 2.4 on accumulators: floor(t) + [u < frac(t)], t = max(acc, 0) / 2^s, decided in exact
    rational arithmetic (Python Fractions; u is a double, hence an exact rational)."""
    from fractions import Fraction
    rng = np.random.default_rng(40 + s)
    fo = 4
    mag = min(61, s + 14)
    acc = rng.integers(-(1 << mag), 1 << mag, 400, dtype=np.int64)
    # remainders next to 0 and next to 2^s, and draws next to the remainder
    special = [0, 1, (1 << s) - 1, 1 << s, (1 << s) + 1, -1, -(1 << s), 3 * (1 << s) - 1]
    special = [v for v in special if abs(v) < (1 << 62)]            # the supported accumulator width
    acc[:len(special)] = special
    u = rng.random(400)
    u[:4] = [0.0, 1.0 - 2.0 ** -53, 0.5, 2.0 ** -40]
    for relu in (True, False):
        code, zeros, sats = oracle.act_stochastic(acc, u, fo + s, 16, 12, fo, relu, with_sat=True)
        want, clipped = [], 0
        for a, uu in zip(acc.tolist(), u.tolist()):
            v = max(a, 0) if relu else a
            t = Fraction(v, 1 << s)
            fl = t.numerator // t.denominator
            r = fl + (1 if Fraction(uu) < t - fl else 0)
            clipped += (r < -32768 or r > 32767)
            want.append(min(max(r, -32768), 32767))
        assert code.tolist() == want
        assert zeros == sum(1 for w in want if w == 0)
        assert sats == clipped


def test_act_stochastic_degenerate_draws_expectation_and_float_quantizer(oracle):
    rng = np.random.default_rng(50)
    acc = rng.integers(-(1 << 20), 1 << 20, 3000, dtype=np.int64)
    s, fo = 9, 6
    fl = acc >> s                                                   # floor division
    on_grid = (acc & ((1 << s) - 1)) == 0
    # u = 0 rounds everything off the grid up, u just below 1 rounds everything down
    up, _ = oracle.act_stochastic(acc, np.zeros(acc.shape), fo + s, 16, 10, fo, False)
    down, _ = oracle.act_stochastic(acc, np.full(acc.shape, 1.0 - 2.0 ** -53), fo + s, 16, 10, fo, False)
    assert np.array_equal(up, np.where(on_grid, fl, fl + 1)) and np.array_equal(down, fl)
    # no rounding to do when the output has at least the accumulator's fraction bits
    c, _ = oracle.act_stochastic(np.array([-3, 0, 5, 40000]), np.array([0.1, 0.9, 0.5, 0.5]), 4, 16, 10, 6, False)
    assert c.tolist() == [-12, 0, 20, 32767]
    # expectation: E[code] = acc / 2^s
    draws = 200000
    a = np.full(draws, 5 * (1 << s) + 333, dtype=np.int64)          # fractional part 333/512
    c, _ = oracle.act_stochastic(a, rng.random(draws), fo + s, 16, 10, fo, True)
    p = 333 / 512
    assert set(np.unique(c).tolist()) == {5, 6}
    assert abs(c.mean() - (5 + p)) < 4 * np.sqrt(p * (1 - p) / draws)
    # an accumulator that is exactly a float (24 significant bits) goes through the float
    # quantizer of the same section to the same code for the same draw
    a = rng.integers(-(1 << 23), 1 << 23, 2000, dtype=np.int64)
    u = rng.random(2000)
    f_acc = 20
    x = (a.astype(np.float64) * 2.0 ** -f_acc).astype(np.float32)   # exact
    via_float, _, _ = oracle.quantize_stochastic(x, u, 16, 8, 8)
    via_acc, _ = oracle.act_stochastic(a, u, f_acc, 16, 8, 8, False)
    assert np.array_equal(via_float, via_acc)
    with pytest.raises(ValueError):
        oracle.act_stochastic(np.array([1]), np.array([1.0]), 12, 16, 8, 8)   # u outside [0, 1)


def test_act_rejects_out_of_range(oracle):
    with pytest.raises(ValueError):
        oracle.act(np.array([1 << 62]), 20, 16, 8, 8)
    with pytest.raises(ValueError):
        oracle.act(np.array([1]), 20, 16, 8, 9)


# ---------------------------------------------------------------------- maxpool

def test_maxpool_against_library(oracle):
    rng = np.random.default_rng(70)
    x = _codes(rng, (2, 3, 8, 6))
    want = F.max_pool2d(torch.from_numpy(x.astype(np.float64)), 2).numpy().astype(np.int32)
    assert np.array_equal(oracle.maxpool2x2(x), want)
    with pytest.raises(ValueError):
        oracle.maxpool2x2(x[:, :, :7])


def test_maxpool_commutes_with_act(oracle):
    """max is monotone, so pooling codes equals requantizing pooled accumulators."""
    rng = np.random.default_rng(71)
    acc = rng.integers(-(1 << 30), 1 << 30, (1, 2, 6, 6)).astype(np.int64)
    code, _ = oracle.act(acc, 23, 16, 8, 8, True)
    pooled_acc = acc.reshape(1, 2, 3, 2, 3, 2).max(axis=(3, 5))
    code2, _ = oracle.act(pooled_acc, 23, 16, 8, 8, True)
    assert np.array_equal(oracle.maxpool2x2(code), code2)


# ------------------------------------------------------------------------ chain

def test_conv_stack_chain_properties():
    """The chain is a composition of pinned steps; check its bookkeeping on a tiny VGG-like net:
    formats sum to n, outputs are non-negative after ReLU, frozen formats reproduce the run,
    sparsity with zero-mean random weights sits near one half."""
    import lp_inputs
    from oracle import vgg

    x = lp_inputs.uniform01((2, 3, 16, 16), seed=9)
    ws = [lp_inputs.he_normal_conv(8, 3, 3, 3, 9, 1), lp_inputs.he_normal_conv(8, 8, 3, 3, 9, 2),
          lp_inputs.he_normal_conv(16, 8, 3, 3, 9, 3)]
    pools = [False, True, True]
    out = vgg.conv_stack(x, ws, pools, n=16, threads=2)
    assert out["mx"] == 1                                   # U(0,1) -> Q1.15
    assert out["final"].shape == (2, 16, 4, 4)
    for L in out["layers"]:
        assert L["mw"] + L["fw"] == 16 and L["mo"] + L["fo"] == 16 and L["mw"] <= 2
        assert L["codes"].min() >= 0
        assert 0.2 < L["zeros"] / L["count"] < 0.8
        # the chosen output format is the tightest one that holds the largest value
        assert L["codes"].max() >= (1 << 14) or L["mo"] == 1
    frozen = [{"mx": out["mx"], "mw": L["mw"], "mo": L["mo"]} for L in out["layers"]]
    again = vgg.conv_stack(x, ws, pools, n=16, formats=frozen)
    assert np.array_equal(again["final"], out["final"])


def test_conv_stack_per_layer_kernel_sizes_and_paddings(oracle):
    """Table 1's Giga1Net mixes kernel sizes 1/7/5/3 with paddings that make the sizes chain up:
    the chain with per-layer paddings must equal the pinned steps composed by hand, layer by layer."""
    import lp_inputs
    from oracle import vgg

    x = lp_inputs.uniform01((2, 3, 20, 20), seed=12)
    ws = [lp_inputs.he_normal_conv(4, 3, 1, 1, 12, 1), lp_inputs.he_normal_conv(6, 4, 7, 7, 12, 2),
          lp_inputs.he_normal_conv(5, 6, 5, 5, 12, 3), lp_inputs.he_normal_conv(7, 5, 3, 3, 12, 4)]
    pools, pads = [True, False, False, True], [0, 1, 1, 1]
    out = vgg.conv_stack(x, ws, pools, n=16, threads=2, pads=pads)
    mx = oracle.range_float(x, 16)[0]
    cur, fx = oracle.quantize(x, 16, mx, 16 - mx)[0], 16 - mx
    for w, pool, pad, L in zip(ws, pools, pads, out["layers"]):
        mw = oracle.range_float(w, 16)[0]
        acc = oracle.conv(cur, oracle.quantize(w, 16, mw, 16 - mw)[0], stride=1, pad=pad)
        assert acc.shape[2] == cur.shape[2] + 2 * pad - w.shape[2] + 1
        mo = oracle.range_acc(acc, fx + 16 - mw, True, 16)[0]
        codes, zeros = oracle.act(acc, fx + 16 - mw, 16, mo, 16 - mo, True, oracle.ROUND_AWAY)
        assert (L["mw"], L["mo"], L["zeros"]) == (mw, mo, zeros) and np.array_equal(L["codes"], codes)
        cur, fx = (oracle.maxpool2x2(codes) if pool else codes), 16 - mo
    assert np.array_equal(out["final"], cur) and out["final"].shape == (2, 7, 2, 2)


def test_fc_stack_equals_hand_composed_steps(oracle):
    """The classifier chain (LPInnerProduct -> LPAct, ReLU on all but the last layer) must equal
    the pinned steps composed by hand, layer by layer, including which layers apply ReLU."""
    import lp_inputs
    from oracle import vgg

    x = lp_inputs.relu_normal((6, 40), seed=13)
    ws = lp_inputs.config5_weights(seed=13, dims=[(40, 24), (24, 24), (24, 10)])
    ws = [w * np.float32(12.0) for w in ws]                       # large enough for non-trivial codes
    relus = [True, True, False]
    out = vgg.fc_stack(x, ws, relus, n=16, threads=2)
    mx = oracle.range_float(x, 16)[0]
    assert out["mx"] == mx
    cur, fx = oracle.quantize(x, 16, mx, 16 - mx)[0], 16 - mx
    assert np.array_equal(out["x_codes"], cur)
    for w, relu, L in zip(ws, relus, out["layers"]):
        mw = oracle.range_float(w, 16)[0]
        wc = oracle.quantize(w, 16, mw, 16 - mw)[0]
        acc = cur.astype(np.int64) @ wc.astype(np.int64).T            # library matmul
        f_acc = fx + 16 - mw
        mo = oracle.range_acc(acc, f_acc, relu, 16)[0]
        codes, zeros = oracle.act(acc, f_acc, 16, mo, 16 - mo, relu, oracle.ROUND_AWAY)
        assert (L["mw"], L["mo"], L["f_acc"], L["zeros"]) == (mw, mo, f_acc, zeros)
        assert np.array_equal(L["acc"], acc) and np.array_equal(L["codes"], codes)
        cur, fx = codes, 16 - mo
    assert np.array_equal(out["final"], cur) and out["final"].shape == (6, 10)
    assert out["layers"][0]["codes"].min() >= 0 and out["final"].min() < 0      # ReLU on fc6/fc7 only
    assert all(L["codes"].any() for L in out["layers"])
