"""GPU parity: lp_quantize, lp_range, lp_range_acc, lp_act, lp_maxpool2x2 against the CPU oracle,
bit for bit, through the C ABI."""
import numpy as np
import pytest
import torch

import lp_inputs
import paper_1711_04713_amd as lp
from gpu_helpers import code_torch_dtype, counter, quantize, to_dev

pytestmark = pytest.mark.gpu


def _mixed_values(count, seed, span):
    """Gaussian body, uniform tails beyond the clip range, exact ties, specials, ~25% zeros."""
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal(count) * span * 0.4).astype(np.float32)
    k = count // 8
    if k:
        x[:k] = rng.uniform(-1.5 * span, 1.5 * span, k).astype(np.float32)
        x[k:2 * k] = ((rng.integers(-70000, 70000, k) + 0.5) * (span / 32768.0)).astype(np.float32)
        x[2 * k:4 * k] = 0.0
    specials = np.array([np.nan, np.inf, -np.inf, 1e-40, -1e-40, 3e38, -3e38, -0.0], np.float32)
    m = min(len(specials), count)
    x[count - m:] = specials[:m]
    return x


@pytest.mark.parametrize("count", [0, 1, 7, 8, 9, 255, 256 * 8 + 3, 100003, 1 << 20])
@pytest.mark.parametrize("q", [(16, 8, 8), (16, 1, 15), (8, 3, 5), (12, 4, 8)])
def test_quantize_matches_oracle(oracle, count, q):
    n, m, f = q
    x = _mixed_values(count, count + n, 2.0 ** (m - 1))
    for mode_gpu, mode_cpu in ((lp.LP_ROUND_NEAREST_AWAY, oracle.ROUND_AWAY), (lp.LP_ROUND_NEAREST_EVEN, oracle.ROUND_EVEN)):
        want, wz, ws = oracle.quantize(x, n, m, f, mode_cpu)
        got, gz, gs = quantize(x, q, mode_gpu)
        assert np.array_equal(got, want)
        assert (gz, gs) == (wz, ws)
    got, _, _ = quantize(x, q, counters=False)       # the no-counter kernel variant
    assert np.array_equal(got, oracle.quantize(x, n, m, f)[0])


def test_quantize_config_tensors(oracle):
    """The tensors of the single-layer and conv1_2-shaped workloads, with formats from lp_range."""
    for x in (*lp_inputs.config1(), *lp_inputs.config2(batch=1, hw=96)):
        fmt, _ = lp.lp_range(to_dev(x.reshape(-1)), 16)
        m, _ = oracle.range_float(x, 16)
        assert fmt.astuple() == (16, m, 16 - m)
        got, gz, gs = quantize(x, fmt.astuple())
        want, wz, ws = oracle.quantize(x, 16, m, 16 - m)
        assert np.array_equal(got, want) and (gz, gs) == (wz, ws)


def test_quantize_rejects_bad_arguments():
    x = torch.zeros(64, device="cuda")
    y = torch.zeros(64, dtype=torch.int16, device="cuda")
    with pytest.raises(lp.LpError):
        lp.lp_quantize(x, y, (16, 8, 9))
    with pytest.raises(lp.LpError):
        lp.lp_quantize(x[1:], y, (16, 8, 8))        # misaligned input
    with pytest.raises(lp.LpError):
        lp.lp_quantize(x, y, (16, 8, 8), r=3)


# ------------------------------------------------------------------ stochastic rounding

def _philox4x32_10(counter, key):
    """The four output words of Philox4x32-10 (Salmon et al., SC'11), written from the published
    round function, vectorised over numpy uint64.  counter: four words (arrays or ints), key: two."""
    mask = np.uint64(0xFFFFFFFF)
    c0, c1, c2, c3 = (np.atleast_1d(np.asarray(c, dtype=np.uint64)) for c in counter)
    c0, c1, c2, c3 = np.broadcast_arrays(c0, c1, c2, c3)
    k0, k1 = np.uint64(key[0]), np.uint64(key[1])
    for _ in range(10):
        p0 = np.uint64(0xD2511F53) * c0
        p1 = np.uint64(0xCD9E8D57) * c2
        c0, c1, c2, c3 = (p1 >> np.uint64(32)) ^ c1 ^ k0, p1 & mask, (p0 >> np.uint64(32)) ^ c3 ^ k1, p0 & mask
        k0 = (k0 + np.uint64(0x9E3779B9)) & mask
        k1 = (k1 + np.uint64(0xBB67AE85)) & mask
    return np.stack([c0, c1, c2, c3], axis=-1)


def _draws(count, seed):
    """The library's draws for elements 0 .. count-1: element i takes word i % 4 of the block with
    counter (i / 4 lo, i / 4 hi, 0, 0) and key (seed lo, seed hi)."""
    blocks = np.arange((count + 3) // 4, dtype=np.uint64)
    words = _philox4x32_10((blocks & np.uint64(0xFFFFFFFF), blocks >> np.uint64(32), 0, 0),
                           (seed & 0xFFFFFFFF, seed >> 32))
    return words.reshape(-1)[:count]


def test_philox_known_answers():
    """The generator's published known-answer vectors: zero counter and key, all ones, and the
    digits of pi."""
    kat = [((0, 0, 0, 0), (0, 0), (0x6627E8D5, 0xE169C58D, 0xBC57AC4C, 0x9B00DBD8)),
           ((0xFFFFFFFF,) * 4, (0xFFFFFFFF,) * 2, (0x408F276D, 0x41C83B0E, 0xA20BC7C6, 0x6D5451FD)),
           ((0x243F6A88, 0x85A308D3, 0x13198A2E, 0x03707344), (0xA4093822, 0x299F31D0),
            (0xD16CFE09, 0x94FDCCEB, 0x5001E420, 0x24126EA1))]
    for counter, key, want in kat:
        assert tuple(int(w) for w in _philox4x32_10(counter, key)[0]) == want
    # the element-to-word map: elements 0..3 are the four words of block 0
    assert tuple(int(w) for w in _draws(4, 0)) == kat[0][2]
    assert int(_draws(6, 0)[5]) == int(_philox4x32_10((1, 0, 0, 0), (0, 0))[0][1])


@pytest.mark.parametrize("q", [(16, 8, 8), (8, 2, 6)])
def test_quantize_stochastic_matches_oracle(oracle, q):
    n, m, f = q
    count = 70001
    x = _mixed_values(count, 77, 2.0 ** (m - 1))
    seed = 0x1234567ABCDEF01
    u = _draws(count, seed).astype(np.float64) * 2.0 ** -32
    want, wz, ws = oracle.quantize_stochastic(x, u, n, m, f)
    got, gz, gs = quantize(x, q, lp.LP_ROUND_STOCHASTIC, seed=seed)
    assert np.array_equal(got, want) and (gz, gs) == (wz, ws)
    other, _, _ = quantize(x, q, lp.LP_ROUND_STOCHASTIC, seed=seed + 1)
    assert not np.array_equal(other, got)


def test_quantize_stochastic_fraction_needs_more_than_float32(oracle):
    """t = x * 2^f = -0.25 + 2^-26 has the fractional part 0.75 + 2^-26, which float32 cannot
    hold; with a draw in [0.75, 0.75 + 2^-26) the exact decision is "up".  Seed and index were
    found by searching the test-side generator for a draw in that window."""
    seed, index, f = 15080025, 7, 8
    w = int(_draws(64, seed)[index])
    assert 3 << 30 <= w < (3 << 30) + 64                    # the draw sits in the window
    t = np.float32(-0.25) + np.float32(2.0 ** -26)
    assert float(t) == -0.25 + 2.0 ** -26                   # representable
    x = np.zeros(64, np.float32)
    x[index] = t * np.float32(2.0 ** -f)
    u = _draws(64, seed).astype(np.float64) * 2.0 ** -32
    want, _, _ = oracle.quantize_stochastic(x, u, 16, 8, f)
    assert want[index] == 0                                 # floor is -1, rounded up
    got, _, _ = quantize(x, (16, 8, f), lp.LP_ROUND_STOCHASTIC, seed=seed)
    assert np.array_equal(got, want)


# --------------------------------------------------------------------------------- range

@pytest.mark.parametrize("count", [0, 1, 3, 4, 5, 1000, 262147])
@pytest.mark.parametrize("scale", [0.01, 1.0, 300.0, 1e6])
def test_range_matches_oracle(oracle, count, scale):
    rng = np.random.default_rng(count)
    x = (rng.standard_normal(count) * scale).astype(np.float32)
    if count > 4:
        x[1] = np.nan
        x[2] = 2.0 ** 3           # exactly a power of two
    for n in (16, 8):
        for thr in (0.0, 0.01, 0.3):
            fmt, lost = lp.lp_range(to_dev(x), n, thr)
            if count == 0:
                assert fmt.astuple() == (n, 1, n - 1)
                continue
            m, want_lost = oracle.range_float(x, n, thr)
            assert fmt.astuple() == (n, m, n - m)
            assert lost[1:] == [int(v) for v in want_lost[1:]]


def test_range_infinity_is_always_lost(oracle):
    x = np.array([0.5, np.inf, -0.25, 0.0], np.float32)
    fmt, lost = lp.lp_range(to_dev(x), 16, 0.0)
    assert fmt.m == 16 and lost[16] == 1
    assert oracle.range_float(x, 16, 0.0)[0] == 16


@pytest.mark.parametrize("count", [1, 2, 3, 1001, 200000])
@pytest.mark.parametrize("f_acc,relu", [(0, False), (23, True), (27, False), (30, True)])
def test_range_acc_matches_oracle(oracle, count, f_acc, relu):
    rng = np.random.default_rng(count + f_acc)
    acc = (rng.standard_normal(count) * 2.0 ** (f_acc + 3)).astype(np.int64)
    acc[0] = 1 << (f_acc + 2)
    if count > 2:
        acc[1] = -(1 << 50)
    for thr in (0.0, 0.02):
        fmt, lost = lp.lp_range_acc(to_dev(acc), f_acc, relu, 16, thr)
        m, want_lost = oracle.range_acc(acc, f_acc, relu, 16, thr)
        assert fmt.astuple() == (16, m, 16 - m)
        assert lost[1:] == [int(v) for v in want_lost[1:]]


# ----------------------------------------------------------------------------------- act

@pytest.mark.parametrize("count", [0, 1, 8, 13, 4099, 300007])
@pytest.mark.parametrize("f_acc,qy,relu", [
    (23, (16, 8, 8), True), (27, (16, 4, 12), True), (27, (16, 4, 12), False), (30, (16, 1, 15), True),
    (12, (8, 3, 5), True), (5, (16, 8, 8), False), (8, (16, 8, 8), True), (40, (16, 14, 2), False),
])
def test_act_matches_oracle(oracle, count, f_acc, qy, relu):
    n, m, fo = qy
    s = f_acc - fo
    rng = np.random.default_rng(count * 7 + f_acc)
    acc = (rng.standard_normal(count) * 2.0 ** (max(s, 0) + n - 2)).astype(np.int64)
    k = count // 4
    if k and s > 0:   # exact ties
        acc[:k] = (rng.integers(-40000, 40000, k) * 2 + 1) * (1 << (s - 1))
    for mode_gpu, mode_cpu in ((lp.LP_ROUND_NEAREST_AWAY, oracle.ROUND_AWAY), (lp.LP_ROUND_NEAREST_EVEN, oracle.ROUND_EVEN)):
        want, wz, wsat = oracle.act(acc, f_acc, n, m, fo, relu, mode_cpu, with_sat=True)
        y = torch.empty(count, dtype=code_torch_dtype(n), device="cuda")
        z, sat = counter(), counter()
        lp.lp_act(to_dev(acc), f_acc, qy, relu, y, mode_gpu, z, sat)
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy().astype(np.int32), want)
        assert (int(z.item()), int(sat.item())) == (wz, wsat)
        if count > 4000:
            assert wsat > 0                              # the sample does reach past the code range
            sat_only = counter()                         # the clipped-value counter on its own
            lp.lp_act(to_dev(acc), f_acc, qy, relu, y, mode_gpu, None, sat_only)
            torch.cuda.synchronize()
            assert int(sat_only.item()) == wsat


def test_act_extremes(oracle):
    acc = np.array([(1 << 62) - 1, -(1 << 62) + 1, 0, 1, -1, 1 << 40, -(1 << 40), (1 << 22), (1 << 22) - 1], np.int64)
    want, wz, wsat = oracle.act(acc, 23, 16, 8, 8, False, oracle.ROUND_AWAY, with_sat=True)
    y = torch.empty(len(acc), dtype=torch.int16, device="cuda")
    z, sat = counter(), counter()
    lp.lp_act(to_dev(acc), 23, (16, 8, 8), False, y, zero_count=z, sat_count=sat)
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy().astype(np.int32), want) and int(z.item()) == wz
    assert int(sat.item()) == wsat == 4                  # the two ends of the width and +-2^40


@pytest.mark.parametrize("count,f_acc,qy,relu", [
    (0, 23, (16, 8, 8), True), (1, 23, (16, 8, 8), True), (9, 23, (16, 8, 8), False),
    (4099, 27, (16, 4, 12), True), (70001, 27, (16, 4, 12), False), (33000, 12, (8, 3, 5), True),
    (5000, 50, (16, 8, 8), False), (5000, 64, (16, 14, 2), True), (3000, 5, (16, 8, 8), False),
])
def test_act_stochastic_matches_oracle(oracle, count, f_acc, qy, relu):
    """Stochastic rounding of accumulators (Sec. 2.4): the draws are the generator's words for
    the element indices, fed to the oracle as numbers; shifts below and above 32 bits, a shift
    of 62, and an output finer than the accumulator (nothing to round)."""
    n, m, fo = qy
    s = f_acc - fo
    rng = np.random.default_rng(count * 11 + f_acc)
    mag = min(61, max(s, 0) + n - 2)
    acc = rng.integers(-(1 << mag), 1 << mag, count, dtype=np.int64) if count else np.zeros(0, np.int64)
    if count > 8 and 0 < s <= 60:
        acc[:4] = [0, (1 << s) - 1, 1 << s, -1]           # remainders 0, 2^s - 1, 0, 2^s - 1
    seed = 0xC0FFEE1234567
    u = _draws(count, seed).astype(np.float64) * 2.0 ** -32
    want, wz, wsat = oracle.act_stochastic(acc, u, f_acc, n, m, fo, relu, with_sat=True)
    y = torch.empty(count, dtype=code_torch_dtype(n), device="cuda")
    z, sat = counter(), counter()
    lp.lp_act_stochastic(to_dev(acc), f_acc, qy, relu, seed, y, z, sat)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.int32)
    assert np.array_equal(got, want) and (int(z.item()), int(sat.item())) == (wz, wsat)
    if count > 1000 and s > 0:
        y2 = torch.empty(count, dtype=code_torch_dtype(n), device="cuda")
        lp.lp_act_stochastic(to_dev(acc), f_acc, qy, relu, seed + 1, y2)
        torch.cuda.synchronize()
        assert not np.array_equal(y2.cpu().numpy().astype(np.int32), got)      # the seed matters
    if s <= 0 and count:
        y3 = torch.empty(count, dtype=code_torch_dtype(n), device="cuda")
        lp.lp_act(to_dev(acc), f_acc, qy, relu, y3)
        torch.cuda.synchronize()
        assert torch.equal(y3, y)


def test_act_stochastic_after_conv_accumulators(oracle):
    """The unfused route for a layer with stochastic rounding: lp_conv_fwd's exact accumulators,
    then lp_act_stochastic, against the oracle's conv followed by its stochastic act."""
    from gpu_helpers import conv
    rng = np.random.default_rng(91)
    x = rng.integers(0, 3000, (2, 64, 12, 12)).astype(np.int32)
    w = rng.integers(-3000, 3000, (64, 64, 3, 3)).astype(np.int32)
    qx, qw, qy = (16, 4, 12), (16, 1, 15), (16, 6, 10)
    got = conv(x, qx, w, qw, qy=qy)
    want_acc = oracle.conv(x, w, threads=8)
    assert np.array_equal(got["acc"], want_acc)
    acc_nhwc = np.ascontiguousarray(want_acc.transpose(0, 2, 3, 1))
    seed = 77
    u = _draws(acc_nhwc.size, seed).astype(np.float64) * 2.0 ** -32
    want, wz = oracle.act_stochastic(acc_nhwc.reshape(-1), u, 27, *qy, True)
    acc_dev = to_dev(np.ascontiguousarray(got["acc"].transpose(0, 2, 3, 1)).reshape(-1))
    y = torch.empty(acc_nhwc.size, dtype=torch.int16, device="cuda")
    z = counter()
    lp.lp_act_stochastic(acc_dev, 27, qy, True, seed, y, z)
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy().astype(np.int32), want) and int(z.item()) == wz


# ------------------------------------------------------------------------------- maxpool

@pytest.mark.parametrize("N,C,H,W,n", [(1, 8, 2, 2, 16), (2, 64, 8, 12, 16), (3, 24, 6, 4, 16), (2, 5, 4, 6, 16),
                                       (2, 32, 8, 8, 8), (1, 7, 4, 4, 8), (2, 128, 28, 28, 16)])
def test_maxpool_matches_oracle(oracle, N, C, H, W, n):
    rng = np.random.default_rng(N * C + H)
    x = rng.integers(-(1 << (n - 1)), 1 << (n - 1), (N, C, H, W)).astype(np.int32)
    want = oracle.maxpool2x2(x)
    dt = np.int16 if n > 8 else np.int8
    xd = to_dev(x.transpose(0, 2, 3, 1).astype(dt))
    yd = torch.empty((N, H // 2, W // 2, C), dtype=code_torch_dtype(n), device="cuda")
    lp.lp_maxpool2x2(xd, yd, N, H, W, C, n)
    torch.cuda.synchronize()
    assert np.array_equal(yd.cpu().numpy().astype(np.int32).transpose(0, 3, 1, 2), want)
    with pytest.raises(lp.LpError):
        lp.lp_maxpool2x2(xd, yd, N, H + 1, W, C, n)
