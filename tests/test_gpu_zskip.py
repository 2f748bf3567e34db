"""GPU parity of zero-tile skipping (lp_conv_fwd_zskip): layers leave per-tile nonzero flags, the
next layer skips input chunks flagged all-zero; codes and counters must equal the oracle's (which
knows nothing of skipping) bit for bit, the flags must equal what the oracle's codes imply, and on
inputs with structured sparsity chunks must really be skipped."""
import numpy as np
import pytest
import torch

import lp_inputs
import paper_1711_04713_amd as lp
from gpu_helpers import to_dev
from oracle import vgg as ovgg
from paper_1711_04713_amd.stack import ConvStack

pytestmark = pytest.mark.gpu

QX, QW, QY = (16, 4, 12), (16, 1, 15), (16, 5, 11)


def _nhwc(a):
    return to_dev(np.ascontiguousarray(a.transpose(0, 2, 3, 1)))


def _expected_flags(codes_nchw, info):
    """flag[pixel tile][channel tile] = the tile of the LPAct output holds a nonzero code."""
    N, C, H, W = codes_nchw.shape
    rh, tw, bn = info["tile_rows"], info["tile_cols"], info["bn"]
    stacked = codes_nchw.transpose(0, 2, 3, 1).reshape(N * H, W, C)          # stacked output rows
    tiles_r, tiles_c, tiles_n = -(-N * H // rh), -(-W // tw), info["tiles_n"]
    assert tiles_r * tiles_c == info["tiles_m"]
    out = np.zeros((tiles_r, tiles_c, tiles_n), np.uint8)
    for r in range(tiles_r):
        for c in range(tiles_c):
            for n in range(tiles_n):
                out[r, c, n] = stacked[r * rh:(r + 1) * rh, c * tw:(c + 1) * tw, n * bn:(n + 1) * bn].any()
    return out.reshape(-1)


def _layer(x_codes, w_codes, qx, qw, qy, x_map=None, pool=0):
    N, Cin, H, W = x_codes.shape
    Cout, _, R, S = w_codes.shape
    d = lp.ConvDesc(N, H, W, Cin, Cout, R, S, 1, R // 2, pool)
    dt = np.int16 if qx[0] > 8 else np.int8
    xd = to_dev(x_codes.transpose(0, 2, 3, 1).astype(dt))
    wd = to_dev(w_codes.transpose(0, 2, 3, 1).astype(np.int16 if qw[0] > 8 else np.int8))
    packed = torch.empty(lp.lp_conv_packed_bytes(d, qx, qw), dtype=torch.uint8, device="cuda")
    lp.lp_conv_pack_weights(d, qx, qw, wd, packed)
    info = lp.lp_conv_plan_info(d, qx, qw)
    y = torch.full((N, H >> pool, W >> pool, Cout), -7, dtype=torch.int16 if qy[0] > 8 else torch.int8, device="cuda")
    z, s, k = (torch.zeros(1, dtype=torch.int64, device="cuda") for _ in range(3))
    flags = torch.full((info["tiles_m"] * info["tiles_n"],), 7, dtype=torch.uint8, device="cuda")
    ws = torch.full((max(lp.lp_conv_workspace_bytes(d, qx, qw), 16),), 0xA5, dtype=torch.uint8, device="cuda")
    lp.lp_conv_fwd_zskip(d, xd, qx, x_map, packed, qw, qy, y, zero_count=z, sat_count=s, y_flags=flags, skipped=k,
                         workspace=ws)
    torch.cuda.synchronize()
    return {"y": y, "y_np": y.cpu().numpy().astype(np.int32).transpose(0, 3, 1, 2), "zeros": int(z.item()),
            "sats": int(s.item()), "skipped": int(k.item()), "flags": flags, "info": info, "W": W}


def _sparse_pair(rng, N, C0, H, W, C1, C2, n=16):
    """Layer-1 input with all-zero regions and layer-1 weights whose upper output channels cannot
    fire (negative weights on non-negative input): whole tiles and whole channel tiles of the
    layer-1 output are zero, while the rest is ordinary."""
    hi = 1 << (n - 3)
    x = rng.integers(0, hi, (N, C0, H, W)).astype(np.int32)
    x[:, :, :, W // 2:] = 0                                   # right half of every image is blank
    x[N // 2:] = 0                                            # and so are the later images altogether
    w1 = rng.integers(-hi, hi, (C1, C0, 3, 3)).astype(np.int32)
    w1[C1 // 2:] = -np.abs(w1[C1 // 2:]) - 1                  # these channels are always <= 0 before ReLU
    w2 = rng.integers(-hi, hi, (C2, C1, 3, 3)).astype(np.int32)
    return x, w1, w2


@pytest.mark.parametrize("shape,pool", [((4, 64, 24, 32, 128, 64), 0), ((4, 64, 24, 32, 256, 96), 1),
                                        ((6, 128, 16, 16, 192, 64), 0), ((2, 64, 12, 12, 256, 64), 0),
                                        ((24, 64, 64, 64, 128, 128), 0), ((24, 64, 64, 64, 128, 128), 1)])
def test_two_layers_with_structured_zeros(oracle, shape, pool):
    N, C0, H, W, C1, C2 = shape
    rng = np.random.default_rng(sum(shape))
    x, w1, w2 = _sparse_pair(rng, N, C0, H, W, C1, C2)
    acc1 = oracle.conv(x, w1, threads=8)
    y1, z1, s1 = oracle.act(acc1, 27, *QY, True, oracle.ROUND_AWAY, with_sat=True)
    a = _layer(x, w1, QX, QW, QY, pool=pool)
    want1 = oracle.maxpool2x2(y1) if pool else y1
    assert np.array_equal(a["y_np"], want1) and (a["zeros"], a["sats"]) == (z1, s1)
    flags = a["flags"].cpu().numpy()
    assert np.array_equal(flags, _expected_flags(y1, a["info"]))               # flags describe the unpooled codes
    assert 0 < flags.sum() < flags.size
    # second layer on the first one's codes, told which of its input tiles are blank
    qx2 = QY
    x_map = lp.zero_map(a["flags"], a["info"], a["W"], 2 if pool else 1)
    b = _layer(want1, w2, qx2, QW, (16, 9, 7), x_map=x_map)
    acc2 = oracle.conv(want1, w2, threads=8)
    y2, z2, s2 = oracle.act(acc2, qx2[2] + QW[2], 16, 9, 7, True, oracle.ROUND_AWAY, with_sat=True)
    assert np.array_equal(b["y_np"], y2) and (b["zeros"], b["sats"]) == (z2, s2)
    assert np.array_equal(b["flags"].cpu().numpy(), _expected_flags(y2, b["info"]))
    if N == 24:
        assert b["info"]["split"] == 1              # a grid of whole rounds: every tile may skip
    if b["info"]["split"] == 1:
        assert b["skipped"] > 0                                                    # chunks were really left out
    # the same layer without a map: same results, nothing skipped
    c = _layer(want1, w2, qx2, QW, (16, 9, 7))
    assert torch.equal(b["y"], c["y"]) and c["skipped"] == 0


@pytest.mark.parametrize("C0,kernel", [(3, "flat"), (16, "rows"), (32, "rows")])
def test_flags_from_the_flat_window_and_window_row_kernels(oracle, C0, kernel):
    """A first layer with few input channels runs on another kernel than the layer it feeds; its flags
    must describe its codes all the same, and the consumer must skip on them."""
    N, H, W, C1, C2 = 24, 32, 32, 128, 64
    rng = np.random.default_rng(C0)
    x, w1, w2 = _sparse_pair(rng, N, C0, H, W, C1, C2)
    a = _layer(x, w1, QX, QW, QY)
    assert a["info"]["kernel"] == {"flat": lp.LP_KERNEL_FLAT, "rows": lp.LP_KERNEL_ROWS}[kernel]
    y1, z1, s1 = oracle.act(oracle.conv(x, w1, threads=8), 27, *QY, True, oracle.ROUND_AWAY, with_sat=True)
    assert np.array_equal(a["y_np"], y1) and (a["zeros"], a["sats"]) == (z1, s1)
    flags = a["flags"].cpu().numpy()
    assert np.array_equal(flags, _expected_flags(y1, a["info"])) and 0 < flags.sum() < flags.size
    b = _layer(y1, w2, QY, QW, (16, 9, 7), x_map=lp.zero_map(a["flags"], a["info"], a["W"]))
    y2, z2, s2 = oracle.act(oracle.conv(y1, w2, threads=8), QY[2] + QW[2], 16, 9, 7, True, oracle.ROUND_AWAY, with_sat=True)
    assert b["info"]["kernel"] == lp.LP_KERNEL_PATCH
    assert np.array_equal(b["y_np"], y2) and (b["zeros"], b["sats"]) == (z2, s2)
    if b["info"]["split"] == 1:
        assert b["skipped"] > 0
    # a map handed to a layer that runs on the window-row kernel is accepted and changes nothing
    if kernel == "rows":
        w3 = rng.integers(-900, 900, (C0, C0, 3, 3)).astype(np.int32)
        xs = x[:, :, :16, :16]
        prev = _layer(rng.integers(0, 50, (N, 64, 16, 16)).astype(np.int32) * 0, rng.integers(-9, 9, (C0, 64, 3, 3)).astype(np.int32),
                      QX, QW, QY)
        c = _layer(xs, w3, QX, QW, QY, x_map=lp.zero_map(prev["flags"], prev["info"], prev["W"]))
        y3, z3 = oracle.act(oracle.conv(xs, w3, threads=8), 27, *QY, True, oracle.ROUND_AWAY)
        assert c["info"]["kernel"] == lp.LP_KERNEL_ROWS and np.array_equal(c["y_np"], y3) and c["zeros"] == z3 and c["skipped"] == 0


def test_flags_from_split_tiles_and_all_zero_input(oracle):
    """A producer whose tail tiles are finished by the second kernel still writes every flag; an input
    that is blank everywhere (every chunk flagged zero) still gives the bias-only output."""
    rng = np.random.default_rng(5)
    x, w1, _ = _sparse_pair(rng, 2, 256, 12, 12, 64, 64)
    a = _layer(x, w1, QX, QW, QY)
    assert a["info"]["split"] > 1
    y1, z1 = oracle.act(oracle.conv(x, w1, threads=8), 27, *QY, True, oracle.ROUND_AWAY)
    assert np.array_equal(a["y_np"], y1) and a["zeros"] == z1
    assert np.array_equal(a["flags"].cpu().numpy(), _expected_flags(y1, a["info"]))
    blank = np.zeros((2, 128, 16, 16), np.int32)
    w = rng.integers(-2000, 2000, (64, 128, 3, 3)).astype(np.int32)
    d = lp.ConvDesc(2, 16, 16, 128, 64, 3, 3, 1, 1)
    info_prev = dict(lp.lp_conv_plan_info(lp.ConvDesc(2, 16, 16, 64, 128, 3, 3, 1, 1), QX, QW))
    zeros = torch.zeros(info_prev["tiles_m"] * info_prev["tiles_n"], dtype=torch.uint8, device="cuda")
    b = _layer(blank, w, QX, QW, QY, x_map=lp.zero_map(zeros, info_prev, 16))
    assert not b["y_np"].any() and b["zeros"] == b["y_np"].size
    assert b["skipped"] > 0 or b["info"]["split"] > 1        # tiles that share their reduction multiply everything
    assert not b["flags"].cpu().numpy().any()


def test_int8_layers_skip_too(oracle):
    rng = np.random.default_rng(8)
    x, w1, w2 = _sparse_pair(rng, 4, 64, 16, 16, 128, 64, n=8)
    qx, qw, qy = (8, 3, 5), (8, 1, 7), (8, 6, 2)
    a = _layer(x, w1, qx, qw, qy)
    y1, z1 = oracle.act(oracle.conv(x, w1, threads=8), 12, *qy, True, oracle.ROUND_AWAY)
    assert a["info"]["limbs"] == 1 and np.array_equal(a["y_np"], y1) and a["zeros"] == z1
    assert np.array_equal(a["flags"].cpu().numpy(), _expected_flags(y1, a["info"]))
    b = _layer(y1, w2, qy, qw, (8, 7, 1), x_map=lp.zero_map(a["flags"], a["info"], a["W"]))
    y2, z2 = oracle.act(oracle.conv(y1, w2, threads=8), 9, 8, 7, 1, True, oracle.ROUND_AWAY)
    assert np.array_equal(b["y_np"], y2) and b["zeros"] == z2
    assert b["skipped"] > 0 or b["info"]["split"] > 1


def test_stack_with_zero_skipping_matches_oracle_chain(oracle):
    """A VGG-like chain run with zskip: blank borders in the images make whole tiles of the early
    layers zero; every layer's codes and counters equal the oracle chain's."""
    x = lp_inputs.uniform01((4, 3, 48, 48), seed=31)
    x[:, :, :, 24:] = 0
    x[2:] = 0
    ws, pools, cin = [], [], 3
    for i, cout in enumerate([64, 64, 128, 128, 128]):
        w = lp_inputs.he_normal_conv(cout, cin, 3, 3, 31, 100 + i)
        if i == 1:
            w[cout // 2:] = -np.abs(w[cout // 2:])          # dead output channels
        ws.append(w)
        pools.append(i in (1, 3))
        cin = cout
    want = ovgg.conv_stack(x, ws, pools, n=16, threads=8)
    for fuse in (False, True):
        st = ConvStack([_nhwc(w) for w in ws], pools, fuse_pool=fuse, zskip=True)
        xd = _nhwc(x)
        st.calibrate(xd)
        st.prepare(4, 48, 48)
        out = st.forward(xd)
        torch.cuda.synchronize()
        for i, (L, G) in enumerate(zip(want["layers"], st.layers)):
            assert (st.qw[i].m, st.qy[i].m) == (L["mw"], L["mo"])
            if G["y"] is not None:
                assert np.array_equal(G["y"].cpu().numpy().astype(np.int32).transpose(0, 3, 1, 2), L["codes"]), i
            if G["pooled"] is not None:
                assert np.array_equal(G["pooled"].cpu().numpy().astype(np.int32).transpose(0, 3, 1, 2), L["pooled"]), i
            assert int(st.zero_counts[i].item()) == L["zeros"] and int(st.sat_counts[i].item()) == L["sats"]
        assert np.array_equal(out.cpu().numpy().astype(np.int32).transpose(0, 3, 1, 2), want["final"])
        assert int(st.skipped[1:].sum().item()) > 0 or all(G["info"]["split"] > 1 for G in st.layers[1:])
