"""GPU parity of whole layer chains against the oracle's chain: formats chosen from the dynamic
range by each side on its own, then every layer's codes and zero count compared bit for bit."""
import numpy as np
import pytest
import torch

import lp_inputs
import paper_1711_04713_amd as lp
from gpu_helpers import fc, to_dev
from oracle import vgg as ovgg
from paper_1711_04713_amd.stack import ConvStack

pytestmark = pytest.mark.gpu


def _nhwc(a):
    return to_dev(np.ascontiguousarray(a.transpose(0, 2, 3, 1)))


def _run_stack(x, ws, pools, n_act=16, n_w=16, calib=None, fuse_pool=False, pad=1):
    st = ConvStack([_nhwc(w) for w in ws], pools, n_act=n_act, n_w=n_w, fuse_pool=fuse_pool, pad=pad)
    xd = _nhwc(x)
    st.calibrate(xd[:calib] if calib else xd)
    N, H, W, _ = xd.shape
    st.prepare(N, H, W)
    out = st.forward(xd)
    torch.cuda.synchronize()
    return st, out


def _compare(st, out, want, n_images=None):
    assert st.qx.astuple()[1] == want["mx"]
    sl = slice(None) if n_images is None else slice(0, n_images)
    for i, (L, G) in enumerate(zip(want["layers"], st.layers)):
        assert st.qw[i].m == L["mw"], "layer %d weight format" % i
        assert st.qy[i].m == L["mo"], "layer %d output format" % i
        if G["y"] is not None:          # a layer with the pooling fused never writes these
            got = G["y"][sl].cpu().numpy().astype(np.int32).transpose(0, 3, 1, 2)
            assert np.array_equal(got, L["codes"]), "layer %d codes" % i
        if G["pooled"] is not None:
            gp = G["pooled"][sl].cpu().numpy().astype(np.int32).transpose(0, 3, 1, 2)
            assert np.array_equal(gp, L["pooled"]), "layer %d pooled codes" % i
        if n_images is None:
            assert int(st.zero_counts[i].item()) == L["zeros"], "layer %d zero count" % i
            assert int(st.sat_counts[i].item()) == L["sats"], "layer %d count of clipped values" % i
        elif G["y"] is not None:  # the counter covers the whole batch: check it against the codes it counted
            assert int(st.zero_counts[i].item()) == int((G["y"] == 0).sum().item())
    assert np.array_equal(out[sl].cpu().numpy().astype(np.int32).transpose(0, 3, 1, 2), want["final"])


def test_small_vgg_like_stack_16bit(oracle):
    """13-layer VGG16 channel plan scaled down (channels / 4, 32x32 input), U(0,1) images, He weights."""
    x = lp_inputs.uniform01((3, 3, 32, 32), seed=21)
    ws, pools = [], []
    cin = 3
    for i, (_, _, cout, _, pool) in enumerate(lp_inputs.VGG16_CONV):
        ws.append(lp_inputs.he_normal_conv(cout // 4, cin, 3, 3, 21, 100 + i))
        pools.append(pool)
        cin = cout // 4
    want = ovgg.conv_stack(x, ws, pools, n=16, threads=8)
    for fuse in (False, True):
        st, out = _run_stack(x, ws, pools, fuse_pool=fuse)
        _compare(st, out, want)
        if fuse:                                    # at least the wide early layers pool in the epilogue
            assert any(G["fused_pool"] for G in st.layers)
    for L in want["layers"]:
        assert 0.2 < L["zeros"] / L["count"] < 0.8       # ~half zeros with zero-mean random weights


def test_giga1net_conv_stack_full_resolution(oracle):
    """The eleven conv layers of Table 1 (kernel sizes 1, 7, 7, 5, 5, 5, 3 x 5; 3..128 channels;
    224x224 down to 18x18; four pools) at their true shapes, two images: every layer's codes, pooled
    codes and zero count against the oracle chain, with the pools as separate kernels and fused."""
    spec = lp_inputs.GIGA1NET_CONV
    x = lp_inputs.config3_input(seed=5, batch=2)
    ws = lp_inputs.giga1net_conv_weights(seed=5)
    pools = [p for (*_, p) in spec]
    pads = [pad for (*_, pad, _) in spec]
    hw = 224
    for (name, cin, cout, k, hw_in, pad, pool), w in zip(spec, ws):   # the table's sizes chain up with these pads
        assert hw == hw_in and w.shape == (cout, cin, k, k), name
        hw = hw + 2 * pad - k + 1
        hw = hw // 2 if pool else hw
    assert hw == 9
    want = ovgg.conv_stack(x, ws, pools, n=16, threads=16, pads=pads)
    for fuse in (False, True):
        st, out = _run_stack(x, ws, pools, fuse_pool=fuse, pad=pads)
        _compare(st, out, want)
        assert all(G["info"]["path"] == 1 for G in st.layers)       # every layer on the MFMA kernel


def test_vgg16_first_two_blocks_full_resolution(oracle):
    """conv1_1..conv2_2 at the real 224x224 resolution and channel counts, one image."""
    x = lp_inputs.config3_input(seed=2, batch=1)
    ws = lp_inputs.vgg16_conv_weights(seed=2, layers=["conv1_1", "conv1_2", "conv2_1", "conv2_2"])
    pools = [False, True, False, True]
    want = ovgg.conv_stack(x, ws, pools, n=16, threads=16)
    for fuse in (False, True):
        st, out = _run_stack(x, ws, pools, fuse_pool=fuse)
        _compare(st, out, want)
        assert [G["fused_pool"] for G in st.layers] == [False, fuse, False, fuse]


def test_frozen_formats_from_a_calibration_subset(oracle):
    """Formats measured on the first image only, then the whole batch runs with them; the oracle
    does the same, and saturation of the other images must agree too."""
    x = lp_inputs.uniform01((4, 3, 24, 24), seed=22) * np.float32(1.0)
    x[1:] *= np.float32(3.0)        # later images exceed the calibrated range
    ws = [lp_inputs.he_normal_conv(16, 3, 3, 3, 22, 1), lp_inputs.he_normal_conv(32, 16, 3, 3, 22, 2),
          lp_inputs.he_normal_conv(32, 32, 3, 3, 22, 3)]
    pools = [False, True, False]
    cal = ovgg.conv_stack(x[:1], ws, pools, n=16)
    frozen = [{"mx": cal["mx"], "mw": L["mw"], "mo": L["mo"]} for L in cal["layers"]]
    want = ovgg.conv_stack(x, ws, pools, n=16, formats=frozen)
    st, out = _run_stack(x, ws, pools, calib=1)
    _compare(st, out, want)
    assert (want["x_codes"] == 32767).any()       # the input really saturated
    assert int(st.input_sat.item()) == oracle.quantize(x, 16, cal["mx"], 16 - cal["mx"])[2] > 0
    assert sum(L["sats"] for L in want["layers"]) > 0      # and so did activations (compared per layer above)


def test_int8_stack_conv3_to_conv5_shapes_small(oracle):
    """8-bit weights (Q1.7 expected) and 8-bit activations on the conv3_1..conv5_3 channel plan,
    small spatial size and batch."""
    x = lp_inputs.relu_normal((2, 128, 16, 16), seed=3, stream=10)
    ws = [lp_inputs.he_normal_conv(co, ci, 3, 3, 3, 100 + i)
          for i, (_, ci, co, _, _) in enumerate(lp_inputs.VGG16_CONV[4:10])]
    pools = [False, False, True, False, False, True]
    want = ovgg.conv_stack(x, ws, pools, n=8, n_w=8, threads=8)
    st, out = _run_stack(x, ws, pools, n_act=8, n_w=8)
    assert all(q.astuple() == (8, 1, 7) for q in st.qw)
    assert all(L["info"]["path"] == 1 and L["info"]["limbs"] == 1 for L in st.layers)
    _compare(st, out, want)


def test_fc_classifier_chain_reduced(oracle):
    """fc6/fc7/fc8-shaped chain at reduced width: 16-bit, N(0, 0.01) weights, ReLU inputs, last layer
    without ReLU; formats from the dynamic range on both sides."""
    M, dims = 64, [(3136, 512), (512, 512), (512, 125)]
    x = lp_inputs.config5_input(seed=4, batch=M, k=dims[0][0])
    ws = lp_inputs.config5_weights(seed=4, dims=dims)
    want = ovgg.fc_stack(x, ws, [True, True, False], n=16, threads=8)
    ws_dev = torch.empty(lp.LP_RANGE_WORKSPACE_WORDS, dtype=torch.int64, device="cuda")
    qx, _ = lp.lp_range(to_dev(x.reshape(-1)), 16, 0.0, ws_dev)
    assert qx.m == want["mx"]
    cur = want["x_codes"]             # same codes as lp_quantize gives (checked elsewhere); keeps the helper simple
    q_in = qx.astuple()
    for w, relu, L in zip(ws, [True, True, False], want["layers"]):
        qw, _ = lp.lp_range(to_dev(w.reshape(-1)), 16, 0.0, ws_dev)
        assert qw.m == L["mw"]
        got = fc(cur, q_in, L["w_codes"], qw.astuple(), qy=None)
        assert np.array_equal(got["acc"], L["acc"])
        qy, _ = lp.lp_range_acc(to_dev(got["acc"].reshape(-1)), L["f_acc"], relu, 16, 0.0, ws_dev)
        assert qy.m == L["mo"]
        got = fc(cur, q_in, L["w_codes"], qw.astuple(), qy=qy.astuple(), relu=relu, want_acc=False)
        assert np.array_equal(got["y"], L["codes"]) and (got["zeros"], got["sats"]) == (L["zeros"], L["sats"])
        cur, q_in = got["y"], qy.astuple()
