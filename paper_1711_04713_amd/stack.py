"""Host-side sequencing of the C-ABI calls for a stack of low-precision layers (Sec. 2.1
workflow: quantize -> [LPConvolution -> LPAct+ReLU -> optional 2x2 max-pool] x L).

Only launches and buffer bookkeeping live here; every number is produced by the kernels
behind include/lp.h.  Activations are NHWC torch tensors on the GPU.
"""
import warnings

import torch

from . import binding as lp


class ConvStack:
    """A chain of stride-1 low-precision conv layers with frozen per-layer formats.

    weights: list of float32 CUDA tensors [Cout][R][S][Cin]; pool_after: list of bool; pad: zero
    padding, one int for all layers or a list (VGG16: 3x3 kernels, pad 1; Table 1's Giga1Net mixes
    kernel sizes 1/3/5/7).  n_act / n_w: total bits of activations / weights.  Formats are fixed
    by calibrate().
    """

    def __init__(self, weights, pool_after, n_act=16, n_w=16, loss_threshold=0.0, r=lp.LP_ROUND_NEAREST_AWAY,
                 pad=1, fuse_pool=True, count_sat=True, zskip=False):
        """fuse_pool: let lp_conv_fwd store the 2x2 maxima directly where its tiling allows it
        (the unpooled codes of such a layer are then never written; layer["y"] is None).
        count_sat: also count, per layer, the activations the frozen output format clips
        (sat_counts; Sec. 2.3's share of lost values, measured on the running batch).
        zskip: every layer leaves per-tile nonzero flags of its output and the next layer skips the
        64-channel chunks of its input patches that are flagged all-zero (lp_conv_fwd_zskip;
        skipped[i] counts the (tile, chunk) pairs layer i did not multiply)."""
        assert len(weights) == len(pool_after)
        self.fuse_pool, self.count_sat, self.zskip = fuse_pool, count_sat, zskip
        self.n_act, self.n_w, self.thr, self.r = n_act, n_w, loss_threshold, r
        self.pads = list(pad) if isinstance(pad, (list, tuple)) else [pad] * len(weights)
        assert len(self.pads) == len(weights)
        self.pool_after = list(pool_after)
        self.w_float = weights
        self.range_ws = torch.empty(lp.LP_RANGE_WORKSPACE_WORDS, dtype=torch.int64, device="cuda")
        # weight formats and codes: Sec. 2.3 rule on the weights themselves (done once, offline)
        self.qw, self.w_codes = [], []
        for w in weights:
            q, _ = lp.lp_range(w.reshape(-1), n_w, loss_threshold, self.range_ws)
            codes = torch.empty(w.shape, dtype=torch.int16 if n_w > 8 else torch.int8, device="cuda")
            lp.lp_quantize(w.reshape(-1), codes, q, r)
            self.qw.append(q)
            self.w_codes.append(codes)
        self.qx = None        # input format
        self.qy = []          # per-layer output formats
        self.plans = None

    def _desc(self, i, N, H, W, pool=0):
        cout, R, S, cin = self.w_float[i].shape
        return lp.ConvDesc(N, H, W, cin, cout, R, S, 1, self.pads[i], pool)

    def _out_hw(self, i, H, W):
        _, R, S, _ = self.w_float[i].shape
        return H + 2 * self.pads[i] - R + 1, W + 2 * self.pads[i] - S + 1

    def calibrate(self, x_float):
        """Fix the input format and every layer's output format from the dynamic range seen on
        this (small) batch: raw int64 accumulators -> lp_range_acc -> lp_act -> pool -> next."""
        N, H, W, _ = x_float.shape
        dt = torch.int16 if self.n_act > 8 else torch.int8
        self.qx, _ = lp.lp_range(x_float.reshape(-1), self.n_act, self.thr, self.range_ws)
        cur = torch.empty(x_float.shape, dtype=dt, device="cuda")
        lp.lp_quantize(x_float.reshape(-1), cur, self.qx, self.r)
        q_in = self.qx
        self.qy = []
        for i, pool in enumerate(self.pool_after):
            d = self._desc(i, N, H, W)
            packed = torch.empty(lp.lp_conv_packed_bytes(d, q_in, self.qw[i]), dtype=torch.uint8, device="cuda")
            lp.lp_conv_pack_weights(d, q_in, self.qw[i], self.w_codes[i], packed)
            H, W = self._out_hw(i, H, W)
            acc = torch.empty((N, H, W, d.Cout), dtype=torch.int64, device="cuda")
            lp.lp_conv_fwd(d, cur, q_in, packed, self.qw[i], acc_out=acc, r=self.r)
            f_acc = q_in.f + self.qw[i].f
            qy, _ = lp.lp_range_acc(acc.reshape(-1), f_acc, True, self.n_act, self.thr, self.range_ws)
            y = torch.empty((N, H, W, d.Cout), dtype=dt, device="cuda")
            lp.lp_act(acc.reshape(-1), f_acc, qy, True, y, self.r)
            if pool:
                p = torch.empty((N, H // 2, W // 2, d.Cout), dtype=dt, device="cuda")
                lp.lp_maxpool2x2(y, p, N, H, W, d.Cout, self.n_act)
                y, H, W = p, H // 2, W // 2
            self.qy.append(qy)
            cur, q_in = y, qy
        torch.cuda.synchronize()
        return self.qx, self.qy

    def set_formats(self, qx, qy):
        as_fmt = lambda q: lp.QFmt(*(q.astuple() if isinstance(q, lp.QFmt) else q))
        self.qx, self.qy = as_fmt(qx), [as_fmt(q) for q in qy]

    def prepare(self, N, H, W):
        """Pack weights for the frozen formats and allocate every buffer of a forward pass."""
        assert self.qx is not None, "calibrate() or set_formats() first"
        dt = torch.int16 if self.n_act > 8 else torch.int8
        self.in_shape = (N, H, W, self.w_float[0].shape[3])
        self.x_codes = torch.empty(self.in_shape, dtype=dt, device="cuda")
        # one buffer for every counter of a pass, so that a pass clears them with one fill
        nl = len(self.pool_after)
        self.counters = torch.zeros(3 * nl + 1, dtype=torch.int64, device="cuda")
        self.zero_counts = self.counters[0:nl]
        self.sat_counts = self.counters[nl:2 * nl]
        self.skipped = self.counters[2 * nl:3 * nl]
        self.input_sat = self.counters[3 * nl:3 * nl + 1]
        self.layers = []
        q_in = self.qx
        for i, pool in enumerate(self.pool_after):
            d = self._desc(i, N, H, W)
            fused = False
            if pool and self.fuse_pool and self.n_act > 8:
                try:                      # status 2: this layer's tiling or arguments cannot pool for free
                    if lp.lp_conv_pool_check(self._desc(i, N, H, W, 1), q_in, self.qw[i], self.qy[i], True, self.r):
                        d, fused = self._desc(i, N, H, W, 1), True
                except lp.LpError as e:
                    if e.status != 2:
                        raise
            packed = torch.empty(lp.lp_conv_packed_bytes(d, q_in, self.qw[i]), dtype=torch.uint8, device="cuda")
            lp.lp_conv_pack_weights(d, q_in, self.qw[i], self.w_codes[i], packed)
            H, W = self._out_hw(i, H, W)      # from here on: the layer's output size
            y = None if fused else torch.empty((N, H, W, d.Cout), dtype=dt, device="cuda")
            p = None
            if pool:
                p = torch.empty((N, H // 2, W // 2, d.Cout), dtype=dt, device="cuda")
            ws = torch.empty(max(lp.lp_conv_workspace_bytes(d, q_in, self.qw[i]), 16), dtype=torch.uint8, device="cuda")
            info = lp.lp_conv_plan_info(d, q_in, self.qw[i])
            if info["path"] != 1:
                warnings.warn("layer %d (%s) is outside the int8-MFMA kernels' shapes and runs on the plain "
                              "one-thread-per-output kernel" % (i, tuple(self.w_float[i].shape)), RuntimeWarning)
            flags = x_map = None
            if self.zskip and info["path"] == 1:
                flags = torch.empty(info["tiles_m"] * info["tiles_n"], dtype=torch.uint8, device="cuda")
                prev = self.layers[-1] if self.layers else None
                if prev is not None and prev["flags"] is not None:
                    x_map = lp.zero_map(prev["flags"], prev["info"], prev["W"], 2 if prev["pooled"] is not None else 1)
            self.layers.append({"flags": flags, "x_map": x_map, "desc": d, "packed": packed, "ws": ws, "qx": q_in, "qw": self.qw[i], "qy": self.qy[i], "y": y,
                                "pooled": p, "fused_pool": fused, "H": H, "W": W, "y_numel": N * H * W * d.Cout,
                                "macs": N * H * W * d.Cout * d.R * d.S * d.Cin,
                                "info": info})
            if pool:
                H, W = H // 2, W // 2
            q_in = self.qy[i]
        torch.cuda.synchronize()

    def forward(self, x_float, events=None):
        """One pass over the batch: input quantize + every conv (+fused LPAct/ReLU/zero count) +
        pools.  events (optional): list to which (label, start_event, end_event) are appended."""
        assert tuple(x_float.shape) == self.in_shape
        self.counters.zero_()

        def timed(label, fn):
            if events is None:
                fn()
                return
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            events.append((label, a, b))

        timed("quantize", lambda: lp.lp_quantize(x_float.reshape(-1), self.x_codes, self.qx, self.r,
                                                 sat_count=self.input_sat if self.count_sat else None))
        cur = self.x_codes
        for i, L in enumerate(self.layers):
            out = L["pooled"] if L["fused_pool"] else L["y"]
            if L["flags"] is not None:
                timed("conv%d" % i, lambda L=L, cur=cur, i=i, out=out: lp.lp_conv_fwd_zskip(
                    L["desc"], cur, L["qx"], L["x_map"], L["packed"], L["qw"], L["qy"], out, relu=True, r=self.r,
                    zero_count=self.zero_counts[i:i + 1], workspace=L["ws"],
                    sat_count=self.sat_counts[i:i + 1] if self.count_sat else None, y_flags=L["flags"],
                    skipped=self.skipped[i:i + 1]))
            else:
                timed("conv%d" % i, lambda L=L, cur=cur, i=i, out=out: lp.lp_conv_fwd(
                    L["desc"], cur, L["qx"], L["packed"], L["qw"], qy=L["qy"], y_codes=out, relu=True, r=self.r,
                    zero_count=self.zero_counts[i:i + 1], workspace=L["ws"],
                    sat_count=self.sat_counts[i:i + 1] if self.count_sat else None))
            cur = out
            if L["pooled"] is not None and not L["fused_pool"]:
                d = L["desc"]
                timed("pool%d" % i, lambda L=L, d=d: lp.lp_maxpool2x2(L["y"], L["pooled"], d.N, L["H"], L["W"], d.Cout,
                                                                       self.n_act))
                cur = L["pooled"]
        return cur
