#!/usr/bin/env python3
"""Benchmark: VGG16 16-bit fixed-point conv-stack forward on one MI355X.

A step = one pass of the whole hot path over one synthetic batch already resident in HBM:
lp_quantize of the float input, 13 x lp_conv_fwd (int8-MFMA implicit GEMM, exact two-limb
16-bit arithmetic, fused LPAct + ReLU + zero count) and the 5 max-pools.  Weights are
quantized/packed and per-layer formats calibrated beforehand (untimed, as the paper does
offline).  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_PEAK_TOPS = 5000.0     # MI355X dense int8 MFMA, published (5.0 POP/s)
HBM_PEAK_GBS = 8000.0

# HBM traffic of the dominant kernel comes from the tracked rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# summary under profiles/ (its last line is a small JSON record: average bytes per launch over the
# patch-kernel launches of one step, scaled by the copy-kernel factor, and the sha256 of the kernel
# sources it was measured on).  For any other source the counters are stale and null is reported.
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "conv_stack_vgg16_batch32_hbm_traffic.txt")
KERNEL_SOURCES = ("lp_conv.hip", "lp_tile.h", "lp_device.h")


def kernel_sources_sha256():
    import hashlib

    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        h.update(open(os.path.join(ROOT, "paper_1711_04713_amd", "csrc", name), "rb").read())
    return h.hexdigest()


def _traffic_for_current_source():
    try:
        lines = [l for l in open(TRAFFIC_PROFILE) if l.startswith("bench_record: ")]
        rec = json.loads(lines[-1][len("bench_record: "):])
        return int(rec["bytes_per_launch"]) if rec["sources_sha256"] == kernel_sources_sha256() else None
    except (OSError, IndexError, KeyError, ValueError):
        return None


EXTRA_SECTIONS = ("elementwise", "conv64", "int8", "giga1net", "fc", "zskip")


def measure_extras(lp, torch, lp_inputs, which=EXTRA_SECTIONS, iters=10):
    """The other steps of the path, each alone against its own roofline (sections, selectable with
    --extras): "elementwise": the HBM-bound kernels at the size of one 8 x 64 x 224 x 224 activation
    tensor; "conv64": the single 64->64 layer at batch 8; "int8": the 8-bit conv3_1..conv5_3 layers
    at batch 64; "giga1net": the conv layers of the paper's Table 1 at batch 32; "fc": the three
    classifier layers at batch 256; "zskip": one 256->256 layer with and without zero-tile skipping.
    Inputs have the distributions of the workload configurations (ReLU(N(0,1)) activations,
    He-normal / N(0, 0.01) weights), quantized by the library with formats from lp_range; parity of
    these shapes is the tests' job."""
    import numpy as np

    def timed(fn, n=iters):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    out = {}
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    rws = torch.empty(lp.LP_RANGE_WORKSPACE_WORDS, dtype=torch.int64, device="cuda")

    def codes_of(xf, n):
        """float tensor on the GPU -> (codes, format) by the Sec. 2.3 rule"""
        q, _ = lp.lp_range(xf.reshape(-1), n, 0.0, rws)
        c = torch.empty(xf.shape, dtype=torch.int16 if n > 8 else torch.int8, device="cuda")
        lp.lp_quantize(xf.reshape(-1), c, q)
        return c, q

    def relu_normal(shape):
        return torch.randn(shape, device="cuda", generator=g).clamp_(min=0)

    if "elementwise" in which:
        shape = (8, 224, 224, 64)
        n = 8 * 224 * 224 * 64
        xf = relu_normal(shape)
        codes = torch.empty(shape, dtype=torch.int16, device="cuda")
        q = (16, 4, 12)
        ms = timed(lambda: lp.lp_quantize(xf.reshape(-1), codes, q))
        out["lp_quantize"] = {"elements": n, "ms": round(ms, 4), "GBps": round(6 * n / ms / 1e6, 1)}
        ms = timed(lambda: lp.lp_quantize(xf.reshape(-1), codes, q, r=lp.LP_ROUND_STOCHASTIC, seed=1))
        out["lp_quantize_stochastic"] = {"elements": n, "ms": round(ms, 4), "GBps": round(6 * n / ms / 1e6, 1)}
        t0 = time.perf_counter()
        for _ in range(iters):
            lp.lp_range(xf.reshape(-1), 16, 0.0, rws)              # returns the format: synchronises
        ms = (time.perf_counter() - t0) * 1e3 / iters
        out["lp_range"] = {"elements": n, "ms": round(ms, 4), "GBps": round(4 * n / ms / 1e6, 1),
                           "note": "includes the host round trip; kernel-only figures: profiles/"}
        acc = (torch.randn(shape, device="cuda", generator=g) * (1 << 24)).to(torch.int64)
        ms = timed(lambda: lp.lp_act(acc.reshape(-1), 27, (16, 6, 10), True, codes))
        out["lp_act"] = {"elements": n, "ms": round(ms, 4), "GBps": round(10 * n / ms / 1e6, 1)}
        ms = timed(lambda: lp.lp_act_stochastic(acc.reshape(-1), 27, (16, 6, 10), True, 1, codes))
        out["lp_act_stochastic"] = {"elements": n, "ms": round(ms, 4), "GBps": round(10 * n / ms / 1e6, 1),
                                    "note": "two Philox4x32-10 blocks per eight elements"}
        t0 = time.perf_counter()
        for _ in range(iters):
            lp.lp_range_acc(acc.reshape(-1), 27, True, 16, 0.0, rws)
        ms = (time.perf_counter() - t0) * 1e3 / iters
        out["lp_range_acc"] = {"elements": n, "ms": round(ms, 4), "GBps": round(8 * n / ms / 1e6, 1),
                               "note": "includes the host round trip; kernel-only figures: profiles/"}
        pooled = torch.empty((8, 112, 112, 64), dtype=torch.int16, device="cuda")
        ms = timed(lambda: lp.lp_maxpool2x2(codes, pooled, 8, 224, 224, 64, 16))
        out["lp_maxpool2x2"] = {"elements": n, "ms": round(ms, 4), "GBps": round(2.5 * n / ms / 1e6, 1)}
        del xf, acc, pooled, codes

    def conv_ms(N, hw, cin, cout, bits, k=3, pad=1):
        """one fused layer: x = ReLU(N(0,1)) codes, He-normal weight codes, output format with 3 integer bits more than x"""
        x, qx = codes_of(relu_normal((N, hw, hw, cin)), bits)
        wf = torch.randn((cout, k, k, cin), device="cuda", generator=g) * (2.0 / (cin * k * k)) ** 0.5
        w, qw = codes_of(wf, bits)
        m = min(bits, qx.m + 2)
        qy = (bits, m, bits - m)
        d = lp.ConvDesc(N, hw, hw, cin, cout, k, k, 1, pad)
        packed = torch.empty(lp.lp_conv_packed_bytes(d, qx, qw), dtype=torch.uint8, device="cuda")
        lp.lp_conv_pack_weights(d, qx, qw, w, packed)
        ho = hw + 2 * pad - k + 1
        y = torch.empty((N, ho, ho, cout), dtype=x.dtype, device="cuda")
        z = torch.zeros(1, dtype=torch.int64, device="cuda")
        ws = torch.empty(max(lp.lp_conv_workspace_bytes(d, qx, qw), 16), dtype=torch.uint8, device="cuda")
        return timed(lambda: lp.lp_conv_fwd(d, x, qx, packed, qw, qy=qy, y_codes=y, zero_count=z, workspace=ws))

    if "conv64" in which:
        ms = conv_ms(8, 224, 64, 64, 16)
        macs = 8 * 224 * 224 * 64 * 9 * 64
        out["conv_64to64_224_batch8_16bit"] = {"ms": round(ms, 4), "int8_tops": round(8 * macs / ms / 1e9, 1)}
    if "int8" in which:
        tot_ms, tot_macs, per = 0.0, 0, {}
        for (name, cin, cout, hw, _) in lp_inputs.VGG16_CONV[4:]:
            ms = conv_ms(64, hw, cin, cout, 8)
            per[name] = round(ms, 4)
            tot_ms += ms
            tot_macs += 64 * hw * hw * cout * 9 * cin
        out["conv3_1_to_conv5_3_batch64_8bit"] = {"ms": round(tot_ms, 4), "int8_tops": round(2 * tot_macs / tot_ms / 1e9, 1),
                                                  "layers_ms": per}
    if "giga1net" in which:
        # Table 1's Giga1Net conv layers (kernel sizes 1/3/5/7, 3..128 channels) at batch 32, 16 bit
        tot_ms, tot_macs, per = 0.0, 0, {}
        for (name, cin, cout, k, hw, pad, _) in lp_inputs.GIGA1NET_CONV:
            ms = conv_ms(32, hw, cin, cout, 16, k, pad)
            per[name] = round(ms, 4)
            tot_ms += ms
            ho = hw + 2 * pad - k + 1
            tot_macs += 32 * ho * ho * cout * k * k * cin
        out["giga1net_conv_layers_batch32_16bit"] = {"ms": round(tot_ms, 4), "int8_tops": round(8 * tot_macs / tot_ms / 1e9, 1),
                                                       "images_per_s": round(32 / tot_ms * 1e3, 1), "layers_ms": per}
    if "fc" in which:
        M = 256
        fc = {}
        for name, K, N, relu in lp_inputs.VGG16_FC:
            x, qx = codes_of(relu_normal((M, K)), 16)
            w, qw = codes_of(torch.randn((N, K), device="cuda", generator=g) * 0.01, 16)
            qy = (16, 8, 8)
            packed = torch.empty(lp.lp_fc_packed_bytes(M, K, N, qx, qw), dtype=torch.uint8, device="cuda")
            lp.lp_fc_pack_weights(M, K, N, qx, qw, w, packed)
            y = torch.empty((M, N), dtype=torch.int16, device="cuda")
            z = torch.zeros(1, dtype=torch.int64, device="cuda")
            ws = torch.empty(max(lp.lp_fc_workspace_bytes(M, K, N, qx, qw), 16), dtype=torch.uint8, device="cuda")
            ms = timed(lambda: lp.lp_fc_fwd(M, K, N, x, qx, packed, qw, qy=qy, y_codes=y, relu=relu,
                                            zero_count=z, workspace=ws), n=2 * iters)
            fc[name] = {"ms": round(ms, 4), "int8_tops": round(8 * M * K * N / ms / 1e9, 1),
                        "weight_GBps": round(2 * K * N / ms / 1e6, 1)}
            del x, w, packed
        out["fc_batch256_16bit"] = fc
    if "zskip" in which:
        # conv3_2's shape with structured zeros: the producer's tile flags are built from the data
        B, hw, cin, cout = 32, 56, 256, 256
        qx, qw, qy = (16, 4, 12), (16, 1, 15), (16, 6, 10)
        d = lp.ConvDesc(B, hw, hw, cin, cout, 3, 3, 1, 1)
        info = lp.lp_conv_plan_info(d, qx, qw)
        w = torch.randint(-2000, 2000, (cout, 3, 3, cin), device="cuda", generator=g).to(torch.int16)
        packed = torch.empty(lp.lp_conv_packed_bytes(d, qx, qw), dtype=torch.uint8, device="cuda")
        lp.lp_conv_pack_weights(d, qx, qw, w, packed)
        y = torch.empty((B, hw, hw, cout), dtype=torch.int16, device="cuda")
        z = torch.zeros(1, dtype=torch.int64, device="cuda")
        k = torch.zeros(1, dtype=torch.int64, device="cuda")
        ws = torch.empty(max(lp.lp_conv_workspace_bytes(d, qx, qw), 16), dtype=torch.uint8, device="cuda")
        fl = torch.empty(info["tiles_m"] * info["tiles_n"], dtype=torch.uint8, device="cuda")
        rh, tw = info["tile_rows"], info["tile_cols"]      # the producer is given this layer's own tile geometry
        tr, tc, tn = -(-B * hw // rh), -(-hw // tw), cin // 64
        res = {}
        for label, kind in (("dense", 0), ("half_of_elements_zero_unstructured", 1), ("2_of_4_channel_chunks_zero", 2),
                            ("right_half_of_images_zero", 3)):
            x = torch.randint(1, 2000, (B * hw, hw, cin), device="cuda", generator=g).to(torch.int16)
            keep = torch.ones((tr, tc, tn), dtype=torch.bool, device="cuda")
            if kind == 1:
                x = x * (torch.rand(x.shape, device="cuda", generator=g) >= 0.5).to(torch.int16)
            if kind == 2:
                keep[:, :, tn // 2:] = False
            if kind == 3:
                keep[:, tc // 2:, :] = False
            m = keep.repeat_interleave(rh, 0)[:B * hw].repeat_interleave(tw, 1)[:, :hw].repeat_interleave(64, 2)
            x = (x * m.to(torch.int16)).reshape(B, hw, hw, cin).contiguous()
            prod = dict(info, tiles_n=tn, bn=64)
            xm = lp.zero_map(keep.to(torch.uint8).reshape(-1).contiguous(), prod, hw)
            run_base = lambda: lp.lp_conv_fwd(d, x, qx, packed, qw, qy=qy, y_codes=y, zero_count=z, workspace=ws)
            run_skip = lambda: lp.lp_conv_fwd_zskip(d, x, qx, xm, packed, qw, qy, y, zero_count=z, workspace=ws,
                                                    y_flags=fl, skipped=k)
            run_base()
            y0 = y.clone()
            k.zero_()
            run_skip()
            per_call = int(k.item())
            # alternate the two so that both see the same clocks
            base = skip = 0.0
            for _ in range(3):
                base += timed(run_base, 2 * iters) / 3
                skip += timed(run_skip, 2 * iters) / 3
            res[label] = {"lp_conv_fwd_ms": round(base, 4), "zskip_ms": round(skip, 4), "speedup": round(base / skip, 3),
                          "same_codes": bool(torch.equal(y, y0)),
                          "chunks_skipped": round(per_call / (info["tiles_m"] * info["tiles_n"] * tn), 3)}
        out["zskip_conv3_2_batch32"] = res
    return out


def copy_probe(torch):
    """A plain 1 GiB device-to-device copy: what FETCH_SIZE / WRITE_SIZE read for it calibrates those counters."""
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    src.zero_()
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--calib", type=int, default=2, help="images used to fix the per-layer formats")
    ap.add_argument("--cpu-images", type=int, default=2, help="images the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--no-extras", action="store_true", help="skip the per-kernel measurements of the other path steps")
    ap.add_argument("--extras", default="all", help="comma list of extra sections to run: " + ", ".join(EXTRA_SECTIONS))
    ap.add_argument("--no-main", action="store_true",
                    help="only the extra sections (for profiling them alone); prints their JSON, not the benchmark line")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy (calibrates FETCH_SIZE/WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: the library runs on exactly one GPU (--gpus 1); more GPUs would each take a share of the batch",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import lp_inputs
    import paper_1711_04713_amd as lp
    from paper_1711_04713_amd.stack import ConvStack

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    lp.load()        # raises if liblp.so is not built: there is no fallback
    torch.cuda.set_device(0)
    B = args.batch
    sections = EXTRA_SECTIONS if args.extras == "all" else tuple(s for s in args.extras.split(",") if s)
    if args.no_main:
        print(json.dumps({"extras": measure_extras(lp, torch, lp_inputs, sections)}))
        if args.copy_probe:
            copy_probe(torch)
        return

    x_np = lp_inputs.config3_input(seed=2, batch=B)                       # U(0,1) images, NCHW
    w_np = lp_inputs.vgg16_conv_weights(seed=2)                           # He-normal
    pools = [p for (_, _, _, _, p) in lp_inputs.VGG16_CONV]
    x = torch.from_numpy(np.ascontiguousarray(x_np.transpose(0, 2, 3, 1))).cuda()
    ws = [torch.from_numpy(np.ascontiguousarray(w.transpose(0, 2, 3, 1))).cuda() for w in w_np]

    stack = ConvStack(ws, pools, n_act=16, n_w=16)
    stack.calibrate(x[:args.calib])
    stack.prepare(B, 224, 224)

    for _ in range(args.warmup):
        stack.forward(x)
    torch.cuda.synchronize()
    # HIP events bracket every launch on one step in four of the timed region (recording them on
    # every step would itself cost about 5 % of the step time)
    events = []
    t0 = time.perf_counter()
    for k in range(args.steps):
        stack.forward(x, events if k % 4 == 0 else None)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps

    if args.copy_probe:
        copy_probe(torch)

    # per-launch durations from the HIP events recorded on the launch stream
    per = {}
    for label, a, b in events:
        per.setdefault(label, []).append(a.elapsed_time(b))
    avg = {k: sum(v) / len(v) for k, v in per.items()}
    zeros = stack.zero_counts.cpu().numpy()
    sats = stack.sat_counts.cpu().numpy()
    layers = []
    total_macs = 0
    kern_ops, kern_ms = {}, {}
    for i, L in enumerate(stack.layers):
        name = lp_inputs.VGG16_CONV[i][0]
        ms = avg["conv%d" % i]
        macs = L["macs"]
        total_macs += macs
        info = L["info"]
        kname = {lp.LP_KERNEL_DIRECT: "conv_direct_kernel", lp.LP_KERNEL_FLAT: "conv_flat_kernel",
                 lp.LP_KERNEL_ROWS: "conv_rows_kernel",
                 lp.LP_KERNEL_PATCH: "conv_mfma_kernel<%d,%d,patch>" % (info["limbs"], info["bn"] // 64)}[info["kernel"]]
        kern_ops[kname] = kern_ops.get(kname, 0) + 8 * macs          # 4 int8 limb MACs = 8 int8 ops per 16-bit MAC
        kern_ms[kname] = kern_ms.get(kname, 0.0) + ms
        layers.append({
            "layer": name, "ms": round(ms, 4), "format_in": repr(L["qx"]), "format_w": repr(L["qw"]),
            "format_out": repr(L["qy"]), "sparsity": round(float(zeros[i]) / L["y_numel"], 4),
            "saturated": round(float(sats[i]) / L["y_numel"], 6), "pool_fused": bool(L["fused_pool"]),
            "int8_tops": round(8 * macs / (ms * 1e-3) / 1e12, 1), "kernel": kname,
            "tile": [info["tile_rows"], info["tile_cols"], info["bn"]], "workgroups": info["workgroups"],
            "split": info["split"],
        })
    dominant = max(kern_ms, key=kern_ms.get)
    achieved = kern_ops[dominant] / (kern_ms[dominant] * 1e-3) / 1e12
    images_per_s = B / (ms_per_step * 1e-3)
    useful_tops = 2 * total_macs / (ms_per_step * 1e-3) / 1e12
    int8_tops = 4 * useful_tops

    out = {
        "metric": "VGG16 16-bit fixed-point conv fwd images/s",
        "value": round(images_per_s, 1),
        "unit": "images/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int16 codes as 2x int8 limbs, int32/int64 accumulate",
        "data": "synthetic",
        "config": {"workload": "VGG16 conv stack (13 conv 3x3 pad 1 + 5 max-pool), 16-bit weights and activations, "
                               "per-layer Qm.f from dynamic range", "batch": B, "input": "3x224x224 U(0,1)",
                   "calibration_images": args.calib},
        "int_mac_tops_useful": round(useful_tops, 2),
        "int8_mfma_tops": round(int8_tops, 1),
        "pct_of_int8_mfma_peak": round(100.0 * int8_tops / INT8_PEAK_TOPS, 2),
        "roofline": {
            "bound": "mfma", "kernel": dominant, "achieved": round(achieved, 1), "peak": INT8_PEAK_TOPS,
            "unit": "TOP/s", "frac": round(achieved / INT8_PEAK_TOPS, 4), "traffic": _traffic_for_current_source(),
            "launches_per_step": sum(1 for l in layers if l["kernel"] == dominant),
            "ms_per_step_in_kernel": round(kern_ms[dominant], 4),
        },
        "other_kernels_ms": {k: round(v, 4) for k, v in avg.items() if not k.startswith("conv")},
        "layers": layers,
    }
    in_bytes = x.numel() * 4 + stack.x_codes.numel() * 2
    out["quantize_gbs"] = round(in_bytes / (avg["quantize"] * 1e-3) / 1e9, 1)

    if args.cpu_images > 0:
        import oracle
        from oracle import vgg as ovgg

        nimg = min(args.cpu_images, B)
        threads = min(os.cpu_count() or 1, len(os.sched_getaffinity(0)), 16)
        frozen = [{"mx": stack.qx.m, "mw": stack.qw[i].m, "mo": stack.qy[i].m} for i in range(len(pools))]
        t0 = time.perf_counter()
        ref = ovgg.conv_stack(x_np[:nimg], w_np, pools, n=16, threads=threads, formats=frozen, keep_codes=False)
        cpu_s = time.perf_counter() - t0
        got = stack.layers[-1]["pooled"][:nimg].cpu().numpy().astype(np.int32).transpose(0, 3, 1, 2)
        # single-thread leg: the same chain on the first image alone
        t0 = time.perf_counter()
        ref1 = ovgg.conv_stack(x_np[:1], w_np, pools, n=16, threads=1, formats=frozen, keep_codes=False)
        cpu1_s = time.perf_counter() - t0
        out["cpu_baseline"] = {
            "value": round(nimg / cpu_s, 4), "unit": "images/s", "cores": threads, "kind": "oracle",
            "single_thread": {"value": round(1.0 / cpu1_s, 4), "unit": "images/s", "cores": 1, "seconds": round(cpu1_s, 2),
                              "sample": "first image of the same batch, same chain",
                              "matches_gpu_final_codes": bool(np.array_equal(got[:1], ref1["final"]))},
            "sample": "first %d image(s) of the same batch, whole 13-layer stack, frozen formats, gcc -O2 direct loops, "
                      "OpenMP over (image, output channel); includes weight quantization" % nimg,
            "seconds": round(cpu_s, 2),
            "matches_gpu_final_codes": bool(np.array_equal(got, ref["final"])),
        }
    if not args.no_extras:
        out["extras"] = measure_extras(lp, torch, lp_inputs, sections)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
