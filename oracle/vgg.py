"""Layer chains composed from the oracle's steps (TEST INFRASTRUCTURE ONLY).

conv_stack: quantize the input, then per layer LPConvolution -> LPAct+ReLU ->
optional 2x2 max-pool, as the workflow of Sec. 2.1 strings the low-precision
layers together.  Per-tensor formats come from the dynamic-range rule of
Sec. 2.3 with a fixed total width n: weights and the input from their float
values, each layer's output from its own exact accumulators on this batch
(the paper measures ranges on a sample of images and then freezes them).
Sparsity is counted on the LPAct output, before pooling (Sec. 3.1).
"""
from . import lp_oracle as orc


def conv_stack(x, weights, pool_after, n=16, n_w=None, threshold=0.0, mode=orc.ROUND_AWAY,
               threads=1, formats=None, keep_codes=True, pads=None):
    """x float32 [N,C,H,W]; weights: list of float32 [Cout,Cin,R,S]; pool_after: list of bool;
    pads: zero padding per layer (default 1 everywhere: the 3x3 layers of VGG16); stride 1.

    formats (optional): list of dicts {"mw","mo"} (+ "mx" in entry 0) to use frozen formats
    instead of measuring them.  Returns {"mx", "layers": [ {mw, fw, mo, fo, f_acc, zeros,
    sats (values clipped by the output format), count, codes (LPAct output, NCHW), pooled (or
    None)} ... ], "x_codes"}.
    """
    n_w = n_w or n
    mx = formats[0]["mx"] if formats else orc.range_float(x, n, threshold)[0]
    fx = n - mx
    cur, _, _ = orc.quantize(x, n, mx, fx, mode)
    out = {"mx": mx, "x_codes": cur if keep_codes else None, "layers": []}
    for i, (w, pool) in enumerate(zip(weights, pool_after)):
        mw = formats[i]["mw"] if formats else orc.range_float(w, n_w, threshold)[0]
        fw = n_w - mw
        wc, _, _ = orc.quantize(w, n_w, mw, fw, mode)
        acc = orc.conv(cur, wc, stride=1, pad=1 if pads is None else pads[i], threads=threads)
        f_acc = fx + fw
        mo = formats[i]["mo"] if formats else orc.range_acc(acc, f_acc, True, n, threshold)[0]
        fo = n - mo
        codes, zeros, sats = orc.act(acc, f_acc, n, mo, fo, True, mode, with_sat=True)
        pooled = orc.maxpool2x2(codes) if pool else None
        out["layers"].append({
            "mw": mw, "fw": fw, "mo": mo, "fo": fo, "f_acc": f_acc, "zeros": zeros, "sats": sats,
            "count": int(codes.size), "w_codes": wc if keep_codes else None,
            "codes": codes if keep_codes else None, "pooled": pooled if keep_codes else None,
        })
        cur = pooled if pool else codes
        fx = fo
    out["final"] = cur
    return out


def fc_stack(x, weights, relu_after, n=16, threshold=0.0, mode=orc.ROUND_AWAY, threads=1):
    """x float32 [M,K]; weights: list of float32 [Nout,K]; LPInnerProduct -> LPAct (+ReLU) chain."""
    mx = orc.range_float(x, n, threshold)[0]
    fx = n - mx
    cur, _, _ = orc.quantize(x, n, mx, fx, mode)
    out = {"mx": mx, "x_codes": cur, "layers": []}
    for w, relu in zip(weights, relu_after):
        mw = orc.range_float(w, n, threshold)[0]
        fw = n - mw
        wc, _, _ = orc.quantize(w, n, mw, fw, mode)
        acc = orc.fc(cur, wc, threads=threads)
        f_acc = fx + fw
        mo = orc.range_acc(acc, f_acc, relu, n, threshold)[0]
        fo = n - mo
        codes, zeros, sats = orc.act(acc, f_acc, n, mo, fo, relu, mode, with_sat=True)
        out["layers"].append({"mw": mw, "fw": fw, "mo": mo, "fo": fo, "f_acc": f_acc, "zeros": zeros, "sats": sats,
                              "count": int(codes.size), "w_codes": wc, "acc": acc, "codes": codes})
        cur, fx = codes, fo
    out["final"] = cur
    return out
