"""ctypes binding of include/lp.h.  Same names as the C entry points; tensors are torch
tensors on the GPU (their data_ptr() is what crosses the ABI), the stream is torch's current
stream.  No arithmetic happens here, and there is no CPU fallback: if liblp.so is missing or
fails to load, every call raises."""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liblp.so")
_lib = None

LP_ROUND_NEAREST_AWAY = 0
LP_ROUND_NEAREST_EVEN = 1
LP_ROUND_STOCHASTIC = 2
LP_RANGE_WORKSPACE_WORDS = 32
LP_KERNEL_DIRECT, LP_KERNEL_PATCH, LP_KERNEL_FLAT, LP_KERNEL_ROWS = 0, 1, 2, 3   # lp_plan_info.kernel


class LpError(RuntimeError):
    def __init__(self, status, what):
        self.status = int(status)
        super().__init__("%s failed: status %d (%s)" % (what, status, lp_status_string(status)))


class QFmt(ctypes.Structure):
    """(n, m, f): n total bits, m integer bits including sign, f fraction bits."""
    _fields_ = [("n", ctypes.c_int32), ("m", ctypes.c_int32), ("f", ctypes.c_int32)]

    def __repr__(self):
        return "Q%d.%d(n=%d)" % (self.m, self.f, self.n)

    def astuple(self):
        return (self.n, self.m, self.f)


class PlanInfo(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int32) for k in ("path", "limbs", "bn", "tile_rows", "tile_cols", "patch_rows",
                                               "patch_cols", "tiles_m", "tiles_n", "lds_bytes", "patch_pitch", "patch_pixel",
                                               "workgroups", "split", "items_per_die", "whole_items_per_die", "kernel")]

    def asdict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class ZeroMap(ctypes.Structure):
    """Per-tile nonzero flags of a tensor and the tile geometry they were written in (lp_zero_map)."""
    _fields_ = [("flags_dev", ctypes.c_void_p)] + [(k, ctypes.c_int32) for k in ("tile_rows", "tile_cols", "tiles_c", "tiles_n",
                                                                             "bn", "scale")]


class ConvDesc(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int32) for k in ("N", "H", "W", "Cin", "Cout", "R", "S", "stride", "pad", "pool")]


_SIGNATURES = {
    "lp_status_string": (ctypes.c_char_p, [ctypes.c_int]),
    "lp_range": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_double,
                                ctypes.POINTER(QFmt), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]),
    "lp_range_acc": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                    ctypes.c_double, ctypes.POINTER(QFmt), ctypes.c_void_p, ctypes.c_void_p,
                                    ctypes.c_void_p]),
    "lp_quantize": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, QFmt, ctypes.c_int,
                                   ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]),
    "lp_act": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, QFmt, ctypes.c_int, ctypes.c_int,
                              ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]),
    "lp_act_stochastic": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, QFmt, ctypes.c_int,
                                         ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_void_p]),
    "lp_conv_packed_bytes": (ctypes.c_int, [ctypes.POINTER(ConvDesc), QFmt, QFmt, ctypes.POINTER(ctypes.c_size_t)]),
    "lp_conv_plan_info": (ctypes.c_int, [ctypes.POINTER(ConvDesc), QFmt, QFmt, ctypes.POINTER(PlanInfo)]),
    "lp_conv_pack_weights": (ctypes.c_int, [ctypes.POINTER(ConvDesc), QFmt, QFmt, ctypes.c_void_p, ctypes.c_void_p,
                                            ctypes.c_size_t, ctypes.c_void_p]),
    "lp_conv_pool_check": (ctypes.c_int, [ctypes.POINTER(ConvDesc), QFmt, QFmt, ctypes.c_int, QFmt, QFmt, ctypes.c_int,
                                          ctypes.c_int]),
    "lp_conv_workspace_bytes": (ctypes.c_int, [ctypes.POINTER(ConvDesc), QFmt, QFmt,
                                               ctypes.POINTER(ctypes.c_size_t)]),
    "lp_conv_fwd": (ctypes.c_int, [ctypes.POINTER(ConvDesc), ctypes.c_void_p, QFmt, ctypes.c_void_p, QFmt,
                                   ctypes.c_void_p, QFmt, ctypes.c_void_p, ctypes.c_void_p, QFmt, ctypes.c_int,
                                   ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                   ctypes.c_void_p]),
    "lp_conv_fwd_zskip": (ctypes.c_int, [ctypes.POINTER(ConvDesc), ctypes.c_void_p, QFmt, ctypes.POINTER(ZeroMap),
                                         ctypes.c_void_p, QFmt, ctypes.c_void_p, QFmt, ctypes.c_void_p, QFmt, ctypes.c_int,
                                         ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "lp_conv_fwd_static": (ctypes.c_int, [ctypes.POINTER(ConvDesc), ctypes.c_void_p, QFmt, ctypes.c_void_p, QFmt,
                                          ctypes.c_void_p, QFmt, ctypes.c_void_p, ctypes.c_void_p, QFmt, ctypes.c_int,
                                          ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]),
    "lp_fc_packed_bytes": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, ctypes.c_int, QFmt, QFmt,
                                          ctypes.POINTER(ctypes.c_size_t)]),
    "lp_fc_pack_weights": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, ctypes.c_int, QFmt, QFmt, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "lp_fc_workspace_bytes": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, ctypes.c_int, QFmt, QFmt,
                                             ctypes.POINTER(ctypes.c_size_t)]),
    "lp_fc_fwd": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, QFmt, ctypes.c_void_p,
                                 QFmt, ctypes.c_void_p, QFmt, ctypes.c_void_p, ctypes.c_void_p, QFmt, ctypes.c_int,
                                 ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                 ctypes.c_void_p]),
    "lp_maxpool2x2": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_int, ctypes.c_int, ctypes.c_void_p]),
}


def lib_path():
    return _LIB_PATH


def exported_symbols():
    return sorted(_SIGNATURES)


def load():
    """Load liblp.so (built beforehand by build.py); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError("liblp.so is not built: run `python -m paper_1711_04713_amd.build` "
                               "(there is no fallback path)")
        lib = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def lp_status_string(status):
    return load().lp_status_string(int(status)).decode()


def _check(status, what):
    if status != 0:
        raise LpError(status, what)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch

    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _q(q):
    return q if isinstance(q, QFmt) else QFmt(*q)


def lp_range(x, n, loss_threshold=0.0, workspace=None):
    """x: float32 CUDA tensor.  Returns (QFmt, lost list with lost[m] for m=1..n)."""
    import torch

    ws = workspace if workspace is not None else torch.empty(LP_RANGE_WORKSPACE_WORDS, dtype=torch.int64, device=x.device)
    out = QFmt()
    lost = (ctypes.c_uint64 * (n + 1))()
    _check(load().lp_range(_ptr(x), x.numel(), n, loss_threshold, ctypes.byref(out), lost, _ptr(ws), _stream()),
           "lp_range")
    return out, list(lost)


def lp_range_acc(acc, f_acc, relu, n, loss_threshold=0.0, workspace=None):
    import torch

    ws = workspace if workspace is not None else torch.empty(LP_RANGE_WORKSPACE_WORDS, dtype=torch.int64, device=acc.device)
    out = QFmt()
    lost = (ctypes.c_uint64 * (n + 1))()
    _check(load().lp_range_acc(_ptr(acc), acc.numel(), f_acc, int(bool(relu)), n, loss_threshold, ctypes.byref(out),
                               lost, _ptr(ws), _stream()), "lp_range_acc")
    return out, list(lost)


def lp_quantize(x, codes, q, r=LP_ROUND_NEAREST_AWAY, seed=0, zero_count=None, sat_count=None):
    _check(load().lp_quantize(_ptr(x), _ptr(codes), x.numel(), _q(q), r, seed, _ptr(zero_count), _ptr(sat_count),
                              _stream()), "lp_quantize")


def lp_act(acc, f_acc, qy, relu, y_codes, r=LP_ROUND_NEAREST_AWAY, zero_count=None, sat_count=None):
    _check(load().lp_act(_ptr(acc), acc.numel(), f_acc, _q(qy), int(bool(relu)), r, _ptr(y_codes), _ptr(zero_count),
                         _ptr(sat_count), _stream()), "lp_act")


def lp_act_stochastic(acc, f_acc, qy, relu, seed, y_codes, zero_count=None, sat_count=None):
    _check(load().lp_act_stochastic(_ptr(acc), acc.numel(), f_acc, _q(qy), int(bool(relu)), seed, _ptr(y_codes),
                                    _ptr(zero_count), _ptr(sat_count), _stream()), "lp_act_stochastic")


def lp_conv_packed_bytes(desc, qx, qw):
    n = ctypes.c_size_t(0)
    _check(load().lp_conv_packed_bytes(ctypes.byref(desc), _q(qx), _q(qw), ctypes.byref(n)), "lp_conv_packed_bytes")
    return n.value


def lp_conv_plan_info(desc, qx, qw):
    out = PlanInfo()
    _check(load().lp_conv_plan_info(ctypes.byref(desc), _q(qx), _q(qw), ctypes.byref(out)), "lp_conv_plan_info")
    return out.asdict()


def lp_conv_pool_check(desc, qx, qw, qy, relu=True, r=LP_ROUND_NEAREST_AWAY, qb=None):
    """True if lp_conv_fwd takes this call with desc.pool = 1."""
    status = load().lp_conv_pool_check(ctypes.byref(desc), _q(qx), _q(qw), int(qb is not None),
                                       _q(qb) if qb is not None else QFmt(), _q(qy), int(bool(relu)), r)
    if status not in (0, 2):
        raise LpError(status, "lp_conv_pool_check")
    return status == 0


def lp_conv_pack_weights(desc, qx, qw, w_codes, packed):
    _check(load().lp_conv_pack_weights(ctypes.byref(desc), _q(qx), _q(qw), _ptr(w_codes), _ptr(packed),
                                       packed.numel() * packed.element_size(), _stream()), "lp_conv_pack_weights")


def lp_conv_workspace_bytes(desc, qx, qw):
    n = ctypes.c_size_t(0)
    _check(load().lp_conv_workspace_bytes(ctypes.byref(desc), _q(qx), _q(qw), ctypes.byref(n)),
           "lp_conv_workspace_bytes")
    return n.value


def lp_conv_fwd(desc, x_codes, qx, w_packed, qw, qy=None, y_codes=None, acc_out=None, relu=True,
                r=LP_ROUND_NEAREST_AWAY, bias_codes=None, qb=None, zero_count=None, workspace=None, sat_count=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().lp_conv_fwd(ctypes.byref(desc), _ptr(x_codes), _q(qx), _ptr(w_packed), _q(qw), _ptr(bias_codes),
                              _q(qb) if qb is not None else QFmt(), _ptr(acc_out), _ptr(y_codes),
                              _q(qy) if qy is not None else QFmt(), int(bool(relu)), r, _ptr(zero_count),
                              _ptr(sat_count), _ptr(workspace), ws_bytes, _stream()), "lp_conv_fwd")


def zero_map(flags, producer_info, Wo, scale=1):
    """lp_zero_map for a tensor whose producer (plan info producer_info, output width Wo) wrote `flags`;
    scale = 2 when the tensor was 2x2-pooled after the flags were taken."""
    return ZeroMap(flags.data_ptr(), producer_info["tile_rows"], producer_info["tile_cols"],
                   (Wo + producer_info["tile_cols"] - 1) // producer_info["tile_cols"], producer_info["tiles_n"],
                   producer_info["bn"], scale)


def lp_conv_fwd_zskip(desc, x_codes, qx, x_map, w_packed, qw, qy, y_codes, relu=True, r=LP_ROUND_NEAREST_AWAY,
                      bias_codes=None, qb=None, zero_count=None, sat_count=None, y_flags=None, skipped=None,
                      workspace=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().lp_conv_fwd_zskip(ctypes.byref(desc), _ptr(x_codes), _q(qx), ctypes.byref(x_map) if x_map is not None else None,
                                    _ptr(w_packed), _q(qw), _ptr(bias_codes), _q(qb) if qb is not None else QFmt(),
                                    _ptr(y_codes), _q(qy), int(bool(relu)), r, _ptr(zero_count), _ptr(sat_count),
                                    _ptr(y_flags), _ptr(skipped), _ptr(workspace), ws_bytes, _stream()),
           "lp_conv_fwd_zskip")


LP_STATIC_WORKSPACE_BYTES = 64 << 20


def lp_conv_fwd_static(desc, x_codes, qx, w_packed, qw, qy=None, y_codes=None, acc_out=None, relu=True,
                       r=LP_ROUND_NEAREST_AWAY, bias_codes=None, qb=None, zero_count=None, sat_count=None):
    _check(load().lp_conv_fwd_static(ctypes.byref(desc), _ptr(x_codes), _q(qx), _ptr(w_packed), _q(qw),
                                     _ptr(bias_codes), _q(qb) if qb is not None else QFmt(), _ptr(acc_out),
                                     _ptr(y_codes), _q(qy) if qy is not None else QFmt(), int(bool(relu)), r,
                                     _ptr(zero_count), _ptr(sat_count), _stream()), "lp_conv_fwd_static")


def lp_fc_packed_bytes(M, K, Nout, qx, qw):
    n = ctypes.c_size_t(0)
    _check(load().lp_fc_packed_bytes(M, K, Nout, _q(qx), _q(qw), ctypes.byref(n)), "lp_fc_packed_bytes")
    return n.value


def lp_fc_pack_weights(M, K, Nout, qx, qw, w_codes, packed):
    _check(load().lp_fc_pack_weights(M, K, Nout, _q(qx), _q(qw), _ptr(w_codes), _ptr(packed),
                                     packed.numel() * packed.element_size(), _stream()), "lp_fc_pack_weights")


def lp_fc_workspace_bytes(M, K, Nout, qx, qw):
    n = ctypes.c_size_t(0)
    _check(load().lp_fc_workspace_bytes(M, K, Nout, _q(qx), _q(qw), ctypes.byref(n)), "lp_fc_workspace_bytes")
    return n.value


def lp_fc_fwd(M, K, Nout, x_codes, qx, w_packed, qw, qy=None, y_codes=None, acc_out=None, relu=True,
              r=LP_ROUND_NEAREST_AWAY, bias_codes=None, qb=None, zero_count=None, workspace=None, sat_count=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().lp_fc_fwd(M, K, Nout, _ptr(x_codes), _q(qx), _ptr(w_packed), _q(qw), _ptr(bias_codes),
                            _q(qb) if qb is not None else QFmt(), _ptr(acc_out), _ptr(y_codes),
                            _q(qy) if qy is not None else QFmt(), int(bool(relu)), r, _ptr(zero_count),
                            _ptr(sat_count), _ptr(workspace), ws_bytes, _stream()), "lp_fc_fwd")


def lp_maxpool2x2(x_codes, y_codes, N, H, W, C, n_bits):
    _check(load().lp_maxpool2x2(_ptr(x_codes), _ptr(y_codes), N, H, W, C, n_bits, _stream()), "lp_maxpool2x2")
