"""ctypes front end of oracle/lp_oracle.c (numpy arrays in, numpy arrays out).

TEST INFRASTRUCTURE ONLY.  Holds no arithmetic of the method: every number is
produced by the C file.  Tensors are NCHW / [Cout][Cin][R][S]; codes are int32,
accumulators int64.
"""
import ctypes
import os
import subprocess

import numpy as np

ROUND_AWAY = 0
ROUND_EVEN = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lp_oracle.c")
_LIB = os.path.join(_HERE, "liblp_oracle.so")
_lib = None


def build(force=True):
    """Compile lp_oracle.c with gcc -O2 (+OpenMP over the outermost loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


class _ConvShape(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int) for k in ("N", "Cin", "H", "W", "Cout", "R", "S", "stride", "pad")]


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(_LIB)
        _lib.orc_num_threads.restype = ctypes.c_int
    return _lib


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _check(rc, what):
    if rc != 0:
        raise ValueError("oracle %s rejected its arguments (rc=%d)" % (what, rc))


def num_threads():
    return int(_load().orc_num_threads())


def quantize(x, n, m, f, mode=ROUND_AWAY):
    """float32 array -> (int32 codes of the same shape, zero_count, sat_count)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    code = np.empty(x.shape, dtype=np.int32)
    z, s = ctypes.c_uint64(0), ctypes.c_uint64(0)
    rc = _load().orc_quantize(_ptr(x), ctypes.c_int64(x.size), n, m, f, mode, _ptr(code),
                              ctypes.byref(z), ctypes.byref(s))
    _check(rc, "quantize")
    return code, int(z.value), int(s.value)


def quantize_stochastic(x, u, n, m, f):
    """u: float64 uniforms in [0,1), one per element."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = np.ascontiguousarray(u, dtype=np.float64)
    assert u.shape == x.shape
    code = np.empty(x.shape, dtype=np.int32)
    z, s = ctypes.c_uint64(0), ctypes.c_uint64(0)
    rc = _load().orc_quantize_stochastic(_ptr(x), _ptr(u), ctypes.c_int64(x.size), n, m, f,
                                         _ptr(code), ctypes.byref(z), ctypes.byref(s))
    _check(rc, "quantize_stochastic")
    return code, int(z.value), int(s.value)


def range_float(v, n, threshold=0.0):
    """-> (m, lost) with lost[m] = number of |v| >= 2^(m-1), m = 1..n (lost[0] unused)."""
    v = np.ascontiguousarray(v, dtype=np.float32)
    lost = np.zeros(n + 1, dtype=np.uint64)
    m = ctypes.c_int(0)
    rc = _load().orc_range(_ptr(v), ctypes.c_int64(v.size), n, ctypes.c_double(threshold),
                           ctypes.byref(m), _ptr(lost))
    _check(rc, "range")
    return int(m.value), lost


def range_acc(acc, f_acc, relu, n, threshold=0.0):
    acc = np.ascontiguousarray(acc, dtype=np.int64)
    lost = np.zeros(n + 1, dtype=np.uint64)
    m = ctypes.c_int(0)
    rc = _load().orc_range_acc(_ptr(acc), ctypes.c_int64(acc.size), f_acc, int(bool(relu)), n,
                               ctypes.c_double(threshold), ctypes.byref(m), _ptr(lost))
    _check(rc, "range_acc")
    return int(m.value), lost


def _shape(x, w, stride, pad):
    N, Cin, H, W = x.shape
    Cout, Cin2, R, S = w.shape
    if Cin != Cin2:
        raise ValueError("channel mismatch")
    cs = _ConvShape(N, Cin, H, W, Cout, R, S, stride, pad)
    Ho, Wo = ctypes.c_int(0), ctypes.c_int(0)
    _check(_load().orc_conv_out_hw(ctypes.byref(cs), ctypes.byref(Ho), ctypes.byref(Wo)), "conv shape")
    return cs, Ho.value, Wo.value


def conv(x, w, bias=None, f_acc=0, fb=0, stride=1, pad=1, threads=1):
    """x [N,Cin,H,W], w [Cout,Cin,R,S] int codes -> int64 acc [N,Cout,Ho,Wo]."""
    x, w, bias = _i32(x), _i32(w), _i32(bias)
    cs, Ho, Wo = _shape(x, w, stride, pad)
    acc = np.empty((cs.N, cs.Cout, Ho, Wo), dtype=np.int64)
    rc = _load().orc_conv(ctypes.byref(cs), _ptr(x), _ptr(w), _ptr(bias), f_acc, fb, _ptr(acc),
                          int(threads))
    _check(rc, "conv")
    return acc


def conv_sampled(x, w, flat_index, bias=None, f_acc=0, fb=0, stride=1, pad=1):
    """Accumulators at flat indices into the [N,Cout,Ho,Wo] output only."""
    x, w, bias = _i32(x), _i32(w), _i32(bias)
    cs, _, _ = _shape(x, w, stride, pad)
    idx = np.ascontiguousarray(flat_index, dtype=np.int64)
    acc = np.empty(idx.shape, dtype=np.int64)
    rc = _load().orc_conv_sampled(ctypes.byref(cs), _ptr(x), _ptr(w), _ptr(bias), f_acc, fb,
                                  _ptr(idx), ctypes.c_int64(idx.size), _ptr(acc))
    _check(rc, "conv_sampled")
    return acc


def fc(x, w, bias=None, f_acc=0, fb=0, threads=1):
    """x [M,K], w [Nout,K] int codes -> int64 acc [M,Nout]."""
    x, w, bias = _i32(x), _i32(w), _i32(bias)
    M, K = x.shape
    Nout, K2 = w.shape
    if K != K2:
        raise ValueError("K mismatch")
    acc = np.empty((M, Nout), dtype=np.int64)
    rc = _load().orc_fc(M, K, Nout, _ptr(x), _ptr(w), _ptr(bias), f_acc, fb, _ptr(acc), int(threads))
    _check(rc, "fc")
    return acc


def act(acc, f_acc, n, m, fo, relu=True, mode=ROUND_AWAY, with_sat=False):
    """int64 accumulators -> (int32 codes, zero_count), plus the count of clipped values if with_sat."""
    acc = np.ascontiguousarray(acc, dtype=np.int64)
    code = np.empty(acc.shape, dtype=np.int32)
    z, s = ctypes.c_uint64(0), ctypes.c_uint64(0)
    rc = _load().orc_act(_ptr(acc), ctypes.c_int64(acc.size), f_acc, n, m, fo, int(bool(relu)), mode,
                         _ptr(code), ctypes.byref(z), ctypes.byref(s))
    _check(rc, "act")
    return (code, int(z.value), int(s.value)) if with_sat else (code, int(z.value))


def act_stochastic(acc, u, f_acc, n, m, fo, relu=True, with_sat=False):
    """int64 accumulators, u in [0,1) per element -> (int32 codes, zero_count) (Sec. 2.4), plus the
    count of clipped values if with_sat."""
    acc = np.ascontiguousarray(acc, dtype=np.int64)
    u = np.ascontiguousarray(u, dtype=np.float64)
    assert u.shape == acc.shape
    code = np.empty(acc.shape, dtype=np.int32)
    z, s = ctypes.c_uint64(0), ctypes.c_uint64(0)
    rc = _load().orc_act_stochastic(_ptr(acc), _ptr(u), ctypes.c_int64(acc.size), f_acc, n, m, fo,
                                    int(bool(relu)), _ptr(code), ctypes.byref(z), ctypes.byref(s))
    _check(rc, "act_stochastic")
    return (code, int(z.value), int(s.value)) if with_sat else (code, int(z.value))


def maxpool2x2(x):
    x = _i32(x)
    N, C, H, W = x.shape
    y = np.empty((N, C, H // 2, W // 2), dtype=np.int32)
    _check(_load().orc_maxpool2x2(_ptr(x), N, C, H, W, _ptr(y)), "maxpool2x2")
    return y
