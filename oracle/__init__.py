"""CPU oracle for the mixed-precision training hot path -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It shares nothing with the HIP library and never imports it.

* conv / FC: fp64 direct definitions in C (``jz_oracle.c``), called via ctypes; inputs are fp16 bit patterns (the
  mixed-precision path) or float32 arrays (the single-precision variant of Section 5.4 / Table 9): same loops.
* LARS: the mixed-precision update of Section 4.1 / Eq. 1, step by step in
  fp64 numpy (``lars.py``).
* the dynamic loss-scale controller around that update (``loss_scale.py``).
* batch normalization + ReLU (Section 4.2's formulas) and its gradient, fp64 numpy (``bn.py``).
* the small layers between the convolutions (residual add, pooling, bias, softmax loss), fp64 numpy (``layers.py``).
"""
import ctypes
import os

import numpy as np

from .bn import bn_add_relu_fwd, bn_relu_bwd, bn_relu_fwd  # noqa: F401
from .layers import (add_fwd, avgpool_bwd, avgpool_fwd, bias_add, bias_grad, maxpool_bwd, maxpool_fwd, pool_out,  # noqa: F401
                     relu_bwd, softmax_xent)
from .lars import lars_mp_update, lars_trust_ratio  # noqa: F401
from .loss_scale import loss_scale_step  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class ConvDesc(ctypes.Structure):
    """x[N,H,W,C] (*) w[K,R,S,C] -> y[N,P,Q,K]; dilation 1, groups 1."""

    _fields_ = [(n, ctypes.c_int) for n in ("N", "H", "W", "C", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w")]

    @property
    def P(self):
        return (self.H + 2 * self.pad_h - self.R) // self.stride_h + 1

    @property
    def Q(self):
        return (self.W + 2 * self.pad_w - self.S) // self.stride_w + 1


def conv_desc(N, H, W, C, K, R, S, stride=1, pad=0):
    sh, sw = (stride, stride) if isinstance(stride, int) else stride
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    return ConvDesc(N, H, W, C, K, R, S, sh, sw, ph, pw)


def lib():
    global _LIB
    if _LIB is None:
        path = os.path.join(_HERE, "liborc.so")
        if not os.path.exists(path):
            from .build_oracle import build

            build()
        L = ctypes.CDLL(path)
        L.orc_half_to_double.restype = ctypes.c_double
        L.orc_half_to_double.argtypes = [ctypes.c_uint16]
        L.orc_double_to_half.restype = ctypes.c_uint16
        L.orc_double_to_half.argtypes = [ctypes.c_double]
        L.orc_num_threads.restype = ctypes.c_int
        _LIB = L
    return _LIB


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _bits(a) -> np.ndarray:
    """fp16 data as a contiguous uint16 array (accepts float16 or uint16)."""
    a = np.asarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError("oracle inputs must be fp16 bit patterns (float16 or uint16), got %s" % a.dtype)
    return np.ascontiguousarray(a)


def _p(a, ty):
    return a.ctypes.data_as(ctypes.POINTER(ty))


def _chk(a, n, what):
    if a.size != n:
        raise ValueError("%s has %d elements, descriptor needs %d" % (what, a.size, n))


def half_to_double(bits) -> np.ndarray:
    b = _bits(bits)
    out = np.empty(b.shape, np.float64)
    lib().orc_halves_to_doubles(_p(b, ctypes.c_uint16), _p(out, ctypes.c_double), ctypes.c_int64(b.size))
    return out


def round_to_half(values) -> np.ndarray:
    """RNE16 of fp64 values, one rounding; returns uint16 bit patterns."""
    v = np.ascontiguousarray(values, dtype=np.float64)
    out = np.empty(v.shape, np.uint16)
    lib().orc_doubles_to_halves(_p(v, ctypes.c_double), _p(out, ctypes.c_uint16), ctypes.c_int64(v.size))
    return out


def _operands(a, b):
    """Two inputs of one dtype: fp16 (float16 or uint16 bit patterns) or float32.  Returns (a, b, ctype, name suffix)."""
    a, b = np.asarray(a), np.asarray(b)
    if a.dtype == np.float32 or b.dtype == np.float32:
        if a.dtype != np.float32 or b.dtype != np.float32:
            raise TypeError("oracle inputs must both be float32 or both be fp16, got %s and %s" % (a.dtype, b.dtype))
        return np.ascontiguousarray(a), np.ascontiguousarray(b), ctypes.c_float, "_f32"
    return _bits(a), _bits(b), ctypes.c_uint16, ""


def conv_fwd(d: ConvDesc, x, w) -> np.ndarray:
    x, w, ty, sfx = _operands(x, w)
    _chk(x, d.N * d.H * d.W * d.C, "x")
    _chk(w, d.K * d.R * d.S * d.C, "w")
    y = np.empty((d.N, d.P, d.Q, d.K), np.float64)
    rc = getattr(lib(), "orc_conv_fwd" + sfx)(ctypes.byref(d), _p(x, ty), _p(w, ty), _p(y, ctypes.c_double))
    assert rc == 0
    return y


def conv_bwd_data(d: ConvDesc, dy, w) -> np.ndarray:
    dy, w, ty, sfx = _operands(dy, w)
    _chk(dy, d.N * d.P * d.Q * d.K, "dy")
    _chk(w, d.K * d.R * d.S * d.C, "w")
    dx = np.empty((d.N, d.H, d.W, d.C), np.float64)
    rc = getattr(lib(), "orc_conv_bwd_data" + sfx)(ctypes.byref(d), _p(dy, ty), _p(w, ty), _p(dx, ctypes.c_double))
    assert rc == 0
    return dx


def conv_bwd_weight(d: ConvDesc, x, dy) -> np.ndarray:
    x, dy, ty, sfx = _operands(x, dy)
    _chk(x, d.N * d.H * d.W * d.C, "x")
    _chk(dy, d.N * d.P * d.Q * d.K, "dy")
    dw = np.empty((d.K, d.R, d.S, d.C), np.float64)
    rc = getattr(lib(), "orc_conv_bwd_weight" + sfx)(ctypes.byref(d), _p(x, ty), _p(dy, ty), _p(dw, ctypes.c_double))
    assert rc == 0
    return dw


def _at(name, d, a, b, idx):
    a, b, ty, sfx = _operands(a, b)
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty(idx.shape, np.float64)
    rc = getattr(lib(), name + sfx)(ctypes.byref(d), _p(a, ty), _p(b, ty), _p(idx, ctypes.c_int64), ctypes.c_int64(idx.size),
                                    _p(out, ctypes.c_double))
    assert rc == 0
    return out


def conv_fwd_at(d, x, w, flat_idx):
    """Selected elements of y (flat NPQK indices), each by the plain definition."""
    _chk(np.asarray(x), d.N * d.H * d.W * d.C, "x")
    _chk(np.asarray(w), d.K * d.R * d.S * d.C, "w")
    return _at("orc_conv_fwd_at", d, x, w, flat_idx)


def conv_bwd_data_at(d, dy, w, flat_idx):
    """Selected elements of dx (flat NHWC indices)."""
    _chk(np.asarray(dy), d.N * d.P * d.Q * d.K, "dy")
    _chk(np.asarray(w), d.K * d.R * d.S * d.C, "w")
    return _at("orc_conv_bwd_data_at", d, dy, w, flat_idx)


def conv_bwd_weight_at(d, x, dy, flat_idx):
    """Selected elements of dw (flat KRSC indices)."""
    _chk(np.asarray(x), d.N * d.H * d.W * d.C, "x")
    _chk(np.asarray(dy), d.N * d.P * d.Q * d.K, "dy")
    return _at("orc_conv_bwd_weight_at", d, x, dy, flat_idx)


def fc_fwd(B, I, O, x, w) -> np.ndarray:
    x, w, ty, sfx = _operands(x, w)
    _chk(x, B * I, "x")
    _chk(w, O * I, "w")
    y = np.empty((B, O), np.float64)
    assert getattr(lib(), "orc_fc_fwd" + sfx)(B, I, O, _p(x, ty), _p(w, ty), _p(y, ctypes.c_double)) == 0
    return y


def fc_bwd_data(B, I, O, dy, w) -> np.ndarray:
    dy, w, ty, sfx = _operands(dy, w)
    _chk(dy, B * O, "dy")
    _chk(w, O * I, "w")
    dx = np.empty((B, I), np.float64)
    assert getattr(lib(), "orc_fc_bwd_data" + sfx)(B, I, O, _p(dy, ty), _p(w, ty), _p(dx, ctypes.c_double)) == 0
    return dx


def fc_bwd_weight(B, I, O, dy, x) -> np.ndarray:
    dy, x, ty, sfx = _operands(dy, x)
    _chk(dy, B * O, "dy")
    _chk(x, B * I, "x")
    dw = np.empty((O, I), np.float64)
    assert getattr(lib(), "orc_fc_bwd_weight" + sfx)(B, I, O, _p(dy, ty), _p(x, ty), _p(dw, ctypes.c_double)) == 0
    return dw
