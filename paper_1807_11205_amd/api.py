"""Thin ctypes binding of libjz (include/jz.h): same entry-point names, argument marshalling only.

torch is used for device memory and streams; every arithmetic step runs in the HIP kernels of
libjz.so.  There is no CPU fallback: if the library has not been built, loading raises.
"""
import ctypes
import os
from typing import Optional, Sequence

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("JZ_LIB_PATH", os.path.join(_PKG, "libjz.so"))

JZ_OK = 0
JZ_ERR_NULL, JZ_ERR_SHAPE, JZ_ERR_UNSUPPORTED, JZ_ERR_WORKSPACE = -1, -2, -3, -4
JZ_ERR_ALIGN, JZ_ERR_ALIAS, JZ_ERR_LAUNCH, JZ_ERR_NOT_PREPARED = -5, -6, -7, -8
JZ_FWD, JZ_BWD_DATA, JZ_BWD_WEIGHT = 0, 1, 2
JZ_PARAM_WEIGHT_DECAY, JZ_PARAM_LARS, JZ_PARAM_GRAD_PRESUMMED = 1, 2, 4

EXPORTS = [
    "jz_conv2d_workspace_bytes", "jz_conv2d_describe_plan", "jz_conv2d_tune_set", "jz_conv2d_tune_use_table", "jz_conv2d_tune_clear", "jz_conv2d_fwd", "jz_conv2d_bwd_data", "jz_conv2d_bwd_weight", "jz_conv2d_bwd_weight_static",
    "jz_conv2d_bwd_weight_sumsq", "jz_gemm_fc_workspace_bytes", "jz_gemm_fc", "jz_gemm_fc_bwd_weight_sumsq",
    "jz_conv2d_f32_workspace_bytes", "jz_conv2d_fwd_f32", "jz_conv2d_bwd_data_f32", "jz_conv2d_bwd_weight_f32",
    "jz_gemm_fc_f32_workspace_bytes", "jz_gemm_fc_f32",
    "jz_lars_workspace_bytes", "jz_lars_prepare", "jz_lars_mp_update", "jz_loss_scale_init", "jz_lars_mp_update_dyn",
    "jz_lars_begin_step", "jz_lars_sumsq_sink", "jz_lars_grad_sumsq", "jz_lars_mp_update_presummed", "jz_lars_mp_update_presummed_dyn",
    "jz_add_fwd", "jz_relu_bwd", "jz_relu_bwd_sum", "jz_maxpool_fwd", "jz_maxpool_bwd", "jz_avgpool_fwd", "jz_avgpool_bwd", "jz_bias_add",
    "jz_bias_grad", "jz_softmax_xent_bwd", "jz_conv2d_bn_relu_fwd_workspace_bytes", "jz_conv2d_bn_relu_fwd",
    "jz_conv2d_bwd_data_bn_relu_bwd_workspace_bytes", "jz_conv2d_bwd_data_bn_relu_bwd", "jz_conv2d_bwd_data_block_end_bwd",
    "jz_bn_workspace_bytes", "jz_bn_relu_fwd", "jz_bn_relu_bwd", "jz_bn_bwd_block_end",
    "jz_status_string", "jz_version",
]


class JzError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s" % (where, status_string(status)))


class jz_conv_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("N", "H", "W", "C", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w")]

    @property
    def P(self):
        return (self.H + 2 * self.pad_h - self.R) // self.stride_h + 1

    @property
    def Q(self):
        return (self.W + 2 * self.pad_w - self.S) // self.stride_w + 1


class jz_lars_hparams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_float) for n in ("lr", "momentum", "weight_decay", "trust_coef", "loss_scale")]


class jz_loss_scale_policy(ctypes.Structure):
    _fields_ = [("growth_factor", ctypes.c_float), ("backoff_factor", ctypes.c_float), ("growth_interval", ctypes.c_int),
                ("min_scale", ctypes.c_float), ("max_scale", ctypes.c_float)]


class jz_sumsq_sink(ctypes.Structure):
    _fields_ = [("sums", ctypes.c_void_p), ("nonfinite", ctypes.c_void_p)]


JZ_SUMSQ_SINK_BYTES = 8192


class jz_param_set(ctypes.Structure):
    _fields_ = [
        ("num_tensors", ctypes.c_int64),
        ("offsets", ctypes.POINTER(ctypes.c_int64)),
        ("flags", ctypes.POINTER(ctypes.c_uint8)),
        ("master_w", ctypes.c_void_p),
        ("momentum", ctypes.c_void_p),
        ("grad16", ctypes.c_void_p),
        ("weight16", ctypes.c_void_p),
    ]


_lib = None


def lib() -> ctypes.CDLL:
    """Open libjz.so; raises (never falls back) when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libjz.so is not built: run `python -m paper_1807_11205_amd.build` (needs hipcc)")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        dp = ctypes.POINTER(jz_conv_desc)
        L.jz_conv2d_workspace_bytes.argtypes = [ci, dp, ctypes.POINTER(sz)]
        L.jz_conv2d_describe_plan.argtypes = [ci, dp, ctypes.c_char_p, sz]
        L.jz_conv2d_tune_set.argtypes = [ci, dp, ci, ci, ci, ci, ci, ci]
        L.jz_conv2d_tune_use_table.argtypes = [ci]
        L.jz_conv2d_tune_clear.argtypes = []
        for name in ("jz_conv2d_fwd", "jz_conv2d_bwd_data", "jz_conv2d_bwd_weight"):
            getattr(L, name).argtypes = [dp, vp, vp, vp, vp, sz, vp]
        L.jz_conv2d_bwd_weight_static.argtypes = [dp, vp, vp, vp, vp]
        sk = ctypes.POINTER(jz_sumsq_sink)
        L.jz_conv2d_bwd_weight_sumsq.argtypes = [dp, vp, vp, vp, vp, sz, sk, vp]
        L.jz_gemm_fc_bwd_weight_sumsq.argtypes = [ci, ci, ci, vp, vp, vp, vp, sz, sk, vp]
        L.jz_conv2d_f32_workspace_bytes.argtypes = [ci, dp, ctypes.POINTER(sz)]
        for name in ("jz_conv2d_fwd_f32", "jz_conv2d_bwd_data_f32", "jz_conv2d_bwd_weight_f32"):
            getattr(L, name).argtypes = [dp, vp, vp, vp, vp, sz, vp]
        L.jz_gemm_fc_f32_workspace_bytes.argtypes = [ci, ci, ci, ci, ctypes.POINTER(sz)]
        L.jz_gemm_fc_f32.argtypes = [ci, ci, ci, ci, vp, vp, vp, vp, sz, vp]
        L.jz_gemm_fc_workspace_bytes.argtypes = [ci, ci, ci, ci, ctypes.POINTER(sz)]
        L.jz_gemm_fc.argtypes = [ci, ci, ci, ci, vp, vp, vp, vp, sz, vp]
        pp = ctypes.POINTER(jz_param_set)
        L.jz_lars_workspace_bytes.argtypes = [pp, ctypes.POINTER(sz)]
        L.jz_lars_prepare.argtypes = [pp, vp, sz, vp]
        L.jz_lars_mp_update.argtypes = [pp, ctypes.POINTER(jz_lars_hparams), vp, vp, sz, vp]
        L.jz_loss_scale_init.argtypes = [vp, ctypes.c_float, vp]
        L.jz_lars_mp_update_dyn.argtypes = [pp, ctypes.POINTER(jz_lars_hparams), ctypes.POINTER(jz_loss_scale_policy), vp, vp,
                                            vp, sz, vp]
        i64, cf = ctypes.c_int64, ctypes.c_float
        L.jz_lars_begin_step.argtypes = [pp, vp, vp, sz, vp]
        L.jz_lars_sumsq_sink.argtypes = [pp, vp, sz, i64, sk]
        L.jz_lars_grad_sumsq.argtypes = [pp, i64, i64, vp, sz, vp]
        L.jz_lars_mp_update_presummed.argtypes = [pp, ctypes.POINTER(jz_lars_hparams), vp, vp, sz, vp]
        L.jz_lars_mp_update_presummed_dyn.argtypes = [pp, ctypes.POINTER(jz_lars_hparams), ctypes.POINTER(jz_loss_scale_policy), vp, vp,
                                                      vp, sz, vp]
        L.jz_bn_workspace_bytes.argtypes = [i64, ci, ctypes.POINTER(sz)]
        L.jz_bn_relu_fwd.argtypes = [i64, ci, vp, vp, vp, cf, ci, vp, vp, vp, vp, sz, vp]
        L.jz_bn_relu_bwd.argtypes = [i64, ci, vp, vp, vp, vp, vp, vp, ci, vp, vp, vp, vp, sz, vp]
        L.jz_add_fwd.argtypes = [i64, vp, vp, ci, vp, vp]
        L.jz_bn_bwd_block_end.argtypes = [i64, ci, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.jz_relu_bwd.argtypes = [i64, vp, vp, vp, vp]
        L.jz_relu_bwd_sum.argtypes = [i64, vp, vp, vp, vp, vp]
        L.jz_maxpool_fwd.argtypes = [ci] * 7 + [vp, vp, vp, vp]
        L.jz_maxpool_bwd.argtypes = [ci] * 7 + [vp, vp, vp, vp, vp]
        L.jz_avgpool_fwd.argtypes = [ci, ci, ci, vp, vp, vp]
        L.jz_avgpool_bwd.argtypes = [ci, ci, ci, vp, vp, vp]
        L.jz_bias_add.argtypes = [i64, ci, vp, vp, vp, vp]
        L.jz_bias_grad.argtypes = [i64, ci, vp, vp, vp]
        L.jz_softmax_xent_bwd.argtypes = [ci, ci, vp, vp, cf, vp, vp, vp, vp]
        L.jz_conv2d_bn_relu_fwd_workspace_bytes.argtypes = [dp, ctypes.POINTER(sz)]
        L.jz_conv2d_bn_relu_fwd.argtypes = [dp, vp, vp, vp, vp, cf, vp, ci, vp, vp, vp, vp, vp, sz, vp]
        L.jz_conv2d_bwd_data_bn_relu_bwd_workspace_bytes.argtypes = [dp, ctypes.POINTER(sz)]
        L.jz_conv2d_bwd_data_bn_relu_bwd.argtypes = [dp] + [vp] * 12 + [sz, vp]
        L.jz_conv2d_bwd_data_block_end_bwd.argtypes = [dp] + [vp] * 13 + [sz, vp]
        L.jz_status_string.argtypes = [ci]
        L.jz_status_string.restype = ctypes.c_char_p
        L.jz_version.argtypes = []
        for name in EXPORTS:
            if name != "jz_status_string":
                getattr(L, name).restype = ci
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().jz_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != JZ_OK:
        raise JzError(status, where)


def conv_desc(N, H, W, C, K, R, S, stride=1, pad=0) -> jz_conv_desc:
    sh, sw = (stride, stride) if isinstance(stride, int) else stride
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    return jz_conv_desc(N, H, W, C, K, R, S, sh, sw, ph, pw)


def _dev_ptr(t: Optional[torch.Tensor], dtype, numel=None, what="tensor") -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError("%s must be a contiguous %s tensor on the GPU" % (what, dtype))
    if numel is not None and t.numel() != numel:
        raise ValueError("%s has %d elements, expected %d" % (what, t.numel(), numel))
    return t.data_ptr() if t.numel() else None


def _ws(ws: Optional[torch.Tensor]):
    if ws is None:
        return None, 0
    if not ws.is_cuda or not ws.is_contiguous():
        raise TypeError("workspace must be a contiguous GPU tensor")
    return ws.data_ptr(), ws.numel() * ws.element_size()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def jz_version() -> int:
    return lib().jz_version()


def jz_conv2d_workspace_bytes(op: int, desc: jz_conv_desc) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().jz_conv2d_workspace_bytes(op, ctypes.byref(desc), ctypes.byref(n)), "jz_conv2d_workspace_bytes")
    return n.value


def jz_conv2d_describe_plan(op: int, desc: jz_conv_desc) -> str:
    buf = ctypes.create_string_buffer(256)
    _check(lib().jz_conv2d_describe_plan(op, ctypes.byref(desc), buf, 256), "jz_conv2d_describe_plan")
    return buf.value.decode()


def jz_bn_workspace_bytes(rows: int, channels: int) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().jz_bn_workspace_bytes(rows, channels, ctypes.byref(n)), "jz_bn_workspace_bytes")
    return n.value


def jz_bn_relu_fwd(rows, channels, x16, gamma, beta, eps, relu, y16, save_mean, save_invstd, ws, stream=None):
    """y16 = [relu](gamma * (x16 - mean) * invstd + beta) with the mini-batch statistics, which are written to save_*."""
    h, f = torch.float16, torch.float32
    wp, wn = _ws(ws)
    _check(lib().jz_bn_relu_fwd(rows, channels, _dev_ptr(x16, h, rows * channels, "x16"), _dev_ptr(gamma, f, channels, "gamma"),
                                _dev_ptr(beta, f, channels, "beta"), float(eps), int(bool(relu)),
                                _dev_ptr(y16, h, rows * channels, "y16"), _dev_ptr(save_mean, f, channels, "save_mean"),
                                _dev_ptr(save_invstd, f, channels, "save_invstd"), wp, wn, _stream(stream)), "jz_bn_relu_fwd")


def jz_bn_relu_bwd(rows, channels, x16, y16, dy16, gamma, save_mean, save_invstd, relu, dx16, dgamma16, dbeta16, ws, stream=None):
    """dx16, dgamma16, dbeta16 of the layer above; y16 (the forward output) is the ReLU mask and may be None without ReLU."""
    h, f = torch.float16, torch.float32
    wp, wn = _ws(ws)
    _check(lib().jz_bn_relu_bwd(rows, channels, _dev_ptr(x16, h, rows * channels, "x16"), _dev_ptr(y16, h, rows * channels, "y16"),
                                _dev_ptr(dy16, h, rows * channels, "dy16"), _dev_ptr(gamma, f, channels, "gamma"),
                                _dev_ptr(save_mean, f, channels, "save_mean"), _dev_ptr(save_invstd, f, channels, "save_invstd"),
                                int(bool(relu)), _dev_ptr(dx16, h, rows * channels, "dx16"), _dev_ptr(dgamma16, h, channels, "dgamma16"),
                                _dev_ptr(dbeta16, h, channels, "dbeta16"), wp, wn, _stream(stream)), "jz_bn_relu_bwd")


def jz_bn_bwd_block_end(rows, channels, x16, y_out16, dya16, dyb16, gamma, save_mean, save_invstd, g16, dx16, dgamma16, dbeta16, ws,
                        stream=None):
    """g16 = relu-masked (dya16 [+ dyb16]); dx16, dgamma16, dbeta16 = batch-norm backward (no ReLU) of dy = g16."""
    h, f, n = torch.float16, torch.float32, rows * channels
    wp, wn = _ws(ws)
    _check(lib().jz_bn_bwd_block_end(rows, channels, _dev_ptr(x16, h, n, "x16"), _dev_ptr(y_out16, h, n, "y_out16"),
                                     _dev_ptr(dya16, h, n, "dya16"), _dev_ptr(dyb16, h, n, "dyb16"), _dev_ptr(gamma, f, channels, "gamma"),
                                     _dev_ptr(save_mean, f, channels, "save_mean"), _dev_ptr(save_invstd, f, channels, "save_invstd"),
                                     _dev_ptr(g16, h, n, "g16"), _dev_ptr(dx16, h, n, "dx16"), _dev_ptr(dgamma16, h, channels, "dgamma16"),
                                     _dev_ptr(dbeta16, h, channels, "dbeta16"), wp, wn, _stream(stream)), "jz_bn_bwd_block_end")


def jz_conv2d_tune_set(op: int, desc: jz_conv_desc, tile_m: int, tile_n: int, k_tile: int, wavefronts: int, ring: int, splits: int):
    _check(lib().jz_conv2d_tune_set(op, ctypes.byref(desc), tile_m, tile_n, k_tile, wavefronts, ring, splits), "jz_conv2d_tune_set")


def jz_conv2d_tune_use_table(on: bool):
    _check(lib().jz_conv2d_tune_use_table(1 if on else 0), "jz_conv2d_tune_use_table")


def jz_conv2d_tune_clear():
    _check(lib().jz_conv2d_tune_clear(), "jz_conv2d_tune_clear")


def jz_conv2d_fwd(desc, x16, w16, y16, ws=None, stream=None):
    d, h = desc, torch.float16
    wp, wn = _ws(ws)
    _check(lib().jz_conv2d_fwd(ctypes.byref(d), _dev_ptr(x16, h, d.N * d.H * d.W * d.C, "x16"),
                               _dev_ptr(w16, h, d.K * d.R * d.S * d.C, "w16"),
                               _dev_ptr(y16, h, d.N * d.P * d.Q * d.K, "y16"), wp, wn, _stream(stream)), "jz_conv2d_fwd")


def jz_conv2d_bwd_data(desc, dy16, w16, dx16, ws=None, stream=None):
    d, h = desc, torch.float16
    wp, wn = _ws(ws)
    _check(lib().jz_conv2d_bwd_data(ctypes.byref(d), _dev_ptr(dy16, h, d.N * d.P * d.Q * d.K, "dy16"),
                                    _dev_ptr(w16, h, d.K * d.R * d.S * d.C, "w16"),
                                    _dev_ptr(dx16, h, d.N * d.H * d.W * d.C, "dx16"), wp, wn, _stream(stream)),
           "jz_conv2d_bwd_data")


def jz_conv2d_bwd_weight(desc, x16, dy16, dw16, ws=None, stream=None):
    d, h = desc, torch.float16
    wp, wn = _ws(ws)
    _check(lib().jz_conv2d_bwd_weight(ctypes.byref(d), _dev_ptr(x16, h, d.N * d.H * d.W * d.C, "x16"),
                                      _dev_ptr(dy16, h, d.N * d.P * d.Q * d.K, "dy16"),
                                      _dev_ptr(dw16, h, d.K * d.R * d.S * d.C, "dw16"), wp, wn, _stream(stream)),
           "jz_conv2d_bwd_weight")


# ---- the single-precision variant (same operations, float tensors) ----------------------------------------------------
def jz_conv2d_f32_workspace_bytes(op: int, desc: jz_conv_desc) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().jz_conv2d_f32_workspace_bytes(op, ctypes.byref(desc), ctypes.byref(n)), "jz_conv2d_f32_workspace_bytes")
    return n.value


def jz_conv2d_f32(op: int, desc: jz_conv_desc, a32, b32, out32, ws=None, stream=None):
    """op JZ_FWD: (x, w) -> y; JZ_BWD_DATA: (dy, w) -> dx; JZ_BWD_WEIGHT: (x, dy) -> dw; float32 GPU tensors."""
    d, f = desc, torch.float32
    nx, ny, nw = d.N * d.H * d.W * d.C, d.N * d.P * d.Q * d.K, d.K * d.R * d.S * d.C
    na, nb, no = {JZ_FWD: (nx, nw, ny), JZ_BWD_DATA: (ny, nw, nx), JZ_BWD_WEIGHT: (nx, ny, nw)}[op]
    fn = {JZ_FWD: lib().jz_conv2d_fwd_f32, JZ_BWD_DATA: lib().jz_conv2d_bwd_data_f32, JZ_BWD_WEIGHT: lib().jz_conv2d_bwd_weight_f32}[op]
    wp, wn = _ws(ws)
    _check(fn(ctypes.byref(d), _dev_ptr(a32, f, na, "first input"), _dev_ptr(b32, f, nb, "second input"), _dev_ptr(out32, f, no, "output"),
              wp, wn, _stream(stream)), "jz_conv2d_f32")


def jz_gemm_fc_f32_workspace_bytes(mode: int, batch: int, in_features: int, out_features: int) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().jz_gemm_fc_f32_workspace_bytes(mode, batch, in_features, out_features, ctypes.byref(n)), "jz_gemm_fc_f32_workspace_bytes")
    return n.value


def jz_gemm_fc_f32(mode: int, batch: int, in_features: int, out_features: int, a32, b32, out32, ws=None, stream=None):
    """mode JZ_FWD: (x, w) -> y; JZ_BWD_DATA: (dy, w) -> dx; JZ_BWD_WEIGHT: (dy, x) -> dw; float32 GPU tensors."""
    B, I, O, f = batch, in_features, out_features, torch.float32
    na, nb, no = {JZ_FWD: (B * I, O * I, B * O), JZ_BWD_DATA: (B * O, O * I, B * I), JZ_BWD_WEIGHT: (B * O, B * I, O * I)}[mode]
    wp, wn = _ws(ws)
    _check(lib().jz_gemm_fc_f32(mode, B, I, O, _dev_ptr(a32, f, na, "first input"), _dev_ptr(b32, f, nb, "second input"),
                                _dev_ptr(out32, f, no, "output"), wp, wn, _stream(stream)), "jz_gemm_fc_f32")


def bind_conv2d_f32(op: int, desc: jz_conv_desc, a32, b32, out32, ws=None):
    """Pre-marshalled jz_conv2d_*_f32 call (see BoundCall)."""
    fn = {JZ_FWD: lib().jz_conv2d_fwd_f32, JZ_BWD_DATA: lib().jz_conv2d_bwd_data_f32, JZ_BWD_WEIGHT: lib().jz_conv2d_bwd_weight_f32}[op]
    wp, wn = _ws(ws)
    return BoundCall(fn, (ctypes.byref(desc), a32.data_ptr(), b32.data_ptr(), out32.data_ptr(), wp, wn), "jz_conv2d_f32", (desc, a32, b32, out32, ws))


def bind_gemm_fc_f32(mode: int, batch: int, in_features: int, out_features: int, a32, b32, out32, ws=None):
    wp, wn = _ws(ws)
    return BoundCall(lib().jz_gemm_fc_f32, (mode, batch, in_features, out_features, a32.data_ptr(), b32.data_ptr(), out32.data_ptr(), wp, wn),
                     "jz_gemm_fc_f32", (a32, b32, out32, ws))


JZ_STATIC_SCRATCH_BYTES = 64 << 20


def jz_conv2d_bwd_weight_static(desc, x16, dy16, dw16, stream=None):
    """jz_conv2d_bwd_weight without a workspace argument: scratch in the library's own fixed array."""
    d, h = desc, torch.float16
    _check(lib().jz_conv2d_bwd_weight_static(ctypes.byref(d), _dev_ptr(x16, h, d.N * d.H * d.W * d.C, "x16"),
                                             _dev_ptr(dy16, h, d.N * d.P * d.Q * d.K, "dy16"),
                                             _dev_ptr(dw16, h, d.K * d.R * d.S * d.C, "dw16"), _stream(stream)),
           "jz_conv2d_bwd_weight_static")


class BoundCall:
    """One entry-point call with its arguments already marshalled: `call(stream)` enqueues it again without
    re-validating the tensors (they are kept alive here).  For launch loops that repeat the same calls every step."""

    __slots__ = ("fn", "args", "where", "keep")

    def __init__(self, fn, args, where, keep):
        self.fn, self.args, self.where, self.keep = fn, args, where, keep

    def __call__(self, stream=None):
        st = self.fn(*self.args, _stream(stream))
        if st != JZ_OK:
            raise JzError(st, self.where)


def bind_conv2d(op: int, desc, a16, b16, out16, ws=None) -> BoundCall:
    """Pre-marshalled jz_conv2d_fwd (x, w -> y), jz_conv2d_bwd_data (dy, w -> dx) or jz_conv2d_bwd_weight (x, dy -> dw)."""
    d, h = desc, torch.float16
    nx, nw, ny = d.N * d.H * d.W * d.C, d.K * d.R * d.S * d.C, d.N * d.P * d.Q * d.K
    name, na, nb, no = {JZ_FWD: ("jz_conv2d_fwd", nx, nw, ny), JZ_BWD_DATA: ("jz_conv2d_bwd_data", ny, nw, nx),
                        JZ_BWD_WEIGHT: ("jz_conv2d_bwd_weight", nx, ny, nw)}[op]
    wp, wn = _ws(ws)
    args = (ctypes.byref(d), _dev_ptr(a16, h, na, "first operand"), _dev_ptr(b16, h, nb, "second operand"),
            _dev_ptr(out16, h, no, "output"), wp, wn)
    return BoundCall(getattr(lib(), name), args, name, (d, a16, b16, out16, ws))


def bind_gemm_fc(mode, batch, in_features, out_features, a16, b16, out16, ws=None) -> BoundCall:
    """Pre-marshalled jz_gemm_fc."""
    B, I, O, h = batch, in_features, out_features, torch.float16
    na, nb, no = {JZ_FWD: (B * I, O * I, B * O), JZ_BWD_DATA: (B * O, O * I, B * I), JZ_BWD_WEIGHT: (B * O, B * I, O * I)}[mode]
    wp, wn = _ws(ws)
    args = (mode, B, I, O, _dev_ptr(a16, h, na, "a16"), _dev_ptr(b16, h, nb, "b16"), _dev_ptr(out16, h, no, "out16"), wp, wn)
    return BoundCall(lib().jz_gemm_fc, args, "jz_gemm_fc", (a16, b16, out16, ws))


def jz_gemm_fc_workspace_bytes(mode: int, batch: int, in_features: int, out_features: int) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().jz_gemm_fc_workspace_bytes(mode, batch, in_features, out_features, ctypes.byref(n)),
           "jz_gemm_fc_workspace_bytes")
    return n.value


def jz_gemm_fc(mode, batch, in_features, out_features, a16, b16, out16, ws=None, stream=None):
    B, I, O, h = batch, in_features, out_features, torch.float16
    na, nb, no = {JZ_FWD: (B * I, O * I, B * O), JZ_BWD_DATA: (B * O, O * I, B * I), JZ_BWD_WEIGHT: (B * O, B * I, O * I)}[mode]
    wp, wn = _ws(ws)
    _check(lib().jz_gemm_fc(mode, B, I, O, _dev_ptr(a16, h, na, "a16"), _dev_ptr(b16, h, nb, "b16"),
                            _dev_ptr(out16, h, no, "out16"), wp, wn, _stream(stream)), "jz_gemm_fc")


class ParamSet:
    """Keeps the host tables of a jz_param_set alive next to the device buffers it points at."""

    def __init__(self, offsets: Sequence[int], flags: Sequence[int], master_w: torch.Tensor, momentum: torch.Tensor,
                 grad16: torch.Tensor, weight16: torch.Tensor):
        self.offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        self.flags = np.ascontiguousarray(flags, dtype=np.uint8)
        T = len(self.flags)
        if len(self.offsets) != T + 1:
            raise ValueError("offsets must have num_tensors + 1 entries")
        P = int(self.offsets[-1]) if T else 0
        self.tensors = (master_w, momentum, grad16, weight16)
        self.c = jz_param_set(
            T, self.offsets.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
            self.flags.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)),
            _dev_ptr(master_w, torch.float32, P, "master_w"), _dev_ptr(momentum, torch.float32, P, "momentum"),
            _dev_ptr(grad16, torch.float16, P, "grad16"), _dev_ptr(weight16, torch.float16, P, "weight16"))
        self.P, self.T = P, T


def jz_lars_workspace_bytes(ps: ParamSet) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().jz_lars_workspace_bytes(ctypes.byref(ps.c), ctypes.byref(n)), "jz_lars_workspace_bytes")
    return n.value


def jz_lars_prepare(ps: ParamSet, ws: torch.Tensor, stream=None):
    wp, wn = _ws(ws)
    _check(lib().jz_lars_prepare(ctypes.byref(ps.c), wp, wn, _stream(stream)), "jz_lars_prepare")


def jz_lars_mp_update(ps: ParamSet, hp: jz_lars_hparams, found_inf: torch.Tensor, ws: torch.Tensor, stream=None):
    if not found_inf.is_cuda or found_inf.dtype != torch.int32 or found_inf.numel() != 1:
        raise TypeError("found_inf must be a one-element int32 GPU tensor")
    wp, wn = _ws(ws)
    _check(lib().jz_lars_mp_update(ctypes.byref(ps.c), ctypes.byref(hp), found_inf.data_ptr(), wp, wn, _stream(stream)),
           "jz_lars_mp_update")


def _ls_state(state: torch.Tensor) -> int:
    # jz_loss_scale_state {float scale; int good_steps;} held in a two-element int32 GPU tensor
    if not state.is_cuda or state.dtype != torch.int32 or state.numel() != 2 or not state.is_contiguous():
        raise TypeError("the loss-scale state must be a contiguous two-element int32 GPU tensor")
    return state.data_ptr()


def jz_loss_scale_init(state: torch.Tensor, initial_scale: float, stream=None):
    _check(lib().jz_loss_scale_init(_ls_state(state), float(initial_scale), _stream(stream)), "jz_loss_scale_init")


def loss_scale_state(state: torch.Tensor):
    """(scale, good_steps) read back from the device state (synchronizes)."""
    h = state.cpu()
    return float(h[:1].view(torch.float32).item()), int(h[1].item())


def loss_scale_policy(growth_factor=2.0, backoff_factor=0.5, growth_interval=2000, min_scale=1.0,
                      max_scale=65536.0) -> jz_loss_scale_policy:
    return jz_loss_scale_policy(growth_factor, backoff_factor, growth_interval, min_scale, max_scale)


def jz_lars_mp_update_dyn(ps: ParamSet, hp: jz_lars_hparams, policy: jz_loss_scale_policy, state: torch.Tensor,
                          found_inf: torch.Tensor, ws: torch.Tensor, stream=None):
    if not found_inf.is_cuda or found_inf.dtype != torch.int32 or found_inf.numel() != 1:
        raise TypeError("found_inf must be a one-element int32 GPU tensor")
    wp, wn = _ws(ws)
    _check(lib().jz_lars_mp_update_dyn(ctypes.byref(ps.c), ctypes.byref(hp), ctypes.byref(policy), _ls_state(state),
                                       found_inf.data_ptr(), wp, wn, _stream(stream)), "jz_lars_mp_update_dyn")


# ---- the update in one launch: gradient norms taken where the gradients are produced --------------------------------------
def sumsq_sink(sums: torch.Tensor, nonfinite: torch.Tensor) -> jz_sumsq_sink:
    """A sink in caller-owned memory: `sums` int64[1024] (8192 bytes, 128-byte aligned), `nonfinite` int32[1]; the caller keeps
    both alive and clears them."""
    if not sums.is_cuda or sums.dtype != torch.int64 or sums.numel() != JZ_SUMSQ_SINK_BYTES // 8 or not sums.is_contiguous():
        raise TypeError("sums must be a contiguous 1024-element int64 GPU tensor")
    if not nonfinite.is_cuda or nonfinite.dtype != torch.int32 or nonfinite.numel() != 1:
        raise TypeError("nonfinite must be a one-element int32 GPU tensor")
    return jz_sumsq_sink(sums.data_ptr(), nonfinite.data_ptr())


def sumsq_sink_units(sums: torch.Tensor) -> int:
    """What a sink holds, read back (synchronizes), as an exact integer count of units of 2^-48: the 64 quadruples of
    base-2^20 digit counters added as integers."""
    a = sums.cpu().numpy().view(np.uint64).reshape(64, 16)
    d = [sum(int(x) for x in a[:, i]) for i in range(4)]
    return (d[3] << 60) + (d[2] << 40) + (d[1] << 20) + d[0]


def jz_conv2d_bwd_weight_sumsq(desc, x16, dy16, dw16, sink: jz_sumsq_sink, ws=None, stream=None):
    d, h = desc, torch.float16
    wp, wn = _ws(ws)
    _check(lib().jz_conv2d_bwd_weight_sumsq(ctypes.byref(d), _dev_ptr(x16, h, d.N * d.H * d.W * d.C, "x16"),
                                            _dev_ptr(dy16, h, d.N * d.P * d.Q * d.K, "dy16"),
                                            _dev_ptr(dw16, h, d.K * d.R * d.S * d.C, "dw16"), wp, wn, ctypes.byref(sink),
                                            _stream(stream)), "jz_conv2d_bwd_weight_sumsq")


def jz_gemm_fc_bwd_weight_sumsq(batch, in_features, out_features, dy16, x16, dw16, sink: jz_sumsq_sink, ws=None, stream=None):
    B, I, O, h = batch, in_features, out_features, torch.float16
    wp, wn = _ws(ws)
    _check(lib().jz_gemm_fc_bwd_weight_sumsq(B, I, O, _dev_ptr(dy16, h, B * O, "dy16"), _dev_ptr(x16, h, B * I, "x16"),
                                             _dev_ptr(dw16, h, O * I, "dw16"), wp, wn, ctypes.byref(sink), _stream(stream)),
           "jz_gemm_fc_bwd_weight_sumsq")


def bind_conv2d_bwd_weight_sumsq(desc, x16, dy16, dw16, sink: jz_sumsq_sink, ws=None) -> BoundCall:
    d, h = desc, torch.float16
    wp, wn = _ws(ws)
    args = (ctypes.byref(d), _dev_ptr(x16, h, d.N * d.H * d.W * d.C, "x16"), _dev_ptr(dy16, h, d.N * d.P * d.Q * d.K, "dy16"),
            _dev_ptr(dw16, h, d.K * d.R * d.S * d.C, "dw16"), wp, wn, ctypes.byref(sink))
    return BoundCall(lib().jz_conv2d_bwd_weight_sumsq, args, "jz_conv2d_bwd_weight_sumsq", (d, x16, dy16, dw16, ws, sink))


def bind_gemm_fc_bwd_weight_sumsq(batch, in_features, out_features, dy16, x16, dw16, sink: jz_sumsq_sink, ws=None) -> BoundCall:
    B, I, O, h = batch, in_features, out_features, torch.float16
    wp, wn = _ws(ws)
    args = (B, I, O, _dev_ptr(dy16, h, B * O, "dy16"), _dev_ptr(x16, h, B * I, "x16"), _dev_ptr(dw16, h, O * I, "dw16"), wp, wn,
            ctypes.byref(sink))
    return BoundCall(lib().jz_gemm_fc_bwd_weight_sumsq, args, "jz_gemm_fc_bwd_weight_sumsq", (dy16, x16, dw16, ws, sink))


def jz_lars_begin_step(ps: ParamSet, ws: torch.Tensor, state: Optional[torch.Tensor] = None, stream=None):
    wp, wn = _ws(ws)
    _check(lib().jz_lars_begin_step(ctypes.byref(ps.c), _ls_state(state) if state is not None else None, wp, wn, _stream(stream)),
           "jz_lars_begin_step")


def jz_lars_sumsq_sink(ps: ParamSet, ws: torch.Tensor, tensor: int) -> jz_sumsq_sink:
    """The sink of tensor `tensor` inside the LARS workspace (host only; valid while `ws` is)."""
    wp, wn = _ws(ws)
    sink = jz_sumsq_sink()
    _check(lib().jz_lars_sumsq_sink(ctypes.byref(ps.c), wp, wn, int(tensor), ctypes.byref(sink)), "jz_lars_sumsq_sink")
    return sink


def jz_lars_grad_sumsq(ps: ParamSet, first_tensor: int, num_tensors: int, ws: torch.Tensor, stream=None):
    wp, wn = _ws(ws)
    _check(lib().jz_lars_grad_sumsq(ctypes.byref(ps.c), int(first_tensor), int(num_tensors), wp, wn, _stream(stream)),
           "jz_lars_grad_sumsq")


def jz_lars_mp_update_presummed(ps: ParamSet, hp: jz_lars_hparams, found_inf: torch.Tensor, ws: torch.Tensor, stream=None):
    if not found_inf.is_cuda or found_inf.dtype != torch.int32 or found_inf.numel() != 1:
        raise TypeError("found_inf must be a one-element int32 GPU tensor")
    wp, wn = _ws(ws)
    _check(lib().jz_lars_mp_update_presummed(ctypes.byref(ps.c), ctypes.byref(hp), found_inf.data_ptr(), wp, wn, _stream(stream)),
           "jz_lars_mp_update_presummed")


def jz_lars_mp_update_presummed_dyn(ps: ParamSet, hp: jz_lars_hparams, policy: jz_loss_scale_policy, state: torch.Tensor,
                                    found_inf: torch.Tensor, ws: torch.Tensor, stream=None):
    if not found_inf.is_cuda or found_inf.dtype != torch.int32 or found_inf.numel() != 1:
        raise TypeError("found_inf must be a one-element int32 GPU tensor")
    wp, wn = _ws(ws)
    _check(lib().jz_lars_mp_update_presummed_dyn(ctypes.byref(ps.c), ctypes.byref(hp), ctypes.byref(policy), _ls_state(state),
                                                 found_inf.data_ptr(), wp, wn, _stream(stream)), "jz_lars_mp_update_presummed_dyn")


def lars_hparams(lr, momentum, weight_decay, trust_coef, loss_scale) -> jz_lars_hparams:
    return jz_lars_hparams(lr, momentum, weight_decay, trust_coef, loss_scale)


# ---------------------------------------------------------------------------------------------
# the small layers between the convolutions (FP16 NHWC tensors; marshalling only)
# ---------------------------------------------------------------------------------------------
def _h(t: torch.Tensor, n: int, what: str) -> int:
    return _dev_ptr(t, torch.float16, n, what)


def jz_add_fwd(a, b, y, relu=True, stream=None):
    n = a.numel()
    _check(lib().jz_add_fwd(n, _h(a, n, "a"), _h(b, n, "b"), int(bool(relu)), _h(y, n, "y"), _stream(stream)), "jz_add_fwd")


def jz_relu_bwd(y, dy, dx, stream=None):
    n = y.numel()
    _check(lib().jz_relu_bwd(n, _h(y, n, "y"), _h(dy, n, "dy"), _h(dx, n, "dx"), _stream(stream)), "jz_relu_bwd")


def jz_relu_bwd_sum(y, dya, dyb, dx, stream=None):
    n = y.numel()
    _check(lib().jz_relu_bwd_sum(n, _h(y, n, "y"), _h(dya, n, "dya"), _h(dyb, n, "dyb"), _h(dx, n, "dx"), _stream(stream)), "jz_relu_bwd_sum")


def pool_out(size, window, stride, pad):
    return (size + 2 * pad - window) // stride + 1


def jz_maxpool_fwd(N, H, W, C, window, stride, pad, x, y, arg=None, stream=None):
    """arg: optional uint8 tensor, one entry per output element, that receives each window's winner for jz_maxpool_bwd."""
    P, Q = pool_out(H, window, stride, pad), pool_out(W, window, stride, pad)
    _check(lib().jz_maxpool_fwd(N, H, W, C, window, stride, pad, _h(x, N * H * W * C, "x"), _h(y, N * P * Q * C, "y"),
                                _dev_ptr(arg, torch.uint8, N * P * Q * C, "arg"), _stream(stream)), "jz_maxpool_fwd")


def jz_maxpool_bwd(N, H, W, C, window, stride, pad, x, dy, dx, arg=None, stream=None):
    """With arg (from jz_maxpool_fwd) x may be None."""
    P, Q = pool_out(H, window, stride, pad), pool_out(W, window, stride, pad)
    _check(lib().jz_maxpool_bwd(N, H, W, C, window, stride, pad, _dev_ptr(x, torch.float16, N * H * W * C, "x"),
                                _dev_ptr(arg, torch.uint8, N * P * Q * C, "arg"), _h(dy, N * P * Q * C, "dy"),
                                _h(dx, N * H * W * C, "dx"), _stream(stream)), "jz_maxpool_bwd")


def jz_avgpool_fwd(N, HW, C, x, y, stream=None):
    _check(lib().jz_avgpool_fwd(N, HW, C, _h(x, N * HW * C, "x"), _h(y, N * C, "y"), _stream(stream)), "jz_avgpool_fwd")


def jz_avgpool_bwd(N, HW, C, dy, dx, stream=None):
    _check(lib().jz_avgpool_bwd(N, HW, C, _h(dy, N * C, "dy"), _h(dx, N * HW * C, "dx"), _stream(stream)), "jz_avgpool_bwd")


def jz_bias_add(rows, C, y, b, out, stream=None):
    _check(lib().jz_bias_add(rows, C, _h(y, rows * C, "y"), _h(b, C, "b"), _h(out, rows * C, "out"), _stream(stream)), "jz_bias_add")


def jz_bias_grad(rows, C, dy, db, stream=None):
    _check(lib().jz_bias_grad(rows, C, _h(dy, rows * C, "dy"), _h(db, C, "db"), _stream(stream)), "jz_bias_grad")


def jz_softmax_xent_bwd(rows, classes, z, labels, dz, loss, loss_scale=1.0, state=None, stream=None):
    if not labels.is_cuda or labels.dtype != torch.int32 or labels.numel() != rows or not labels.is_contiguous():
        raise TypeError("labels must be a contiguous int32 GPU tensor with one entry per row")
    _check(lib().jz_softmax_xent_bwd(rows, classes, _h(z, rows * classes, "z"), labels.data_ptr(), float(loss_scale),
                                     _ls_state(state) if state is not None else None, _h(dz, rows * classes, "dz"),
                                     _dev_ptr(loss, torch.float32, rows, "loss"), _stream(stream)), "jz_softmax_xent_bwd")


def jz_conv2d_bn_relu_fwd_workspace_bytes(desc: jz_conv_desc) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().jz_conv2d_bn_relu_fwd_workspace_bytes(ctypes.byref(desc), ctypes.byref(n)), "jz_conv2d_bn_relu_fwd_workspace_bytes")
    return n.value


def jz_conv2d_bn_relu_fwd(desc, x16, w16, gamma, beta, eps, relu, conv_out16, y16, save_mean, save_invstd, ws, residual16=None,
                          stream=None):
    """y16 = [relu](bn(conv(x16, w16)) [+ residual16]); conv_out16 receives the convolution output."""
    d, h, f = desc, torch.float16, torch.float32
    n_out = d.N * d.P * d.Q * d.K
    wp, wn = _ws(ws)
    _check(lib().jz_conv2d_bn_relu_fwd(ctypes.byref(d), _dev_ptr(x16, h, d.N * d.H * d.W * d.C, "x16"),
                                       _dev_ptr(w16, h, d.K * d.R * d.S * d.C, "w16"), _dev_ptr(gamma, f, d.K, "gamma"),
                                       _dev_ptr(beta, f, d.K, "beta"), float(eps), _dev_ptr(residual16, h, n_out, "residual16"),
                                       int(bool(relu)), _dev_ptr(conv_out16, h, n_out, "conv_out16"),
                                       _dev_ptr(y16, h, n_out, "y16"), _dev_ptr(save_mean, f, d.K, "save_mean"),
                                       _dev_ptr(save_invstd, f, d.K, "save_invstd"), wp, wn, _stream(stream)), "jz_conv2d_bn_relu_fwd")


def jz_conv2d_bwd_data_bn_relu_bwd_workspace_bytes(desc: jz_conv_desc) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().jz_conv2d_bwd_data_bn_relu_bwd_workspace_bytes(ctypes.byref(desc), ctypes.byref(n)),
           "jz_conv2d_bwd_data_bn_relu_bwd_workspace_bytes")
    return n.value


def jz_conv2d_bwd_data_bn_relu_bwd(desc, dy16, w16, bn_x16, bn_y16, gamma, save_mean, save_invstd, dz16, bn_dx16, dgamma16, dbeta16, ws,
                                   stream=None):
    """dz16 = bwd_data(dy16, w16); bn_dx16, dgamma16, dbeta16 = backward of the batch norm + ReLU (input bn_x16, output
    bn_y16 = this convolution's forward input) for the incoming gradient dz16."""
    d, h, f = desc, torch.float16, torch.float32
    n_in, C = d.N * d.H * d.W * d.C, d.C
    wp, wn = _ws(ws)
    _check(lib().jz_conv2d_bwd_data_bn_relu_bwd(ctypes.byref(d), _dev_ptr(dy16, h, d.N * d.P * d.Q * d.K, "dy16"),
                                                _dev_ptr(w16, h, d.K * d.R * d.S * d.C, "w16"), _dev_ptr(bn_x16, h, n_in, "bn_x16"),
                                                _dev_ptr(bn_y16, h, n_in, "bn_y16"), _dev_ptr(gamma, f, C, "gamma"),
                                                _dev_ptr(save_mean, f, C, "save_mean"), _dev_ptr(save_invstd, f, C, "save_invstd"),
                                                _dev_ptr(dz16, h, n_in, "dz16"), _dev_ptr(bn_dx16, h, n_in, "bn_dx16"),
                                                _dev_ptr(dgamma16, h, C, "dgamma16"), _dev_ptr(dbeta16, h, C, "dbeta16"), wp, wn,
                                                _stream(stream)), "jz_conv2d_bwd_data_bn_relu_bwd")


def jz_conv2d_bwd_data_block_end_bwd(desc, dy16, w16, dyb16, bn_x16, y_out16, gamma, save_mean, save_invstd, g16, bn_dx16, dgamma16, dbeta16,
                                     ws, stream=None):
    """g16 = relu-masked (bwd_data(dy16, w16) [+ dyb16]) by y_out16 > 0; bn_dx16, dgamma16, dbeta16 = batch-norm backward
    (no ReLU, input bn_x16) of dy = g16."""
    d, h, f = desc, torch.float16, torch.float32
    n_in, C = d.N * d.H * d.W * d.C, d.C
    wp, wn = _ws(ws)
    _check(lib().jz_conv2d_bwd_data_block_end_bwd(ctypes.byref(d), _dev_ptr(dy16, h, d.N * d.P * d.Q * d.K, "dy16"),
                                                  _dev_ptr(w16, h, d.K * d.R * d.S * d.C, "w16"), _dev_ptr(dyb16, h, n_in, "dyb16"),
                                                  _dev_ptr(bn_x16, h, n_in, "bn_x16"), _dev_ptr(y_out16, h, n_in, "y_out16"),
                                                  _dev_ptr(gamma, f, C, "gamma"), _dev_ptr(save_mean, f, C, "save_mean"),
                                                  _dev_ptr(save_invstd, f, C, "save_invstd"), _dev_ptr(g16, h, n_in, "g16"),
                                                  _dev_ptr(bn_dx16, h, n_in, "bn_dx16"), _dev_ptr(dgamma16, h, C, "dgamma16"),
                                                  _dev_ptr(dbeta16, h, C, "dbeta16"), wp, wn, _stream(stream)),
           "jz_conv2d_bwd_data_block_end_bwd")
