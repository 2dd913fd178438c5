"""Seeded synthetic inputs with the shapes and value distributions of the paper's
workloads (ImageNet-sized activations of AlexNet / ResNet-50, He-normal filters,
loss-scaled fp16 gradients).  The dataset itself is not used: kernel time does
not depend on the pixel values and parity is judged against the CPU oracle.

This module only draws random numbers and rounds them to the storage types; it
contains none of the training method's arithmetic, so the HIP path's callers
and the oracle's tests can both take their inputs from it.  Everything is
generated on the host with numpy so that the same bits reach both sides.
"""
from dataclasses import dataclass
from typing import Dict, List, Optional

import numpy as np

from . import shapes

BASE_SEED = 180711205   # the paper's arXiv number


def rng_for(*key: int) -> np.random.Generator:
    return np.random.default_rng([BASE_SEED, *[int(k) for k in key]])


def normal_f16(rng: np.random.Generator, shape, std: float = 1.0) -> np.ndarray:
    """fp16 array ~ N(0, std^2): drawn in fp32, scaled, rounded to nearest even."""
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a.astype(np.float16)


def he_normal_f32(rng: np.random.Generator, shape, fan_in: int) -> np.ndarray:
    return rng.standard_normal(size=shape, dtype=np.float32) * np.float32(np.sqrt(2.0 / fan_in))


@dataclass
class ConvCase:
    """One convolution layer's operands: x and dy in fp16, fp32 master filter and its fp16 rounding."""
    N: int
    H: int
    W: int
    C: int
    K: int
    R: int
    S: int
    stride: int
    pad: int
    x: np.ndarray          # [N,H,W,C] fp16
    w32: np.ndarray        # [K,R,S,C] fp32 master
    w16: np.ndarray        # [K,R,S,C] fp16 = RNE16(w32)
    dy: np.ndarray         # [N,P,Q,K] fp16 = RNE16(S_loss * z)
    loss_scale: float

    @property
    def P(self):
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self):
        return (self.W + 2 * self.pad - self.S) // self.stride + 1


def conv_case(seed_key, N, H, W, C, K, R, S, stride=1, pad=0, loss_scale=1.0, dy_std=1.0) -> ConvCase:
    """x ~ N(0,1), filter He-normal std sqrt(2/(R*S*C)), dy ~ N(0,dy_std^2) * loss_scale; draw order x, w, dy."""
    rng = rng_for(*seed_key)
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    x = normal_f16(rng, (N, H, W, C))
    w32 = he_normal_f32(rng, (K, R, S, C), R * S * C)
    dy = normal_f16(rng, (N, P, Q, K), std=dy_std * loss_scale)
    return ConvCase(N, H, W, C, K, R, S, stride, pad, x, w32, w32.astype(np.float16), dy, loss_scale)


def conv_case_for(cs: shapes.ConvShape, N: int, seed_key, loss_scale=1.0) -> ConvCase:
    return conv_case(seed_key, N, cs.H, cs.H, cs.C, cs.K, cs.R, cs.R, cs.stride, cs.pad, loss_scale)


@dataclass
class FcCase:
    B: int
    I: int
    O: int
    x: np.ndarray      # [B,I] fp16
    w32: np.ndarray    # [O,I] fp32
    w16: np.ndarray
    dy: np.ndarray     # [B,O] fp16
    loss_scale: float


def fc_case(seed_key, B, I, O, loss_scale=1.0) -> FcCase:
    rng = rng_for(*seed_key)
    x = normal_f16(rng, (B, I))
    w32 = he_normal_f32(rng, (O, I), I)
    dy = normal_f16(rng, (B, O), std=loss_scale)
    return FcCase(B, I, O, x, w32, w32.astype(np.float16), dy, loss_scale)


@dataclass
class ParamSet:
    """Fused flat parameter buffers of a model plus the per-tensor table."""
    names: List[str]
    offsets: np.ndarray    # int64 [T+1]
    flags: np.ndarray      # uint8 [T]
    master_w: np.ndarray   # fp32 [P]
    momentum: np.ndarray   # fp32 [P]
    grad16: np.ndarray     # fp16 [P], already multiplied by the loss scale
    weight16: np.ndarray   # fp16 [P] = RNE16(master_w)
    loss_scale: float
    inf_index: Optional[int] = None

    @property
    def P(self):
        return int(self.offsets[-1])

    @property
    def T(self):
        return len(self.flags)


# hyper-parameters every configuration shares (lr, momentum, weight decay, LARS coefficient eta = 0.001 of Section 5.2)
HPARAMS: Dict[str, float] = dict(lr=0.1, momentum=0.9, weight_decay=5e-5, trust_coef=0.001)


def resnet50_param_set(loss_scale=1024.0, grad_std=1e-3, inject_inf=False, seed_key=(1,), variant="v1",
                       momentum_std=0.0) -> ParamSet:
    """ResNet-50's 161 trainable tensors (25,557,032 parameters) as one fused buffer.

    Filters and the classifier weight are He-normal, gamma = 1, beta = 0, bias = 0;
    fp16 gradients ~ N(0, grad_std^2) * loss_scale.  With inject_inf one seeded
    element of the gradient buffer is set to +Inf.  momentum_std > 0 fills the
    momentum buffer with N(0, momentum_std^2) instead of zeros (later steps).
    """
    tensors = shapes.resnet50_param_tensors(variant)
    off = np.asarray(shapes.offsets_of(tensors), dtype=np.int64)
    rng = rng_for(*seed_key)
    P = int(off[-1])
    w = np.zeros(P, np.float32)
    for i, (_, shp, kind, _) in enumerate(tensors):
        a, b = int(off[i]), int(off[i + 1])
        if kind == "conv":
            w[a:b] = he_normal_f32(rng, (b - a,), shp[1] * shp[2] * shp[3])
        elif kind == "fc":
            w[a:b] = he_normal_f32(rng, (b - a,), shp[1])
        elif kind == "gamma":
            w[a:b] = 1.0
    g = normal_f16(rng, (P,), std=grad_std * loss_scale)
    inf_index = None
    if inject_inf:
        inf_index = int(rng.integers(P))
        g[inf_index] = np.float16(np.inf)
    if momentum_std > 0:
        v = rng.standard_normal(size=P, dtype=np.float32) * np.float32(momentum_std)
    else:
        v = np.zeros(P, np.float32)
    return ParamSet([t[0] for t in tensors], off, np.asarray([t[3] for t in tensors], np.uint8), w, v, g,
                    w.astype(np.float16), loss_scale, inf_index)


def param_set_from_tensors(weights32: List[np.ndarray], grads16: List[np.ndarray], flags: List[int], loss_scale: float,
                           names: Optional[List[str]] = None) -> ParamSet:
    """Pack given per-tensor fp32 weights and fp16 gradients into one fused buffer (zero momentum)."""
    sizes = [int(w.size) for w in weights32]
    off = np.zeros(len(sizes) + 1, np.int64)
    off[1:] = np.cumsum(sizes)
    w = np.concatenate([np.asarray(a, np.float32).ravel() for a in weights32]) if sizes else np.zeros(0, np.float32)
    g = np.concatenate([np.asarray(a, np.float16).ravel() for a in grads16]) if sizes else np.zeros(0, np.float16)
    return ParamSet(names or ["t%d" % i for i in range(len(sizes))], off, np.asarray(flags, np.uint8), w,
                    np.zeros_like(w), g, w.astype(np.float16), loss_scale)


def random_param_set(seed_key, sizes: List[int], loss_scale=1024.0, grad_std=1e-3, flags: Optional[List[int]] = None,
                     momentum_std=0.0) -> ParamSet:
    """Generic fused buffer: tensor t ~ N(0, 2/size_t) weights, N(0, grad_std^2)*S gradients."""
    rng = rng_for(*seed_key)
    ws = [he_normal_f32(rng, (n,), max(n, 1)) for n in sizes]
    gs = [normal_f16(rng, (n,), std=grad_std * loss_scale) for n in sizes]
    ps = param_set_from_tensors(ws, gs, flags if flags is not None else [3] * len(sizes), loss_scale)
    if momentum_std > 0:
        ps.momentum = rng.standard_normal(size=ps.P, dtype=np.float32) * np.float32(momentum_std)
    return ps
