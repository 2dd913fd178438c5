"""fp64 oracle of training-mode batch normalization with an optional ReLU -- TEST INFRASTRUCTURE ONLY.

Section 4.2 of Jia et al. 2018 writes the layer as two formulas: each value is centred by the mini-batch mean and
divided by sqrt(mini-batch variance + eps), then scaled by gamma and shifted by beta (the two trainable parameter
sets the paper leaves out of weight decay).  Mean and variance are taken per channel over all N*H*W positions of the
mini-batch; the variance is the plain (biased) mean of squared deviations.  The backward pass is the exact gradient
of that map.  Everything is evaluated in fp64 on the fp16 inputs, in the order the formulas are written.

Conventions this oracle defines (the paper is silent on them):
  * tensors are [rows, C] with rows = N*H*W (NHWC flattened), activations and activation gradients in FP16;
  * gamma, beta and the saved statistics are FP32 (master precision), the parameter gradients are returned in fp64
    and as FP16 (they join the loss-scaled FP16 gradient buffer the optimizer reads);
  * with relu = True the output is max(z, 0) and the backward pass masks the incoming gradient with (y16 > 0), y16
    being the FP16 output that the forward pass wrote (passed in, so both sides use the same mask bits).
"""
import numpy as np


def _f16(a):
    a = np.asarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.float16)
    if a.dtype != np.float16:
        raise TypeError("expected fp16 data, got %s" % a.dtype)
    return a


def bn_relu_fwd(x16, gamma32, beta32, eps, relu=True):
    """Returns (y64, y16, mean64, invstd64): y = [relu](gamma * (x - mean) / sqrt(var + eps) + beta)."""
    x = _f16(x16).astype(np.float64)
    if x.ndim != 2:
        raise ValueError("x must be [rows, C]")
    g = np.asarray(gamma32, dtype=np.float32).astype(np.float64)
    b = np.asarray(beta32, dtype=np.float32).astype(np.float64)
    mean = x.sum(axis=0) / x.shape[0]
    dev = x - mean
    var = (dev * dev).sum(axis=0) / x.shape[0]
    invstd = 1.0 / np.sqrt(var + float(eps))
    z = g * (dev * invstd) + b
    y = np.maximum(z, 0.0) if relu else z
    with np.errstate(over="ignore"):
        y16 = y.astype(np.float16)
    return y, y16, mean, invstd


def bn_add_relu_fwd(x16, res16, gamma32, beta32, eps, relu=True):
    """The end of a bottleneck block: y = [relu](bn(x) + res), the sum formed before the one rounding to FP16.
    Returns (y64, y16, mean64, invstd64)."""
    z, _, mean, invstd = bn_relu_fwd(x16, gamma32, beta32, eps, relu=False)
    y = z + _f16(res16).astype(np.float64)
    if relu:
        y = np.maximum(y, 0.0)
    with np.errstate(over="ignore"):
        return y, y.astype(np.float16), mean, invstd


def bn_relu_bwd(x16, y16, dy16, gamma32, mean32, invstd32, relu=True):
    """Gradient of the map above for the saved statistics (FP32 values, widened).  Returns
    (dx64, dx16, dgamma64, dbeta64, dgamma16, dbeta16)."""
    x = _f16(x16).astype(np.float64)
    dy = _f16(dy16).astype(np.float64)
    g = np.asarray(gamma32, dtype=np.float32).astype(np.float64)
    mean = np.asarray(mean32, dtype=np.float32).astype(np.float64)
    invstd = np.asarray(invstd32, dtype=np.float32).astype(np.float64)
    M = x.shape[0]
    if relu:
        dy = dy * (_f16(y16).astype(np.float64) > 0.0)
    xhat = (x - mean) * invstd
    dbeta = dy.sum(axis=0)
    dgamma = (dy * xhat).sum(axis=0)
    dx = g * invstd * (dy - dbeta / M - xhat * (dgamma / M))
    with np.errstate(over="ignore"):
        return dx, dx.astype(np.float16), dgamma, dbeta, dgamma.astype(np.float16), dbeta.astype(np.float16)
