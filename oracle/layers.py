"""fp64 oracle of the small layers between the convolutions of ResNet-50 -- TEST INFRASTRUCTURE ONLY.

The paper trains stock ResNet-50 / AlexNet (Section 5) and does not restate these layers; each function below is the
layer's textbook definition written out, evaluated in fp64 on the FP16 inputs, with one rounding to FP16 at the end
(the storage type of every forward / backward tensor in Section 4.1).  Tensors are NHWC.

Conventions this oracle defines:
  * max pooling ignores padding (a window is clipped to the image); its gradient goes to the FIRST maximum of the
    window in (row, column) scan order, and a pixel that wins several windows receives the sum;
  * the global average pool divides by H*W; its gradient spreads dy / (H*W) over the positions;
  * the bias gradient is the column sum over all rows;
  * softmax cross-entropy: loss_n = log(sum_j exp(z_nj)) - z_n,label; the gradient handed to the backward pass is
    loss_scale * (softmax(z_n) - onehot(label_n)) / N, i.e. the gradient of the batch-mean loss times the loss scale
    of Section 4.1.
"""
import numpy as np


def _f16(a):
    a = np.asarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.float16)
    if a.dtype != np.float16:
        raise TypeError("expected fp16 data, got %s" % a.dtype)
    return a


def _to16(v):
    with np.errstate(over="ignore"):
        return np.asarray(v, dtype=np.float64).astype(np.float16)


def add_fwd(a16, b16, relu=True):
    """y = [relu](a + b): the residual connection.  Returns (y64, y16)."""
    y = _f16(a16).astype(np.float64) + _f16(b16).astype(np.float64)
    if relu:
        y = np.maximum(y, 0.0)
    return y, _to16(y)


def relu_bwd(y16, dy16):
    """dx = dy where the forward output was positive, else 0 (exact: returns FP16)."""
    y, dy = _f16(y16), _f16(dy16)
    return np.where(y.astype(np.float64) > 0.0, dy, np.float16(0.0))


def pool_out(size, window, stride, pad):
    return (size + 2 * pad - window) // stride + 1


def maxpool_fwd(x16, window, stride, pad):
    """x[N,H,W,C] -> y[N,P,Q,C] (FP16, exact) and the flat (h*W + w) index of each window's first maximum."""
    x = _f16(x16).astype(np.float64)
    N, H, W, C = x.shape
    P, Q = pool_out(H, window, stride, pad), pool_out(W, window, stride, pad)
    y = np.full((N, P, Q, C), -np.inf)
    arg = np.full((N, P, Q, C), -1, np.int64)
    for p in range(P):
        for q in range(Q):
            for r in range(window):
                for s in range(window):
                    h, w = p * stride - pad + r, q * stride - pad + s
                    if 0 <= h < H and 0 <= w < W:
                        v = x[:, h, w, :]
                        better = (v > y[:, p, q, :]) | (arg[:, p, q, :] < 0)
                        y[:, p, q, :] = np.where(better, v, y[:, p, q, :])
                        arg[:, p, q, :] = np.where(better, h * W + w, arg[:, p, q, :])
    return y.astype(np.float16), arg


def maxpool_bwd(x16, dy16, window, stride, pad):
    """dx[N,H,W,C]: every dy goes to its window's first maximum.  Returns (dx64, dx16)."""
    x = _f16(x16)
    N, H, W, C = x.shape
    dy = _f16(dy16).astype(np.float64)
    _, arg = maxpool_fwd(x, window, stride, pad)
    dx = np.zeros((N, H * W, C))
    n_idx = np.arange(N)[:, None]
    c_idx = np.arange(C)[None, :]
    for p in range(arg.shape[1]):
        for q in range(arg.shape[2]):
            np.add.at(dx, (n_idx, arg[:, p, q, :], c_idx), dy[:, p, q, :])
    dx = dx.reshape(N, H, W, C)
    return dx, _to16(dx)


def avgpool_fwd(x16):
    """Global average pool x[N,H,W,C] -> y[N,C].  Returns (y64, y16)."""
    x = _f16(x16).astype(np.float64)
    y = x.sum(axis=(1, 2)) / (x.shape[1] * x.shape[2])
    return y, _to16(y)


def avgpool_bwd(dy16, H, W):
    """dy[N,C] -> dx[N,H,W,C] = dy / (H*W) at every position.  Returns (dx64, dx16)."""
    dy = _f16(dy16).astype(np.float64)
    dx = np.broadcast_to((dy / (H * W))[:, None, None, :], (dy.shape[0], H, W, dy.shape[1])).copy()
    return dx, _to16(dx)


def bias_add(y16, b16):
    """y[rows,C] + b[C].  Returns (out64, out16)."""
    out = _f16(y16).astype(np.float64) + _f16(b16).astype(np.float64)[None, :]
    return out, _to16(out)


def bias_grad(dy16):
    """db[C] = sum over rows of dy[rows,C].  Returns (db64, db16)."""
    db = _f16(dy16).astype(np.float64).sum(axis=0)
    return db, _to16(db)


def softmax_xent(z16, labels, loss_scale):
    """Per-sample losses (fp64) and the loss-scaled gradient of their mean with respect to the logits:
    returns (loss64[N], dz64[N,classes], dz16)."""
    z = _f16(z16).astype(np.float64)
    N = z.shape[0]
    lab = np.asarray(labels, dtype=np.int64)
    m = z.max(axis=1, keepdims=True)
    e = np.exp(z - m)
    se = e.sum(axis=1, keepdims=True)
    loss = (np.log(se) + m)[:, 0] - z[np.arange(N), lab]
    p = e / se
    p[np.arange(N), lab] -= 1.0
    dz = float(loss_scale) * p / N
    return loss, dz, _to16(dz)
