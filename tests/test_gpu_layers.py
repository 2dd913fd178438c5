"""GPU parity of the small layers (residual add, ReLU gradient, pooling, bias, softmax cross-entropy gradient) through
the C ABI against oracle/layers.py.  Bars: bit-exact where FP32 arithmetic on FP16 inputs is exact (add, ReLU
gradient, max pooling forward, bias add); at most one FP16 step from the oracle's rounding, and rel-L2 <= 1e-3, where
an FP32 sum or quotient is rounded a second time on the FP16 store."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_1807_11205_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def jz():
    from paper_1807_11205_amd import api
    api.lib()
    assert torch.cuda.is_available()
    return api


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def h16(key, shape, std=1.0):
    return inputs.normal_f16(inputs.rng_for(5, *key), shape, std=std)


def same_bits(a, b):
    return np.array_equal(np.ascontiguousarray(a).view(np.uint16), np.ascontiguousarray(b).view(np.uint16))


def within_one_step(got16, ref64, ref16, what):
    """Every value is the oracle's FP16 or one of its two neighbours, few differ at all, and the tensor is within 1e-3."""
    g, r16, r64 = got16.ravel(), ref16.ravel(), np.asarray(ref64).ravel()
    diff = np.nonzero(g.view(np.uint16) != r16.view(np.uint16))[0]
    if diff.size:
        up, dn = np.nextafter(r16[diff], np.float16(np.inf)), np.nextafter(r16[diff], np.float16(-np.inf))
        ok = (g[diff] == up) | (g[diff] == dn)
        assert np.all(ok), "%s: %d values more than one FP16 step away" % (what, int((~ok).sum()))
    assert diff.size <= 0.01 * g.size + 2, "%s: %d of %d values differ from the oracle's rounding" % (what, diff.size, g.size)
    den = np.linalg.norm(r64)
    fin = np.isfinite(r64)
    rel = np.linalg.norm(g.astype(np.float64)[fin] - r64[fin]) / den if den > 0 else 0.0
    assert rel <= 1e-3, "%s: rel-L2 %.3g" % (what, rel)


@pytest.mark.parametrize("n", [8, 2048, 8 * 12345, 64 * 56 * 56 * 64])
@pytest.mark.parametrize("relu", [True, False])
def test_add_is_bit_exact(jz, n, relu):
    a, b = h16((1, n), (n,), 2.0), h16((2, n), (n,), 2.0)
    a[:4] = [65504, -65504, 0.0, -0.0]; b[:4] = [65504, -65504, -0.0, -0.0]      # overflow to Inf on the store, signed zeros
    y = torch.empty(n, dtype=torch.float16, device="cuda")
    jz.jz_add_fwd(dev(a), dev(b), y, relu=relu)
    ref = oracle.add_fwd(a, b, relu=relu)[1]
    got = host(y)
    assert np.array_equal(got, ref) and np.isinf(got[0])
    # in place on the first operand
    ta = dev(a)
    jz.jz_add_fwd(ta, dev(b), ta, relu=relu)
    assert np.array_equal(host(ta), ref)


@pytest.mark.parametrize("n", [8, 8 * 777, 64 * 28 * 28 * 512])
def test_relu_gradient_is_bit_exact(jz, n):
    y = np.maximum(h16((3, n), (n,)), np.float16(0))
    y[:6] = np.array([0.0, -0.0, 6e-8, np.inf, np.nan, -1.0], np.float16)        # zero, signed zero, subnormal, Inf, NaN
    dy = h16((4, n), (n,), 8.0)
    dx = torch.empty(n, dtype=torch.float16, device="cuda")
    jz.jz_relu_bwd(dev(y), dev(dy), dx)
    assert same_bits(host(dx), oracle.relu_bwd(y, dy))
    tdy = dev(dy)
    jz.jz_relu_bwd(dev(y), tdy, tdy)                                              # in place on dy
    assert same_bits(host(tdy), oracle.relu_bwd(y, dy))
    # two gradient contributions: the add (one rounding, may overflow to Inf) and the mask in one pass
    dy2 = h16((44, n), (n,), 8.0)
    dy2[:8] = np.array([65504, -65504, 1, 2, 3, 4, 5, 6], np.float16); dy[:8] = np.array([65504, -65504, 1, 2, 3, 4, 5, 6], np.float16)
    y[6:8] = np.float16(1.0)
    want = oracle.relu_bwd(y, oracle.add_fwd(dy, dy2, relu=False)[1])
    jz.jz_relu_bwd_sum(dev(y), dev(dy), dev(dy2), dx)
    assert same_bits(host(dx), want)
    ta = dev(dy)
    jz.jz_relu_bwd_sum(dev(y), ta, dev(dy2), ta)
    assert same_bits(host(ta), want)


POOLS = [(2, 112, 112, 64, 3, 2, 1),      # the ResNet-50 stem pool at a small batch
         (3, 13, 9, 8, 3, 2, 1), (2, 7, 7, 16, 3, 2, 0), (1, 8, 8, 24, 2, 2, 0), (2, 6, 5, 8, 3, 1, 1), (1, 5, 5, 8, 5, 3, 2),
         (2, 55, 55, 96, 3, 2, 0)]       # AlexNet's overlapping pool


@pytest.mark.parametrize("N,H,W,C,window,stride,pad", POOLS)
def test_maxpool_forward_and_backward(jz, N, H, W, C, window, stride, pad):
    x = h16((5, N, H, W, C), (N, H, W, C))
    x = np.maximum(x, np.float16(0))        # after a ReLU: about half the values are zero, so windows tie all the time
    x[0, :, :, 1] = np.round(x[0, :, :, 1])
    P, Q = oracle.pool_out(H, window, stride, pad), oracle.pool_out(W, window, stride, pad)
    y = torch.empty(N * P * Q * C, dtype=torch.float16, device="cuda")
    y2 = torch.empty_like(y)
    arg = torch.full((N * P * Q * C,), 255, dtype=torch.uint8, device="cuda")
    tx = dev(x.ravel())
    jz.jz_maxpool_fwd(N, H, W, C, window, stride, pad, tx, y)
    jz.jz_maxpool_fwd(N, H, W, C, window, stride, pad, tx, y2, arg)
    ry, rarg = oracle.maxpool_fwd(x, window, stride, pad)
    assert same_bits(host(y).reshape(ry.shape), ry) and same_bits(host(y2).reshape(ry.shape), ry)
    # the saved winner (position r * window + s inside the window) names the oracle's first maximum exactly
    a = host(arg).reshape(ry.shape).astype(np.int64)
    pp, qq = np.arange(P)[None, :, None, None], np.arange(Q)[None, None, :, None]
    flat = (pp * stride - pad + a // window) * W + (qq * stride - pad + a % window)
    assert np.array_equal(flat, rarg)
    dy = h16((6, N, H, W, C), ry.shape, 4.0)
    dx = torch.empty(N * H * W * C, dtype=torch.float16, device="cuda")
    jz.jz_maxpool_bwd(N, H, W, C, window, stride, pad, tx, dev(dy.ravel()), dx)
    r64, r16 = oracle.maxpool_bwd(x, dy, window, stride, pad)
    got = host(dx)
    within_one_step(got, r64, r16, "maxpool dx")
    # from the saved winners, without x: the same bits as the re-derivation
    dx2 = torch.empty_like(dx)
    jz.jz_maxpool_bwd(N, H, W, C, window, stride, pad, None, dev(dy.ravel()), dx2, arg)
    assert same_bits(host(dx2), got)
    # no gradient lost: the column sums of dx and dy agree (fp64 sums of the FP16 values, up to the roundings of summed cells)
    assert np.allclose(got.reshape(N, -1, C).astype(np.float64).sum(axis=1), dy.reshape(N, -1, C).astype(np.float64).sum(axis=1),
                       rtol=2e-3, atol=0.5)


def test_maxpool_negative_inputs_and_signed_zero(jz):
    x = -np.abs(h16((7,), (1, 6, 6, 8))) - np.float16(1.0)      # all negative: padding must not win with a zero
    x[0, 0, 0, :] = -0.0
    x[0, 0, 1, :] = 0.0
    y = torch.empty(1 * 3 * 3 * 8, dtype=torch.float16, device="cuda")
    jz.jz_maxpool_fwd(1, 6, 6, 8, 3, 2, 1, dev(x.ravel()), y)
    ry, _ = oracle.maxpool_fwd(x, 3, 2, 1)
    got = host(y).reshape(ry.shape)
    assert same_bits(got, ry) and np.all(got[0, 1:, 1:, :] < 0)


@pytest.mark.parametrize("N,HW,C", [(4, 49, 2048), (3, 1, 8), (2, 36, 256), (64, 49, 2048)])
def test_global_average_pool(jz, N, HW, C):
    x = h16((8, N, HW, C), (N, HW, 1, C), 3.0) + np.float16(1.0)
    y = torch.empty(N * C, dtype=torch.float16, device="cuda")
    jz.jz_avgpool_fwd(N, HW, C, dev(x.ravel()), y)
    r64, r16 = oracle.avgpool_fwd(x)
    within_one_step(host(y), r64, r16, "avgpool y")
    dy = h16((9, N, C), (N, C))
    dx = torch.empty(N * HW * C, dtype=torch.float16, device="cuda")
    jz.jz_avgpool_bwd(N, HW, C, dev(dy.ravel()), dx)
    d64, d16 = oracle.avgpool_bwd(dy, HW, 1)
    within_one_step(host(dx), d64, d16, "avgpool dx")


@pytest.mark.parametrize("rows,C", [(64, 1000), (1, 8), (130, 40), (4096, 96)])
def test_bias_add_and_gradient(jz, rows, C):
    y, b, dy = h16((10, rows, C), (rows, C)), h16((11, C), (C,)), h16((12, rows, C), (rows, C))
    out = torch.empty(rows * C, dtype=torch.float16, device="cuda")
    jz.jz_bias_add(rows, C, dev(y.ravel()), dev(b), out)
    assert same_bits(host(out).reshape(rows, C), oracle.bias_add(y, b)[1])
    ty = dev(y.ravel())
    jz.jz_bias_add(rows, C, ty, dev(b), ty)
    assert same_bits(host(ty).reshape(rows, C), oracle.bias_add(y, b)[1])
    db = torch.empty(C, dtype=torch.float16, device="cuda")
    jz.jz_bias_grad(rows, C, dev(dy.ravel()), db)
    r64, r16 = oracle.bias_grad(dy)
    within_one_step(host(db), r64, r16, "bias gradient")


@pytest.mark.parametrize("rows,K,S", [(64, 1000, 1024.0), (5, 10, 1.0), (3, 1, 8.0), (7, 1003, 65536.0), (2, 5000, 128.0)])
def test_softmax_cross_entropy_gradient(jz, rows, K, S):
    z = h16((13, rows, K), (rows, K), 3.0)
    z[0, 0] = 60000.0 if K > 1 else z[0, 0]
    lab = inputs.rng_for(5, 14, rows, K).integers(0, K, size=rows).astype(np.int32)
    dz = torch.empty(rows * K, dtype=torch.float16, device="cuda")
    loss = torch.empty(rows, dtype=torch.float32, device="cuda")
    jz.jz_softmax_xent_bwd(rows, K, dev(z.ravel()), dev(lab), dz, loss, loss_scale=S)
    l64, d64, d16 = oracle.softmax_xent(z, lab, S)
    gl, gd = host(loss), host(dz).reshape(rows, K)
    assert np.allclose(gl, l64, rtol=2e-6, atol=2e-6 * (1 + np.abs(z.astype(np.float64)).max()))
    # FP32 exp / divide: relative error of a few 1e-7 before the FP16 rounding
    fin = np.isfinite(d16.astype(np.float64))
    assert np.all(fin) and np.all(np.isfinite(gd))
    err = np.abs(gd.astype(np.float64) - d64)
    assert np.all(err <= 2.0 ** -10 * np.abs(d64) + 2.0 ** -25), "max err %.3g" % err.max()   # half an FP16 step (+ fp32 slack), or the subnormal step
    assert np.linalg.norm(gd.astype(np.float64) - d64) <= 1e-3 * np.linalg.norm(d64)
    # the scale from device memory gives the same bits as the same scale passed by value
    st = torch.zeros(2, dtype=torch.int32, device="cuda")
    jz.jz_loss_scale_init(st, S)
    dz2 = torch.empty_like(dz)
    jz.jz_softmax_xent_bwd(rows, K, dev(z.ravel()), dev(lab), dz2, loss, loss_scale=3.0, state=st)
    assert same_bits(host(dz2), host(dz))


def test_softmax_label_out_of_range(jz):
    z = h16((15,), (3, 16))
    lab = np.array([2, 16, -1], np.int32)
    dz = torch.full((48,), 7.0, dtype=torch.float16, device="cuda")
    loss = torch.zeros(3, dtype=torch.float32, device="cuda")
    jz.jz_softmax_xent_bwd(3, 16, dev(z.ravel()), dev(lab), dz, loss, loss_scale=2.0)
    gl, gd = host(loss), host(dz).reshape(3, 16)
    assert np.isfinite(gl[0]) and np.isnan(gl[1]) and np.isnan(gl[2])
    assert np.all(gd[1:] == 0) and np.any(gd[0] != 0)


def test_argument_errors(jz):
    L = jz.lib()
    t = torch.zeros(4096, dtype=torch.float16, device="cuda")
    u = torch.zeros(4096, dtype=torch.float16, device="cuda")
    v = torch.zeros(4096, dtype=torch.float16, device="cuda")
    p, q, r = t.data_ptr(), u.data_ptr(), v.data_ptr()
    assert L.jz_add_fwd(12, p, q, 1, r, None) == jz.JZ_ERR_SHAPE            # not a multiple of 8
    assert L.jz_add_fwd(-8, p, q, 1, r, None) == jz.JZ_ERR_SHAPE
    assert L.jz_add_fwd(16, None, q, 1, r, None) == jz.JZ_ERR_NULL
    assert L.jz_add_fwd(16, p + 2, q, 1, r, None) == jz.JZ_ERR_ALIGN
    assert L.jz_add_fwd(64, p, q, 1, p + 16, None) == jz.JZ_ERR_ALIAS       # partial overlap is not "in place"
    assert L.jz_add_fwd(0, None, None, 1, None, None) == jz.JZ_OK
    assert L.jz_relu_bwd(64, p, q, p, None) == jz.JZ_ERR_ALIAS              # dx must not be y
    assert L.jz_relu_bwd(64, p, q, q, None) == jz.JZ_OK
    assert L.jz_maxpool_fwd(1, 8, 8, 12, 3, 2, 1, p, q, None, None) == jz.JZ_ERR_SHAPE      # C not a multiple of 8
    assert L.jz_maxpool_fwd(1, 8, 8, 8, 3, 2, 3, p, q, None, None) == jz.JZ_ERR_SHAPE       # pad >= window
    assert L.jz_maxpool_fwd(1, 2, 2, 8, 5, 1, 1, p, q, None, None) == jz.JZ_ERR_SHAPE       # window larger than the padded image
    assert L.jz_maxpool_fwd(1, 40, 40, 8, 17, 1, 0, p, q, None, None) == jz.JZ_ERR_UNSUPPORTED
    assert L.jz_maxpool_fwd(1, 8, 8, 8, 3, 2, 1, p, p, None, None) == jz.JZ_ERR_ALIAS
    assert L.jz_maxpool_fwd(1, 8, 8, 8, 3, 2, 1, p, q, q, None) == jz.JZ_ERR_ALIAS          # the winners must not overlap y
    assert L.jz_maxpool_fwd(1, 8, 8, 8, 3, 2, 1, p, q, r + 4, None) == jz.JZ_ERR_ALIGN
    assert L.jz_maxpool_bwd(1, 8, 8, 8, 3, 2, 1, p, None, q, p, None) == jz.JZ_ERR_ALIAS
    assert L.jz_maxpool_bwd(1, 8, 8, 8, 3, 2, 1, None, None, q, r, None) == jz.JZ_ERR_NULL  # neither x nor the winners
    assert L.jz_maxpool_bwd(1, 8, 8, 8, 3, 2, 1, None, p, q, r, None) == jz.JZ_OK
    assert L.jz_avgpool_fwd(2, 0, 8, p, q, None) == jz.JZ_ERR_SHAPE
    assert L.jz_avgpool_bwd(2, 4, 8, p, p, None) == jz.JZ_ERR_ALIAS
    assert L.jz_bias_add(4, 8, p, p, q, None) == jz.JZ_OK                   # the bias may alias the input, not the output
    assert L.jz_bias_add(4, 8, p, q, q, None) == jz.JZ_ERR_ALIAS
    assert L.jz_bias_grad(4, 12, p, q, None) == jz.JZ_ERR_SHAPE
    assert L.jz_bias_grad(4, 8, p, None, None) == jz.JZ_ERR_NULL
    lab = torch.zeros(8, dtype=torch.int32, device="cuda")
    loss = torch.zeros(8, dtype=torch.float32, device="cuda")
    f = ctypes.c_float
    assert L.jz_softmax_xent_bwd(8, 16, p, lab.data_ptr(), f(0.0), None, q, loss.data_ptr(), None) == jz.JZ_ERR_SHAPE
    assert L.jz_softmax_xent_bwd(8, 0, p, lab.data_ptr(), f(1.0), None, q, loss.data_ptr(), None) == jz.JZ_ERR_SHAPE
    assert L.jz_softmax_xent_bwd(8, 16, p, None, f(1.0), None, q, loss.data_ptr(), None) == jz.JZ_ERR_NULL
    assert L.jz_softmax_xent_bwd(8, 16, p, lab.data_ptr(), f(1.0), None, p, loss.data_ptr(), None) == jz.JZ_ERR_ALIAS
    assert L.jz_softmax_xent_bwd(8, 16, p, lab.data_ptr(), f(1.0), None, q, loss.data_ptr(), None) == jz.JZ_OK
    torch.cuda.synchronize()


def _pool_geometries():
    rng = np.random.default_rng(2024)
    out = []
    while len(out) < 20:
        window, stride = int(rng.integers(1, 8)), int(rng.integers(1, 5))
        pad = int(rng.integers(0, window))
        H, W = int(rng.integers(1, 21)), int(rng.integers(1, 21))
        if window > H + 2 * pad or window > W + 2 * pad:
            continue
        out.append((int(rng.integers(1, 4)), H, W, 8 * int(rng.integers(1, 4)), window, stride, pad))
    return out


@pytest.mark.parametrize("N,H,W,C,window,stride,pad", _pool_geometries())
def test_maxpool_seeded_geometries(jz, N, H, W, C, window, stride, pad):
    """Window 1 to 7 (the compile-time 2 and 3 and the general kernel), strides larger than the window (positions no
    window covers get zero gradient), padding up to window - 1, images smaller than the window."""
    x = np.round(h16((20, N, H, W, C, window), (N, H, W, C)) * np.float16(2)) / np.float16(2)      # coarse values: many ties
    P, Q = oracle.pool_out(H, window, stride, pad), oracle.pool_out(W, window, stride, pad)
    y = torch.empty(N * P * Q * C, dtype=torch.float16, device="cuda")
    arg = torch.empty(N * P * Q * C, dtype=torch.uint8, device="cuda")
    tx = dev(x.ravel())
    jz.jz_maxpool_fwd(N, H, W, C, window, stride, pad, tx, y, arg)
    ry, rarg = oracle.maxpool_fwd(x, window, stride, pad)
    assert same_bits(host(y).reshape(ry.shape), ry)
    a = host(arg).reshape(ry.shape).astype(np.int64)
    pp, qq = np.arange(P)[None, :, None, None], np.arange(Q)[None, None, :, None]
    assert np.array_equal((pp * stride - pad + a // window) * W + (qq * stride - pad + a % window), rarg)
    dy = np.round(h16((21, N, H, W, C, window), ry.shape, 4.0))                                    # integers: the sums are exact
    r64, r16 = oracle.maxpool_bwd(x, dy, window, stride, pad)
    for use_arg in (False, True):
        dx = torch.full((N * H * W * C,), float("nan"), dtype=torch.float16, device="cuda")
        jz.jz_maxpool_bwd(N, H, W, C, window, stride, pad, None if use_arg else tx, dev(dy.ravel()), dx, arg if use_arg else None)
        assert same_bits(host(dx).reshape(r16.shape), r16), "winners from %s" % ("the forward pass" if use_arg else "x")
