"""Pins of oracle/layers.py: explicit loops on tiny inputs, hand-worked cases (ties, padding), closed forms, and the
adjoint identities that tie every backward function to its forward one.  No GPU."""
import math

import numpy as np
import pytest

import oracle


def rnd(seed, shape, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float16)


def test_add_and_relu_backward_hand_values():
    a = np.array([1.5, -2.0, 0.25, 3.0, -0.0], np.float16)
    b = np.array([0.5, 1.0, -0.25, -4.0, 0.0], np.float16)
    y, y16 = oracle.add_fwd(a, b, relu=True)
    assert y.tolist() == [2.0, 0.0, 0.0, 0.0, 0.0] and y16.dtype == np.float16
    assert oracle.add_fwd(a, b, relu=False)[0].tolist() == [2.0, -1.0, 0.0, -1.0, 0.0]
    dy = np.array([7, 8, 9, 10, 11], np.float16)
    assert oracle.relu_bwd(y16, dy).tolist() == [7.0, 0.0, 0.0, 0.0, 0.0]
    # 65504 + 65504 overflows FP16 on the write, as any FP16 store would
    assert np.isinf(oracle.add_fwd(np.array([65504], np.float16), np.array([65504], np.float16))[1][0])


def loops_maxpool(x, window, stride, pad):
    N, H, W, C = x.shape
    P, Q = oracle.pool_out(H, window, stride, pad), oracle.pool_out(W, window, stride, pad)
    y = np.zeros((N, P, Q, C), np.float16)
    arg = np.zeros((N, P, Q, C), np.int64)
    for n in range(N):
        for c in range(C):
            for p in range(P):
                for q in range(Q):
                    best, where = None, None
                    for r in range(window):
                        for s in range(window):
                            h, w = p * stride - pad + r, q * stride - pad + s
                            if 0 <= h < H and 0 <= w < W and (best is None or float(x[n, h, w, c]) > best):
                                best, where = float(x[n, h, w, c]), h * W + w
                    y[n, p, q, c], arg[n, p, q, c] = best, where
    return y, arg


@pytest.mark.parametrize("H,W,window,stride,pad", [(7, 9, 3, 2, 1), (8, 8, 3, 2, 1), (5, 5, 2, 2, 0), (6, 4, 3, 1, 1)])
def test_maxpool_against_explicit_loops(H, W, window, stride, pad):
    x = rnd(H * 100 + W, (2, H, W, 3))
    x[0, :, :, 1] = np.round(x[0, :, :, 1])          # many ties
    y, arg = oracle.maxpool_fwd(x, window, stride, pad)
    ry, rarg = loops_maxpool(x, window, stride, pad)
    assert np.array_equal(y, ry) and np.array_equal(arg, rarg)
    dy = rnd(5, y.shape)
    dx, dx16 = oracle.maxpool_bwd(x, dy, window, stride, pad)
    ref = np.zeros((2, H * W, 3))
    for n in range(2):
        for c in range(3):
            for p in range(y.shape[1]):
                for q in range(y.shape[2]):
                    ref[n, rarg[n, p, q, c], c] += float(dy[n, p, q, c])
    assert np.array_equal(dx.reshape(2, H * W, 3), ref)
    assert np.array_equal(dx16, dx.astype(np.float16))


def test_maxpool_hand_worked_ties_and_padding():
    # one channel, 4x4, window 3 stride 2 pad 1 -> 2x2 windows over rows/cols {-1..1} and {1..3}
    x = np.array([[1, 1, 0, 2],
                  [1, 0, 0, 2],
                  [0, 0, 0, 0],
                  [3, 0, 0, 0]], np.float16).reshape(1, 4, 4, 1)
    y, arg = oracle.maxpool_fwd(x, 3, 2, 1)
    assert y.reshape(2, 2).tolist() == [[1.0, 2.0], [3.0, 2.0]]
    # first maximum in scan order: (0,0); (0,3); (3,0); (1,3)
    assert arg.reshape(2, 2).tolist() == [[0, 3], [12, 7]]
    dy = np.array([[10, 20], [30, 40]], np.float16).reshape(1, 2, 2, 1)
    dx = oracle.maxpool_bwd(x, dy, 3, 2, 1)[0].reshape(4, 4)
    want = np.zeros((4, 4)); want[0, 0] = 10; want[0, 3] = 20; want[3, 0] = 30; want[1, 3] = 40
    assert np.array_equal(dx, want)
    # an all-equal image: every window's gradient lands on its first valid position, and the shared one gets the sum
    x0 = np.zeros((1, 3, 3, 1), np.float16)
    dx0 = oracle.maxpool_bwd(x0, np.array([1, 2, 4, 8], np.float16).reshape(1, 2, 2, 1), 3, 2, 1)[0].reshape(3, 3)
    want0 = np.zeros((3, 3)); want0[0, 0] = 1; want0[0, 1] = 2; want0[1, 0] = 4; want0[1, 1] = 8
    assert np.array_equal(dx0, want0)


def test_maxpool_adjoint_and_mass():
    x = rnd(11, (3, 12, 10, 4))
    dy = rnd(12, (3, 6, 5, 4))
    y, _ = oracle.maxpool_fwd(x, 3, 2, 1)
    dx, _ = oracle.maxpool_bwd(x, dy, 3, 2, 1)
    # y = x[arg], hence <y, dy> = <x, dx>; and no gradient is lost or invented
    assert math.isclose(float((y.astype(np.float64) * dy).sum()), float((x.astype(np.float64) * dx).sum()), rel_tol=1e-12)
    assert np.allclose(dx.sum(axis=(1, 2)), dy.astype(np.float64).sum(axis=(1, 2)), rtol=0, atol=1e-12)


def test_avgpool_closed_forms_and_adjoint():
    x = np.empty((2, 7, 7, 3), np.float16)
    x[..., 0] = 2.5
    x[..., 1] = np.arange(49).reshape(7, 7)                 # mean 24
    x[..., 2] = (np.arange(49).reshape(7, 7) % 2) * 2 - 1   # 24 ones, 25 minus ones
    y, y16 = oracle.avgpool_fwd(x)
    assert np.allclose(y[0], [2.5, 24.0, -1.0 / 49.0], rtol=0, atol=1e-15)
    dy = rnd(3, (2, 3))
    dx, dx16 = oracle.avgpool_bwd(dy, 7, 7)
    assert dx.shape == (2, 7, 7, 3) and np.array_equal(dx[:, 3, 4, :], dy.astype(np.float64) / 49.0)
    xr = rnd(4, (2, 7, 7, 3))
    assert math.isclose(float((oracle.avgpool_fwd(xr)[0] * dy).sum()), float((xr.astype(np.float64) * dx).sum()), rel_tol=1e-12)
    assert np.array_equal(dx16, dx.astype(np.float16))


def test_bias_add_and_gradient():
    dy = rnd(6, (50, 8))
    db, db16 = oracle.bias_grad(dy)
    for c in range(8):
        assert math.isclose(db[c], math.fsum(float(v) for v in dy[:, c]), rel_tol=1e-14, abs_tol=1e-14)
    b = rnd(7, (8,))
    out, out16 = oracle.bias_add(np.zeros((50, 8), np.float16), b)
    assert math.isclose(float((out * dy).sum()), float((b.astype(np.float64) * db).sum()), rel_tol=1e-12)
    y = rnd(8, (50, 8))
    assert np.array_equal(oracle.bias_add(y, b)[0][17], y[17].astype(np.float64) + b.astype(np.float64))


def test_softmax_closed_forms():
    N, K, S = 4, 10, 128.0
    z = np.full((N, K), 3.0, np.float16)
    lab = np.array([0, 3, 9, 3])
    loss, dz, dz16 = oracle.softmax_xent(z, lab, S)
    assert np.allclose(loss, math.log(K), rtol=1e-15)
    want = np.full((N, K), S / K / N); want[np.arange(N), lab] -= S / N
    assert np.allclose(dz, want, rtol=1e-14)
    # two classes: the sigmoid
    z2 = np.array([[1.5, -0.5]], np.float16)
    loss2, dz2, _ = oracle.softmax_xent(z2, [0], 1.0)
    p0 = 1.0 / (1.0 + math.exp(-2.0))
    assert math.isclose(loss2[0], -math.log(p0), rel_tol=1e-14) and np.allclose(dz2[0], [p0 - 1.0, 1.0 - p0], rtol=1e-13)
    # the largest FP16 logits do not overflow, and a shift of all logits changes nothing
    zl = np.array([[60000.0, 59990.0, -60000.0]], np.float16)
    l3, d3, _ = oracle.softmax_xent(zl, [1], 1.0)
    assert np.isfinite(l3[0]) and np.all(np.isfinite(d3))
    za = np.array([[8.0, -2.0, 0.0]], np.float16)
    l4, d4, _ = oracle.softmax_xent(za, [1], 1.0)
    l5, d5, _ = oracle.softmax_xent((za + np.float16(16.0)).astype(np.float16), [1], 1.0)
    assert math.isclose(l4[0], l5[0], rel_tol=1e-13) and np.allclose(d4, d5, rtol=1e-12)
    assert math.isclose(l4[0], math.log(math.exp(8.0) + math.exp(-2.0) + 1.0) + 2.0, rel_tol=1e-14)


def test_softmax_gradient_against_central_differences():
    rng = np.random.default_rng(9)
    N, K, S = 3, 6, 4.0
    z = (rng.integers(-256, 257, size=(N, K)) / 128.0).astype(np.float16)     # multiples of 2^-7, |z| <= 2: z +- 2^-7 is exact
    lab = np.array([1, 5, 0])
    _, dz, dz16 = oracle.softmax_xent(z, lab, S)
    assert np.allclose(dz.sum(axis=1), 0.0, atol=1e-15)
    h = 2.0 ** -7
    for n in range(N):
        for j in range(K):
            zp, zm = z.copy(), z.copy()
            zp[n, j] += np.float16(h); zm[n, j] -= np.float16(h)
            lp = oracle.softmax_xent(zp, lab, S)[0].mean()
            lm = oracle.softmax_xent(zm, lab, S)[0].mean()
            assert abs(S * (lp - lm) / (2 * h) - dz[n, j]) < 2e-5 * S
    assert np.array_equal(dz16, dz.astype(np.float16))
