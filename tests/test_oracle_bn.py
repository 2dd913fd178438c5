"""Pins of the batch-normalization oracle (oracle/bn.py): brute force, the invariants the two formulas of the paper's
Section 4.2 imply, and finite differences of the forward map for the backward pass.  No GPU."""
import numpy as np
import pytest

import oracle


def _case(seed, rows, C, shift=0.0, scale=1.0):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((rows, C)) * scale + shift).astype(np.float16)
    gamma = (1.0 + 0.5 * rng.standard_normal(C)).astype(np.float32)
    beta = (0.3 * rng.standard_normal(C)).astype(np.float32)
    dy = rng.standard_normal((rows, C)).astype(np.float16)
    return x, gamma, beta, dy


def test_forward_against_explicit_loops():
    x, gamma, beta, _ = _case(1, 7, 3, shift=0.7, scale=2.0)
    eps = 1e-3
    y, y16, mean, invstd = oracle.bn_relu_fwd(x, gamma, beta, eps, relu=True)
    for c in range(3):
        col = [float(v) for v in x[:, c]]
        mu = sum(col) / 7
        var = sum((v - mu) ** 2 for v in col) / 7
        assert abs(mean[c] - mu) < 1e-14 and abs(invstd[c] - (var + eps) ** -0.5) < 1e-13
        for r in range(7):
            z = float(gamma[c]) * (col[r] - mu) / (var + eps) ** 0.5 + float(beta[c])
            assert abs(y[r, c] - max(z, 0.0)) < 1e-13
    assert np.array_equal(y16, y.astype(np.float16))


def test_normalised_output_has_the_moments_the_formulas_imply():
    x, gamma, beta, _ = _case(2, 500, 8, shift=-1.5, scale=3.0)
    eps = 1e-5
    y, _, mean, invstd = oracle.bn_relu_fwd(x, gamma, beta, eps, relu=False)
    xf = x.astype(np.float64)
    var = xf.var(axis=0)
    assert np.allclose(y.mean(axis=0), beta.astype(np.float64), atol=1e-12)
    assert np.allclose(y.var(axis=0), gamma.astype(np.float64) ** 2 * var / (var + eps), rtol=1e-12)
    assert np.allclose(mean, xf.mean(axis=0)) and np.allclose(invstd, 1 / np.sqrt(var + eps))


def test_constant_channel_gives_beta_and_relu_clips():
    x = np.full((10, 8), 2.5, np.float16)
    gamma = np.arange(1, 9, dtype=np.float32)
    beta = np.array([-1, 1, -2, 2, -3, 3, 0, 0.5], np.float32)
    y, y16, mean, invstd = oracle.bn_relu_fwd(x, gamma, beta, 1e-5, relu=True)
    assert np.all(mean == 2.5) and np.allclose(invstd, 1e-5 ** -0.5)
    assert np.array_equal(y, np.broadcast_to(np.maximum(beta, 0).astype(np.float64), (10, 8)))


def test_affine_invariance_without_eps():
    # exact in fp16: powers of two and small integers
    rng = np.random.default_rng(3)
    x = rng.integers(-8, 9, size=(64, 8)).astype(np.float16)
    gamma = np.ones(8, np.float32)
    beta = np.zeros(8, np.float32)
    y0 = oracle.bn_relu_fwd(x, gamma, beta, 0.0, relu=False)[0]
    y1 = oracle.bn_relu_fwd((4 * x + 16).astype(np.float16), gamma, beta, 0.0, relu=False)[0]
    assert np.allclose(y0, y1, atol=1e-13)


@pytest.mark.parametrize("relu", [False, True])
def test_backward_is_the_gradient_of_the_forward_map(relu):
    x, gamma, beta, dy = _case(4, 12, 4, shift=0.2)
    eps = 1e-2
    xf, dyf = x.astype(np.float64), dy.astype(np.float64)

    def fwd64(xv, gv, bv):      # the two formulas again, on fp64 perturbed values (the oracle takes fp16 / fp32 inputs)
        mu = xv.mean(axis=0)
        var = ((xv - mu) ** 2).mean(axis=0)
        z = gv * (xv - mu) / np.sqrt(var + eps) + bv
        return np.maximum(z, 0) if relu else z

    y, y16, mean, invstd = oracle.bn_relu_fwd(x, gamma, beta, eps, relu=relu)
    z = fwd64(xf, gamma.astype(np.float64), beta.astype(np.float64))
    if relu:
        assert np.min(np.abs(z[z != 0])) > 1e-3          # no value sits on the kink
    # the saved statistics enter as fp32: widen them exactly as the oracle does, but compare against the gradient taken
    # with the exact fp64 statistics (difference ~1e-7 relative)
    dx, _, dgamma, dbeta, _, _ = oracle.bn_relu_bwd(x, y16, dy, gamma, mean.astype(np.float32), invstd.astype(np.float32), relu=relu)
    L = lambda xv, gv, bv: float(np.sum(dyf * fwd64(xv, gv, bv)))
    h = 1e-6
    g64, b64 = gamma.astype(np.float64), beta.astype(np.float64)
    for (r, c) in [(0, 0), (3, 1), (7, 2), (11, 3), (5, 0)]:
        e = np.zeros_like(xf); e[r, c] = h
        fd = (L(xf + e, g64, b64) - L(xf - e, g64, b64)) / (2 * h)
        assert abs(fd - dx[r, c]) <= 1e-5 * max(1.0, abs(fd)), (r, c, fd, dx[r, c])
    for c in range(4):
        e = np.zeros(4); e[c] = h
        fdg = (L(xf, g64 + e, b64) - L(xf, g64 - e, b64)) / (2 * h)
        fdb = (L(xf, g64, b64 + e) - L(xf, g64, b64 - e)) / (2 * h)
        assert abs(fdg - dgamma[c]) <= 1e-5 * max(1.0, abs(fdg)) and abs(fdb - dbeta[c]) <= 1e-5 * max(1.0, abs(fdb))


def test_backward_invariants_and_mask():
    x, gamma, beta, dy = _case(5, 300, 16, shift=1.0, scale=2.0)
    y, y16, mean, invstd = oracle.bn_relu_fwd(x, gamma, beta, 1e-5, relu=True)
    m32, i32 = mean.astype(np.float32), invstd.astype(np.float32)
    dx, dx16, dgamma, dbeta, dg16, db16 = oracle.bn_relu_bwd(x, y16, dy, gamma, m32, i32, relu=True)
    xhat = (x.astype(np.float64) - m32.astype(np.float64)) * i32.astype(np.float64)
    # the gradient with respect to x is orthogonal to the two directions batch normalization removes
    assert np.allclose(dx.sum(axis=0), 0, atol=1e-5)                                      # exact only for exact statistics
    assert np.allclose((dx * xhat).sum(axis=0), 0, atol=1e-3 * np.abs(dgamma).max())
    masked = dy.astype(np.float64) * (y16.astype(np.float64) > 0)
    assert np.allclose(dbeta, masked.sum(axis=0)) and np.allclose(dgamma, (masked * xhat).sum(axis=0))
    # positions the ReLU switched off contribute nothing: zeroing dy there changes no output
    dy2 = dy.copy(); dy2[y16 <= 0] = 0
    again = oracle.bn_relu_bwd(x, y16, dy2, gamma, m32, i32, relu=True)
    assert np.array_equal(again[0], dx) and np.array_equal(again[2], dgamma)
    assert np.array_equal(dx16, dx.astype(np.float16)) and np.array_equal(dg16, dgamma.astype(np.float16)) and np.array_equal(db16, dbeta.astype(np.float16))
    # gamma = 0 stops all gradient to x
    assert np.all(oracle.bn_relu_bwd(x, y16, dy, np.zeros(16, np.float32), m32, i32, relu=False)[0] == 0)


def test_residual_variant_adds_before_the_relu_and_rounds_once():
    x, gamma, beta, _ = _case(21, 9, 4, shift=0.3, scale=1.5)
    res = np.random.default_rng(22).standard_normal((9, 4)).astype(np.float16)
    eps = 1e-4
    z = oracle.bn_relu_fwd(x, gamma, beta, eps, relu=False)[0]
    y, y16, mean, invstd = oracle.bn_add_relu_fwd(x, res, gamma, beta, eps, relu=True)
    for r in range(9):
        for c in range(4):
            assert y[r, c] == max(z[r, c] + float(res[r, c]), 0.0)
    assert np.array_equal(y16, y.astype(np.float16))
    # the sum is NOT rounded in between: a residual that cancels z to within an FP16 step of z leaves the small remainder
    big = (-z).astype(np.float16)
    y2 = oracle.bn_add_relu_fwd(x, big, gamma, beta, eps, relu=False)[0]
    assert np.array_equal(y2, z + big.astype(np.float64)) and np.any(y2 != 0) and np.all(np.abs(y2) <= np.abs(z) * 2.0 ** -10 + 1e-7)
    # zero residual: the plain layer; statistics never depend on the residual
    y3, _, m3, i3 = oracle.bn_add_relu_fwd(x, np.zeros_like(res), gamma, beta, eps, relu=True)
    assert np.array_equal(y3, oracle.bn_relu_fwd(x, gamma, beta, eps, relu=True)[0]) and np.array_equal(m3, mean) and np.array_equal(i3, invstd)
