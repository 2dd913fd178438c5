"""Pins for the float32 entry points of the conv/FC oracle (the single-precision variant compared with in Section 5.4 /
Table 9): against an independent library (torch CPU fp64 conv2d and its autograd), numpy matmul, the adjoint
identities, and the fp16 entry points on inputs both can represent.  Random float32 inputs use all 24 significand
bits, so an entry point that narrowed its inputs to fp16 anywhere would miss the 1e-12 bars by nine orders."""
import numpy as np
import pytest

import oracle
from oracle import conv_desc
from test_oracle_conv import ASYM, torch_ref


def rnd32(rng, shape, scale=1.0):
    return (rng.standard_normal(shape) * scale).astype(np.float32)


@pytest.mark.parametrize("cfg", ASYM)
def test_against_independent_library(cfg):
    N, H, W, C, K, R, S, st, pad = cfg
    d = conv_desc(N, H, W, C, K, R, S, st, pad)
    rng = np.random.default_rng(hash(cfg) % 2**32 + 1)
    x, w, dy = rnd32(rng, (N, H, W, C)), rnd32(rng, (K, R, S, C)), rnd32(rng, (N, d.P, d.Q, K))
    assert np.any(x != x.astype(np.float16).astype(np.float32))          # really more than fp16 holds
    y_ref, dx_ref, dw_ref = torch_ref(d, x, w, dy)
    np.testing.assert_allclose(oracle.conv_fwd(d, x, w), y_ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.conv_bwd_data(d, dy, w), dx_ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.conv_bwd_weight(d, x, dy), dw_ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("cfg", ASYM)
def test_adjoint_identities(cfg):
    N, H, W, C, K, R, S, st, pad = cfg
    d = conv_desc(N, H, W, C, K, R, S, st, pad)
    rng = np.random.default_rng(17)
    x, w, dy = rnd32(rng, (N, H, W, C)), rnd32(rng, (K, R, S, C)), rnd32(rng, (N, d.P, d.Q, K))
    a = np.sum(oracle.conv_fwd(d, x, w) * dy.astype(np.float64))
    b = np.sum(x.astype(np.float64) * oracle.conv_bwd_data(d, dy, w))
    c = np.sum(w.astype(np.float64) * oracle.conv_bwd_weight(d, x, dy))
    scale = abs(a) + 1.0
    assert abs(a - b) <= 1e-11 * scale and abs(a - c) <= 1e-11 * scale


@pytest.mark.parametrize("cfg", ASYM[:5])
def test_same_results_as_the_fp16_entry_points_on_fp16_values(cfg):
    # values both formats hold exactly: the two families must agree to the last bit (same loops, same order)
    N, H, W, C, K, R, S, st, pad = cfg
    d = conv_desc(N, H, W, C, K, R, S, st, pad)
    rng = np.random.default_rng(19)
    x, w, dy = (rng.standard_normal(s).astype(np.float16) for s in ((N, H, W, C), (K, R, S, C), (N, d.P, d.Q, K)))
    f = lambda a: a.astype(np.float32)
    assert np.array_equal(oracle.conv_fwd(d, f(x), f(w)), oracle.conv_fwd(d, x, w))
    assert np.array_equal(oracle.conv_bwd_data(d, f(dy), f(w)), oracle.conv_bwd_data(d, dy, w))
    assert np.array_equal(oracle.conv_bwd_weight(d, f(x), f(dy)), oracle.conv_bwd_weight(d, x, dy))


@pytest.mark.parametrize("cfg", ASYM[:5])
def test_single_element_routines_agree_with_full_tensors(cfg):
    N, H, W, C, K, R, S, st, pad = cfg
    d = conv_desc(N, H, W, C, K, R, S, st, pad)
    rng = np.random.default_rng(23)
    x, w, dy = rnd32(rng, (N, H, W, C)), rnd32(rng, (K, R, S, C)), rnd32(rng, (N, d.P, d.Q, K))
    y, dx, dw = oracle.conv_fwd(d, x, w), oracle.conv_bwd_data(d, dy, w), oracle.conv_bwd_weight(d, x, dy)
    for full, fn, a, b in ((y, oracle.conv_fwd_at, x, w), (dx, oracle.conv_bwd_data_at, dy, w), (dw, oracle.conv_bwd_weight_at, x, dy)):
        idx = np.arange(full.size, dtype=np.int64)
        np.testing.assert_allclose(fn(d, a, b, idx), full.ravel(), rtol=1e-12, atol=1e-12)


def test_fc_is_matmul_and_a_1x1_conv():
    rng = np.random.default_rng(29)
    B, I, O = 5, 24, 7
    x, w, dy = rnd32(rng, (B, I)), rnd32(rng, (O, I)), rnd32(rng, (B, O))
    x64, w64, dy64 = (a.astype(np.float64) for a in (x, w, dy))
    np.testing.assert_allclose(oracle.fc_fwd(B, I, O, x, w), x64 @ w64.T, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.fc_bwd_data(B, I, O, dy, w), dy64 @ w64, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.fc_bwd_weight(B, I, O, dy, x), dy64.T @ x64, rtol=1e-13, atol=1e-13)
    d = conv_desc(B, 1, 1, I, O, 1, 1)
    np.testing.assert_allclose(oracle.conv_fwd(d, x, w).reshape(B, O), oracle.fc_fwd(B, I, O, x, w), rtol=1e-13, atol=1e-13)
