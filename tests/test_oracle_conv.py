"""Pins for the fp64 conv/FC oracle against things other than itself: closed forms,
identities, an independent library (torch CPU fp64 conv2d and its autograd), numpy
matmul, and linear-algebra invariants.  Asymmetric shapes (H != W, R != S, different
strides and pads per axis, C != K) make a swapped index or operand visible."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from oracle import conv_desc


def rnd16(rng, shape, scale=1.0):
    return (rng.standard_normal(shape) * scale).astype(np.float16)


ASYM = [
    # N, H, W, C, K, R, S, stride, pad
    (2, 9, 7, 3, 5, 3, 2, (2, 1), (1, 0)),
    (1, 8, 11, 4, 2, 1, 3, (1, 2), (0, 2)),
    (3, 6, 6, 16, 16, 3, 3, (1, 1), (1, 1)),
    (2, 10, 9, 1, 3, 5, 4, (3, 2), (2, 3)),
    (1, 7, 7, 3, 1, 7, 7, (2, 2), (3, 3)),
    (2, 5, 6, 8, 4, 1, 1, (2, 2), (0, 0)),
    (1, 12, 5, 2, 3, 4, 5, (1, 1), (3, 4)),   # pad >= R-1: whole taps in the border
]


def torch_ref(d, x16, w16, dy16=None):
    """conv2d in fp64 from an independent library, NCHW/KCRS, plus its autograd adjoints."""
    x = torch.from_numpy(x16.astype(np.float64)).permute(0, 3, 1, 2).contiguous().requires_grad_(True)
    w = torch.from_numpy(w16.astype(np.float64)).permute(0, 3, 1, 2).contiguous().requires_grad_(True)
    y = F.conv2d(x, w, stride=(d.stride_h, d.stride_w), padding=(d.pad_h, d.pad_w))
    out = [y.detach().permute(0, 2, 3, 1).numpy()]
    if dy16 is not None:
        dy = torch.from_numpy(dy16.astype(np.float64)).permute(0, 3, 1, 2).contiguous()
        gx, gw = torch.autograd.grad(y, (x, w), dy)
        out += [gx.permute(0, 2, 3, 1).numpy(), gw.permute(0, 2, 3, 1).numpy()]
    return out


@pytest.mark.parametrize("cfg", ASYM)
def test_against_independent_library(cfg):
    N, H, W, C, K, R, S, st, pad = cfg
    d = conv_desc(N, H, W, C, K, R, S, st, pad)
    rng = np.random.default_rng(hash(cfg) % 2**32)
    x, w, dy = rnd16(rng, (N, H, W, C)), rnd16(rng, (K, R, S, C)), rnd16(rng, (N, d.P, d.Q, K))
    y_ref, dx_ref, dw_ref = torch_ref(d, x, w, dy)
    assert y_ref.shape == (N, d.P, d.Q, K)
    np.testing.assert_allclose(oracle.conv_fwd(d, x, w), y_ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.conv_bwd_data(d, dy, w), dx_ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.conv_bwd_weight(d, x, dy), dw_ref, rtol=1e-12, atol=1e-12)


def test_delta_kernel_reproduces_input_exactly():
    # W[k,r0,s0,c] = [k==c] at the centre tap, stride 1, "same" padding  =>  Y == X
    rng = np.random.default_rng(1)
    N, H, W, C = 2, 6, 5, 4
    x = rnd16(rng, (N, H, W, C), 30.0)
    w = np.zeros((C, 3, 3, C), np.float16)
    for k in range(C):
        w[k, 1, 1, k] = 1.0
    d = conv_desc(N, H, W, C, C, 3, 3, 1, 1)
    y = oracle.conv_fwd(d, x, w)
    assert np.array_equal(y, x.astype(np.float64))
    assert np.array_equal(oracle.round_to_half(y), x.view(np.uint16))
    # shifted delta: tap (0,2) reads x[h-1, w+1]
    w2 = np.zeros_like(w)
    for k in range(C):
        w2[k, 0, 2, k] = 1.0
    y2 = oracle.conv_fwd(d, x, w2)
    xp = np.zeros((N, H + 2, W + 2, C))
    xp[:, 1:-1, 1:-1] = x
    assert np.array_equal(y2, xp[:, 0:H, 2:W + 2])


@pytest.mark.parametrize("R,S,st,pad", [(3, 3, 1, 1), (5, 3, 2, (2, 1)), (7, 7, 2, 3), (2, 4, (1, 3), (1, 2))])
def test_all_ones_counts_valid_taps(R, S, st, pad):
    # X = 1, W = 1  =>  Y[n,p,q,k] = C * #(taps inside the image): a closed form that needs no convolution code
    N, H, W, C, K = 1, 9, 8, 3, 2
    d = conv_desc(N, H, W, C, K, R, S, st, pad)
    y = oracle.conv_fwd(d, np.ones((N, H, W, C), np.float16), np.ones((K, R, S, C), np.float16))
    for p in range(d.P):
        nh = sum(0 <= p * d.stride_h - d.pad_h + r < H for r in range(R))
        for q in range(d.Q):
            nw = sum(0 <= q * d.stride_w - d.pad_w + s < W for s in range(S))
            assert np.all(y[0, p, q, :] == C * nh * nw)
    # the adjoints of the all-ones problem have closed forms too
    dy = np.ones((N, d.P, d.Q, K), np.float16)
    dw = oracle.conv_bwd_weight(d, np.ones((N, H, W, C), np.float16), dy)
    for r in range(R):
        nh = sum(0 <= p * d.stride_h - d.pad_h + r < H for p in range(d.P))
        for s in range(S):
            nw = sum(0 <= q * d.stride_w - d.pad_w + s < W for q in range(d.Q))
            assert np.all(dw[:, r, s, :] == N * nh * nw)
    # sum over dX counts every forward term once per (k,c), exactly as sum over Y does
    assert oracle.conv_bwd_data(d, dy, np.ones((K, R, S, C), np.float16)).sum() == y.sum()


@pytest.mark.parametrize("cfg", ASYM)
def test_adjoint_identities(cfg):
    # <fwd(X,W), dY> = <X, bwd_data(dY,W)> = <W, bwd_weight(X,dY)>  (bilinear map => this pins both adjoints)
    N, H, W, C, K, R, S, st, pad = cfg
    d = conv_desc(N, H, W, C, K, R, S, st, pad)
    rng = np.random.default_rng(7)
    x, w, dy = rnd16(rng, (N, H, W, C)), rnd16(rng, (K, R, S, C)), rnd16(rng, (N, d.P, d.Q, K))
    a = np.sum(oracle.conv_fwd(d, x, w) * dy.astype(np.float64))
    b = np.sum(x.astype(np.float64) * oracle.conv_bwd_data(d, dy, w))
    c = np.sum(w.astype(np.float64) * oracle.conv_bwd_weight(d, x, dy))
    scale = abs(a) + 1.0
    assert abs(a - b) <= 1e-11 * scale and abs(a - c) <= 1e-11 * scale


def test_one_by_one_conv_is_a_gemm():
    rng = np.random.default_rng(3)
    N, H, W, C, K = 2, 5, 4, 24, 10
    x, w = rnd16(rng, (N, H, W, C)), rnd16(rng, (K, 1, 1, C))
    d = conv_desc(N, H, W, C, K, 1, 1)
    y = oracle.conv_fwd(d, x, w).reshape(N * H * W, K)
    ref = x.reshape(-1, C).astype(np.float64) @ w.reshape(K, C).astype(np.float64).T
    np.testing.assert_allclose(y, ref, rtol=1e-13, atol=1e-13)
    dy = rnd16(rng, (N, H, W, K))
    np.testing.assert_allclose(oracle.conv_bwd_data(d, dy, w).reshape(-1, C),
                               dy.reshape(-1, K).astype(np.float64) @ w.reshape(K, C).astype(np.float64), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.conv_bwd_weight(d, x, dy).reshape(K, C),
                               dy.reshape(-1, K).astype(np.float64).T @ x.reshape(-1, C).astype(np.float64), rtol=1e-13, atol=1e-13)


def test_strided_backward_data_leaves_unreached_pixels_zero():
    # 1x1 stride 2: only even (h,w) are read by the forward pass, so only they can receive gradient
    rng = np.random.default_rng(4)
    d = conv_desc(2, 8, 8, 4, 6, 1, 1, 2, 0)
    dx = oracle.conv_bwd_data(d, rnd16(rng, (2, d.P, d.Q, 6)), rnd16(rng, (6, 1, 1, 4)))
    mask = np.zeros((8, 8), bool)
    mask[::2, ::2] = True
    assert np.all(dx[:, ~mask, :] == 0.0)
    assert np.all(dx[:, mask, :] != 0.0)
    # 2x2 filter, stride 3, no pad: rows/cols 2, 5 are never touched
    d = conv_desc(1, 8, 8, 2, 3, 2, 2, 3, 0)
    dx = oracle.conv_bwd_data(d, rnd16(rng, (1, d.P, d.Q, 3)), rnd16(rng, (3, 2, 2, 2)))
    assert np.all(dx[:, [2, 5], :, :] == 0) and np.all(dx[:, :, [2, 5], :] == 0) and np.all(dx[:, 0, 0, :] != 0)


def test_linearity_in_each_argument():
    rng = np.random.default_rng(8)
    d = conv_desc(1, 6, 7, 4, 3, 3, 3, 1, 1)
    x1, x2 = rnd16(rng, (1, 6, 7, 4)), rnd16(rng, (1, 6, 7, 4))
    w = rnd16(rng, (3, 3, 3, 4))
    xs = (x1.astype(np.float32) * 2 + x2.astype(np.float32) * 0.5)
    # keep the combination exactly representable: use values on a coarse grid
    x1 = (np.round(x1.astype(np.float32) * 8) / 8).astype(np.float16)
    x2 = (np.round(x2.astype(np.float32) * 8) / 8).astype(np.float16)
    xs = (2 * x1.astype(np.float32) + 0.5 * x2.astype(np.float32)).astype(np.float16)
    assert np.array_equal(xs.astype(np.float64), 2 * x1.astype(np.float64) + 0.5 * x2.astype(np.float64))
    np.testing.assert_allclose(oracle.conv_fwd(d, xs, w), 2 * oracle.conv_fwd(d, x1, w) + 0.5 * oracle.conv_fwd(d, x2, w),
                               rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("cfg", ASYM[:5])
def test_single_element_routines_agree_with_full_tensors(cfg):
    # the *_at routines are written differently (gather / brute-force match of coordinates); pin them to the full ones,
    # which are themselves pinned above
    N, H, W, C, K, R, S, st, pad = cfg
    d = conv_desc(N, H, W, C, K, R, S, st, pad)
    rng = np.random.default_rng(11)
    x, w, dy = rnd16(rng, (N, H, W, C)), rnd16(rng, (K, R, S, C)), rnd16(rng, (N, d.P, d.Q, K))
    y, dx, dw = oracle.conv_fwd(d, x, w), oracle.conv_bwd_data(d, dy, w), oracle.conv_bwd_weight(d, x, dy)
    for full, fn, a, b in ((y, oracle.conv_fwd_at, x, w), (dx, oracle.conv_bwd_data_at, dy, w), (dw, oracle.conv_bwd_weight_at, x, dy)):
        idx = np.arange(full.size, dtype=np.int64)
        np.testing.assert_allclose(fn(d, a, b, idx), full.ravel(), rtol=1e-12, atol=1e-12)


def test_fc_is_matmul_and_a_1x1_conv():
    rng = np.random.default_rng(9)
    B, I, O = 5, 24, 7
    x, w, dy = rnd16(rng, (B, I)), rnd16(rng, (O, I)), rnd16(rng, (B, O))
    x64, w64, dy64 = (a.astype(np.float64) for a in (x, w, dy))
    np.testing.assert_allclose(oracle.fc_fwd(B, I, O, x, w), x64 @ w64.T, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.fc_bwd_data(B, I, O, dy, w), dy64 @ w64, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.fc_bwd_weight(B, I, O, dy, x), dy64.T @ x64, rtol=1e-13, atol=1e-13)
    d = conv_desc(B, 1, 1, I, O, 1, 1)
    np.testing.assert_allclose(oracle.conv_fwd(d, x, w).reshape(B, O), oracle.fc_fwd(B, I, O, x, w), rtol=1e-13, atol=1e-13)


def test_input_size_is_checked():
    d = conv_desc(1, 4, 4, 2, 2, 3, 3, 1, 1)
    with pytest.raises(ValueError):
        oracle.conv_fwd(d, np.zeros((1, 4, 4, 3), np.float16), np.zeros((2, 3, 3, 2), np.float16))
    with pytest.raises(TypeError):
        oracle.conv_fwd(d, np.zeros((1, 4, 4, 2), np.float32), np.zeros((2, 3, 3, 2), np.float16))
