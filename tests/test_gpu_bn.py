"""GPU parity of jz_bn_relu_fwd / jz_bn_relu_bwd (through the C ABI) against the fp64 oracle of Section 4.2's formulas.

Tolerances: FP16 tensors (y, dx) relative L2 <= 1e-3 like every other FP16 output of the library (one rounding to FP16
contributes ~2.8e-4); the FP32 statistics: mean within 1e-5 of the channel's scale (|mean| + std), invstd within 1e-4
relative (the variance is formed as E[x^2] - mean^2 from FP32 slab sums); the FP16 parameter gradients within 2e-3 of
max(|value|, sqrt(rows) * 1e-2) (their own FP16 rounding is 4.9e-4 relative)."""
import numpy as np
import pytest
import torch

from paper_1807_11205_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def jz():
    from paper_1807_11205_amd import api
    api.lib()
    assert torch.cuda.is_available()
    return api


def _inputs(key, rows, C, shift=0.5, scale=1.5, dy_std=4.0):
    rng = inputs.rng_for(30, *key)
    x = (rng.standard_normal((rows, C), dtype=np.float32) * np.float32(scale) + np.float32(shift) *
         rng.standard_normal(C, dtype=np.float32)).astype(np.float16)
    gamma = (1.0 + 0.3 * rng.standard_normal(C, dtype=np.float32)).astype(np.float32)
    beta = (0.2 * rng.standard_normal(C, dtype=np.float32)).astype(np.float32)
    dy = inputs.normal_f16(rng, (rows, C), std=dy_std)
    return x, gamma, beta, dy


def _run(jz, x, gamma, beta, dy, eps, relu):
    import jzt
    import oracle
    rows, C = x.shape
    dev = jzt.DEV
    X, G, B, DY = jzt.to_dev(x), jzt.to_dev(gamma), jzt.to_dev(beta), jzt.to_dev(dy)
    Y = torch.empty_like(X); DX = torch.empty_like(X)
    mean = torch.empty(C, dtype=torch.float32, device=dev); invstd = torch.empty_like(mean)
    dg = torch.empty(C, dtype=torch.float16, device=dev); db = torch.empty_like(dg)
    ws = torch.empty(max(jz.jz_bn_workspace_bytes(rows, C), 16), dtype=torch.uint8, device=dev)
    jz.jz_bn_relu_fwd(rows, C, X, G, B, eps, relu, Y, mean, invstd, ws)
    ws.fill_(0xCD)   # the workspace carries nothing from the forward to the backward call
    jz.jz_bn_relu_bwd(rows, C, X, Y if relu else None, DY, G, mean, invstd, relu, DX, dg, db, ws)
    torch.cuda.synchronize()
    y_gpu, mean_gpu, invstd_gpu = Y.cpu().numpy(), mean.cpu().numpy(), invstd.cpu().numpy()
    # forward against the oracle
    y64, y16, m64, i64 = oracle.bn_relu_fwd(x, gamma, beta, eps, relu=relu)
    std = 1.0 / i64
    assert np.all(np.abs(mean_gpu - m64) <= 1e-5 * (np.abs(m64) + std)), np.max(np.abs(mean_gpu - m64))
    assert np.all(np.abs(invstd_gpu - i64) <= 1e-4 * i64), np.max(np.abs(invstd_gpu - i64) / i64)
    assert jzt.rel_l2(y_gpu, y64) <= 1e-3
    # backward against the oracle on the same inputs: the GPU's own y16 (mask) and statistics
    dx64, _, dg64, db64, _, _ = oracle.bn_relu_bwd(x, y_gpu, dy, gamma, mean_gpu, invstd_gpu, relu=relu)
    assert jzt.rel_l2(DX.cpu().numpy(), dx64) <= 1e-3
    floor = np.sqrt(rows) * 1e-2
    for got, ref in ((dg.cpu().numpy(), dg64), (db.cpu().numpy(), db64)):
        err = np.abs(got.astype(np.float64) - ref)
        assert np.all(err <= 2e-3 * np.maximum(np.abs(ref), floor)), float(np.max(err / np.maximum(np.abs(ref), floor)))
    return y_gpu, y16


@pytest.mark.parametrize("rows,C", [(2 * 14 * 14, 16), (3 * 9 * 9, 64), (1000, 96), (5 * 7 * 7, 2048), (4099, 256), (1, 8), (777, 384)])
@pytest.mark.parametrize("relu", [True, False])
def test_bn_relu_against_the_oracle(jz, rows, C, relu):
    x, gamma, beta, dy = _inputs((rows, C), rows, C)
    _run(jz, x, gamma, beta, dy, 1e-5, relu)


def test_resnet_sized_layer_and_determinism(jz):
    # 64 x 56 x 56 positions of 64 channels (the first batch normalization of ResNet-50 at batch 64 has 4x this): many
    # slabs, the grid-stride apply kernels, and two runs must agree bit for bit
    rows, C = 64 * 28 * 28, 64
    x, gamma, beta, dy = _inputs((1,), rows, C, shift=2.0)
    y1, _ = _run(jz, x, gamma, beta, dy, 1e-5, True)
    y2, _ = _run(jz, x, gamma, beta, dy, 1e-5, True)
    assert np.array_equal(y1.view(np.uint16), y2.view(np.uint16))


def test_constant_channels_and_exact_cases(jz):
    import jzt
    rows, C = 256, 16
    x = np.zeros((rows, C), np.float16)
    x[:, :8] = 3.0                                     # constant channels: variance 0, output = beta exactly
    x[:, 8:] = np.where(np.arange(rows)[:, None] % 2 == 0, 1.0, -1.0)   # +-1: mean 0, variance 1
    gamma = np.full(C, 2.0, np.float32)
    beta = np.linspace(-1, 1, C).astype(np.float32)
    dev = jzt.DEV
    X, G, B = jzt.to_dev(x), jzt.to_dev(gamma), jzt.to_dev(beta)
    Y = torch.empty_like(X)
    mean = torch.empty(C, dtype=torch.float32, device=dev); invstd = torch.empty_like(mean)
    ws = torch.empty(jz.jz_bn_workspace_bytes(rows, C), dtype=torch.uint8, device=dev)
    jz.jz_bn_relu_fwd(rows, C, X, G, B, 0.0625, False, Y, mean, invstd, ws)
    torch.cuda.synchronize()
    y = Y.cpu().numpy().astype(np.float64)
    assert np.array_equal(mean.cpu().numpy(), np.r_[np.full(8, 3.0), np.zeros(8)].astype(np.float32))
    assert np.array_equal(invstd.cpu().numpy()[:8], np.full(8, 4.0, np.float32))          # 1 / sqrt(0 + 1/16)
    assert np.array_equal(y[:, :8], np.broadcast_to(beta[:8].astype(np.float16).astype(np.float64), (rows, 8)))
    expect = (2.0 * x[:, 8:].astype(np.float64) / np.sqrt(1.0625) + beta[8:]).astype(np.float16)
    assert np.array_equal(Y.cpu().numpy()[:, 8:].view(np.uint16), expect.view(np.uint16))


def test_bn_argument_errors(jz):
    import jzt
    dev = jzt.DEV
    with pytest.raises(jz.JzError):
        jz.jz_bn_workspace_bytes(0, 64)
    with pytest.raises(jz.JzError):
        jz.jz_bn_workspace_bytes(100, 60)          # not a multiple of 8
    with pytest.raises(jz.JzError):
        jz.jz_bn_workspace_bytes(100, 4096)        # more than 2048 channels
    rows, C = 64, 64
    X = torch.zeros(rows * C, dtype=torch.float16, device=dev)
    f = lambda: torch.zeros(C, dtype=torch.float32, device=dev)
    small = torch.empty(16, dtype=torch.uint8, device=dev)
    with pytest.raises(jz.JzError):
        jz.jz_bn_relu_fwd(rows, C, X, f(), f(), 1e-5, True, torch.empty_like(X), f(), f(), small)      # workspace too small
    ws = torch.empty(jz.jz_bn_workspace_bytes(rows, C), dtype=torch.uint8, device=dev)
    with pytest.raises(jz.JzError):
        jz.jz_bn_relu_fwd(rows, C, X, f(), f(), 1e-5, True, X, f(), f(), ws)                             # output aliases input
    with pytest.raises(jz.JzError):
        jz.jz_bn_relu_fwd(rows, C, X, f(), f(), -1.0, True, torch.empty_like(X), f(), f(), ws)          # negative eps


@pytest.mark.parametrize("rows,C,two", [(2 * 14 * 14, 64, True), (5 * 7 * 7, 2048, True), (4099, 256, False), (3 * 9 * 9, 96, True), (1, 8, False)])
def test_block_end_backward_equals_relu_gradient_then_batch_norm_backward(jz, rows, C, two):
    """jz_bn_bwd_block_end against (a) the two separate calls, bit for bit, and (b) the oracle's composition."""
    import jzt
    import oracle
    x, gamma, beta, dya = _inputs((9, rows, C), rows, C)
    rng = inputs.rng_for(31, rows, C)
    dyb = inputs.normal_f16(rng, (rows, C), std=4.0) if two else None
    out = np.maximum(inputs.normal_f16(rng, (rows, C)), np.float16(0))           # the block's output: about half zeros
    dev = jzt.DEV
    X, G, B, OUT, DA = jzt.to_dev(x), jzt.to_dev(gamma), jzt.to_dev(beta), jzt.to_dev(out), jzt.to_dev(dya)
    DB = jzt.to_dev(dyb) if two else None
    Y = torch.empty_like(X)
    mean = torch.empty(C, dtype=torch.float32, device=dev); invstd = torch.empty_like(mean)
    ws = torch.empty(max(jz.jz_bn_workspace_bytes(rows, C), 16), dtype=torch.uint8, device=dev)
    jz.jz_bn_relu_fwd(rows, C, X, G, B, 1e-5, False, Y, mean, invstd, ws)
    res = []
    for fused in (True, False):
        g = torch.full_like(X, float("nan")); dx = torch.full_like(X, float("nan"))
        dg = torch.empty(C, dtype=torch.float16, device=dev); db = torch.empty_like(dg)
        ws.fill_(0xCD)
        if fused:
            jz.jz_bn_bwd_block_end(rows, C, X, OUT, DA, DB, G, mean, invstd, g, dx, dg, db, ws)
        else:
            if two:
                jz.jz_relu_bwd_sum(OUT.reshape(-1), DA.reshape(-1), DB.reshape(-1), g.reshape(-1)) if rows * C % 8 == 0 else None
            else:
                jz.jz_relu_bwd(OUT.reshape(-1), DA.reshape(-1), g.reshape(-1))
            jz.jz_bn_relu_bwd(rows, C, X, None, g, G, mean, invstd, False, dx, dg, db, ws)
        torch.cuda.synchronize()
        res.append([t.cpu().numpy() for t in (g, dx, dg, db)])
    for a, b in zip(*res):
        assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    g16 = oracle.relu_bwd(out, oracle.add_fwd(dya, dyb, relu=False)[1] if two else dya)
    assert np.array_equal(res[0][0].view(np.uint16), g16.view(np.uint16))
    dx64, _, dg64, db64, _, _ = oracle.bn_relu_bwd(x, None, g16, gamma, mean.cpu().numpy(), invstd.cpu().numpy(), relu=False)
    assert jzt.rel_l2(res[0][1], dx64) <= 1e-3
    floor = np.sqrt(rows) * 1e-2
    for got, ref in ((res[0][2], dg64), (res[0][3], db64)):
        err = np.abs(got.astype(np.float64) - ref)
        assert np.all(err <= 2e-3 * np.maximum(np.abs(ref), floor))
