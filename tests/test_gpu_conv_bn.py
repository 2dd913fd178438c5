"""GPU parity of jz_conv2d_bn_relu_fwd (forward convolution with the batch-norm statistics taken in its epilogue): the
convolution output must be the bits jz_conv2d_fwd writes, and mean / invstd / y must meet the bars of the stand-alone
batch normalization against the oracle evaluated on that convolution output.  Every kernel variant is forced through
the planner's tuning hook, and a shape that cannot take the sums in the epilogue (split reduction) must give the same
results through the fallback pass."""
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


def run_case(jz, N, H, C, K, R, stride, pad, relu=True, key=0, eps=1e-5, residual=False, variant=None, splits=1):
    import jzt
    if variant is not None:
        with jzt.forced_variant(jz.conv_desc(N, H, H, C, K, R, R, stride, pad), *variant, splits=splits, ops=(jz.JZ_FWD,)):
            return run_case(jz, N, H, C, K, R, stride, pad, relu, key, eps, residual)
    rng = inputs.rng_for(41, key, N, H, C, K, R)
    x = inputs.normal_f16(rng, (N * H * H * C,))
    w = inputs.normal_f16(rng, (K * R * R * C,), std=(2.0 / (R * R * C)) ** 0.5)
    gamma = (1.0 + 0.3 * rng.standard_normal(K, dtype=np.float32)).astype(np.float32)
    beta = (0.2 * rng.standard_normal(K, dtype=np.float32)).astype(np.float32)
    d = jz.conv_desc(N, H, H, C, K, R, R, stride, pad)
    rows = N * d.P * d.Q
    X, W, G, B = jzt.to_dev(x), jzt.to_dev(w), jzt.to_dev(gamma), jzt.to_dev(beta)
    c_ref = torch.empty(rows * K, dtype=torch.float16, device="cuda")
    ws0 = torch.zeros(max(jz.jz_conv2d_workspace_bytes(jz.JZ_FWD, d), 16), dtype=torch.uint8, device="cuda")
    jz.bind_conv2d(jz.JZ_FWD, d, X, W, c_ref, ws0)()
    c = torch.full((rows * K,), float("nan"), dtype=torch.float16, device="cuda")
    y = torch.full((rows * K,), float("nan"), dtype=torch.float16, device="cuda")
    mean = torch.empty(K, dtype=torch.float32, device="cuda"); invstd = torch.empty_like(mean)
    ws = torch.full((max(jz.jz_conv2d_bn_relu_fwd_workspace_bytes(d), 16),), 0xCD, dtype=torch.uint8, device="cuda")
    res = inputs.normal_f16(rng, (rows * K,), std=1.5) if residual else None
    jz.jz_conv2d_bn_relu_fwd(d, X, W, G, B, eps, relu, c, y, mean, invstd, ws, jzt.to_dev(res) if residual else None)
    torch.cuda.synchronize()
    c_np = c.cpu().numpy()
    assert np.array_equal(c_np.view(np.uint16), c_ref.cpu().numpy().view(np.uint16)), "convolution output differs from jz_conv2d_fwd"
    if residual:
        y64, _, m64, i64 = oracle.bn_add_relu_fwd(c_np.reshape(rows, K), res.reshape(rows, K), gamma, beta, eps, relu=relu)
    else:
        y64, _, m64, i64 = oracle.bn_relu_fwd(c_np.reshape(rows, K), gamma, beta, eps, relu=relu)
    mg, ig = mean.cpu().numpy(), invstd.cpu().numpy()
    assert np.all(np.abs(mg - m64) <= 1e-5 * (np.abs(m64) + 1.0 / i64)), float(np.max(np.abs(mg - m64)))
    assert np.all(np.abs(ig - i64) <= 1e-4 * i64), float(np.max(np.abs(ig - i64) / i64))
    assert jzt.rel_l2(y.cpu().numpy(), y64) <= 1e-3
    return jz.lib()


SHAPES = [
    (2, 14, 64, 64, 3, 1, 1),        # 392 rows: ragged against every tile height
    (3, 9, 32, 96, 3, 1, 1),         # K not a multiple of 64
    (2, 28, 256, 128, 1, 1, 0),      # 1x1
    (2, 28, 256, 512, 1, 2, 0),      # strided 1x1 (projection shortcut)
    (2, 32, 3, 64, 7, 2, 3),         # the stem's small-channel path
    (1, 7, 512, 2048, 1, 1, 0),      # widest layer, 49 rows
    (4, 56, 64, 64, 3, 1, 1),        # several row tiles
]


@pytest.mark.parametrize("N,H,C,K,R,stride,pad", SHAPES)
@pytest.mark.parametrize("relu", [True, False])
def test_fused_statistics_against_the_oracle(jz, N, H, C, K, R, stride, pad, relu):
    run_case(jz, N, H, C, K, R, stride, pad, relu=relu)
    run_case(jz, N, H, C, K, R, stride, pad, relu=relu, residual=True, key=7)


@pytest.mark.parametrize("variant", [(128, 128, 32, 4, 4), (128, 64, 32, 4, 4), (64, 128, 32, 4, 3), (64, 64, 64, 4, 4),
                                     (128, 128, 64, 4, 4), (256, 128, 32, 8, 4), (256, 128, 64, 8, 3), (256, 256, 32, 8, 4),
                                     (128, 128, 32, 8, 3), (128, 128, 64, 8, 4)], ids=lambda v: "x".join(str(i) for i in v))
def test_every_kernel_variant_leaves_the_same_statistics(jz, variant):
    run_case(jz, 5, 24, 64, 192, 3, 1, 1, key=1, variant=variant)       # 2880 rows: 22.5 tiles of 128, 11.25 of 256
    run_case(jz, 2, 10, 128, 72, 1, 1, 0, key=2, variant=variant)       # 200 rows, 72 channels: ragged both ways


def test_split_reduction_falls_back_to_the_statistics_pass(jz):
    run_case(jz, 2, 14, 256, 64, 3, 1, 1, key=3, variant=(128, 64, 32, 4, 4), splits=3)


def test_argument_errors(jz):
    import ctypes
    L = jz.lib()
    d = jz.conv_desc(2, 8, 8, 16, 32, 3, 3, 1, 1)
    n = ctypes.c_size_t(0)
    assert L.jz_conv2d_bn_relu_fwd_workspace_bytes(ctypes.byref(d), None) == jz.JZ_ERR_NULL
    assert L.jz_conv2d_bn_relu_fwd_workspace_bytes(ctypes.byref(d), ctypes.byref(n)) == jz.JZ_OK and n.value > 0
    h, f = torch.float16, torch.float32
    x = torch.zeros(2 * 8 * 8 * 16, dtype=h, device="cuda"); w = torch.zeros(32 * 9 * 16, dtype=h, device="cuda")
    c = torch.zeros(2 * 8 * 8 * 32, dtype=h, device="cuda"); y = torch.zeros_like(c)
    g = torch.ones(32, dtype=f, device="cuda"); b = torch.zeros(32, dtype=f, device="cuda")
    m = torch.zeros(32, dtype=f, device="cuda"); s = torch.zeros(32, dtype=f, device="cuda")
    ws = torch.zeros(n.value, dtype=torch.uint8, device="cuda")
    ptr = lambda t: t.data_ptr()

    def call(**o):
        a = dict(x=ptr(x), w=ptr(w), g=ptr(g), b=ptr(b), eps=1e-5, c=ptr(c), y=ptr(y), m=ptr(m), s=ptr(s), ws=ptr(ws), n=n.value)
        a.update(o)
        return L.jz_conv2d_bn_relu_fwd(ctypes.byref(d), a["x"], a["w"], a["g"], a["b"], a["eps"], a.get("r"), 1, a["c"], a["y"], a["m"], a["s"],
                                       a["ws"], a["n"], None)

    assert call(x=None) == jz.JZ_ERR_NULL and call(y=None) == jz.JZ_ERR_NULL and call(m=None) == jz.JZ_ERR_NULL
    assert call(eps=-1.0) == jz.JZ_ERR_SHAPE
    assert call(n=n.value - 1) == jz.JZ_ERR_WORKSPACE and call(ws=None) == jz.JZ_ERR_WORKSPACE
    assert call(y=ptr(c)) == jz.JZ_ERR_ALIAS and call(s=ptr(m)) == jz.JZ_ERR_ALIAS and call(y=ptr(x)) == jz.JZ_ERR_ALIAS
    assert call(y=ptr(y) + 2) == jz.JZ_ERR_ALIGN
    assert call(r=ptr(y)) == jz.JZ_ERR_ALIAS and call(r=ptr(c)) == jz.JZ_ERR_ALIAS and call(r=ptr(x) + 2) == jz.JZ_ERR_ALIGN
    assert call() == jz.JZ_OK
    torch.cuda.synchronize()
    dbad = jz.conv_desc(2, 8, 8, 16, 36, 3, 3, 1, 1)      # 36 channels: not a multiple of 8 for the normalization
    assert L.jz_conv2d_bn_relu_fwd_workspace_bytes(ctypes.byref(dbad), ctypes.byref(n)) == jz.JZ_ERR_UNSUPPORTED
