"""GPU parity of the single-precision variant (jz_conv2d_*_f32, jz_gemm_fc_f32: FP32 storage, FP32 accumulate; the
FP32 side of the comparison in Section 5.4 / Table 9) against the fp64 oracle on the same float32 inputs.

Bars (the design doc derives them): relative L2 error <= 1e-5 (an FP32 sum of K products carries about sqrt(K) * 2^-24
relative to the root-sum-square of its terms; the longest reduction here has 800 k terms), and for EVERY element
|got - ref| <= 2^-23 |ref| + 8 * 2^-24 * sum|terms|  (one output rounding, accumulation in any order)."""
import numpy as np
import pytest
import torch

import oracle
from paper_1807_11205_amd import inputs, shapes

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def jz():
    from paper_1807_11205_amd import api
    api.lib()
    assert torch.cuda.is_available()
    return api


def check_f32(got, ref64, mag64, what, tol=1e-5):
    got = np.asarray(got, np.float64).ravel()
    ref = np.asarray(ref64, np.float64).ravel()
    mag = np.asarray(mag64, np.float64).ravel()
    assert got.shape == ref.shape and not np.any(np.isnan(got)), what + ": unwritten or NaN output"
    den = np.linalg.norm(ref)
    err = float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got))
    assert err <= tol, "%s: relative L2 error %.3e > %.1e" % (what, err, tol)
    bound = 2.0 ** -23 * np.abs(ref) + 8 * 2.0 ** -24 * mag + 1e-37
    worst = float(np.max(np.abs(got - ref) / bound))
    assert worst <= 1.0, "%s: an element is %.2f x its bound" % (what, worst)
    return err, worst


def run_f32(jz, op, d, a, b, out_shape):
    ta, tb = torch.from_numpy(np.ascontiguousarray(a)).to(DEV), torch.from_numpy(np.ascontiguousarray(b)).to(DEV)
    out = torch.full(out_shape, float("nan"), dtype=torch.float32, device=DEV)      # poison: every element must be written
    n = jz.jz_conv2d_f32_workspace_bytes(op, d)
    ws = torch.empty(max(n, 16), dtype=torch.uint8, device=DEV) if n else None
    jz.jz_conv2d_f32(op, d, ta, tb, out, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def all_ops(jz, N, H, W, C, K, R, S, st, pad, key, ops=(0, 1, 2), full=True, n_sample=32768):
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    od = oracle.conv_desc(N, H, W, C, K, R, S, st, (ph, pw))
    d = jz.conv_desc(N, H, W, C, K, R, S, st, (ph, pw))
    rng = inputs.rng_for(91, key, N, H, C, K, R)
    x = rng.standard_normal((N, H, W, C), dtype=np.float32)
    w = (rng.standard_normal((K, R, S, C), dtype=np.float32) * np.float32((2.0 / (R * S * C)) ** 0.5))
    dy = rng.standard_normal((N, od.P, od.Q, K), dtype=np.float32) * np.float32(4.0)
    res = {}
    cases = {jz.JZ_FWD: ("fwd", x, w, (N, od.P, od.Q, K), oracle.conv_fwd, oracle.conv_fwd_at),
             jz.JZ_BWD_DATA: ("bwd_data", dy, w, (N, H, W, C), oracle.conv_bwd_data, oracle.conv_bwd_data_at),
             jz.JZ_BWD_WEIGHT: ("bwd_weight", x, dy, (K, R, S, C), oracle.conv_bwd_weight, oracle.conv_bwd_weight_at)}
    for op in ops:
        name, a, b, shp, fn, fn_at = cases[op]
        got = run_f32(jz, op, d, a, b, shp)
        if full or op == jz.JZ_BWD_WEIGHT:      # the weight gradient is always compared as a whole tensor
            res[name] = check_f32(got, fn(od, a, b), fn(od, np.abs(a), np.abs(b)), name)
        else:
            idx = np.unique(np.concatenate([rng.integers(0, got.size, size=min(n_sample, got.size)),
                                            np.arange(min(got.size, 4096)), np.arange(max(0, got.size - 4096), got.size)]))
            res[name] = check_f32(got.ravel()[idx], fn_at(od, a, b, idx), fn_at(od, np.abs(a), np.abs(b), idx), name)
    return res


SHAPES = [
    # N, H, W, C, K, R, S, stride, pad
    (2, 13, 13, 64, 192, 3, 3, 1, 1),      # several tiles, ragged in m and n
    (3, 14, 14, 128, 64, 1, 1, 1, 0),      # 1x1
    (2, 14, 14, 256, 128, 1, 1, 2, 0),     # strided 1x1: backward-data leaves the odd pixels zero
    (1, 15, 15, 64, 64, 5, 5, 1, 2),       # 5x5 pad 2
    (2, 9, 9, 64, 128, 3, 3, 2, 1),        # 3x3 stride 2
    (4, 7, 7, 192, 320, 3, 3, 1, 1),       # deep reduction, few pixels
    (2, 6, 10, 128, 200, 3, 1, 1, (1, 0)), # R != S, H != W
    (2, 9, 7, 3, 5, 3, 2, (2, 1), (1, 0)), # element-wise fetches: 3 channels, 5 filters
    (1, 23, 23, 3, 64, 7, 7, 2, 3),        # stem-like
    (3, 6, 6, 24, 40, 3, 3, 1, 1),         # multiples of 4 only
    (1, 1, 1, 5, 7, 1, 1, 1, 0),           # one dot product per output
    (5, 4, 4, 130, 129, 1, 1, 1, 0),       # just over one tile, odd sizes
    (16, 20, 20, 8, 8, 3, 3, 1, 1),        # long reduction into a small weight gradient: split across workgroups
]


@pytest.mark.parametrize("cfg", SHAPES)
def test_small_shapes_whole_tensors(jz, cfg):
    res = all_ops(jz, *cfg, key=SHAPES.index(cfg))
    print(res)


def test_split_reduction_is_planned_and_deterministic(jz):
    d = jz.conv_desc(16, 20, 20, 8, 8, 3, 3, 1, 1)
    assert jz.jz_conv2d_f32_workspace_bytes(jz.JZ_BWD_WEIGHT, d) > 0       # the reduction over 6400 pixels is split
    rng = inputs.rng_for(92)
    x = rng.standard_normal((16, 20, 20, 8), dtype=np.float32)
    dy = rng.standard_normal((16, 20, 20, 8), dtype=np.float32)
    a = run_f32(jz, jz.JZ_BWD_WEIGHT, d, x, dy, (8, 3, 3, 8))
    b = run_f32(jz, jz.JZ_BWD_WEIGHT, d, x, dy, (8, 3, 3, 8))
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


@pytest.mark.parametrize("B,I,O", [(64, 2048, 1000), (5, 24, 7), (130, 192, 72)])
def test_fully_connected_modes(jz, B, I, O):
    rng = inputs.rng_for(93, B, I, O)
    x = rng.standard_normal((B, I), dtype=np.float32)
    w = rng.standard_normal((O, I), dtype=np.float32) * np.float32((2.0 / I) ** 0.5)
    dy = rng.standard_normal((B, O), dtype=np.float32)
    for mode, a, b, shp, fn in ((jz.JZ_FWD, x, w, (B, O), oracle.fc_fwd), (jz.JZ_BWD_DATA, dy, w, (B, I), oracle.fc_bwd_data),
                                (jz.JZ_BWD_WEIGHT, dy, x, (O, I), oracle.fc_bwd_weight)):
        ta, tb = torch.from_numpy(a).to(DEV), torch.from_numpy(b).to(DEV)
        out = torch.full(shp, float("nan"), dtype=torch.float32, device=DEV)
        n = jz.jz_gemm_fc_f32_workspace_bytes(mode, B, I, O)
        ws = torch.empty(max(n, 16), dtype=torch.uint8, device=DEV) if n else None
        jz.jz_gemm_fc_f32(mode, B, I, O, ta, tb, out, ws)
        torch.cuda.synchronize()
        check_f32(out.cpu().numpy(), fn(B, I, O, a, b), fn(B, I, O, np.abs(a), np.abs(b)), "fc mode %d" % mode)


FULL_SIZE = [cs for cs in shapes.resnet50_convs() if cs.name in ("stem", "s2b1b", "s2b1c", "s3b1a", "s4b1b", "s5b1c")]


@pytest.mark.parametrize("cs", FULL_SIZE, ids=lambda c: c.name)
def test_resnet50_layers_batch64_sampled(jz, cs):
    # the sizes the FP32 bench line runs: outputs sampled (random, plus the first and last 4096 elements), the weight
    # gradient as a whole tensor
    res = all_ops(jz, 64, cs.H, cs.H, cs.C, cs.K, cs.R, cs.R, cs.stride, cs.pad, key=100 + cs.H + cs.C,
                  ops=(0, 2) if cs.first else (0, 1, 2), full=False)
    print(cs.name, res)


def test_argument_errors(jz):
    import ctypes
    L = jz.lib()
    d = jz.conv_desc(2, 8, 8, 64, 64, 3, 3, 1, 1)
    A = 0x10000000
    n = ctypes.c_size_t(0)
    assert L.jz_conv2d_fwd_f32(ctypes.byref(d), None, A, A + (1 << 24), None, 0, None) == jz.JZ_ERR_NULL
    assert L.jz_conv2d_fwd_f32(ctypes.byref(d), A + 4, A + (1 << 24), A + (1 << 25), None, 0, None) == jz.JZ_ERR_ALIGN
    assert L.jz_conv2d_fwd_f32(ctypes.byref(d), A, A + (1 << 24), A, None, 0, None) == jz.JZ_ERR_ALIAS
    bad = jz.conv_desc(2, 8, 8, 64, 64, 3, 3, 1, 3)
    assert L.jz_conv2d_f32_workspace_bytes(0, ctypes.byref(bad), ctypes.byref(n)) == jz.JZ_ERR_SHAPE
    big = jz.conv_desc(64, 56, 56, 64, 64, 3, 3, 1, 1)
    assert L.jz_conv2d_f32_workspace_bytes(2, ctypes.byref(big), ctypes.byref(n)) == jz.JZ_OK and n.value > 0
    assert L.jz_conv2d_bwd_weight_f32(ctypes.byref(big), A, A + (1 << 28), A + (1 << 29), None, 0, None) == jz.JZ_ERR_WORKSPACE
    assert L.jz_gemm_fc_f32(7, 4, 4, 4, A, A + 4096, A + 8192, None, 0, None) == jz.JZ_ERR_UNSUPPORTED
