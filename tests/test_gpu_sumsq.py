"""GPU tests of the gradient sum-of-squares sinks (the ||g_t|| of Eq. 1 taken where the gradient is produced) and of the
one-launch update that consumes them: jz_conv2d_bwd_weight_sumsq / jz_gemm_fc_bwd_weight_sumsq, jz_lars_begin_step,
jz_lars_sumsq_sink, jz_lars_grad_sumsq, jz_lars_mp_update_presummed, all through the C ABI.

What is compared with what: the weight gradient of a *_sumsq call with the plain call's (bit for bit) and with the fp64
oracle; a sink's content with the sum of squares of the fp16 gradient it belongs to, added up in Python integers (the
sinks are exact, so the comparison is for equality); the update with oracle.lars_mp_update on the gradient
buffer the GPU produced."""
import ctypes
import re
from fractions import Fraction

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


def new_sink(jz):
    # 8192 bytes, 128-byte aligned: a slice of a larger allocation that starts on such a boundary
    raw = torch.zeros(1024 + 16, dtype=torch.int64, device="cuda")
    skip = (-raw.data_ptr() // 8) % 16
    sums = raw[skip:skip + 1024]
    assert sums.data_ptr() % 128 == 0
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    return jz.sumsq_sink(sums, flag), sums, flag, raw


# (N, H, C, K, R, stride, pad): a split reduction, a small-channel layer (padded copy + split), a 1x1 that is reduced in
# one piece when forced to, a shape only the element-wise kernel takes
CONV_CASES = [
    (16, 28, 128, 128, 3, 1, 1),
    (8, 14, 256, 512, 1, 1, 0),
    (4, 64, 3, 64, 7, 2, 3),
    (8, 20, 3, 5, 3, 1, 1),
]


@pytest.mark.parametrize("case", CONV_CASES, ids=lambda c: "x".join(map(str, c)))
@pytest.mark.parametrize("one_piece", [False, True], ids=["planned", "unsplit"])
def test_weight_gradient_and_its_sum_of_squares(jz, case, one_piece):
    import jzt
    N, H, C, K, R, stride, pad = case
    c = inputs.conv_case((9, 1, *case), N, H, H, C, K, R, R, stride, pad, loss_scale=64.0, dy_std=0.05)
    d, od = jzt.desc_of(c), jzt.odesc_of(c)
    x, dy = jzt.to_dev(c.x), jzt.to_dev(c.dy)
    try:
        if one_piece:
            # the planner's own variant with the reduction in one piece: the gradient leaves the GEMM kernel as fp16 and the
            # sum of squares is taken by the separate pass
            plan = jz.jz_conv2d_describe_plan(jz.JZ_BWD_WEIGHT, d)
            if "vector tile" not in plan:
                pytest.skip("element-wise plan has no tunable variant: " + plan)
            m = re.search(r"tile (\d+)x(\d+)x(\d+), (\d+) wavefronts, ring (\d+)", plan)
            jz.jz_conv2d_tune_set(jz.JZ_BWD_WEIGHT, d, *[int(v) for v in m.groups()], 1)
            assert ", 1 splits" in jz.jz_conv2d_describe_plan(jz.JZ_BWD_WEIGHT, d)
        ws = jzt._ws_tensor(jz.jz_conv2d_workspace_bytes(jz.JZ_BWD_WEIGHT, d))
        plain = torch.full((K, R, R, C), float("nan"), dtype=torch.float16, device="cuda")
        jz.jz_conv2d_bwd_weight(d, x, dy, plain, ws)
        sink, sums, flag, _keep = new_sink(jz)
        dw = torch.full((K, R, R, C), float("nan"), dtype=torch.float16, device="cuda")
        jz.jz_conv2d_bwd_weight_sumsq(d, x, dy, dw, sink, ws)
        torch.cuda.synchronize()
        g = dw.cpu().numpy()
        assert np.array_equal(jzt.bits(g), jzt.bits(plain.cpu().numpy())), "the gradient must be the plain call's, bit for bit"
        ref = oracle.conv_bwd_weight(od, c.x, c.dy)
        mag = oracle.conv_bwd_weight(od, jzt.abs16(c.x), jzt.abs16(c.dy))
        jzt.check_half_output(g, ref, what="dw", mag64=mag)
        once = jz.sumsq_sink_units(sums)
        assert int(flag.item()) == 0
        assert once == jzt.exact_units(g), "sink != exact sum of squares of the gradient written"
        assert abs(float(Fraction(once, 2 ** 48)) - float(np.sum(g.astype(np.float64) ** 2))) <= 1e-12 * float(Fraction(once, 2 ** 48))
        # a second call adds to the sink
        jz.jz_conv2d_bwd_weight_sumsq(d, x, dy, dw, sink, ws)
        torch.cuda.synchronize()
        assert jz.sumsq_sink_units(sums) == 2 * once, "same contributions in another arrival order must give the same digits"
    finally:
        jz.jz_conv2d_tune_clear()


@pytest.mark.parametrize("bad", [np.inf, np.nan])
def test_non_finite_gradient_raises_the_sink_flag(jz, bad):
    import jzt
    c = inputs.conv_case((9, 2), 8, 14, 14, 64, 64, 3, 3, 1, 1, loss_scale=8.0, dy_std=0.1)
    c.dy[3, 5, 7, 11] = np.float16(bad)
    d = jzt.desc_of(c)
    ws = jzt._ws_tensor(jz.jz_conv2d_workspace_bytes(jz.JZ_BWD_WEIGHT, d))
    sink, sums, flag, _keep = new_sink(jz)
    dw = torch.zeros((64, 3, 3, 64), dtype=torch.float16, device="cuda")
    jz.jz_conv2d_bwd_weight_sumsq(d, jzt.to_dev(c.x), jzt.to_dev(c.dy), dw, sink, ws)
    torch.cuda.synchronize()
    g = dw.cpu().numpy().astype(np.float64)
    assert not np.all(np.isfinite(g)) and int(flag.item()) == 1


def test_fully_connected_weight_gradient(jz):
    import jzt
    B, I, O = 64, 2048, 1000
    f = inputs.fc_case((9, 3), B, I, O, loss_scale=32.0)
    dy, x = jzt.to_dev(f.dy), jzt.to_dev(f.x)
    ws = jzt._ws_tensor(jz.jz_gemm_fc_workspace_bytes(jz.JZ_BWD_WEIGHT, B, I, O))
    plain = torch.zeros((O, I), dtype=torch.float16, device="cuda")
    jz.jz_gemm_fc(jz.JZ_BWD_WEIGHT, B, I, O, dy, x, plain, ws)
    sink, sums, flag, _keep = new_sink(jz)
    dw = torch.zeros((O, I), dtype=torch.float16, device="cuda")
    jz.jz_gemm_fc_bwd_weight_sumsq(B, I, O, dy, x, dw, sink, ws)
    torch.cuda.synchronize()
    g = dw.cpu().numpy()
    assert np.array_equal(jzt.bits(g), jzt.bits(plain.cpu().numpy()))
    jzt.check_half_output(g, oracle.fc_bwd_weight(B, I, O, f.dy, f.x), what="fc dw",
                          mag64=oracle.fc_bwd_weight(B, I, O, jzt.abs16(f.dy), jzt.abs16(f.x)))
    assert jz.sumsq_sink_units(sums) == jzt.exact_units(g)
    assert int(flag.item()) == 0


def test_grad_sumsq_fills_the_workspace_sinks(jz):
    import jzt
    sizes = [5000, 64, 0, 300000, 4096, 7]
    ps = inputs.random_param_set((9, 4), sizes, loss_scale=256.0, grad_std=2e-3)
    ps.grad16[5000 + 17] = np.float16(np.inf)      # tensor 1
    r = jzt.LarsRun(ps, path="presummed")
    jz.jz_lars_begin_step(r.ps, r.ws)
    jz.jz_lars_grad_sumsq(r.ps, 0, 2, r.ws)          # tensors in two calls, each tensor once
    jz.jz_lars_grad_sumsq(r.ps, 2, 4, r.ws)
    torch.cuda.synchronize()
    off = ps.offsets
    for t, n in enumerate(sizes):
        sink = jz.jz_lars_sumsq_sink(r.ps, r.ws, t)
        base = sink.sums - r.ws.data_ptr()
        assert base % 128 == 0
        sums = r.ws[base:base + jz.JZ_SUMSQ_SINK_BYTES].view(torch.int64)
        fl = int(r.ws[sink.nonfinite - r.ws.data_ptr():sink.nonfinite - r.ws.data_ptr() + 4].view(torch.int32).item())
        g = ps.grad16[off[t]:off[t + 1]]
        assert fl == (1 if t == 1 else 0)
        if t != 1:
            assert jz.sumsq_sink_units(sums) == jzt.exact_units(g)
    # begin_step clears them again
    jz.jz_lars_begin_step(r.ps, r.ws)
    torch.cuda.synchronize()
    for t in range(len(sizes)):
        sink = jz.jz_lars_sumsq_sink(r.ps, r.ws, t)
        base = sink.sums - r.ws.data_ptr()
        assert int(r.ws[base:base + jz.JZ_SUMSQ_SINK_BYTES].view(torch.int64).abs().sum().item()) == 0


def test_update_from_sinks_filled_by_the_producing_kernels(jz):
    """Three convolution layers write their weight gradients straight into the fused gradient buffer and their sums of
    squares into the workspace sinks; batch-norm style tensors in between go through jz_lars_grad_sumsq; then ONE launch
    updates everything.  Checked against the oracle update on the gradient buffer the GPU produced, twice in a row (the second
    step runs on carried sums of squares of the weights), and run to run."""
    import jzt
    layers = [(16, 28, 128, 128, 3, 1, 1), (8, 14, 256, 512, 1, 1, 0), (4, 64, 3, 64, 7, 2, 3)]
    cases = [inputs.conv_case((9, 5, i), N, H, H, C, K, R, R, st, pd, loss_scale=128.0, dy_std=0.02) for i, (N, H, C, K, R, st, pd) in enumerate(layers)]
    sizes, flags = [], []
    for c in cases:
        sizes += [c.K * c.R * c.S * c.C, c.K, c.K]      # filter, gamma, beta
        flags += [3, 2, 2]
    ps = inputs.random_param_set((9, 6), sizes, loss_scale=128.0, grad_std=1e-3, flags=flags, momentum_std=1e-3)

    def one_run():
        r = jzt.LarsRun(ps, path="presummed")
        out = []
        descs = [jzt.desc_of(c) for c in cases]
        xs, dys = [jzt.to_dev(c.x) for c in cases], [jzt.to_dev(c.dy) for c in cases]
        wss = [jzt._ws_tensor(jz.jz_conv2d_workspace_bytes(jz.JZ_BWD_WEIGHT, d)) for d in descs]
        hp = jz.lars_hparams(inputs.HPARAMS["lr"], inputs.HPARAMS["momentum"], inputs.HPARAMS["weight_decay"], inputs.HPARAMS["trust_coef"], 128.0)
        for step in range(2):
            jz.jz_lars_begin_step(r.ps, r.ws)
            for i, c in enumerate(cases):
                t = 3 * i
                lo, hi = int(ps.offsets[t]), int(ps.offsets[t + 1])
                dw = r.g[lo:hi].view(c.K, c.R, c.S, c.C)
                jz.jz_conv2d_bwd_weight_sumsq(descs[i], xs[i], dys[i], dw, jz.jz_lars_sumsq_sink(r.ps, r.ws, t), wss[i])
                jz.jz_lars_grad_sumsq(r.ps, t + 1, 2, r.ws)
            gbuf = r.g.cpu().numpy().copy()
            before = (r.w.cpu().numpy().copy(), r.v.cpu().numpy().copy(), r.w16.cpu().numpy().copy())
            jz.jz_lars_mp_update_presummed(r.ps, hp, r.flag, r.ws)
            torch.cuda.synchronize()
            got = (r.w.cpu().numpy(), r.v.cpu().numpy(), r.w16.cpu().numpy(), int(r.flag.item()))
            host = inputs.ParamSet(names=ps.names, offsets=ps.offsets, flags=ps.flags, master_w=before[0], momentum=before[1],
                                   grad16=gbuf, weight16=before[2], loss_scale=128.0)
            res = jzt.check_lars_against_oracle(host, got, loss_scale=128.0)
            assert res["flag"] == 0
            out.append(tuple(a.copy() for a in got[:3]))
        return out

    a, b = one_run(), one_run()
    for sa, sb in zip(a, b):
        for x, y in zip(sa, sb):
            assert np.array_equal(x.view(np.uint8), y.view(np.uint8)), "not bit-identical from run to run"


def test_both_update_paths_can_share_a_workspace(jz):
    import jzt
    ps = inputs.random_param_set((9, 7), [70000, 64, 9000], loss_scale=512.0, flags=[3, 2, 1], momentum_std=1e-3)
    r = jzt.LarsRun(ps, path="three_launches")
    for step, path in enumerate(["three_launches", "presummed", "presummed", "three_launches", "presummed"]):
        g = inputs.normal_f16(inputs.rng_for(9, 7, step), (ps.P,), std=1e-3 * 512.0)
        if step == 2:
            g[777] = np.float16(np.nan)         # a skipped presummed step in the middle
        ps.grad16 = g
        r.g.copy_(torch.from_numpy(g))
        r.path = path
        got = r.step()
        res = jzt.check_lars_against_oracle(ps, got)
        assert res["flag"] == (1 if step == 2 else 0)
        ps.master_w, ps.momentum, ps.weight16 = got[0].copy(), got[1].copy(), got[2].copy()


def test_argument_errors(jz):
    import jzt
    L, c = jz.lib(), ctypes.byref
    ps = inputs.random_param_set((9, 8), [4096, 64])
    r = jzt.LarsRun(ps, path="presummed")
    hp = jz.lars_hparams(0.1, 0.9, 5e-5, 0.001, 1024.0)
    wp, wn, fp = r.ws.data_ptr(), r.ws.numel(), r.flag.data_ptr()
    # the one-launch update needs jz_lars_begin_step first, once per update, with the same loss-scale state
    assert L.jz_lars_mp_update_presummed(c(r.ps.c), c(hp), fp, wp, wn, None) == jz.JZ_ERR_NOT_PREPARED
    jz.jz_lars_begin_step(r.ps, r.ws)
    jz.jz_lars_grad_sumsq(r.ps, 0, 2, r.ws)
    assert L.jz_lars_mp_update_presummed(c(r.ps.c), c(hp), fp, wp, wn, None) == jz.JZ_OK
    assert L.jz_lars_mp_update_presummed(c(r.ps.c), c(hp), fp, wp, wn, None) == jz.JZ_ERR_NOT_PREPARED
    state = torch.zeros(2, dtype=torch.int32, device="cuda")
    jz.jz_loss_scale_init(state, 64.0)
    pol = jz.loss_scale_policy()
    jz.jz_lars_begin_step(r.ps, r.ws)             # begun without a device-resident scale ...
    assert L.jz_lars_mp_update_presummed_dyn(c(r.ps.c), c(hp), c(pol), state.data_ptr(), fp, wp, wn, None) == jz.JZ_ERR_NOT_PREPARED
    # a workspace that was never prepared, tensor ranges, sinks
    other = torch.zeros(wn, dtype=torch.uint8, device="cuda")
    assert L.jz_lars_begin_step(c(r.ps.c), None, other.data_ptr(), wn, None) == jz.JZ_ERR_NOT_PREPARED
    assert L.jz_lars_begin_step(c(r.ps.c), None, wp, 64, None) == jz.JZ_ERR_WORKSPACE
    assert L.jz_lars_grad_sumsq(c(r.ps.c), 1, 2, wp, wn, None) == jz.JZ_ERR_SHAPE
    assert L.jz_lars_grad_sumsq(c(r.ps.c), -1, 1, wp, wn, None) == jz.JZ_ERR_SHAPE
    sk = jz.jz_sumsq_sink()
    assert L.jz_lars_sumsq_sink(c(r.ps.c), wp, wn, 2, c(sk)) == jz.JZ_ERR_SHAPE
    assert L.jz_lars_sumsq_sink(c(r.ps.c), wp, wn, 0, None) == jz.JZ_ERR_NULL
    d = jz.conv_desc(4, 8, 8, 16, 16, 3, 3, 1, 1)
    x = torch.zeros(4 * 8 * 8 * 16, dtype=torch.float16, device="cuda")
    dw = torch.zeros(16 * 3 * 3 * 16, dtype=torch.float16, device="cuda")
    ws = jzt._ws_tensor(max(jz.jz_conv2d_workspace_bytes(jz.JZ_BWD_WEIGHT, d), 16))
    good, sums, flag, _keep = new_sink(jz)

    def conv(sink):
        return L.jz_conv2d_bwd_weight_sumsq(c(d), x.data_ptr(), x.data_ptr(), dw.data_ptr(), ws.data_ptr(), ws.numel(),
                                            c(sink) if sink is not None else None, None)

    assert conv(None) == jz.JZ_ERR_NULL
    assert conv(jz.jz_sumsq_sink(None, flag.data_ptr())) == jz.JZ_ERR_NULL
    assert conv(jz.jz_sumsq_sink(sums.data_ptr() + 8, flag.data_ptr())) == jz.JZ_ERR_ALIGN
    assert conv(jz.jz_sumsq_sink(dw.data_ptr() + ((-dw.data_ptr()) % 128), flag.data_ptr())) == jz.JZ_ERR_ALIAS
    assert conv(good) == jz.JZ_OK
    torch.cuda.synchronize()
