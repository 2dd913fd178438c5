"""The chained ResNet-50 step (paper_1807_11205_amd/resnet50.py: forward, loss gradient, backward, LARS update with the
dynamic loss scale, every tensor produced by the launch before it) against the oracle, launch by launch: each launch's
outputs are compared with the oracle evaluated on the inputs that launch actually read on the GPU, with the bar of
that operation's own parity test.  Small image and batch so that the fp64 oracle finishes in seconds; the network,
its 161 parameter tensors and the order of the launches are those of the full-size step."""
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


def np16(t):
    return t.detach().cpu().numpy()


def rel_l2(got, ref):
    got, ref = np.asarray(got, np.float64).ravel(), np.asarray(ref, np.float64).ravel()
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got))


def one_step_of_fp16(got16, ref64, ref16, what):
    g, r16 = got16.ravel(), np.asarray(ref16).ravel()
    diff = np.nonzero(g.view(np.uint16) != r16.view(np.uint16))[0]
    if diff.size:
        up, dn = np.nextafter(r16[diff], np.float16(np.inf)), np.nextafter(r16[diff], np.float16(-np.inf))
        assert np.all((g[diff] == up) | (g[diff] == dn)), what
    assert diff.size <= 0.01 * g.size + 2, what
    assert rel_l2(g, ref64) <= 1e-3, what


def check_op(op, counts, check_conv=True):
    import jzt
    k, p = op.kind, op.params
    what = "%s %s" % (k, op.name)
    ins = [None if t is None else np16(t) for t in op.ins]
    outs = [np16(t) for t in op.outs]
    counts[k] = counts.get(k, 0) + 1
    if k in ("conv_fwd", "conv_bwd_data", "conv_bwd_weight"):
        d = p["desc"]
        od = oracle.conv_desc(d.N, d.H, d.W, d.C, d.K, d.R, d.S, (d.stride_h, d.stride_w), (d.pad_h, d.pad_w))
        fn = {"conv_fwd": oracle.conv_fwd, "conv_bwd_data": oracle.conv_bwd_data, "conv_bwd_weight": oracle.conv_bwd_weight}[k]
        jzt.check_half_output(outs[0], fn(od, ins[0], ins[1]), tol=1e-3, what=what, mag64=fn(od, jzt.abs16(ins[0]), jzt.abs16(ins[1])))
    elif k == "conv_bn_fwd":
        d = p["desc"]
        od = oracle.conv_desc(d.N, d.H, d.W, d.C, d.K, d.R, d.S, (d.stride_h, d.stride_w), (d.pad_h, d.pad_w))
        jzt.check_half_output(outs[0], oracle.conv_fwd(od, ins[0], ins[1]), tol=1e-3, what=what,
                              mag64=oracle.conv_fwd(od, jzt.abs16(ins[0]), jzt.abs16(ins[1])))
        rows, C = p["rows"], p["C"]
        if ins[4] is None:
            y64, _, m64, i64 = oracle.bn_relu_fwd(outs[0].reshape(rows, C), ins[2], ins[3], p["eps"], relu=p["relu"])
        else:
            y64, _, m64, i64 = oracle.bn_add_relu_fwd(outs[0].reshape(rows, C), ins[4].reshape(rows, C), ins[2], ins[3], p["eps"], relu=p["relu"])
        assert np.all(np.abs(outs[2] - m64) <= 1e-5 * (np.abs(m64) + 1.0 / i64)), what
        assert np.all(np.abs(outs[3] - i64) <= 1e-4 * i64), what
        assert rel_l2(outs[1], y64) <= 1e-3, what
    elif k.startswith("fc_"):
        fn = {"fc_fwd": oracle.fc_fwd, "fc_bwd_data": oracle.fc_bwd_data, "fc_bwd_weight": oracle.fc_bwd_weight}[k]
        jzt.check_half_output(outs[0], fn(p["B"], p["I"], p["O"], ins[0], ins[1]), tol=1e-3, what=what,
                              mag64=fn(p["B"], p["I"], p["O"], jzt.abs16(ins[0]), jzt.abs16(ins[1])))
    elif k == "bn_fwd":
        rows, C = p["rows"], p["C"]
        y64, _, m64, i64 = oracle.bn_relu_fwd(ins[0].reshape(rows, C), ins[1], ins[2], p["eps"], relu=p["relu"])
        assert np.all(np.abs(outs[1] - m64) <= 1e-5 * (np.abs(m64) + 1.0 / i64)), what
        assert np.all(np.abs(outs[2] - i64) <= 1e-4 * i64), what
        assert rel_l2(outs[0], y64) <= 1e-3, what
    elif k == "bn_bwd":
        rows, C = p["rows"], p["C"]
        x, dy = ins[0].reshape(rows, C), ins[2].reshape(rows, C)
        y = ins[1].reshape(rows, C) if p["relu"] else None
        dx64, _, dg64, db64, _, _ = oracle.bn_relu_bwd(x, y, dy, ins[3], ins[4], ins[5], relu=p["relu"])
        assert rel_l2(outs[0], dx64) <= 1e-3, what
        # gamma / beta gradients: FP32 sums rounded to FP16; the floor is the rounding noise of a sum of `rows` terms
        rms = float(np.sqrt(np.mean(dy.astype(np.float64) ** 2)))
        floor = np.sqrt(rows) * rms * 2.5e-3 + 2.0 ** -24
        for got, ref in ((outs[1], dg64), (outs[2], db64)):
            err = np.abs(got.astype(np.float64) - ref)
            assert np.all(err <= 2e-3 * np.maximum(np.abs(ref), floor)), what
    elif k == "conv_bwd_data_bn_bwd":
        # the convolution's gradient like any backward-data launch, then the batch-norm backward on that gradient as it
        # was written (ins: dy, w, bn x, bn y, gamma, mean, invstd; outs: dz, dx, dgamma, dbeta)
        d = p["desc"]
        od = oracle.conv_desc(d.N, d.H, d.W, d.C, d.K, d.R, d.S, (d.stride_h, d.stride_w), (d.pad_h, d.pad_w))
        if check_conv:      # (at full size the caller samples this output instead)
            jzt.check_half_output(outs[0], oracle.conv_bwd_data(od, ins[0], ins[1]), tol=1e-3, what=what,
                                  mag64=oracle.conv_bwd_data(od, jzt.abs16(ins[0]), jzt.abs16(ins[1])))
        rows, C = p["rows"], p["C"]
        x, y, dz = ins[2].reshape(rows, C), ins[3].reshape(rows, C), outs[0].reshape(rows, C)
        dx64, _, dg64, db64, _, _ = oracle.bn_relu_bwd(x, y, dz, ins[4], ins[5], ins[6], relu=True)
        assert rel_l2(outs[1], dx64) <= 1e-3, what
        rms = float(np.sqrt(np.mean(dz.astype(np.float64) ** 2)))
        floor = np.sqrt(rows) * rms * 2.5e-3 + 2.0 ** -24
        for got, ref in ((outs[2], dg64), (outs[3], db64)):
            err = np.abs(got.astype(np.float64) - ref)
            assert np.all(err <= 2e-3 * np.maximum(np.abs(ref), floor)), what
        counts["conv_bwd_data"] = counts.get("conv_bwd_data", 0) + 1
        counts["bn_bwd"] = counts.get("bn_bwd", 0) + 1
    elif k == "conv_bwd_data_block_end":
        # ins: dy, w, dyb, bn x, y_out, gamma, mean, invstd; outs: g, dx, dgamma, dbeta.  The convolution's own result is
        # never stored, so g is compared with what the oracle makes of the oracle's convolution: equal bits except where the
        # convolution's FP16 rounding fell the other way (at most one FP16 step of the sum, on a small share of the elements)
        d = p["desc"]
        od = oracle.conv_desc(d.N, d.H, d.W, d.C, d.K, d.R, d.S, (d.stride_h, d.stride_w), (d.pad_h, d.pad_w))
        rows, C = p["rows"], p["C"]
        if check_conv:
            dxa64 = oracle.conv_bwd_data(od, ins[0], ins[1])
            dxa16 = np.asarray(dxa64, np.float64).astype(np.float16).ravel()
            tot = oracle.add_fwd(dxa16, ins[2], relu=False)[1] if ins[2] is not None else dxa16
            g_ref = oracle.relu_bwd(ins[4], tot)
            mask = ins[4].ravel() > 0
            assert np.array_equal(outs[0].ravel()[~mask].view(np.uint16), np.zeros(int((~mask).sum()), np.uint16)), what
            exact64 = (np.asarray(dxa64, np.float64).ravel() + (ins[2].astype(np.float64).ravel() if ins[2] is not None else 0.0)) * mask
            jzt.check_half_output(outs[0], exact64, tol=1e-3, what=what)
            assert np.mean(outs[0].ravel().view(np.uint16) != g_ref.ravel().view(np.uint16)) <= 0.02, what
        x, g = ins[3].reshape(rows, C), outs[0].reshape(rows, C)
        dx64, _, dg64, db64, _, _ = oracle.bn_relu_bwd(x, None, g, ins[5], ins[6], ins[7], relu=False)
        assert rel_l2(outs[1], dx64) <= 1e-3, what
        rms = float(np.sqrt(np.mean(g.astype(np.float64) ** 2)))
        floor = np.sqrt(rows) * rms * 2.5e-3 + 2.0 ** -24
        for got, ref in ((outs[2], dg64), (outs[3], db64)):
            err = np.abs(got.astype(np.float64) - ref)
            assert np.all(err <= 2e-3 * np.maximum(np.abs(ref), floor)), what
        counts["conv_bwd_data"] = counts.get("conv_bwd_data", 0) + 1
        counts["bn_bwd_block_end"] = counts.get("bn_bwd_block_end", 0) + 1
    elif k == "add_fwd":
        assert np.array_equal(outs[0].view(np.uint16), oracle.add_fwd(ins[0], ins[1], relu=p["relu"])[1].view(np.uint16)), what
    elif k == "relu_bwd":
        assert np.array_equal(outs[0].view(np.uint16), oracle.relu_bwd(ins[0], ins[1]).view(np.uint16)), what
    elif k == "bn_bwd_block_end":
        rows, C = p["rows"], p["C"]
        dy = oracle.add_fwd(ins[2], ins[3], relu=False)[1] if ins[3] is not None else ins[2]
        g16 = oracle.relu_bwd(ins[1], dy)
        assert np.array_equal(outs[0].view(np.uint16), g16.view(np.uint16)), what
        x, g = ins[0].reshape(rows, C), g16.reshape(rows, C)
        dx64, _, dg64, db64, _, _ = oracle.bn_relu_bwd(x, None, g, ins[4], ins[5], ins[6], relu=False)
        assert rel_l2(outs[1], dx64) <= 1e-3, what
        rms = float(np.sqrt(np.mean(g.astype(np.float64) ** 2)))
        floor = np.sqrt(rows) * rms * 2.5e-3 + 2.0 ** -24
        for got, ref in ((outs[2], dg64), (outs[3], db64)):
            err = np.abs(got.astype(np.float64) - ref)
            assert np.all(err <= 2e-3 * np.maximum(np.abs(ref), floor)), what
    elif k == "relu_bwd_sum":
        want = oracle.relu_bwd(ins[0], oracle.add_fwd(ins[1], ins[2], relu=False)[1])
        assert np.array_equal(outs[0].view(np.uint16), want.view(np.uint16)), what
    elif k == "maxpool_fwd":
        x = ins[0].reshape(p["N"], p["H"], p["W"], p["C"])
        ry, rarg = oracle.maxpool_fwd(x, p["window"], p["stride"], p["pad"])
        assert np.array_equal(outs[0].view(np.uint16), ry.ravel().view(np.uint16)), what
        a = outs[1].reshape(ry.shape).astype(np.int64)
        P = ry.shape[1]
        pp, qq = np.arange(P)[None, :, None, None], np.arange(P)[None, None, :, None]
        flat = (pp * p["stride"] - p["pad"] + a // p["window"]) * p["W"] + (qq * p["stride"] - p["pad"] + a % p["window"])
        assert np.array_equal(flat, rarg), what
    elif k == "maxpool_bwd":
        x = ins[0].reshape(p["N"], p["H"], p["W"], p["C"])
        P = oracle.pool_out(p["H"], p["window"], p["stride"], p["pad"])
        r64, r16 = oracle.maxpool_bwd(x, ins[1].reshape(p["N"], P, P, p["C"]), p["window"], p["stride"], p["pad"])
        one_step_of_fp16(outs[0], r64, r16, what)
    elif k == "avgpool_fwd":
        r64, r16 = oracle.avgpool_fwd(ins[0].reshape(p["N"], p["HW"], 1, p["C"]))
        one_step_of_fp16(outs[0], r64, r16, what)
    elif k == "avgpool_bwd":
        r64, r16 = oracle.avgpool_bwd(ins[0].reshape(p["N"], p["C"]), p["HW"], 1)
        one_step_of_fp16(outs[0], r64, r16, what)
    elif k == "bias_add":
        assert np.array_equal(outs[0].view(np.uint16), oracle.bias_add(ins[0].reshape(p["rows"], p["C"]), ins[1])[1].ravel().view(np.uint16)), what
    elif k == "bias_grad":
        r64, r16 = oracle.bias_grad(ins[0].reshape(p["rows"], p["C"]))
        one_step_of_fp16(outs[0], r64, r16, what)
    elif k == "softmax_xent":
        S = float(ins[2][:1].view(np.float32)[0])
        l64, d64, _ = oracle.softmax_xent(ins[0].reshape(p["rows"], p["classes"]), ins[1], S)
        assert np.allclose(outs[1], l64, rtol=2e-6, atol=2e-5), what
        err = np.abs(outs[0].astype(np.float64).reshape(d64.shape) - d64)
        assert np.all(err <= 2.0 ** -10 * np.abs(d64) + 2.0 ** -25), what
    elif k in ("lars_begin", "lars_grad_sumsq"):
        pass        # what they leave in the optimiser's workspace is checked as a whole, behind the backward pass
    else:
        raise AssertionError("no check for " + k)


@pytest.mark.parametrize("fused,block_end,presummed,bwd_stats", [(True, True, True, True), (True, True, True, False), (True, True, False, True),
                                                                 (True, False, True, True), (False, False, True, False)])
def test_every_launch_of_a_chained_step_against_the_oracle(jz, fused, block_end, presummed, bwd_stats):
    import jzt
    from paper_1807_11205_amd import resnet50
    net = resnet50.ResNet50Chain(batch=4, image=64, initial_loss_scale=256.0, policy=dict(growth_interval=1), fused=fused,
                                 block_end=block_end, presummed=presummed, bwd_stats=bwd_stats)
    assert len(net.fwd_ops) == (53 if fused else 53 * 2 + 16) + 1 + 1 + 3 + (1 if presummed else 0) and net.trace[-1].kind == "lars_dyn"
    assert (net.fwd_ops[0].kind == "lars_begin" and net.bwd_ops[-1].kind == "lars_grad_sumsq") == presummed
    for op in net.trace[:-1]:
        op.call()
    torch.cuda.synchronize()
    counts = {}
    for op in net.trace[:-1]:
        check_op(op, counts)
    assert counts.get("conv_bn_fwd", 0) + counts.get("conv_fwd", 0) == 53 and counts.get("conv_fwd", 0) == counts.get("bn_fwd", 0)
    assert counts["conv_bwd_weight"] == 53 and counts["conv_bwd_data"] == 52
    assert counts.get("conv_bwd_data_bn_bwd", 0) == (32 if bwd_stats else 0)    # the a and b layers of the 16 blocks
    assert counts.get("conv_bwd_data_block_end", 0) == (15 if bwd_stats and block_end else 0)   # every block end but the last
    assert counts["bn_bwd"] + counts.get("bn_bwd_block_end", 0) == 53 and counts["add_fwd"] == (1 if fused else 32)
    assert counts.get("relu_bwd", 0) + counts.get("relu_bwd_sum", 0) + counts.get("bn_bwd_block_end", 0) == 16
    assert counts.get("bn_bwd_block_end", 0) == (16 if block_end else 0) and counts.get("relu_bwd_sum", 0) == (15 if fused and not block_end else 0)
    # every parameter tensor received a gradient from this step (none was left at its initial zero)
    g = np16(net.grad)
    for i, (name, _, _, _) in enumerate(net.tensors):
        assert np.any(g[net.offsets[i]:net.offsets[i + 1]] != 0), name
    if presummed:
        # every tensor's sink holds exactly the sum of squares of its gradient: the filters' from the weight-gradient GEMMs
        # (split reduction, unsplit + separate pass, small-channel stem alike), the rest from the pass behind the backward
        for i, (name, _, _, _) in enumerate(net.tensors):
            units, bad = jzt.sink_units(net.ps, net.lars_ws, i)
            assert bad == 0 and units == jzt.exact_units(g[net.offsets[i]:net.offsets[i + 1]]), name
    # the update: LARS against the oracle with the scale the step ran with, then the controller
    before = inputs.ParamSet(names=[t[0] for t in net.tensors], offsets=np.asarray(net.offsets, np.int64),
                             flags=np.asarray(net.flags, np.uint8), master_w=np16(net.master), momentum=np16(net.momentum),
                             grad16=g, weight16=np16(net.w16), loss_scale=256.0)
    net.update()
    torch.cuda.synchronize()
    got = (np16(net.master), np16(net.momentum), np16(net.w16), int(net.found_inf.item()))
    out = jzt.check_lars_against_oracle(before, got, loss_scale=256.0, plain_rtol=1e-6, plain_floor=0.1, **net.hp)
    assert out["flag"] == 0
    assert jz.loss_scale_state(net.ls_state) == oracle.loss_scale_step(256.0, 0, 0, growth_interval=1)


def test_the_chained_step_learns_a_fixed_batch(jz):
    """Twenty steps on one fixed batch of eight images: the initial loss scale is too large, so the first steps overflow
    and are skipped while the controller (on the device throughout) halves the scale; from then on no step is skipped
    and the network memorises the batch: the mean loss falls from about log(1000) to well under 1."""
    from paper_1807_11205_amd import resnet50
    net = resnet50.ResNet50Chain(batch=8, image=64, initial_loss_scale=65536.0, hparams=dict(lr=2.0),
                                 policy=dict(growth_interval=1000, max_scale=2.0 ** 24))
    losses, flags = [], []
    for _ in range(20):
        net.step()
        losses.append(net.mean_loss())
        flags.append(int(net.found_inf.item()))
    print("losses", ["%.3f" % v for v in losses], "flags", flags, "scale", jz.loss_scale_state(net.ls_state), flush=True)
    assert abs(losses[0] - np.log(1000.0)) < 1.5
    assert all(np.isfinite(losses)) and all(f in (0, 1) for f in flags) and sum(flags[-10:]) == 0
    assert 1 <= sum(flags) <= 10 and losses[sum(flags)] == losses[0]        # skipped steps change nothing
    assert losses[-1] < 1.0 and min(losses) == min(losses[-6:])


def test_side_stream_schedule_gives_the_same_bits(jz):
    """The weight-gradient GEMMs on a side stream: same launches, same order of every reduction, so three steps leave
    exactly the same parameters as on one stream."""
    from paper_1807_11205_amd import resnet50
    out = []
    for use_side, proj in ((False, False), (True, False), (True, True)):
        net = resnet50.ResNet50Chain(batch=4, image=64, initial_loss_scale=512.0, hparams=dict(lr=1.0), proj_side=proj)
        side = torch.cuda.Stream() if use_side else None
        for _ in range(3):
            net.step(side=side)
        torch.cuda.synchronize()
        out.append((np16(net.master), np16(net.momentum), np16(net.w16), np16(net.grad), net.mean_loss()))
    for other in out[1:]:
        for a, b in zip(out[0][:4], other[:4]):
            assert np.array_equal(a.view(np.uint32 if a.dtype == np.float32 else np.uint16), b.view(np.uint32 if b.dtype == np.float32 else np.uint16))
        assert out[0][4] == other[4]


def test_full_size_chained_step_on_sampled_outputs(jz):
    """The step bench.py --workload chain times (N = 64, 224x224, fused calls): the GPU computes whole tensors, the oracle
    (a) a seeded sample of convolution outputs one by one, on the operands that launch read, (b) whole tensors of the
    cheap layers, exactly, and (c) the statistics, gamma / beta gradients and outputs of three batch normalizations."""
    import jzt
    from paper_1807_11205_amd import resnet50
    net = resnet50.ResNet50Chain(batch=64, image=224, initial_loss_scale=1024.0)
    net.forward(); net.backward()
    torch.cuda.synchronize()
    assert np.isfinite(net.mean_loss())
    rng = np.random.default_rng(5)
    ops = {(o.kind, o.name): o for o in net.trace}
    odesc = lambda d: oracle.conv_desc(d.N, d.H, d.W, d.C, d.K, d.R, d.S, (d.stride_h, d.stride_w), (d.pad_h, d.pad_w))

    # (a) sampled convolution outputs: forward (inside the fused call), backward-data, backward-weight
    for name in ("stem", "s2b1c", "s2b1p", "s3b1a", "s4b2a", "s4b3b", "s5b3c"):
        op = ops[("conv_bn_fwd", name)]
        d = op.params["desc"]
        x, w, c = np16(op.ins[0]), np16(op.ins[1]), np16(op.outs[0])
        idx = rng.integers(0, c.size, size=8192)
        jzt.check_half_output(c[idx], oracle.conv_fwd_at(odesc(d), x, w, idx), 1e-3, "fwd " + name,
                              mag64=oracle.conv_fwd_at(odesc(d), jzt.abs16(x), jzt.abs16(w), idx))
        ow = ops[("conv_bwd_weight", name)]          # the whole weight gradient
        xw, dyw = np16(ow.ins[0]), np16(ow.ins[1])
        jzt.check_half_output(np16(ow.outs[0]), oracle.conv_bwd_weight(odesc(d), xw, dyw), 1e-3, "bwd_weight " + name,
                              mag64=oracle.conv_bwd_weight(odesc(d), jzt.abs16(xw), jzt.abs16(dyw)))
        if name != "stem":
            od_ = ops.get(("conv_bwd_data", name)) or next(o for o in net.trace if o.kind in ("conv_bwd_data_bn_bwd", "conv_bwd_data_block_end")
                                                           and o.name.startswith(name + " + "))
            dx = np16(od_.outs[0])
            idx = rng.integers(0, dx.size, size=8192)
            gy, ww = np16(od_.ins[0]), np16(od_.ins[1])
            ref = oracle.conv_bwd_data_at(odesc(d), gy, ww, idx)
            if od_.kind == "conv_bwd_data_block_end":
                # the convolution's result exists only inside g = relu-masked (result + the shortcut's contribution): two
                # roundings to FP16, so the norm-wise bar only
                ref = (ref + np16(od_.ins[2])[idx].astype(np.float64)) * (np16(od_.ins[4])[idx] > 0)
                jzt.check_half_output(dx[idx], ref, 1e-3, "bwd_data + block end " + name)
            else:
                jzt.check_half_output(dx[idx], ref, 1e-3, "bwd_data " + name,
                                      mag64=oracle.conv_bwd_data_at(odesc(d), jzt.abs16(gy), jzt.abs16(ww), idx))

    # (b) whole tensors of the cheap layers (per-image layers on the first images, where the oracle loops in Python)
    counts = {}
    fused_end = next(o for o in net.trace if o.kind == "conv_bwd_data_block_end" and o.name.endswith(" + s4b6c.bn"))
    check_op(fused_end, counts, check_conv=False)       # (g of such calls is sampled under (a): s3b1a through the in-place pass, s4b2a from the epilogue)
    for key in (("bn_bwd_block_end", "s5b3c.bn"), ("add_fwd", "s2b1.dx"), ("avgpool_fwd", "pool5"), ("avgpool_bwd", "pool5"),
                ("bias_add", "fc.b"), ("bias_grad", "fc.b"), ("softmax_xent", "loss"), ("fc_fwd", "fc"), ("fc_bwd_data", "fc"), ("fc_bwd_weight", "fc")):
        check_op(ops[key], counts)
    mp, mb = ops[("maxpool_fwd", "pool1")], ops[("maxpool_bwd", "pool1")]
    p = mp.params
    n2, per_in, per_out = 2, p["H"] * p["W"] * p["C"], 56 * 56 * p["C"]
    x = np16(mp.ins[0])[:n2 * per_in].reshape(n2, p["H"], p["W"], p["C"])
    ry, rarg = oracle.maxpool_fwd(x, 3, 2, 1)
    assert np.array_equal(np16(mp.outs[0])[:n2 * per_out].view(np.uint16), ry.ravel().view(np.uint16))
    r64, r16 = oracle.maxpool_bwd(x, np16(mb.ins[1])[:n2 * per_out].reshape(n2, 56, 56, p["C"]), 3, 2, 1)
    one_step_of_fp16(np16(mb.outs[0])[:n2 * per_in], r64, r16, "maxpool_bwd")

    # (c) batch normalization on whole tensors: a plain one, one with the residual, and their backward passes
    for name in ("s2b1a", "s4b1a", "s5b3c"):
        op = ops[("conv_bn_fwd", name)]
        rows, C = op.params["rows"], op.params["C"]
        c = np16(op.outs[0]).reshape(rows, C)
        if op.ins[4] is None:
            y64, _, m64, i64 = oracle.bn_relu_fwd(c, np16(op.ins[2]), np16(op.ins[3]), op.params["eps"], relu=op.params["relu"])
        else:
            y64, _, m64, i64 = oracle.bn_add_relu_fwd(c, np16(op.ins[4]).reshape(rows, C), np16(op.ins[2]), np16(op.ins[3]), op.params["eps"],
                                                      relu=op.params["relu"])
        assert np.all(np.abs(np16(op.outs[2]) - m64) <= 1e-5 * (np.abs(m64) + 1.0 / i64)), name
        assert np.all(np.abs(np16(op.outs[3]) - i64) <= 1e-4 * i64), name
        assert rel_l2(np16(op.outs[1]), y64) <= 1e-3, name
        del y64
        if name.endswith("c"):
            check_op(ops[("bn_bwd_block_end", name + ".bn")], counts)
        else:       # the a layers' backward is the second half of the call that holds the b layers' backward-data
            check_op(next(o for o in net.trace if o.kind == "conv_bwd_data_bn_bwd" and o.name.endswith(" + " + name + ".bn")), counts,
                     check_conv=False)


def test_a_new_batch_changes_the_step_and_the_old_one_reproduces_it(jz):
    from paper_1807_11205_amd import resnet50
    net = resnet50.ResNet50Chain(batch=4, image=64, initial_loss_scale=128.0)
    x0, l0 = net.x.clone(), net.labels.clone()
    net.forward(); net.backward(); torch.cuda.synchronize()
    g0, loss0 = np16(net.grad).copy(), net.mean_loss()
    gen = torch.Generator().manual_seed(9)
    net.set_batch(torch.randn(x0.numel(), generator=gen).to(torch.float16).cuda(), torch.randint(0, 1000, (4,), generator=gen).cuda())
    net.forward(); net.backward(); torch.cuda.synchronize()
    assert net.mean_loss() != loss0 and not np.array_equal(np16(net.grad).view(np.uint16), g0.view(np.uint16))
    net.set_batch(x0, l0)
    net.forward(); net.backward(); torch.cuda.synchronize()
    assert net.mean_loss() == loss0 and np.array_equal(np16(net.grad).view(np.uint16), g0.view(np.uint16))
    with pytest.raises(ValueError):
        net.set_batch(x0[:-8], l0)


def test_whole_step_replays_from_a_hip_graph_including_the_loss_scale_decisions(jz):
    """With the loss scale and its controller on the device nothing in a step depends on the host, so the step can be
    captured once and replayed: every replay (overflowing steps that are skipped and halve the scale, then clean steps)
    leaves the same bits as the eager step on a second network, with eager work and synchronisations in between."""
    from paper_1807_11205_amd import resnet50
    kw = dict(batch=4, image=64, initial_loss_scale=2.0 ** 18, hparams=dict(lr=1.0), policy=dict(growth_interval=3, max_scale=2.0 ** 24))
    net, ref = resnet50.ResNet50Chain(**kw), resnet50.ResNet50Chain(**kw)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        net.step(s)                      # first launches load the code objects: not inside a capture
        s.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            net.step(s)
        s.synchronize()
    ref.step()
    torch.cuda.synchronize()
    flags = []
    for k in range(10):
        g.replay()
        ref.step()
        torch.cuda.synchronize()
        flags.append(int(net.found_inf.item()))
        assert flags[-1] == int(ref.found_inf.item())
        assert jz.loss_scale_state(net.ls_state) == jz.loss_scale_state(ref.ls_state)
        for a, b in ((net.master, ref.master), (net.momentum, ref.momentum), (net.w16, ref.w16), (net.grad, ref.grad)):
            assert np.array_equal(np16(a).view(np.uint32 if a.dtype == torch.float32 else np.uint16),
                                  np16(b).view(np.uint32 if b.dtype == torch.float32 else np.uint16)), "replay %d" % k
        assert net.mean_loss() == ref.mean_loss()
    assert 1 in flags and 0 in flags, flags    # the oversized scale overflowed at first, then steps went through
