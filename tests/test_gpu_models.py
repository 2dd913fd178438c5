"""GPU parity at the paper's model shapes (Table 3: AlexNet and ResNet-50), in the launch configuration the benchmark
times: whole tensors on the GPU, the oracle on the full tensor where that takes seconds and on a seeded sample of
output elements (each by its plain definition) where it would take minutes."""
import numpy as np
import pytest
import torch

from paper_1807_11205_amd import inputs, shapes

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def jz():
    from paper_1807_11205_amd import api
    api.lib()
    assert torch.cuda.is_available()
    return api


def distinct(convs):
    seen, out = set(), []
    for c in convs:
        key = (c.H, c.C, c.K, c.R, c.stride, c.pad)
        if key not in seen:
            seen.add(key)
            out.append(c)
    return out


BOTTLENECK = [shapes.ConvShape("a", 56, 256, 64, 1, 1, 0), shapes.ConvShape("b", 56, 64, 64, 3, 1, 1),
              shapes.ConvShape("c", 56, 64, 256, 1, 1, 0)]


@pytest.mark.parametrize("cs", BOTTLENECK, ids=lambda c: c.name)
def test_stage2_bottleneck_full_tensor_literal_loss_scale(jz, cs):
    # N = 32, 56x56, dy ~ N(0,1)*1024: most of the weight gradient overflows fp16, which is what the oracle's fp16
    # rounding says too; forward and backward-data stay finite
    import jzt
    c = inputs.conv_case_for(cs, 32, (2, ord(cs.name)), loss_scale=1024.0)
    res = jzt.conv_all_ops_full(c)
    print(cs.name, res)
    assert res["bwd_weight"]["n_inf"] > 0 and res["fwd"]["n_inf"] == 0 and res["bwd_data"]["n_inf"] == 0


def test_stage2_bottleneck_weight_gradient_after_back_off(jz):
    # halving S until the flag clears reaches S = 32 for this block: the weight gradients are finite and feed LARS
    import jzt
    import oracle
    grads, weights = [], []
    for cs in BOTTLENECK:
        c = inputs.conv_case_for(cs, 32, (2, ord(cs.name)), loss_scale=32.0)
        d = jzt.desc_of(c)
        dw = jzt.run_conv(jz.JZ_BWD_WEIGHT, d, c.x, c.dy, (c.K, c.R, c.S, c.C))
        ref = oracle.conv_bwd_weight(jzt.odesc_of(c), c.x, c.dy)
        r = jzt.check_half_output(dw, ref, what=cs.name)
        assert r["n_inf"] == 0
        grads.append(dw)
        weights.append(c.w32)
    ps = inputs.param_set_from_tensors(weights, grads, [3, 3, 3], 32.0)
    assert ps.P == 69632
    out = jzt.check_lars_against_oracle(ps, jzt.LarsRun(ps).step(), plain_rtol=1e-6)
    assert out["flag"] == 0


@pytest.mark.parametrize("cs", distinct(shapes.resnet50_convs()), ids=lambda c: "%s_%dx%d_%d_%d_%dx%d_s%d" % (c.name, c.H, c.H, c.C, c.K, c.R, c.R, c.stride))
def test_resnet50_layers_batch64_sampled(jz, cs):
    import jzt
    c = inputs.conv_case_for(cs, 64, (4, cs.H, cs.C, cs.K, cs.R, cs.stride), loss_scale=1.0)
    res = jzt.conv_all_ops_sampled(c, seed=cs.H * 1000 + cs.C + cs.K, skip_bwd_data=cs.first)
    print(cs.name, {k: "%.2e / %.2f of the element bound / %d compared" % (v["rel_l2"], v["worst_elem"], v["n"]) for k, v in res.items()})
    assert res["bwd_weight"]["n"] == cs.weight_count()     # the whole weight gradient, not a sample


V15_ONLY = [c for c in distinct(shapes.resnet50_convs("v1.5"))
            if (c.H, c.C, c.K, c.R, c.stride) not in {(v.H, v.C, v.K, v.R, v.stride) for v in shapes.resnet50_convs()}]


@pytest.mark.parametrize("cs", V15_ONLY, ids=lambda c: "%s_%dx%d_%d_%d_%dx%d_s%d" % (c.name, c.H, c.H, c.C, c.K, c.R, c.R, c.stride))
def test_resnet50_v15_layers_batch64_sampled(jz, cs):
    """The six shapes only the v1.5 placement of the stride has (stride 2 on the 3x3 of a stage's first block, whose
    backward-data runs as one launch per parity class; the 1x1 in front of it at unit stride), through their table entries."""
    import jzt
    c = inputs.conv_case_for(cs, 64, (5, cs.H, cs.C, cs.K, cs.R, cs.stride), loss_scale=1.0)
    res = jzt.conv_all_ops_sampled(c, seed=cs.H * 1000 + cs.C + cs.K + 15)
    assert res["bwd_weight"]["n"] == cs.weight_count()
    if cs.R > 1:
        assert "parity class" in jz.jz_conv2d_describe_plan(jz.JZ_BWD_DATA, jzt.desc_of(c))


OTHER_BATCH = [(n, cs) for n in (32, 128) for cs in distinct(shapes.resnet50_convs())
               if cs.name in ("s2b1b", "s2b1c", "s3b1a", "s3b1p", "s4b1b", "s5b1c", "s5b1b")]


@pytest.mark.parametrize("n,cs", OTHER_BATCH, ids=lambda v: str(v) if isinstance(v, int) else v.name)
def test_resnet50_layers_other_batch_sizes_sampled(jz, n, cs):
    """Batch 32 and 128 have planner tables of their own (keyed by GEMM shape): a sample of layer kinds through them."""
    import jzt
    c = inputs.conv_case_for(cs, n, (6, n, cs.H, cs.C, cs.K, cs.R, cs.stride), loss_scale=1.0)
    jzt.conv_all_ops_sampled(c, n_fwd=16384, n_bwd_data=16384, seed=n + cs.H * 1000 + cs.C + cs.K)


def test_resnet50_classifier_batch64(jz):
    import jzt
    import oracle
    B, I, O = 64, 2048, 1000
    c = inputs.fc_case((4, 9999), B, I, O, loss_scale=1024.0)
    r = jzt.fc_all_modes(B, I, O, c)["bwd_weight"]
    assert r["n_inf"] == 0     # std of dW is S*sqrt(64) = 8192: inside fp16


def test_resnet50_layer_with_literal_loss_scale_overflow_pattern(jz):
    # one deep layer at the literal S = 1024: about a quarter of dW overflows; the pattern must match the oracle's
    import jzt
    cs = shapes.ConvShape("s5b1c", 7, 512, 2048, 1, 1, 0)
    c = inputs.conv_case_for(cs, 64, (4, 7), loss_scale=1024.0)
    d, od = jzt.desc_of(c), jzt.odesc_of(c)
    import oracle
    dw = jzt.run_conv(jz.JZ_BWD_WEIGHT, d, c.x, c.dy, (c.K, c.R, c.S, c.C))
    r = jzt.check_half_output(dw, oracle.conv_bwd_weight(od, c.x, c.dy), what="dW at S=1024")
    print(r)
    assert 0.1 < r["n_inf"] / dw.size < 0.5


@pytest.mark.parametrize("cs", shapes.alexnet_convs(), ids=lambda c: c.name)
def test_alexnet_layers_batch128_sampled(jz, cs):
    import jzt
    c = inputs.conv_case_for(cs, 128, (3, cs.H, cs.C, cs.K), loss_scale=1.0)
    res = jzt.conv_all_ops_sampled(c, seed=cs.H + cs.C, skip_bwd_data=cs.first, n_fwd=32768, n_bwd_data=32768)
    print(cs.name, {k: "%.2e / %.2f of the element bound / %d compared" % (v["rel_l2"], v["worst_elem"], v["n"]) for k, v in res.items()})
    assert res["bwd_weight"]["n"] == cs.weight_count()


@pytest.mark.parametrize("fc", shapes.ALEXNET_FCS, ids=lambda f: f.name)
def test_alexnet_classifier_batch128(jz, fc):
    import jzt
    import oracle
    B, I, O = 128, fc.I, fc.O
    c = inputs.fc_case((3, I, O), B, I, O, loss_scale=1.0)
    rng = np.random.default_rng(I + O)
    y = jzt.run_fc(jz.JZ_FWD, B, I, O, c.x, c.w16, (B, O))
    dx = jzt.run_fc(jz.JZ_BWD_DATA, B, I, O, c.dy, c.w16, (B, I))
    dw = jzt.run_fc(jz.JZ_BWD_WEIGHT, B, I, O, c.dy, c.x, (O, I))
    od = oracle.conv_desc(B, 1, 1, I, O, 1, 1)      # the oracle's sampled routines take the 1x1-conv view of the same GEMM
    for name, out, fn, a, b in (("fwd", y, oracle.conv_fwd_at, c.x, c.w16), ("bwd_data", dx, oracle.conv_bwd_data_at, c.dy, c.w16),
                                ("bwd_weight", dw, oracle.conv_bwd_weight_at, c.x, c.dy)):
        assert not np.any(np.isnan(out))
        idx = rng.integers(0, out.size, size=min(out.size, 65536))
        jzt.check_half_output(out.ravel()[idx], fn(od, a, b, idx), what=fc.name + " " + name, mag64=fn(od, jzt.abs16(a), jzt.abs16(b), idx))
