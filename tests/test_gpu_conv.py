"""GPU parity of the convolution and fully connected entry points (through the C ABI) against the fp64 oracle.
Tolerance: relative L2 error <= 1e-3 (fp16 rounding of the result alone contributes about 2e-4)."""
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


def test_config0_layer_literal_loss_scale(jz):
    # 3x3, stride 1, pad 1, [2,14,14,16] -> 16 channels, dy ~ N(0,1) * 1024: the weight gradient overflows fp16 in a
    # few entries; the overflow pattern has to match the oracle's
    import jzt
    c = inputs.conv_case((0,), 2, 14, 14, 16, 16, 3, 3, 1, 1, loss_scale=1024.0)
    res = jzt.conv_all_ops_full(c)
    print(res)


def test_config0_layer_backed_off_loss_scale(jz):
    import jzt
    c = inputs.conv_case((0,), 2, 14, 14, 16, 16, 3, 3, 1, 1, loss_scale=256.0)
    res = jzt.conv_all_ops_full(c)
    assert res["bwd_weight"]["n_inf"] == 0
    print(res)


GENERIC = [
    # N, H, W, C, K, R, S, stride, pad   -- none of these meets the vector paths' channel multiples
    (2, 9, 7, 3, 5, 3, 2, (2, 1), (1, 0)),
    (1, 8, 11, 4, 2, 1, 3, (1, 2), (0, 2)),
    (2, 10, 9, 1, 3, 5, 4, (3, 2), (2, 3)),
    (1, 23, 23, 3, 64, 7, 7, 2, 3),          # stem-like: 3 input channels, 7x7 stride 2
    (2, 35, 35, 3, 96, 11, 11, 4, 0),        # AlexNet conv1-like
    (3, 6, 6, 24, 40, 3, 3, 1, 1),           # channels multiple of 8 but not of 64
    (1, 1, 1, 5, 7, 1, 1, 1, 0),             # a single dot product per output
    (5, 4, 4, 130, 129, 1, 1, 1, 0),         # just over one tile in n and k
    (8, 20, 20, 3, 5, 3, 3, 1, 1),           # long reduction (3200 pixels) into 5 x 27 weight gradients: the element-wise
                                             # kernel splits it, and the partial-sum slabs are not 16-byte multiples
]


@pytest.mark.parametrize("cfg", GENERIC)
def test_generic_shapes(jz, cfg):
    import jzt
    N, H, W, C, K, R, S, st, pad = cfg
    c = inputs.conv_case((10, abs(hash(cfg)) % 10000), N, H, W, C, K, R, S, 1, 0)
    # conv_case only knows symmetric stride/pad: build asymmetric descriptors by hand
    sh, sw = (st, st) if isinstance(st, int) else st
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    rng = inputs.rng_for(10, 1, abs(hash(cfg)) % 10000)
    import oracle
    od = oracle.conv_desc(N, H, W, C, K, R, S, (sh, sw), (ph, pw))
    d = jz.conv_desc(N, H, W, C, K, R, S, (sh, sw), (ph, pw))
    x = inputs.normal_f16(rng, (N, H, W, C))
    w = inputs.he_normal_f32(rng, (K, R, S, C), R * S * C).astype(np.float16)
    dy = inputs.normal_f16(rng, (N, od.P, od.Q, K), std=4.0)
    if cfg[0] == 8:
        assert " 1 splits" not in jz.jz_conv2d_describe_plan(jz.JZ_BWD_WEIGHT, d) and "element-wise" in jz.jz_conv2d_describe_plan(jz.JZ_BWD_WEIGHT, d)
    res = jzt.all_ops_against_the_oracle(d, od, x, w, dy)


VECTOR = [
    # N, H, W, C, K, R, S, stride, pad  -- channel counts that take the vector loaders; several tiles and ragged tails
    (2, 13, 13, 64, 192, 3, 3, 1, 1),      # M = 338 (2.6 tiles), N = 192 (1.5 tiles)
    (3, 14, 14, 128, 64, 1, 1, 1, 0),      # 1x1, 64 output channels (narrow tile)
    (2, 14, 14, 256, 128, 1, 1, 2, 0),     # 1x1 stride 2 (ResNet downsample): backward-data leaves odd pixels zero
    (1, 15, 15, 64, 64, 5, 5, 1, 2),       # 5x5 pad 2
    (2, 9, 9, 64, 128, 3, 3, 2, 1),        # 3x3 stride 2 (the v1.5 placement)
    (4, 7, 7, 192, 320, 3, 3, 1, 1),       # deep reduction, few pixels: split-K in fwd / bwd_data
    (1, 8, 8, 64, 8, 1, 1, 1, 0),          # K = 8: vector path of backward-weight with a tiny m
    (2, 6, 10, 128, 200, 3, 1, 1, (1, 0)), # R != S, H != W, K not a multiple of 64 (bwd_data falls back)
    (3, 10, 10, 40, 24, 1, 1, 1, 0),       # 1x1 with channel counts that are multiples of 8 only: ragged last k tile
    (2, 9, 9, 72, 40, 1, 1, 2, 0),         # the same with stride 2 (scatter epilogue in backward-data)
    (2, 5, 5, 1000, 136, 1, 1, 1, 0),      # long ragged reduction (31 full k tiles + 8 channels)
    (1, 12, 12, 32, 64, 7, 7, 1, 3),       # 49 taps: more than the 32-bit tap mask holds (per-load tap arithmetic)
    (2, 11, 11, 64, 64, 3, 3, 1, 0),       # no padding: backward-data reads outside dy on every border
    (2, 12, 12, 64, 96, 4, 4, 2, 1),       # even filter, stride 2
]


@pytest.mark.parametrize("cfg", VECTOR)
def test_vector_path_shapes(jz, cfg):
    import jzt
    import oracle
    N, H, W, C, K, R, S, st, pad = cfg
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    od = oracle.conv_desc(N, H, W, C, K, R, S, st, (ph, pw))
    d = jz.conv_desc(N, H, W, C, K, R, S, st, (ph, pw))
    rng = inputs.rng_for(11, abs(hash(cfg)) % 10000)
    x = inputs.normal_f16(rng, (N, H, W, C))
    w = inputs.he_normal_f32(rng, (K, R, S, C), R * S * C).astype(np.float16)
    dy = inputs.normal_f16(rng, (N, od.P, od.Q, K), std=8.0)
    res = jzt.all_ops_against_the_oracle(d, od, x, w, dy)
    print({k: (v["rel_l2"], v["worst_elem"]) for k, v in res.items()})


STRIDED = [
    # N, H, W, C, K, R, S, (stride_h, stride_w), (pad_h, pad_w): multi-tap strided layers, backward-data only
    (2, 14, 14, 64, 64, 3, 3, (2, 2), (1, 1)),     # the v1.5 placement: classes of 1, 2, 2 and 4 taps
    (2, 15, 13, 64, 96, 3, 3, (2, 2), (1, 1)),     # odd sizes: the classes' grids differ by one row / column
    (2, 14, 14, 64, 64, 3, 3, (2, 2), (0, 0)),     # no padding: the last row of the odd class meets no output pixel
    (1, 23, 23, 64, 64, 7, 7, (2, 2), (3, 3)),     # 49 taps, 16 / 12 / 12 / 9 per class
    (2, 12, 12, 64, 96, 4, 4, (2, 2), (1, 1)),     # even filter
    (2, 16, 16, 32, 64, 3, 3, (3, 3), (1, 1)),     # stride 3: nine single-tap classes
    (2, 17, 11, 64, 160, 5, 5, (3, 2), (2, 1)),    # different strides and pads along the two axes
    (2, 12, 12, 64, 64, 3, 3, (2, 1), (1, 1)),     # strided along h only
    (2, 12, 12, 64, 64, 3, 5, (1, 2), (1, 2)),     # strided along w only
    (2, 9, 9, 128, 96, 5, 3, (4, 2), (2, 1)),      # 8 classes
    (2, 9, 9, 64, 40, 3, 3, (2, 2), (1, 1)),       # 40 output channels: no 16-byte k tiles, the element-wise kernel
    (1, 13, 13, 64, 64, 2, 2, (3, 3), (0, 0)),     # filter smaller than the stride: some pixels meet no tap (per-load variant)
    (3, 5, 5, 64, 64, 3, 3, (2, 2), (1, 1)),       # tiny grids: classes of 3x3, 3x2, 2x3 and 2x2 pixels
]


@pytest.mark.parametrize("cfg", STRIDED, ids=lambda c: "x".join(str(v) for v in c).replace(" ", ""))
def test_strided_backward_data_parity_classes(jz, cfg):
    """Strided multi-tap backward-data runs as one unit-stride launch per parity class of the stride: every input pixel is
    written exactly once (the output is poisoned with NaN first) and meets the oracle element by element."""
    import jzt
    import oracle
    N, H, W, C, K, R, S, st, pad = cfg
    od = oracle.conv_desc(N, H, W, C, K, R, S, st, pad)
    d = jz.conv_desc(N, H, W, C, K, R, S, st, pad)
    plan = jz.jz_conv2d_describe_plan(jz.JZ_BWD_DATA, d)
    assert ("parity class" in plan) == (R >= st[0] and S >= st[1] and K % 32 == 0), plan
    rng = inputs.rng_for(14, abs(hash(cfg)) % 10000)
    w = inputs.he_normal_f32(rng, (K, R, S, C), R * S * C).astype(np.float16)
    dy = inputs.normal_f16(rng, (N, od.P, od.Q, K), std=8.0)
    x = np.zeros((N, H, W, C), np.float16)      # (not used by backward-data)
    jzt.all_ops_against_the_oracle(d, od, x, w, dy, ops=(jz.JZ_BWD_DATA,))
    # all-ones data: every input pixel's value is the number of (tap, output pixel) pairs it meets, exactly
    ones_w = np.ones((K, R, S, C), np.float16)
    ones_dy = np.ones((N, od.P, od.Q, K), np.float16)
    got = jzt.run_conv(jz.JZ_BWD_DATA, d, ones_dy, ones_w, (N, H, W, C)).astype(np.float64)
    want = np.asarray(oracle.conv_bwd_data(od, ones_dy, ones_w), np.float64).reshape(got.shape)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("variant", [(128, 128, 32, 4, 4), (64, 64, 32, 4, 3), (128, 64, 64, 4, 4), (256, 128, 32, 8, 4), (128, 128, 64, 8, 4),
                                     (256, 256, 32, 8, 4)], ids=lambda v: "x".join(str(i) for i in v))
def test_parity_class_launches_in_every_kernel_family(jz, variant):
    import jzt
    import oracle
    N, H, W, C, K, R, S, st, pad = 3, 30, 30, 64, 128, 3, 3, (2, 2), (1, 1)       # 675 pixels per class
    od = oracle.conv_desc(N, H, W, C, K, R, S, st, pad)
    d = jz.conv_desc(N, H, W, C, K, R, S, st, pad)
    rng = inputs.rng_for(15, *variant)
    w = inputs.he_normal_f32(rng, (K, R, S, C), R * S * C).astype(np.float16)
    dy = inputs.normal_f16(rng, (N, od.P, od.Q, K), std=8.0)
    with jzt.forced_variant(d, *variant, ops=(jz.JZ_BWD_DATA,)):
        jzt.all_ops_against_the_oracle(d, od, np.zeros((N, H, W, C), np.float16), w, dy, ops=(jz.JZ_BWD_DATA,))


def test_delta_filter_copies_the_input_bit_exactly(jz):
    import jzt
    rng = inputs.rng_for(12)
    N, H, W, C = 2, 10, 9, 64
    x = inputs.normal_f16(rng, (N, H, W, C), std=30.0)
    w = np.zeros((C, 3, 3, C), np.float16)
    w[np.arange(C), 1, 1, np.arange(C)] = 1.0
    y = jzt.run_conv(jz.JZ_FWD, jz.conv_desc(N, H, W, C, C, 3, 3, 1, 1), x, w, (N, H, W, C))
    assert np.array_equal(y.view(np.uint16), x.view(np.uint16))


def test_subnormal_inputs_and_outputs_are_kept(jz):
    # 2^-24 (the paper's underflow threshold) times 1, 2, 3 ... must come out as the exact subnormal, not zero
    import jzt
    C = 64
    x = np.zeros((1, 1, 1, C), np.float16)
    x[0, 0, 0, 0] = np.float16(2.0 ** -24)
    w = np.zeros((8, 1, 1, C), np.float16)
    w[:, 0, 0, 0] = np.arange(1, 9)
    y = jzt.run_conv(jz.JZ_FWD, jz.conv_desc(1, 1, 1, C, 8, 1, 1), x, w, (1, 1, 1, 8))
    assert np.array_equal(y.ravel().view(np.uint16), np.arange(1, 9, dtype=np.uint16))


def test_adjoint_identities_on_gpu_outputs(jz):
    import jzt
    c = inputs.conv_case((13,), 2, 12, 12, 64, 128, 3, 3, 1, 1, loss_scale=1.0)
    d = jzt.desc_of(c)
    y = jzt.run_conv(jz.JZ_FWD, d, c.x, c.w16, (c.N, c.P, c.Q, c.K)).astype(np.float64)
    dx = jzt.run_conv(jz.JZ_BWD_DATA, d, c.dy, c.w16, (c.N, c.H, c.W, c.C)).astype(np.float64)
    dw = jzt.run_conv(jz.JZ_BWD_WEIGHT, d, c.x, c.dy, (c.K, c.R, c.S, c.C)).astype(np.float64)
    a = np.sum(y * c.dy.astype(np.float64))
    b = np.sum(c.x.astype(np.float64) * dx)
    e = np.sum(c.w16.astype(np.float64) * dw)
    scale = np.linalg.norm(y) * np.linalg.norm(c.dy.astype(np.float64))
    assert abs(a - b) <= 1e-3 * scale and abs(a - e) <= 1e-3 * scale


def test_same_inputs_give_identical_bits(jz):
    import jzt
    c = inputs.conv_case((14,), 4, 7, 7, 192, 320, 3, 3, 1, 1, loss_scale=16.0)   # split-K in every op
    d = jzt.desc_of(c)
    for op, a, b, shp in ((jz.JZ_FWD, c.x, c.w16, (c.N, c.P, c.Q, c.K)), (jz.JZ_BWD_DATA, c.dy, c.w16, (c.N, c.H, c.W, c.C)),
                          (jz.JZ_BWD_WEIGHT, c.x, c.dy, (c.K, c.R, c.S, c.C))):
        r1 = jzt.run_conv(op, d, a, b, shp)
        r2 = jzt.run_conv(op, d, a, b, shp)
        assert np.array_equal(r1.view(np.uint16), r2.view(np.uint16))


KERNEL_VARIANTS = [
    # (tile_m, tile_n, k tile, wavefronts, ring): every LDS-direct kernel variant, forced through the planner's tuning
    # hook so that each one is compared with the oracle whatever the planner would have picked
    (128, 128, 32, 4, 4), (128, 64, 32, 4, 4), (64, 128, 32, 4, 4), (64, 64, 32, 4, 4),
    (128, 128, 64, 4, 4), (128, 64, 64, 4, 4), (64, 128, 64, 4, 4), (64, 64, 64, 4, 4),
    (128, 128, 64, 8, 4), (256, 128, 64, 8, 3), (256, 128, 32, 8, 4), (256, 256, 32, 8, 4),
]


@pytest.mark.parametrize("splits", [1, 3])
@pytest.mark.parametrize("variant", KERNEL_VARIANTS, ids=lambda v: "x".join(str(i) for i in v))
def test_every_kernel_variant_against_the_oracle(jz, variant, splits):
    import jzt
    import oracle
    # M = 675 pixels (2.6 tiles of 256 rows), 128 -> 320 channels (1.25 tiles of 256 columns), 3x3 with padding
    N, H, W, C, K, R, S, st, pad = 3, 15, 15, 128, 320, 3, 3, 1, 1
    od = oracle.conv_desc(N, H, W, C, K, R, S, st, (pad, pad))
    d = jz.conv_desc(N, H, W, C, K, R, S, st, (pad, pad))
    rng = inputs.rng_for(16, *variant)
    x = inputs.normal_f16(rng, (N, H, W, C))
    w = inputs.he_normal_f32(rng, (K, R, S, C), R * S * C).astype(np.float16)
    dy = inputs.normal_f16(rng, (N, od.P, od.Q, K), std=8.0)
    with jzt.forced_variant(d, *variant, splits=splits):
        if splits > 1:
            assert "%d splits" % splits in jz.jz_conv2d_describe_plan(jz.JZ_FWD, d)
        jzt.all_ops_against_the_oracle(d, od, x, w, dy)
    if splits > 1:
        return
    # a strided 1x1 layer: the scatter epilogue of backward-data, also in its slabbed form
    N, H, W, C, K = 2, 14, 14, 256, 128
    od = oracle.conv_desc(N, H, W, C, K, 1, 1, 2, (0, 0))
    d = jz.conv_desc(N, H, W, C, K, 1, 1, 2, (0, 0))
    w = inputs.he_normal_f32(rng, (K, 1, 1, C), C).astype(np.float16)
    dy = inputs.normal_f16(rng, (N, od.P, od.Q, K), std=8.0)
    with jzt.forced_variant(d, *variant, ops=(jz.JZ_BWD_DATA,)):
        assert "scatter epilogue" in jz.jz_conv2d_describe_plan(jz.JZ_BWD_DATA, d)
        jzt.all_ops_against_the_oracle(d, od, x, w, dy, ops=(jz.JZ_BWD_DATA,))   # x is not an input of this op


@pytest.mark.parametrize("tile", [(128, 128), (128, 64), (64, 128), (64, 64)], ids=lambda t: "%dx%d" % t)
def test_three_stage_ring_variants_against_the_oracle(jz, tile):
    # the short-ring variants (three stages, three to six workgroups per compute unit), on a short and a long reduction
    import jzt
    import oracle
    for (N, H, W, C, K, R, pad) in ((5, 12, 12, 64, 192, 1, 0), (2, 13, 13, 128, 192, 3, 1), (1, 9, 9, 32, 64, 1, 0)):
        od = oracle.conv_desc(N, H, W, C, K, R, R, 1, (pad, pad))
        d = jz.conv_desc(N, H, W, C, K, R, R, 1, (pad, pad))
        rng = inputs.rng_for(18, tile[0] * 1000 + tile[1], C, R)
        x = inputs.normal_f16(rng, (N, H, W, C))
        w = inputs.he_normal_f32(rng, (K, R, R, C), R * R * C).astype(np.float16)
        dy = inputs.normal_f16(rng, (N, od.P, od.Q, K), std=8.0)
        with jzt.forced_variant(d, tile[0], tile[1], 32, 4, 3, splits={jz.JZ_BWD_WEIGHT: 2}):
            jzt.all_ops_against_the_oracle(d, od, x, w, dy)


@pytest.mark.parametrize("tile,nst", [((256, 128), 3), ((128, 128), 4), ((128, 128), 3)])
def test_eight_wavefront_32_deep_variants_against_the_oracle(jz, tile, nst):
    # 8 wavefronts on 32-deep tiles with rings short enough for two or three workgroups per compute unit
    import jzt
    import oracle
    for (N, H, W, C, K, R, pad) in ((3, 15, 15, 128, 320, 3, 1), (5, 12, 12, 64, 192, 1, 0), (2, 9, 9, 32, 64, 1, 0)):
        od = oracle.conv_desc(N, H, W, C, K, R, R, 1, (pad, pad))
        d = jz.conv_desc(N, H, W, C, K, R, R, 1, (pad, pad))
        rng = inputs.rng_for(21, tile[0] * 1000 + tile[1], nst, C, R)
        x = inputs.normal_f16(rng, (N, H, W, C))
        w = inputs.he_normal_f32(rng, (K, R, R, C), R * R * C).astype(np.float16)
        dy = inputs.normal_f16(rng, (N, od.P, od.Q, K), std=8.0)
        with jzt.forced_variant(d, tile[0], tile[1], 32, 8, nst, splits={jz.JZ_BWD_WEIGHT: 2}):
            jzt.all_ops_against_the_oracle(d, od, x, w, dy)


@pytest.mark.parametrize("tile", [(128, 128), (128, 64), (64, 128), (64, 64)], ids=lambda t: "%dx%d" % t)
@pytest.mark.parametrize("nst", [4, 3])
def test_small_channel_kernel_variants_against_the_oracle(jz, tile, nst):
    # 3-channel stems run on a padded 4-channel copy: every masked forward variant, and backward-weight both with a split
    # reduction (the reduction kernel writes the real filter entries) and without (separate unpacking kernel)
    import jzt
    import oracle
    for (N, H, C, K, R, st, pad, splits) in ((3, 37, 3, 64, 7, 2, 3, 4), (2, 23, 3, 72, 7, 2, 3, 1), (4, 39, 3, 96, 11, 4, 0, 2),
                                             (4, 20, 4, 64, 5, 2, 2, 3), (1, 30, 1, 64, 3, 2, 1, 2)):
        od = oracle.conv_desc(N, H, H, C, K, R, R, st, (pad, pad))
        d = jz.conv_desc(N, H, H, C, K, R, R, st, (pad, pad))
        rng = inputs.rng_for(20, tile[0] * 1000 + tile[1], nst, H, R)
        x = inputs.normal_f16(rng, (N, H, H, C))
        w = inputs.he_normal_f32(rng, (K, R, R, C), R * R * C).astype(np.float16)
        dy = inputs.normal_f16(rng, (N, od.P, od.Q, K), std=8.0)
        bk_fwd = 32 if 4 * R <= 32 else 64           # one filter row of the padded copy is one k tile
        with jzt.forced_variant(d, tile[0], tile[1], bk_fwd, 4, nst if bk_fwd == 32 else 4, ops=(jz.JZ_FWD,)):
            assert "4-channel padded copy" in jz.jz_conv2d_describe_plan(jz.JZ_FWD, d)
            jzt.all_ops_against_the_oracle(d, od, x, w, dy, ops=(jz.JZ_FWD,))
        with jzt.forced_variant(d, tile[0], tile[1], 32, 4, nst, splits=splits, ops=(jz.JZ_BWD_WEIGHT,)):
            plan_bw = jz.jz_conv2d_describe_plan(jz.JZ_BWD_WEIGHT, d)
            assert "4-channel padded copy" in plan_bw and ("%d splits" % splits) in plan_bw, plan_bw
            jzt.all_ops_against_the_oracle(d, od, x, w, dy, ops=(jz.JZ_BWD_WEIGHT,))


PATCH_KERNEL = [
    # N, H, W, C, K, R, S, stride, pad
    (3, 37, 37, 3, 64, 7, 7, 2, 3),             # the ResNet stem's geometry: 361 pixels per image, one ragged block each
    (2, 75, 75, 3, 64, 7, 7, 2, 3),             # 1444 pixels: three blocks per image, blocks that start mid-row
    (4, 39, 39, 3, 96, 11, 11, 4, 0),           # the AlexNet stem's geometry: 3 channel tiles, stride 4
    (2, 83, 83, 3, 96, 11, 11, 4, 2),           # 361 pixels in blocks of 256
    (4, 20, 20, 4, 64, 5, 5, 2, 2),             # 4 real channels
    (1, 30, 30, 1, 32, 3, 3, 2, 1),             # one channel, one channel tile, a single k step per filter row
    (2, 41, 29, 3, 128, 7, 5, (3, 2), (3, 1)),  # 4 channel tiles, odd row stride, H != W, R != S, unequal pads
    (2, 33, 45, 2, 64, 4, 6, (1, 4), (0, 2)),   # even filter sizes, unit row stride
    (1, 40, 40, 3, 32, 13, 13, 2, 6),           # 13 taps per row: four k steps
    (1, 9, 9, 3, 32, 3, 3, 2, 1),               # 25 output pixels: less than one 32-pixel tile
    (1, 12, 400, 3, 64, 3, 3, (1, 2), 1),       # wide and flat: a block is little more than one output row
    (3, 21, 21, 3, 64, 7, 7, (4, 2), (3, 3)),   # row stride larger than the column stride, 6 x 11 output pixels
]


@pytest.mark.parametrize("shape", PATCH_KERNEL, ids=lambda t: "x".join(str(v) for v in t[:9]).replace(" ", ""))
def test_small_channel_forward_from_a_patch_in_lds(jz, shape):
    # the forward pass of small-channel strided layers reads its operands out of an input patch in LDS (whole filter
    # resident); whole output against the oracle, norm-wise and element by element
    import jzt
    import oracle
    N, H, W, C, K, R, S, st, pad = shape
    od = oracle.conv_desc(N, H, W, C, K, R, S, st, pad)
    d = jz.conv_desc(N, H, W, C, K, R, S, st, pad)
    assert "patch kernel" in jz.jz_conv2d_describe_plan(jz.JZ_FWD, d)
    rng = inputs.rng_for(27, H, W, K, R)
    x = inputs.normal_f16(rng, (N, H, W, C))
    w = inputs.he_normal_f32(rng, (K, R, S, C), R * S * C).astype(np.float16)
    jzt.all_ops_against_the_oracle(d, od, x, w, np.zeros((N, od.P, od.Q, K), np.float16), ops=(jz.JZ_FWD,))


def test_patch_kernel_workgroups_walk_through_several_blocks(jz):
    # more blocks than resident workgroups (1080 blocks of 256 pixels, 768 workgroups): every workgroup reloads its patch and reuses the
    # filter; all-ones inputs count the taps exactly, seeded inputs go against the oracle
    import jzt
    import oracle
    N, H, W, C, K, R, S, st, pad = 60, 131, 131, 3, 64, 7, 7, 2, 3
    od = oracle.conv_desc(N, H, W, C, K, R, S, st, pad)
    d = jz.conv_desc(N, H, W, C, K, R, S, st, pad)
    assert "patch kernel" in jz.jz_conv2d_describe_plan(jz.JZ_FWD, d)
    ones_x = np.ones((N, H, W, C), np.float16)
    ones_w = np.ones((K, R, S, C), np.float16)
    y = jzt.run_conv(jz.JZ_FWD, d, ones_x, ones_w, (N, od.P, od.Q, K)).astype(np.float64)
    rows = np.minimum(np.arange(od.P) * 2 - 3 + R, H) - np.maximum(np.arange(od.P) * 2 - 3, 0)
    cols = np.minimum(np.arange(od.Q) * 2 - 3 + S, W) - np.maximum(np.arange(od.Q) * 2 - 3, 0)
    want = (rows[:, None] * cols[None, :] * C).astype(np.float64)
    assert np.array_equal(y, np.broadcast_to(want[None, :, :, None], y.shape))
    rng = inputs.rng_for(28)
    x = inputs.normal_f16(rng, (N, H, W, C))
    w = inputs.he_normal_f32(rng, (K, R, S, C), R * S * C).astype(np.float16)
    jzt.all_ops_against_the_oracle(d, od, x, w, np.zeros((N, od.P, od.Q, K), np.float16), ops=(jz.JZ_FWD,))


def test_small_channel_layers_the_patch_kernel_does_not_take(jz):
    # output channels that are no multiple of 32 stay on the implicit-GEMM kernel, and so does a layer with a variant
    # set through the tuning hook
    d = jz.conv_desc(2, 23, 23, 3, 72, 7, 7, 2, 3)
    assert "patch kernel" not in jz.jz_conv2d_describe_plan(jz.JZ_FWD, d)
    d = jz.conv_desc(1, 64, 600, 3, 128, 31, 15, 2, 0)          # a filter of 508 KB does not fit the LDS
    assert "patch kernel" not in jz.jz_conv2d_describe_plan(jz.JZ_FWD, d)
    d = jz.conv_desc(1, 64, 64, 3, 160, 7, 7, 2, 3)             # more than 128 output channels
    assert "patch kernel" not in jz.jz_conv2d_describe_plan(jz.JZ_FWD, d)
    d = jz.conv_desc(2, 23, 23, 3, 64, 7, 7, 2, 3)
    assert "patch kernel" in jz.jz_conv2d_describe_plan(jz.JZ_FWD, d)
    import jzt
    with jzt.forced_variant(d, 128, 64, 32, 4, 4, ops=(jz.JZ_FWD,)):
        assert "patch kernel" not in jz.jz_conv2d_describe_plan(jz.JZ_FWD, d)
    assert "patch kernel" in jz.jz_conv2d_describe_plan(jz.JZ_FWD, d)


def test_run_time_tuning_hook_runs_the_chosen_kernel_correctly(jz):
    # a choice recorded with jz_conv2d_tune_set is what runs (no environment override involved), and the result still
    # agrees with the oracle; clearing restores the planner's own choice
    import jzt
    import oracle
    N, H, W, C, K, R, S, st, pad = 2, 14, 14, 128, 256, 3, 3, 1, 1
    od = oracle.conv_desc(N, H, W, C, K, R, S, st, (pad, pad))
    d = jz.conv_desc(N, H, W, C, K, R, S, st, (pad, pad))
    rng = inputs.rng_for(22)
    x = inputs.normal_f16(rng, (N, H, W, C))
    w = inputs.he_normal_f32(rng, (K, R, S, C), R * S * C).astype(np.float16)
    dy = inputs.normal_f16(rng, (N, od.P, od.Q, K), std=8.0)
    before = jz.jz_conv2d_describe_plan(jz.JZ_BWD_WEIGHT, d)
    try:
        jz.jz_conv2d_tune_set(jz.JZ_FWD, d, 256, 128, 32, 8, 3, 2)
        jz.jz_conv2d_tune_set(jz.JZ_BWD_DATA, d, 64, 128, 64, 4, 4, 1)
        jz.jz_conv2d_tune_set(jz.JZ_BWD_WEIGHT, d, 128, 128, 32, 8, 4, 3)
        assert "tile 256x128x32, 8 wavefronts, ring 3" in jz.jz_conv2d_describe_plan(jz.JZ_FWD, d)
        assert "tile 128x128x32, 8 wavefronts, ring 4" in jz.jz_conv2d_describe_plan(jz.JZ_BWD_WEIGHT, d)
        assert " 3 splits" in jz.jz_conv2d_describe_plan(jz.JZ_BWD_WEIGHT, d)
        res = jzt.all_ops_against_the_oracle(d, od, x, w, dy)
    finally:
        jz.jz_conv2d_tune_clear()
    assert jz.jz_conv2d_describe_plan(jz.JZ_BWD_WEIGHT, d) == before


@pytest.mark.parametrize("B,I,O", [(64, 2048, 1000), (128, 1024, 520), (5, 24, 7), (1, 64, 64), (130, 192, 72)])
def test_fully_connected_modes(jz, B, I, O):
    import jzt
    import oracle
    c = inputs.fc_case((15, B, I, O), B, I, O, loss_scale=32.0)
    jzt.fc_all_modes(B, I, O, c)


def test_fc_equals_one_by_one_conv_bit_for_bit(jz):
    import jzt
    c = inputs.fc_case((16,), 96, 256, 192)
    y1 = jzt.run_fc(jz.JZ_FWD, 96, 256, 192, c.x, c.w16, (96, 192))
    y2 = jzt.run_conv(jz.JZ_FWD, jz.conv_desc(96, 1, 1, 256, 192, 1, 1), c.x, c.w16, (96, 1, 1, 192))
    assert np.array_equal(y1.view(np.uint16).ravel(), y2.view(np.uint16).ravel())


def test_argument_errors(jz):
    import jzt
    api = jz
    d = api.conv_desc(2, 8, 8, 64, 64, 3, 3, 1, 1)
    x = torch.zeros(2 * 8 * 8 * 64, dtype=torch.float16, device=jzt.DEV)
    w = torch.zeros(64 * 9 * 64, dtype=torch.float16, device=jzt.DEV)
    y = torch.zeros(2 * 8 * 8 * 64, dtype=torch.float16, device=jzt.DEV)
    L = api.lib()
    import ctypes
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert L.jz_conv2d_fwd(ctypes.byref(d), None, w.data_ptr(), y.data_ptr(), None, 0, st) == api.JZ_ERR_NULL
    assert L.jz_conv2d_fwd(ctypes.byref(d), x.data_ptr() + 2, w.data_ptr(), y.data_ptr(), None, 0, st) == api.JZ_ERR_ALIGN
    assert L.jz_conv2d_fwd(ctypes.byref(d), x.data_ptr(), w.data_ptr(), x.data_ptr(), None, 0, st) == api.JZ_ERR_ALIAS
    bad = api.conv_desc(2, 8, 8, 64, 64, 3, 3, 1, 3)     # pad >= filter size
    assert L.jz_conv2d_fwd(ctypes.byref(bad), x.data_ptr(), w.data_ptr(), y.data_ptr(), None, 0, st) == api.JZ_ERR_SHAPE
    bad = api.conv_desc(2, 2, 2, 64, 64, 5, 5, 1, 0)     # filter larger than the padded image
    assert L.jz_conv2d_fwd(ctypes.byref(bad), x.data_ptr(), w.data_ptr(), y.data_ptr(), None, 0, st) == api.JZ_ERR_SHAPE
    dw = api.conv_desc(64, 7, 7, 64, 64, 3, 3, 1, 1)     # backward-weight needs a split-K workspace here
    need = api.jz_conv2d_workspace_bytes(api.JZ_BWD_WEIGHT, dw)
    assert need > 0
    xx = torch.zeros(64 * 49 * 64, dtype=torch.float16, device=jzt.DEV)
    assert L.jz_conv2d_bwd_weight(ctypes.byref(dw), xx.data_ptr(), xx.data_ptr() , w.data_ptr(), None, 0, st) == api.JZ_ERR_WORKSPACE
    assert L.jz_gemm_fc(7, 4, 4, 4, x.data_ptr(), w.data_ptr(), y.data_ptr(), None, 0, st) == api.JZ_ERR_UNSUPPORTED
    assert L.jz_gemm_fc(0, 0, 4, 4, x.data_ptr(), w.data_ptr(), y.data_ptr(), None, 0, st) == api.JZ_ERR_SHAPE
    torch.cuda.synchronize()
