"""Host-only checks of the C ABI: the library loads and exports every symbol include/jz.h declares, and
argument validation that needs no GPU returns the documented codes."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def jzlib():
    from paper_1807_11205_amd import api
    if not os.path.exists(api.LIB_PATH):
        from paper_1807_11205_amd import build
        build.build()
    return api


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "jz.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(jz_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(jzlib):
    L = jzlib.lib()
    names = declared_symbols()
    assert len(names) >= 11
    for n in names:
        assert hasattr(L, n), n
    assert sorted(jzlib.EXPORTS) == names


def test_status_strings_and_version(jzlib):
    assert jzlib.jz_version() >= 100
    assert jzlib.status_string(0) == "JZ_OK"
    for code in range(-8, 0):
        assert jzlib.status_string(code).startswith("JZ_ERR_")
    assert "unknown" in jzlib.status_string(-99)


def test_lars_table_validation_on_the_host(jzlib):
    import numpy as np
    L = jzlib.lib()
    n = ctypes.c_size_t(0)

    def ps(offsets, flags):
        o = np.asarray(offsets, np.int64)
        f = np.asarray(flags, np.uint8)
        s = jzlib.jz_param_set(len(flags), o.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                               f.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), None, None, None, None)
        s._keep = (o, f)
        return s

    assert L.jz_lars_workspace_bytes(ctypes.byref(ps([0, 64, 4160], [3, 2])), ctypes.byref(n)) == 0 and n.value > 0
    small = n.value
    assert L.jz_lars_workspace_bytes(ctypes.byref(ps([0, 64, 4160000], [3, 2])), ctypes.byref(n)) == 0 and n.value > small
    assert L.jz_lars_workspace_bytes(ctypes.byref(ps([0], [])), ctypes.byref(n)) == 0
    assert L.jz_lars_workspace_bytes(ctypes.byref(ps([8, 64], [3])), ctypes.byref(n)) == jzlib.JZ_ERR_SHAPE       # offsets[0] != 0
    assert L.jz_lars_workspace_bytes(ctypes.byref(ps([0, 64, 32], [3, 3])), ctypes.byref(n)) == jzlib.JZ_ERR_SHAPE  # decreasing
    assert L.jz_lars_workspace_bytes(ctypes.byref(ps([0, 2 ** 31], [3])), ctypes.byref(n)) == jzlib.JZ_ERR_UNSUPPORTED
    assert L.jz_lars_workspace_bytes(None, ctypes.byref(n)) == jzlib.JZ_ERR_NULL
    assert L.jz_lars_workspace_bytes(ctypes.byref(ps([0, 8], [3])), None) == jzlib.JZ_ERR_NULL


def test_describe_plan_for_every_resnet50_and_alexnet_layer(jzlib):
    # host logic only: the planner must produce a runnable plan (a kernel variant that exists, a workspace size) for
    # every layer of the two models of the paper's Table 3, with and without its table of measured choices
    import re
    from paper_1807_11205_amd import shapes
    known = {(128, 128, 32, 4), (128, 64, 32, 4), (64, 128, 32, 4), (64, 64, 32, 4), (128, 128, 64, 8), (256, 128, 64, 8),
             (256, 128, 32, 8), (256, 256, 32, 8), (128, 128, 64, 4), (128, 64, 64, 4), (64, 128, 64, 4), (64, 64, 64, 4),
             (128, 128, 32, 8)}
    layers = [(64, c) for c in shapes.resnet50_convs()] + [(128, c) for c in shapes.alexnet_convs()]
    for use_table in (True, False):
        jzlib.jz_conv2d_tune_use_table(use_table)
        try:
            for batch, cs in layers:
                d = jzlib.conv_desc(batch, cs.H, cs.H, cs.C, cs.K, cs.R, cs.R, cs.stride, cs.pad)
                for op in (jzlib.JZ_FWD, jzlib.JZ_BWD_DATA, jzlib.JZ_BWD_WEIGHT):
                    text = jzlib.jz_conv2d_describe_plan(op, d)
                    if "patch kernel" in text:      # the forward pass of the two 3-channel stems
                        assert op == jzlib.JZ_FWD and cs.C == 3 and "padded copy" in text, text
                        assert re.search(r"(256 pixels x 64|256 pixels x 96) channels per block", text), text
                        assert jzlib.jz_conv2d_workspace_bytes(op, d) > 0
                        continue
                    m = re.search(r"(vector|element-wise) tile (\d+)x(\d+)x(\d+), (\d+) wavefronts, ring \d+, (\d+) x (\d+) tiles, (\d+) splits of (\d+) k tiles", text)
                    assert m, text
                    bm, bn, bk, wv, tm, tn, sp, kps = (int(v) for v in m.groups()[1:])
                    if m.group(1) == "vector":
                        assert (bm, bn, bk, wv) in known, text
                    assert tm >= 1 and tn >= 1 and sp >= 1 and kps >= 1
                    ws = jzlib.jz_conv2d_workspace_bytes(op, d)
                    assert (ws > 0) == (sp > 1 or "padded copy" in text), text
        finally:
            jzlib.jz_conv2d_tune_clear()


def test_tensor_size_limit_is_checked_on_the_host(jzlib):
    # the kernels form byte offsets in 32 bits: a tensor of 2^30 or more elements is refused before any launch, through
    # every query and for each of the three tensors of a layer; one element less is planned
    L = jzlib.lib()
    n = ctypes.c_size_t(0)
    ok = jzlib.conv_desc(1, 1, 1 << 15, (1 << 15) - 8, 8, 1, 1)                   # x: 2^30 - 2^18 elements
    big_x = jzlib.conv_desc(1, 1, 1 << 15, 1 << 15, 8, 1, 1)                      # x: exactly 2^30 elements
    big_y = jzlib.conv_desc(1, 1, 1 << 15, 8, 1 << 15, 1, 1)                      # y: 2^30
    big_w = jzlib.conv_desc(1, 1, 1, 1 << 15, 1 << 15, 1, 1)                      # w: 2^30
    for op in (jzlib.JZ_FWD, jzlib.JZ_BWD_DATA, jzlib.JZ_BWD_WEIGHT):
        assert L.jz_conv2d_workspace_bytes(op, ctypes.byref(ok), ctypes.byref(n)) == jzlib.JZ_OK
        for d in (big_x, big_y, big_w):
            assert L.jz_conv2d_workspace_bytes(op, ctypes.byref(d), ctypes.byref(n)) == jzlib.JZ_ERR_UNSUPPORTED
            assert L.jz_conv2d_describe_plan(op, ctypes.byref(d), ctypes.create_string_buffer(256), 256) == jzlib.JZ_ERR_UNSUPPORTED
    A = 0x10000000                                                               # never dereferenced: refused first
    assert L.jz_conv2d_fwd(ctypes.byref(big_x), A, A + (1 << 32), A + (1 << 33), None, 0, None) == jzlib.JZ_ERR_UNSUPPORTED
    # a padded multi-tap layer just under the limit: descriptor size + padding margin stay below 2^32 bytes
    pad = jzlib.conv_desc(1, 1 << 10, (1 << 10) - 1, 1 << 10, 8, 3, 3, 1, 1)
    assert L.jz_conv2d_workspace_bytes(jzlib.JZ_FWD, ctypes.byref(pad), ctypes.byref(n)) == jzlib.JZ_OK


def test_tuned_table_is_used_for_the_benchmark_shapes(jzlib):
    # a stage-4 3x3 layer of ResNet-50 at batch 64 is in the table of measured choices; switching the table off must be
    # able to change the plan, switching it on must give the table's entry
    d = jzlib.conv_desc(64, 14, 14, 256, 256, 3, 3, 1, 1)
    with_table = jzlib.jz_conv2d_describe_plan(jzlib.JZ_BWD_WEIGHT, d)
    assert "M 256 N 2304 K 12544" in with_table
    assert "tile 128x128x64, 8 wavefronts, ring 4" in with_table   # the table's entry for this shape
    # a shape next to it that is in no table gets the cost model's plan, and switching the table off must still plan
    other = jzlib.conv_desc(48, 14, 14, 256, 256, 3, 3, 1, 1)
    assert "M 256 N 2304 K 9408" in jzlib.jz_conv2d_describe_plan(jzlib.JZ_BWD_WEIGHT, other)
    jzlib.jz_conv2d_tune_use_table(False)
    try:
        assert "M 256 N 2304 K 12544" in jzlib.jz_conv2d_describe_plan(jzlib.JZ_BWD_WEIGHT, d)
    finally:
        jzlib.jz_conv2d_tune_clear()
    assert jzlib.jz_conv2d_describe_plan(jzlib.JZ_BWD_WEIGHT, d) == with_table


def test_run_time_tuning_hook_changes_the_plan_and_can_be_cleared(jzlib):
    d = jzlib.conv_desc(64, 14, 14, 256, 256, 3, 3, 1, 1)
    before = jzlib.jz_conv2d_describe_plan(jzlib.JZ_FWD, d)
    try:
        jzlib.jz_conv2d_tune_set(jzlib.JZ_FWD, d, 64, 64, 32, 4, 3, 2)
        assert "tile 64x64x32, 4 wavefronts, ring 3" in jzlib.jz_conv2d_describe_plan(jzlib.JZ_FWD, d)
        assert "2 splits" in jzlib.jz_conv2d_describe_plan(jzlib.JZ_FWD, d)
        jzlib.jz_conv2d_tune_set(jzlib.JZ_FWD, d, 256, 128, 64, 8, 3, 1)      # replaces the entry for this shape
        assert "tile 256x128x64, 8 wavefronts, ring 3" in jzlib.jz_conv2d_describe_plan(jzlib.JZ_FWD, d)
        assert jzlib.jz_conv2d_describe_plan(jzlib.JZ_BWD_DATA, d) != ""       # other ops of the layer are untouched
        with pytest.raises(jzlib.JzError):
            jzlib.jz_conv2d_tune_set(jzlib.JZ_FWD, d, 96, 96, 32, 4, 4, 1)    # no such kernel
        with pytest.raises(jzlib.JzError):
            jzlib.jz_conv2d_tune_set(jzlib.JZ_FWD, jzlib.conv_desc(2, 9, 7, 3, 5, 3, 2, (2, 1), (1, 0)), 64, 64, 32, 4, 4, 1)  # element-wise path
        # the 3-channel stem runs the 4-wavefront kernels at its own k tile depth
        stem = jzlib.conv_desc(64, 224, 224, 3, 64, 7, 7, 2, 3)
        jzlib.jz_conv2d_tune_set(jzlib.JZ_BWD_WEIGHT, stem, 64, 128, 32, 4, 4, 64)
        assert "tile 64x128x32" in jzlib.jz_conv2d_describe_plan(jzlib.JZ_BWD_WEIGHT, stem)
        with pytest.raises(jzlib.JzError):
            jzlib.jz_conv2d_tune_set(jzlib.JZ_BWD_WEIGHT, stem, 128, 128, 64, 8, 4, 64)
    finally:
        jzlib.jz_conv2d_tune_clear()
    assert jzlib.jz_conv2d_describe_plan(jzlib.JZ_FWD, d) == before


def test_every_table_entry_belongs_to_a_layer_and_is_what_the_planner_runs(jzlib):
    # the generated tables are keyed by GEMM dimensions: a key that no layer produces would silently never be used, and
    # an entry the planner cannot honour (no such kernel) would silently fall back to the cost model
    from paper_1807_11205_amd import tune
    pkg = os.path.dirname(os.path.abspath(tune.__file__))
    ops = {"fwd": jzlib.JZ_FWD, "bwd_data": jzlib.JZ_BWD_DATA, "bwd_weight": jzlib.JZ_BWD_WEIGHT}
    for model, inc, other_batch in (("resnet50", "jz_tuned.inc", None), ("alexnet", "jz_tuned_alexnet.inc", None),
                                    ("resnet50", "jz_tuned_resnet50_n32.inc", 32), ("resnet50", "jz_tuned_resnet50_n128.inc", 128),
                                    ("resnet50", "jz_tuned_resnet50_n256.inc", 256)):
        batch, layers = tune.model_layers(model)
        batch = other_batch or batch
        by_name = {cs.name: cs for cs in layers}
        entries = 0
        for line in open(os.path.join(pkg, "csrc", inc)):
            m = re.match(r"\{(\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+)\},\s*// (\S+) (\S+):", line)
            if not m:
                assert line.startswith("//") or not line.strip(), line
                continue
            entries += 1
            op, M, N, K, taps, sc, bm, bn, bk, wv, nst, sp = (int(v) for v in m.groups()[:12])
            cs = by_name[m.group(13)]
            opn = m.group(14)
            assert tune.OPS.index(opn) == op
            rec = dict(H=cs.H, C=cs.C, K=cs.K, R=cs.R, stride=cs.stride, pad=cs.pad, batch=batch, op=opn)
            assert tune.gemm_dims(rec) == (M, N, K, taps, sc), line
            d = jzlib.conv_desc(batch, cs.H, cs.H, cs.C, cs.K, cs.R, cs.R, cs.stride, cs.pad)
            plan = jzlib.jz_conv2d_describe_plan(ops[opn], d)
            assert "M %d N %d K %d:" % (M, N, K) in plan, (line, plan)
            assert "tile %dx%dx%d, %d wavefronts, ring %d," % (bm, bn, bk, wv, nst) in plan, (line, plan)
        assert entries == 3 * len(layers) - sum(1 for cs in layers if cs.first), (model, entries)


def test_layer_entry_points_validate_on_the_host_before_any_launch(jzlib):
    """Shape, null, alignment and aliasing mistakes are caught from the arguments alone (the pointers below are never
    dereferenced: every call returns before a launch), and empty inputs are accepted without touching the GPU."""
    L, E = jzlib.lib(), jzlib
    A, B, C_ = 0x10000000, 0x20000000, 0x30000000       # fake, well separated, 16-byte aligned device addresses
    f = ctypes.c_float
    assert L.jz_add_fwd(0, None, None, 1, None, None) == E.JZ_OK
    assert L.jz_add_fwd(12, A, B, 1, C_, None) == E.JZ_ERR_SHAPE
    assert L.jz_add_fwd(16, A, None, 1, C_, None) == E.JZ_ERR_NULL
    assert L.jz_add_fwd(16, A, B + 8, 1, C_, None) == E.JZ_ERR_ALIGN
    assert L.jz_add_fwd(64, A, B, 0, A + 32, None) == E.JZ_ERR_ALIAS
    assert L.jz_relu_bwd(0, None, None, None, None) == E.JZ_OK
    assert L.jz_relu_bwd(64, A, B, A, None) == E.JZ_ERR_ALIAS
    assert L.jz_relu_bwd_sum(0, None, None, None, None, None) == E.JZ_OK
    assert L.jz_relu_bwd_sum(64, A, B, None, C_, None) == E.JZ_ERR_NULL
    assert L.jz_relu_bwd_sum(64, A, B, C_, A, None) == E.JZ_ERR_ALIAS      # dx must not be y
    assert L.jz_maxpool_fwd(0, 8, 8, 8, 3, 2, 1, None, None, None, None) == E.JZ_OK
    assert L.jz_maxpool_fwd(1, 8, 8, 8, 3, 0, 1, A, B, None, None) == E.JZ_ERR_SHAPE
    assert L.jz_maxpool_fwd(1, 8, 8, 8, 3, 2, 1, A, B, C_ + 4, None) == E.JZ_ERR_ALIGN
    assert L.jz_maxpool_bwd(1, 8, 8, 8, 3, 2, 1, None, None, A, B, None) == E.JZ_ERR_NULL
    assert L.jz_avgpool_fwd(0, 49, 2048, None, None, None) == E.JZ_OK
    assert L.jz_avgpool_fwd(2, 49, 2044, A, B, None) == E.JZ_ERR_SHAPE
    assert L.jz_avgpool_bwd(2, 49, 2048, None, B, None) == E.JZ_ERR_NULL
    assert L.jz_bias_add(0, 8, None, None, None, None) == E.JZ_OK
    assert L.jz_bias_add(4, 8, A, B, B, None) == E.JZ_ERR_ALIAS
    assert L.jz_bias_grad(4, 8, A, None, None) == E.JZ_ERR_NULL
    assert L.jz_softmax_xent_bwd(0, 1000, None, None, f(1.0), None, None, None, None) == E.JZ_OK
    assert L.jz_softmax_xent_bwd(4, 1000, A, B, f(-1.0), None, C_, C_ + 0x100000, None) == E.JZ_ERR_SHAPE
    assert L.jz_softmax_xent_bwd(4, 1000, A, B, f(1.0), None, A, C_, None) == E.JZ_ERR_ALIAS
    assert L.jz_softmax_xent_bwd(4, 1000, A, B, f(1.0), 0x40000004, C_, C_ + 0x100000, None) == E.JZ_ERR_ALIGN
    n = ctypes.c_size_t(0)
    assert L.jz_bn_workspace_bytes(64, 16, ctypes.byref(n)) == E.JZ_OK
    D = [0x10000000 + i * 0x1000000 for i in range(12)]
    be = lambda **o: L.jz_bn_bwd_block_end(64, 16, o.get("x", D[0]), o.get("y", D[1]), o.get("a", D[2]), o.get("b", D[3]), D[4], D[5], D[6],
                                           o.get("g", D[7]), o.get("dx", D[8]), D[9], D[9] + 0x1000, D[10], o.get("n", n.value), None)
    assert be(y=None) == E.JZ_ERR_NULL and be(g=None) == E.JZ_ERR_NULL
    assert be(n=n.value - 1) == E.JZ_ERR_WORKSPACE
    assert be(b=D[3] + 2) == E.JZ_ERR_ALIGN
    assert be(g=D[2]) == E.JZ_ERR_ALIAS and be(dx=D[7]) == E.JZ_ERR_ALIAS and be(g=D[0]) == E.JZ_ERR_ALIAS
    assert L.jz_bn_bwd_block_end(64, 12, D[0], D[1], D[2], None, D[4], D[5], D[6], D[7], D[8], D[9], D[9] + 0x1000, D[10], n.value,
                                 None) == E.JZ_ERR_UNSUPPORTED
    assert L.jz_loss_scale_init(None, f(1.0), None) == E.JZ_ERR_NULL
    assert L.jz_loss_scale_init(A, f(0.0), None) == E.JZ_ERR_SHAPE
    assert L.jz_loss_scale_init(A + 4, f(1.0), None) == E.JZ_ERR_ALIGN


def test_fused_convolution_batch_norm_workspace_and_validation(jzlib):
    L, E = jzlib.lib(), jzlib
    n, m = ctypes.c_size_t(0), ctypes.c_size_t(0)
    for cs_args in ((64, 56, 56, 64, 64, 3, 3, 1, 1), (64, 56, 56, 64, 256, 1, 1, 1, 0), (64, 224, 224, 3, 64, 7, 7, 2, 3)):
        d = jzlib.conv_desc(*cs_args)
        assert L.jz_conv2d_bn_relu_fwd_workspace_bytes(ctypes.byref(d), ctypes.byref(n)) == E.JZ_OK
        assert L.jz_conv2d_workspace_bytes(E.JZ_FWD, ctypes.byref(d), ctypes.byref(m)) == E.JZ_OK
        # room for the convolution's own workspace, the per-tile (or per-slab) sums and the coefficients
        assert n.value >= m.value + 4 * d.K * 4 and n.value < m.value + (64 << 20)
    d = jzlib.conv_desc(2, 8, 8, 16, 4096, 1, 1, 1, 0)                  # more channels than the normalization handles
    assert L.jz_conv2d_bn_relu_fwd_workspace_bytes(ctypes.byref(d), ctypes.byref(n)) == E.JZ_ERR_UNSUPPORTED
    d = jzlib.conv_desc(2, 8, 8, 16, 32, 3, 3, 1, 1)
    assert L.jz_conv2d_bn_relu_fwd_workspace_bytes(ctypes.byref(d), ctypes.byref(n)) == E.JZ_OK
    A = 0x10000000
    f = ctypes.c_float
    args = lambda **o: [o.get(k, A + i * 0x1000000) for i, k in enumerate(("x", "w", "g", "b"))]
    assert L.jz_conv2d_bn_relu_fwd(ctypes.byref(d), *args(), f(1e-5), None, 1, A + 0x5000000, None, A + 0x7000000, A + 0x8000000,
                                   A + 0x9000000, n.value, None) == E.JZ_ERR_NULL
    assert L.jz_conv2d_bn_relu_fwd(ctypes.byref(d), *args(), f(-1.0), None, 1, A + 0x5000000, A + 0x6000000, A + 0x7000000, A + 0x8000000,
                                   A + 0x9000000, n.value, None) == E.JZ_ERR_SHAPE
    assert L.jz_conv2d_bn_relu_fwd(ctypes.byref(d), *args(), f(1e-5), None, 1, A + 0x5000000, A + 0x6000000, A + 0x7000000, A + 0x8000000,
                                   A + 0x9000000, n.value - 1, None) == E.JZ_ERR_WORKSPACE
    assert L.jz_conv2d_bn_relu_fwd(ctypes.byref(d), *args(), f(1e-5), A + 0x6000000, 1, A + 0x5000000, A + 0x6000000, A + 0x7000000,
                                   A + 0x8000000, A + 0x9000000, n.value, None) == E.JZ_ERR_ALIAS


def test_fused_backward_data_batch_norm_validation_on_the_host(jzlib):
    """jz_conv2d_bwd_data_bn_relu_bwd / jz_conv2d_bwd_data_block_end_bwd: workspace sizes and every argument mistake are
    settled on the host (fake, well separated device addresses that are never dereferenced)."""
    L, E = jzlib.lib(), jzlib
    n, m = ctypes.c_size_t(0), ctypes.c_size_t(0)
    for cs_args in ((64, 56, 56, 64, 64, 3, 3, 1, 1), (64, 14, 14, 1024, 256, 1, 1, 1, 0), (64, 56, 56, 256, 128, 1, 1, 2, 0)):
        d = jzlib.conv_desc(*cs_args)
        assert L.jz_conv2d_bwd_data_bn_relu_bwd_workspace_bytes(ctypes.byref(d), ctypes.byref(n)) == E.JZ_OK
        assert L.jz_conv2d_workspace_bytes(E.JZ_BWD_DATA, ctypes.byref(d), ctypes.byref(m)) == E.JZ_OK
        assert n.value >= m.value + 4 * d.C * 4 and n.value < m.value + (64 << 20)
    assert L.jz_conv2d_bwd_data_bn_relu_bwd_workspace_bytes(ctypes.byref(d), None) == E.JZ_ERR_NULL
    d = jzlib.conv_desc(2, 8, 8, 4096, 32, 1, 1, 1, 0)                  # more channels than the normalization handles
    assert L.jz_conv2d_bwd_data_bn_relu_bwd_workspace_bytes(ctypes.byref(d), ctypes.byref(n)) == E.JZ_ERR_UNSUPPORTED
    d = jzlib.conv_desc(2, 8, 8, 16, 32, 3, 3, 1, 1)
    assert L.jz_conv2d_bwd_data_bn_relu_bwd_workspace_bytes(ctypes.byref(d), ctypes.byref(n)) == E.JZ_OK
    D = [0x10000000 + i * 0x1000000 for i in range(14)]
    names = ("dy", "w", "x", "y", "g", "m", "s", "dz", "dx", "dg", "db", "ws")

    def plain(**o):
        a = {k: D[i] for i, k in enumerate(names)}
        a.update(o)
        return L.jz_conv2d_bwd_data_bn_relu_bwd(ctypes.byref(d), a["dy"], a["w"], a["x"], a["y"], a["g"], a["m"], a["s"], a["dz"], a["dx"],
                                                a["dg"], a["db"], a["ws"], o.get("n", n.value), None)

    def end(**o):
        a = {k: D[i] for i, k in enumerate(names)}
        a["add"] = D[12]
        a.update(o)
        return L.jz_conv2d_bwd_data_block_end_bwd(ctypes.byref(d), a["dy"], a["w"], a["add"], a["x"], a["y"], a["g"], a["m"], a["s"], a["dz"],
                                                  a["dx"], a["dg"], a["db"], a["ws"], o.get("n", n.value), None)

    for call in (plain, end):
        for k in names[:-1]:
            assert call(**{k: None}) == E.JZ_ERR_NULL, k
        assert call(ws=None) == E.JZ_ERR_WORKSPACE and call(n=n.value - 1) == E.JZ_ERR_WORKSPACE
        assert call(x=D[2] + 2) == E.JZ_ERR_ALIGN and call(dx=D[8] + 8) == E.JZ_ERR_ALIGN
        assert call(dx=D[7]) == E.JZ_ERR_ALIAS and call(dz=D[3]) == E.JZ_ERR_ALIAS and call(db=D[9]) == E.JZ_ERR_ALIAS
        assert call(dz=D[11]) == E.JZ_ERR_ALIAS                        # an output inside the workspace
    assert end(add=D[12] + 2) == E.JZ_ERR_ALIGN and end(add=D[7]) == E.JZ_ERR_ALIAS
    # strided multi-tap backward-data asks for room for its repacked filter; the strided 1x1 form and unit stride do not
    for cs_args, want in (((64, 56, 56, 128, 128, 3, 3, 2, 1), 128 * 9 * 128 * 2), ((64, 56, 56, 256, 128, 1, 1, 2, 0), 0),
                          ((64, 28, 28, 128, 128, 3, 3, 1, 1), 0)):
        d2 = jzlib.conv_desc(*cs_args)
        assert L.jz_conv2d_workspace_bytes(E.JZ_BWD_DATA, ctypes.byref(d2), ctypes.byref(m)) == E.JZ_OK
        assert m.value == want, (cs_args, m.value)
    buf = ctypes.create_string_buffer(256)
    d2 = jzlib.conv_desc(64, 56, 56, 128, 128, 3, 3, 2, 1)
    assert L.jz_conv2d_describe_plan(E.JZ_BWD_DATA, ctypes.byref(d2), buf, 256) == E.JZ_OK and b"parity class" in buf.value
    d2 = jzlib.conv_desc(4, 13, 13, 64, 64, 2, 2, 3, 0)               # a filter smaller than its stride keeps the per-load variant
    assert L.jz_conv2d_describe_plan(E.JZ_BWD_DATA, ctypes.byref(d2), buf, 256) == E.JZ_OK and b"per-load" in buf.value


def test_parity_class_keys_of_the_tuner_match_the_planner(jzlib):
    """tune.py records a strided multi-tap backward-data layer's choice under the GEMM key of every parity class; the
    first class's key must be the GEMM the planner reports for the layer, and with the table built in the three such
    layers of ResNet-50 v1.5 at batch 64 come out with the table's variant, not the cost model's."""
    import re
    from paper_1807_11205_amd import shapes, tune
    strided = [c for c in shapes.resnet50_convs("v1.5") if c.R > 1 and c.stride > 1 and not c.first]
    assert len(strided) == 3
    table = open(os.path.join(os.path.dirname(tune.__file__), "csrc", "jz_tuned_resnet50_v15.inc")).read()
    for cs in strided:
        rec = dict(H=cs.H, C=cs.C, K=cs.K, R=cs.R, stride=cs.stride, pad=cs.pad, batch=64, op="bwd_data")
        keys = tune.class_dims(rec)
        assert len(keys) == 4 and sorted(k[3] for k in keys) == [1, 2, 2, 4]           # a 3x3 stride-2 filter: classes of 1, 2, 2, 4 taps
        d = jzlib.conv_desc(64, cs.H, cs.H, cs.C, cs.K, cs.R, cs.R, cs.stride, cs.pad)
        text = jzlib.jz_conv2d_describe_plan(jzlib.JZ_BWD_DATA, d)
        assert "parity class" in text and ("M %d N %d K %d:" % keys[0][:3]) in text, text
        row = re.search(r"\{1, %d, %d, %d, %d, 1, (\d+), (\d+), (\d+), (\d+), (\d+), 1\}" % keys[0], table)
        assert row, keys[0]
        bm, bn, bk, wv, nst = (int(v) for v in row.groups())
        assert ("tile %dx%dx%d, %d wavefronts, ring %d," % (bm, bn, bk, wv, nst)) in text, text
