"""jz_conv2d_bwd_weight_static (backward-weight with its scratch in a fixed array inside the library, for callers
that cannot allocate) against jz_conv2d_bwd_weight through the C ABI: same kernels, so the same bits; and against the
oracle to the conv bar.  Two calls in a row on the shared array, the second with a smaller input."""
import ctypes

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


def both_ways(jz, N, H, C, K, R, stride, pad, key):
    """dw through the workspace entry point and through the static one, raw C ABI calls; returns the two results."""
    import jzt
    c = inputs.conv_case((71, key), N, H, H, C, K, R, R, stride, pad, loss_scale=8.0)
    d = jzt.desc_of(c)
    L = jz.lib()
    x, dy = jzt.to_dev(c.x), jzt.to_dev(c.dy)
    need = jz.jz_conv2d_workspace_bytes(jz.JZ_BWD_WEIGHT, d)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=jzt.DEV)
    ref = torch.full((K * R * R * C,), float("nan"), dtype=torch.float16, device=jzt.DEV)
    got = torch.full((K * R * R * C,), float("nan"), dtype=torch.float16, device=jzt.DEV)
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert L.jz_conv2d_bwd_weight(ctypes.byref(d), x.data_ptr(), dy.data_ptr(), ref.data_ptr(), ws.data_ptr(), ws.numel(), st) == jz.JZ_OK
    assert L.jz_conv2d_bwd_weight_static(ctypes.byref(d), x.data_ptr(), dy.data_ptr(), got.data_ptr(), st) == jz.JZ_OK
    torch.cuda.synchronize()
    return c, need, ref.cpu().numpy(), got.cpu().numpy()


def test_static_scratch_entry_point_matches_the_workspace_one_twice_in_a_row(jz):
    import jzt
    import oracle
    # first a layer whose reduction is split 12 ways (7 MB of partial sums), then a much smaller one that
    # reuses the head of the same array, then the small-channel path (padded copy + partial sums in the array)
    for key, (N, H, C, K, R, stride, pad) in enumerate(((16, 28, 128, 128, 3, 1, 1), (4, 14, 64, 64, 3, 1, 1), (4, 64, 3, 64, 7, 2, 3))):
        c, need, ref, got = both_ways(jz, N, H, C, K, R, stride, pad, key)
        assert need > 0, "the case has to use scratch"
        assert np.array_equal(ref.view(np.uint16), got.view(np.uint16)), "static-scratch result differs from the workspace one"
        od = jzt.odesc_of(c)
        jzt.check_half_output(got, oracle.conv_bwd_weight(od, c.x, c.dy), what="bwd_weight (static scratch)",
                              mag64=oracle.conv_bwd_weight(od, jzt.abs16(c.x), jzt.abs16(c.dy)))


def test_static_scratch_entry_point_rejects_what_does_not_fit_and_checks_arguments(jz):
    import jzt
    L = jz.lib()
    A = 0x10000000
    big = jz.conv_desc(64, 112, 112, 64, 64, 3, 3, 1, 1)          # needs far more than the array holds when split
    need = jz.jz_conv2d_workspace_bytes(jz.JZ_BWD_WEIGHT, big)
    if need <= jz.JZ_STATIC_SCRATCH_BYTES:                        # make it so through the tuning hook: 512 splits
        jz.jz_conv2d_tune_set(jz.JZ_BWD_WEIGHT, big, 64, 64, 32, 4, 4, 512)
        need = jz.jz_conv2d_workspace_bytes(jz.JZ_BWD_WEIGHT, big)
    try:
        assert need > jz.JZ_STATIC_SCRATCH_BYTES
        assert L.jz_conv2d_bwd_weight_static(ctypes.byref(big), A, A + (1 << 30), A + (1 << 31), None) == jz.JZ_ERR_WORKSPACE
    finally:
        jz.jz_conv2d_tune_clear()
    d = jz.conv_desc(2, 8, 8, 64, 64, 3, 3, 1, 1)
    assert L.jz_conv2d_bwd_weight_static(ctypes.byref(d), None, A, A + (1 << 20), None) == jz.JZ_ERR_NULL
    assert L.jz_conv2d_bwd_weight_static(ctypes.byref(d), A + 2, A + (1 << 20), A + (1 << 21), None) == jz.JZ_ERR_ALIGN
    assert L.jz_conv2d_bwd_weight_static(None, A, A + (1 << 20), A + (1 << 21), None) == jz.JZ_ERR_NULL
