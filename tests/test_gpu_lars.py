"""GPU parity of jz_lars_mp_update (through the C ABI) against the fp64 oracle."""
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


@pytest.fixture(autouse=True, params=["three_launches", "presummed"])
def lars_path(request):
    """Every test of this module runs on both update paths (see jzt.LARS_PATH)."""
    import jzt
    old, jzt.LARS_PATH = jzt.LARS_PATH, request.param
    yield request.param
    jzt.LARS_PATH = old


def run_and_check(ps, plain_rtol=None, plain_floor=0.0, **hp):
    import jzt
    r = jzt.LarsRun(ps)
    got = r.step(**hp)
    return jzt.check_lars_against_oracle(ps, got, plain_rtol=plain_rtol, plain_floor=plain_floor, **hp)


def test_config0_sized_single_tensor(jz):
    # one 3x3x16x16 filter (2,304 parameters), He-normal, grads of order S
    ps = inputs.random_param_set((0, 1), [2304], loss_scale=1024.0, grad_std=0.02)
    out = run_and_check(ps, plain_rtol=1e-6)
    assert out["flag"] == 0


@pytest.mark.parametrize("sizes", [
    [64, 4096, 8, 4104, 8192, 12296],                 # chunk-size multiples and one-vector tails
    [1, 7, 13, 4097, 3, 8191, 5, 100003],             # ragged: nothing aligned to 8
    [0, 64, 0, 0, 256, 0],                            # empty tensors between real ones
    [300000],                                         # one tensor spanning many chunks
])
def test_ragged_and_multi_tensor(jz, sizes):
    n = len(sizes)
    flags = [(3, 2, 1, 0)[i % 4] for i in range(n)]
    ps = inputs.random_param_set((0, 2, n, sum(sizes) % 1000), sizes, loss_scale=128.0, grad_std=3e-3, flags=flags,
                                 momentum_std=1e-3)
    out = run_and_check(ps)
    assert out["flag"] == 0


def test_empty_parameter_set(jz):
    import jzt
    ps = inputs.random_param_set((0, 3), [])
    r = jzt.LarsRun(ps)
    w, v, w16, flag = r.step()
    assert flag == 0 and w.size == 0
    ps = inputs.random_param_set((0, 3), [0, 0])
    assert jzt.LarsRun(ps).step()[3] == 0


@pytest.mark.parametrize("bad,where", [(np.inf, 0), (-np.inf, -1), (np.nan, 5000), (np.inf, 4095), (np.nan, 4096)])
def test_overflow_flag_skips_the_whole_update(jz, bad, where):
    import jzt
    ps = inputs.random_param_set((0, 4), [4096, 64, 9000, 777], loss_scale=1024.0, momentum_std=1e-3)
    ps.grad16[where] = np.float16(bad)
    # stale fp16 weights that are NOT the rounding of the master copy: a skipped step must not refresh them
    stale = inputs.normal_f16(inputs.rng_for(0, 44), (ps.P,))
    ps.weight16 = stale
    got = jzt.LarsRun(ps).step()
    out = jzt.check_lars_against_oracle(ps, got)
    assert out["flag"] == 1


def test_largest_finite_gradient_is_not_an_overflow(jz):
    ps = inputs.random_param_set((0, 5), [1024, 64])
    ps.grad16[17] = np.float16(65504.0)
    ps.grad16[1030] = np.float16(-65504.0)
    assert run_and_check(ps)["flag"] == 0


def test_zero_norm_guards(jz):
    # beta = 0 tensor (||w|| = 0) and a tensor with zero gradient (||g|| = 0): rho falls back to 1
    ps = inputs.random_param_set((0, 6), [256, 512, 64], loss_scale=64.0)
    ps.master_w[0:256] = 0.0
    ps.weight16[0:256] = 0.0
    ps.grad16[256:768] = 0.0
    assert run_and_check(ps)["flag"] == 0


def test_flag_bits_and_hyper_parameters(jz):
    ps = inputs.random_param_set((0, 7), [4096 * 3 + 40, 1000], loss_scale=256.0, flags=[1, 2], momentum_std=1e-2)
    run_and_check(ps, lr=3.2, momentum=0.5, weight_decay=1e-4, trust_coef=0.01)
    run_and_check(ps, momentum=0.0, weight_decay=0.0)


def test_loss_scale_not_a_power_of_two(jz):
    ps = inputs.random_param_set((0, 8), [5000, 64], loss_scale=1000.0)
    run_and_check(ps)   # 1/S is rounded to fp32 once on the host: still inside 1e-6


def test_loss_scale_invariance_is_bit_exact_on_the_gpu(jz):
    import jzt
    ps = inputs.random_param_set((0, 9), [10000, 64], loss_scale=256.0, grad_std=1e-3, momentum_std=1e-3)
    a = jzt.LarsRun(ps).step()
    ps2 = inputs.random_param_set((0, 9), [10000, 64], loss_scale=256.0, grad_std=1e-3, momentum_std=1e-3)
    ps2.grad16 = (ps.grad16.astype(np.float32) * 2).astype(np.float16)
    ps2.loss_scale = 512.0
    b = jzt.LarsRun(ps2).step()
    for x, y in zip(a[:3], b[:3]):
        assert np.array_equal(x, y)


def test_three_steps_with_momentum(jz):
    import jzt
    ps = inputs.random_param_set((0, 10), [70000, 64, 64], loss_scale=1024.0, flags=[3, 2, 2])
    r = jzt.LarsRun(ps)
    for step in range(3):
        g = inputs.normal_f16(inputs.rng_for(0, 10, step), (ps.P,), std=1e-3 * 1024.0)
        ps.grad16 = g
        r.g.copy_(torch.from_numpy(g))
        got = r.step()
        jzt.check_lars_against_oracle(ps, got)
        # next step starts from the library's own state
        ps.master_w, ps.momentum, ps.weight16 = got[0].copy(), got[1].copy(), got[2].copy()
    assert np.count_nonzero(ps.momentum) > 0.99 * ps.P


def test_carried_weight_norms_match_recomputed_ones_bit_for_bit(jz):
    # The workspace carries sum(w^2) per tensor from one update to the next.  A run that re-prepares its workspace
    # before every update (so that the norms are recomputed from the weights) must give identical bits, also across
    # a skipped step (Inf in the gradient: nothing may change, and the carried sums must still be right afterwards).
    import jzt
    ps = inputs.random_param_set((0, 13), [70000, 64, 9000, 64], loss_scale=1024.0, flags=[3, 2, 3, 2], momentum_std=1e-3)
    a, b = jzt.LarsRun(ps), jzt.LarsRun(ps)
    for step in range(4):
        g = inputs.normal_f16(inputs.rng_for(0, 13, step), (ps.P,), std=1e-3 * 1024.0)
        if step == 1:
            g[12345] = np.float16(np.inf)
        for r in (a, b):
            r.g.copy_(torch.from_numpy(g))
        jz.jz_lars_prepare(b.ps, b.ws)
        ga, gb = a.step(), b.step()
        assert ga[3] == gb[3] == (1 if step == 1 else 0)
        for x, y in zip(ga[:3], gb[:3]):
            assert np.array_equal(x.view(np.uint8), y.view(np.uint8)), "step %d" % step
        ps.grad16 = g
        jzt.check_lars_against_oracle(ps, ga)
        ps.master_w, ps.momentum, ps.weight16 = ga[0].copy(), ga[1].copy(), ga[2].copy()


def test_prepare_again_after_an_outside_write_of_the_master_weights(jz):
    import jzt
    ps = inputs.random_param_set((0, 14), [50000, 64], loss_scale=1024.0, flags=[3, 2])
    r = jzt.LarsRun(ps)
    got = r.step()
    jzt.check_lars_against_oracle(ps, got)
    # restore different weights from outside, as a checkpoint load would, then prepare again as the header demands
    ps2 = inputs.random_param_set((0, 15), [50000, 64], loss_scale=1024.0, flags=[3, 2])
    r.w.copy_(torch.from_numpy(ps2.master_w)); r.v.copy_(torch.from_numpy(ps2.momentum))
    r.g.copy_(torch.from_numpy(ps2.grad16)); r.w16.copy_(torch.from_numpy(ps2.weight16))
    jz.jz_lars_prepare(r.ps, r.ws)
    jzt.check_lars_against_oracle(ps2, r.step())


def test_same_inputs_give_identical_bits(jz):
    import jzt
    ps = inputs.random_param_set((0, 11), [123457, 64, 2048], momentum_std=1e-3)
    a = jzt.LarsRun(ps).step()
    b = jzt.LarsRun(ps).step()
    for x, y in zip(a[:3], b[:3]):
        assert np.array_equal(x.view(np.uint8), y.view(np.uint8))


def test_resnet50_parameter_set_full_size(jz):
    # 161 tensors, 25,557,032 parameters, the configuration the LARS bandwidth figure is quoted on
    ps = inputs.resnet50_param_set(loss_scale=1024.0, grad_std=1e-3)
    assert ps.T == 161 and ps.P == 25557032
    # the stated bar, literally: |w32 - w64| <= 1e-6 |w64|, for every parameter that the step does not cancel (among 25.6 M
    # He-normal weights a few dozen are as small as their own update; those are held to the operand-scale bound)
    out = run_and_check(ps, plain_rtol=1e-6, plain_floor=0.1)
    assert out["flag"] == 0
    print("boundary-band fp16 elements: %d of %d; max rel err w %.2e v %.2e" % (out["n_boundary"], ps.P, out["max_rel_w"], out["max_rel_v"]))


def test_resnet50_parameter_set_with_injected_inf(jz):
    ps = inputs.resnet50_param_set(loss_scale=1024.0, grad_std=1e-3, inject_inf=True)
    assert ps.inf_index is not None
    assert run_and_check(ps)["flag"] == 1


def test_argument_errors(jz):
    import jzt
    api = jz
    ps = inputs.random_param_set((0, 12), [4096, 64])
    r = jzt.LarsRun(ps)
    hp = api.lars_hparams(0.1, 0.9, 5e-5, 0.001, 1024.0)
    other = torch.zeros(r.ws.numel() + 256, dtype=torch.uint8, device=jzt.DEV)
    with pytest.raises(api.JzError) as e:       # workspace never prepared
        api.jz_lars_mp_update(r.ps, hp, r.flag, other[:r.ws.numel()])
    assert e.value.status == api.JZ_ERR_NOT_PREPARED
    with pytest.raises(api.JzError) as e:       # too small
        api.jz_lars_mp_update(r.ps, hp, r.flag, r.ws[:64])
    assert e.value.status == api.JZ_ERR_WORKSPACE
    with pytest.raises(api.JzError) as e:       # loss scale must be positive
        api.jz_lars_mp_update(r.ps, api.lars_hparams(0.1, 0.9, 5e-5, 0.001, 0.0), r.flag, r.ws)
    assert e.value.status == api.JZ_ERR_SHAPE
    bad = api.ParamSet(ps.offsets, ps.flags, r.w, r.v, r.g, r.g)   # fp16 output aliases the gradient input
    with pytest.raises(api.JzError) as e:
        api.jz_lars_mp_update(bad, hp, r.flag, r.ws)
    assert e.value.status == api.JZ_ERR_ALIAS
    wmis = torch.zeros(ps.P + 4, dtype=torch.float32, device=jzt.DEV)[1:ps.P + 1]
    with pytest.raises(api.JzError) as e:
        api.jz_lars_mp_update(api.ParamSet(ps.offsets, ps.flags, wmis, r.v, r.g, r.w16), hp, r.flag, r.ws)
    assert e.value.status == api.JZ_ERR_ALIGN
    # a different table with the same workspace is refused
    ps_b = inputs.random_param_set((0, 12), [4096, 64])
    ps_b.flags = np.array([3, 2], np.uint8)
    rb = api.ParamSet(ps_b.offsets, ps_b.flags, r.w, r.v, r.g, r.w16)
    with pytest.raises(api.JzError) as e:
        api.jz_lars_mp_update(rb, hp, r.flag, r.ws)
    assert e.value.status == api.JZ_ERR_NOT_PREPARED
    torch.cuda.synchronize()
