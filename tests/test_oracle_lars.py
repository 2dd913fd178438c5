"""Pins for the fp64 LARS oracle: the closed form of Eq. 1 on constant vectors, invariants
that follow from Eq. 1, the textbook momentum-SGD special case, the skip-on-overflow rule,
and the paper's reason for the fp32 copy (Sections 4.1 and 5.2: the local rate with
eta = 0.001 leaves the fp16 range)."""
import numpy as np
import pytest

from oracle import lars_mp_update, lars_trust_ratio

HP = dict(lr=0.1, momentum=0.9, weight_decay=5e-5, trust_coef=0.001)


def one(w, g16, v=None, flags=3, S=1024.0, **hp):
    w = np.asarray(w, np.float32)
    v = np.zeros_like(w) if v is None else np.asarray(v, np.float32)
    kw = dict(HP, loss_scale=S)
    kw.update(hp)
    return lars_mp_update([0, w.size], [flags], w, v, np.asarray(g16, np.float16), w.astype(np.float16), **kw)


def test_closed_form_on_constant_vectors():
    # w = a*1, g16 = S*b*1, v = 0  =>  rho = eta*a/b ; v' = lr*rho*(b + lam*a) ; w' = a - v'   for every element.
    # The 2-norm of a constant vector is sqrt(n)*|a|, and sqrt(n) cancels in the ratio: no summation code needed.
    n, a, b, S = 64, 0.5, 2.0 ** -6, 1024.0
    w32, v32, w16, inf, info = one(np.full(n, a), np.full(n, S * b, np.float16), S=S)
    eta, lr, lam = HP["trust_coef"], HP["lr"], HP["weight_decay"]
    rho = eta * a / b
    v_exp = lr * rho * (b + lam * a)
    assert inf == 0
    assert abs(info["rho"][0] - rho) <= 1e-15 * rho
    assert np.all(v32 == np.float32(v_exp))
    assert np.all(w32 == np.float32(a - v_exp))
    assert np.all(w16 == np.float32(a - v_exp).astype(np.float16))
    # numbers worked by hand: eta*a/b = 0.001*0.5*64 = 0.032 ; b + lam*a = 0.015625 + 2.5e-5 = 0.01565
    assert abs(v_exp - 0.1 * 0.032 * 0.01565) < 1e-18
    assert abs(float(v32[0]) - 5.008e-5) < 1e-11


def test_step_length_is_lr_eta_norm_w():
    # Eq. 1 with no decay and no momentum: ||w' - w|| = lr * eta * ||w|| whatever the gradient is
    rng = np.random.default_rng(0)
    w = rng.standard_normal(4096).astype(np.float32)
    for gs in (1e-4, 1.0, 20.0):
        g = (rng.standard_normal(4096) * gs).astype(np.float16)
        _, _, _, inf, info = one(w, g, S=1.0, weight_decay=0.0, momentum=0.0)
        step = np.linalg.norm(info["w64"] - w.astype(np.float64))
        assert inf == 0 and abs(step / (0.1 * 0.001 * np.linalg.norm(w.astype(np.float64))) - 1) < 1e-12


def test_loss_scale_invariance_is_bit_exact():
    rng = np.random.default_rng(1)
    w = rng.standard_normal(1000).astype(np.float32)
    v = (rng.standard_normal(1000) * 1e-3).astype(np.float32)
    g = (rng.standard_normal(1000)).astype(np.float16)
    a = one(w, g, v, S=256.0)
    b = one(w, (g.astype(np.float32) * 2).astype(np.float16), v, S=512.0)
    for x, y in zip(a[:3], b[:3]):
        assert np.array_equal(x, y)


def test_gradient_scale_invariance_without_decay():
    rng = np.random.default_rng(2)
    w = rng.standard_normal(512).astype(np.float32)
    g = rng.standard_normal(512).astype(np.float16)
    a = one(w, g, S=1.0, weight_decay=0.0)
    b = one(w, (g.astype(np.float32) * 4).astype(np.float16), S=1.0, weight_decay=0.0)
    np.testing.assert_allclose(a[4]["w64"], b[4]["w64"], rtol=1e-15)
    assert abs(a[4]["rho"][0] / b[4]["rho"][0] - 4.0) < 1e-14


def test_flag_bits():
    rng = np.random.default_rng(3)
    w = rng.standard_normal(256).astype(np.float32)
    v = (rng.standard_normal(256) * 1e-2).astype(np.float32)
    g = (rng.standard_normal(256) * 100).astype(np.float16)
    # decay bit off == run with lambda = 0 (bias / batch-norm tensors, Section 4.2)
    a, b = one(w, g, v, flags=2), one(w, g, v, flags=3, weight_decay=0.0)
    assert all(np.array_equal(x, y) for x, y in zip(a[:3], b[:3]))
    c = one(w, g, v, flags=3)
    assert not np.array_equal(a[0], c[0])
    # LARS bit off == textbook momentum SGD with L2 decay: v' = m v + lr (g + lam w), w' = w - v'
    w32, v32, _, _, info = one(w, g, v, flags=1, S=128.0)
    g64 = g.astype(np.float64) / 128.0
    v_ref = 0.9 * v.astype(np.float64) + 0.1 * (g64 + 5e-5 * w.astype(np.float64))
    assert info["rho"][0] == 1.0
    assert np.array_equal(v32, v_ref.astype(np.float32))
    assert np.array_equal(w32, (w.astype(np.float64) - v_ref).astype(np.float32))


def test_zero_norm_guards():
    g = np.full(64, 3.0, np.float16)
    # ||w|| = 0 (batch-norm beta starts at 0): rho = 1, so the tensor can still move
    w32, v32, _, _, info = one(np.zeros(64), g, S=1.0)
    assert info["rho"][0] == 1.0 and np.all(v32 == np.float32(0.1 * 3.0)) and np.all(w32 == -np.float32(0.1 * 3.0))
    # ||g|| = 0: rho = 1, only decay acts
    w32, v32, _, _, info = one(np.full(64, 2.0), np.zeros(64, np.float16), S=1.0)
    assert info["rho"][0] == 1.0 and np.all(v32 == np.float32(0.1 * 5e-5 * 2.0))


@pytest.mark.parametrize("bad", [np.inf, -np.inf, np.nan])
def test_overflow_skips_everything(bad):
    rng = np.random.default_rng(4)
    off, flags = [0, 64, 200, 264], [3, 2, 3]
    w = rng.standard_normal(264).astype(np.float32)
    v = rng.standard_normal(264).astype(np.float32)
    g = rng.standard_normal(264).astype(np.float16)
    w16_old = rng.standard_normal(264).astype(np.float16)      # deliberately NOT RNE16(w): must come back untouched
    g[137] = bad                                                # in tensor 1; tensors 0 and 2 must be skipped too
    w32, v32, w16, inf, _ = lars_mp_update(off, flags, w, v, g, w16_old, loss_scale=1024.0, **HP)
    assert inf == 1
    assert np.array_equal(w32, w) and np.array_equal(v32, v) and np.array_equal(w16.view(np.uint16), w16_old.view(np.uint16))
    g[137] = 65504.0                                            # largest finite value is not an overflow
    assert lars_mp_update(off, flags, w, v, g, w16_old, loss_scale=1024.0, **HP)[3] == 0


def test_tensors_are_independent_and_use_their_own_norms():
    rng = np.random.default_rng(5)
    sizes = [64, 1000, 8, 333]
    off = np.concatenate([[0], np.cumsum(sizes)])
    w = rng.standard_normal(off[-1]).astype(np.float32)
    v = (rng.standard_normal(off[-1]) * 1e-3).astype(np.float32)
    g = (rng.standard_normal(off[-1]) * np.repeat([1.0, 10.0, 0.1, 3.0], sizes)).astype(np.float16)
    flags = [3, 2, 3, 1]
    full = lars_mp_update(off, flags, w, v, g, w.astype(np.float16), loss_scale=8.0, **HP)
    for t in range(4):
        a, b = off[t], off[t + 1]
        solo = lars_mp_update([0, b - a], [flags[t]], w[a:b], v[a:b], g[a:b], w[a:b].astype(np.float16), loss_scale=8.0, **HP)
        assert np.array_equal(full[0][a:b], solo[0]) and np.array_equal(full[1][a:b], solo[1]) and np.array_equal(full[2][a:b], solo[2])
        rho = lars_trust_ratio(w[a:b], g[a:b], 8.0, 0.001, use_lars=bool(flags[t] & 2))
        assert abs(full[4]["rho"][t] - rho) <= 1e-15 * rho


def test_brute_force_scalar_loop():
    # the same update written element by element with python floats (fp64) and math.fsum for the norms
    import math
    rng = np.random.default_rng(6)
    n, S = 37, 64.0
    w = rng.standard_normal(n).astype(np.float32)
    v = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    g = (rng.standard_normal(n) * S * 0.01).astype(np.float16)
    w32, v32, w16, _, _ = one(w, g, v, S=S)
    nw = math.sqrt(math.fsum(float(a) ** 2 for a in w))
    ng = math.sqrt(math.fsum((float(a) / S) ** 2 for a in g))
    rho = 0.001 * nw / ng
    for i in range(n):
        vi = 0.9 * float(v[i]) + 0.1 * rho * (float(g[i]) / S + 5e-5 * float(w[i]))
        assert v32[i] == np.float32(vi)
        assert w32[i] == np.float32(float(w[i]) - vi)
        assert w16[i] == np.float16(np.float32(float(w[i]) - vi))


def test_fp16_lars_would_stall_but_the_fp32_copy_does_not():
    # Sections 4.1 / 5.2: evaluated in fp16, the local rate of Eq. 1 leaves the format's range and the step vanishes;
    # with the fp32 copies it does not.
    rng = np.random.default_rng(7)
    n = 100_000
    w = (rng.standard_normal(n) * 0.02).astype(np.float32)
    g16 = (rng.standard_normal(n) * 1e-3 * 1024.0).astype(np.float16)      # loss-scaled, O(1) entries
    # (a) the norm in Eq. 1's denominator, accumulated in fp16, overflows (sum of n ~ 1e5 squares of O(1) numbers
    #     exceeds 65504), so an fp16 ratio is eta*||w||/Inf = 0: "the computed learning rate is out of the dynamic range"
    ss = np.float16(0)
    with np.errstate(over="ignore"):
        for chunk in np.array_split(g16, 100):
            ss = np.float16(ss + np.sum(chunk.astype(np.float16) ** 2, dtype=np.float16))
    assert np.isinf(ss) and np.float16(0.001) * np.float16(np.linalg.norm(w)) / np.sqrt(ss) == 0
    w32, v32, w16, inf, info = one(w, g16, S=1024.0)
    assert inf == 0 and np.isfinite(info["rho"][0]) and 0.01 < info["rho"][0] < 0.03   # eta*0.02/1e-3 = 0.02
    # (b) the per-element step lr*rho*g ~ 2e-6 is below half an fp16 ulp of most weights (ulp(0.02) = 2^-16), so
    #     weights kept only in fp16 would not move, while the fp32 master copy accumulates every step
    step16 = v32.astype(np.float16)
    w16_naive = (w.astype(np.float16) - step16).astype(np.float16)
    assert np.count_nonzero(w16_naive != w.astype(np.float16)) < 0.25 * n
    assert np.count_nonzero(w32 != w) > 0.95 * n
    # (c) and for a layer with small weights the step itself is under the 2^-24 threshold the paper quotes
    ws = (w * 1e-2).astype(np.float32)
    _, v32s, _, _, _ = one(ws, g16, S=1024.0)
    assert np.count_nonzero(v32s.astype(np.float16) == 0) > 0.5 * n and np.count_nonzero(v32s) > 0.99 * n


def test_write_back_is_the_rounding_of_the_fp32_master():
    rng = np.random.default_rng(8)
    w = rng.standard_normal(5000).astype(np.float32)
    g = (rng.standard_normal(5000) * 50).astype(np.float16)
    w32, _, w16, _, _ = one(w, g)
    assert np.array_equal(w16, w32.astype(np.float16))
