"""Pins of the loss-scale controller oracle: hand-worked trajectories and the clamps.  The policy itself is a
convention (the paper names loss scaling in Sections 4.1 and 5.3 but no policy); what is pinned is that the oracle
implements the policy its header states.  No GPU."""
import oracle


def _run(scale, flags, **kw):
    good, out = 0, []
    for f in flags:
        scale, good = oracle.loss_scale_step(scale, good, f, **kw)
        out.append((scale, good))
    return out


def test_hand_worked_trajectory():
    # interval 3: clean, clean, clean -> grow; overflow -> halve and restart the count; two clean; overflow; three clean
    got = _run(1024.0, [0, 0, 0, 1, 0, 0, 1, 0, 0, 0], growth_interval=3)
    want = [(1024.0, 1), (1024.0, 2), (2048.0, 0), (1024.0, 0), (1024.0, 1), (1024.0, 2), (512.0, 0), (512.0, 1), (512.0, 2),
            (1024.0, 0)]
    assert got == want


def test_clamps_and_other_factors():
    assert _run(2.0, [1, 1, 1], min_scale=1.0) == [(1.0, 0), (1.0, 0), (1.0, 0)]
    assert _run(32768.0, [0, 0, 0], growth_interval=1, max_scale=65536.0) == [(65536.0, 0), (65536.0, 0), (65536.0, 0)]
    # growth 4, backoff 1/4, interval 2
    assert _run(16.0, [0, 0, 1, 0, 0], growth_factor=4.0, backoff_factor=0.25, growth_interval=2) == \
        [(16.0, 1), (64.0, 0), (16.0, 0), (16.0, 1), (64.0, 0)]


def test_back_off_reaches_the_scale_the_bench_uses():
    # the benchmark's gradients overflow at S = 1024 and first fit FP16 at S = 16: six halvings
    scale, good = 1024.0, 0
    for s in (1024, 512, 256, 128, 64, 32):
        assert scale == s
        scale, good = oracle.loss_scale_step(scale, good, 1)
    assert (scale, good) == (16.0, 0)
    assert oracle.loss_scale_step(scale, good, 0) == (16.0, 1)
