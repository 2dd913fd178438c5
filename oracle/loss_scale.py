"""Oracle of the dynamic loss-scale controller -- TEST INFRASTRUCTURE ONLY.

Section 4.1 of Jia et al. 2018 keeps small gradients representable in FP16 by multiplying the loss by a scale S before
the backward pass and dividing the gradients by S before the update; Section 5.3 says this is required at large batch
sizes but gives neither a value nor a policy.  The controller here is the usual one for such training (skip the step
and shrink S when a gradient overflowed, grow S again after a run of clean steps); every constant is a parameter:

    overflow seen:   S <- max(S * backoff_factor, min_scale),  good_steps <- 0        (the LARS update was skipped)
    otherwise:       good_steps <- good_steps + 1;
                     if good_steps >= growth_interval:  S <- min(S * growth_factor, max_scale),  good_steps <- 0

S is held in FP32 (the products are formed in FP32, as the kernel does; with factors 2 and 1/2 they are exact).  These
are conventions this oracle defines: the paper fixes none of them.
"""
import numpy as np


def loss_scale_step(scale, good_steps, found_inf, *, growth_factor=2.0, backoff_factor=0.5, growth_interval=2000,
                    min_scale=1.0, max_scale=65536.0):
    """One controller step; returns (scale', good_steps')."""
    s = np.float32(scale)
    if found_inf:
        s = np.float32(s * np.float32(backoff_factor))
        return float(max(s, np.float32(min_scale))), 0
    good = int(good_steps) + 1
    if good >= int(growth_interval):
        s = np.float32(s * np.float32(growth_factor))
        return float(min(s, np.float32(max_scale))), 0
    return float(s), good
