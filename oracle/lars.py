"""fp64 oracle of the mixed-precision LARS update -- TEST INFRASTRUCTURE ONLY.

Follows Section 4.1 of Jia et al. 2018: gradients arrive in FP16 (multiplied by
the loss scale S), weights live in an FP32 master copy; both are widened, the
layer-wise adaptive rate of Eq. 1 is applied, and the result is cast back to
FP16 for the next forward pass.  Every step below is in fp64 so that it is the
algorithm itself rather than one particular fp32 evaluation order.

Readings the paper leaves open (each is a convention this oracle *defines*):
  * Eq. 1 is followed literally: rho = eta * ||w|| / ||g||, g = gradient after
    un-scaling, without the weight-decay term in the denominator.
  * Eq. 2 gives E = E0 + (lambda/2) * sum w^2, so dE/dw = g + lambda*w; this is
    what the local rate multiplies (Eq. 3 as typeset would count the decay
    twice).  lambda is applied only to tensors whose flag bit0 is set (bias and
    batch-norm gamma/beta are left unregularised, Section 4.2).
  * Momentum is not in the paper; the usual LARS form is used:
    v <- m*v + lr*rho*(g + lambda*w), w <- w - v.
  * rho = 1 when ||w|| = 0 or ||g|| = 0, or when flag bit1 is clear.
  * Any Inf/NaN in the fp16 gradient buffer (anywhere) skips the whole update.
"""
import numpy as np

FLAG_WEIGHT_DECAY = 1
FLAG_LARS = 2


def _as_f16(a):
    a = np.asarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.float16)
    if a.dtype != np.float16:
        raise TypeError("expected fp16 data (float16 or uint16 bits), got %s" % a.dtype)
    return a


def lars_trust_ratio(w32, g16, loss_scale, trust_coef, use_lars=True):
    """rho of Eq. 1 for one tensor: eta*||w||/||g|| with g = g16/S, fp64."""
    w = np.asarray(w32, dtype=np.float32).astype(np.float64)
    g = _as_f16(g16).astype(np.float64) / float(loss_scale)
    nw = np.sqrt(np.sum(w * w))
    ng = np.sqrt(np.sum(g * g))
    if use_lars and nw > 0.0 and ng > 0.0:
        return float(trust_coef) * nw / ng
    return 1.0


def lars_mp_update(offsets, flags, master_w, momentum_buf, grad16, weight16, *, lr, momentum, weight_decay, trust_coef,
                   loss_scale):
    """One mixed-precision LARS step over a fused flat parameter buffer.

    offsets[T+1] are element offsets of the T tensors, flags[T] the per-tensor
    bits.  Returns (w32', v32', w16', found_inf, info); inputs are not modified.
    w16' is RNE16 of the *fp32* master value (the cast-back of Section 4.1).
    info holds the fp64 pre-rounding weights and the per-tensor rho for tests.
    """
    offsets = np.asarray(offsets, dtype=np.int64)
    flags = np.asarray(flags, dtype=np.uint8)
    T = len(flags)
    assert len(offsets) == T + 1 and offsets[0] == 0
    w_in = np.asarray(master_w, dtype=np.float32)
    v_in = np.asarray(momentum_buf, dtype=np.float32)
    g_in = _as_f16(grad16)
    w16_in = _as_f16(weight16)
    P = int(offsets[-1])
    assert w_in.size == P and v_in.size == P and g_in.size == P and w16_in.size == P

    g_all = g_in.astype(np.float64)
    found_inf = int(not np.all(np.isfinite(g_all)))
    if found_inf:  # overflow under loss scaling: leave every state buffer as it was
        return w_in.copy(), v_in.copy(), w16_in.copy(), 1, {"rho": None, "w64": None}

    S = float(loss_scale)
    w64_out = np.empty(P, np.float64)
    v64_out = np.empty(P, np.float64)
    vmag = np.empty(P, np.float64)      # |m*v| + lr*rho*(|g| + |lam*w|): operand scale of v', for error bounds under cancellation
    rho = np.empty(T, np.float64)
    for t in range(T):
        a, b = int(offsets[t]), int(offsets[t + 1])
        w = w_in[a:b].astype(np.float64)
        v = v_in[a:b].astype(np.float64)
        g = g_all[a:b] / S                              # un-scale
        nw = np.sqrt(np.sum(w * w))
        ng = np.sqrt(np.sum(g * g))
        if (flags[t] & FLAG_LARS) and nw > 0.0 and ng > 0.0:
            rho[t] = float(trust_coef) * nw / ng        # Eq. 1 local rate
        else:
            rho[t] = 1.0
        lam = float(weight_decay) if (flags[t] & FLAG_WEIGHT_DECAY) else 0.0
        u = g + lam * w                                 # Eq. 2 differentiated
        v_new = float(momentum) * v + float(lr) * rho[t] * u
        w64_out[a:b] = w - v_new
        v64_out[a:b] = v_new
        vmag[a:b] = np.abs(float(momentum) * v) + np.abs(float(lr) * rho[t]) * (np.abs(g) + np.abs(lam * w))
    w32_out = w64_out.astype(np.float32)                # RNE to the fp32 master copy
    v32_out = v64_out.astype(np.float32)
    w16_out = w32_out.astype(np.float16)                # cast back from the fp32 value
    return w32_out, v32_out, w16_out, 0, {"rho": rho, "w64": w64_out, "v64": v64_out, "vmag": vmag}
