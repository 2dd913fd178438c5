"""Helpers shared by the GPU parity tests: move seeded host inputs to the GPU, call libjz through its
binding, bring results back, and compare against the CPU oracle with the stated tolerances."""
import numpy as np
import torch

import oracle
from paper_1807_11205_amd import api, inputs

DEV = "cuda:0"


def to_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def bits(t) -> np.ndarray:
    """fp16 tensor/array -> uint16 bit patterns on the host."""
    if isinstance(t, torch.Tensor):
        t = t.detach().cpu().numpy()
    return np.ascontiguousarray(t).view(np.uint16)


def rel_l2(got: np.ndarray, ref64: np.ndarray) -> float:
    """||got - ref|| / ||ref|| in fp64 (the conv/FC tolerance is 1e-3 on this number)."""
    g = np.asarray(got, dtype=np.float64).ravel()
    r = np.asarray(ref64, dtype=np.float64).ravel()
    den = np.linalg.norm(r)
    return float(np.linalg.norm(g - r) / den) if den > 0 else float(np.linalg.norm(g))


class LarsRun:
    """Device copies of a fused parameter set plus a prepared workspace."""

    def __init__(self, ps: inputs.ParamSet, weight16_init=None):
        self.host = ps
        self.w = to_dev(ps.master_w)
        self.v = to_dev(ps.momentum)
        self.g = to_dev(ps.grad16)
        self.w16 = to_dev(ps.weight16 if weight16_init is None else weight16_init)
        self.flag = torch.full((1,), 7, dtype=torch.int32, device=DEV)
        self.ps = api.ParamSet(ps.offsets, ps.flags, self.w, self.v, self.g, self.w16)
        nbytes = api.jz_lars_workspace_bytes(self.ps)
        self.ws = torch.zeros(max(nbytes, 16), dtype=torch.uint8, device=DEV)
        api.jz_lars_prepare(self.ps, self.ws)

    def step(self, loss_scale=None, **hp):
        kw = dict(inputs.HPARAMS)
        kw.update(hp)
        S = self.host.loss_scale if loss_scale is None else loss_scale
        api.jz_lars_mp_update(self.ps, api.lars_hparams(kw["lr"], kw["momentum"], kw["weight_decay"], kw["trust_coef"], S),
                              self.flag, self.ws)
        torch.cuda.synchronize()
        return self.w.cpu().numpy(), self.v.cpu().numpy(), self.w16.cpu().numpy(), int(self.flag.item())


def check_lars_against_oracle(ps: inputs.ParamSet, got, loss_scale=None, rtol=1e-6, **hp):
    """The LARS parity bar: flag bit-exact; fp32 master weights and momentum within rtol element-wise;
    fp16 write-back == RNE16(own fp32 master) everywhere, and == the oracle's fp16 except where the fp64
    value sits within 2e-6 (relative to the operand scale, see below) of an fp16 rounding midpoint, where the
    neighbouring fp16 value is allowed."""
    kw = dict(inputs.HPARAMS)
    kw.update(hp)
    S = ps.loss_scale if loss_scale is None else loss_scale
    w32, v32, w16, flag = got
    rw, rv, rw16, rflag, info = oracle.lars_mp_update(ps.offsets, ps.flags, ps.master_w, ps.momentum, ps.grad16,
                                                      ps.weight16, loss_scale=S, **kw)
    assert flag == rflag, "overflow flag %d, oracle %d" % (flag, rflag)
    if rflag:
        assert np.array_equal(w32.view(np.uint32), ps.master_w.view(np.uint32)), "skip must leave master weights untouched"
        assert np.array_equal(v32.view(np.uint32), ps.momentum.view(np.uint32)), "skip must leave momentum untouched"
        assert np.array_equal(bits(w16), bits(ps.weight16)), "skip must leave fp16 weights untouched"
        return dict(flag=1)
    w64, v64 = info["w64"], info["v64"]
    ew = np.abs(w32.astype(np.float64) - w64)
    ev = np.abs(v32.astype(np.float64) - v64)
    # Relative to the operand scale: w' = w - (m*v + lr*rho*u) is a three-term sum that can cancel, and an fp32
    # evaluation is only accurate relative to the terms it adds.  Without cancellation (|v'| << |w|, the usual case
    # and all of the ResNet-50 configuration) wscale is |w'| to within 1e-4, i.e. the plain element-wise relative error.
    vscale = info["vmag"]
    wscale = np.abs(ps.master_w.astype(np.float64)) + vscale
    assert np.all(ew <= rtol * wscale + 1e-30), "master weights: max rel err %.3g" % np.max(ew / (wscale + 1e-300))
    assert np.all(ev <= rtol * vscale + 1e-30), "momentum: max rel err %.3g" % np.max(ev / (vscale + 1e-300))
    # (1) the write-back is exactly the rounding of the library's own fp32 master value
    assert np.array_equal(bits(w16), oracle.round_to_half(w32.astype(np.float64))), "w16 != RNE16(w32)"
    # (2) against the oracle's fp16
    diff = np.nonzero(bits(w16) != bits(rw16))[0]
    if diff.size:
        a = w16[diff].astype(np.float64)
        b = rw16[diff].astype(np.float64)
        assert np.array_equal(np.nextafter(w16[diff], rw16[diff]), rw16[diff]), "w16 differs by more than one fp16 step"
        mid = 0.5 * (a + b)
        assert np.all(np.abs(w64[diff] - mid) <= 2e-6 * wscale[diff]), "w16 differs away from a rounding boundary"
    return dict(flag=0, n_boundary=int(diff.size), max_rel_w=float(np.max(ew / (wscale + 1e-300), initial=0.0)),
                max_rel_v=float(np.max(ev / (vscale + 1e-300), initial=0.0)),
                max_rel_w_plain=float(np.max(ew / (np.abs(w64) + 1e-300), initial=0.0)))
