"""Helpers shared by the GPU parity tests: move seeded host inputs to the GPU, call libjz through its
binding, bring results back, and compare against the CPU oracle with the stated tolerances."""
from contextlib import contextmanager

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


def exact_units(g16: np.ndarray) -> int:
    """sum of squares of finite fp16 values as an exact integer count of units of 2^-48 (every fp16 value is an integer
    multiple of 2^-24, below 2^40 of them): k = value * 2^24 is exact in fp64 and in int64; k^2 is split as
    (hi 2^20 + lo)^2 so that every partial sum stays inside int64, and the three sums are combined as Python integers."""
    k = np.abs(np.rint(g16.astype(np.float64).ravel() * 2.0 ** 24)).astype(np.int64)
    hi, lo = k >> 20, k & 0xFFFFF
    total = 0
    for s in range(0, k.size, 1 << 20):     # 2^20 elements per slice: hi * hi < 2^40, so a slice's sum < 2^61
        h, l = hi[s:s + (1 << 20)], lo[s:s + (1 << 20)]
        total += (int(np.sum(h * h)) << 40) + (int(np.sum(2 * h * l)) << 20) + int(np.sum(l * l))
    return total


def sink_units(ps, ws, tensor) -> int:
    """What the sink of `tensor` inside a LARS workspace holds (exact integer units of 2^-48) and its non-finite flag."""
    sink = api.jz_lars_sumsq_sink(ps, ws, tensor)
    base, fl = sink.sums - ws.data_ptr(), sink.nonfinite - ws.data_ptr()
    return api.sumsq_sink_units(ws[base:base + api.JZ_SUMSQ_SINK_BYTES].view(torch.int64)), int(ws[fl:fl + 4].view(torch.int32).item())


# which update LarsRun.step runs: "three_launches" (jz_lars_mp_update) or "presummed" (jz_lars_begin_step, jz_lars_grad_sumsq
# over every tensor, jz_lars_mp_update_presummed); the LARS test modules run every test both ways
LARS_PATH = "three_launches"


class LarsRun:
    """Device copies of a fused parameter set plus a prepared workspace."""

    def __init__(self, ps: inputs.ParamSet, weight16_init=None, path=None):
        self.path = LARS_PATH if path is None else path
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
        hpc = api.lars_hparams(kw["lr"], kw["momentum"], kw["weight_decay"], kw["trust_coef"], S)
        if self.path == "presummed":
            api.jz_lars_begin_step(self.ps, self.ws)
            api.jz_lars_grad_sumsq(self.ps, 0, self.ps.T, self.ws)
            api.jz_lars_mp_update_presummed(self.ps, hpc, self.flag, self.ws)
        else:
            api.jz_lars_mp_update(self.ps, hpc, self.flag, self.ws)
        torch.cuda.synchronize()
        return self.w.cpu().numpy(), self.v.cpu().numpy(), self.w16.cpu().numpy(), int(self.flag.item())


def check_lars_against_oracle(ps: inputs.ParamSet, got, loss_scale=None, rtol=1e-6, plain_rtol=None, plain_floor=0.0, **hp):
    """The LARS parity bar: flag bit-exact; fp32 master weights and momentum within rtol element-wise;
    fp16 write-back == RNE16(own fp32 master) everywhere, and == the oracle's fp16 except where the fp64
    value sits within 2e-6 (relative to the operand scale, see below) of an fp16 rounding midpoint, where the
    neighbouring fp16 value is allowed.  plain_rtol: also assert the plain element-wise relative error
    |w32 - w64| <= plain_rtol * |w64| (the stated 1e-6) on every element whose new value is at least plain_floor times
    its operand scale (0: every element; a real training step has a few weights that the update happens to cancel, and
    the one fp32 rounding of w - v, 6e-8 of the larger operand, is only within 1e-6 of a difference that is not more
    than about ten times smaller than the operands: hence a floor of 0.1 there)."""
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
    keep = np.abs(w64) >= plain_floor * wscale
    plain = float(np.max((ew / (np.abs(w64) + 1e-300))[keep], initial=0.0))
    if plain_rtol is not None:
        assert plain <= plain_rtol, "master weights: plain relative error %.3g > %.1g" % (plain, plain_rtol)
        assert np.count_nonzero(~keep) <= 1e-3 * keep.size, "too many cancelled weights left out of the plain bound"
    return dict(flag=0, n_boundary=int(diff.size), max_rel_w=float(np.max(ew / (wscale + 1e-300), initial=0.0)),
                max_rel_v=float(np.max(ev / (vscale + 1e-300), initial=0.0)), max_rel_w_plain=plain)


# ---------------------------------------------------------------------------------------------
# convolution / fully connected
# ---------------------------------------------------------------------------------------------
def _ws_tensor(nbytes):
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=DEV) if nbytes else None


def desc_of(c) -> "api.jz_conv_desc":
    return api.conv_desc(c.N, c.H, c.W, c.C, c.K, c.R, c.S, c.stride, c.pad)


def odesc_of(c):
    return oracle.conv_desc(c.N, c.H, c.W, c.C, c.K, c.R, c.S, c.stride, c.pad)


def run_conv(op, d, a: np.ndarray, b: np.ndarray, out_shape):
    """Call one conv entry point through the C ABI; a, b are the two fp16 inputs in the order the entry point takes."""
    ta, tb = to_dev(a), to_dev(b)
    out = torch.full(out_shape, float("nan"), dtype=torch.float16, device=DEV)   # poison: every element must be written
    ws = _ws_tensor(api.jz_conv2d_workspace_bytes(op, d))
    fn = {api.JZ_FWD: api.jz_conv2d_fwd, api.JZ_BWD_DATA: api.jz_conv2d_bwd_data, api.JZ_BWD_WEIGHT: api.jz_conv2d_bwd_weight}[op]
    fn(d, ta, tb, out, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def run_fc(mode, B, I, O, a, b, out_shape):
    ta, tb = to_dev(a), to_dev(b)
    out = torch.full(out_shape, float("nan"), dtype=torch.float16, device=DEV)
    ws = _ws_tensor(api.jz_gemm_fc_workspace_bytes(mode, B, I, O))
    api.jz_gemm_fc(mode, B, I, O, ta, tb, out, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@contextmanager
def forced_variant(d, tile_m, tile_n, k_tile, wavefronts, ring, splits=1, ops=(api.JZ_FWD, api.JZ_BWD_DATA, api.JZ_BWD_WEIGHT)):
    """Make the planner run one kernel variant for the ops of layer `d` (jz_conv2d_tune_set), whatever it would have
    picked; splits: one number or {op: number}.  Everything recorded is forgotten on exit."""
    try:
        for op in ops:
            sp = splits.get(op, 1) if isinstance(splits, dict) else splits
            api.jz_conv2d_tune_set(op, d, tile_m, tile_n, k_tile, wavefronts, ring, sp)
            want = "tile %dx%dx%d, %d wavefronts, ring %d" % (tile_m, tile_n, k_tile, wavefronts, ring)
            plan = api.jz_conv2d_describe_plan(op, d)
            assert want in plan, (want, plan)
        yield
    finally:
        api.jz_conv2d_tune_clear()


FP16_OVERFLOW = 65520.0      # |v| >= this rounds to +-Inf


ELEMENT_C = 8.0               # per-element bound: multiples of 2^-24 * sum|terms| allowed for fp32 accumulation


def abs16(a: np.ndarray) -> np.ndarray:
    """|a| of fp16 data as bit patterns (sign bit cleared): the oracle run on these gives sum |term| per output."""
    return np.ascontiguousarray(a).view(np.uint16) & np.uint16(0x7FFF)


def check_half_output(got16: np.ndarray, ref64: np.ndarray, tol=1e-3, what="", mag64=None):
    """The conv/FC parity bar: relative L2 error <= tol against the fp64 oracle over every entry that is finite in
    the oracle's fp16 rounding, and the +-Inf pattern of fp16 overflow must match exactly, except for entries whose
    exact magnitude lies within 2^-10 (relative) of the overflow threshold 65520, where fp32 accumulation order may
    legitimately tip the rounding either way (such an entry must then be +-Inf or within 2^-9 of the exact value).

    mag64 (the oracle evaluated on |inputs|: sum of |term| for every output) adds a bound on EVERY finite element:
      |got - ref| <= 2^-10 |ref| + ELEMENT_C 2^-24 mag + 2^-24
    one fp16 rounding (2^-11, doubled for a second rounding at an fp32 / fp16 midpoint), fp32 accumulation in any
    order (each of the K - 1 additions errs by at most 2^-24 of a partial sum that is at most mag; as a random walk that
    is about 0.6 * 2^-24 * mag in total, ELEMENT_C leaves six standard deviations), and the spacing of fp16 subnormals."""
    got = np.asarray(got16).astype(np.float64).ravel()
    ref = np.asarray(ref64, dtype=np.float64).ravel()
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert not np.any(np.isnan(got)) or np.any(np.isnan(ref)), what + ": NaN in output (element never written?)"
    mag = np.abs(ref)
    band = np.abs(mag - FP16_OVERFLOW) <= FP16_OVERFLOW * 2.0 ** -10
    ref_inf = mag >= FP16_OVERFLOW
    got_inf = np.isinf(got)
    strict = ~band
    assert np.array_equal(got_inf[strict], ref_inf[strict]), what + ": fp16 overflow pattern differs"
    assert np.all(np.sign(got[ref_inf & strict]) == np.sign(ref[ref_inf & strict])), what + ": sign of overflow"
    if np.any(band):
        ok = got_inf[band] | (np.abs(got[band] - ref[band]) <= 2.0 ** -9 * mag[band])
        assert np.all(ok), what + ": near-threshold entry is neither Inf nor the neighbouring finite value"
    fin = ~ref_inf & ~got_inf
    err = rel_l2(got[fin], ref[fin]) if np.any(fin) else 0.0
    assert err <= tol, "%s: relative L2 error %.3e > %.1e" % (what, err, tol)
    worst = 0.0
    if mag64 is not None:
        mag_t = np.asarray(mag64, dtype=np.float64).ravel()
        assert mag_t.shape == ref.shape
        bound = 2.0 ** -10 * mag[fin] + ELEMENT_C * 2.0 ** -24 * mag_t[fin] + 2.0 ** -24
        ratio = np.abs(got[fin] - ref[fin]) / bound
        worst = float(np.max(ratio, initial=0.0))
        bad = np.nonzero(ratio > 1.0)[0]
        assert bad.size == 0, "%s: %d elements beyond the per-element bound, worst %.2f x at finite index %d (got %r, ref %r)" % (
            what, bad.size, worst, int(bad[0]), got[fin][bad[0]], ref[fin][bad[0]])
    return dict(rel_l2=err, n_inf=int(np.count_nonzero(ref_inf)), n_band=int(np.count_nonzero(band)), worst_elem=worst)


def conv_all_ops_full(case, tol=1e-3, ops=(0, 1, 2)):
    """fwd / bwd_data / bwd_weight of one layer against the full-tensor oracle."""
    d, od = desc_of(case), odesc_of(case)
    res = {}
    ax, aw, ady = abs16(case.x), abs16(case.w16), abs16(case.dy)
    if api.JZ_FWD in ops:
        y = run_conv(api.JZ_FWD, d, case.x, case.w16, (case.N, case.P, case.Q, case.K))
        res["fwd"] = check_half_output(y, oracle.conv_fwd(od, case.x, case.w16), tol, "fwd", oracle.conv_fwd(od, ax, aw))
    if api.JZ_BWD_DATA in ops:
        dx = run_conv(api.JZ_BWD_DATA, d, case.dy, case.w16, (case.N, case.H, case.W, case.C))
        res["bwd_data"] = check_half_output(dx, oracle.conv_bwd_data(od, case.dy, case.w16), tol, "bwd_data",
                                            oracle.conv_bwd_data(od, ady, aw))
    if api.JZ_BWD_WEIGHT in ops:
        dw = run_conv(api.JZ_BWD_WEIGHT, d, case.x, case.dy, (case.K, case.R, case.S, case.C))
        res["bwd_weight"] = check_half_output(dw, oracle.conv_bwd_weight(od, case.x, case.dy), tol, "bwd_weight",
                                              oracle.conv_bwd_weight(od, ax, ady))
    return res


def plan_tiles(op, d):
    """(tile_m, tile_n, tiles_m, tiles_n, splits, scatter) of the plan the library would run for `op` on `d`."""
    import re
    text = api.jz_conv2d_describe_plan(op, d)
    m = re.search(r"patch kernel, (\d+) pixels x (\d+) channels per block, (\d+) blocks per image", text)
    if m:   # blocks of consecutive pixels that never straddle an image: ("patch", pixels per block, channels, blocks per image)
        return ("patch",) + tuple(int(v) for v in m.groups())
    m = re.search(r"tile (\d+)x(\d+)x\d+, \d+ wavefronts, ring \d+, (\d+) x (\d+) tiles, (\d+) splits", text)
    assert m, text
    if "parity class" in text:   # strided multi-tap backward-data: one launch per class, the text shows the first class's tiles
        return ("classes", int(m.group(1)), int(m.group(2)))
    return tuple(int(v) for v in m.groups()) + ("scatter epilogue" in text,)


def class_edge_pixels(case, bm, max_tiles_per_class=384):
    """Flat input-pixel indices (n, h, w) at the first and last row of the row tiles of every parity class of a strided
    multi-tap backward-data layer: class (ca, cb) holds the pixels h = ca + s i, w = cb + s l in (n, i, l) order."""
    s_h = s_w = case.stride
    rows = set()
    for ca in range(s_h):
        for cb in range(s_w):
            ha, wb = -(-(case.H - ca) // s_h), -(-(case.W - cb) // s_w)
            mc = case.N * ha * wb
            if mc <= 0:
                continue
            tm = -(-mc // bm)
            tiles = range(tm) if tm <= max_tiles_per_class else np.unique(np.linspace(0, tm - 1, max_tiles_per_class).astype(int))
            for t in tiles:
                for j in (int(t) * bm, min((int(t) + 1) * bm, mc) - 1):
                    n, rem = divmod(j, ha * wb)
                    i, l = divmod(rem, wb)
                    rows.add((n * case.H + ca + s_h * i) * case.W + cb + s_w * l)
    return np.asarray(sorted(rows), np.int64)


def structured_rows_cols(M, N, plan, max_row_tiles=1536, pq=None):
    """Rows and columns of the GEMM output where a tiling bug would show: the first and last row of (up to max_row_tiles,
    evenly spaced, always the first and last two) row tiles, of the row tiles at which one XCD's run of consecutive
    workgroups ends and the next begins, and the first and last column of every column tile (ragged last tiles
    included by construction)."""
    if plan[0] == "patch":
        # the forward kernel of small-channel layers: the first and last pixel of (up to max_row_tiles, evenly spaced) blocks,
        # among them every image's ragged last block; the first and last channel of every 32-channel tile
        _, mb, k, bpi = plan
        assert k == N and M % pq == 0 and bpi == -(-pq // mb), (M, N, pq, plan)
        nblk = (M // pq) * bpi
        blocks = set(range(nblk)) if nblk <= max_row_tiles else set(np.linspace(0, nblk - 1, max_row_tiles).astype(int).tolist()) | {bpi - 1, nblk - bpi}
        rows = sorted({r for b in blocks for r in ((b // bpi) * pq + (b % bpi) * mb, (b // bpi) * pq + min((b % bpi + 1) * mb, pq) - 1)})
        cols = sorted({c for t in range(N // 32) for c in (t * 32, t * 32 + 31)})
        return np.asarray(rows, np.int64), np.asarray(cols, np.int64)
    bm, bn, tm, tn, splits, _ = plan
    assert tm == -(-M // bm) and tn == -(-N // bn), (M, N, plan)
    tiles = set(range(tm)) if tm <= max_row_tiles else set(np.linspace(0, tm - 1, max_row_tiles).astype(int).tolist()) | {1, tm - 2}
    grid = tm * tn * splits
    q, rem = divmod(grid, 8)
    for x in range(1, 8):                                 # first workgroup of XCD x's run and the one before it
        for L in (x * q + min(x, rem), x * q + min(x, rem) - 1):
            if 0 <= L < grid:
                tiles.add((L % (tm * tn)) // tn)
    rows = sorted({r for t in tiles for r in (t * bm, min((t + 1) * bm, M) - 1)})
    cols = sorted({c for t in range(tn) for c in (t * bn, min((t + 1) * bn, N) - 1)})
    return np.asarray(rows, np.int64), np.asarray(cols, np.int64)


def conv_all_ops_sampled(case, n_fwd=65536, n_bwd_data=65536, seed=0, tol=1e-3, skip_bwd_data=False):
    """Full-size layer in the launch configuration the planner picks for it: the GPU computes whole tensors; for the
    forward and backward-data outputs the oracle computes, one by one, a seeded random sample PLUS the rows and columns
    at the edges of the kernel's output tiles and XCD runs; the weight gradient (small output, long reduction, split
    across workgroups) is compared as a WHOLE tensor.  Every compared element also has to meet the per-element bound."""
    d, od = desc_of(case), odesc_of(case)
    rng = np.random.default_rng(seed)
    res = {}
    ax, aw, ady = abs16(case.x), abs16(case.w16), abs16(case.dy)

    def sample(out, op, M, Ncol, to_flat):
        rows, cols = structured_rows_cols(M, Ncol, plan_tiles(op, d), pq=case.P * case.Q)
        edge = to_flat(np.repeat(rows, cols.size), np.tile(cols, rows.size))
        return np.unique(np.concatenate([rng.integers(0, out.size, size=min(n_fwd if op == api.JZ_FWD else n_bwd_data, out.size)), edge]))

    y = run_conv(api.JZ_FWD, d, case.x, case.w16, (case.N, case.P, case.Q, case.K))
    assert not np.any(np.isnan(y)), "fwd: unwritten output"
    idx = sample(y, api.JZ_FWD, case.N * case.P * case.Q, case.K, lambda r, c: r * case.K + c)
    res["fwd"] = check_half_output(y.ravel()[idx], oracle.conv_fwd_at(od, case.x, case.w16, idx), tol, "fwd",
                                   oracle.conv_fwd_at(od, ax, aw, idx))
    res["fwd"]["n"] = int(idx.size)
    if not skip_bwd_data:
        dx = run_conv(api.JZ_BWD_DATA, d, case.dy, case.w16, (case.N, case.H, case.W, case.C))
        assert not np.any(np.isnan(dx)), "bwd_data: unwritten output"
        bd_plan = plan_tiles(api.JZ_BWD_DATA, d)
        if bd_plan[0] == "classes":
            rows = class_edge_pixels(case, bd_plan[1])
            cols = np.asarray(sorted({c for t in range(-(-case.C // bd_plan[2])) for c in (t * bd_plan[2], min((t + 1) * bd_plan[2], case.C) - 1)}), np.int64)
            edge = np.repeat(rows, cols.size) * case.C + np.tile(cols, rows.size)
            idx = np.unique(np.concatenate([rng.integers(0, dx.size, size=min(n_bwd_data, dx.size)), edge]))
            res["bwd_data"] = check_half_output(dx.ravel()[idx], oracle.conv_bwd_data_at(od, case.dy, case.w16, idx), tol, "bwd_data",
                                                oracle.conv_bwd_data_at(od, ady, aw, idx))
            res["bwd_data"]["n"] = int(idx.size)
        elif bd_plan[5]:
            # strided 1x1 layer: the GEMM's rows are the output pixels (n, p, q); row m lands on input pixel
            # (n, p * stride, q * stride), and the pixel diagonally behind it (when inside) must hold the zero
            def to_flat(r, c):
                n, rem = np.divmod(r, case.P * case.Q)
                p, q = np.divmod(rem, case.Q)
                hit = ((n * case.H + p * case.stride) * case.W + q * case.stride) * case.C + c
                h1, w1 = np.minimum(p * case.stride + 1, case.H - 1), np.minimum(q * case.stride + 1, case.W - 1)
                return np.concatenate([hit, ((n * case.H + h1) * case.W + w1) * case.C + c])
            M = case.N * case.P * case.Q
        else:
            to_flat = lambda r, c: r * case.C + c
            M = case.N * case.H * case.W
        if bd_plan[0] != "classes":
            idx = sample(dx, api.JZ_BWD_DATA, M, case.C, to_flat)
            res["bwd_data"] = check_half_output(dx.ravel()[idx], oracle.conv_bwd_data_at(od, case.dy, case.w16, idx), tol, "bwd_data",
                                                oracle.conv_bwd_data_at(od, ady, aw, idx))
            res["bwd_data"]["n"] = int(idx.size)
    dw = run_conv(api.JZ_BWD_WEIGHT, d, case.x, case.dy, (case.K, case.R, case.S, case.C))
    res["bwd_weight"] = check_half_output(dw, oracle.conv_bwd_weight(od, case.x, case.dy), tol, "bwd_weight (whole tensor)",
                                          oracle.conv_bwd_weight(od, ax, ady))
    res["bwd_weight"]["n"] = int(dw.size)
    return res


def fc_all_modes(B, I, O, c, tol=1e-3):
    """The three fully connected GEMMs of one layer against the oracle's triple loops, norm-wise and element by element."""
    ax, aw, ady = abs16(c.x), abs16(c.w16), abs16(c.dy)
    res = {}
    res["fwd"] = check_half_output(run_fc(api.JZ_FWD, B, I, O, c.x, c.w16, (B, O)), oracle.fc_fwd(B, I, O, c.x, c.w16), tol, "fc fwd",
                                   oracle.fc_fwd(B, I, O, ax, aw))
    res["bwd_data"] = check_half_output(run_fc(api.JZ_BWD_DATA, B, I, O, c.dy, c.w16, (B, I)), oracle.fc_bwd_data(B, I, O, c.dy, c.w16), tol,
                                        "fc bwd_data", oracle.fc_bwd_data(B, I, O, ady, aw))
    res["bwd_weight"] = check_half_output(run_fc(api.JZ_BWD_WEIGHT, B, I, O, c.dy, c.x, (O, I)), oracle.fc_bwd_weight(B, I, O, c.dy, c.x), tol,
                                          "fc bwd_weight", oracle.fc_bwd_weight(B, I, O, ady, ax))
    return res


def all_ops_against_the_oracle(d, od, x, w, dy, ops=(api.JZ_FWD, api.JZ_BWD_DATA, api.JZ_BWD_WEIGHT), tol=1e-3):
    """fwd / bwd_data / bwd_weight of an arbitrary descriptor pair (library, oracle) on given arrays: whole tensors,
    norm-wise and element by element."""
    N, H, W, C, K, R, S = od.N, od.H, od.W, od.C, od.K, od.R, od.S
    ax, aw, ady = abs16(x), abs16(w), abs16(dy)
    res = {}
    if api.JZ_FWD in ops:
        res["fwd"] = check_half_output(run_conv(api.JZ_FWD, d, x, w, (N, od.P, od.Q, K)), oracle.conv_fwd(od, x, w), tol, "fwd",
                                       oracle.conv_fwd(od, ax, aw))
    if api.JZ_BWD_DATA in ops:
        res["bwd_data"] = check_half_output(run_conv(api.JZ_BWD_DATA, d, dy, w, (N, H, W, C)), oracle.conv_bwd_data(od, dy, w), tol,
                                            "bwd_data", oracle.conv_bwd_data(od, ady, aw))
    if api.JZ_BWD_WEIGHT in ops:
        res["bwd_weight"] = check_half_output(run_conv(api.JZ_BWD_WEIGHT, d, x, dy, (K, R, S, C)), oracle.conv_bwd_weight(od, x, dy), tol,
                                              "bwd_weight", oracle.conv_bwd_weight(od, ax, ady))
    return res
