"""Tuning sweep for the implicit-GEMM planner: python -m paper_1807_11205_amd.tune [--json FILE] [--write] [--in-place]

For every distinct convolution shape of ResNet-50 (batch 64) and each of forward / backward-data / backward-weight it
times every kernel variant (output tile, k tile depth, wavefronts per workgroup) at every admissible split of the
reduction, through the planner's tuning hook (jz_conv2d_tune_set), with the caches flushed before each timed launch (inside a
training step every layer finds them cold).  `--write` turns the measurements into csrc/jz_tuned.inc, the table the
planner consults before its cost model; `--json FILE` re-uses saved measurements instead of running on the GPU.

`--in-place` refines those choices inside the whole training step of bench.py (three streams, the network's own
dependency order): a layer that runs beside others does not always want the variant that is fastest alone (fewer
splits leave compute units and bandwidth to its neighbours).  For every layer shape, heaviest first, it tries the few
best variants of the layer-by-layer sweep and smaller split counts through jz_conv2d_tune_set, times the GEMM phase of
the step and keeps a change only if a second measurement confirms it; it starts from the choices compiled into the
library, so it can be repeated.
"""
import argparse
import json
import os
import re
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
# (tile, k tile depth, wavefronts, ring depth)
VARIANTS = [(128128, 32, 4, 4), (128064, 32, 4, 4), (64128, 32, 4, 4), (64064, 32, 4, 4), (128128, 64, 8, 4), (256128, 64, 8, 3),
            (256128, 32, 8, 4), (256256, 32, 8, 4), (128128, 64, 4, 4), (128064, 64, 4, 4), (64128, 64, 4, 4), (64064, 64, 4, 4),
            (128128, 32, 4, 3), (128064, 32, 4, 3), (64128, 32, 4, 3), (64064, 32, 4, 3),
            (256128, 32, 8, 3), (128128, 32, 8, 4), (128128, 32, 8, 3)]
SPLITS = [1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 14, 16, 20, 24, 28, 32, 40, 48, 56, 64, 80, 96, 112, 128]
OPS = ("fwd", "bwd_data", "bwd_weight")
BATCH = 64
VARIANT = "v1"     # where ResNet-50's stride-2 steps sit (--variant)


def gemm_dims(rec):
    """(M, N, K, taps, scatter) of the GEMM the library runs for this record (see jz_igemm.h)."""
    H, C, K, R, st = rec["H"], rec["C"], rec["K"], rec["R"], rec["stride"]
    pad, B = rec.get("pad", (R - 1) // 2), rec.get("batch", BATCH)
    P = (H + 2 * pad - R) // st + 1
    if rec["op"] == "fwd":
        return B * P * P, K, R * R * C, R * R, 0
    if rec["op"] == "bwd_data":
        if R == 1 and st > 1:
            return B * P * P, C, K, 1, 1
        return B * H * H, C, R * R * K, R * R, 0
    return K, R * R * C, B * P * P, R * R, 0


def class_dims(rec):
    """(M, N, K, taps) of the GEMM of every parity class of a strided multi-tap backward-data layer (square image, filter,
    stride): input pixels h = ca + s i, w = cb + s l meet the taps r = (ca + pad) mod s + s j (and likewise along w)."""
    H, C, K, R, st = rec["H"], rec["C"], rec["K"], rec["R"], rec["stride"]
    pad, B = rec.get("pad", (R - 1) // 2), rec.get("batch", BATCH)
    out = []
    for ca in range(st):
        for cb in range(st):
            ha, wb = -(-(H - ca) // st), -(-(H - cb) // st)
            ra, sb = -(-(R - (ca + pad) % st) // st), -(-(R - (cb + pad) % st) // st)
            if ha > 0 and wb > 0:
                out.append((B * ha * wb, C, ra * sb * K, ra * sb))
    return out


def model_layers(model):
    """(batch, layers) swept for a model: every distinct convolution shape except the 3-channel stem (it runs on a padded
    copy and has its own entries), fully connected layers as 1x1 convolutions over a 1x1 image."""
    from . import shapes
    if model == "alexnet":
        convs = [c for c in shapes.alexnet_convs() if not c.first]
        return 128, convs + [shapes.ConvShape(f.name, 1, f.I, f.O, 1, 1, 0) for f in shapes.ALEXNET_FCS]
    seen, layers = set(), []
    if VARIANT != "v1":     # only what the v1 table does not already hold
        seen = {(c.H, c.C, c.K, c.R, c.stride) for c in shapes.resnet50_convs("v1")}
    for c in shapes.resnet50_convs(VARIANT):
        key = (c.H, c.C, c.K, c.R, c.stride)
        if key in seen or c.first:
            continue
        seen.add(key)
        layers.append(c)
    return BATCH, layers


def sweep(path, variants=VARIANTS, model="resnet50"):
    import torch
    from . import api
    h, dev = torch.float16, "cuda:0"
    BATCH, layers = model_layers(model)
    junk = torch.zeros(192 << 20, dtype=torch.float32, device=dev)
    ws = torch.empty(1 << 30, dtype=torch.uint8, device=dev)

    def timeit(fn, iters=3):
        fn()
        torch.cuda.synchronize()
        best = 1e9
        for _ in range(iters):
            junk.sum()  # read-only pass over 768 MB: evicts L2 and the last-level cache without leaving dirty lines
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1))
        return best * 1e3

    out = []
    for cs in layers:
        d = api.conv_desc(BATCH, cs.H, cs.H, cs.C, cs.K, cs.R, cs.R, cs.stride, cs.pad)
        x = torch.randn(BATCH * cs.H * cs.H * cs.C, device=dev).to(h)
        w = (torch.randn(cs.K * cs.R * cs.R * cs.C, device=dev) * 0.05).to(h)
        dy = torch.randn(BATCH * cs.P * cs.P * cs.K, device=dev).to(h)
        y, dx, dw = torch.empty_like(dy), torch.empty_like(x), torch.empty_like(w)
        for opn, op in zip(OPS, (api.JZ_FWD, api.JZ_BWD_DATA, api.JZ_BWD_WEIGHT)):
            def run():
                if opn == "fwd":
                    api.jz_conv2d_fwd(d, x, w, y, ws)
                elif opn == "bwd_data":
                    api.jz_conv2d_bwd_data(d, dy, w, dx, ws)
                else:
                    api.jz_conv2d_bwd_weight(d, x, dy, dw, ws)
            api.jz_conv2d_tune_clear()
            res = {"planner": round(timeit(run), 1)}
            api.jz_conv2d_tune_use_table(False)
            res["model"] = round(timeit(run), 1)
            for (t, bk, wv, nst) in variants:
                prev_need = None
                for sp in SPLITS:
                    try:
                        api.jz_conv2d_tune_set(op, d, t // 1000, t % 1000, bk, wv, nst, sp)
                        need = api.jz_conv2d_workspace_bytes(op, d)
                    except api.JzError:
                        continue  # no such kernel for this layer
                    if need > ws.numel() or (sp > 1 and need in (0, prev_need)):
                        continue  # too large, or the planner could not honour this split count
                    prev_need = need
                    plan = api.jz_conv2d_describe_plan(op, d)
                    want = "tile %dx%dx%d, %d wavefronts, ring %d," % (t // 1000, t % 1000, bk, wv, nst)
                    if want not in plan:
                        continue  # the planner could not honour this combination for this layer
                    res["%d.%d.%d.%d/%d" % (t, bk, wv, nst, sp)] = round(timeit(run), 1)
            api.jz_conv2d_tune_clear()
            cands = [k for k in res if k not in ("planner", "model")]
            best = min(cands, key=res.get)
            out.append(dict(layer=cs.name, H=cs.H, C=cs.C, K=cs.K, R=cs.R, stride=cs.stride, pad=cs.pad, batch=BATCH, op=opn, best=best,
                            best_us=res[best], all=res))
            print(cs.name, opn, "planner", res["planner"], "model", res["model"], "best", best, res[best], flush=True)
            with open(path, "w") as f:
                json.dump(out, f)
    return out


def write_table(recs, path, choice=None):
    """choice: {(layer, op): "tile.bk.waves.ring/splits"} from the in-place pass; default: the fastest alone."""
    lines = ["// Generated by `python -m paper_1807_11205_amd.tune --write` from cold-cache timings on one MI355X (ResNet-50 layer",
             "// shapes at batch 64 or --batch, or with --model alexnet the AlexNet-shaped layers at batch 128; with --in-place: refined inside",
             "// the whole training step).  {op, M, N, K, taps, scatter, BM, BN, k tile, wavefronts, ring depth, splits}; the planner",
             "// looks a GEMM up here first and falls back to its cost model."]
    for r in recs:
        cands = {k: v for k, v in r["all"].items() if k not in ("planner", "model")}
        best = min(cands, key=cands.get)
        if choice and (r["layer"], r["op"]) in choice:
            best = choice[(r["layer"], r["op"])]
        fam, sp = best.split("/")
        tile, bk, wv, nst = (int(v) for v in fam.split(".")[:4])
        note = "%.1f us alone" % cands[best] if best in cands else "chosen in the step"
        if r["op"] == "bwd_data" and r["R"] > 1 and r["stride"] > 1:
            # one launch per parity class of the stride, each a unit-stride GEMM of its own with a scatter epilogue: the
            # variant is recorded under every class's key (what jz_conv2d_tune_set does at run time), reductions unsplit
            keys = []
            for key in class_dims(r):
                if key not in keys:
                    keys.append(key)
                    lines.append("{1, %d, %d, %d, %d, 1, %d, %d, %d, %d, %d, 1},  // %s bwd_data, a parity class: %s for the layer" % (
                        key + (tile // 1000, tile % 1000, bk, wv, nst, r["layer"], note)))
            continue
        M, N, K, taps, sc = gemm_dims(r)
        lines.append("{%d, %d, %d, %d, %d, %d, %d, %d, %d, %d, %d, %s},  // %s %s: %s" % (
            OPS.index(r["op"]), M, N, K, taps, sc, tile // 1000, tile % 1000, bk, wv, nst, sp, r["layer"], r["op"], note))
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")


def in_place(recs, steps=100, top=3, gain=0.001, passes=2, n_side=2, model="resnet50"):
    """Coordinate descent over the layer shapes with the GEMM phase of the bench step as the objective."""
    import torch
    from . import api, shapes
    sys.path.insert(0, os.path.dirname(PKG))
    import bench
    api.lib()
    torch.cuda.set_device(0)
    big = 1 << 30
    if model == "alexnet":
        batch = 128
        wl = bench.AlexNetStep(batch, n_side, ws_bytes=big)                 # room for any split count
    else:
        batch = BATCH
        wl = bench.ResNet50Step(batch=BATCH, variant=VARIANT)
        wl.ws = torch.empty(big, dtype=torch.uint8, device="cuda:0")
        wl.side_ws = [torch.empty(big, dtype=torch.uint8, device="cuda:0") for _ in range(3)]
        for _ in range(12):                                                 # the loss-scale back-off of bench.py
            wl.step()
            torch.cuda.synchronize()
            if int(wl.found_inf.item()) == 0:
                break
            wl.halve_loss_scale()
    stream = torch.cuda.Stream()
    side = [torch.cuda.Stream() for _ in range(n_side)]
    ops = {"fwd": api.JZ_FWD, "bwd_data": api.JZ_BWD_DATA, "bwd_weight": api.JZ_BWD_WEIGHT}

    def measure():
        with torch.cuda.stream(stream):
            for _ in range(3):
                wl.run_gemms(side)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(steps):
                wl.run_gemms(side)
            e1.record(stream)
            stream.synchronize()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps

    def apply(d, op, key):
        fam, sp = key.split("/")
        tile, bk, wv, nst = (int(v) for v in fam.split("."))
        try:
            api.jz_conv2d_tune_set(op, d, tile // 1000, tile % 1000, bk, wv, nst, int(sp))
        except api.JzError:
            return False
        plan = api.jz_conv2d_describe_plan(op, d)
        # (the split count the plan reports can be a little lower: splits that would be empty are dropped)
        return ("tile %dx%dx%d, %d wavefronts, ring %d," % (tile // 1000, tile % 1000, bk, wv, nst)) in plan and \
            api.jz_conv2d_workspace_bytes(op, d) <= big

    convs = model_layers(model)[1] if model == "alexnet" else list(shapes.resnet50_convs(VARIANT))
    count = {}
    for c in convs:
        count[(c.H, c.C, c.K, c.R, c.stride)] = count.get((c.H, c.C, c.K, c.R, c.stride), 0) + 1
    pad_of = {(c.H, c.C, c.K, c.R, c.stride): c.pad for c in convs}
    work = []
    for r in recs:
        cands = {k: v for k, v in r["all"].items() if k not in ("planner", "model")}
        best = min(cands, key=cands.get)
        work.append((cands[best] * count[(r["H"], r["C"], r["K"], r["R"], r["stride"])], r, cands, best))
    # the 3-channel stems are not part of the layer-by-layer sweep (they run on a padded copy, forward on the patch
    # kernel): a few candidates by hand; their entries live beside the generated tables, so the result is only reported
    # (the times beside the candidates are rough figures alone, in us: they only order the candidates)
    if model == "alexnet":
        stem = dict(layer="conv1", H=227, C=3, K=96, R=11, stride=4, by_hand=True)
        pad_of[(227, 3, 96, 11, 4)] = 0
        by_hand = {"128128.32.4.3/128": 108.0, "128128.32.4.4/128": 110.0, "128128.32.4.3/64": 115.0, "128128.32.4.4/64": 115.0,
                   "128064.32.4.4/128": 120.0, "128064.32.4.4/64": 125.0, "64128.32.4.4/128": 125.0, "64128.32.4.4/64": 130.0,
                   "64064.32.4.4/128": 140.0}
        work.append((110.0, dict(stem, op="bwd_weight"), by_hand, "128128.32.4.3/128"))
    else:
        stem = dict(layer="stem", H=224, C=3, K=64, R=7, stride=2, by_hand=True)
        work.append((67.0, dict(stem, op="bwd_weight"), {"64064.32.4.4/256": 67.0, "64128.32.4.4/384": 69.0, "128064.32.4.4/192": 88.7},
                     "64064.32.4.4/256"))
    work.sort(key=lambda w: -w[0])

    def current(d, op):                                                     # what the library would run now, as a key
        m = re.search(r"tile (\d+)x(\d+)x(\d+), (\d+) wavefronts, ring (\d+), \d+ x \d+ tiles, (\d+) splits", api.jz_conv2d_describe_plan(op, d))
        bm, bn, bk, wv, nst, sp = (int(v) for v in m.groups())
        return "%d.%d.%d.%d/%d" % (bm * 1000 + bn, bk, wv, nst, sp)

    choice = {}
    base = min(measure(), measure())
    print("in-place: GEMM phase %.4f ms with the library's current choices" % base, flush=True)
    for p in range(passes):
        changed = 0
        for _, r, cands, alone in work:
            d = api.conv_desc(batch, r["H"], r["H"], r["C"], r["K"], r["R"], r["R"], r["stride"],
                              pad_of[(r["H"], r["C"], r["K"], r["R"], r["stride"])])
            op = ops[r["op"]]
            start = current(d, op)
            fam, sp = start.split("/")
            snap = lambda x: max((s for s in SPLITS if s <= max(1.0, x + 0.01)), default=1)
            fams = {}                                                       # variant -> (its best time alone, at which split)
            for k, v in cands.items():
                f, n = k.split("/")
                if f not in fams or v < fams[f][0]:
                    fams[f] = (v, int(n))
            tries = []
            for f in sorted(fams, key=lambda f: fams[f][0])[:top]:          # the best variants alone, also with fewer splits
                for scale in (1.0, 0.5, 0.25):
                    tries.append("%s/%d" % (f, snap(fams[f][1] * scale)))
            for scale in (1.5, 0.75, 0.5, 0.33):                            # the current variant with other split counts
                tries.append("%s/%d" % (fam, snap(int(sp) * scale)))
            tries = [k for i, k in enumerate(tries) if k != start and k not in tries[:i]]
            cur, cur_t = start, base
            for k in tries:
                if not apply(d, op, k) or current(d, op) == start:
                    continue
                t = measure()
                if t < cur_t * (1.0 - gain):
                    t2 = measure()                                          # confirm before believing it
                    if t2 < cur_t * (1.0 - gain):
                        cur, cur_t = k, max(t, t2)
            apply(d, op, cur)
            if cur != start:
                base = cur_t
                changed += 1
            if not r.get("by_hand"):
                choice[(r["layer"], r["op"])] = cur
            print("pass %d %s %s: %s -> %s  GEMM phase %.4f ms" % (p + 1, r["layer"], r["op"], start, cur, base), flush=True)
        if not changed:
            break
    final = min(measure(), measure())
    print("in-place: GEMM phase %.4f ms after refinement" % final, flush=True)
    return choice


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--json", default=None, help="saved measurements to use instead of running the sweep")
    ap.add_argument("--out-json", default="tune_sweep.json", help="where the sweep saves its measurements")
    ap.add_argument("--write", action="store_true", help="write csrc/jz_tuned.inc")
    ap.add_argument("--in-place", action="store_true", help="refine the choices inside the whole step of bench.py")
    ap.add_argument("--streams", type=int, default=3, help="--in-place: streams of the step (as bench.py --streams)")
    ap.add_argument("--passes", type=int, default=2, help="--in-place: passes over the launches (stops early when a pass changes nothing)")
    ap.add_argument("--top", type=int, default=3, help="--in-place: how many of a launch's best variants alone are tried in the step "
                                                       "(the AlexNet table: 8; the step has 22 launches, each long enough to matter)")
    ap.add_argument("--table", default=os.path.join(PKG, "csrc", "jz_tuned.inc"), help="where --write puts the table")
    ap.add_argument("--model", default="resnet50", choices=("resnet50", "alexnet"), help="whose layer shapes to sweep")
    ap.add_argument("--only", default=None, help="sweep only these variants, e.g. 256128.32.8.3,128128.32.8.4; with --json: "
                                                 "add the new timings to those saved measurements")
    ap.add_argument("--batch", type=int, default=None, help="resnet50: batch size of the swept shapes (default 64; the table is keyed "
                                                            "by GEMM shape, so tables of several batch sizes can sit side by side)")
    ap.add_argument("--variant", default="v1", choices=("v1", "v1.5"), help="resnet50: the network variant whose shapes are swept (the table is "
                                                                            "keyed by GEMM shape: a v1.5 table only needs the shapes v1 does not have)")
    a = ap.parse_args()
    global BATCH, VARIANT
    if a.batch:
        BATCH = a.batch
    VARIANT = a.variant
    if a.only:
        sel = [tuple(int(x) for x in v.split(".")) for v in a.only.split(",")]
        assert all(v in VARIANTS for v in sel), "unknown variant"
        fresh = sweep(a.out_json, sel, a.model)
        recs = json.load(open(a.json)) if a.json else fresh
        if a.json:
            by = {(r["layer"], r["op"]): r for r in fresh}
            for r in recs:
                extra = by[(r["layer"], r["op"])]["all"]
                r["all"].update({k: v for k, v in extra.items() if k not in ("planner", "model")})
                cands = {k: v for k, v in r["all"].items() if k not in ("planner", "model")}
                r["best"] = min(cands, key=cands.get)
                r["best_us"] = cands[r["best"]]
            with open(a.out_json, "w") as f:
                json.dump(recs, f)
    else:
        recs = json.load(open(a.json)) if a.json else sweep(a.out_json, VARIANTS, a.model)
    choice = None
    if a.in_place:
        choice = in_place(recs, n_side=a.streams - 1, model=a.model, top=a.top, passes=a.passes)
    if a.write:
        write_table(recs, a.table, choice)
    tp = sum(r["all"]["planner"] for r in recs)
    tb = sum(r["best_us"] for r in recs)
    print("sum over distinct layer shapes: planner %.0f us, best variant %.0f us" % (tp, tb), file=sys.stderr)


if __name__ == "__main__":
    main()
