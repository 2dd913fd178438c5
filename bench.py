#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X: ResNet-50 (v1) N=64, fp16 storage / fp32 accumulate.

One step = forward of all 53 convolutions and the classifier, then backward-data (not for the stem) and
backward-weight of every layer in reverse order with the weight gradients written straight into the fused flat
gradient buffer, then one mixed-precision LARS update over all 161 tensors (25,557,032 parameters).  Batch norm,
ReLU, pooling and the residual adds are not part of this path, so every layer has its own seeded synthetic input
and output gradient of the right shape (a chained stack without normalisation would overflow fp16).  Launches are
eager (replaying the step from a HIP graph measured slower here) and follow the network's dependency graph: the
projection shortcuts and the backward-weight launches run on side streams (--streams).

Prints ONE JSON line.  `value` is images/s of the whole step with all inputs resident in HBM; `roofline` is for
the implicit-GEMM kernel family (all conv/FC launches of a step, algorithmic flops / their time between HIP events
on the launch stream); `lars` gives the update's GB/s against HBM; `cpu_baseline` times the fp64 oracle on the
host cores on an eight-image sample of the same stack.
"""
import argparse
import json
import sys
import time

import numpy as np
import torch

from paper_1807_11205_amd import api, inputs, shapes

FP16_MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense fp16 matrix peak
FP32_MFMA_PEAK_TFLOPS = 157.3    # MI355X dense fp32 matrix peak
HBM_PEAK_GBPS = 8000.0           # MI355X HBM3E
LARS_BYTES_PER_PARAM = 20        # read w32 4 + g16 2 + v32 4, write w32 4 + v32 4 + w16 2
# HBM bytes per step are never literals here: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summaries live under profiles/,
# and the headline line quotes one only when it was taken with the kernel plans of the run (measured_traffic).


class ResNet50Step:
    """All device buffers of one ResNet-50 N=batch step and the launch sequence."""

    def __init__(self, batch=64, loss_scale=1024.0, seed=180711205, variant="v1", device="cuda:0", dtype="f16", lars_path="presummed",
                 sumsq_from="split"):
        """dtype "f32": the single-precision variant of the GEMM phase (float32 activations, filters = the master weights,
        float32 weight gradients in a buffer of their own; the LARS update still runs on the fp16 gradient buffer).
        lars_path "presummed": the update is one launch (jz_lars_mp_update_presummed).  The gradient sums of squares it needs
        come from two places.  sumsq_from "split": a backward-weight launch whose reduction is split leaves its gradient's
        sum of squares in the optimiser's workspace from inside the kernel that adds the partial sums (the values are in
        registers there); every other tensor (unsplit filters, batch-norm scale / shift, bias) is covered by one
        jz_lars_grad_sumsq launch behind the last backward-data launch, beside the last backward-weight launches.
        "all": every backward-weight launch leaves its sum (unsplit ones through a separate pass over the gradient).
        "three_launches": plain backward-weight, jz_lars_mp_update."""
        self.f32 = dtype == "f32"
        self.presummed = lars_path == "presummed" and not self.f32
        self.sumsq_from = sumsq_from
        self.N = batch
        self.dev = device
        self.loss_scale = float(loss_scale)
        self.ls_state = self.ls_policy = None
        gen = torch.Generator(device=device)
        gen.manual_seed(seed)
        self.gen = gen
        self.convs = shapes.resnet50_convs(variant)
        self.fc = shapes.RESNET50_FC
        tensors = shapes.resnet50_param_tensors(variant)
        self.offsets = shapes.offsets_of(tensors)
        self.flags = [t[3] for t in tensors]   # the presummed path marks the tensors whose producer supplies the sum (below)
        P = self.offsets[-1]
        h = torch.float32 if self.f32 else torch.float16

        def randn(n, std=1.0, dt=None):
            return (torch.randn(n, generator=gen, device=device, dtype=torch.float32) * std).to(dt or h)

        # fused flat parameter state: fp32 master (He-normal filters, gamma 1, beta 0, bias 0), momentum 0, fp16 copies
        self.master = torch.zeros(P, dtype=torch.float32, device=device)
        for i, (_, shp, kind, _) in enumerate(tensors):
            a, b = self.offsets[i], self.offsets[i + 1]
            if kind in ("conv", "fc"):
                fan_in = shp[1] * shp[2] * shp[3] if kind == "conv" else shp[1]
                self.master[a:b] = torch.randn(b - a, generator=gen, device=device) * float(np.sqrt(2.0 / fan_in))
            elif kind == "gamma":
                self.master[a:b] = 1.0
        self.momentum = torch.zeros(P, dtype=torch.float32, device=device)
        self.w16 = self.master.to(torch.float16)
        # gradients of batch-norm and bias tensors are not produced on this path: fixed synthetic values ~ N(0,1e-3)*S
        self.grad = randn(P, 1e-3 * self.loss_scale, torch.float16)
        self.grad32 = torch.zeros(P, dtype=torch.float32, device=device) if self.f32 else None
        self.master0, self.w16_0 = self.master.clone(), self.w16.clone()
        wsrc, gdst = (self.master, self.grad32) if self.f32 else (self.w16, self.grad)
        ws_conv = api.jz_conv2d_f32_workspace_bytes if self.f32 else api.jz_conv2d_workspace_bytes
        ws_fc = api.jz_gemm_fc_f32_workspace_bytes if self.f32 else api.jz_gemm_fc_workspace_bytes

        self.layers = []
        ws_bytes = 0
        self.flops = 0
        for li, cs in enumerate(self.convs):
            d = api.conv_desc(batch, cs.H, cs.H, cs.C, cs.K, cs.R, cs.R, cs.stride, cs.pad)
            ti = 3 * li
            a, b = self.offsets[ti], self.offsets[ti + 1]
            L = dict(kind="conv", name=cs.name, d=d, first=cs.first, tensor=ti,
                     x=randn(batch * cs.H * cs.H * cs.C), dy=randn(batch * cs.P * cs.P * cs.K, self.loss_scale),
                     y=torch.empty(batch * cs.P * cs.P * cs.K, dtype=h, device=device),
                     dx=None if cs.first else torch.empty(batch * cs.H * cs.H * cs.C, dtype=h, device=device),
                     w=wsrc[a:b], dw=gdst[a:b], calls={})
            for op in (api.JZ_FWD, api.JZ_BWD_DATA, api.JZ_BWD_WEIGHT):
                ws_bytes = max(ws_bytes, ws_conv(op, d))
            self.flops += 2 * cs.macs(batch) * (2 if cs.first else 3)
            self.layers.append(L)
        ti = 3 * len(self.convs)
        a, b = self.offsets[ti], self.offsets[ti + 1]
        B, I, O = batch, self.fc.I, self.fc.O
        self.layers.append(dict(kind="fc", name="fc", tensor=ti, x=randn(B * I), dy=randn(B * O, self.loss_scale),
                                y=torch.empty(B * O, dtype=h, device=device), dx=torch.empty(B * I, dtype=h, device=device),
                                w=wsrc[a:b], dw=gdst[a:b], calls={}))
        for op in (api.JZ_FWD, api.JZ_BWD_DATA, api.JZ_BWD_WEIGHT):
            ws_bytes = max(ws_bytes, ws_fc(op, B, I, O))
        self.flops += 2 * self.fc.macs(batch) * 3
        self.ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=device)
        self.side_ws = [torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=device) for _ in range(3)]

        if self.presummed:
            for L in self.layers:
                d = L["d"] if L["kind"] == "conv" else api.conv_desc(B, 1, 1, I, O, 1, 1)
                split = ", 1 splits" not in api.jz_conv2d_describe_plan(api.JZ_BWD_WEIGHT, d)
                L["sumsq"] = self.sumsq_from == "all" or (self.sumsq_from == "split" and split)
                if L["sumsq"]:
                    self.flags[L["tensor"]] |= api.JZ_PARAM_GRAD_PRESUMMED
        self.found_inf = torch.zeros(1, dtype=torch.int32, device=device)
        self.ps = api.ParamSet(self.offsets, self.flags, self.master, self.momentum, self.grad, self.w16)
        self.lars_ws = torch.zeros(api.jz_lars_workspace_bytes(self.ps), dtype=torch.uint8, device=device)
        api.jz_lars_prepare(self.ps, self.lars_ws)
        self.P = P
        self.programs = {}

    def hparams(self):
        hp = inputs.HPARAMS
        return api.lars_hparams(hp["lr"], hp["momentum"], hp["weight_decay"], hp["trust_coef"], self.loss_scale)

    def _bound(self, L, op, ws):
        """The layer's forward / backward-data / backward-weight call with its arguments marshalled once."""
        B, I, O = self.N, self.fc.I, self.fc.O
        key = (op, ws.data_ptr())
        if key not in L["calls"]:
            if self.presummed and op == api.JZ_BWD_WEIGHT and L.get("sumsq"):
                sink = api.jz_lars_sumsq_sink(self.ps, self.lars_ws, L["tensor"])
                if L["kind"] == "conv":
                    L["calls"][key] = api.bind_conv2d_bwd_weight_sumsq(L["d"], L["x"], L["dy"], L["dw"], sink, ws)
                else:
                    L["calls"][key] = api.bind_gemm_fc_bwd_weight_sumsq(B, I, O, L["dy"], L["x"], L["dw"], sink, ws)
            elif L["kind"] == "conv":
                a, b, o = {api.JZ_FWD: ("x", "w", "y"), api.JZ_BWD_DATA: ("dy", "w", "dx"), api.JZ_BWD_WEIGHT: ("x", "dy", "dw")}[op]
                L["calls"][key] = (api.bind_conv2d_f32 if self.f32 else api.bind_conv2d)(op, L["d"], L[a], L[b], L[o], ws)
            else:
                a, b, o = {api.JZ_FWD: ("x", "w", "y"), api.JZ_BWD_DATA: ("dy", "w", "dx"), api.JZ_BWD_WEIGHT: ("dy", "x", "dw")}[op]
                L["calls"][key] = (api.bind_gemm_fc_f32 if self.f32 else api.bind_gemm_fc)(op, B, I, O, L[a], L[b], L[o], ws)
        return L["calls"][key]

    def build_program(self, n_side):
        """The launch sequence of the GEMM phase as a flat list of (kind, object, stream index) with kind in
        launch / record / wait; stream 0 is the caller's stream, 1 .. n_side the side streams.

        Forward of every layer, then the backward pass, ordered the way the network's own dependency graph allows
        (every layer has independent buffers here, but nothing is started earlier than a real ResNet-50 could start it).
        Forward: the projection shortcut of a stage's first block reads the block input, like conv a of that block, so it
        runs on a side stream beside a-b-c.  Backward: dW of layer l needs only dy of layer l, which the backward-data
        of layer l+1 produces, so the backward-weight launches go round-robin to the side streams while the
        backward-data chain stays on stream 0.  Each side stream has its own workspace."""
        prog = []
        ev = lambda: torch.cuda.Event()
        names = [L["name"] for L in self.layers]
        begin = ("launch", lambda st: api.jz_lars_begin_step(self.ps, self.lars_ws, self.ls_state, stream=st))
        # every tensor whose sum of squares no backward-weight launch supplies, in one launch behind the last backward-data
        # launch (their gradients exist by then, or are being written by launches this one is ordered behind)
        rest = ("launch", lambda st: api.jz_lars_grad_sumsq(self.ps, 0, self.ps.T, self.lars_ws, stream=st), 0)
        pending = None
        block_in = None
        begun = not self.presummed
        if self.presummed and not n_side:
            prog.append(begin + (0,))   # the step starts: clear the gradient sinks, add up the carried sums of squares of the weights
            begun = True
        for L in self.layers:                                   # forward
            if n_side and L["kind"] == "conv" and L["name"].endswith("p"):
                prog += [("wait", block_in, 1), ("launch", self._bound(L, api.JZ_FWD, self.side_ws[0]), 1)]
                if not begun:
                    # jz_lars_begin_step costs the step nothing here: side stream 1 has nothing else to do, block_in orders
                    # it behind the previous update, and the main stream waits for `pending` long before anything touches
                    # a sink
                    prog.append(begin + (1,))
                    begun = True
                pending = ev()
                prog.append(("record", pending, 1))
                continue
            if n_side and L["kind"] == "conv" and L["name"].endswith("a"):
                if pending is not None:                         # the residual add of the previous block needs its shortcut
                    prog.append(("wait", pending, 0))
                    pending = None
                if L["name"][:-1] + "p" in names:               # only a block with a projection shortcut has a second reader
                    block_in = ev()                             # (an event record costs the stream 4-6 us)
                    prog.append(("record", block_in, 0))
            prog.append(("launch", self._bound(L, api.JZ_FWD, self.ws), 0))
        if pending is not None:
            prog.append(("wait", pending, 0))
        if not begun:
            prog.append(begin + (0,))
        if not n_side:
            for L in reversed(self.layers):                     # backward, one stream
                if not L.get("first"):
                    prog.append(("launch", self._bound(L, api.JZ_BWD_DATA, self.ws), 0))
                prog.append(("launch", self._bound(L, api.JZ_BWD_WEIGHT, self.ws), 0))
            return prog + ([rest] if self.presummed else [])
        ready = ev()
        prog.append(("record", ready, 0))                       # the loss gradient exists
        unsplit_done = {}
        for k, L in enumerate(reversed(self.layers)):
            si = 1 + k % n_side
            prog += [("wait", ready, si), ("launch", self._bound(L, api.JZ_BWD_WEIGHT, self.side_ws[si - 1]), si)]
            if self.presummed and not L.get("sumsq"):
                unsplit_done[si] = len(prog)                    # the last launch on this side stream that `rest` reads from
            if not L.get("first"):
                prog.append(("launch", self._bound(L, api.JZ_BWD_DATA, self.ws), 0))
                ready = ev()
                prog.append(("record", ready, 0))               # dy of the layer below exists
        if self.presummed:
            # `rest` reads the unsplit filters' gradients: behind the last such launch of each side stream (they are early in
            # the backward pass, so these waits do not hold the main stream up)
            for si, pos in sorted(unsplit_done.items(), key=lambda kv: -kv[1]):
                e = ev()
                prog.insert(pos, ("record", e, si))
                prog.append(("wait", e, 0))
            prog.append(rest)
        for si in range(1, n_side + 1):
            done = ev()
            prog += [("record", done, si), ("wait", done, 0)]
        return prog

    def run_gemms(self, sides=()):
        n_side = len(sides)
        if n_side not in self.programs:
            self.programs[n_side] = self.build_program(n_side)
        streams = [torch.cuda.current_stream(), *sides]
        for kind, obj, si in self.programs[n_side]:
            if kind == "launch":
                obj(streams[si])
            elif kind == "record":
                obj.record(streams[si])
            else:
                streams[si].wait_event(obj)

    def run_lars(self):
        if self.presummed:
            if self.ls_state is not None:
                api.jz_lars_mp_update_presummed_dyn(self.ps, self.hparams(), self.ls_policy, self.ls_state, self.found_inf, self.lars_ws)
            else:
                api.jz_lars_mp_update_presummed(self.ps, self.hparams(), self.found_inf, self.lars_ws)
        elif self.ls_state is not None:
            api.jz_lars_mp_update_dyn(self.ps, self.hparams(), self.ls_policy, self.ls_state, self.found_inf, self.lars_ws)
        else:
            api.jz_lars_mp_update(self.ps, self.hparams(), self.found_inf, self.lars_ws)

    def use_dynamic_loss_scale(self):
        """The update reads S from device memory and the controller kernel runs behind it.  The growth interval is set
        beyond the run's length so that S stays at the value the synthetic gradients were scaled with."""
        self.ls_state = torch.zeros(2, dtype=torch.int32, device=self.found_inf.device)
        self.ls_policy = api.loss_scale_policy(growth_interval=1 << 30)
        api.jz_loss_scale_init(self.ls_state, self.loss_scale)
        self.programs = {}   # jz_lars_begin_step takes the state

    def step(self):
        self.run_gemms()
        self.run_lars()

    def halve_loss_scale(self):
        """Back off after an overflow: every loss-scaled quantity is halved (exact in fp16 short of underflow)."""
        self.loss_scale *= 0.5
        for L in self.layers:
            L["dy"].mul_(0.5)
        self.grad.mul_(0.5)

    def reset_state(self):
        self.master.copy_(self.master0)
        self.w16.copy_(self.w16_0)
        self.momentum.zero_()
        api.jz_lars_prepare(self.ps, self.lars_ws)   # the master weights were written from outside: drop the carried sums


class _LayerView:
    """What per_layer_report needs of a workload that is not a ResNet50Step: the layer records, how to bind a call."""

    def __init__(self, layers, bound, ws, N, dev, title):
        self.layers, self._bound_fn, self.ws, self.N, self.dev, self.title, self.f32, self.fc = layers, bound, ws, N, dev, title, False, None

    def _bound(self, L, op, ws):
        return self._bound_fn(L, op, ws)


def per_layer_report(wl, iters=20, out_path=None, peak=FP16_MFMA_PEAK_TFLOPS):
    """Time every launch of the step on its own (HIP events) and print one line per layer and op: time warm (`iters`
    back-to-back repeats) and cold (caches flushed by a 768 MB read before each of three launches, the fastest: inside
    the step every layer finds its operands cold), TFLOP/s, the layer's own roofline min(matrix peak, flop / compulsory
    bytes * HBM peak), the fraction of it reached (warm), and the kernel plan.  Compulsory bytes = both inputs read
    once + the output written once.  Returns the rows as dicts; out_path: also written there as a text table."""
    B = wl.N
    title = getattr(wl, "title", "ResNet-50 v1")
    rows = []
    junk = torch.zeros(192 << 20, dtype=torch.float32, device=wl.dev)
    esz = 4 if wl.f32 else 2

    def timeit(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        warm = e0.elapsed_time(e1) / iters
        cold = 1e9
        for _ in range(3):
            junk.sum()      # read-only pass over 768 MB: evicts L2 and the last-level cache without leaving dirty lines
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            cold = min(cold, e0.elapsed_time(e1))
        return warm, cold

    lines = ["# per-layer, per-op timing of the %s step (%s, N = %d): every launch alone on an idle GPU" % ("fp32" if wl.f32 else "fp16", title, wl.N),
             "# command: python3 " + " ".join(sys.argv),
             "# us warm = mean of %d back-to-back launches; us cold = fastest of 3 launches behind a 768 MB cache flush;" % iters,
             "# roofline = min(%.1f TFLOP/s, flop / (bytes of both inputs + output) * 8 TB/s); frac = warm TFLOP/s / roofline;" % peak,
             "# us@roof = the time that roofline allows; plan = the library's kernel choice (jz_conv2d_describe_plan)",
             "# layer   shape                    op          us warm  us cold  TFLOP/s  roofline  frac   us@roof  plan"]
    opname = {api.JZ_FWD: "fwd", api.JZ_BWD_DATA: "bwd_data", api.JZ_BWD_WEIGHT: "bwd_weight"}
    for L in wl.layers:
        if L["kind"] == "conv":
            d = L["d"]
            macs = d.N * d.P * d.Q * d.K * d.R * d.S * d.C
            desc = "%dx%d %d->%d %dx%d s%d" % (d.H, d.W, d.C, d.K, d.R, d.S, d.stride_h)
        else:
            I, O = (L["I"], L["O"]) if "I" in L else (wl.fc.I, wl.fc.O)
            d = api.conv_desc(B, 1, 1, I, O, 1, 1)
            macs = B * I * O
            desc = "fc %d->%d" % (I, O)
        nbytes = esz * (L["x"].numel() + L["w"].numel() + L["y"].numel())
        for op in (api.JZ_FWD, api.JZ_BWD_DATA, api.JZ_BWD_WEIGHT):
            if op == api.JZ_BWD_DATA and L.get("first"):
                continue
            call = wl._bound(L, op, wl.ws)
            warm, cold = timeit(call)
            tf = 2 * macs / (warm * 1e-3) / 1e12
            roof = min(peak, 2 * macs / nbytes * HBM_PEAK_GBPS / 1e3)
            plan = "" if wl.f32 else api.jz_conv2d_describe_plan(op, d).split(": ", 1)[1]
            r = dict(layer=L["name"], shape=desc, op=opname[op], us=warm * 1e3, us_cold=cold * 1e3, tflops=tf, roofline_tflops=roof,
                     frac=tf / roof, us_roofline=2 * macs / roof / 1e6, plan=plan)
            rows.append(r)
            line = "%-7s %-24s %-10s %8.1f %8.1f %8.1f %9.1f %6.3f %8.1f  %s" % (r["layer"], desc, r["op"], r["us"], r["us_cold"], tf, roof,
                                                                               r["frac"], r["us_roofline"], plan)
            lines.append(line)
            print(line, file=sys.stderr, flush=True)
    lines.append("# sums over the step's launches (us): warm %.1f, cold %.1f, at the per-layer rooflines %.1f" % (
        sum(r["us"] for r in rows), sum(r["us_cold"] for r in rows), sum(r["us_roofline"] for r in rows)))
    for opn in ("fwd", "bwd_data", "bwd_weight"):
        sel = [r for r in rows if r["op"] == opn]
        lines.append("#   %-10s warm %.1f  cold %.1f  roofline %.1f" % (opn, sum(r["us"] for r in sel), sum(r["us_cold"] for r in sel),
                                                                        sum(r["us_roofline"] for r in sel)))
    for ln in lines[-4:]:
        print(ln, file=sys.stderr)
    if out_path:
        with open(out_path, "w") as f:
            f.write("\n".join(lines) + "\n")
    return rows


class AlexNetStep:
    """configs[3]: the AlexNet-shaped layers (five convolutions, ungrouped, and the three FC GEMMs) at N = 128, forward,
    backward-data and backward-weight of every layer on independent seeded N(0,1) inputs, He-normal weights.  Same launch
    scheme as the ResNet-50 step: forward and the backward-data chain in network order on one stream, backward-weight
    round-robin on the side streams.  ws_bytes: size of each stream's workspace (default: what the current plans need;
    a tuning run that tries other split counts passes more)."""

    def __init__(self, batch=128, n_side=2, ws_bytes=None):
        B, h, dev = batch, torch.float16, "cuda:0"
        self.N, self.dev, self.n_side = B, dev, n_side
        gen = torch.Generator(device=dev)
        gen.manual_seed(7)
        randn = lambda n, std=1.0: (torch.randn(n, generator=gen, device=dev) * std).to(h)
        layers, flops, need = [], 0, 0
        for cs in shapes.alexnet_convs():
            d = api.conv_desc(B, cs.H, cs.H, cs.C, cs.K, cs.R, cs.R, cs.stride, cs.pad)
            nx, ny, nw = B * cs.H * cs.H * cs.C, B * cs.P * cs.P * cs.K, cs.K * cs.R * cs.R * cs.C
            layers.append(dict(kind="conv", name=cs.name, d=d, first=cs.first, x=randn(nx), dy=randn(ny),
                               w=randn(nw, float(np.sqrt(2.0 / (cs.R * cs.R * cs.C)))), y=torch.empty(ny, dtype=h, device=dev),
                               dx=None if cs.first else torch.empty(nx, dtype=h, device=dev), dw=torch.empty(nw, dtype=h, device=dev)))
            need = max([need] + [api.jz_conv2d_workspace_bytes(op, d) for op in (api.JZ_FWD, api.JZ_BWD_DATA, api.JZ_BWD_WEIGHT)])
            flops += 2 * cs.macs(B) * (2 if cs.first else 3)
        for fc in shapes.ALEXNET_FCS:
            layers.append(dict(kind="fc", name=fc.name, I=fc.I, O=fc.O, first=False, x=randn(B * fc.I), dy=randn(B * fc.O),
                               w=randn(fc.I * fc.O, float(np.sqrt(2.0 / fc.I))), y=torch.empty(B * fc.O, dtype=h, device=dev),
                               dx=torch.empty(B * fc.I, dtype=h, device=dev), dw=torch.empty(fc.I * fc.O, dtype=h, device=dev)))
            need = max([need] + [api.jz_gemm_fc_workspace_bytes(op, B, fc.I, fc.O) for op in (api.JZ_FWD, api.JZ_BWD_DATA, api.JZ_BWD_WEIGHT)])
            flops += 2 * fc.macs(B) * 3
        self.layers, self.flops = layers, flops
        self.wss = [torch.empty(max(ws_bytes or need, 16), dtype=torch.uint8, device=dev) for _ in range(n_side + 1)]
        prog = [("launch", self.bound(L, api.JZ_FWD, self.wss[0]), 0) for L in layers]
        ready = torch.cuda.Event()
        prog.append(("record", ready, 0))
        for k, L in enumerate(reversed(layers)):
            si = 1 + k % n_side if n_side else 0
            if n_side:
                prog.append(("wait", ready, si))
            prog.append(("launch", self.bound(L, api.JZ_BWD_WEIGHT, self.wss[si]), si))
            if not L["first"]:
                prog.append(("launch", self.bound(L, api.JZ_BWD_DATA, self.wss[0]), 0))
                if n_side:
                    ready = torch.cuda.Event()
                    prog.append(("record", ready, 0))
        for si in range(1, n_side + 1):
            done = torch.cuda.Event()
            prog += [("record", done, si), ("wait", done, 0)]
        self.prog = prog

    def bound(self, L, op, ws):
        if L["kind"] == "conv":
            a, b, o = {api.JZ_FWD: ("x", "w", "y"), api.JZ_BWD_DATA: ("dy", "w", "dx"), api.JZ_BWD_WEIGHT: ("x", "dy", "dw")}[op]
            return api.bind_conv2d(op, L["d"], L[a], L[b], L[o], ws)
        a, b, o = {api.JZ_FWD: ("x", "w", "y"), api.JZ_BWD_DATA: ("dy", "w", "dx"), api.JZ_BWD_WEIGHT: ("dy", "x", "dw")}[op]
        return api.bind_gemm_fc(op, self.N, L["I"], L["O"], L[a], L[b], L[o], ws)

    def run_gemms(self, sides=()):
        """One step: main chain on the current stream, backward-weight launches on `sides` (as many as n_side)."""
        streams = [torch.cuda.current_stream(), *sides]
        for kind, obj, si in self.prog:
            if kind == "launch":
                obj(streams[si])
            elif kind == "record":
                obj.record(streams[si])
            else:
                streams[si].wait_event(obj)


def alexnet_workload(args):
    """bench.py --workload alexnet: times AlexNetStep.  One JSON line; no LARS phase (the configuration names none)."""
    B = args.batch
    n_side = max(0, min(args.streams, 4) - 1)
    wl = AlexNetStep(B, n_side)
    layers, flops, prog = wl.layers, wl.flops, wl.prog
    rows = None
    if args.per_layer or args.per_layer_file:
        rows = per_layer_report(_LayerView(layers, wl.bound, wl.wss[0], B, wl.dev, "AlexNet-shaped layers"), out_path=args.per_layer_file)
    stream = torch.cuda.Stream()
    sides = [torch.cuda.Stream() for _ in range(n_side)]
    run = lambda: wl.run_gemms(sides)

    with torch.cuda.stream(stream):
        for _ in range(max(args.warmup, 1)):
            run()
        stream.synchronize()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        for _ in range(args.steps):
            run()
        e1.record(stream)
        stream.synchronize()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    ms = wall * 1e3 / args.steps
    tflops = flops / (e0.elapsed_time(e1) / args.steps * 1e-3) / 1e12
    n_launch = sum(1 for e in prog if e[0] == "launch")
    out = {
        "metric": "AlexNet-shaped layers N=%d fp16 fwd+bwd images/s" % B, "value": B / (ms * 1e-3), "unit": "images/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 storage, f32 accumulate", "data": "synthetic",
        "config": {"workload": "configs[3]: AlexNet-shaped layers (5 convs ungrouped + 3 FC), fwd + bwd_data + bwd_weight per layer on "
                               "independent seeded N(0,1) inputs", "batch": B, "launch": "eager", "streams": args.streams},
        "roofline": {"kernel": "igemm_kernel (all %d conv/FC launches of a step)" % n_launch, "bound": "mfma", "achieved": tflops,
                     "peak": FP16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tflops / FP16_MFMA_PEAK_TFLOPS, "traffic": None,
                     "flop_per_step": flops}}
    if rows is not None:
        worst = sorted(rows, key=lambda r: r["us"] - r["us_roofline"], reverse=True)[:10]
        out["per_layer_worst"] = [{k: r[k] for k in ("layer", "shape", "op", "us", "us_roofline", "tflops", "roofline_tflops", "frac", "plan")}
                                  for r in worst]
    print(json.dumps(out))


def bn_workload(args):
    """The 53 batch-normalization + ReLU layers of ResNet-50 v1 at N = 64 (one behind every convolution, on that
    convolution's output shape), forward of all, then backward of all in reverse order, on independent seeded inputs.
    HBM-bound: algorithmic bytes are 4 per element forward (x read, y written) and 8 backward (x, y, dy read, dx written)."""
    B, h, dev = args.batch, torch.float16, "cuda:0"
    gen = torch.Generator(device=dev)
    gen.manual_seed(11)
    layers, elems, ws_bytes = [], 0, 16
    for cs in shapes.resnet50_convs():
        rows, C = B * cs.P * cs.P, cs.K
        n = rows * C
        layers.append(dict(rows=rows, C=C, x=(torch.randn(n, generator=gen, device=dev) * 1.5 + 0.3).to(h),
                           dy=torch.randn(n, generator=gen, device=dev).to(h), y=torch.empty(n, dtype=h, device=dev),
                           dx=torch.empty(n, dtype=h, device=dev), gamma=torch.ones(C, device=dev), beta=torch.zeros(C, device=dev),
                           mean=torch.empty(C, device=dev), invstd=torch.empty(C, device=dev),
                           dg=torch.empty(C, dtype=h, device=dev), db=torch.empty(C, dtype=h, device=dev)))
        elems += n
        ws_bytes = max(ws_bytes, api.jz_bn_workspace_bytes(rows, C))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    def run():
        for L in layers:
            api.jz_bn_relu_fwd(L["rows"], L["C"], L["x"], L["gamma"], L["beta"], 1e-5, True, L["y"], L["mean"], L["invstd"], ws)
        for L in reversed(layers):
            api.jz_bn_relu_bwd(L["rows"], L["C"], L["x"], L["y"], L["dy"], L["gamma"], L["mean"], L["invstd"], True, L["dx"],
                               L["dg"], L["db"], ws)

    for _ in range(max(args.warmup, 1)):
        run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    gbps = 12.0 * elems / (e0.elapsed_time(e1) / args.steps * 1e-3) / 1e9
    print(json.dumps({
        "metric": "ResNet-50 N=%d batch-norm + ReLU fwd+bwd GB/s (algorithmic)" % B, "value": gbps, "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 storage, f32 statistics (f64 across slabs)", "data": "synthetic",
        "config": {"workload": "the 53 batch-normalization + ReLU layers of ResNet-50 v1 (training mode), forward then backward, "
                               "independent seeded inputs", "batch": B, "elements_per_pass": elems, "launch": "eager", "streams": 1},
        "roofline": {"kernel": "bn_stats / bn_apply / bn_bwd_apply (6 launches per layer)", "bound": "hbm", "achieved": gbps,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS,
                     "traffic": None,
                     "traffic_note": "not measured in this run; profiles/bench_bn_resnet50_n64_kernel_stats.txt holds the HBM-counter "
                                     "summary of this workload (20.9 bytes per element moved against 12 algorithmic when it was taken)",
                     "bytes_per_element": 12}}))


def chain_workload(args):
    """One complete, chained training step of ResNet-50 v1 (every tensor produced by the launch before it): forward with
    training-mode batch normalization, ReLU, pooling and residual adds, softmax cross-entropy gradient times the loss
    scale, backward into the fused FP16 gradient buffer, LARS update with the dynamic loss scale on the device.  Eager
    launches, the weight-gradient GEMMs on a side stream (--streams 1: everything on one), the same fixed synthetic
    batch every step."""
    from paper_1807_11205_amd import resnet50
    net = resnet50.ResNet50Chain(batch=args.batch, image=224, initial_loss_scale=65536.0,
                                 policy=dict(growth_interval=1 << 30, max_scale=2.0 ** 24), fused=not args.unfused,
                                 block_end=not args.no_block_end, bwd_stats=not args.no_bwd_stats)
    skipped = 0
    for _ in range(24):                                   # let the controller bring the scale down until steps go through
        net.step()
        torch.cuda.synchronize()
        if int(net.found_inf.item()) == 0:
            break
        skipped += 1
    assert int(net.found_inf.item()) == 0, "the loss scale did not settle"
    for _ in range(max(args.warmup, 1)):
        net.step()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    # one side stream for the weight gradients: two or three measured slower (7.36, 7.38 against 7.23 ms)
    side = [torch.cuda.Stream()] if args.streams > 1 else None
    for _ in range(2):
        net.step(side=side)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for e in ev:
        e[0].record(); net.forward(side=side); e[1].record(); net.backward(side=side); e[2].record(); net.update(); e[3].record()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    assert int(net.found_inf.item()) == 0
    ph = [float(np.mean([e[i].elapsed_time(e[i + 1]) for e in ev])) for i in range(3)]
    gpu_ms = float(np.mean([e[0].elapsed_time(e[3]) for e in ev]))
    tflops = net.flops_per_step() / (gpu_ms * 1e-3) / 1e12
    kinds = {}
    for op in net.trace:
        kinds[op.kind] = kinds.get(op.kind, 0) + 1
    print(json.dumps({
        "metric": "ResNet-50 N=%d chained training step images/s" % args.batch, "value": args.batch / (ms * 1e-3), "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 storage, f32 accumulate, f32 master weights", "data": "synthetic",
        "config": {"workload": "ResNet-50 v1 chained step: conv + batch norm + ReLU + pooling + residual adds + classifier + "
                               "softmax loss gradient, backward, LARS with dynamic loss scale", "batch": args.batch, "image": 224,
                   "launch": "eager", "streams": 1 + (len(side) if side else 0), "launches_per_step": len(net.trace), "launches_by_kind": kinds,
                   "conv_bn_forward": "one call, statistics in the convolution epilogue" if net.fused else "two calls",
                   "loss_scale": api.loss_scale_state(net.ls_state)[0], "steps_skipped_while_the_scale_settled": skipped,
                   "mean_loss": net.mean_loss()},
        "phases_ms": {"forward_and_loss": ph[0], "backward": ph[1], "lars_update": ph[2], "gpu_total": gpu_ms},
        "roofline": {"kernel": "whole step (GEMM flops of the convolutions and the classifier over the step's GPU time)",
                     "bound": "mfma", "achieved": tflops, "peak": FP16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": tflops / FP16_MFMA_PEAK_TFLOPS, "traffic": None},
        "hbm": {"bytes_per_step": None, "note": "not measured in this run; profiles/bench_chain_resnet50_n64_hbm_traffic.txt holds the "
                                                  "HBM-counter summary of this workload"}}))


def cpu_baseline(sample_batch=8):
    """The fp64 oracle, as it stands, on the host cores: the same 53-conv + FC stack at a small batch, plus LARS."""
    import oracle
    gemm_s = 0.0
    for li, cs in enumerate(shapes.resnet50_convs()):
        c = inputs.conv_case_for(cs, sample_batch, (77, li), loss_scale=1.0)
        od = oracle.conv_desc(c.N, c.H, c.W, c.C, c.K, c.R, c.S, c.stride, c.pad)
        t1 = time.perf_counter()
        oracle.conv_fwd(od, c.x, c.w16)
        if not cs.first:
            oracle.conv_bwd_data(od, c.dy, c.w16)
        oracle.conv_bwd_weight(od, c.x, c.dy)
        gemm_s += time.perf_counter() - t1
    fc = shapes.RESNET50_FC
    f = inputs.fc_case((77, 99), sample_batch, fc.I, fc.O)
    t1 = time.perf_counter()
    oracle.fc_fwd(sample_batch, fc.I, fc.O, f.x, f.w16)
    oracle.fc_bwd_data(sample_batch, fc.I, fc.O, f.dy, f.w16)
    oracle.fc_bwd_weight(sample_batch, fc.I, fc.O, f.dy, f.x)
    gemm_s += time.perf_counter() - t1
    ps = inputs.resnet50_param_set(loss_scale=1024.0)
    t1 = time.perf_counter()
    oracle.lars_mp_update(ps.offsets, ps.flags, ps.master_w, ps.momentum, ps.grad16, ps.weight16, loss_scale=1024.0, **inputs.HPARAMS)
    lars_s = time.perf_counter() - t1
    total = gemm_s + lars_s
    return {"value": sample_batch / total, "unit": "images/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "fp64 oracle, all 53 convs + FC fwd/bwd_data/bwd_weight at N=%d (%.1f s; its backward-data routine "
                      "threads over images only) plus one LARS update over all 25,557,032 parameters (%.2f s); input "
                      "generation not timed" % (sample_batch, gemm_s, lars_s),
            "lars_gbps": LARS_BYTES_PER_PARAM * ps.P / lars_s / 1e9}


def time_steps(wl, stream, side, steps, warmup, graph=0):
    """`warmup` untimed steps, then `steps` timed ones: host wall clock around all of them (the reported ms_per_step)
    and HIP events on the launch stream around the GEMM phase and the LARS update of every step."""
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    with torch.cuda.stream(stream):
        for _ in range(max(warmup, 1)):
            wl.run_gemms(side)
            wl.run_lars()
        stream.synchronize()
        graphs = None
        if graph:
            # two graphs (GEMM phase, LARS phase) so that HIP events can separate the phases between replays
            g1, g2 = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
            with torch.cuda.graph(g1, stream=stream):
                wl.run_gemms(side)
            with torch.cuda.graph(g2, stream=stream):
                wl.run_lars()
            graphs = (g1, g2)
            for _ in range(2):
                g1.replay(); g2.replay()
            stream.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            ev[k][0].record(stream)
            if graphs:
                graphs[0].replay()
            else:
                wl.run_gemms(side)
            ev[k][1].record(stream)
            if graphs:
                graphs[1].replay()
            else:
                wl.run_lars()
            ev[k][2].record(stream)
        stream.synchronize()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    assert int(wl.found_inf.item()) == 0
    g = np.array([e[0].elapsed_time(e[1]) for e in ev])
    l = np.array([e[1].elapsed_time(e[2]) for e in ev])
    return {"wall_ms": wall * 1e3 / steps, "gemm_ms": float(g.mean()), "gemm_ms_median": float(np.median(g)), "gemm_ms_min": float(g.min()),
            "lars_ms": float(l.mean()), "lars_ms_median": float(np.median(l)), "lars_ms_min": float(l.min()),
            "step_ms_mean": float((g + l).mean()), "step_ms_median": float(np.median(g + l)), "step_ms_min": float((g + l).min())}


def plans_digest(wl):
    """A fingerprint of how the library would run every launch of the step (kernel variant, tiles, splits per layer and
    op): a traffic figure measured under one set of plans says nothing about another."""
    import hashlib
    hsh = hashlib.sha256()
    B, I, O = wl.N, wl.fc.I, wl.fc.O
    for L in wl.layers:
        for op in (api.JZ_FWD, api.JZ_BWD_DATA, api.JZ_BWD_WEIGHT):
            if L.get("first") and op == api.JZ_BWD_DATA:
                continue
            d = L["d"] if L["kind"] == "conv" else api.conv_desc(B, 1, 1, I, O, 1, 1)
            hsh.update(api.jz_conv2d_describe_plan(op, d).encode())
    return hsh.hexdigest()[:16]


TRAFFIC_PROFILE = "profiles/bench_resnet50_n64_hbm_traffic.txt"


def measured_traffic(wl):
    """HBM bytes per step from the rocprofv3 counter summary under profiles/ (FETCH_SIZE / WRITE_SIZE, copy-kernel
    scaled), but only if that summary was taken with the kernel plans this run uses: the summary records their digest."""
    import os
    import re
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), TRAFFIC_PROFILE)
    if not os.path.exists(path):
        return None
    text = open(path).read()
    m = re.search(r"^# machine-readable: plans_digest=(\w+) gemm_phase_hbm_bytes_per_step=([\d.e+]+) lars_hbm_bytes_per_update=([\d.e+]+)", text, re.M)
    if not m or m.group(1) != plans_digest(wl):
        return None
    return {"bytes": float(m.group(2)), "lars_bytes": float(m.group(3)),
            "note": "HBM bytes per step of all these launches from %s (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, copy-kernel scaled), "
                    "taken with the same kernel plans as this run (digest %s)" % (TRAFFIC_PROFILE, m.group(1))}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--batch", type=int, default=None, help="default: 64 (resnet50), 128 (alexnet)")
    ap.add_argument("--workload", default="resnet50", choices=("resnet50", "alexnet", "bn", "chain"),
                    help="resnet50: the full step the headline metric is quoted on; alexnet: the AlexNet-shaped layers of configs[3]; "
                         "bn: the batch-normalization + ReLU layers of ResNet-50 (not part of the headline step); chain: a complete chained "
                         "ResNet-50 training step with every layer between the convolutions (not the headline step either)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--variant", default="v1", choices=("v1", "v1.5"),
                    help="where a stage's stride 2 sits: v1 (the network the paper cites: on the first 1x1 of the stage's first block) or "
                         "v1.5 (on its 3x3; 6 %% more multiply-adds; its shapes have no entries in the planner's table)")
    ap.add_argument("--no-alt", action="store_true", help="skip the run with the other LARS update path")
    ap.add_argument("--per-layer", action="store_true", help="also print a per-layer, per-op timing table to stderr (the ResNet-50 step does "
                    "by default: its ten launches furthest from their rooflines go into the JSON line as per_layer_worst)")
    ap.add_argument("--no-per-layer", action="store_true", help="ResNet-50 step: skip the per-layer table (about ten seconds)")
    ap.add_argument("--per-layer-file", default=None, help="write the per-layer table (time, TFLOP/s, the layer's own roofline, "
                    "fraction, kernel plan) to this file as well; implies --per-layer")
    ap.add_argument("--lars-path", default="presummed", choices=("presummed", "three_launches"),
                    help="presummed: the backward-weight launches leave each filter gradient's sum of squares with the optimiser "
                         "and the update is one launch; three_launches: jz_lars_mp_update (reduce, rates, update)")
    ap.add_argument("--sumsq-from", default="split", choices=("split", "all"),
                    help="presummed path: which backward-weight launches leave their gradient's sum of squares (see ResNet50Step)")
    ap.add_argument("--dtype", default="f16", choices=("f16", "f32"), help="f16: the mixed-precision path (the headline); f32: the "
                    "single-precision variant of the same step (Table 9's comparison)")
    ap.add_argument("--no-fp32", action="store_true", help="skip the short single-precision run that the default line reports beside the headline")
    ap.add_argument("--plans-digest", action="store_true", help="print the fingerprint of this workload's kernel plans and exit")
    ap.add_argument("--streams", type=int, default=3, help="1: everything in order on one stream; n > 1: n-1 side streams "
                    "for the projection shortcuts (forward) and the backward-weight launches (at most 4)")
    ap.add_argument("--graph", type=int, default=0, help="replay the step from a HIP graph (1) or launch eagerly (0); eager launches measured faster here")
    ap.add_argument("--no-block-end", action="store_true", help="chain workload: ReLU gradient and batch-norm backward at a block's end as two calls")
    ap.add_argument("--no-bwd-stats", action="store_true",
                    help="chain workload: backward-data convolution and the batch-norm backward underneath it as two calls")
    ap.add_argument("--unfused", action="store_true", help="chain workload: convolution and batch normalization as two calls")
    ap.add_argument("--dynamic-loss-scale", action="store_true",
                    help="time jz_lars_mp_update_dyn (loss scale and its controller on the device) instead of jz_lars_mp_update")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run ten 1 GiB device-to-device copies and exit: the known-size kernel that the HBM byte counters "
                         "(FETCH_SIZE / WRITE_SIZE under rocprofv3 --pmc) are scaled by")
    args = ap.parse_args()
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4, "copies": 10}))
        return
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives are part of it); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    api.lib()
    torch.cuda.set_device(0)
    if args.plans_digest:
        print(plans_digest(ResNet50Step(batch=args.batch or 64)))
        return
    if args.batch is None:
        args.batch = 128 if args.workload == "alexnet" else 64
    if args.workload == "alexnet":
        alexnet_workload(args)
        return
    if args.workload == "bn":
        bn_workload(args)
        return
    if args.workload == "chain":
        chain_workload(args)
        return
    wl = ResNet50Step(batch=args.batch, dtype=args.dtype, lars_path=args.lars_path, sumsq_from=args.sumsq_from, variant=args.variant)

    # loss-scale back-off: halve S until the weight gradients stay inside fp16 and the update is not skipped
    for _ in range(12):
        wl.step()
        torch.cuda.synchronize()
        if int(wl.found_inf.item()) == 0:
            break
        wl.halve_loss_scale()
    assert int(wl.found_inf.item()) == 0, "loss-scale back-off did not clear the overflow flag"
    wl.reset_state()
    if args.dynamic_loss_scale:
        wl.use_dynamic_loss_scale()

    rows = None
    if args.per_layer or args.per_layer_file or not args.no_per_layer:
        rows = per_layer_report(wl, out_path=args.per_layer_file, peak=FP32_MFMA_PEAK_TFLOPS if wl.f32 else FP16_MFMA_PEAK_TFLOPS)
        wl.reset_state()

    stream = torch.cuda.Stream()
    side = [torch.cuda.Stream() for _ in range(max(0, min(args.streams, 4) - 1))]
    t = time_steps(wl, stream, side, args.steps, args.warmup, graph=args.graph)
    gemm_ms, lars_ms, ms_per_step = t["gemm_ms"], t["lars_ms"], t["wall_ms"]
    n_gemm = sum(3 if not L.get("first") else 2 for L in wl.layers)
    default_workload = args.batch == 64 and not wl.f32
    peak = FP32_MFMA_PEAK_TFLOPS if wl.f32 else FP16_MFMA_PEAK_TFLOPS
    tflops = wl.flops / (gemm_ms * 1e-3) / 1e12
    lars_gbps = LARS_BYTES_PER_PARAM * wl.P / (lars_ms * 1e-3) / 1e9
    traffic = measured_traffic(wl) if default_workload else None
    out = {
        "metric": "ResNet-50 N=%d %s fwd+bwd images/s" % (args.batch, "fp32" if wl.f32 else "fp16"),
        "value": args.batch / (ms_per_step * 1e-3),
        "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32 storage, f32 accumulate (LARS as in the mixed-precision step)" if wl.f32 else
                 "f16 storage, f32 accumulate (LARS in f32, norms f64)",
        "data": "synthetic",
        "config": {"workload": "configs[4]: ResNet-50 %s, 53 convs + FC, fwd + bwd_data + bwd_weight per layer on "
                               "independent seeded N(0,1) inputs, then fused LARS over 161 tensors / 25,557,032 params" % args.variant,
                   "batch": args.batch, "loss_scale_after_back_off": wl.loss_scale, "loss_scale_control": "device" if args.dynamic_loss_scale else "fixed", "launch": "hip graph" if args.graph else "eager", "streams": args.streams},
        "ms_per_step_stats": {"gpu_mean": t["step_ms_mean"], "gpu_median": t["step_ms_median"], "gpu_min": t["step_ms_min"],
                              "note": "per-step HIP-event times (GEMM phase + LARS) over the timed steps; ms_per_step is host wall clock / steps"},
        "pct_fp16_mfma_peak": 100.0 * (wl.flops / (ms_per_step * 1e-3) / 1e12) / FP16_MFMA_PEAK_TFLOPS,
        "roofline": {"kernel": "%s (all %d conv/FC launches of a step)" % ("igemm_f32_kernel" if wl.f32 else "igemm_dma_kernel", n_gemm),
                     "bound": "mfma", "achieved": tflops, "peak": peak, "unit": "TFLOP/s", "frac": tflops / peak,
                     "peak_note": ("dense FP32 MFMA: 256 CU x 4 SIMD x 64 flop/clk (v_mfma_f32_32x32x2_f32) x 2.4 GHz = 157.3 TFLOP/s" if wl.f32 else
                                   "dense FP16 MFMA, the published 2.5 PFLOP/s: 256 CU x 4 SIMD x 1024 flop/clk (v_mfma_f32_32x32x16_f16) x 2.4 GHz = 2.52; "
                                   "a loop of nothing but MFMAs sustains 1.94 on this chip (effective clock 1.85 GHz)"),
                     "traffic": traffic["bytes"] if traffic else None,
                     "traffic_note": (traffic["note"] if traffic else "no HBM-counter summary under profiles/ matches this run's kernel plans") +
                                     "; algorithmic 2(|x|+|w|+|y|) per pass is 7.99e9 at fp16 storage",
                     "flop_per_step": wl.flops, "ms_per_step_gemm_phase": gemm_ms, "ms_gemm_phase_median": t["gemm_ms_median"],
                     "ms_gemm_phase_min": t["gemm_ms_min"], "avg_launch_us": gemm_ms * 1e3 / n_gemm},
        "lars": {"bound": "hbm", "achieved": lars_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": lars_gbps / HBM_PEAK_GBPS,
                 "path": "one launch, gradient norms from the backward-weight kernels' sinks" if wl.presummed else
                         "three launches (reduce, per-tensor rates, update)",
                 "bytes_per_param": LARS_BYTES_PER_PARAM, "params": wl.P, "us_per_update": lars_ms * 1e3,
                 "us_per_update_median": t["lars_ms_median"] * 1e3, "us_per_update_min": t["lars_ms_min"] * 1e3,
                 "traffic": traffic["lars_bytes"] if traffic else None},
    }
    if rows is not None:
        worst = sorted(rows, key=lambda r: r["us"] - r["us_roofline"], reverse=True)[:10]
        out["per_layer_worst"] = [{k: r[k] for k in ("layer", "shape", "op", "us", "us_roofline", "tflops", "roofline_tflops", "frac", "plan")}
                                  for r in worst]
    if wl.presummed and not args.no_alt:
        # the same step with the other update path (plain backward-weight launches, three-launch update), a run of its own:
        # what the one-launch update costs the GEMM phase and what it saves behind it
        wl3 = ResNet50Step(batch=args.batch, loss_scale=wl.loss_scale, lars_path="three_launches", variant=args.variant)   # the scale after back-off
        if args.dynamic_loss_scale:
            wl3.use_dynamic_loss_scale()
        t3 = time_steps(wl3, stream, side, args.steps, args.warmup)
        out["lars"]["three_launch_path"] = {"us_per_update": t3["lars_ms"] * 1e3, "ms_gemm_phase": t3["gemm_ms"], "ms_per_step": t3["wall_ms"],
                                            "images_per_s": args.batch / (t3["wall_ms"] * 1e-3),
                                            "note": "jz_lars_mp_update behind plain backward-weight launches, same run, same inputs"}
        del wl3
    if not wl.f32 and not args.no_fp32:
        # Table 9's comparison on this chip: the same step with the single-precision kernels (a short run of its own)
        wl32 = ResNet50Step(batch=args.batch, dtype="f32", variant=args.variant)
        t32 = time_steps(wl32, stream, side, max(3, args.steps // 4), 2)
        v32 = args.batch / (t32["wall_ms"] * 1e-3)
        tf32 = wl32.flops / (t32["gemm_ms"] * 1e-3) / 1e12
        out["fp32_variant"] = {"value": v32, "unit": "images/s", "ms_per_step": t32["wall_ms"], "steps": max(3, args.steps // 4),
                               "achieved": tf32, "peak": FP32_MFMA_PEAK_TFLOPS, "frac": tf32 / FP32_MFMA_PEAK_TFLOPS,
                               "mixed_over_fp32": out["value"] / v32,
                               "paper_table9": {"fp32_images_per_s": 172, "mixed_images_per_s": 218, "ratio": 218.0 / 172.0,
                                                "hardware": "one Tesla P40 node (no FP16 matrix units)"}}
        del wl32
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
