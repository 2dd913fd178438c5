"""A chained ResNet-50 training step as a sequence of libjz calls (sequencing and buffer bookkeeping only: every
arithmetic step runs in the library's kernels).

One step = forward through the 53 convolutions with training-mode batch normalization (+ ReLU), the stem max pool,
the residual adds, the global average pool and the classifier; softmax cross-entropy gradient times the loss scale
(Section 4.1 of Jia et al. 2018); backward through all of it into the fused FP16 gradient buffer; the mixed-precision
LARS update with the device-resident dynamic loss scale.  The network is the stock ResNet-50 the paper trains
(Table 3); gamma, beta and the bias are exempt from weight decay (Section 4.2) through the parameter flags.

Every intermediate tensor has a buffer of its own and every launch is recorded in `self.trace` with the tensors it
read and wrote, so that a test can check each launch against an independent implementation on the inputs that launch
actually saw.
"""
from typing import List

import numpy as np
import torch

from . import api, inputs, shapes

BN_EPS = 1e-5


class Op:
    """One library call of the step: what it is, the tensors it reads and writes, and the launch itself."""

    __slots__ = ("kind", "name", "params", "ins", "outs", "call", "side_call", "lane", "joins_side")

    def __init__(self, kind, name, params, ins, outs, call, side_call=None):
        self.kind, self.name, self.params, self.ins, self.outs, self.call = kind, name, params, ins, outs, call
        self.side_call = side_call      # workspace -> the same launch bound to that workspace, for a side stream
        self.lane = "main"              # "side": a weight gradient, "proj": the projection-shortcut branch (both may run on a side stream)
        self.joins_side = False         # reads what the side stream's projection branch wrote: waits for it


class ResNet50Chain:
    def __init__(self, batch=64, image=224, variant="v1", seed=180711205, initial_loss_scale=1024.0, hparams=None,
                 policy=None, device="cuda:0", fused=True, block_end=True, proj_side=False, presummed=True, bwd_stats=True):
        """fused: forward convolution + batch normalization as one call (statistics in the convolution's epilogue)
        instead of two.  bwd_stats (with fused): a backward-data convolution and the batch-norm backward that consumes its
        output as one call (the statistics of that backward in the convolution's epilogue).  presummed: the weight-gradient GEMMs whose reduction is split leave their gradient's sum of squares
        in the optimiser's workspace (from inside the kernel that adds the partial sums), the remaining tensors' sums are
        taken by one launch behind the last gradient of the backward pass, and the update is one launch (else: the update's
        own reduce pass reads every gradient again, three launches)."""
        self.presummed = bool(presummed)
        self.N, self.image, self.device, self.fused = int(batch), int(image), torch.device(device), bool(fused)
        self.block_end = bool(block_end) and self.fused
        self.bwd_stats = bool(bwd_stats) and self.fused
        self.proj_side = bool(proj_side)      # projection-shortcut branches on the side stream too (measured: no gain)
        self.convs = shapes.resnet50_convs(variant, image)
        self.fc = shapes.RESNET50_FC
        self.hp = dict(inputs.HPARAMS)
        self.hp.update(hparams or {})
        h, f = torch.float16, torch.float32
        dev = self.device

        # parameters: FP32 master weights, momentum, FP16 working copy and FP16 gradients, one fused buffer each
        host = inputs.resnet50_param_set(loss_scale=1.0, seed_key=(seed % 1000003,), variant=variant)
        self.tensors = shapes.resnet50_param_tensors(variant)
        self.offsets = [int(o) for o in host.offsets]
        self.flags = [int(x) for x in host.flags]
        self.index = {name: i for i, (name, _, _, _) in enumerate(self.tensors)}
        if self.presummed:      # filters whose weight-gradient reduction is split: their producer supplies the sum of squares
            for cs in self.convs:
                d = api.conv_desc(self.N, cs.H, cs.H, cs.C, cs.K, cs.R, cs.R, cs.stride, cs.pad)
                if ", 1 splits" not in api.jz_conv2d_describe_plan(api.JZ_BWD_WEIGHT, d):
                    self.flags[self.index[cs.name + ".w"]] |= api.JZ_PARAM_GRAD_PRESUMMED
            d = api.conv_desc(self.N, 1, 1, self.fc.I, self.fc.O, 1, 1)
            if ", 1 splits" not in api.jz_conv2d_describe_plan(api.JZ_BWD_WEIGHT, d):
                self.flags[self.index["fc.w"]] |= api.JZ_PARAM_GRAD_PRESUMMED
        self.master = torch.from_numpy(host.master_w).to(dev)
        self.momentum = torch.zeros_like(self.master)
        self.w16 = self.master.to(h)
        self.grad = torch.zeros(self.master.numel(), dtype=h, device=dev)
        self.ps = api.ParamSet(self.offsets, self.flags, self.master, self.momentum, self.grad, self.w16)
        self.lars_ws = torch.zeros(max(api.jz_lars_workspace_bytes(self.ps), 16), dtype=torch.uint8, device=dev)
        api.jz_lars_prepare(self.ps, self.lars_ws)
        self.found_inf = torch.zeros(1, dtype=torch.int32, device=dev)
        self.ls_state = torch.zeros(2, dtype=torch.int32, device=dev)
        self.policy = api.loss_scale_policy(**(policy or {}))
        api.jz_loss_scale_init(self.ls_state, initial_loss_scale)

        # data: a fixed synthetic batch
        g = torch.Generator(device="cpu").manual_seed(seed)
        self.x = torch.randn(self.N * image * image * 3, generator=g, dtype=f).to(h).to(dev)
        self.labels = torch.randint(0, self.fc.O, (self.N,), generator=g, dtype=torch.int32).to(dev)
        self.loss = torch.zeros(self.N, dtype=f, device=dev)

        self._ws_bytes = 16
        self._pending_ws = []
        self.fwd_ops: List[Op] = []
        self.bwd_ops: List[Op] = []
        self._build()
        if self.presummed:
            # first launch of a step: clear the gradient sinks, add up the carried sums of squares of the weights, note the
            # loss scale; last launch of the backward pass: the tensors no GEMM produces (batch-norm scale / shift, bias)
            self.fwd_ops.insert(0, Op("lars_begin", "begin", {}, [], [],
                                      lambda stream=None: api.jz_lars_begin_step(self.ps, self.lars_ws, self.ls_state, stream)))
            self.bwd_ops.append(Op("lars_grad_sumsq", "rest", {}, [self.grad], [],
                                   lambda stream=None: api.jz_lars_grad_sumsq(self.ps, 0, self.ps.T, self.lars_ws, stream)))
        self.ws = torch.zeros(self._ws_bytes, dtype=torch.uint8, device=dev)
        self.side_ws = []               # one workspace per side stream, made on first use
        self._side_calls = {}
        self._events = {}
        for bind in self._pending_ws:
            bind(self.ws)
        self.trace = self.fwd_ops + self.bwd_ops + [self._lars_op()]

    # ---- buffers and parameter views --------------------------------------------------------------------------------
    def _buf(self, n, dtype=torch.float16):
        return torch.zeros(int(n), dtype=dtype, device=self.device)

    def _param(self, buf, name):
        i = self.index[name]
        return buf[self.offsets[i]:self.offsets[i + 1]]

    # ---- op constructors ---------------------------------------------------------------------------------------------
    def _later(self, make):
        """Calls that need the shared workspace are bound once its size is known."""
        box = {}
        self._pending_ws.append(lambda ws: box.__setitem__("call", make(ws)))
        return lambda stream=None: box["call"](stream)

    def _conv(self, op, cs, a, b, out, name):
        d = api.conv_desc(self.N, cs.H, cs.H, cs.C, cs.K, cs.R, cs.R, cs.stride, cs.pad)
        self._ws_bytes = max(self._ws_bytes, api.jz_conv2d_workspace_bytes(op, d))
        kind = {api.JZ_FWD: "conv_fwd", api.JZ_BWD_DATA: "conv_bwd_data", api.JZ_BWD_WEIGHT: "conv_bwd_weight"}[op]
        bind = lambda ws: api.bind_conv2d(op, d, a, b, out, ws)
        if op == api.JZ_BWD_WEIGHT and self.presummed and self.flags[self.index[name + ".w"]] & api.JZ_PARAM_GRAD_PRESUMMED:
            sink = api.jz_lars_sumsq_sink(self.ps, self.lars_ws, self.index[name + ".w"])
            bind = lambda ws: api.bind_conv2d_bwd_weight_sumsq(d, a, b, out, sink, ws)
        o = Op(kind, name, dict(desc=d), [a, b], [out], self._later(bind), bind)
        if op == api.JZ_BWD_WEIGHT:
            o.lane = "side"
        return o

    def _fc(self, mode, a, b, out, name):
        B, I, O = self.N, self.fc.I, self.fc.O
        self._ws_bytes = max(self._ws_bytes, api.jz_gemm_fc_workspace_bytes(mode, B, I, O))
        kind = {api.JZ_FWD: "fc_fwd", api.JZ_BWD_DATA: "fc_bwd_data", api.JZ_BWD_WEIGHT: "fc_bwd_weight"}[mode]
        bind = lambda ws: api.bind_gemm_fc(mode, B, I, O, a, b, out, ws)
        if mode == api.JZ_BWD_WEIGHT and self.presummed and self.flags[self.index[name + ".w"]] & api.JZ_PARAM_GRAD_PRESUMMED:
            sink = api.jz_lars_sumsq_sink(self.ps, self.lars_ws, self.index[name + ".w"])
            bind = lambda ws: api.bind_gemm_fc_bwd_weight_sumsq(B, I, O, a, b, out, sink, ws)
        o = Op(kind, name, dict(B=B, I=I, O=O), [a, b], [out], self._later(bind), bind)
        if mode == api.JZ_BWD_WEIGHT:
            o.lane = "side"
        return o

    def _bn_fwd(self, cs, x, y, relu, name):
        rows, C = self.N * cs.P * cs.P, cs.K
        gamma, beta = self._param(self.master, cs.name + ".gamma"), self._param(self.master, cs.name + ".beta")
        mean, invstd = self._buf(C, torch.float32), self._buf(C, torch.float32)
        self._ws_bytes = max(self._ws_bytes, api.jz_bn_workspace_bytes(rows, C))
        run = lambda ws, stream: api.jz_bn_relu_fwd(rows, C, x, gamma, beta, BN_EPS, relu, y, mean, invstd, ws, stream)
        return Op("bn_fwd", name, dict(rows=rows, C=C, relu=relu, eps=BN_EPS), [x, gamma, beta], [y, mean, invstd],
                  lambda stream=None: run(self.ws, stream), lambda ws: (lambda stream=None: run(ws, stream))), mean, invstd

    def _conv_bn_fwd(self, cs, x, w, c, y, relu, residual=None):
        d = api.conv_desc(self.N, cs.H, cs.H, cs.C, cs.K, cs.R, cs.R, cs.stride, cs.pad)
        rows, C = self.N * cs.P * cs.P, cs.K
        gamma, beta = self._param(self.master, cs.name + ".gamma"), self._param(self.master, cs.name + ".beta")
        mean, invstd = self._buf(C, torch.float32), self._buf(C, torch.float32)
        self._ws_bytes = max(self._ws_bytes, api.jz_conv2d_bn_relu_fwd_workspace_bytes(d))
        run = lambda ws, stream: api.jz_conv2d_bn_relu_fwd(d, x, w, gamma, beta, BN_EPS, relu, c, y, mean, invstd, ws, residual, stream)
        return Op("conv_bn_fwd", cs.name, dict(desc=d, rows=rows, C=C, relu=relu, eps=BN_EPS), [x, w, gamma, beta, residual],
                  [c, y, mean, invstd], lambda stream=None: run(self.ws, stream),
                  lambda ws: (lambda stream=None: run(ws, stream))), mean, invstd

    def _block_end(self, cs, x, mean, invstd, dx, end, name):
        """ReLU gradient of the block output (one or two incoming contributions, named in `end`) and the batch-norm
        backward of branch c in one call; end["g"] receives the gradient of the sum for the shortcut branch."""
        rows, C = self.N * cs.P * cs.P, cs.K
        gamma = self._param(self.master, cs.name + ".gamma")
        dgamma, dbeta = self._param(self.grad, cs.name + ".gamma"), self._param(self.grad, cs.name + ".beta")
        op = Op("bn_bwd_block_end", name, dict(rows=rows, C=C), [x, end["out"], end["dya"], end["dyb"], gamma, mean, invstd],
                [end["g"], dx, dgamma, dbeta], None)
        op.call = lambda stream=None: api.jz_bn_bwd_block_end(rows, C, x, end["out"], end["dya"], end["dyb"], gamma, mean, invstd, end["g"],
                                                              dx, dgamma, dbeta, self.ws, stream)
        end["op"] = op
        return op

    def _bn_bwd(self, cs, x, y, dy, mean, invstd, dx, relu, name):
        rows, C = self.N * cs.P * cs.P, cs.K
        gamma = self._param(self.master, cs.name + ".gamma")
        dgamma, dbeta = self._param(self.grad, cs.name + ".gamma"), self._param(self.grad, cs.name + ".beta")
        run = lambda ws, stream: api.jz_bn_relu_bwd(rows, C, x, y if relu else None, dy, gamma, mean, invstd, relu, dx, dgamma, dbeta,
                                                    ws, stream)
        return Op("bn_bwd", name, dict(rows=rows, C=C, relu=relu), [x, y, dy, gamma, mean, invstd], [dx, dgamma, dbeta],
                  lambda stream=None: run(self.ws, stream), lambda ws: (lambda stream=None: run(ws, stream)))

    def _fuse_bwd_pairs(self, seg):
        """A backward-data convolution directly followed by the batch-norm (+ ReLU) backward that reads its output becomes
        one call, jz_conv2d_bwd_data_bn_relu_bwd."""
        out, i = [], 0
        while i < len(seg):
            a = seg[i]
            b = seg[i + 1] if i + 1 < len(seg) else None
            if (a.kind == "conv_bwd_data" and b is not None and b.kind == "bn_bwd" and b.params["relu"] and b.lane == a.lane == "main"
                    and b.ins[2].data_ptr() == a.outs[0].data_ptr()):
                d = a.params["desc"]
                dy, w = a.ins
                x, y, dz, gamma, mean, invstd = b.ins
                dx, dgamma, dbeta = b.outs
                self._ws_bytes = max(self._ws_bytes, api.jz_conv2d_bwd_data_bn_relu_bwd_workspace_bytes(d))
                run = lambda stream=None, t=(d, dy, w, x, y, gamma, mean, invstd, dz, dx, dgamma, dbeta): \
                    api.jz_conv2d_bwd_data_bn_relu_bwd(*t, self.ws, stream)
                op = Op("conv_bwd_data_bn_bwd", a.name + " + " + b.name, dict(desc=d, rows=b.params["rows"], C=b.params["C"]),
                        [dy, w, x, y, gamma, mean, invstd], [dz, dx, dgamma, dbeta], run)
                op.joins_side = a.joins_side or b.joins_side
                out.append(op)
                i += 2
            elif (a.kind == "conv_bwd_data" and b is not None and b.kind == "bn_bwd_block_end" and b.lane == a.lane == "main"
                    and b.ins[2].data_ptr() == a.outs[0].data_ptr()):
                # the first convolution of a block and the end of the block underneath: the convolution's result is one of the
                # two contributions to that block's output gradient and is never stored
                d = a.params["desc"]
                dy, w = a.ins
                x, y_out, _, dyb, gamma, mean, invstd = b.ins
                g, dx, dgamma, dbeta = b.outs
                self._ws_bytes = max(self._ws_bytes, api.jz_conv2d_bwd_data_bn_relu_bwd_workspace_bytes(d))
                run = lambda stream=None, t=(d, dy, w, dyb, x, y_out, gamma, mean, invstd, g, dx, dgamma, dbeta): \
                    api.jz_conv2d_bwd_data_block_end_bwd(*t, self.ws, stream)
                op = Op("conv_bwd_data_block_end", a.name + " + " + b.name, dict(desc=d, rows=b.params["rows"], C=b.params["C"]),
                        [dy, w, dyb, x, y_out, gamma, mean, invstd], [g, dx, dgamma, dbeta], run)
                op.joins_side = a.joins_side or b.joins_side
                out.append(op)
                i += 2
            else:
                out.append(a)
                i += 1
        return out

    # ---- the network -------------------------------------------------------------------------------------------------
    def _build(self):
        N, F = self.N, self.fwd_ops
        segments = []                            # backward ops per network segment, each list in execution order
        by_name = {cs.name: cs for cs in self.convs}
        W = lambda cs: self._param(self.w16, cs.name + ".w")
        DW = lambda cs: self._param(self.grad, cs.name + ".w")

        def conv_bn(cs, x_in, dx_in, relu, dz=None, residual=None, end=None):
            """conv -> batch norm (-> ReLU), appended to the forward list.  Returns (z, dz, back): the output, the buffer
            the consumer of z writes z's gradient to, and this pair's backward ops in execution order.  dx_in is where
            the gradient with respect to x_in goes (None for the first layer)."""
            n_out = N * cs.P * cs.P * cs.K
            c, z, dc = self._buf(n_out), self._buf(n_out), self._buf(n_out)
            dz = self._buf(n_out) if dz is None else dz
            if self.fused:     # with a residual: z = relu(bn(c) + residual), the block's output
                op, mean, invstd = self._conv_bn_fwd(cs, x_in, W(cs), c, z, relu or residual is not None, residual)
                F.append(op)
            else:
                F.append(self._conv(api.JZ_FWD, cs, x_in, W(cs), c, cs.name))
                op, mean, invstd = self._bn_fwd(cs, c, z, relu, cs.name + ".bn")
                F.append(op)
            if end is not None:   # block end: the ReLU gradient of z and this batch-norm backward are one call
                end["out"] = z
                first = self._block_end(cs, c, mean, invstd, dc, end, cs.name + ".bn")
            else:
                first = self._bn_bwd(cs, c, z if relu else None, dz, mean, invstd, dc, relu, cs.name + ".bn")
            back = [first, self._conv(api.JZ_BWD_WEIGHT, cs, x_in, dc, DW(cs), cs.name)]
            if dx_in is not None:
                back.append(self._conv(api.JZ_BWD_DATA, cs, dc, W(cs), dx_in, cs.name))
            return z, dz, back

        def add_op(name, a, b, out, relu):
            return Op("add_fwd", name, dict(relu=relu), [a, b], [out], lambda stream=None: api.jz_add_fwd(a, b, out, relu, stream))

        stem = self.convs[0]
        a0, da0, back_stem = conv_bn(stem, self.x, None, True)
        Hp = stem.P
        Hq = api.pool_out(Hp, 3, 2, 1)
        pool = dict(N=N, H=Hp, W=Hp, C=64, window=3, stride=2, pad=1)
        cur, dcur = self._buf(N * Hq * Hq * 64), self._buf(N * Hq * Hq * 64)
        arg = self._buf(N * Hq * Hq * 64, torch.uint8)     # each window's winner, saved for the backward pass
        F.append(Op("maxpool_fwd", "pool1", pool, [a0], [cur, arg],
                    lambda stream=None, y=cur: api.jz_maxpool_fwd(N, Hp, Hp, 64, 3, 2, 1, a0, y, arg, stream)))
        segments.append([Op("maxpool_bwd", "pool1", pool, [a0, dcur, arg], [da0],
                            lambda stream=None, dy=dcur: api.jz_maxpool_bwd(N, Hp, Hp, 64, 3, 2, 1, None, dy, da0, arg, stream))] + back_stem)

        blocks = sorted({cs.name[:-1] for cs in self.convs[1:]}, key=lambda n: (int(n[1]), int(n[3:])))
        below = None      # the block underneath (fused form): where its ReLU gradient takes its incoming gradient(s) from
        for nm in blocks:
            a, b, c = by_name[nm + "a"], by_name[nm + "b"], by_name[nm + "c"]
            p = by_name.get(nm + "p")
            x_in, dx_out = cur, dcur                       # dx_out: gradient of the block input, read by the segment below
            dxa = self._buf(x_in.numel())                  # branch a's contribution to it
            n_out = N * c.P * c.P * c.K
            ds = self._buf(n_out)                          # gradient of the sum in front of the block's last ReLU
            if p is not None:      # the projection shortcut first: on a side stream it runs beside branch a - b
                dxp = self._buf(x_in.numel())
                n_fwd = len(F)
                shortcut, _, back_p = conv_bn(p, x_in, dxp, False, dz=ds)
                for o in F[n_fwd:] + back_p:
                    o.lane = "proj"
                dshort = dxp
            else:
                shortcut, back_p, dshort = x_in, [], ds
            za, dza, back_a = conv_bn(a, x_in, dxa, True)
            zb, dzb, back_b = conv_bn(b, za, dza, True)
            dout = self._buf(n_out)
            end = None
            if self.fused:     # the residual add and the block's ReLU happen in the normalization pass of branch c
                end = dict(dya=dout, dyb=None, g=ds, at=(2, 3))
                out, _, back_c = conv_bn(c, zb, dzb, False, dz=ds, residual=shortcut, end=end if self.block_end else None)
                if back_p:
                    F[-1].joins_side = True        # the residual is the projection branch's output
                if self.block_end:     # ... and the ReLU gradient in the statistics pass of branch c's backward
                    seg = back_c[:1] + back_p + back_c[1:] + back_b + back_a
                else:
                    op = Op("relu_bwd", nm + ".add", {}, [out, dout, None], [ds], None)
                    op.call = lambda stream=None, e=end, y=out: (
                        api.jz_relu_bwd_sum(y, e["dya"], e["dyb"], e["g"], stream) if e["dyb"] is not None
                        else api.jz_relu_bwd(y, e["dya"], e["g"], stream))
                    end["op"], end["at"] = op, (1, 2)
                    seg = [op] + back_p + back_c + back_b + back_a
            else:
                zc, _, back_c = conv_bn(c, zb, dzb, False, dz=ds)
                out = self._buf(n_out)
                F.append(add_op(nm + ".add", zc, shortcut, out, True))
                F[-1].joins_side = bool(back_p)
                seg = [Op("relu_bwd", nm + ".add", {}, [out, dout], [ds],
                          lambda stream=None, y=out, dy=dout, dx=ds: api.jz_relu_bwd(y, dy, dx, stream))] + back_p + back_c + back_b + back_a
            if self.fused and below is not None:
                # the two contributions to this block's input gradient are added inside the ReLU gradient of the block
                # underneath (which runs after this segment) instead of by a launch of their own
                below["dya"], below["dyb"] = dxa, dshort
                i, j = below["at"]
                below["op"].ins[i], below["op"].ins[j] = dxa, dshort
                below["op"].joins_side = bool(back_p)   # dshort then comes from the projection branch
                if below["op"].kind == "relu_bwd":
                    below["op"].kind = "relu_bwd_sum"
            else:
                seg.append(add_op(nm + ".dx", dxa, dshort, dx_out, False))
                seg[-1].joins_side = bool(back_p)
            segments.append(self._fuse_bwd_pairs(seg) if self.bwd_stats else seg)
            below = end
            cur, dcur = out, dout

        last = by_name[blocks[-1] + "c"]
        HW, C = last.P * last.P, last.K
        pooled, dpooled = self._buf(N * C), self._buf(N * C)
        F.append(Op("avgpool_fwd", "pool5", dict(N=N, HW=HW, C=C), [cur], [pooled],
                    lambda stream=None, x=cur: api.jz_avgpool_fwd(N, HW, C, x, pooled, stream)))
        O = self.fc.O
        fw, fb = self._param(self.w16, "fc.w"), self._param(self.w16, "fc.b")
        dfw, dfb = self._param(self.grad, "fc.w"), self._param(self.grad, "fc.b")
        raw, self.logits, self.dlogits = self._buf(N * O), self._buf(N * O), self._buf(N * O)
        F.append(self._fc(api.JZ_FWD, pooled, fw, raw, "fc"))
        F.append(Op("bias_add", "fc.b", dict(rows=N, C=O), [raw, fb], [self.logits],
                    lambda stream=None: api.jz_bias_add(N, O, raw, fb, self.logits, stream)))
        F.append(Op("softmax_xent", "loss", dict(rows=N, classes=O), [self.logits, self.labels, self.ls_state], [self.dlogits, self.loss],
                    lambda stream=None: api.jz_softmax_xent_bwd(N, O, self.logits, self.labels, self.dlogits, self.loss,
                                                                state=self.ls_state, stream=stream)))
        segments.append([Op("bias_grad", "fc.b", dict(rows=N, C=O), [self.dlogits], [dfb],
                            lambda stream=None: api.jz_bias_grad(N, O, self.dlogits, dfb, stream)),
                         self._fc(api.JZ_BWD_WEIGHT, self.dlogits, pooled, dfw, "fc"),
                         self._fc(api.JZ_BWD_DATA, self.dlogits, fw, dpooled, "fc"),
                         Op("avgpool_bwd", "pool5", dict(N=N, HW=HW, C=C), [dpooled], [dcur],
                            lambda stream=None, dx=dcur: api.jz_avgpool_bwd(N, HW, C, dpooled, dx, stream))])
        for seg in reversed(segments):
            self.bwd_ops.extend(seg)
        if self.bwd_stats and self.block_end:     # pairs across block boundaries: a block's first convolution + the end of the block below
            self.bwd_ops = self._fuse_bwd_pairs(self.bwd_ops)
        if not self.proj_side:     # the projection branches stay on the main stream, their weight gradients go with the others
            for o in self.fwd_ops + self.bwd_ops:
                if o.lane == "proj":
                    o.lane = "side" if o.kind.endswith("bwd_weight") else "main"

    def _lars_op(self):
        hp = api.lars_hparams(self.hp["lr"], self.hp["momentum"], self.hp["weight_decay"], self.hp["trust_coef"], 1.0)
        fn = api.jz_lars_mp_update_presummed_dyn if self.presummed else api.jz_lars_mp_update_dyn
        call = lambda stream=None: fn(self.ps, hp, self.policy, self.ls_state, self.found_inf, self.lars_ws, stream)
        return Op("lars_dyn", "update", dict(hp=dict(self.hp)), [self.master, self.momentum, self.grad, self.w16, self.ls_state],
                  [self.master, self.momentum, self.w16, self.found_inf, self.ls_state], call)

    # ---- running -----------------------------------------------------------------------------------------------------
    def _run(self, ops, stream, side, which):
        """Launches ops in order; with side streams, those of lane "side" go there round-robin (each after an event that
        says the main stream has produced what it reads), and an op that reads the projection branch's output first
        waits for the side streams.  which: "fwd" or "bwd" (keys of the pre-created events)."""
        if side is None:
            for op in ops:
                op.call(stream)
            return
        sides = list(side) if isinstance(side, (list, tuple)) else [side]
        while len(self.side_ws) < len(sides):
            self.side_ws.append(torch.zeros(self._ws_bytes, dtype=torch.uint8, device=self.device))
        main = stream if stream is not None else torch.cuda.current_stream()

        def event(key):
            ev = self._events.get(key)
            if ev is None:
                ev = self._events[key] = torch.cuda.Event()
            return ev

        k, dirty = 0, [False] * len(sides)
        for i, op in enumerate(ops):
            if op.lane == "main":
                if op.joins_side:
                    for j, s_ in enumerate(sides):
                        if dirty[j]:
                            ev = event((which, "join", i, j))
                            ev.record(s_)
                            main.wait_event(ev)
                op.call(main)
                continue
            # weight gradients go round-robin; the projection branches (their weight gradients included) stay in order
            # on the first side stream
            j = 0
            if op.lane == "side":
                j = k % len(sides)
                k += 1
            call = self._side_calls.get((which, i, j))
            if call is None:
                call = self._side_calls[(which, i, j)] = op.side_call(self.side_ws[j])
            ev = event((which, i))
            ev.record(main)                 # what this op reads has just been produced on the main stream
            sides[j].wait_event(ev)
            call(sides[j])
            dirty[j] = True
        for j, s_ in enumerate(sides):
            if dirty[j]:
                done = event((which, "done", j))
                done.record(s_)
                main.wait_event(done)

    def forward(self, stream=None, side=None):
        """With side streams the projection-shortcut branch of a stage's first block runs beside branch a - b."""
        self._run(self.fwd_ops, stream, side, "fwd")

    def backward(self, stream=None, side=None):
        """With side streams the weight-gradient GEMMs (which nothing in the backward pass waits for) and the backward
        of the projection-shortcut branches run there, beside the chain of activation gradients."""
        self._run(self.bwd_ops, stream, side, "bwd")

    def update(self, stream=None):
        self.trace[-1].call(stream)

    def step(self, stream=None, side=None):
        self.forward(stream, side)
        self.backward(stream, side)
        self.update(stream)

    def set_batch(self, images16: torch.Tensor, labels: torch.Tensor, stream=None):
        """Copies a new mini-batch (FP16 NHWC images, int32 labels) into the buffers the launches are bound to."""
        if images16.dtype != torch.float16 or images16.numel() != self.x.numel() or labels.numel() != self.N:
            raise ValueError("expected %d FP16 image values and %d labels" % (self.x.numel(), self.N))
        with torch.cuda.stream(stream if stream is not None else torch.cuda.current_stream()):
            self.x.copy_(images16.reshape(-1), non_blocking=True)
            self.labels.copy_(labels.reshape(-1).to(torch.int32), non_blocking=True)

    def mean_loss(self) -> float:
        torch.cuda.synchronize()
        return float(self.loss.double().mean().item())

    def flops_per_step(self) -> float:
        """Multiply-adds x 2 of the convolution / classifier GEMMs: forward, backward-data (not for the first layer) and
        backward-weight."""
        macs = sum(cs.macs(self.N) * (2 if cs.first else 3) for cs in self.convs) + 3 * self.fc.macs(self.N)
        return 2.0 * macs
