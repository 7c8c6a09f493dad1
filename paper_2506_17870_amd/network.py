"""A whole quantised CNN on the nested-integer path: ResNet-101 shaped (bottleneck blocks
[3, 4, 23, 3], stride on the 3x3 convolution, batch norm folded into a bias), random He-normal
weights, every layer INT-n nesting INT-h.  The paper evaluates such CNNs with 8-bit activations
(Sec. 4.1, 4.2) and switches the whole model between full-bit and part-bit by paging every
layer's lower-bit page (Sec. 3.3); it gives no layer code, so the graph below is this
repository's reading.

This module only describes the graph and walks it, handing each layer to the C ABI
(`nq_conv_*`, `nq_gemm_*`, `nq_maxpool_i8`, `nq_avgpool_i8`).  Nothing is computed in Python:
residual add, ReLU and requantisation are part of the fused epilogue.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as nq
from . import inputs


def resnet101_plan(num_classes: int = 1000):
    """Layer table.  Tensors are numbered; every op names its input/output tensor ids."""
    ops = []
    t = 0  # tensor 0 = network input, NHWC int8, 3 channels

    def conv(src, cin, cout, k, stride, pad, relu, residual=None):
        nonlocal t
        t += 1
        ops.append(dict(op="conv", src=src, dst=t, cin=cin, cout=cout, k=k, stride=stride, pad=pad, relu=relu,
                        residual=residual))
        return t

    x = conv(0, 3, 64, 7, 2, 3, True)
    t += 1
    ops.append(dict(op="maxpool", src=x, dst=t, k=3, stride=2, pad=1))
    x = t
    cin = 64
    for width, blocks, stride in ((64, 3, 1), (128, 4, 2), (256, 23, 2), (512, 3, 2)):
        for b in range(blocks):
            s = stride if b == 0 else 1
            skip = x
            if b == 0:
                skip = conv(x, cin, 4 * width, 1, s, 0, False)          # projection shortcut
            a = conv(x, cin, width, 1, 1, 0, True)
            m = conv(a, width, width, 3, s, 1, True)
            x = conv(m, width, 4 * width, 1, 1, 0, True, residual=skip)  # add + ReLU in the epilogue
            cin = 4 * width
    t += 1
    ops.append(dict(op="avgpool", src=x, dst=t))
    x = t
    t += 1
    ops.append(dict(op="fc", src=x, dst=t, cin=cin, cout=num_classes))
    return ops


def plan_float_weights(ops, seed: int = 0):
    """fp32 He-normal weights [Cout, KH*KW*Cin] and a small bias for every conv / fc of the plan (NumPy draws)."""
    out = []
    for i, op in enumerate(ops):
        if op["op"] not in ("conv", "fc"):
            out.append(None)
            continue
        k = op.get("k", 1)
        K = k * k * op["cin"]
        w = inputs.float_weights(op["cout"], K, inputs.he_sigma(K), seed=seed + i)
        bias = inputs.small_floats(op["cout"], 0.02, seed=seed + 7 * i)
        out.append((w, bias))
    return out


def quantize_tensor(x_float, n_bits: int = 8):
    """Per-tensor int8 codes of an fp32 activation tensor (NumPy or torch), on the device (nq_quantize_tensor,
    Eq. 1).  Returns (codes, cuda int8, same shape; step, float)."""
    d_x = torch.as_tensor(x_float, dtype=torch.float32).cuda().contiguous()
    codes = torch.empty(d_x.shape, dtype=torch.int8, device="cuda")
    step = torch.empty(1, dtype=torch.float32, device="cuda")
    nq.nq_quantize_tensor(d_x, d_x.numel(), n_bits, codes, step)
    return codes, float(step.cpu()[0])


def out_hw(h, w, k, stride, pad):
    return (h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1


class NestedCNN:
    """Device-side owner of the nested weights of a plan and walker of the graph."""

    def __init__(self, ops, weights, n_bits=8, l_bits=2):
        """weights: per op None or (fp32 weights [N,K], fp32 bias [N]), as plan_float_weights() returns them; they
        are quantised to INT-n on the device (nq_quantize, Eq. 1), decomposed and packed."""
        self.ops, self.n_bits, self.l_bits = ops, n_bits, l_bits
        self.cfg = nq.make_cfg(n_bits, l_bits)
        # every layer's lower-bit page is a slice of one device arena and one pinned host arena, in the
        # same order, so that the model is paged in with a single copy (nq_page_in_low_batch)
        sizes = [0 if w is None else max(nq.nq_packed_bytes(w[0].shape[0], w[0].shape[1], l_bits), 16)
                 for w in weights]
        sizes = [(s + 255) // 256 * 256 if s else 0 for s in sizes]
        total = sum(sizes)
        self.low_arena = torch.zeros(total, dtype=torch.uint8, device="cuda")
        self.low_arena_host = torch.zeros(total, dtype=torch.uint8, pin_memory=True)
        self.layers = []
        off = 0
        for op, w, size in zip(ops, weights, sizes):
            if w is None:
                self.layers.append(None)
                continue
            w_float, bias = w
            N, K = w_float.shape
            need = max(nq.nq_packed_bytes(N, K, l_bits), 16)
            W = nq.NestedWeight(N, K, self.cfg, low=self.low_arena[off:off + need],
                                low_host=self.low_arena_host[off:off + need], init=False)
            W.desc.low_bytes = size            # the slot reaches up to the next page: contiguous runs
            off += size
            self.layers.append((W, torch.from_numpy(bias).cuda()))
        self.descs = [L[0].desc for L in self.layers if L is not None]
        nq.nq_weight_init_group(self.descs)
        # every layer is quantised per output channel on the device; all layers are then decomposed and packed by
        # one batched call, and the arena of lower-bit pages is copied once to its pinned master copy
        jobs, keep = [], []
        for L, w in zip(self.layers, weights):
            if L is not None:
                d_w = torch.from_numpy(w[0]).cuda()
                d_w_int = torch.empty(w[0].shape, dtype=torch.int8, device="cuda")
                nq.nq_quantize(d_w, L[0].N, L[0].K, n_bits, d_w_int, L[0].scale)
                keep.append(d_w_int)
                jobs.append((d_w_int, L[0].N, L[0].K, L[0].high, L[0].low))
        nq.nq_decompose_pack_batch(jobs, self.cfg)
        self.low_arena_host.copy_(self.low_arena)
        torch.cuda.synchronize()
        for L in self.layers:
            if L is not None:
                L[0].desc.low_resident = 1
        self.out_scale = [None] * (max(op["dst"] for op in ops) + 1)   # step of every int8 tensor
        self.channels = {0: ops[0]["cin"]}                             # channels of every NHWC tensor
        for op in ops:
            self.channels[op["dst"]] = op["cout"] if op["op"] in ("conv", "fc") else self.channels[op["src"]]

    def low_page_bytes(self) -> int:
        return sum(nq.nq_packed_bytes(L[0].N, L[0].K, self.l_bits) for L in self.layers if L is not None)

    def page_out_low(self, stream=None):
        nq.nq_page_out_low_batch(self.descs, stream)

    def page_in_low(self, copy_stream=None):
        nq.nq_page_in_low_batch(self.descs, copy_stream)

    def allocate(self, B: int, H: int, W: int):
        """Output tensors of every op for a batch of B images of H x W pixels, allocated once, so that a
        forward pass allocates nothing (and can be captured into a HIP graph)."""
        self.batch, self.in_hw = B, (H, W)
        self.hw = {0: (H, W)}
        self.buf = {}
        for op in self.ops:
            hs, ws = self.hw[op["src"]]
            if op["op"] in ("conv", "maxpool"):
                ho, wo = out_hw(hs, ws, op["k"], op["stride"], op["pad"])
                c = op["cout"] if op["op"] == "conv" else self.channels[op["src"]]
                self.buf[op["dst"]] = torch.empty((B, ho, wo, c), dtype=torch.int8, device="cuda")
                self.hw[op["dst"]] = (ho, wo)
            elif op["op"] == "avgpool":
                self.buf[op["dst"]] = torch.empty((B, 1, 1, self.channels[op["src"]]), dtype=torch.int8, device="cuda")
                self.hw[op["dst"]] = (1, 1)
            else:
                self.buf[op["dst"]] = torch.empty((B, op["cout"]), dtype=torch.float32, device="cuda")
        # ops that are a branch of the graph: convolutions whose output is used only as the residual of a later layer
        # (the projection shortcuts of the first block of every stage)
        used_as_residual = {op["residual"] for op in self.ops if op.get("residual") is not None}
        used_as_input = {op["src"] for op in self.ops}
        self.branch_ops = {i for i, op in enumerate(self.ops)
                           if op["op"] == "conv" and op["dst"] in used_as_residual and op["dst"] not in used_as_input}
        self.branch_events = {i: (torch.cuda.Event(), torch.cuda.Event()) for i in self.branch_ops}
        return self

    def calibrate(self, x, in_scale: float):
        """Fixes the int8 step of every activation tensor for this input batch (per tensor, symmetric): each
        convolution runs once in full-bit mode with fp32 output, nq_tensor_scale reduces it to absmax / 127
        on the device, and the layer is run again with that step to feed the next one."""
        B, H, W, _ = x.shape
        if getattr(self, "batch", None) != B or self.in_hw != (H, W):
            self.allocate(B, H, W)
        d_step = torch.zeros(1, dtype=torch.float32, device="cuda")
        self.out_scale[0] = float(in_scale)
        for op, L in zip(self.ops, self.layers):
            if op["op"] == "conv":
                src = x if op["src"] == 0 else self.buf[op["src"]]
                hs, ws = self.hw[op["src"]]
                ho, wo = self.hw[op["dst"]]
                Wt, bias = L
                shape = nq.nq_conv_shape(B, hs, ws, op["cin"], op["cout"], op["k"], op["k"], op["stride"], op["pad"])
                res, s_r = None, 0.0
                if op["residual"] is not None:
                    res, s_r = self.buf[op["residual"]], self.out_scale[op["residual"]]
                yf = torch.empty((B, ho, wo, op["cout"]), dtype=torch.float32, device="cuda")
                nq.nq_conv_full(src, shape, Wt.desc, nq.make_epilogue(self.out_scale[op["src"]], bias, res, s_r,
                                                                      op["relu"]), yf)
                nq.nq_tensor_scale(yf, yf.numel(), 8, d_step)
                self.out_scale[op["dst"]] = float(d_step.cpu()[0])
                del yf
            elif op["op"] in ("maxpool", "avgpool"):
                self.out_scale[op["dst"]] = self.out_scale[op["src"]]   # neither a maximum nor a mean exceeds the input range
            self._run_op(op, L, x, B, True, None)
        torch.cuda.synchronize()

    def _run_op(self, op, L, x, B, full, stream):
        src = x if op["src"] == 0 else self.buf[op["src"]]
        hs, ws = self.hw[op["src"]]
        s_in = self.out_scale[op["src"]]
        y = self.buf[op["dst"]]
        if op["op"] == "maxpool":
            nq.nq_maxpool_i8(src, B, hs, ws, src.shape[3], op["k"], op["stride"], op["pad"], y, stream)
        elif op["op"] == "avgpool":
            nq.nq_avgpool_i8(src, B, hs * ws, src.shape[3], s_in, 1.0 / self.out_scale[op["dst"]], y, stream)
        elif op["op"] == "fc":
            Wt, bias = L
            (nq.nq_gemm_full if full else nq.nq_gemm_part)(src.view(B, -1), B, Wt.desc, nq.make_epilogue(s_in, bias), y,
                                                           stream)
        else:
            Wt, bias = L
            shape = nq.nq_conv_shape(B, hs, ws, op["cin"], op["cout"], op["k"], op["k"], op["stride"], op["pad"])
            res, s_r = None, 0.0
            if op["residual"] is not None:
                res, s_r = self.buf[op["residual"]], self.out_scale[op["residual"]]
            epi = nq.make_epilogue(s_in, bias, res, s_r, op["relu"], True, 1.0 / self.out_scale[op["dst"]])
            (nq.nq_conv_full if full else nq.nq_conv_part)(src, shape, Wt.desc, epi, y, stream)

    def forward(self, x, in_scale: float, full: bool, keep=None, stream=None, branch_stream=None):
        """x: int8 NHWC device tensor.  Returns the fp32 logits [B, classes] (a buffer of the model: the next
        forward overwrites it).  The int8 step of every tensor (out_scale) must have been set, by calibrate()
        or by the caller.  keep, if a dict, receives every op's output tensor.
        branch_stream: a second stream (torch.cuda.Stream) for the branches of the graph: the projection shortcut of
        a block does not depend on the block's main path, so it is issued there and joined (events, also under HIP
        graph capture) before the layer that adds it; its launch, prologue and tail then overlap the main path."""
        B, H, W, _ = x.shape
        if getattr(self, "batch", None) != B or self.in_hw != (H, W):
            self.allocate(B, H, W)
        self.out_scale[0] = float(in_scale)
        logits = None
        main = stream if stream is not None else torch.cuda.current_stream()
        joins = {}                                   # tensor id -> event its branch recorded
        for i, (op, L) in enumerate(zip(self.ops, self.layers)):
            on_branch = branch_stream is not None and i in self.branch_ops
            if on_branch:
                fork, join = self.branch_events[i]
                fork.record(main)                    # the branch starts from what the main path has produced so far
                branch_stream.wait_event(fork)
                self._run_op(op, L, x, B, full, branch_stream)
                join.record(branch_stream)
                joins[op["dst"]] = join
            else:
                if op.get("residual") in joins:
                    main.wait_event(joins.pop(op["residual"]))
                self._run_op(op, L, x, B, full, stream)
            if op["op"] == "fc":
                logits = self.buf[op["dst"]]
            if keep is not None:
                keep[op["dst"]] = self.buf[op["dst"]]
        return logits
