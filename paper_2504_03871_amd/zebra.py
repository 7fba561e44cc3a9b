"""The expert side of zebra parallelism on one GPU (Section 4.1 of the paper; engine paragraph of Section 5).

The paper runs every GPU with one compute stream and two communication streams (dispatch and combine
all-to-alls go in opposite directions and do not contend), orders streams with events, keeps one
receive buffer per micro-batch, and feeds the compute stream in the order of its Theorem 1: for the
expert GPUs all micro-batches of layer 1 forward, ..., layer L forward, then layer L backward, ..., layer 1
backward.  This module does the same with what one GPU has: the all-to-alls become device-to-device
copies on the two communication streams (the "attention side" is a set of plain buffers; there is no
attention computation, a layer's output is the next layer's input), and the expert computation is the
library's MoE layer, one call sequence per (layer, micro-batch) on the compute stream.

Nothing is computed here: the copies are `Tensor.copy_` on a stream, everything else is a library call.
Weight gradients of a layer are accumulated over its micro-batches by the library (accumulate flag).
All streams have the default priority.
"""
from __future__ import annotations

import torch

from . import binding as B
from .layer import MoELayer


def expert_stream_order(L: int, R: int):
    """Compute-stream order of an expert GPU (Theorem 1): ('F' | 'B', layer, micro-batch), 0-based."""
    fwd = [("F", i, j) for i in range(L) for j in range(R)]
    bwd = [("B", i, j) for i in reversed(range(L)) for j in range(R)]
    return fwd + bwd


def attention_stream_forward_order(L: int, R: int, offload):
    """Forward compute-stream order of an ATTENTION GPU under asymmetric expert assignment (Section 4.2):
    ('A', layer, micro-batch) for attention, ('X', layer, micro-batch) for the experts that expert block
    `layer` (0-based, L - 1 of them between L attention blocks) has offloaded to this GPU.  A layer's
    offloaded experts run after that layer's attention of ALL micro-batches, because their tokens come from
    the other attention GPUs with the dispatch.  The library side of such a task is the same call sequence
    the expert GPUs use, restricted by the slice arguments that moe_asymea_shares returns for role 1."""
    order = []
    for i in range(L):
        order += [("A", i, j) for j in range(R)]
        if i < L - 1 and offload[i] > 0:
            order += [("X", i, j) for j in range(R)]
    return order


class ZebraExpertEngine:
    def __init__(self, L, R, T_mb, d_model, d_ff, E, k, dtype=B.DTYPE_BF16, act=B.ACT_GELU, device="cuda:0"):
        self.L, self.R, self.T_mb = L, R, T_mb
        self.device = torch.device(device)
        # one parameter set per layer; one set of activation buffers per (layer, micro-batch)
        self.params = [MoELayer(T_mb, d_model, d_ff, E, k, dtype, act, device=device) for _ in range(L)]
        self.mb = [[self.params[i] if j == 0 else
                    MoELayer(T_mb, d_model, d_ff, E, k, dtype, act, device=device, params=self.params[i])
                    for j in range(R)] for i in range(L)]
        td = self.params[0].tdtype
        buf = lambda: [torch.empty(T_mb, d_model, dtype=td, device=self.device) for _ in range(R)]
        # the attention side: what it sends into layer i (act[i]), what comes out of the last layer
        # (act[L]), and the gradients travelling the other way (grad[i] = gradient w.r.t. act[i])
        self.act = [buf() for _ in range(L + 1)]
        self.grad = [buf() for _ in range(L + 1)]
        self.compute = torch.cuda.Stream(device=self.device)
        self.dispatch = torch.cuda.Stream(device=self.device)   # attention -> expert in the forward pass
        self.combine = torch.cuda.Stream(device=self.device)    # expert -> attention in the forward pass
        ev = lambda: [[torch.cuda.Event() for _ in range(R)] for _ in range(L)]
        self.recv_f, self.done_f, self.back_f = ev(), ev(), ev()
        self.recv_b, self.done_b, self.back_b = ev(), ev(), ev()

    def run_iteration(self):
        """One training iteration: inputs in act[0][j], upstream gradients in grad[L][j]; leaves outputs in
        act[L][j], input gradients in grad[0][j] and the summed weight gradients in params[i]."""
        L, R = self.L, self.R
        start = torch.cuda.Event()
        start.record(torch.cuda.current_stream(self.device))
        for s in (self.compute, self.dispatch, self.combine):
            s.wait_event(start)
        for kind, i, j in expert_stream_order(L, R):
            m = self.mb[i][j]
            if kind == "F":
                with torch.cuda.stream(self.dispatch):           # dispatch all-to-all of (i, j)
                    if i > 0:
                        self.dispatch.wait_event(self.back_f[i - 1][j])   # the previous layer's output has arrived
                    m.x.copy_(self.act[i][j], non_blocking=True)
                    self.recv_f[i][j].record(self.dispatch)
                with torch.cuda.stream(self.compute):            # E^F_{i,j}
                    self.compute.wait_event(self.recv_f[i][j])
                    m.forward()
                    self.done_f[i][j].record(self.compute)
                with torch.cuda.stream(self.combine):            # combine all-to-all of (i, j)
                    self.combine.wait_event(self.done_f[i][j])
                    self.act[i + 1][j].copy_(m.out, non_blocking=True)
                    self.back_f[i][j].record(self.combine)
            else:
                # backward: the directions are reversed, the gradient of the combine travels first
                with torch.cuda.stream(self.combine):
                    if i < L - 1:
                        self.combine.wait_event(self.back_b[i + 1][j])
                    m.d_out.copy_(self.grad[i + 1][j], non_blocking=True)
                    self.recv_b[i][j].record(self.combine)
                with torch.cuda.stream(self.compute):            # E^B_{i,j}
                    self.compute.wait_event(self.recv_b[i][j])
                    m.backward(accumulate=1 if j > 0 else 0)
                    self.done_b[i][j].record(self.compute)
                with torch.cuda.stream(self.dispatch):
                    self.dispatch.wait_event(self.done_b[i][j])
                    self.grad[i][j].copy_(m.dx, non_blocking=True)
                    self.back_b[i][j].record(self.dispatch)
        cur = torch.cuda.current_stream(self.device)
        for s in (self.compute, self.dispatch, self.combine):
            done = torch.cuda.Event()
            done.record(s)
            cur.wait_event(done)
