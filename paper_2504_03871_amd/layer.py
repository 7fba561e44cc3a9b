"""Call sequencing of one MoE layer step (forward + backward) on top of the C-ABI binding.

Owns the device buffers (torch is used for memory and streams only) and issues the library calls in
the order of the paper's MoE block: gate, dispatch, expert FFN, combine (Section 2.1), then the two
backward branches of Section 5.  Nothing is computed here.
"""
from __future__ import annotations

import torch

from . import binding as B


class MoELayer:
    def __init__(self, T, d_model, d_ff, E, k, dtype=B.DTYPE_BF16, act=B.ACT_GELU, capacity=0, device="cuda:0",
                 params=None):
        """`params`: another MoELayer whose weights and weight-gradient buffers this one aliases (one
        layer seen by several micro-batches, each with activation buffers of its own)."""
        self.cfg = B.make_cfg(T, d_model, d_ff, E, k, dtype, act, capacity)
        self.T, self.d, self.f, self.E, self.k, self.act = T, d_model, d_ff, E, k, act
        self.tdtype = {B.DTYPE_BF16: torch.bfloat16, B.DTYPE_F16: torch.float16}.get(dtype, torch.float32)
        self.device = torch.device(device)
        A = T * k
        dev, td = self.device, self.tdtype
        i32 = dict(dtype=torch.int32, device=dev)
        f32 = dict(dtype=torch.float32, device=dev)
        e = lambda *s, **kw: torch.empty(*s, **kw)
        # parameters and inputs (filled by the caller)
        self.x = e(T, d_model, dtype=td, device=dev)
        if params is None:
            self.Wr = e(d_model, E, **f32)
            self.bias = None
            self.W1 = e(E, d_model, d_ff, dtype=td, device=dev)
            self.W1b = e(E, d_model, d_ff, dtype=td, device=dev) if act == B.ACT_SWIGLU else None
            self.W2 = e(E, d_ff, d_model, dtype=td, device=dev)
        else:
            self.Wr, self.bias, self.W1, self.W1b, self.W2 = params.Wr, params.bias, params.W1, params.W1b, params.W2
        self.d_out = e(T, d_model, dtype=td, device=dev)
        # forward state
        self.logits = e(T, E, **f32)
        self.topk_idx = e(T, k, **i32)
        self.topk_w = e(T, k, **f32)
        self.counts, self.kept, self.offsets = e(E, **i32), e(E, **i32), e(E + 1, **i32)
        self.row_of, self.src_of = e(A, **i32), e(A, **i32)
        self.slice_lo = self.slice_hi = None
        self.side = None
        self.x_perm = e(A, d_model, dtype=td, device=dev)
        self.saved = torch.empty(B.moe_saved_bytes(self.cfg), dtype=torch.uint8, device=dev)
        self.y_perm = e(A, d_model, dtype=td, device=dev)
        self.out = e(T, d_model, dtype=td, device=dev)
        self.ws = torch.empty(max(B.moe_workspace_bytes(self.cfg), 256), dtype=torch.uint8, device=dev)
        # backward state
        self.dy_perm = e(A, d_model, dtype=td, device=dev)
        self.d_topk_w = e(T, k, **f32)
        self.dx_perm = e(A, d_model, dtype=td, device=dev)
        if params is None:
            self.dW1 = e(E, d_model, d_ff, **f32)
            self.dW1b = e(E, d_model, d_ff, **f32) if act == B.ACT_SWIGLU else None
            self.dW2 = e(E, d_ff, d_model, **f32)
            self.dWr = e(d_model, E, **f32)
        else:
            self.dW1, self.dW1b, self.dW2, self.dWr = params.dW1, params.dW1b, params.dW2, params.dWr
        self.d_logits = e(T, E, **f32)
        self.dx = e(T, d_model, dtype=td, device=dev)

    def saved_plane(self, i):
        """Plane i of the saved activations as a [T*k, d_ff] tensor (GELU: A, H; SwiGLU: G, U, H)."""
        A, f = self.T * self.k, self.f
        n = A * f * self.x.element_size()
        return self.saved[i * n:(i + 1) * n].view(self.tdtype).view(A, f)

    def set_slices(self, lo, hi):
        """Per-expert [lo, hi) shares as int32 device tensors, or None/None for everything."""
        if lo is None:
            self.slice_lo = self.slice_hi = None
        else:
            self.slice_lo = torch.as_tensor(lo, dtype=torch.int32).to(self.device).contiguous()
            self.slice_hi = torch.as_tensor(hi, dtype=torch.int32).to(self.device).contiguous()

    # ---- the hot path, one library call per line -------------------------------------------------
    def route(self, logits_in=None):
        B.moe_route(self.cfg, self.x, self.Wr, self.bias, logits_in, self.logits, self.topk_idx, self.topk_w, self.ws)

    def dispatch(self, gather=True):
        B.moe_dispatch(self.cfg, self.x, self.topk_idx, self.slice_lo, self.slice_hi, self.counts, self.kept,
                       self.offsets, self.row_of, self.src_of, self.x_perm if gather else None, self.ws)

    def ffn_fwd(self):
        B.moe_expert_ffn_fwd(self.cfg, self.x_perm, self.W1, self.W1b, self.W2, self.offsets, self.kept,
                             self.slice_lo, self.slice_hi, self.saved, self.y_perm, self.ws)

    def ffn_fwd_light(self):
        """Forward of a checkpointed layer: only the hidden activation is kept (in its plane of `saved`)."""
        planes = 3 if self.cfg.act == B.ACT_SWIGLU else 2
        B.moe_expert_ffn_fwd_light(self.cfg, self.x_perm, self.W1, self.W1b, self.W2, self.offsets, self.kept,
                                   self.slice_lo, self.slice_hi, self.saved_plane(planes - 1), self.y_perm, self.ws)

    def ffn_recompute(self):
        """Activation checkpointing: refill the saved planes from x_perm (first half of ffn_fwd)."""
        B.moe_expert_ffn_recompute(self.cfg, self.x_perm, self.W1, self.W1b, self.offsets, self.kept,
                                   self.slice_lo, self.slice_hi, self.saved, self.ws)

    def combine(self):
        B.moe_combine(self.cfg, self.y_perm, self.topk_w, self.topk_idx, self.row_of, self.offsets, self.kept,
                      self.slice_lo, self.slice_hi, self.out, 0)

    def combine_bwd(self):
        B.moe_combine_bwd(self.cfg, self.d_out, self.y_perm, self.topk_w, self.topk_idx, self.row_of, self.offsets,
                          self.kept, self.slice_lo, self.slice_hi, self.dy_perm, self.d_topk_w)

    def ffn_bwd(self, accumulate=0):
        B.moe_expert_ffn_bwd(self.cfg, self.dy_perm, self.x_perm, self.saved, self.W1, self.W1b, self.W2,
                             self.offsets, self.kept, self.slice_lo, self.slice_hi, self.dx_perm, self.dW1,
                             self.dW1b, self.dW2, accumulate, self.ws)

    def dispatch_bwd(self):
        # the input-gradient un-permute is a combine with unit weights
        B.moe_combine(self.cfg, self.dx_perm, None, self.topk_idx, self.row_of, self.offsets, self.kept,
                      self.slice_lo, self.slice_hi, self.dx, 0)

    def route_bwd(self, accumulate=0):
        B.moe_route_bwd(self.cfg, self.x, self.Wr, self.topk_idx, self.topk_w, self.d_topk_w, self.d_logits,
                        self.dWr, self.dx, self.ws, accumulate)

    def forward(self, logits_in=None):
        self.route(logits_in)
        self.dispatch()
        self.ffn_fwd()
        self.combine()

    def backward(self, accumulate=0):
        """accumulate = 1 adds this batch's weight gradients (experts and gate) to the buffers."""
        if self.side is not None:
            return self.backward_overlapped(accumulate)
        self.combine_bwd()
        self.ffn_bwd(accumulate)
        self.dispatch_bwd()
        self.route_bwd(accumulate)

    def enable_gate_overlap(self):
        """Run the gate's weight gradient on a second stream next to the expert backward (both need only
        d_topk_w); it gets a workspace and a d_logits buffer of its own."""
        self.side = torch.cuda.Stream(device=self.device)
        self.side_ws = torch.empty_like(self.ws)
        self.side_d_logits = torch.empty_like(self.d_logits)
        self.ev_fork, self.ev_join = torch.cuda.Event(), torch.cuda.Event()

    def backward_overlapped(self, accumulate=0):
        main = torch.cuda.current_stream(self.device)
        self.combine_bwd()
        self.ev_fork.record(main)
        self.side.wait_event(self.ev_fork)
        with torch.cuda.stream(self.side):     # d_logits and dWr = x^T d_logits
            B.moe_route_bwd(self.cfg, self.x, self.Wr, self.topk_idx, self.topk_w, self.d_topk_w, self.d_logits,
                            self.dWr, None, self.side_ws, accumulate)
            self.ev_join.record(self.side)
        self.ffn_bwd(accumulate)
        self.dispatch_bwd()
        # dx += d_logits Wr^T once the gradient through the experts is in dx
        B.moe_route_bwd(self.cfg, self.x, self.Wr, self.topk_idx, self.topk_w, self.d_topk_w, self.side_d_logits,
                        None, self.dx, self.ws, 0)
        main.wait_event(self.ev_join)

    def step(self):
        self.forward()
        self.backward()

    def step_checkpointed(self):
        """Forward, then the backward of a checkpointed layer: gate, dispatch and the saved activations
        are computed again from the layer input before the gradients (y_perm is kept: the combine
        backward needs the expert outputs).  The forward keeps only the hidden activation."""
        self.route()
        self.dispatch()
        self.ffn_fwd_light()
        self.combine()
        self.route()
        self.dispatch()
        self.ffn_recompute()
        self.backward()
