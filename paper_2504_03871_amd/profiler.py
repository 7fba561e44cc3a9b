"""Time of an expert module on this GPU, for the planner of the asymmetric expert assignment.

The paper's profiler (Section 5) takes one expert FFN out of a layer, feeds it random inputs of the batch
size B that a GPU sees per micro-batch, and times it; those times (on an attention GPU and on an expert
GPU) are inputs of Algorithm 1 (`moe_asymea_plan`).  This is the same measurement for the library's own
kernels: the expert FFN forward (`moe_expert_ffn_fwd`) of `n_experts` experts with B tokens in all, timed
with HIP events on the current stream.  Nothing is computed here; the buffers are filled with random
numbers by torch only because their values do not matter.
"""
from __future__ import annotations

import torch

from . import binding as B


def expert_module_time_ms(tokens, d_model, d_ff, n_experts=1, dtype=B.DTYPE_BF16, act=B.ACT_GELU, iters=20, warmup=5,
                          device="cuda:0"):
    """Median time in milliseconds of the forward expert FFN over `tokens` rows spread evenly over
    `n_experts` experts (T_E of the paper's Algorithm 1 for this GPU: n_experts = the experts the GPU
    holds for a layer, tokens = the tokens it receives per micro-batch)."""
    dev = torch.device(device)
    td = torch.bfloat16 if dtype == B.DTYPE_BF16 else torch.float32
    cfg = B.make_cfg(tokens, d_model, d_ff, n_experts, 1, dtype, act)
    per = tokens // n_experts
    kept = torch.full((n_experts,), per, dtype=torch.int32, device=dev)
    kept[: tokens - per * n_experts] += 1
    offsets = torch.zeros(n_experts + 1, dtype=torch.int32, device=dev)
    offsets[1:] = torch.cumsum(kept, 0)
    x = torch.randn(tokens, d_model, device=dev).to(td)
    W1 = (0.02 * torch.randn(n_experts, d_model, d_ff, device=dev)).to(td)
    W1b = (0.02 * torch.randn(n_experts, d_model, d_ff, device=dev)).to(td) if act == B.ACT_SWIGLU else None
    W2 = (0.02 * torch.randn(n_experts, d_ff, d_model, device=dev)).to(td)
    saved = torch.empty(B.moe_saved_bytes(cfg), dtype=torch.uint8, device=dev)
    y = torch.empty(tokens, d_model, dtype=td, device=dev)
    ws = torch.empty(max(B.moe_workspace_bytes(cfg), 256), dtype=torch.uint8, device=dev)
    call = lambda: B.moe_expert_ffn_fwd(cfg, x, W1, W1b, W2, offsets, kept, None, None, saved, y, ws)
    for _ in range(warmup):
        call()
    times = []
    for _ in range(iters):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        call()
        e1.record()
        e1.synchronize()
        times.append(e0.elapsed_time(e1))
    times.sort()
    return times[len(times) // 2]
