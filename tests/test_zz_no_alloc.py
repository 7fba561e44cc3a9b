"""moe_dispatch_static, the entry point for callers that cannot allocate (its per-block histograms live in a
device array of the library instead of a workspace), against moe_dispatch through the C ABI: same index
arrays and the same gathered rows, bit for bit, on two calls in a row, the second on a smaller input, so
that what the first call left in the shared array must not matter.  Collected last on purpose."""
import numpy as np
import pytest

from paper_2504_03871_amd import binding as B
from paper_2504_03871_amd import synth as S

pytestmark = pytest.mark.gpu


def _both(T, d, E, k, cap, seed, partial):
    import torch
    rng = np.random.default_rng(seed)
    dev = "cuda:0"
    cfg = B.make_cfg(T, d, 64, E, k, capacity=cap)
    idx_np = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    idx = torch.from_numpy(idx_np).to(dev)
    x = torch.from_numpy(S.f32_to_bf16_bits(rng.normal(size=(T, d)).astype(np.float32)).view(np.int16)).to(dev).view(torch.bfloat16)
    lo = hi = None
    if partial:
        lo = torch.from_numpy(rng.integers(0, 40, size=E).astype(np.int32)).to(dev)
        hi = torch.from_numpy(rng.integers(30, 4000, size=E).astype(np.int32)).to(dev)
    out = []
    for static in (False, True):
        i32 = dict(dtype=torch.int32, device=dev)
        counts, kept, offsets = torch.full((E,), -7, **i32), torch.full((E,), -7, **i32), torch.full((E + 1,), -7, **i32)
        row_of, src_of = torch.full((T * k,), -7, **i32), torch.full((T * k,), -7, **i32)
        x_perm = torch.full((T * k, d), 12288.0, dtype=torch.bfloat16, device=dev)
        if static:
            B.moe_dispatch_static(cfg, x, idx, lo, hi, counts, kept, offsets, row_of, src_of, x_perm)
        else:
            ws = torch.empty(B.moe_workspace_bytes(cfg), dtype=torch.uint8, device=dev)
            B.moe_dispatch(cfg, x, idx, lo, hi, counts, kept, offsets, row_of, src_of, x_perm, ws)
        torch.cuda.synchronize()
        out.append((counts, kept, offsets, row_of, src_of, x_perm.view(torch.int16)))
    return out, idx_np


def test_static_scratch_dispatch_equals_workspace_dispatch_twice_in_a_row():
    import torch
    from oracle import moe_oracle as O
    # first a long assignment list (scanned-prefix path, 118 blocks), then a much smaller one (in-block scan)
    for T, d, E, k, cap, seed, partial in ((30000, 128, 40, 4, 2900, 1, True), (700, 64, 8, 2, 0, 2, False)):
        (a, b), idx_np = _both(T, d, E, k, cap, seed, partial)
        for name, ta, tb in zip(("counts", "kept", "offsets", "row_of", "src_of", "x_perm"), a, b):
            assert torch.equal(ta, tb), (T, name)
        ref = O.dispatch_plan(idx_np, E, cap)        # and both against the oracle's plan
        for name, tb, r in zip(("counts", "kept", "offsets", "row_of", "src_of"), b, ref):
            assert (tb.cpu().numpy() == r).all(), (T, name)
