"""The one-GPU zebra engine (Section 4.1; engine paragraph of Section 5): R micro-batches through L expert
layers on a compute stream and two copy streams, in the order of Theorem 1, against the same layers run on
the whole batch on one stream.  Tokens are independent and every per-token sum of the library has a fixed
order, so outputs and input gradients must agree bit for bit; the weight gradients are sums over
micro-batches (accumulate flag) and agree to fp32 summation error."""
from dataclasses import replace

import numpy as np
import pytest

from paper_2504_03871_amd import synth as S
from tests import gpu_util as U

pytestmark = pytest.mark.gpu

CASES = {
    "bf16_gelu_L2_R3": (S.WORKLOADS["cfg1"].scaled(T=768, d=128, f=256, E=8, k=2), 2, 3),
    "bf16_swiglu_L3_R2": (S.WORKLOADS["cfg3"].scaled(T=512, d=128, f=192, E=6, k=3), 3, 2),
    "f32_L2_R4": (S.WORKLOADS["cfg0"].scaled(T=512, d=64, f=96, E=8, k=2), 2, 4),
    "f16_gelu_L2_R2": (S.WORKLOADS["cfg1"].scaled(T=512, d=128, f=256, E=8, k=2, dtype=S.DT_F16), 2, 2),
}


def bits(t):
    import torch
    return t.contiguous().view(torch.int16 if t.element_size() == 2 else torch.int32)


@pytest.mark.parametrize("name", list(CASES))
def test_micro_batched_streams_equal_the_whole_batch(name):
    import torch
    from paper_2504_03871_amd.zebra import ZebraExpertEngine
    w, L, R = CASES[name]
    print(f"\n[case {name}] {w} L={L} R={R}", flush=True)
    assert w.T % R == 0
    T_mb = w.T // R
    inps = [S.make_inputs(replace(w, cid=w.cid + 10 * i)) for i in range(L)]   # one weight set per layer
    # whole batch, one stream, layer after layer
    full = [U.make_layer(w, inps[i]) for i in range(L)]
    for i in range(L):
        if i > 0:
            full[i].x.copy_(full[i - 1].out)
        full[i].forward()
    for i in reversed(range(L)):
        if i < L - 1:
            full[i].d_out.copy_(full[i + 1].dx)
        full[i].backward()
    torch.cuda.synchronize()
    # the reference the engine is compared with is itself checked against the oracle: every layer on the
    # input and the upstream gradient it actually received (its GPU-side values, as stored)
    for i in range(L):
        li = dict(inps[i])
        li["x"] = full[i].x.float().cpu().numpy()
        li["d_out"] = full[i].d_out.float().cpu().numpy()
        ref = U.run_oracle(w, li, gpu_logits=full[i].logits.cpu().numpy())
        assert (U.host(full[i].topk_idx) == ref["idx"]).all()
        for n, key in (("out", "out"), ("dx", "dx"), ("dW1", "dW1"), ("dW2", "dW2"), ("dWr", "dWr")) + \
                ((("dW1b", "dW1b"),) if w.act == S.ACT_SWIGLU else ()):
            U.assert_close(f"layer {i} {n} vs oracle", U.host(getattr(full[i], n)), ref[key], U.TOL[w.dtype])

    eng = ZebraExpertEngine(L, R, T_mb, w.d, w.f, w.E, w.k, dtype=w.dtype, act=w.act)
    for i in range(L):
        for n in ("Wr", "W1", "W2") + (("W1b",) if w.act == S.ACT_SWIGLU else ()):
            getattr(eng.params[i], n).copy_(getattr(full[i], n))
        for n in ("dW1", "dW2", "dWr"):
            getattr(eng.params[i], n).fill_(U.SENTINEL)
    for j in range(R):
        eng.act[0][j].copy_(full[0].x[j * T_mb:(j + 1) * T_mb])
        eng.grad[L][j].copy_(full[L - 1].d_out[j * T_mb:(j + 1) * T_mb])
    torch.cuda.synchronize()
    for it in range(2):          # twice: the second iteration reuses every buffer and event
        eng.run_iteration()
        torch.cuda.synchronize()
        for j in range(R):
            rows = slice(j * T_mb, (j + 1) * T_mb)
            assert torch.equal(bits(eng.act[L][j]), bits(full[L - 1].out[rows])), f"output of micro-batch {j}"
            assert torch.equal(bits(eng.grad[0][j]), bits(full[0].dx[rows])), f"input gradient of micro-batch {j}"
        for i in range(L):
            for n in ("dW1", "dW2", "dWr") + (("dW1b",) if w.act == S.ACT_SWIGLU else ()):
                U.assert_close(f"layer {i} {n}", U.host(getattr(eng.params[i], n)), U.host(getattr(full[i], n)), 1e-4)
    # the engine's own results against the oracle (layer 0: its input is an input of the test)
    li = dict(inps[0])
    li["d_out"] = full[0].d_out.float().cpu().numpy()
    ref = U.run_oracle(w, li, gpu_logits=full[0].logits.cpu().numpy())
    g0 = torch.cat([eng.grad[0][j] for j in range(R)])
    U.assert_close("engine input gradient vs oracle", U.host(g0), ref["dx"], U.TOL[w.dtype])
    for n, key in (("dW1", "dW1"), ("dW2", "dW2"), ("dWr", "dWr")) + ((("dW1b", "dW1b"),) if w.act == S.ACT_SWIGLU else ()):
        U.assert_close(f"engine layer 0 {n} vs oracle", U.host(getattr(eng.params[0], n)), ref[key], U.TOL[w.dtype])
