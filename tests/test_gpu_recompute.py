"""Activation checkpointing (Section 6.1 of the paper: all runs use it): the recompute entry point must
refill the saved activations with the very bits the forward wrote, so that the backward of a checkpointed
layer equals the backward of a layer that kept them."""
import pytest

from paper_2504_03871_amd import synth as S
from tests import gpu_util as U

pytestmark = pytest.mark.gpu

W = S.WORKLOADS
CASES = {
    "f32": W["cfg0"],
    "bf16_gelu": W["cfg1"].scaled(T=1000, d=256, f=512),
    "bf16_gelu_split_k": W["cfg1"].scaled(T=620, d=128, f=2560, E=4, k=2),
    "bf16_swiglu_partial_cap": W["cfg3"].scaled(T=1200, d=256, f=320, E=6, k=3, capacity_factor=0.8, partial=True,
                                                zipf_s=0.7),
    "f16_gelu": W["cfg1"].scaled(T=1000, d=256, f=512, dtype=S.DT_F16),
    "f16_swiglu": W["cfg3"].scaled(T=900, d=256, f=320, E=6, k=3, dtype=S.DT_F16),
}


@pytest.mark.parametrize("name", list(CASES))
def test_recomputed_activations_and_gradients_are_bit_identical(name):
    import torch
    w = CASES[name]
    print(f"\n[case {name}] {w}", flush=True)
    inp = S.make_inputs(w)
    L = U.make_layer(w, inp)
    if w.partial:
        L.route()
        L.dispatch(gather=False)
        torch.cuda.synchronize()
        L.set_slices(*S.partial_slices(w, U.host(L.kept)))
    U.fill_sentinels(L)
    L.step()
    torch.cuda.synchronize()
    grads = ["dx", "dx_perm", "dW1", "dW2", "dWr", "d_logits", "d_topk_w"] + (["dW1b"] if w.act == S.ACT_SWIGLU else [])
    keep = {n: getattr(L, n).clone() for n in grads + ["out", "y_perm", "row_of", "src_of", "x_perm"]}
    saved = L.saved.clone()
    assert not torch.equal(saved, torch.full_like(saved, 0))

    # a checkpointed layer: the saved planes are gone (another layer used the buffer), the gate and
    # the dispatch run again on the layer input, the planes are recomputed, then the usual backward
    y = L.y_perm.clone()
    U.fill_sentinels(L)
    L.y_perm.copy_(y)                       # expert outputs are what a checkpointing caller keeps
    L.route()
    L.dispatch()
    L.ffn_recompute()
    torch.cuda.synchronize()
    assert torch.equal(L.saved, saved), "recomputed activations differ from the forward's"
    # the recomputed planes against the oracle's forward intermediates (routing replayed from the GPU's logits)
    kept = U.host(L.kept)
    lo, hi = S.partial_slices(w, kept) if w.partial else (None, None)
    ref = U.run_oracle(w, inp, gpu_logits=L.logits.cpu().numpy(), lo=lo, hi=hi)
    assert (U.host(L.row_of) == ref["row_of"]).all()
    planes = ("A", "H") if w.act == S.ACT_GELU else ("G", "U", "H")
    for i, p in enumerate(planes):
        U.assert_close("recomputed " + p, U.host(L.saved_plane(i)), ref["fw"][p], U.TOL[w.dtype])
    assert torch.equal(L.row_of, keep["row_of"]) and torch.equal(L.x_perm.view(torch.int16), keep["x_perm"].view(torch.int16))
    L.backward()
    torch.cuda.synchronize()
    for n in grads:
        a, b = getattr(L, n), keep[n]
        assert torch.equal(a.view(torch.int16 if a.element_size() == 2 else torch.int32),
                           b.view(torch.int16 if b.element_size() == 2 else torch.int32)), n
    # and the gradients of the checkpointed backward against the oracle
    for n, key in (("dx", "dx"), ("dW1", "dW1"), ("dW2", "dW2"), ("dWr", "dWr")) + \
            ((("dW1b", "dW1b"),) if w.act == S.ACT_SWIGLU else ()):
        U.assert_close("checkpointed " + n, U.host(getattr(L, n)), ref[key], U.TOL[w.dtype])


@pytest.mark.parametrize("name", list(CASES))
def test_light_forward_keeps_only_the_hidden_activation(name):
    """moe_expert_ffn_fwd_light: H and y_perm bit-identical to the saving forward's, the other planes untouched;
    the checkpointed step built on it gives the gradients of the plain step, bit for bit."""
    import torch
    w = CASES[name]
    print(f"\n[case {name}] {w}", flush=True)
    inp = S.make_inputs(w)
    L = U.make_layer(w, inp)
    if w.partial:
        L.route()
        L.dispatch(gather=False)
        torch.cuda.synchronize()
        L.set_slices(*S.partial_slices(w, U.host(L.kept)))
    bits = lambda t: t.view(torch.int16 if t.element_size() == 2 else torch.int32)
    U.fill_sentinels(L)
    L.step()
    torch.cuda.synchronize()
    nplanes = 3 if w.act == S.ACT_SWIGLU else 2
    grads = ["dx", "dW1", "dW2", "dWr"] + (["dW1b"] if w.act == S.ACT_SWIGLU else [])
    keep = {n: getattr(L, n).clone() for n in grads + ["out", "y_perm"]}
    hidden = L.saved_plane(nplanes - 1).clone()

    U.fill_sentinels(L)
    sentinel = L.saved_plane(0).clone()
    L.route()
    L.dispatch()
    L.ffn_fwd_light()
    torch.cuda.synchronize()
    assert torch.equal(bits(L.saved_plane(nplanes - 1)), bits(hidden)), "hidden activation differs"
    assert torch.equal(bits(L.y_perm), bits(keep["y_perm"])), "expert outputs differ"
    for i in range(nplanes - 1):
        assert torch.equal(bits(L.saved_plane(i)), bits(sentinel)), "a pre-activation plane was written"

    U.fill_sentinels(L)
    L.step_checkpointed()
    torch.cuda.synchronize()
    for n in grads + ["out"]:
        assert torch.equal(bits(getattr(L, n)), bits(keep[n])), n
