"""Host-side checks of the C ABI: the library loads, exports every declared symbol, and rejects bad
arguments before launching anything (so these run without a GPU)."""
import ctypes
import os
import re

import pytest

from paper_2504_03871_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert set(names) == set(B.SYMBOLS), (names, B.SYMBOLS)
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_error_strings():
    lib = B.lib()
    assert lib.moe_error_string(0) == b"ok"
    for code in range(-7, 0):
        assert len(lib.moe_error_string(code)) > 3
    assert b"unknown" in lib.moe_error_string(-99)
    assert lib.moe_last_hip_error() == 0


def test_cfg_validation():
    ok = dict(T=8, d_model=64, d_ff=128, E=4, k=2, dtype=B.DTYPE_BF16, act=B.ACT_GELU)
    assert B.moe_workspace_bytes(B.make_cfg(**ok)) > 0
    assert B.moe_saved_bytes(B.make_cfg(**ok)) == 2 * 16 * 128 * 2
    assert B.moe_saved_bytes(B.make_cfg(**{**ok, "act": B.ACT_SWIGLU, "dtype": B.DTYPE_F32})) == 3 * 16 * 128 * 4
    bad = [dict(k=5), dict(k=0), dict(E=0), dict(E=257), dict(k=9, E=16), dict(d_model=72), dict(d_ff=100),
           dict(T=-1), dict(d_model=0)]
    for b in bad:
        with pytest.raises(B.MoeError) as ei:
            B.moe_workspace_bytes(B.make_cfg(**{**ok, **b}))
        assert ei.value.code == -2, b
    assert B.moe_saved_bytes(B.make_cfg(**{**ok, "dtype": B.DTYPE_F16})) == 2 * 16 * 128 * 2     # fp16 storage
    for b in (dict(dtype=3), dict(act=7)):
        with pytest.raises(B.MoeError) as ei:
            B.moe_workspace_bytes(B.make_cfg(**{**ok, **b}))
        assert ei.value.code == -3
    # fp32 accepts multiples of 4
    assert B.moe_workspace_bytes(B.make_cfg(**{**ok, "dtype": B.DTYPE_F32, "d_model": 68, "d_ff": 100})) > 0


def test_pointer_validation_happens_before_any_launch():
    """Fake (never dereferenced) device addresses: every call must fail in validation."""
    cfg = B.make_cfg(8, 64, 128, 4, 2)
    P, Q = 0x10000, 0x10008       # aligned / misaligned fake addresses
    s = ctypes.c_void_p(0)
    with pytest.raises(B.MoeError) as ei:
        B.moe_route(cfg, None, P, None, None, P, P, P, stream=s)
    assert ei.value.code == -1
    with pytest.raises(B.MoeError) as ei:
        B.moe_route(cfg, P, P, None, None, P, Q, P, ws=P, stream=s)
    assert ei.value.code == -5
    with pytest.raises(B.MoeError) as ei:
        B.moe_route(cfg, P, P, None, None, P, P, P, ws=None, stream=s)      # bf16 gate needs the workspace
    assert ei.value.code == -1
    with pytest.raises(B.MoeError) as ei:                                       # and so does the fp16 gate
        B.moe_route(B.make_cfg(8, 64, 128, 4, 2, dtype=B.DTYPE_F16), P, P, None, None, P, P, P, ws=None, stream=s)
    assert ei.value.code == -1
    with pytest.raises(B.MoeError) as ei:
        B.moe_dispatch(cfg, P, P, P, None, P, P, P, P, P, P, P, stream=s)      # only one slice bound
    assert ei.value.code == -4
    with pytest.raises(B.MoeError) as ei:
        B.moe_dispatch(cfg, None, P, None, None, P, P, P, P, P, P, P, stream=s)  # x_perm without x
    assert ei.value.code == -1
    with pytest.raises(B.MoeError) as ei:
        B.moe_expert_ffn_fwd(cfg, P, P, P, P, P, P, None, None, P, P, P, stream=s)   # W1b given for GELU
    assert ei.value.code == -3
    with pytest.raises(B.MoeError) as ei:
        B.moe_expert_ffn_fwd_light(cfg, P, P, None, P, P, P, None, None, None, P, P, stream=s)   # no hidden buffer
    assert ei.value.code == -1
    with pytest.raises(B.MoeError) as ei:
        B.moe_expert_ffn_recompute(cfg, P, P, None, P, P, None, None, None, P, stream=s)   # no saved buffer
    assert ei.value.code == -1
    with pytest.raises(B.MoeError) as ei:
        B.moe_expert_ffn_recompute(cfg, P, P, None, P, P, None, None, Q, P, stream=s)
    assert ei.value.code == -5
    sw = B.make_cfg(8, 64, 128, 4, 2, act=B.ACT_SWIGLU)
    with pytest.raises(B.MoeError) as ei:
        B.moe_expert_ffn_fwd(sw, P, P, None, P, P, P, None, None, P, P, P, stream=s)  # SwiGLU without W1b
    assert ei.value.code == -1
    with pytest.raises(B.MoeError) as ei:
        B.moe_combine(cfg, P, P, P, P, P, P, None, None, None, 0, stream=s)
    assert ei.value.code == -1
    with pytest.raises(B.MoeError) as ei:
        B.moe_combine_bwd(cfg, P, P, None, P, P, P, P, None, None, P, P, stream=s)
    assert ei.value.code == -1
    with pytest.raises(B.MoeError) as ei:
        B.moe_expert_ffn_bwd(cfg, P, P, P, P, None, P, P, P, None, None, P, P, None, None, 0, P, stream=s)
    assert ei.value.code == -1
    with pytest.raises(B.MoeError) as ei:
        B.moe_route_bwd(cfg, P, P, P, P, P, P, P, Q, P, stream=s)
    assert ei.value.code == -5
    with pytest.raises(B.MoeError) as ei:
        B.moe_route_bwd(cfg, P, P, P, P, P, None, P, P, P, stream=s)     # d_logits is always written
    assert ei.value.code == -1
    with pytest.raises(B.MoeError) as ei:
        B.moe_route_bwd(cfg, P, P, P, P, P, P, None, None, None, stream=s)   # both parts skipped is fine, no workspace is not
    assert ei.value.code == -1


def test_too_small_workspace_is_rejected_before_any_launch():
    """Every call that takes the workspace also takes its size: one byte short is MOE_ERR_WORKSPACE."""
    cfg = B.make_cfg(8, 64, 128, 4, 2)
    need = B.moe_workspace_bytes(cfg)
    P = 0x10000
    s = ctypes.c_void_p(0)
    calls = [
        lambda n: B.moe_route(cfg, P, P, None, None, P, P, P, ws=P, stream=s, ws_bytes=n),
        lambda n: B.moe_dispatch(cfg, P, P, None, None, P, P, P, P, P, P, P, stream=s, ws_bytes=n),
        lambda n: B.moe_expert_ffn_fwd(cfg, P, P, None, P, P, P, None, None, P, P, P, stream=s, ws_bytes=n),
        lambda n: B.moe_expert_ffn_fwd_light(cfg, P, P, None, P, P, P, None, None, P, P, P, stream=s, ws_bytes=n),
        lambda n: B.moe_expert_ffn_recompute(cfg, P, P, None, P, P, None, None, P, P, stream=s, ws_bytes=n),
        lambda n: B.moe_expert_ffn_bwd(cfg, P, P, P, P, None, P, P, P, None, None, P, P, None, P, 0, P, stream=s, ws_bytes=n),
        lambda n: B.moe_route_bwd(cfg, P, P, P, P, P, P, P, P, P, stream=s, ws_bytes=n),
    ]
    for call in calls:
        for n in (0, need - 1):
            with pytest.raises(B.MoeError) as ei:
                call(n)
            assert ei.value.code == -7
    assert b"workspace" in B.lib().moe_error_string(-7)


def test_shapes_whose_byte_offsets_pass_32_bits_are_rejected():
    """The grouped GEMMs use 32-bit byte offsets into one expert's share and one expert's weights."""
    ok = dict(T=32768, d_model=4096, d_ff=14336, E=8, k=2, dtype=B.DTYPE_BF16, act=B.ACT_SWIGLU)
    assert B.moe_workspace_bytes(B.make_cfg(**ok)) > 0
    # T*k*max(d, f)*2 bytes: 2^16 * 2 * 2^14 * 2 = 2^32 exactly is out, one row tile less is in
    edge = dict(T=1 << 16, d_model=64, d_ff=1 << 14, E=8, k=2, dtype=B.DTYPE_BF16, act=B.ACT_GELU)
    with pytest.raises(B.MoeError) as ei:
        B.moe_workspace_bytes(B.make_cfg(**edge))
    assert ei.value.code == -2
    assert B.moe_workspace_bytes(B.make_cfg(**{**edge, "T": (1 << 16) - 1})) > 0
    with pytest.raises(B.MoeError) as ei:       # the same element count in fp32 is twice the bytes
        B.moe_workspace_bytes(B.make_cfg(**{**edge, "T": 1 << 15, "dtype": B.DTYPE_F32}))
    assert ei.value.code == -2
    with pytest.raises(B.MoeError) as ei:       # d * f * 4 bytes of one expert's fp32 weight gradient
        B.moe_workspace_bytes(B.make_cfg(T=8, d_model=1 << 15, d_ff=1 << 15, E=2, k=1))
    assert ei.value.code == -2


def test_clock_probe_validation():
    s = ctypes.c_void_p(0)
    lib = B.lib()
    assert lib.moe_bench_clock_probe(None, 10, 1, s) == -1
    assert lib.moe_bench_clock_probe(0x10008, 10, 1, s) == -5
    assert lib.moe_bench_clock_probe(0x10000, 0, 1, s) == -2
    assert lib.moe_bench_clock_probe(0x10000, 10, 1001, s) == -2
    assert lib.moe_bench_mfma_loop(0, 10, None, 0x10000, s) == -1
    assert lib.moe_bench_mfma_loop(2, 10, 0x10000, 0x20000, s) == -2
    assert lib.moe_bench_mfma_loop(0, 0, 0x10000, 0x20000, s) == -2
    assert lib.moe_bench_mfma_loop(1, 10, 0x10000, 0x20008, s) == -5


def test_bench_stream_validation():
    s = ctypes.c_void_p(0)
    lib = B.lib()
    assert lib.moe_bench_stream(None, 0x10000, 1024, 0, s) == -1
    assert lib.moe_bench_stream(0x10000, None, 1024, 0, s) == -1
    assert lib.moe_bench_stream(0x10000, 0x20008, 1024, 0, s) == -5
    assert lib.moe_bench_stream(0x10000, 0x20000, 1000, 0, s) == -2
    assert lib.moe_bench_stream(0x10000, 0x20000, 1024, 2, s) == -3
    assert lib.moe_bench_stream(0x10000, None, 0, 1, s) == 0


def test_static_scratch_limit_is_checked_before_any_launch():
    P = 0x10000
    s = ctypes.c_void_p(0)
    big = B.make_cfg(1 << 20, 64, 64, 256, 1)       # (1024 + 1) * 256 * 4 bytes > 1 MiB
    with pytest.raises(B.MoeError) as ei:
        B.moe_dispatch_static(big, P, P, None, None, P, P, P, P, P, P, stream=s)
    assert ei.value.code == -7
    with pytest.raises(B.MoeError) as ei:
        B.moe_dispatch_static(B.make_cfg(8, 64, 64, 4, 2), P, None, None, None, P, P, P, P, P, P, stream=s)
    assert ei.value.code == -1
