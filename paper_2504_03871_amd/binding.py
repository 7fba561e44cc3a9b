"""ctypes binding of the C-ABI MoE library (include/moe.h): argument marshalling only.

Each function has the name and the argument order of its C entry point, takes torch tensors (or
None for optional pointers) and enqueues on torch's current HIP stream.  No arithmetic of the
layer happens in Python, and there is no fallback: if the library has not been built, or a call
returns an error code, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_hip.so")

DTYPE_F32, DTYPE_BF16, DTYPE_F16 = 0, 1, 2
ACT_GELU, ACT_SWIGLU = 0, 1
MAX_E, MAX_K = 256, 8

SYMBOLS = ("moe_error_string", "moe_last_hip_error", "moe_workspace_bytes", "moe_saved_bytes", "moe_route",
           "moe_dispatch", "moe_dispatch_static", "moe_expert_ffn_fwd", "moe_expert_ffn_fwd_light", "moe_expert_ffn_recompute", "moe_combine", "moe_combine_bwd", "moe_expert_ffn_bwd",
           "moe_route_bwd", "moe_asymea_plan", "moe_asymea_shares", "moe_bench_stream", "moe_bench_clock_probe", "moe_bench_mfma_loop", "moe_gemm_block_tile")

PROF = {"gemm1_fwd": 0, "gemm2_fwd": 1, "dh_bwd": 2, "dw2_bwd": 3, "dw1_bwd": 4, "dx_bwd": 5, "gather": 6,
        "combine": 7, "combine_bwd": 8, "route": 9}


PROF_COUNT = 10


class MoeProf(ctypes.Structure):
    """Caller-owned timing brackets (moe_prof): per kernel, arrays of hipEvent_t handles and a launch counter."""
    _fields_ = [("start", ctypes.POINTER(ctypes.c_void_p) * PROF_COUNT), ("stop", ctypes.POINTER(ctypes.c_void_p) * PROF_COUNT),
                ("n", ctypes.c_int32 * PROF_COUNT), ("count", ctypes.c_int64 * PROF_COUNT)]


class MoeCfg(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("T", "d_model", "d_ff", "E", "k", "dtype", "act", "capacity")] + \
               [("prof", ctypes.POINTER(MoeProf))]


class MoeError(RuntimeError):
    def __init__(self, fn, code, text, hip):
        super().__init__(f"{fn} failed: {code} ({text})" + (f", hipError {hip}" if code == -6 else ""))
        self.code = code


_lib = None


def lib():
    """The loaded shared library; raises if it has not been built (run __graft_entry__.build())."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2504_03871_amd.build`")
        l = ctypes.CDLL(LIB_PATH)
        l.moe_error_string.restype = ctypes.c_char_p
        l.moe_error_string.argtypes = [ctypes.c_int]
        l.moe_last_hip_error.restype = ctypes.c_int
        p, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        cfgp = ctypes.POINTER(MoeCfg)
        sig = {
            "moe_workspace_bytes": [cfgp, ctypes.POINTER(ctypes.c_size_t)],
            "moe_saved_bytes": [cfgp, ctypes.POINTER(ctypes.c_size_t)],
            "moe_route": [cfgp] + [p] * 8 + [sz, p],
            "moe_dispatch": [cfgp] + [p] * 11 + [sz, p],
            "moe_dispatch_static": [cfgp] + [p] * 11,
            "moe_expert_ffn_fwd": [cfgp] + [p] * 11 + [sz, p],
            "moe_expert_ffn_fwd_light": [cfgp] + [p] * 11 + [sz, p],
            "moe_expert_ffn_recompute": [cfgp] + [p] * 9 + [sz, p],
            "moe_combine": [cfgp] + [p] * 9 + [i32, p],
            "moe_combine_bwd": [cfgp] + [p] * 12,
            "moe_expert_ffn_bwd": [cfgp] + [p] * 14 + [i32, p, sz, p],
            "moe_route_bwd": [cfgp] + [p] * 8 + [i32, p, sz, p],
            "moe_asymea_plan": [i32] * 4 + [ctypes.c_double] * 3 + [i32, i32, ctypes.POINTER(i32)],
            "moe_asymea_shares": [i32] * 6 + [ctypes.POINTER(i32), ctypes.POINTER(i32)],
            "moe_bench_stream": [p, p, sz, i32, p],
            "moe_bench_clock_probe": [p, i32, i32, p],
            "moe_bench_mfma_loop": [i32, i32, p, p, p],
            "moe_gemm_block_tile": [i32, ctypes.c_int64, i32, i32, i32, i32, i32, ctypes.POINTER(i32)],
        }
        for name, args in sig.items():
            fn = getattr(l, name)
            fn.restype = ctypes.c_int
            fn.argtypes = args
        _lib = l
    return _lib


def make_cfg(T, d_model, d_ff, E, k, dtype=DTYPE_BF16, act=ACT_GELU, capacity=0) -> MoeCfg:
    return MoeCfg(int(T), int(d_model), int(d_ff), int(E), int(k), int(dtype), int(act), int(capacity))


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _nbytes(t):
    """Size of a workspace argument: a tensor's byte count; 0 for None; for a raw address the caller vouches."""
    if t is None:
        return 0
    if isinstance(t, int):
        return (1 << 62)
    return t.numel() * t.element_size()


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(name, rc):
    if rc != 0:
        l = lib()
        raise MoeError(name, rc, l.moe_error_string(rc).decode(), l.moe_last_hip_error())


def moe_workspace_bytes(cfg) -> int:
    n = ctypes.c_size_t(0)
    _check("moe_workspace_bytes", lib().moe_workspace_bytes(ctypes.byref(cfg), ctypes.byref(n)))
    return n.value


def moe_saved_bytes(cfg) -> int:
    n = ctypes.c_size_t(0)
    _check("moe_saved_bytes", lib().moe_saved_bytes(ctypes.byref(cfg), ctypes.byref(n)))
    return n.value


def moe_route(cfg, x, Wr, bias, logits_in, logits_out, topk_idx, topk_w, ws=None, stream=None, ws_bytes=None):
    _check("moe_route", lib().moe_route(ctypes.byref(cfg), _ptr(x), _ptr(Wr), _ptr(bias), _ptr(logits_in),
                                        _ptr(logits_out), _ptr(topk_idx), _ptr(topk_w), _ptr(ws),
                                        _nbytes(ws) if ws_bytes is None else ws_bytes,
                                        _stream() if stream is None else stream))


def moe_dispatch(cfg, x, topk_idx, slice_lo, slice_hi, counts, kept, offsets, row_of, src_of, x_perm, ws,
                 stream=None, ws_bytes=None):
    _check("moe_dispatch", lib().moe_dispatch(ctypes.byref(cfg), _ptr(x), _ptr(topk_idx), _ptr(slice_lo),
                                              _ptr(slice_hi), _ptr(counts), _ptr(kept), _ptr(offsets), _ptr(row_of),
                                              _ptr(src_of), _ptr(x_perm), _ptr(ws),
                                              _nbytes(ws) if ws_bytes is None else ws_bytes,
                                              _stream() if stream is None else stream))


def moe_dispatch_static(cfg, x, topk_idx, slice_lo, slice_hi, counts, kept, offsets, row_of, src_of, x_perm, stream=None):
    _check("moe_dispatch_static", lib().moe_dispatch_static(ctypes.byref(cfg), _ptr(x), _ptr(topk_idx), _ptr(slice_lo),
                                                            _ptr(slice_hi), _ptr(counts), _ptr(kept), _ptr(offsets),
                                                            _ptr(row_of), _ptr(src_of), _ptr(x_perm),
                                                            _stream() if stream is None else stream))


def moe_expert_ffn_fwd(cfg, x_perm, W1, W1b, W2, offsets, kept, slice_lo, slice_hi, saved, y_perm, ws, stream=None,
                       ws_bytes=None):
    _check("moe_expert_ffn_fwd", lib().moe_expert_ffn_fwd(ctypes.byref(cfg), _ptr(x_perm), _ptr(W1), _ptr(W1b),
                                                          _ptr(W2), _ptr(offsets), _ptr(kept), _ptr(slice_lo),
                                                          _ptr(slice_hi), _ptr(saved), _ptr(y_perm), _ptr(ws),
                                                          _nbytes(ws) if ws_bytes is None else ws_bytes,
                                                          _stream() if stream is None else stream))


def moe_expert_ffn_fwd_light(cfg, x_perm, W1, W1b, W2, offsets, kept, slice_lo, slice_hi, hidden, y_perm, ws,
                             stream=None, ws_bytes=None):
    """moe_expert_ffn_fwd that keeps only the hidden activation (for activation-checkpointed layers)."""
    _check("moe_expert_ffn_fwd_light", lib().moe_expert_ffn_fwd_light(
        ctypes.byref(cfg), _ptr(x_perm), _ptr(W1), _ptr(W1b), _ptr(W2), _ptr(offsets), _ptr(kept), _ptr(slice_lo),
        _ptr(slice_hi), _ptr(hidden), _ptr(y_perm), _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes,
        _stream() if stream is None else stream))


def moe_expert_ffn_recompute(cfg, x_perm, W1, W1b, offsets, kept, slice_lo, slice_hi, saved, ws, stream=None,
                             ws_bytes=None):
    _check("moe_expert_ffn_recompute", lib().moe_expert_ffn_recompute(
        ctypes.byref(cfg), _ptr(x_perm), _ptr(W1), _ptr(W1b), _ptr(offsets), _ptr(kept), _ptr(slice_lo),
        _ptr(slice_hi), _ptr(saved), _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes,
        _stream() if stream is None else stream))


def moe_combine(cfg, y_perm, topk_w, topk_idx, row_of, offsets, kept, slice_lo, slice_hi, out, accumulate=0,
                stream=None):
    _check("moe_combine", lib().moe_combine(ctypes.byref(cfg), _ptr(y_perm), _ptr(topk_w), _ptr(topk_idx),
                                            _ptr(row_of), _ptr(offsets), _ptr(kept), _ptr(slice_lo), _ptr(slice_hi),
                                            _ptr(out), int(accumulate), _stream() if stream is None else stream))


def moe_combine_bwd(cfg, d_out, y_perm, topk_w, topk_idx, row_of, offsets, kept, slice_lo, slice_hi, dy_perm,
                    d_topk_w, stream=None):
    _check("moe_combine_bwd", lib().moe_combine_bwd(ctypes.byref(cfg), _ptr(d_out), _ptr(y_perm), _ptr(topk_w),
                                                    _ptr(topk_idx), _ptr(row_of), _ptr(offsets), _ptr(kept),
                                                    _ptr(slice_lo), _ptr(slice_hi), _ptr(dy_perm), _ptr(d_topk_w),
                                                    _stream() if stream is None else stream))


def moe_expert_ffn_bwd(cfg, dy_perm, x_perm, saved, W1, W1b, W2, offsets, kept, slice_lo, slice_hi, dx_perm, dW1,
                       dW1b, dW2, accumulate, ws, stream=None, ws_bytes=None):
    _check("moe_expert_ffn_bwd", lib().moe_expert_ffn_bwd(ctypes.byref(cfg), _ptr(dy_perm), _ptr(x_perm), _ptr(saved),
                                                          _ptr(W1), _ptr(W1b), _ptr(W2), _ptr(offsets), _ptr(kept),
                                                          _ptr(slice_lo), _ptr(slice_hi), _ptr(dx_perm), _ptr(dW1),
                                                          _ptr(dW1b), _ptr(dW2), int(accumulate), _ptr(ws),
                                                          _nbytes(ws) if ws_bytes is None else ws_bytes,
                                                          _stream() if stream is None else stream))


def moe_route_bwd(cfg, x, Wr, topk_idx, topk_w, d_topk_w, d_logits, dWr, dx, ws, accumulate=0, stream=None,
                  ws_bytes=None):
    _check("moe_route_bwd", lib().moe_route_bwd(ctypes.byref(cfg), _ptr(x), _ptr(Wr), _ptr(topk_idx), _ptr(topk_w),
                                                _ptr(d_topk_w), _ptr(d_logits), _ptr(dWr), _ptr(dx), int(accumulate), _ptr(ws),
                                                _nbytes(ws) if ws_bytes is None else ws_bytes,
                                                _stream() if stream is None else stream))


def moe_asymea_plan(n, L, M, N, T_A_attn, T_E_attn, T_E_exp, n_min=0, n_max=-1):
    """Experts each expert GPU offloads at every layer (host-only call; list of L ints)."""
    o = (ctypes.c_int32 * max(int(L), 1))()
    _check("moe_asymea_plan", lib().moe_asymea_plan(int(n), int(L), int(M), int(N), float(T_A_attn), float(T_E_attn),
                                                    float(T_E_exp), int(n_min), int(n_max), o))
    return list(o)[:int(L)]


def moe_asymea_shares(n, M, N, o_l, role, rank):
    """Host-side slice bounds (lo, hi lists of n ints) of one GPU for a layer that offloads o_l experts."""
    lo, hi = (ctypes.c_int32 * max(int(n), 1))(), (ctypes.c_int32 * max(int(n), 1))()
    _check("moe_asymea_shares", lib().moe_asymea_shares(int(n), int(M), int(N), int(o_l), int(role), int(rank),
                                                        lo, hi))
    return list(lo)[:int(n)], list(hi)[:int(n)]


def moe_bench_stream(dst, src, nbytes, mode=0, stream=None):
    """Benchmark aid: the library's streaming copy (mode 0) or zero fill (mode 1) over nbytes bytes."""
    _check("moe_bench_stream", lib().moe_bench_stream(_ptr(dst), _ptr(src), int(nbytes), int(mode),
                                                      _stream() if stream is None else stream))


def moe_bench_clock_probe(samples, n, sleeps, stream=None):
    """Benchmark aid: n (shader clock, 100 MHz clock) counter pairs into the uint64 tensor `samples`."""
    _check("moe_bench_clock_probe", lib().moe_bench_clock_probe(_ptr(samples), int(n), int(sleeps),
                                                                _stream() if stream is None else stream))


def moe_bench_mfma_loop(kind, iters, operand, sink, stream=None):
    """Benchmark aid: a kernel of nothing but MFMAs (kind 0: 16x16x32, 1: 32x32x16); FLOP = 1024*8*iters*32*16384."""
    _check("moe_bench_mfma_loop", lib().moe_bench_mfma_loop(int(kind), int(iters), _ptr(operand), _ptr(sink),
                                                            _stream() if stream is None else stream))


def moe_gemm_block_tile(kind, block, n_rt=0, n_full_rt=0, n_split=0, ntm=1, ntn=1):
    """Host-only: the tile that block `block` of a grouped-GEMM launch computes (list of 6 ints, see moe.h)."""
    out = (ctypes.c_int32 * 6)()
    _check("moe_gemm_block_tile", lib().moe_gemm_block_tile(int(kind), int(block), int(n_rt), int(n_full_rt), int(n_split),
                                                            int(ntm), int(ntn), out))
    return list(out)
