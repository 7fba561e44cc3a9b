#!/usr/bin/env python3
"""Benchmark of the MoE expert layer hot path on one MI355X.

One "step" = one forward + backward pass of the whole layer (gate, dispatch, expert FFN, combine and
their backward) over one batch of seeded synthetic input that is already resident in HBM.
Prints ONE JSON line: whole-layer tokens/s, plus a roofline object for the dominant kernel (the bf16
MFMA grouped GEMM) measured with HIP events inside the timed region, per-stage timings, and the CPU
oracle timed on the host cores as a reported baseline.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg1] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3       # fp32 vector / matrix
PEAK_HBM_GBS = 8000.0

STAGES = ("route", "dispatch", "ffn_fwd", "combine", "combine_bwd", "ffn_bwd", "dispatch_bwd", "route_bwd")


def stage_bytes(w, S_rows, s):
    """Algorithmic HBM bytes of each bandwidth-bound stage (unique reads + writes)."""
    T, d, E, k, A = w.T, w.d, w.E, w.k, w.T * w.k
    return {
        "route": T * d * s + d * E * 4 + T * E * 4 + T * k * 8,
        "dispatch": T * d * s + S_rows * d * s + A * 12,
        "combine": S_rows * d * s + A * 8 + T * d * s,
        "combine_bwd": T * d * s + 2 * S_rows * d * s + A * 4,
        "dispatch_bwd": S_rows * d * s + T * d * s,
        "route_bwd": 3 * T * d * s + T * E * 4 + d * E * 4,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--overlap-gate-bwd", action="store_true",
                    help="run the gate's weight gradient on a second stream next to the expert backward "
                         "(measured: no gain; not the default)")
    ap.add_argument("--checkpoint", action="store_true",
                    help="time the step of an activation-checkpointed layer: gate, dispatch and the saved "
                         "activations are computed again before the backward (not the default metric)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 256 MiB device copy three times (calibrates rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2504_03871_amd import synth as S
    from paper_2504_03871_amd import binding as B
    from paper_2504_03871_amd.layer import MoELayer

    B.lib()   # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    w = S.WORKLOADS[args.workload]
    inp = S.make_inputs(w, threads=16)
    bf = w.dtype == S.DT_BF16
    dev = "cuda:0"
    L = MoELayer(w.T, w.d, w.f, w.E, w.k, dtype=w.dtype, act=w.act, capacity=w.capacity, device=dev)
    if args.overlap_gate_bwd:
        L.enable_gate_overlap()

    def up(name):
        if bf:
            return torch.from_numpy(inp[name + "_bits"].view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(inp[name]).to(dev)

    for name in ("x", "W1", "W2", "d_out") + (("W1b",) if w.act == S.ACT_SWIGLU else ()):
        getattr(L, name).copy_(up(name))
    L.Wr.copy_(torch.from_numpy(inp["Wr"]).to(dev))
    if inp["bias"] is not None:
        L.bias = torch.from_numpy(inp["bias"]).to(dev)

    # this GPU's shares need the kept counts once (untimed read-back); routing is fixed by the inputs
    L.route()
    L.dispatch(gather=False)
    torch.cuda.synchronize()
    kept = L.kept.cpu().numpy()
    lo, hi = S.partial_slices(w, kept)
    if w.partial:
        L.set_slices(lo, hi)
    S_rows = int((hi - lo).sum())

    step = L.step_checkpointed if args.checkpoint else L.step
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- HIP events around individual kernels (the library brackets the launches it is armed for)
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    per_step = {"combine": 2}     # launches per step (combine also serves the input-gradient un-permute)

    def make_events(n):
        arr = (ctypes.c_void_p * n)()
        for i in range(n):
            h = ctypes.c_void_p()
            assert hip.hipEventCreate(ctypes.byref(h)) == 0
            arr[i] = h
        return arr

    def arm(names):
        armed = {}
        for name in names:
            n = args.steps * per_step.get(name, 1)
            st, sp = make_events(n), make_events(n)
            B.moe_profile_kernel(B.PROF[name], st, sp, n)
            armed[name] = (st, sp, n)
        return armed

    def read(armed):
        out = {}
        for name, (st, sp, n) in armed.items():
            B.moe_profile_kernel(B.PROF[name], None, None, 0)
            tot, cnt = 0.0, 0
            for i in range(n):
                f = ctypes.c_float()
                if hip.hipEventElapsedTime(ctypes.byref(f), st[i], sp[i]) == 0:   # never recorded: no such launch
                    tot += f.value
                    cnt += 1
            if cnt:
                out[name] = tot / cnt
        hip.hipGetLastError()   # asking an unrecorded event for its time leaves an error behind: clear it
        return out

    calls = (L.route, L.dispatch, L.ffn_fwd, L.combine, L.combine_bwd, L.ffn_bwd, L.dispatch_bwd, L.route_bwd)
    # detail pass (untimed): every kernel bracketed, plus per-call events; also finds the dominant kernel
    armed = arm(list(B.PROF))
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)] for _ in range(args.steps)]
    for s in range(args.steps):
        e = ev[s]
        e[0].record()
        for i, fn in enumerate(calls):
            fn()
            e[i + 1].record()
    torch.cuda.synchronize()
    kern_ms = read(armed)
    stage_ms = {n: float(np.mean([ev[s][i].elapsed_time(ev[s][i + 1]) for s in range(args.steps)]))
                for i, n in enumerate(STAGES)}
    # bf16 with few tiles: dH shares its launch with dW2 (both under "dh_bwd"), dx with dW1 (under "dx_bwd")
    gemm_names = [n for n in ("gemm1_fwd", "gemm2_fwd", "dh_bwd", "dw2_bwd", "dw1_bwd", "dx_bwd") if n in kern_ms]
    dom = max(gemm_names, key=lambda n: kern_ms[n])

    # timed region: exactly K steps, only the dominant kernel carries its event pair
    armed = arm([dom])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    dom_ms = read(armed)[dom]
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # ---- per-kernel algorithmic work (per launch) and the roofline of the dominant kernel
    swi = w.act == S.ACT_SWIGLU
    per = 18 if swi else 12
    unit = 2 * S_rows * w.d * w.f
    flops = {"gemm1_fwd": unit * (2 if swi else 1), "gemm2_fwd": unit, "dh_bwd": unit, "dw2_bwd": unit,
             "dw1_bwd": unit * (2 if swi else 1), "dx_bwd": unit * (2 if swi else 1)}
    if bf:
        # the library's rule (moe_expert_ffn_bwd): a row-tile GEMM of at most 2048 tiles shares its launch
        # with the weight-gradient GEMM after it, and the shared launch is bracketed under the row-tile GEMM
        max_tiles = (w.T * w.k + 255) // 256 + w.E
        if ((w.f + 255) // 256) * max_tiles <= 2048:
            flops["dh_bwd"] += flops.pop("dw2_bwd")
        if ((w.d + 255) // 256) * max_tiles <= 2048:
            flops["dx_bwd"] += unit
            flops["dw1_bwd"] -= unit
    flops = {n: v for n, v in flops.items() if n in kern_ms}
    es = 2 if bf else 4
    sb = stage_bytes(w, S_rows, es)
    kbytes = {"gather": w.T * w.d * es + S_rows * w.d * es + w.T * w.k * 8, "combine": sb["combine"],
              "combine_bwd": sb["combine_bwd"], "route": sb["route"]}
    peak = PEAK_BF16_TFLOPS if bf else PEAK_F32_TFLOPS
    kernels = {}
    for name, ms in kern_ms.items():
        d = {"us": round(ms * 1e3, 2)}
        if name in flops:
            tf = flops[name] / (ms * 1e-3) / 1e12
            d.update(flops=flops[name], TFLOPs=round(tf, 1), frac_mfma=round(tf / peak, 4))
        else:
            gb = kbytes[name] / (ms * 1e-3) / 1e9
            d.update(bytes=kbytes[name], GBps=round(gb, 1), frac_hbm=round(gb / PEAK_HBM_GBS, 4))
        kernels[name] = d
    kernels[dom].update(us_timed_region=round(dom_ms * 1e3, 2))
    dom_tf = flops[dom] / (dom_ms * 1e-3) / 1e12
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        tj = json.load(open(tpath))
        traffic = tj.get(w.name, {}).get(dom)
    paired = bf and ((dom == "dh_bwd" and "dw2_bwd" not in kern_ms) or (dom == "dx_bwd" and flops[dom] > unit * (2 if swi else 1)))
    kname = ("gemm_bf16_pair_kernel" if paired else "gemm_bf16_kernel") if bf else "gemm_f32_kernel"
    roofline = {"bound": "mfma", "kernel": f"{kname} ({dom})",
                "achieved": round(dom_tf, 1), "peak": peak, "unit": "TFLOP/s",
                "frac": round(dom_tf / peak, 4), "traffic": traffic, "flops_per_launch": flops[dom],
                "us_per_launch": round(dom_ms * 1e3, 2),
                "all_gemms": {"flops_per_step": per * S_rows * w.d * w.f,
                              "us_per_step": round(sum(kern_ms[n] for n in flops) * 1e3, 1),
                              "TFLOPs": round(per * S_rows * w.d * w.f / sum(kern_ms[n] for n in flops) / 1e9, 1),
                              "frac": round(per * S_rows * w.d * w.f / sum(kern_ms[n] for n in flops) / 1e9 / peak, 4)}}
    stages = {}
    for n in STAGES:
        d = {"ms": round(stage_ms[n], 4)}
        if n in sb:
            gbs = sb[n] / (stage_ms[n] * 1e-3) / 1e9
            d.update(bytes=sb[n], GBps=round(gbs, 1), frac_hbm=round(gbs / PEAK_HBM_GBS, 4))
        stages[n] = d

    # ---- the box itself: CU count and clock behind the MFMA peak, and what a plain device-to-device copy of
    # 1 GiB reaches (read + write bytes over time), the practical ceiling of the HBM-bound kernels
    props = torch.cuda.get_device_properties(dev)
    big_src = torch.empty(512 * 1024 * 1024, dtype=torch.uint8, device=dev)
    big_dst = torch.empty_like(big_src)
    for _ in range(2):
        big_dst.copy_(big_src)
    ce = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ce[0].record()
    for _ in range(5):
        big_dst.copy_(big_src)
    ce[1].record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * big_src.numel() / (ce[0].elapsed_time(ce[1]) * 1e-3) / 1e9
    del big_src, big_dst
    max_clock = None
    try:   # rocminfo: the GPU agent's "Max Clock Freq. (MHz)"
        import re
        import subprocess
        txt = subprocess.run(["rocminfo"], capture_output=True, text=True, timeout=30).stdout
        for agent in txt.split("Agent ")[1:]:
            if "gfx" in agent and "Device Type:             GPU" in agent:
                m = re.search(r"Max Clock Freq\. \(MHz\):\s*(\d+)", agent)
                if m:
                    max_clock = int(m.group(1))
                    break
    except Exception:
        pass
    device = {"name": props.name, "compute_units": props.multi_processor_count, "max_clock_MHz": max_clock,
              "copy_512MiB_GBps": round(copy_gbs, 1), "copy_frac_hbm": round(copy_gbs / PEAK_HBM_GBS, 4)}

    if args.copy_probe:
        src = torch.zeros(64 * 1024 * 1024, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    # ---- CPU baseline: the oracle as it stands, on the host cores
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import moe_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        # bounded sample: the first Ts tokens of the same workload (all experts, same weights)
        target_flops = 1.0e12
        Ts = int(min(w.T, max(256, target_flops // (per * w.k * w.d * w.f))))
        tc = time.perf_counter()
        O.moe_layer(inp["x"][:Ts], inp["Wr"], inp["bias"], inp["W1"], inp.get("W1b"), inp["W2"], inp["d_out"][:Ts],
                    w.k, w.act, capacity=w.capacity)
        dt = time.perf_counter() - tc
        cpu = {"value": round(Ts / dt, 2), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
               "sample": f"first {Ts} of {w.T} tokens of {w.name}, full layer fwd+bwd, numpy fp64, {dt:.1f} s"}

    out = {
        "metric": "moe_layer_fwd_bwd_tokens_per_s",
        "value": round(w.T / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if bf else "f32",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: T={w.T} d_model={w.d} d_ff={w.f} E={w.E} top-{w.k} "
                               f"{'SwiGLU' if w.act == S.ACT_SWIGLU else 'GELU'} rows_computed={S_rows}"
                               + (", activation checkpointing (gate, dispatch, GEMM1 repeated)" if args.checkpoint else "")},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": kernels,
        "stages": stages,
        "device": device,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
