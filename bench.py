#!/usr/bin/env python3
"""Benchmark of the MoE expert layer hot path on one MI355X.

One "step" = one forward + backward pass of the whole layer (gate, dispatch, expert FFN, combine and
their backward) over one batch of seeded synthetic input that is already resident in HBM.
Prints ONE JSON line: whole-layer tokens/s of the headline workload (the largest single-GPU
configuration, cfg3), a roofline object for its dominant kernel (the bf16 MFMA grouped GEMM) measured
with HIP events inside the timed region, per-kernel and per-stage timings (mean, median, min; the
HBM-bound kernels cold and warm), the CPU oracle timed on the host cores as a reported baseline, and
the step time and all-GEMM fraction of the other benchmark configurations under `other_workloads`.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3] [--also cfg1,cfg2,cfg4|none]
                  [--no-cpu-baseline] [--full-oracle] [--checkpoint] [--f16] [--overlap-gate-bwd]
                  [--clock-probe] [--mfma-loop] [--copy-probe]
"""
from __future__ import annotations

import argparse
import ctypes
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
HBM_STAGES = ("route", "dispatch", "combine", "combine_bwd", "dispatch_bwd", "route_bwd")
EVICT_BYTES = 1 << 30         # written between cold iterations: four times the 256 MB memory-side cache


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


def stats(xs):
    import numpy as np
    a = np.asarray(xs, dtype=np.float64)
    return {"mean": float(a.mean()), "median": float(np.median(a)), "min": float(a.min())}


class Events:
    """hipEvent_t handles for the library's timing brackets (a caller-owned moe_prof)."""

    def __init__(self, B):
        self.B = B
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.prof = B.MoeProf()
        self.arrays = {}

    def _make(self, n):
        arr = (ctypes.c_void_p * n)()
        for i in range(n):
            h = ctypes.c_void_p()
            assert self.hip.hipEventCreate(ctypes.byref(h)) == 0
            arr[i] = h
        return arr

    def arm(self, cfg, counts):
        """counts: kernel name -> number of launches to bracket."""
        self.disarm(cfg)
        for name, n in counts.items():
            i = self.B.PROF[name]
            st, sp = self._make(n), self._make(n)
            self.arrays[name] = (st, sp, n)
            self.prof.start[i] = ctypes.cast(st, ctypes.POINTER(ctypes.c_void_p))
            self.prof.stop[i] = ctypes.cast(sp, ctypes.POINTER(ctypes.c_void_p))
            self.prof.n[i] = n
            self.prof.count[i] = 0
        cfg.prof = ctypes.pointer(self.prof)

    def disarm(self, cfg):
        cfg.prof = None
        for i in range(self.B.PROF_COUNT):
            self.prof.n[i] = 0
        for st, sp, n in self.arrays.values():
            for i in range(n):
                self.hip.hipEventDestroy(st[i])
                self.hip.hipEventDestroy(sp[i])
        self.arrays = {}

    def read(self, cfg):
        """kernel name -> list of milliseconds, one per bracketed launch that was recorded, in launch order."""
        out = {}
        for name, (st, sp, n) in self.arrays.items():
            ms = []
            for i in range(min(n, int(self.prof.count[self.B.PROF[name]]))):
                f = ctypes.c_float()
                if self.hip.hipEventElapsedTime(ctypes.byref(f), st[i], sp[i]) == 0:
                    ms.append(f.value)
            if ms:
                out[name] = ms
        self.hip.hipGetLastError()
        self.disarm(cfg)
        return out


def gemm_flops(w, S_rows, S, present):
    """Algorithmic FLOPs per launch of each GEMM bracket (the library's launch-sharing rule applied)."""
    swi = w.act == S.ACT_SWIGLU
    unit = 2 * S_rows * w.d * w.f
    flops = {"gemm1_fwd": unit * (2 if swi else 1), "gemm2_fwd": unit, "dh_bwd": unit, "dw2_bwd": unit,
             "dw1_bwd": unit * (2 if swi else 1), "dx_bwd": unit * (2 if swi else 1)}
    if w.dtype != S.DT_F32:
        # moe_expert_ffn_bwd: a row-tile GEMM of at most 2048 tiles shares its launch with the weight-gradient
        # GEMM after it, and the shared launch is bracketed under the row-tile GEMM
        max_tiles = (w.T * w.k + 255) // 256 + w.E
        if ((w.f + 255) // 256) * max_tiles <= 2048:
            flops["dh_bwd"] += flops.pop("dw2_bwd")
        if ((w.d + 255) // 256) * max_tiles <= 2048:
            flops["dx_bwd"] += unit
            flops["dw1_bwd"] -= unit
    return {n: v for n, v in flops.items() if n in present and v > 0}


def run_workload(name, steps, warmup, args, full):
    """Times one workload.  full: detail pass, cold pass and roofline; otherwise step time and GEMM brackets only."""
    import numpy as np
    import torch
    from paper_2504_03871_amd import synth as S
    from paper_2504_03871_amd import binding as B
    from paper_2504_03871_amd.layer import MoELayer

    w = S.WORKLOADS[name]
    if args.f16 and w.dtype == S.DT_BF16:
        w = w.scaled(dtype=S.DT_F16)
    inp = S.make_inputs(w, threads=16)
    bf = w.dtype != S.DT_F32      # 16-bit storage: the MFMA path
    dev = "cuda:0"
    L = MoELayer(w.T, w.d, w.f, w.E, w.k, dtype=w.dtype, act=w.act, capacity=w.capacity, device=dev)
    if args.overlap_gate_bwd:
        L.enable_gate_overlap()

    def up(nm):
        if bf:
            return torch.from_numpy(inp[nm + "_bits"].view(np.int16)).to(dev).view(torch.float16 if w.dtype == S.DT_F16 else torch.bfloat16)
        return torch.from_numpy(inp[nm]).to(dev)

    for nm in ("x", "W1", "W2", "d_out") + (("W1b",) if w.act == S.ACT_SWIGLU else ()):
        getattr(L, nm).copy_(up(nm))
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
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()

    evs = Events(B)
    calls = (L.route, L.dispatch, L.ffn_fwd, L.combine, L.combine_bwd, L.ffn_bwd, L.dispatch_bwd, L.route_bwd)
    # ---- detail pass (untimed): every kernel bracketed, plus events around every library call
    per_step = {n: (2 if n == "combine" else 1) for n in B.PROF}   # combine also serves the input-gradient un-permute
    evs.arm(L.cfg, {n: steps * per_step[n] for n in B.PROF})
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)] for _ in range(steps)]
    for s in range(steps):
        e = ev[s]
        e[0].record()
        for i, fn in enumerate(calls):
            fn()
            e[i + 1].record()
    torch.cuda.synchronize()
    kern_ms = evs.read(L.cfg)
    if "combine" in kern_ms:   # launches alternate: combine, then the un-permute of the input gradient
        kern_ms["dispatch_bwd"] = kern_ms["combine"][1::2]
        kern_ms["combine"] = kern_ms["combine"][0::2]
    stage_ms = {n: [ev[s][i].elapsed_time(ev[s][i + 1]) for s in range(steps)] for i, n in enumerate(STAGES)}
    flops = gemm_flops(w, S_rows, S, kern_ms)
    dom = max(flops, key=lambda n: np.mean(kern_ms[n]))

    # ---- optional: the shader clock the chip sustains under this work.  One-wave samplers on side streams record
    # (shader counter, 100 MHz counter) pairs; single samples on the work's own stream before and after the steps
    # bracket the loaded interval in the same 100 MHz time base, so only samples taken inside it are counted (a side
    # stream that happens to share a hardware queue with the work runs before or after it and contributes none).
    if full and args.clock_probe:
        n_s, sleeps, n_side = 8000, 10, 3    # about 35-50 us between samples, 0.3-0.4 s per sampler
        sides = [torch.cuda.Stream(device=dev) for _ in range(n_side)]
        samples = [torch.zeros(2 * n_s, dtype=torch.int64, device=dev) for _ in range(n_side)]
        marks = torch.zeros(4, dtype=torch.int64, device=dev)
        torch.cuda.synchronize()
        for st_, sm_ in zip(sides, samples):
            with torch.cuda.stream(st_):
                B.moe_bench_clock_probe(sm_, n_s, sleeps)
        time.sleep(0.02)               # the first samples see an idle chip
        B.moe_bench_clock_probe(marks[0:2], 1, 0)
        n_probe_steps = 4
        for _ in range(n_probe_steps):
            step()
        B.moe_bench_clock_probe(marks[2:4], 1, 0)
        torch.cuda.synchronize()
        mk = marks.cpu().numpy()
        t_lo, t_hi = int(mk[1]), int(mk[3])
        loaded, idle = [], []
        for sm_ in samples:
            sm = sm_.cpu().numpy().reshape(n_s, 2).astype(np.int64)
            dt_, dr_ = np.diff(sm[:, 0]).astype(np.float64), np.diff(sm[:, 1]).astype(np.float64)
            ok = dr_ > 0
            mhz = np.where(ok, dt_ / np.maximum(dr_, 1.0) * 100.0, 0.0)
            inside = ok & (sm[:-1, 1] >= t_lo) & (sm[1:, 1] <= t_hi)
            before = ok & (sm[1:, 1] < t_lo)
            loaded.append(mhz[inside]); idle.append(mhz[before])
        loaded, idle = np.concatenate(loaded), np.concatenate(idle)
        res_clock = {"samples_under_load": int(len(loaded)), "samples_idle": int(len(idle)),
                     "idle_MHz_median": round(float(np.median(idle)), 1) if len(idle) else None,
                     "under_load_MHz_median": round(float(np.median(loaded)), 1) if len(loaded) else None,
                     "under_load_MHz_p10": round(float(np.percentile(loaded, 10)), 1) if len(loaded) else None,
                     "under_load_MHz_p90": round(float(np.percentile(loaded, 90)), 1) if len(loaded) else None,
                     "loaded_interval_ms": round((t_hi - t_lo) / 1e5, 2),
                     "steps_in_interval": n_probe_steps, "nominal_MHz": 2400}
    else:
        res_clock = None

    # ---- timed region: exactly K steps, only the dominant kernel carries its event pair
    evs.arm(L.cfg, {dom: steps})
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    dom_ms = evs.read(L.cfg)[dom]
    ms_per_step = (t1 - t0) * 1e3 / steps

    swi = w.act == S.ACT_SWIGLU
    per = 18 if swi else 12
    peak = PEAK_BF16_TFLOPS if bf else PEAK_F32_TFLOPS
    gemm_us = sum(float(np.mean(kern_ms[n])) for n in flops) * 1e3
    all_gemms = {"flops_per_step": per * S_rows * w.d * w.f, "us_per_step": round(gemm_us, 1),
                 "TFLOPs": round(per * S_rows * w.d * w.f / gemm_us / 1e6, 1),
                 "frac": round(per * S_rows * w.d * w.f / gemm_us / 1e6 / peak, 4)}
    workload = (f"{w.name}: T={w.T} d_model={w.d} d_ff={w.f} E={w.E} top-{w.k} "
                f"{'SwiGLU' if swi else 'GELU'} rows_computed={S_rows}"
                + (", activation checkpointing (gate, dispatch, GEMM1 repeated)" if args.checkpoint else ""))
    res = {"w": w, "inp": inp, "S_rows": S_rows, "clock_probe": res_clock, "ms_per_step": ms_per_step, "all_gemms": all_gemms, "workload": workload,
           "dtype": {S.DT_BF16: "bf16", S.DT_F16: "f16"}.get(w.dtype, "f32")}
    if not full:
        del L
        torch.cuda.empty_cache()
        return res

    # ---- cold pass for the HBM-bound stages: a 1 GiB fill by the library's streaming kernel (untimed) pushes
    # the inputs out of the L2s and the memory-side cache before every timed call
    cold_iters = max(20, min(steps, 30))
    scratch = torch.empty(EVICT_BYTES, dtype=torch.uint8, device=dev)
    hbm_calls = {"route": L.route, "dispatch": L.dispatch, "combine": L.combine, "combine_bwd": L.combine_bwd,
                 "dispatch_bwd": L.dispatch_bwd, "route_bwd": L.route_bwd}
    evs.arm(L.cfg, {"route": cold_iters, "gather": cold_iters, "combine": 2 * cold_iters, "combine_bwd": cold_iters})
    cev = {n: [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(cold_iters)]
           for n in HBM_STAGES}
    for it in range(cold_iters):
        for n in HBM_STAGES:
            B.moe_bench_stream(scratch, None, EVICT_BYTES, 1)
            cev[n][it][0].record()
            hbm_calls[n]()
            cev[n][it][1].record()
    torch.cuda.synchronize()
    cold_kern = evs.read(L.cfg)
    if "combine" in cold_kern:
        cold_kern["dispatch_bwd"] = cold_kern["combine"][1::2]
        cold_kern["combine"] = cold_kern["combine"][0::2]
    cold_stage = {n: [a.elapsed_time(b) for a, b in cev[n]] for n in HBM_STAGES}

    # ---- per-kernel report
    es = 2 if bf else 4
    sb = stage_bytes(w, S_rows, es)
    kbytes = {"gather": w.T * w.d * es + S_rows * w.d * es + w.T * w.k * 8, "combine": sb["combine"],
              "combine_bwd": sb["combine_bwd"], "route": sb["route"], "dispatch_bwd": sb["dispatch_bwd"]}
    kernels = {}
    for nm, ms in kern_ms.items():
        st = stats(ms)
        d = {"us": round(st["mean"] * 1e3, 2), "us_median": round(st["median"] * 1e3, 2), "us_min": round(st["min"] * 1e3, 2)}
        if nm in flops:
            tf = flops[nm] / (st["mean"] * 1e-3) / 1e12
            d.update(flops=flops[nm], TFLOPs=round(tf, 1), frac_mfma=round(tf / peak, 4))
        elif nm in kbytes:
            warm = kbytes[nm] / (st["median"] * 1e-3) / 1e9
            d.update(bytes=kbytes[nm], warm_GBps=round(warm, 1))
            if nm in cold_kern:
                cs = stats(cold_kern[nm])
                cold = kbytes[nm] / (cs["median"] * 1e-3) / 1e9
                d.update(cold_us_median=round(cs["median"] * 1e3, 2), cold_us_min=round(cs["min"] * 1e3, 2),
                         cold_GBps=round(cold, 1), frac_hbm=round(cold / PEAK_HBM_GBS, 4))
        kernels[nm] = d
    dom_st = stats(dom_ms)
    kernels[dom].update(us_timed_region=round(dom_st["mean"] * 1e3, 2))
    dom_tf = flops[dom] / (dom_st["mean"] * 1e-3) / 1e12
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(w.name, {}).get(dom)
    paired = bf and ((dom == "dh_bwd" and "dw2_bwd" not in kern_ms) or (dom == "dx_bwd" and flops[dom] > 2 * S_rows * w.d * w.f * (2 if swi else 1)))
    kname = ("gemm_bf16_pair_kernel" if paired else "gemm_bf16_kernel") if bf else "gemm_f32_kernel"
    res["roofline"] = {"bound": "mfma", "kernel": f"{kname} ({dom})", "achieved": round(dom_tf, 1), "peak": peak,
                       "unit": "TFLOP/s", "frac": round(dom_tf / peak, 4), "traffic": traffic,
                       "flops_per_launch": flops[dom], "us_per_launch": round(dom_st["mean"] * 1e3, 2),
                       "us_per_launch_median": round(dom_st["median"] * 1e3, 2),
                       "us_per_launch_min": round(dom_st["min"] * 1e3, 2), "all_gemms": all_gemms}
    stages = {}
    for n in STAGES:
        st = stats(stage_ms[n])
        d = {"ms": round(st["mean"], 4), "ms_median": round(st["median"], 4), "ms_min": round(st["min"], 4)}
        if n in sb:
            warm = sb[n] / (st["median"] * 1e-3) / 1e9
            cs = stats(cold_stage[n])
            cold = sb[n] / (cs["median"] * 1e-3) / 1e9
            d.update(bytes=sb[n], warm_GBps=round(warm, 1), cold_ms_median=round(cs["median"], 4),
                     cold_ms_min=round(cs["min"], 4), cold_GBps=round(cold, 1), frac_hbm=round(cold / PEAK_HBM_GBS, 4))
        stages[n] = d
    res["kernels"], res["stages"] = kernels, stages

    # ---- the box itself: CU count and clock behind the MFMA peak, and what a plain streaming copy of 512 MiB
    # reaches with the library's own kernel (read + write bytes over time): the practical HBM ceiling
    props = torch.cuda.get_device_properties(dev)
    n_copy = 512 << 20
    src, dst = scratch[:n_copy], scratch[n_copy:2 * n_copy]
    for _ in range(2):
        B.moe_bench_stream(dst, src, n_copy, 0)
    ce = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
    for a, b in ce:
        a.record()
        B.moe_bench_stream(dst, src, n_copy, 0)
        b.record()
    te = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    te[0].record()
    for _ in range(5):
        dst.copy_(src)
    te[1].record()
    torch.cuda.synchronize()
    own = 2 * n_copy / (float(np.median([a.elapsed_time(b) for a, b in ce])) * 1e-3) / 1e9
    blit = 5 * 2 * n_copy / (te[0].elapsed_time(te[1]) * 1e-3) / 1e9
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
    res["device"] = {"name": props.name, "compute_units": props.multi_processor_count, "max_clock_MHz": max_clock,
                     "copy_kernel_512MiB_GBps": round(own, 1), "copy_kernel_frac_hbm": round(own / PEAK_HBM_GBS, 4),
                     "runtime_copy_512MiB_GBps": round(blit, 1)}
    if args.mfma_loop:
        # the rate of a kernel of nothing but MFMAs, per instruction shape: what the chip's power management allows
        opnd = (torch.randn(64 * 1024, device=dev) * 0.5).to(torch.bfloat16)
        sink = torch.zeros(1024 * 512, dtype=torch.float32, device=dev)
        iters = 10000
        flop = 1024 * 8 * iters * 32 * 16384
        res["device"]["mfma_loop"] = {}
        for kind, nm in ((0, "16x16x32"), (1, "32x32x16")):
            B.moe_bench_mfma_loop(kind, 2000, opnd, sink)
            torch.cuda.synchronize()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            for i in range(3):
                ev[i].record()
                B.moe_bench_mfma_loop(kind, iters, opnd, sink)
            ev[3].record()
            torch.cuda.synchronize()
            ms = float(np.median([ev[i].elapsed_time(ev[i + 1]) for i in range(3)]))
            res["device"]["mfma_loop"][nm + "_bf16_TFLOPs"] = round(flop / ms / 1e9, 1)
    for nm in ("gather", "combine", "combine_bwd", "dispatch_bwd", "route"):
        if nm in kernels and "cold_GBps" in kernels[nm]:
            kernels[nm]["frac_copy_kernel"] = round(kernels[nm]["cold_GBps"] / own, 4)
    for n in HBM_STAGES:
        stages[n]["frac_copy_kernel"] = round(stages[n]["cold_GBps"] / own, 4)
    del L, scratch
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg3",
                    help="headline workload (default: cfg3, the largest configuration that fits one GPU)")
    ap.add_argument("--also", default="cfg1,cfg2,cfg4",
                    help="comma-separated workloads whose step time and all-GEMM fraction are reported under "
                         "other_workloads ('none' to skip)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--overlap-gate-bwd", action="store_true",
                    help="run the gate's weight gradient on a second stream next to the expert backward "
                         "(measured: no gain; not the default)")
    ap.add_argument("--checkpoint", action="store_true",
                    help="time the step of an activation-checkpointed layer: gate, dispatch and the saved "
                         "activations are computed again before the backward (not the default metric)")
    ap.add_argument("--f16", action="store_true",
                    help="run the bf16 workloads with fp16 storage instead (the paper's FP16 mixed precision; not the default metric)")
    ap.add_argument("--clock-probe", action="store_true",
                    help="sample the shader clock with a one-wave kernel on a second stream while steps run "
                         "(evidence for the clock the chip sustains under the GEMMs; not part of the timed region)")
    ap.add_argument("--full-oracle", action="store_true",
                    help="time the CPU oracle on the whole batch instead of a bounded token sample "
                         "(cfg1: under a minute; cfg3: about an hour of host time)")
    ap.add_argument("--mfma-loop", action="store_true",
                    help="also time a kernel of nothing but MFMAs for both bf16 instruction shapes "
                         "(device.mfma_loop: the matrix-core rate the chip's power management allows)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 256 MiB copy with the library's streaming kernel three times "
                         "(calibrates rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2504_03871_amd import binding as B

    B.lib()   # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)

    r = run_workload(args.workload, args.steps, args.warmup, args, full=True)
    w, inp = r["w"], r["inp"]

    if args.copy_probe:
        src = torch.zeros(64 * 1024 * 1024, dtype=torch.int32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            B.moe_bench_stream(dst, src, src.numel() * 4, 0)
        torch.cuda.synchronize()
        del src, dst

    # ---- CPU baseline: the oracle as it stands, on the host cores
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import moe_oracle as O
        from paper_2504_03871_amd import synth as S
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        # bounded sample: the first Ts tokens of the same workload (all experts, same weights)
        per = 18 if w.act == S.ACT_SWIGLU else 12
        target_flops = 1.2e13
        Ts = int(min(w.T, max(256, target_flops // (per * w.k * w.d * w.f))))
        if args.full_oracle:
            Ts = w.T
        tc = time.perf_counter()
        O.moe_layer(inp["x"][:Ts], inp["Wr"], inp["bias"], inp["W1"], inp.get("W1b"), inp["W2"], inp["d_out"][:Ts],
                    w.k, w.act, capacity=w.capacity)
        dt = time.perf_counter() - tc
        cpu = {"value": round(Ts / dt, 2), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
               "sample": (f"all {w.T} tokens of {w.name}, full layer fwd+bwd, numpy fp64, {dt:.1f} s" if Ts == w.T else
                          f"first {Ts} of {w.T} tokens of {w.name} through all {w.E} experts, full layer fwd+bwd, "
                          f"numpy fp64, {dt:.1f} s; tokens/s = sample tokens / that time (extrapolated to the batch)")}
    del inp
    r.pop("inp")

    others = {}
    if args.also and args.also != "none":
        for nm in args.also.split(","):
            nm = nm.strip()
            if not nm or nm == args.workload:
                continue
            o = run_workload(nm, max(5, args.steps // 2), args.warmup, args, full=False)
            others[nm] = {"workload": o["workload"], "ms_per_step": round(o["ms_per_step"], 4),
                          "tokens_per_s": round(o["w"].T / (o["ms_per_step"] * 1e-3), 1), "all_gemms": o["all_gemms"]}
            del o

    out = {
        "metric": "moe_layer_fwd_bwd_tokens_per_s",
        "value": round(w.T / (r["ms_per_step"] * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(r["ms_per_step"], 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": r["dtype"],
        "data": "synthetic",
        "config": {"workload": r["workload"]},
        "roofline": r["roofline"],
        "cpu_baseline": cpu,
        "kernels": r["kernels"],
        "stages": r["stages"],
        "device": r["device"],
        "clock_probe": r.get("clock_probe"),
        "other_workloads": others,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
