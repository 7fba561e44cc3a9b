"""Turns rocprofv3 CSV output of `bench.py` runs into the short text summaries kept under profiles/.

  python -m paper_2504_03871_amd.profsummary --workload cfg3 [--trace DIR] [--fetch DIR --write DIR] [--busy DIR]
                                             [--bench-json FILE] [--out profiles]

DIR is the `-d` directory of a rocprofv3 run made with `--output-format csv -o <workload>`:
  (all runs with -M, mangled kernel names: the demangler garbles the bf16 template argument)
  --trace  rocprofv3 -M --kernel-trace --stats ... -- python3 bench.py --workload W --also none --no-cpu-baseline
  --fetch  rocprofv3 --pmc FETCH_SIZE ...       -- python3 bench.py --workload W --also none --no-cpu-baseline --steps 3 --warmup 1
  --write  rocprofv3 --pmc WRITE_SIZE ...       (same bench command)
  --busy   rocprofv3 --pmc SQ_BUSY_CU_CYCLES SQ_VALU_MFMA_BUSY_CYCLES SQ_WAVE_CYCLES SQ_WAIT_ANY
           SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_VMEM_TA_ADDR_FIFO_FULL SQ_LDS_BANK_CONFLICT SQ_ACTIVE_INST_LDS ... (same)
Byte counters are calibrated on the library's own streaming copy, which bench.py runs on 512 MiB for its
`device` entry in every run: the largest per-dispatch value of `bench_stream_kernel<false>` stands for
524288 KiB read (FETCH_SIZE) and written (WRITE_SIZE).
Also updates profiles/hbm_traffic.json (bytes per launch of each GEMM bracket), which bench.py reads for
`roofline.traffic`.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re


def find_csv(d, suffix):
    hits = glob.glob(os.path.join(d, "**", f"*{suffix}"), recursive=True)
    if not hits:
        raise SystemExit(f"no *{suffix} under {d}")
    return sorted(hits)[-1]


def gemm_role(name, nth=0):
    """(bench bracket, description) of a grouped-GEMM kernel from its MANGLED name (rocprofv3 -M: its demangler
    does not know the bf16 type); nth = index of the launch within a step for the weight-gradient kernel, which
    serves dW2, dW1 (and dW1b) in that order."""
    m = re.search(r"gemm_bf16_pair_kernelIDF16[b_]Li(\d)ELi(\d)ELb([01])E", name)
    if m:
        epi, chain = int(m.group(2)), m.group(3) == "1"
        if epi in (3, 4):
            return "dh_bwd", "dH = dy W2^T with the activation-derivative epilogue, and dW2 = H^T dy, one launch"
        return "dx_bwd", "dx = dA W1^T" + (" (two chained products)" if chain else "") + ", and dW1 = x_perm^T dA, one launch"
    m = re.search(r"gemm_bf16_kernelIDF16[b_]Li(\d)ELi(\d)ELb([01])ELb([01])E", name)
    if not m:
        return None, ""
    mode, epi, dual, chain = int(m.group(1)), int(m.group(2)), m.group(3) == "1", m.group(4) == "1"
    if mode == 0 and epi == 1:
        return "gemm1_fwd", "A = x_perm W1, H = gelu(A)"
    if mode == 0 and epi == 2:
        return "gemm1_fwd", "G = x_perm W1, U = x_perm W1b, H = silu(G) U (two accumulator sets)"
    if mode == 0 and epi == 0:
        return "gemm2_fwd", "y_perm = H W2"
    if mode == 1 and epi in (3, 4):
        return "dh_bwd", "dH = dy W2^T with the activation-derivative epilogue"
    if mode == 1 and epi == 0:
        return "dx_bwd", "dx_perm = dA W1^T" + (" (dG W1^T + dU W1b^T chained)" if chain else "")
    if mode == 2:
        return ("dw2_bwd", "dw1_bwd", "dw1_bwd")[min(nth, 2)], "weight gradient x^T dy (dW2, then dW1, then dW1b for SwiGLU)"
    return None, ""


def short(n):
    """Readable form of a mangled kernel name: the function name and, for the GEMMs, the integer template arguments
    <MODE, EPI, DUAL, CHAIN, BM, BN, BK, waves M, waves N, stages> (pair: <MODE1, EPI1, CHAIN1, BK1, NB1, MODE2, ...>)."""
    m = re.search(r"_ZN3moe\d+([a-z_0-9]+?)I(.*?)EEv", n)
    if m and m.group(1).startswith("gemm_bf16"):
        args = re.findall(r"L[ib](\d+)E", m.group(2))
        st = "bf16" if "DF16b" in m.group(2) else ("f16" if "DF16_" in m.group(2) else "")
        return f"{m.group(1)}<{st}, {', '.join(args)}>"
    m = re.search(r"_ZN3moe\d+([a-z_0-9]+?)(?:I|E)", n)
    if m:
        return m.group(1)
    return n.split("(")[0].replace("void ", "")


def per_kernel(path, counter=None):
    """kernel name -> list of (dispatch id, {counter: value}) in dispatch order."""
    rows = collections.OrderedDict()
    for r in csv.DictReader(open(path)):
        key = (int(r["Dispatch_Id"]), r["Kernel_Name"])
        rows.setdefault(key, {})[r["Counter_Name"]] = float(r["Counter_Value"])
    out = collections.OrderedDict()
    for (did, name), v in sorted(rows.items()):
        out.setdefault(name, []).append((did, v))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--title", default="")
    ap.add_argument("--trace")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--busy")
    ap.add_argument("--bench-json")
    ap.add_argument("--clock-log", help="output of bench.py --clock-probe: writes <workload>_shader_clock.md")
    ap.add_argument("--mfma-log", help="output of bench.py --mfma-loop: writes mfma_loop_rates.md")
    ap.add_argument("--out", default="profiles")
    ap.add_argument("--f16", action="store_true", help="the runs were made with bench.py --f16: files are named <workload>_f16_...")
    a = ap.parse_args()
    w = a.workload
    title = a.title or w
    bench = None
    if a.bench_json:
        line = [x for x in open(a.bench_json) if x.startswith("{")][-1]
        bench = json.loads(line)
        title = bench["config"]["workload"]
    bench_cmd = f"python3 bench.py --workload {w} --also none --no-cpu-baseline" + (" --f16" if a.f16 else "")
    tag = w + ("_f16" if a.f16 else "")   # file name stem
    if a.f16:
        title += " (fp16 storage)"

    if a.mfma_log:
        j = json.loads([x for x in open(a.mfma_log) if x.startswith("{")][-1])
        m = j["device"]["mfma_loop"]
        r16, r32 = m["16x16x32_bf16_TFLOPs"], m["32x32x16_bf16_TFLOPs"]
        out = ["# Rate of a kernel of nothing but bf16 MFMAs, by instruction shape", "",
               f"Command: `{bench_cmd} --mfma-loop` (the kernel is the library's `moe_bench_mfma_loop`: 1024 blocks of eight",
               "waves, 32 independent accumulations per round on register operands drawn from random bf16 data, no memory",
               "traffic in the loop; median of three launches of 10000 rounds).", "",
               "| instruction | TFLOP/s | of the published 2500 | implied clock (256 CUs x 4096 FLOP per clock) |", "|---|---|---|---|",
               f"| v_mfma_f32_16x16x32_bf16 | {r16} | {r16 / 2500:.3f} | {r16 / 2500 * 2.4:.2f} GHz |",
               f"| v_mfma_f32_32x32x16_bf16 | {r32} | {r32 / 2500:.3f} | {r32 / 2500 * 2.4:.2f} GHz |", "",
               "Both shapes do the same FLOP per cycle, and in both loops the SQ counters show the matrix cores busy 99 % of",
               "the cycles (SQ_VALU_MFMA_BUSY_CYCLES / (4 x SQ_BUSY_CU_CYCLES) = 0.99), so the difference is the clock the chip",
               f"holds: the 32 x 32 x 16 shape moves twice the accumulator registers per FLOP and runs {r16 / r32:.2f} times slower.",
               "This is why the grouped GEMM uses 16 x 16 x 32, and it bounds what any bf16 GEMM can reach on this box:",
               f"{r16 / 2500:.2f} of the published peak before a single operand byte is moved."]
        open(os.path.join(a.out, "mfma_loop_rates.md"), "w").write("\n".join(out) + "\n")

    if a.clock_log:
        j = json.loads([x for x in open(a.clock_log) if x.startswith("{")][-1])
        c, g = j["clock_probe"], j["roofline"]["all_gemms"]
        ceil = 2500.0 * c["under_load_MHz_median"] / 2400.0
        out = [f"# Shader clock under the {w} step (bench.py --clock-probe)", "",
               f"Command: `{bench_cmd} --clock-probe` (committed files only).  The sampler is the library's",
               "`moe_bench_clock_probe`: one wave per side stream (three of them) that stores the shader cycle counter and the",
               "100 MHz counter every 35-50 us; single samples on the work's own stream before and after four steps bracket",
               "the loaded interval in the same time base, and only samples inside it count as \"under load\".", "",
               "| quantity | value |", "|---|---|",
               f"| samples before the load (idle chip) | {c['samples_idle']} |",
               f"| idle clock, median | {c['idle_MHz_median']} MHz |",
               f"| samples inside the loaded interval | {c['samples_under_load']} |",
               f"| clock under load, median | {c['under_load_MHz_median']} MHz |",
               f"| clock under load, 10th / 90th percentile | {c['under_load_MHz_p10']} / {c['under_load_MHz_p90']} MHz |",
               f"| loaded interval ({c['steps_in_interval']} steps) | {c['loaded_interval_ms']} ms |",
               f"| ms per step in the timed region of the same run | {j['ms_per_step']} |",
               f"| all GEMMs of a step | {g['TFLOPs']} TFLOP/s = {g['frac']} of 2500 |", "",
               "The published 2.5 PFLOP/s bf16 figure is 256 CUs x 4 matrix cores x 1024 FLOP per clock at 2.4 GHz.  Under this",
               f"workload the chip holds about {c['under_load_MHz_median'] / 2400.0:.2f} of that clock (power management, not something a kernel sets",
               f"directly), which puts the matrix-core ceiling of this run at about {ceil:.0f} TFLOP/s; the GEMMs of a step reach",
               f"{g['TFLOPs'] / ceil:.2f} of that.  bench.py's `frac` stays priced against the published 2500.", "",
               "The clock depends on the instruction mix.  With the 32 x 32 x 16 MFMA the same probe read a median of 1656 MHz",
               "under the same workload; a loop of nothing but MFMAs (matrix cores busy 99 % of cycles by the SQ counters in",
               "both cases) runs at 1880 TFLOP/s with 32 x 32 x 16 and at 2140 TFLOP/s with 16 x 16 x 32."]
        open(os.path.join(a.out, f"{tag}_shader_clock.md"), "w").write("\n".join(out) + "\n")

    if a.trace:
        rows = list(csv.DictReader(open(find_csv(a.trace, "kernel_stats.csv"))))
        out = [f"# {title}: per-kernel durations", "",
               "Command (run from /tmp with TMPDIR=/tmp on the MI355X box):", "",
               f"    rocprofv3 -M --kernel-trace --stats --output-format csv -d <out> -o {w} -- {bench_cmd}", "",
               "bench.py runs its warm-up steps, a detail pass (every kernel bracketed by events), the timed steps and a",
               "cold pass of the HBM-bound calls; durations in microseconds over all of them.", "",
               "| kernel | calls | avg us | min us | max us | % of GPU time | role |", "|---|---|---|---|---|---|---|"]
        for r in rows:
            if "at::native" in r["Name"] or "rocclr" in r["Name"]:
                continue
            role, desc = gemm_role(r["Name"])
            if role and role.startswith("dw"):
                role = "dw2_bwd / dw1_bwd"
            out.append(f"| `{short(r['Name'])}` | {r['Calls']} | {float(r['AverageNs'])/1e3:.1f} | {float(r['MinNs'])/1e3:.1f} | "
                       f"{float(r['MaxNs'])/1e3:.1f} | {float(r['Percentage']):.2f} | {((role or '') + '  ' + desc).strip()} |")
        if bench:
            rf = bench["roofline"]
            out += ["", f"bench.py line of the same run: {bench['ms_per_step']} ms/step, {bench['value']:.0f} tokens/s; dominant kernel "
                    f"{rf['kernel']}: {rf['us_per_launch']} us per launch by HIP events in the timed region (median "
                    f"{rf['us_per_launch_median']}, min {rf['us_per_launch_min']}), {rf['achieved']} TFLOP/s "
                    f"({rf['frac']*100:.1f} % of the {rf['peak']:.0f} TFLOP/s bf16 / fp16 peak); all GEMM launches of a step: "
                    f"{rf['all_gemms']['us_per_step']} us, {rf['all_gemms']['TFLOPs']} TFLOP/s ({rf['all_gemms']['frac']*100:.1f} %)."]
        open(os.path.join(a.out, f"{tag}_kernel_trace_stats.md"), "w").write("\n".join(out) + "\n")

    if a.fetch and a.write:
        pf = per_kernel(find_csv(a.fetch, "counter_collection.csv"))
        pw = per_kernel(find_csv(a.write, "counter_collection.csv"))
        copy = [k for k in pf if "bench_stream_kernelILb0E" in k]
        if not copy:
            raise SystemExit("no copy dispatch (bench_stream_kernel<false>) found for calibration")
        cf = max(v["FETCH_SIZE"] for _, v in pf[copy[0]])
        cw = max(v["WRITE_SIZE"] for _, v in pw[copy[0]])
        sf, sw = 524288.0 / cf, 524288.0 / cw
        lines = [f"# {title}: HBM traffic of the grouped-GEMM kernels from rocprofv3 counters", "",
                 "Commands (each counter in a run of its own; run from /tmp with TMPDIR=/tmp):", "",
                 f"    rocprofv3 -M --pmc FETCH_SIZE --output-format csv -d <out> -o {w} -- {bench_cmd} --steps 3 --warmup 1",
                 f"    rocprofv3 -M --pmc WRITE_SIZE --output-format csv -d <out> -o {w} -- {bench_cmd} --steps 3 --warmup 1", "",
                 "Calibration: the library's 512 MiB streaming copy that bench.py times for its `device` entry (524288 KiB read,",
                 f"524288 KiB written) reads FETCH_SIZE = {cf:.1f} and WRITE_SIZE = {cw:.1f} per dispatch, so FETCH_SIZE is scaled",
                 f"by {sf:.3f} and WRITE_SIZE by {sw:.3f} to get KiB.  Averages over the dispatches of each kind.", "",
                 "| launch | read MiB | written MiB | total bytes | role |", "|---|---|---|---|---|"]
        tj = {}
        for k in pf:
            role0, _ = gemm_role(k)
            if role0 is None or k not in pw:
                continue
            groups = collections.OrderedDict()
            tn = role0.startswith("dw")
            n_per = 1
            if tn and bench:     # launches per step of the weight-gradient kernel
                n_per = 3 if "SwiGLU" in bench["config"]["workload"] else 2
            for i, ((_, vf), (_, vw)) in enumerate(zip(pf[k], pw[k])):
                role, desc = gemm_role(k, i % n_per if tn else 0)
                groups.setdefault((role, desc), []).append((vf["FETCH_SIZE"] * sf, vw["WRITE_SIZE"] * sw))
            for (role, desc), vals in groups.items():
                rd = sum(x for x, _ in vals) / len(vals)
                wr = sum(y for _, y in vals) / len(vals)
                tot = int((rd + wr) * 1024)
                if tn and n_per == 3 and role == "dw1_bwd":
                    tot *= 2     # the bracket holds both launches (dW1 and dW1b)
                tj[role] = tot
                lines.append(f"| {role} | {rd/1024:.1f} | {wr/1024:.1f} | {tot} | {desc} |")
        lines += ["", "Reads above the algorithmic figure are operand panels fetched again by tiles whose L2 (4 MB per XCD) no longer",
                  "holds them; the counter sits between the L2s and the memory-side cache, so part of it never reaches HBM."]
        open(os.path.join(a.out, f"{tag}_gemm_hbm_traffic.md"), "w").write("\n".join(lines) + "\n")
        tpath = os.path.join(a.out, "hbm_traffic.json")
        cur = json.load(open(tpath)) if os.path.exists(tpath) else {}
        cur[w] = tj
        cur["_note"] = ("bytes per launch of each GEMM bracket (FETCH_SIZE and WRITE_SIZE scaled to KiB by the copy "
                        "calibration), written by paper_2504_03871_amd/profsummary.py; see <workload>_gemm_hbm_traffic.md")
        json.dump(cur, open(tpath, "w"), indent=1)

    if a.busy:
        pk = per_kernel(find_csv(a.busy, "counter_collection.csv"))
        lines = [f"# {title}: matrix-core occupancy of the grouped-GEMM launches from rocprofv3 counters", "",
                 "Command (run from /tmp with TMPDIR=/tmp on the MI355X box):", "",
                 "    rocprofv3 -M --pmc SQ_BUSY_CU_CYCLES SQ_VALU_MFMA_BUSY_CYCLES SQ_WAVE_CYCLES SQ_WAIT_ANY SQ_INSTS_VALU_MFMA_MOPS_BF16 "
                 f"SQ_VMEM_TA_ADDR_FIFO_FULL SQ_LDS_BANK_CONFLICT SQ_ACTIVE_INST_LDS --output-format csv -d <out> -o {w} -- {bench_cmd} --steps 3 --warmup 1", "",
                 "Averages per dispatch.  SQ_VALU_MFMA_BUSY_CYCLES counts the four SIMDs of a compute unit separately, so",
                 "busy / (4 x SQ_BUSY_CU_CYCLES) is the share of a busy compute unit's cycles in which a matrix core works.", "",
                 "| launch | MFMA busy / (4 x busy CU cycles) | wait-any / wave cycles | LDS bank-conflict cycles / busy CU cycles | address FIFO full / busy CU cycles | MFMA MOPS (bf16) |",
                 "|---|---|---|---|---|---|"]
        for k, lst in pk.items():
            role0, _ = gemm_role(k)
            if role0 is None:
                continue
            acc = collections.Counter()
            for _, v in lst:
                acc.update(v)
            n = len(lst)
            b = acc["SQ_BUSY_CU_CYCLES"] / n
            name = "dW (all weight gradients)" if role0.startswith("dw") else role0
            lines.append(f"| {name} `{short(k)}` | {acc['SQ_VALU_MFMA_BUSY_CYCLES']/n/b/4:.2f} | {acc['SQ_WAIT_ANY']/max(acc['SQ_WAVE_CYCLES'],1):.2f} | "
                         f"{acc['SQ_LDS_BANK_CONFLICT']/n/b:.3f} | {acc['SQ_VMEM_TA_ADDR_FIFO_FULL']/n/b:.3f} | {acc['SQ_INSTS_VALU_MFMA_MOPS_BF16']/n:.0f} |")
        open(os.path.join(a.out, f"{tag}_gemm_mfma_busy.md"), "w").write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
