"""Turns rocprofv3 output of `bench.py` runs into the short summaries kept under profiles/.

    python -m paper_2305_17423_amd.profile_summary --trace DIR --fetch DIR --write DIR --mfma DIR --out profiles/NAME

Each DIR is the `-d` directory of one rocprofv3 run of bench.py on the headline workload (the commands are printed
into the summaries).  Only library kernels (`fise::`) of masked steps in the steady state are counted.  Written:

  NAME_kernel_trace.md    per-kernel launches per step / average duration (from --kernel-trace)
  NAME_hbm_traffic.md     per-kernel HBM bytes per launch (FETCH_SIZE, WRITE_SIZE scaled by a plain copy kernel)
  NAME_traffic.json       the same per fise_profile_read kind, with the sha1 of the kernel sources measured
  NAME_mfma_counters.md   MFMA busy cycles / MFMA ops / GPU-active cycles per kernel (--pmc run)

The JSON is what bench.py quotes as `roofline.traffic`; it refuses the figure when the kernel sources changed.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import hashlib
import json
import os
import re

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")

TRACE_CMD = ("rocprofv3 --kernel-trace --stats --output-format csv -d gpurun_out/kt -o run -- "
             "python3 bench.py --no-cpu-baseline --no-dense --no-sweeps --caches 1 --steps 20 --warmup 3")
PMC_CMD = ("rocprofv3 --pmc {c} --output-format csv -d gpurun_out/{d} -o run -- "
           "python3 bench.py --no-cpu-baseline --no-dense --no-sweeps --steps 3 --warmup 1 --caches 1 --calibrate-copy")


def kernel_sources_sha1() -> str:
    """sha1 over the library's kernel sources (names and contents, in name order)."""
    h = hashlib.sha1()
    for f in sorted(os.listdir(CSRC)):
        if f.endswith((".hip", ".h", ".cpp")):
            h.update(f.encode())
            h.update(open(os.path.join(CSRC, f), "rb").read())
    return h.hexdigest()


def short(name: str) -> str:
    name = re.sub(r"^void ", "", name)
    name = re.sub(r"\(.*$", "", name)
    return name


def kind_of(name: str):
    """The fise_profile_read kind (as bench.py names it) a profiler kernel name belongs to, or None."""
    n = short(name)
    if "igemm_wsk_kernel" in n:
        return "igemm_wsk_kernel<32|64,NW,3>"
    if "igemm_dma_kernel<64, 64, 2, 2" in n:
        return "igemm_dma_kernel<64,64,2,2,3,*>"
    if "igemm_dma_kernel<64, 128, 2, 2" in n or "igemm_dma_kernel<32, 256" in n:
        return "igemm_dma_kernel<64,128,2,2,3,*> / <32,256,1,4,3,*> (GEGLU)"
    if "igemm_dma_kernel<64, 128, 2, 4" in n:
        return "igemm_dma_kernel<64,128,2,4,3,*>"
    if "igemm_dma_kernel<32, 128" in n:
        return "igemm_dma_kernel<32,128,1,4,3,*>"
    if "igemm_reduce" in n:
        return "igemm_reduce_kernel / igemm_reduce_ln_kernel"
    if "igemm_kernel" in n:
        return "igemm_kernel<...> (GroupNorm prologue)"
    if "attention_merge" in n:
        return "attention_merge_kernel"
    if "attention_kernel" in n:
        return "attention_kernel"
    return None


def _rows(d, pattern):
    f = glob.glob(os.path.join(d, "**", pattern), recursive=True)
    if not f:
        raise FileNotFoundError(f"{pattern} under {d}")
    return list(csv.DictReader(open(f[0])))


def _steps(rows, key_start="Start_Timestamp"):
    """Index ranges of whole steps: each begins with the mask-detection kernel."""
    rows.sort(key=lambda r: int(r[key_start]))
    starts = [i for i, r in enumerate(rows) if "pixel_diff_kernel" in r["Kernel_Name"]]
    return [(a, b) for a, b in zip(starts[:-1], starts[1:])]


def summarize_trace(d, out):
    rows = _rows(d, "*kernel_trace.csv")
    steps = _steps(rows)
    sizes = collections.Counter(b - a for a, b in steps)
    n_launch = sizes.most_common(1)[0][0]                       # the steady-state masked step
    steady = [(a, b) for a, b in steps if b - a == n_launch][2:]
    agg = collections.OrderedDict()
    span = 0.0
    for a, b in steady:
        span += (int(rows[b]["Start_Timestamp"]) - int(rows[a]["Start_Timestamp"])) / 1e3
        for r in rows[a:b]:
            if "fise::" not in r["Kernel_Name"]:
                continue
            e = agg.setdefault(short(r["Kernel_Name"]), [0, 0.0, 1e30, 0.0])
            dur = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
            e[0] += 1; e[1] += dur; e[2] = min(e[2], dur); e[3] = max(e[3], dur)
    ns = len(steady)
    total = sum(v[1] for v in agg.values()) / ns
    lines = ["# Masked UNet step (SD-1.5 shapes, batch 2, 64x64 latent, 10 % blob = 12 of 64 tiles): per-kernel times", "",
             "Command (on the MI355X box, from the repository root, after `cd /tmp && export TMPDIR=/tmp`):", "", "```", TRACE_CMD, "```", "",
             f"Steady state: {ns} consecutive masked steps of `run_kernel_trace.csv`, {n_launch} launches per step "
             f"(mask detection + UNet step), summed kernel durations {total / 1e3:.3f} ms per step, start-to-start "
             f"{span / ns / 1e3:.3f} ms per step under the profiler.", "",
             "| kernel | launches/step | average us | min us | max us | ms/step | % of step |", "|---|---:|---:|---:|---:|---:|---:|"]
    for k, v in sorted(agg.items(), key=lambda kv: -kv[1][1]):
        lines.append(f"| `{k}` | {v[0] / ns:.0f} | {v[1] / v[0]:.2f} | {v[2]:.2f} | {v[3]:.2f} | {v[1] / ns / 1e3:.3f} | {100 * v[1] / ns / total:.1f} |")
    by_kind = collections.OrderedDict()
    for k, v in agg.items():
        kd = kind_of(k)
        if kd:
            e = by_kind.setdefault(kd, [0, 0.0])
            e[0] += v[0]; e[1] += v[1]
    lines += ["", "By `fise_profile_read` kind (what bench.py's `kernels` / `roofline` entries are set against):", "",
              "| kind | launches/step | average us |", "|---|---:|---:|"]
    for k, v in sorted(by_kind.items(), key=lambda kv: -kv[1][1]):
        lines.append(f"| {k} | {v[0] / ns:.0f} | {v[1] / v[0]:.2f} |")
    open(out + "_kernel_trace.md", "w").write("\n".join(lines) + "\n")
    return {k: v[1] / v[0] for k, v in by_kind.items()}


def _pmc(d, counter):
    """[(kernel name, value)] in dispatch order, and the masked steps among them."""
    rows = [r for r in _rows(d, "*counter_collection.csv") if r["Counter_Name"] == counter]
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    return rows


def _after_copy(rows):
    """Steady masked steps after the calibration copy kernel (bench.py --calibrate-copy), and that kernel's row."""
    cal = [i for i, r in enumerate(rows) if "CUDAFunctor_add" in r["Kernel_Name"] or "AddFunctor" in r["Kernel_Name"] or
           ("vectorized_elementwise_kernel" in r["Kernel_Name"] and int(r["Grid_Size"]) >= (64 << 20) // 8)]
    if not cal:
        raise RuntimeError("calibration copy kernel not found (run bench.py with --calibrate-copy)")
    ci = cal[-1]
    starts = [i for i, r in enumerate(rows) if "pixel_diff_kernel" in r["Kernel_Name"] and i > ci]
    steps = [(a, b) for a, b in zip(starts[:-1], starts[1:])]
    sizes = collections.Counter(b - a for a, b in steps)
    n_launch = sizes.most_common(1)[0][0]
    return rows[ci], [(a, b) for a, b in steps if b - a == n_launch]


def summarize_traffic(df, dw, out):
    res = {}
    factors = {}
    nsteps = 0
    for counter, d in (("FETCH_SIZE", df), ("WRITE_SIZE", dw)):
        rows = _pmc(d, counter)
        cal, steps = _after_copy(rows)
        factors[counter] = 262144.0 / float(cal["Counter_Value"])          # the copy reads and writes 256 MiB = 262144 KiB
        nsteps = len(steps)
        for a, b in steps:
            for r in rows[a:b]:
                if "fise::" not in r["Kernel_Name"]:
                    continue
                e = res.setdefault(short(r["Kernel_Name"]), {"n": {"FETCH_SIZE": 0, "WRITE_SIZE": 0}, "FETCH_SIZE": 0.0, "WRITE_SIZE": 0.0})
                e["n"][counter] += 1; e[counter] += float(r["Counter_Value"]) * factors[counter]
    lines = ["# HBM traffic of the masked UNet step's kernels (SD-1.5 shapes, 10 % blob): FETCH_SIZE / WRITE_SIZE", "",
             "Commands (two runs, one counter each; on the MI355X box, from the repository root, after `cd /tmp && export TMPDIR=/tmp`):", "", "```",
             PMC_CMD.format(c="FETCH_SIZE", d="pmc_f"), PMC_CMD.format(c="WRITE_SIZE", d="pmc_w"), "```", "",
             "`--calibrate-copy` adds one plain elementwise kernel that reads 256 MiB and writes 256 MiB (262144 KiB each): the counters are "
             f"scaled by what they read for it (FETCH_SIZE x {factors['FETCH_SIZE']:.3f}, WRITE_SIZE x {factors['WRITE_SIZE']:.3f}).  "
             f"Masked steps after that kernel ({nsteps}), scaled, per launch and per step:", "",
             "| kernel | launches/step | fetched KiB/launch | written KiB/launch | fetched MiB/step | written MiB/step |", "|---|---:|---:|---:|---:|---:|"]
    tot_f = tot_w = 0.0
    for k, e in sorted(res.items(), key=lambda kv: -(kv[1]["FETCH_SIZE"] + kv[1]["WRITE_SIZE"])):
        nf, nw = max(e["n"]["FETCH_SIZE"], 1), max(e["n"]["WRITE_SIZE"], 1)
        lines.append(f"| `{k}` | {nf / nsteps:.0f} | {e['FETCH_SIZE'] / nf:.1f} | {e['WRITE_SIZE'] / nw:.1f} | "
                     f"{e['FETCH_SIZE'] / nsteps / 1024:.1f} | {e['WRITE_SIZE'] / nsteps / 1024:.1f} |")
        tot_f += e["FETCH_SIZE"] / nsteps / 1024; tot_w += e["WRITE_SIZE"] / nsteps / 1024
    lines.append(f"| all library kernels | | | | {tot_f:.1f} | {tot_w:.1f} |")
    per_kind = {}
    for k, e in res.items():
        kd = kind_of(k)
        if kd:
            p = per_kind.setdefault(kd, {"launches": 0, "fetch_kib": 0.0, "write_kib": 0.0})
            p["launches"] += e["n"]["FETCH_SIZE"]; p["fetch_kib"] += e["FETCH_SIZE"]; p["write_kib"] += e["WRITE_SIZE"]
    js = {"workload": "config 5, SD-1.5 shapes, 64x64 latent, 10 % blob, 8x8 base tiles",
          "command": "rocprofv3 --pmc FETCH_SIZE | WRITE_SIZE -- python3 bench.py --no-cpu-baseline --no-dense --no-sweeps --steps 3 --warmup 1 --caches 1 --calibrate-copy",
          "kernel_sources_sha1": kernel_sources_sha1(), "scale": factors, "steps_counted": nsteps, "per_kind": {}}
    for kd, p in per_kind.items():
        n = max(p["launches"], 1)
        js["per_kind"][kd] = {"launches_per_step": p["launches"] / nsteps, "fetch_kib_per_launch": p["fetch_kib"] / n,
                              "write_kib_per_launch": p["write_kib"] / n, "hbm_bytes_per_launch": (p["fetch_kib"] + p["write_kib"]) / n * 1024}
    open(out + "_hbm_traffic.md", "w").write("\n".join(lines) + "\n")
    json.dump(js, open(out + "_traffic.json", "w"), indent=1)


def summarize_mfma(d, out, avg_us):
    names = ("SQ_VALU_MFMA_BUSY_CYCLES", "SQ_INSTS_VALU_MFMA_MOPS_BF16", "SQ_BUSY_CYCLES", "GRBM_GUI_ACTIVE")
    per = {}
    nsteps = 0
    for c in names:
        rows = _pmc(d, c)
        if not rows:
            continue
        starts = [i for i, r in enumerate(rows) if "pixel_diff_kernel" in r["Kernel_Name"]]
        steps = [(a, b) for a, b in zip(starts[:-1], starts[1:])]
        sizes = collections.Counter(b - a for a, b in steps)
        n_launch = sizes.most_common(1)[0][0]
        steps = [(a, b) for a, b in steps if b - a == n_launch][1:]
        nsteps = len(steps)
        for a, b in steps:
            for r in rows[a:b]:
                if "fise::" not in r["Kernel_Name"]:
                    continue
                e = per.setdefault(short(r["Kernel_Name"]), collections.defaultdict(float))
                e[c] += float(r["Counter_Value"]); e["n_" + c] += 1
    lines = ["# MFMA counters of the masked UNet step's kernels (SD-1.5 shapes, 10 % blob)", "",
             "Command (its own run: counters only; on the MI355X box, from the repository root, after `cd /tmp && export TMPDIR=/tmp`):", "", "```",
             "rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_BUSY_CYCLES GRBM_GUI_ACTIVE --output-format csv "
             "-d gpurun_out/pmc_m -o run -- python3 bench.py --no-cpu-baseline --no-dense --no-sweeps --steps 3 --warmup 1 --caches 1", "```", "",
             f"Per launch, averaged over {nsteps} masked steps.  `MFMA busy` = SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE x 1024 SIMDs): the share "
             "of SIMD-cycles, while the kernel had the GPU, in which a matrix unit was executing (the profiler's MfmaUtil).  `GFLOP` = "
             "SQ_INSTS_VALU_MFMA_MOPS_BF16 x 512 / 1e9, the bf16 matrix operations actually issued (padding included).", "",
             "| kernel | launches/step | GPU-active cycles | MFMA busy % | MFMA GFLOP/launch | TFLOP/s while active (2.4 GHz) |", "|---|---:|---:|---:|---:|---:|"]
    for k, e in sorted(per.items(), key=lambda kv: -kv[1]["GRBM_GUI_ACTIVE"]):
        n = max(e["n_GRBM_GUI_ACTIVE"], 1)
        act = e["GRBM_GUI_ACTIVE"] / n
        busy = e["SQ_VALU_MFMA_BUSY_CYCLES"] / max(e["n_SQ_VALU_MFMA_BUSY_CYCLES"], 1)
        gflop = e["SQ_INSTS_VALU_MFMA_MOPS_BF16"] / max(e["n_SQ_INSTS_VALU_MFMA_MOPS_BF16"], 1) * 512 / 1e9
        util = 100.0 * busy / (act * 1024) if act else 0.0
        tf = gflop / (act / 2.4e9) / 1e3 if act else 0.0
        lines.append(f"| `{k}` | {n / nsteps:.0f} | {act:.0f} | {util:.2f} | {gflop:.4f} | {tf:.1f} |")
    open(out + "_mfma_counters.md", "w").write("\n".join(lines) + "\n")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--trace"); ap.add_argument("--fetch"); ap.add_argument("--write"); ap.add_argument("--mfma")
    ap.add_argument("--out", required=True, help="output prefix, e.g. profiles/masked_unet_step_sd15_10pct")
    a = ap.parse_args()
    avg = summarize_trace(a.trace, a.out) if a.trace else {}
    if a.fetch and a.write:
        summarize_traffic(a.fetch, a.write, a.out)
    if a.mfma:
        summarize_mfma(a.mfma, a.out, avg)


if __name__ == "__main__":
    main()
