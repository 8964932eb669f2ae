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

TRACE_CMD = ("rocprofv3 --kernel-trace --stats --output-format csv -d {d} -o run -- "
             "python3 bench.py --no-cpu-baseline --no-dense --no-sweeps --caches 1 --steps 20 --warmup 3")
PMC_CMD = ("rocprofv3 --pmc {c} --output-format csv -d {d} -o run -- "
           "python3 bench.py --no-cpu-baseline --no-dense --no-sweeps --steps 3 --warmup 1 --caches 1")
COPY_KIB = 1048576.0        # bench.py ends with fise_calibrate_peaks on a 2 GiB scratch: each copy launch reads and writes 1 GiB


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
             "Command (on the MI355X box, from the repository root, after `cd /tmp && export TMPDIR=/tmp`):", "", "```", TRACE_CMD.format(d=os.path.normpath(d)), "```", "",
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
    per_kernel = {k: v[1] / v[0] for k, v in agg.items()}
    for r in rows:                                    # the calibration kernels run once, after the steps
        if "calib_" in r["Kernel_Name"]:
            e = per_kernel.setdefault("_n_" + short(r["Kernel_Name"]), [0, 0.0])
            e[0] += 1; e[1] += (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
    for k in [k for k in per_kernel if k.startswith("_n_")]:
        n, tot = per_kernel.pop(k)
        per_kernel[k[3:]] = tot / n
    return per_kernel


def _pmc(d, counter):
    """[(kernel name, value)] in dispatch order, and the masked steps among them."""
    rows = [r for r in _rows(d, "*counter_collection.csv") if r["Counter_Name"] == counter]
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    return rows


def _steady_steps(rows):
    """Index ranges of the steady-state masked steps (each begins with the mask-detection kernel; the most common
    launch count is the masked step's)."""
    starts = [i for i, r in enumerate(rows) if "pixel_diff_kernel" in r["Kernel_Name"]]
    steps = [(a, b) for a, b in zip(starts[:-1], starts[1:])]
    n_launch = collections.Counter(b - a for a, b in steps).most_common(1)[0][0]
    return [(a, b) for a, b in steps if b - a == n_launch][1:]


def _copy_scale(rows):
    """What the counter reads for the library's own plain copy kernel of known size (median over its launches)."""
    v = sorted(float(r["Counter_Value"]) for r in rows if "calib_copy_kernel" in r["Kernel_Name"])
    if not v:
        raise RuntimeError("fise::calib_copy_kernel not in the run (bench.py calls fise_calibrate_peaks at its end)")
    return COPY_KIB / v[len(v) // 2]


def summarize_traffic(df, dw, out):
    res = {}
    factors = {}
    nsteps = 0
    for counter, d in (("FETCH_SIZE", df), ("WRITE_SIZE", dw)):
        rows = _pmc(d, counter)
        steps = _steady_steps(rows)
        factors[counter] = _copy_scale(rows)
        nsteps = len(steps)
        for a, b in steps:
            for r in rows[a:b]:
                if "fise::" not in r["Kernel_Name"]:
                    continue
                e = res.setdefault(short(r["Kernel_Name"]), {"n": {"FETCH_SIZE": 0, "WRITE_SIZE": 0}, "FETCH_SIZE": 0.0, "WRITE_SIZE": 0.0})
                e["n"][counter] += 1; e[counter] += float(r["Counter_Value"]) * factors[counter]
    lines = ["# HBM traffic of the masked UNet step's kernels (SD-1.5 shapes, 10 % blob): FETCH_SIZE / WRITE_SIZE", "",
             "Commands (two runs, one counter each; on the MI355X box, from the repository root, after `cd /tmp && export TMPDIR=/tmp`):", "", "```",
             PMC_CMD.format(c="FETCH_SIZE", d=os.path.normpath(df)), PMC_CMD.format(c="WRITE_SIZE", d=os.path.normpath(dw)), "```", "",
             "bench.py ends with `fise_calibrate_peaks`, whose plain copy kernel (`fise::calib_copy_kernel`) reads 1 GiB and writes 1 GiB per "
             f"launch: the counters are scaled by what they read for it (FETCH_SIZE x {factors['FETCH_SIZE']:.3f}, WRITE_SIZE x "
             f"{factors['WRITE_SIZE']:.3f}).  Steady-state masked steps ({nsteps}), scaled, per launch and per step:", "",
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
          "command": "rocprofv3 --pmc FETCH_SIZE | WRITE_SIZE -- python3 bench.py --no-cpu-baseline --no-dense --no-sweeps --steps 3 --warmup 1 --caches 1",
          "kernel_sources_sha1": kernel_sources_sha1(), "scale": factors, "steps_counted": nsteps, "per_kind": {}}
    for kd, p in per_kind.items():
        n = max(p["launches"], 1)
        js["per_kind"][kd] = {"launches_per_step": p["launches"] / nsteps, "fetch_kib_per_launch": p["fetch_kib"] / n,
                              "write_kib_per_launch": p["write_kib"] / n, "hbm_bytes_per_launch": (p["fetch_kib"] + p["write_kib"]) / n * 1024}
    open(out + "_hbm_traffic.md", "w").write("\n".join(lines) + "\n")
    json.dump(js, open(out + "_traffic.json", "w"), indent=1)


def summarize_mfma(d, out, avg_us):
    """avg_us: kernel name -> average duration from the kernel-trace run (the counter run serialises and slows kernels)."""
    names = ("MfmaUtil", "SQ_INSTS_VALU_MFMA_MOPS_BF16", "GRBM_GUI_ACTIVE")
    per = {}
    nsteps = 0
    for c in names:
        rows = _pmc(d, c)
        if not rows:
            continue
        steps = _steady_steps(rows)
        nsteps = len(steps)
        for a, b in steps:
            for r in rows[a:b]:
                if "fise::" not in r["Kernel_Name"]:
                    continue
                e = per.setdefault(short(r["Kernel_Name"]), collections.defaultdict(float))
                e[c] += float(r["Counter_Value"]); e["n_" + c] += 1
        for r in rows:                                # reference rows: the calibration kernels at the end of the run
            if "calib_" in r["Kernel_Name"]:
                e = per.setdefault(short(r["Kernel_Name"]), collections.defaultdict(float))
                e[c] += float(r["Counter_Value"]); e["n_" + c] += 1
    lines = ["# MFMA counters of the masked UNet step's kernels (SD-1.5 shapes, 10 % blob)", "",
             "Command (its own run: counters only; on the MI355X box, from the repository root, after `cd /tmp && export TMPDIR=/tmp`):", "", "```",
             PMC_CMD.format(c="MfmaUtil SQ_INSTS_VALU_MFMA_MOPS_BF16 GRBM_GUI_ACTIVE", d=os.path.normpath(d)), "```", "",
             f"Per launch, averaged over {nsteps} steady-state masked steps.  `MfmaUtil` is the profiler's derived counter "
             "100 x SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE x SIMDs): the share of SIMD-cycles, while the kernel had the GPU, in which a "
             "matrix unit was executing.  `MFMA GFLOP` = SQ_INSTS_VALU_MFMA_MOPS_BF16 x 512 / 1e9: the bf16 matrix operations actually issued "
             "(tile padding included).  `TFLOP/s` divides it by the kernel's average duration in the kernel-trace run (the counter run "
             "serialises dispatches and is slower); `% of peak` is against 2.5 PFLOP/s.  The last rows are bench.py's calibration kernels "
             "(a register-resident MFMA loop and a plain copy) as a check of what the counters read at the two extremes.", "",
             "| kernel | launches/step | MfmaUtil % | MFMA GFLOP/launch | average us | issued TFLOP/s | % of MFMA peak |", "|---|---:|---:|---:|---:|---:|---:|"]

    def row(k, e, n_steps):
        n = max(e["n_MfmaUtil"], 1)
        util = e["MfmaUtil"] / n
        gflop = e["SQ_INSTS_VALU_MFMA_MOPS_BF16"] / max(e["n_SQ_INSTS_VALU_MFMA_MOPS_BF16"], 1) * 512 / 1e9
        us = avg_us.get(k)
        tf = gflop / us * 1e3 if us else float("nan")
        per_step = f"{n / n_steps:.0f}" if n_steps else "-"
        return f"| `{k}` | {per_step} | {util:.2f} | {gflop:.4f} | {us if us is None else round(us, 2)} | {tf:.1f} | {tf / 2500 * 100:.2f} |"
    main_rows = {k: e for k, e in per.items() if "calib_" not in k}
    for k, e in sorted(main_rows.items(), key=lambda kv: -kv[1]["SQ_INSTS_VALU_MFMA_MOPS_BF16"]):
        lines.append(row(k, e, nsteps))
    for k, e in per.items():
        if "calib_" in k:
            lines.append(row(k, e, 0))
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
