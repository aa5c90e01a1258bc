"""Summaries of rocprofv3 runs of ``bench.py`` and their look-up at benchmark time.

``summarize(run_dir, md_path)`` turns the CSV files of four rocprofv3 passes over the same
``bench.py`` command (kernel trace statistics, FETCH_SIZE, WRITE_SIZE + L2 hits, shader counters;
the commands are written into the summary) into a short Markdown file.  The file ends in a JSON
block that names the workload, feature width, plan options and the digest of the library sources
the run was made with, and gives per kernel the average duration and the calibrated HBM-side
bytes per launch.  ``lookup`` finds the block that matches a benchmark run exactly -- workload,
width, plan options and library sources -- so that a bench line can only ever quote counter traffic
that was measured for the code and plan it is timing; anything else yields ``None``.
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import os

from . import build as _build

PROFILE_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "..", "profiles")
PASSES = {
    "stats": "--kernel-trace --stats",
    "pmc_fetch": "--pmc FETCH_SIZE",
    "pmc_write": "--pmc WRITE_SIZE TCC_HIT_sum TCC_MISS_sum",
    "pmc_sq": "--pmc SQ_WAVES SQ_BUSY_CYCLES SQ_INSTS_VALU SQ_INSTS_VMEM_RD SQ_INSTS_LDS SQ_INSTS_MFMA "
              "SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_SALU GRBM_GUI_ACTIVE",
}
_MARK = "<!-- profile-data -->"


def _short(name: str) -> str:
    return name.split("(")[0].replace("void ", "").strip()


def _find(run_dir: str, sub: str, pattern: str):
    found = glob.glob(os.path.join(run_dir, sub, "**", pattern), recursive=True)
    return found[0] if found else None


def _bench_line(run_dir: str) -> dict:
    """The JSON line bench.py printed under the kernel-trace pass (its stdout is kept as stats.log)."""
    with open(os.path.join(run_dir, "stats.log")) as f:
        lines = [l for l in f.read().splitlines() if l.startswith("{")]
    return json.loads(lines[-1])


def summarize(run_dir: str, md_path: str, bench_args: str) -> dict:
    """Write the summary of the passes found under ``run_dir`` (sub-directories named as PASSES)."""
    line = _bench_line(run_dir)
    cfg = line["config"]
    bench = "python3 bench.py " + bench_args
    out = [f"# rocprofv3 summary: workload `{cfg['workload']}`, N = {cfg['N']}, plan options {json.dumps(cfg['plan_options'])}: "
           "all kernels of one `rsh_spmm` call", "",
           "Commands (run from the repository root on one MI355X; `cd /tmp && export TMPDIR=/tmp` first), then",
           f"`python3 bench.py --summarize-profile OUT --profile-out {os.path.relpath(md_path, os.path.join(PROFILE_DIR, '..'))} "
           f"--profile-args \"{bench_args}\"`:", ""]
    for sub, flags in PASSES.items():
        out.append(f"    rocprofv3 {flags} -d OUT/{sub} -o p --output-format csv -- {bench}   > OUT/{sub}.log")
    out += ["", "## Kernel trace statistics (`--kernel-trace --stats`)", "",
            "| kernel | calls | average (us) | min (us) | max (us) |", "|---|---|---|---|---|"]
    kernels: dict = collections.defaultdict(dict)
    with open(_find(run_dir, "stats", "*kernel_stats.csv")) as f:
        for r in csv.DictReader(f):
            if "rsh::" in r["Name"]:
                k = _short(r["Name"])
                kernels[k].update(calls=int(r["Calls"]), avg_us=float(r["AverageNs"]) / 1e3)
                out.append(f"| `{k}` | {r['Calls']} | {float(r['AverageNs']) / 1e3:.1f} | {float(r['MinNs']) / 1e3:.1f} | "
                           f"{float(r['MaxNs']) / 1e3:.1f} |")
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for sub in ("pmc_fetch", "pmc_write", "pmc_sq"):
        path = _find(run_dir, sub, "*counter_collection.csv")
        if path is None:
            continue
        with open(path) as f:
            for r in csv.DictReader(f):
                if "rsh::" in r["Kernel_Name"]:
                    agg[_short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    mean = {k: {c: sum(v) / len(v) for c, v in d.items()} for k, d in agg.items()}
    probe = mean.get("rsh::rsh_copy_probe_kernel", {})
    if not probe.get("FETCH_SIZE") or not probe.get("WRITE_SIZE"):
        raise RuntimeError("the run holds no calibration copy (bench.py --calibrate-copy)")
    f_scale, w_scale = (1 << 20) / probe["FETCH_SIZE"], (1 << 20) / probe["WRITE_SIZE"]
    out += ["", "## HBM-side traffic per launch (`--pmc FETCH_SIZE`, `--pmc WRITE_SIZE`)", "",
            f"Calibration: `rsh_copy_probe_kernel` copies exactly 1 GiB (reads 1048576 KiB, writes 1048576 KiB); the counters "
            f"read FETCH_SIZE = {probe['FETCH_SIZE']:.0f} and WRITE_SIZE = {probe['WRITE_SIZE']:.0f}, so the scale factors are "
            f"{f_scale:.3f} (fetch) and {w_scale:.3f} (write) KiB per count.", "",
            "| kernel | FETCH_SIZE (raw) | WRITE_SIZE (raw) | fetched (MB) | written (MB) | L2 hit / (hit+miss) |",
            "|---|---|---|---|---|---|"]
    for k, d in mean.items():
        if "copy_probe" in k:
            continue
        fetched, written = d.get("FETCH_SIZE", 0) * f_scale * 1024, d.get("WRITE_SIZE", 0) * w_scale * 1024
        hit = d.get("TCC_HIT_sum", 0) / max(1.0, d.get("TCC_HIT_sum", 0) + d.get("TCC_MISS_sum", 0))
        kernels[k].update(fetched_bytes=int(fetched), written_bytes=int(written), l2_hit=round(hit, 4))
        out.append(f"| `{k}` | {d.get('FETCH_SIZE', 0):.0f} | {d.get('WRITE_SIZE', 0):.0f} | {fetched / 1e6:.1f} | {written / 1e6:.1f} | {hit:.3f} |")
    out += ["", "## Shader counters per launch (`--pmc SQ_*`)", "",
            "MFMA utilisation = SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE x 32 CUs x 4 SIMDs); GRBM_GUI_ACTIVE is the sum over "
            "the 8 XCDs, each with 32 CUs.", "",
            "| kernel | waves | VALU insts | VMEM read insts | LDS insts | SALU insts | MFMA insts | MFMA busy cycles | GPU active cycles | MFMA utilisation |",
            "|---|---|---|---|---|---|---|---|---|---|"]
    for k, d in mean.items():
        if "copy_probe" in k:
            continue
        util = d.get("SQ_VALU_MFMA_BUSY_CYCLES", 0) / max(1.0, d.get("GRBM_GUI_ACTIVE", 0) * 32 * 4)
        kernels[k].update(mfma_util=round(util, 4))
        out.append(f"| `{k}` | {d.get('SQ_WAVES', 0):.0f} | {d.get('SQ_INSTS_VALU', 0):.0f} | {d.get('SQ_INSTS_VMEM_RD', 0):.0f} | "
                   f"{d.get('SQ_INSTS_LDS', 0):.0f} | {d.get('SQ_INSTS_SALU', 0):.0f} | {d.get('SQ_INSTS_MFMA', 0):.0f} | "
                   f"{d.get('SQ_VALU_MFMA_BUSY_CYCLES', 0):.0f} | {d.get('GRBM_GUI_ACTIVE', 0):.0f} | {util:.3f} |")
    keep = ("value", "unit", "ms_per_step", "kernel_ms", "roofline", "hbm_useful_GBps", "bytes_min")
    out += ["", "## The benchmark's own line under the kernel-trace run", "", "```", json.dumps({k: line[k] for k in keep if k in line}), "```"]
    data = {"workload": cfg["workload"], "N": cfg["N"], "plan_options": cfg["plan_options"],
            "library_sources": line.get("library_sources"), "bench_args": bench_args, "kernels": {k: v for k, v in kernels.items() if "copy_probe" not in k}}
    out += ["", "## Machine-readable (read by `bench.py` for `roofline.traffic`)", "", _MARK, "```json", json.dumps(data, sort_keys=True), "```"]
    with open(md_path, "w") as f:
        f.write("\n".join(out) + "\n")
    return data


def _blocks():
    for path in sorted(glob.glob(os.path.join(PROFILE_DIR, "*.md"))):
        with open(path) as f:
            text = f.read()
        at = text.find(_MARK)
        if at < 0:
            continue
        body = text[at:].split("```json", 1)[1].split("```", 1)[0]
        yield os.path.basename(path), json.loads(body)


def lookup(workload: str, N: int, plan_options: dict, kernel_family: str):
    """(traffic bytes per launch, summary file, kernel name) of the kernel whose name contains
    ``kernel_family`` in the summary made for exactly this workload, width, plan options and
    library build; ``None`` when there is none."""
    digest = _build.source_digest()
    # a summary of the plain command first, one that also ran other entry points after it
    for name, data in sorted(_blocks(), key=lambda b: ("--epilogue" in b[1].get("bench_args", ""), b[0])):
        if (data["workload"], data["N"], data["plan_options"], data.get("library_sources")) != (workload, N, plan_options, digest):
            continue
        for kernel, d in data["kernels"].items():
            # rsh_spmm's kernels write fp32 rows (OutPlain); a run with --epilogue also holds the fused ones
            if kernel_family in kernel and "OutPlain" in kernel and "fetched_bytes" in d:
                return d["fetched_bytes"] + d["written_bytes"], name, kernel
    return None
