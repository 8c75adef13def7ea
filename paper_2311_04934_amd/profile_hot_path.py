"""rocprofv3 profile of the benchmark's hot path: kernel durations, HBM bytes per launch, matrix-unit counters.

    python -m paper_2311_04934_amd.profile_hot_path [--workload long_doc_8k] [--out profile_out] [bench flags ...]

Runs `bench.py` once by itself and four times under rocprofv3 (one run per counter group: the profiler does not
split counters over passes) and writes, under --out:

    <workload>[_<tag>]_hot_path.md   a summary in text: the commands, kernel statistics, FETCH_SIZE / WRITE_SIZE per
                                     launch scaled by what the same counter reads for a plain copy of known size
                                     (bench.py --calibrate runs one), and the SQ counters of the attention kernel
    traffic_<workload>[_<tag>].json  the HBM bytes per launch that `bench.py` reports as roofline.traffic, with the
                                     hash of the sources they were measured on

Copy both into profiles/ (merge the json into profiles/traffic.json with --merge) to have them reported; bench.py
prints `null` for a traffic whose source hash is not the one of the library it runs.
Needs a GPU and rocprofv3.  The program under the profiler is `python3 bench.py ...` itself (no shell in between).
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re
import statistics
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SQ_COUNTERS = ["SQ_VALU_MFMA_BUSY_CYCLES", "SQ_INSTS_VALU", "SQ_INSTS_MFMA", "SQ_WAVE_CYCLES", "SQ_WAIT_INST_ANY",
               "SQ_LDS_BANK_CONFLICT", "SQ_LDS_IDX_ACTIVE", "SQ_WAVES", "GRBM_GUI_ACTIVE"]


def kernel_key(name: str):
    """Short name of the library's kernels (None for anything else)."""
    for tag, key in (("attn_bf16_dma_kernel", "attn"), ("attn_bf16_kernel", "attn"), ("attn_combine", "combine"),
                     ("gather_layers_kernel", "gather"), ("gather_append_kernel", "gather"), ("gather_kv_kernel", "gather"),
                     ("append_kernel", "append"), ("calib_copy_kernel", "calib_copy")):
        if tag in name:
            return key
    return None


def short_name(name: str) -> str:
    """Kernel name without its namespaces and parameter list."""
    m = re.match(r"(?:void )?(?:pc::)?(?:\(anonymous namespace\)::)?([A-Za-z_0-9]+(?:<[^>]*>)?)", name)
    return m.group(1) if m else name


def run(cmd, log):
    print("+ " + " ".join(cmd), flush=True)
    with open(log, "w") as f:
        r = subprocess.run(cmd, cwd=ROOT, stdout=f, stderr=subprocess.STDOUT, timeout=900)
    if r.returncode != 0:
        raise RuntimeError(f"{cmd[0]} failed ({r.returncode}), see {log}")


def counters(path):
    """{kernel: {counter: [value per dispatch]}} from a rocprofv3 counter_collection csv."""
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        k = kernel_key(r["Kernel_Name"])
        if k:
            acc[k][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return acc


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="long_doc_8k")
    ap.add_argument("--out", default="profile_out", help="folder for the raw profiler output and the summaries (relative to the repository root)")
    ap.add_argument("--tag", default="", help="suffix of the output names (e.g. the bench mode)")
    ap.add_argument("--merge", default=None, help="traffic json to merge the result into (e.g. profiles/traffic.json)")
    args, bench_flags = ap.parse_known_args(argv)
    sys.path.insert(0, ROOT)
    from paper_2311_04934_amd import build as pc_build
    pc_build.ensure_built()
    out = args.out    # relative to the repository root, where every command runs
    os.makedirs(os.path.join(ROOT, out), exist_ok=True)
    os.chdir(ROOT)
    name = args.workload + ("_" + args.tag if args.tag else "")
    bench = ["python3", "bench.py", "--workload", args.workload, "--no-other-form", "--no-cpu-baseline"] + bench_flags
    short = ["--steps", "2", "--warmup", "1", "--no-full-prefill", "--calibrate"]
    cmds = {}

    # 0. the benchmark by itself: what its HIP events read without a profiler attached
    cmds["plain"] = bench
    run(cmds["plain"], os.path.join(out, name + "_plain.log"))
    # 1. durations
    d_stats = os.path.join(out, name + "_stats")
    cmds["stats"] = ["rocprofv3", "--kernel-trace", "--stats", "--output-format", "csv", "-d", d_stats, "-o", "bench", "--"] + bench
    run(cmds["stats"], d_stats + ".log")
    # 2.-4. counters, one group per run
    groups = {"fetch": ["FETCH_SIZE"], "write": ["WRITE_SIZE"], "sq": SQ_COUNTERS}
    dirs = {}
    for g, names in groups.items():
        dirs[g] = os.path.join(out, f"{name}_pmc_{g}")
        cmds[g] = ["rocprofv3", "--pmc"] + names + ["--kernel-trace", "--output-format", "csv", "-d", dirs[g], "-o", g, "--"] + bench + short
        run(cmds[g], dirs[g] + ".log")

    def find(d, suffix):
        hits = glob.glob(os.path.join(d, "**", "*" + suffix), recursive=True)
        if not hits:
            raise RuntimeError(f"no *{suffix} under {d}")
        return hits[0]

    # ---- kernel statistics
    lines = [f"# rocprofv3 summary: hot path on `{args.workload}`" + (f" ({args.tag})" if args.tag else ""), "",
             f"Sources: hash `{pc_build.source_hash()}` (paper_2311_04934_amd.build.source_hash).  Commands run from the repository root.", "",
             "## Kernel durations", "", "Command: `" + " ".join(cmds["stats"]) + "`", "",
             "| kernel | calls | avg us | min us | max us | % of GPU time |", "|---|---|---|---|---|---|"]
    for r in csv.DictReader(open(find(d_stats, "kernel_stats.csv"))):
        if kernel_key(r["Name"]):
            lines.append(f'| {short_name(r["Name"])} | {r["Calls"]} | {float(r["AverageNs"]) / 1e3:.2f} | {float(r["MinNs"]) / 1e3:.2f} | '
                         f'{float(r["MaxNs"]) / 1e3:.2f} | {r["Percentage"]} |')
    # the attention kernel without the full-prefill comparison's launches (the long ones)
    durs = collections.defaultdict(list)
    for r in csv.DictReader(open(find(d_stats, "kernel_trace.csv"))):
        k = kernel_key(r["Kernel_Name"])
        if k:
            durs[k].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    if durs["attn"]:
        med = statistics.median(durs["attn"])
        hot = [x for x in durs["attn"] if x < 5 * med]
        lines += ["", f"Attention kernel over its {len(hot)} hot-path launches alone (launches shorter than 5x the median; the others "
                      f"are the full-prefill comparison): average **{sum(hot) / len(hot):.2f} us**, median {statistics.median(hot):.2f} us."]
    bench_line = None
    for ln in open(os.path.join(out, name + "_plain.log")):
        if ln.startswith("{"):
            bench_line = json.loads(ln)
    if bench_line:
        lines += ["", "`" + " ".join(cmds["plain"]) + "` just before, on the same machine, without the profiler (HIP events carried by the "
                  "launches; average us per launch): " + json.dumps(bench_line.get("kernels_us")) +
                  f", {bench_line['per_layer']['cached_us']} us per layer, value {bench_line['value']}, roofline.frac {bench_line.get('roofline', {}).get('frac')}.",
                  "The profiler's own cost per dispatch is inside its durations; a kernel that does nothing measures 3.9 us with either method."]

    # ---- HBM traffic
    fetch, write = counters(find(dirs["fetch"], "counter_collection.csv")), counters(find(dirs["write"], "counter_collection.csv"))
    calib_bytes = float(1 << 30)    # bench.py --calibrate copies 1 GiB: that many bytes fetched and as many written per launch
    f_raw = statistics.median(fetch["calib_copy"]["FETCH_SIZE"]) * 1024.0
    w_raw = statistics.median(write["calib_copy"]["WRITE_SIZE"]) * 1024.0
    f_scale, w_scale = calib_bytes / f_raw, calib_bytes / w_raw
    lines += ["", "## HBM traffic per launch", "", "Commands (one counter per run):", "`" + " ".join(cmds["fetch"]) + "`", "and the same with `--pmc WRITE_SIZE`.", "",
              f"Calibration: `calib_copy_kernel` copies 1 GiB; FETCH_SIZE reads {f_raw / 1024:.0f} KiB for it (factor {f_scale:.3f}), "
              f"WRITE_SIZE {w_raw / 1024:.0f} KiB (factor {w_scale:.3f}).", "",
              "| kernel | launches | FETCH_SIZE raw KiB (median) | fetched MB | WRITE_SIZE raw KiB (median) | written MB |", "|---|---|---|---|---|---|"]
    if bench_line:
        pl = bench_line["per_layer"]
        lines += ["", f"Algorithmic bytes (`bench.py`, per layer): assembly {pl['assemble_mbytes']} MB (written + unique read), attention "
                  f"{pl.get('attn_mbytes')} MB (K and V once, Q read, output written; the partial results of KV splits, "
                  "n_splits x rows x heads x 264 B written by the attention kernel and read by the merge, come on top)."]
    traffic = {}
    for k in ("gather", "append", "attn", "combine"):
        if k not in fetch:
            continue
        fr, wr = statistics.median(fetch[k]["FETCH_SIZE"]), statistics.median(write[k]["WRITE_SIZE"])
        fb, wb = fr * 1024 * f_scale, wr * 1024 * w_scale
        traffic[k] = {"fetched_bytes": round(fb), "written_bytes": round(wb)}
        lines.append(f"| {k} | {len(fetch[k]['FETCH_SIZE'])} | {fr:.1f} | {fb / 1e6:.2f} | {wr:.1f} | {wb / 1e6:.2f} |")

    # ---- SQ counters of the attention kernel
    sq = counters(find(dirs["sq"], "counter_collection.csv"))
    lines += ["", "## Attention kernel, SQ counters (median per launch)", "", "Command: `" + " ".join(cmds["sq"]) + "`", "", "| counter | value |", "|---|---|"]
    for c in sorted(sq.get("attn", {})):
        lines.append(f"| {c} | {statistics.median(sq['attn'][c]):.0f} |")
    a = sq.get("attn", {})
    if "SQ_VALU_MFMA_BUSY_CYCLES" in a and "GRBM_GUI_ACTIVE" in a:
        cycles = statistics.median(a["GRBM_GUI_ACTIVE"]) / 8.0    # the counter is summed over the 8 XCDs
        lines += ["", f"GRBM_GUI_ACTIVE is summed over the 8 XCDs: {cycles:.0f} cycles per XCD.  Matrix pipes busy = SQ_VALU_MFMA_BUSY_CYCLES / "
                      f"(cycles x 1024 SIMDs) = {statistics.median(a['SQ_VALU_MFMA_BUSY_CYCLES']) / (cycles * 1024):.3f} of the launch "
                      "(launch, prologue and epilogue included; counters slow the kernel down a little)."]

    if "SQ_LDS_BANK_CONFLICT" in a and "SQ_LDS_IDX_ACTIVE" in a:
        lines += [f"LDS: {statistics.median(a['SQ_LDS_BANK_CONFLICT']) / max(statistics.median(a['SQ_LDS_IDX_ACTIVE']), 1):.3f} of the LDS-active cycles are "
                  "bank-conflict cycles (SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE)."]
    md = os.path.join(out, name + "_hot_path.md")
    with open(md, "w") as f:
        f.write("\n".join(lines) + "\n")
    cfg = (bench_line or {}).get("config", {})
    entry = {"source_hash": pc_build.source_hash(), "workload": args.workload, "kv_path": cfg.get("kv_path"), "assembly": cfg.get("assembly"),
             "q_rotation": cfg.get("q_rotation"), "fetch_scale": round(f_scale, 4), "write_scale": round(w_scale, 4), "kernels": traffic}
    tj = os.path.join(out, f"traffic_{name}.json")
    with open(tj, "w") as f:
        json.dump(entry, f, indent=1)
    if args.merge:
        path = os.path.join(ROOT, args.merge)
        allt = json.load(open(path)) if os.path.exists(path) else {}
        allt[name] = entry
        with open(path, "w") as f:
            json.dump(allt, f, indent=1, sort_keys=True)
    print(open(md).read())
    return 0


if __name__ == "__main__":
    sys.exit(main())
