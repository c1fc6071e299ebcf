"""Turns the rocprofv3 counter runs of ``bench.py`` into the tracked summary ``profiles/kernel_counters.txt``.

    python3 -m paper_2305_18513_amd.profile_counters OUT/pc > profiles/kernel_counters.txt

(``OUT`` is any scratch folder.)  ``OUT/pc`` holds, for every profiled configuration C, the output folders of three runs (each started
from the repository root after ``cd /tmp && export TMPDIR=/tmp``, one counter set per run):

    rocprofv3 --pmc SQ_INSTS_VALU SQ_INSTS_SALU -d OUT/pc/cfgC_insts -o r --output-format csv -- \\
        python3 bench.py --config C --steps 1 --warmup 0 --no-cpu-baseline --no-extras --no-other-configs
    rocprofv3 --pmc FETCH_SIZE -d OUT/pc/cfgC_fetch -o r --output-format csv -- \\
        python3 bench.py --config C --steps 1 --warmup 0 --no-cpu-baseline --no-extras --no-other-configs --calibrate-copy
    rocprofv3 --pmc WRITE_SIZE -d OUT/pc/cfgC_write -o r --output-format csv -- \\
        python3 bench.py --config C --steps 1 --warmup 0 --no-cpu-baseline --no-extras --no-other-configs --calibrate-copy

and, for the operations bench.py times outside the step (its "extras"), two more runs of the default configuration
with the extras left in:

    rocprofv3 --pmc FETCH_SIZE -d OUT/pc/extras_fetch -o r --output-format csv -- \\
        python3 bench.py --steps 1 --warmup 0 --no-cpu-baseline --no-other-configs --calibrate-copy
    rocprofv3 --pmc WRITE_SIZE -d OUT/pc/extras_write -o r --output-format csv -- \\
        python3 bench.py --steps 1 --warmup 0 --no-cpu-baseline --no-other-configs --calibrate-copy

The byte counters (KiB per dispatch) are scaled by what the same counter reads for the 1 GiB device copies of
``--calibrate-copy`` in the same run.  ``bench.py`` reads the ``DATA`` lines of the summary (HBM traffic of the
dominant kernel, instructions per row for the bound rule); nothing here is needed to run the library.
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import re
import sys

from . import synth

GIB_KIB = 1048576.0

# bench.py's kernel names -> the library kernels behind them
KERNELS = {
    "prune_scores": r"prune_rows(_short)?_kernel",
    "layer_delta": r"layer_delta_partials_kernel",
    "quant_pack": r"quant_pack_kernel",
    "dequant_unpack": r"dequant_unpack_kernel",
}


# bench.py's extras -> (kernels of one call, the kernel that runs once per call)
EXTRAS = {
    "restore_scores": (r"restore_tile_kernel", r"restore_tile_kernel"),
    "quant_pack[scores, fixed 4.4]": (r"quant_pack_kernel<\w+, 8, false", r"quant_pack_kernel<\w+, 8, false"),
    "prune_global[ln_in, 10%]": (r"(hist|bracket|count|write)_kernel<\w+, true, false", r"write_kernel<\w+, true, false"),
    "restore_global[ln_in, tile pointers]": (r"restore_tiles_kernel", r"restore_tiles_kernel"),
    "restore_global[ln_in, zeros+scatter]": (r"(zero|scatter)_kernel", r"scatter_kernel"),
    "gelu_quant_pack[gelu_in]": (r"quant_pack_kernel<[^>]*, true>", r"quant_pack_kernel<[^>]*, true>"),
    "gelu_backward_dequant[gelu_in]": (r"dequant_unpack_kernel<[^>]*, true>", r"dequant_unpack_kernel<[^>]*, true>"),
    "softmax_prune[scores as logits]": (r"prune_rows_kernel<\w+, \d+, \w+, \w+, true>", r"prune_rows_kernel<\w+, \d+, \w+, \w+, true>"),
    "softmax_backward_pruned[scores]": (r"softmax_backward_(tile|small)_kernel", r"softmax_backward_(tile|small)_kernel"),
    "layernorm_forward[ln_in]": (r"layernorm_forward_kernel", r"layernorm_forward_kernel"),
    "prune_global_standardized[ln_in, 10%]": (r"(hist|bracket|count|write)_kernel<\w+, true, true", r"write_kernel<\w+, true, true"),
    "layernorm_backward_pruned[ln_in]": (r"layernorm_backward_pruned_kernel", r"layernorm_backward_pruned_kernel"),
    "layernorm_forward_quant_pack[ln_in]": (r"layernorm_forward_quant_kernel", r"layernorm_forward_quant_kernel"),
    "layernorm_backward_dequant[ln_in]": (r"layernorm_backward_dequant_kernel", r"layernorm_backward_dequant_kernel"),
    "apply_update_layer_delta[all weight tensors]": (r"layer_delta_partials_kernel<\w+, \w+, \w+, true>", r"layer_delta_partials_kernel<\w+, \w+, \w+, true>"),
}


def _per_call(rows, counter, pat_all, pat_once):
    """Sum of the counter over a call's kernels, averaged over the calls of the run."""
    total, calls = 0.0, 0
    for r in rows:
        if r.get("Counter_Name") != counter:
            continue
        if re.search(pat_all, r["Kernel_Name"]):
            total += float(r["Counter_Value"])
        if re.search(pat_once, r["Kernel_Name"]):
            calls += 1
    return (total / calls, calls) if calls else (None, 0)


def summarise_extras(root):
    fetch = _rows(os.path.join(root, "extras_fetch"))
    write = _rows(os.path.join(root, "extras_write"))
    if not (fetch and write):
        return [], []
    fs, _ = _copy_scale(fetch, "FETCH_SIZE")
    wsc, _ = _copy_scale(write, "WRITE_SIZE")
    if not (fs and wsc):
        return [], []
    lines = ["operations outside the timed step (bench.py's extras), default configuration: HBM bytes per call"]
    data = []
    for name, (pat_all, pat_once) in EXTRAS.items():
        f, calls = _per_call(fetch, "FETCH_SIZE", pat_all, pat_once)
        w, _ = _per_call(write, "WRITE_SIZE", pat_all, pat_once)
        if f is None or w is None:
            continue
        fb, wb = f * fs * 1024.0, w * wsc * 1024.0
        lines.append("  %-46s fetched %.1f MB + written %.1f MB = %.1f MB (mean of %d calls)" % (name, fb / 1e6, wb / 1e6, (fb + wb) / 1e6, calls))
        data.append("DATA config=-1 kernel=%s fetch_bytes=%.6g write_bytes=%.6g launches=%d" % (name.replace(" ", "_"), fb, wb, calls))
    lines.append("")
    return lines, data


def _rows(folder):
    paths = glob.glob(os.path.join(folder, "**", "*counter_collection.csv"), recursive=True)
    if not paths:
        return []
    with open(paths[0]) as fh:
        return list(csv.DictReader(fh))


def _by_kernel(rows, counter):
    """{bench kernel name: [values per launch]}; quant / dequant split by launch size into [gelu_in] and [ln_in]."""
    groups = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in rows:
        if r.get("Counter_Name") != counter:
            continue
        for name, pat in KERNELS.items():
            if re.search(pat, r["Kernel_Name"]):
                groups[name][int(r.get("Grid_Size", 0) or 0)].append(float(r["Counter_Value"]))
    out = {}
    for name, by_grid in groups.items():
        if name in ("quant_pack", "dequant_unpack") and len(by_grid) > 1:
            grids = sorted(by_grid)
            out[name + "[gelu_in]"] = by_grid[grids[-1]]
            out[name + "[ln_in]"] = [v for g in grids[:-1] for v in by_grid[g]]
        elif name in ("quant_pack", "dequant_unpack"):
            out[name + "[gelu_in]"] = [v for vs in by_grid.values() for v in vs]
        else:
            out[name] = [v for vs in by_grid.values() for v in vs]
    return out


def _copy_scale(rows, counter):
    vals = [float(r["Counter_Value"]) for r in rows if r.get("Counter_Name") == counter and "copyBuffer" in r["Kernel_Name"]]
    return (GIB_KIB / max(vals), max(vals)) if vals and max(vals) > 0 else (None, None)


def summarise(root):
    lines, data = [], []
    for cfg in synth.CONFIGS:
        c = cfg.index
        insts = _rows(os.path.join(root, "cfg%d_insts" % c))
        fetch = _rows(os.path.join(root, "cfg%d_fetch" % c))
        write = _rows(os.path.join(root, "cfg%d_write" % c))
        if not (insts or fetch or write):
            continue
        lines.append("config %d (%s-shaped): score rows %d x %d, keep %d" % (c, cfg.name, cfg.score_rows, cfg.score_cols, cfg.keep_k))
        valu, salu = _by_kernel(insts, "SQ_INSTS_VALU"), _by_kernel(insts, "SQ_INSTS_SALU")
        fs, fraw = _copy_scale(fetch, "FETCH_SIZE")
        wsc, wraw = _copy_scale(write, "WRITE_SIZE")
        if fs and wsc:
            lines.append("  calibration: a 1 GiB device copy reads FETCH_SIZE %.0f KiB, WRITE_SIZE %.0f KiB -> scale fetch x%.4f, write x%.4f"
                         % (fraw, wraw, fs, wsc))
        fb, wb = _by_kernel(fetch, "FETCH_SIZE"), _by_kernel(write, "WRITE_SIZE")
        for name in sorted(set(valu) | set(fb) | set(wb)):
            fields = {}
            if name == "prune_scores" and name in valu:
                fields["rows"] = cfg.score_rows
                fields["valu_per_row"] = sum(valu[name]) / len(valu[name]) / cfg.score_rows
                fields["salu_per_row"] = sum(salu[name]) / len(salu[name]) / cfg.score_rows
            if fs and wsc and name in fb and name in wb:
                fields["fetch_bytes"] = sum(fb[name]) / len(fb[name]) * fs * 1024.0
                fields["write_bytes"] = sum(wb[name]) / len(wb[name]) * wsc * 1024.0
                fields["launches"] = len(fb[name])
            if not fields:
                continue
            human = []
            if "valu_per_row" in fields:
                human.append("wave instructions per row: VALU %.1f, SALU %.1f" % (fields["valu_per_row"], fields["salu_per_row"]))
            if "fetch_bytes" in fields:
                human.append("HBM per launch: fetched %.1f MB + written %.1f MB = %.1f MB (mean of %d launches)"
                             % (fields["fetch_bytes"] / 1e6, fields["write_bytes"] / 1e6,
                                (fields["fetch_bytes"] + fields["write_bytes"]) / 1e6, fields["launches"]))
            lines.append("  %-26s %s" % (name, "; ".join(human)))
            data.append("DATA config=%d kernel=%s " % (c, name) + " ".join(
                "%s=%s" % (k, ("%d" % v) if k in ("rows", "launches") else ("%.6g" % v)) for k, v in fields.items()))
        lines.append("")
    return lines, data


def trace_summary(folder, bench_json, plain_json=None):
    """The kernel-trace statistics of one `rocprofv3 --kernel-trace --stats` run of bench.py, next to the run's own
    JSON line (HIP-event timing inside bench.py), for profiles/bench_config3_bert_large.txt:

        rocprofv3 --kernel-trace --stats -d OUT/prof -o bench --output-format csv -- \\
            python3 bench.py --steps 3 --warmup 1 > OUT/prof/bench_stdout.json
        python3 bench.py > OUT/bench_plain.json
        python3 -m paper_2305_18513_amd.profile_counters --trace OUT/prof OUT/prof/bench_stdout.json \\
            OUT/bench_plain.json

    The second JSON line comes from a run without the profiler (whose per-launch overhead shows in the small
    configurations and in the multi-launch operations): the other configurations and the extras are quoted from it.
    """
    import json
    stats = glob.glob(os.path.join(folder, "**", "*kernel_stats.csv"), recursive=True)
    traces = glob.glob(os.path.join(folder, "**", "*kernel_trace.csv"), recursive=True)
    with open(bench_json) as fh:
        bench = json.loads([l for l in fh if l.startswith("{")][-1])
    plain = bench
    if plain_json:
        with open(plain_json) as fh:
            plain = json.loads([l for l in fh if l.startswith("{")][-1])

    def short(n):
        n = re.sub(r"\(anonymous namespace\)::", "", n)
        return re.sub(r"^void ", "", n)[:118]
    print("rocprofv3 kernel trace of bench.py (default workload: %s), one MI355X" % bench["config"]["workload"])
    print("=" * 84)
    print()
    print("Commands (from the repository root, after `cd /tmp && export TMPDIR=/tmp`):")
    print("  rocprofv3 --kernel-trace --stats -d %s -o bench --output-format csv -- \\" % folder)
    print("      python3 bench.py --steps 3 --warmup 1 > %s" % bench_json)
    print("  python3 bench.py > %s" % (plain_json or "(not given)"))
    print("  python3 -m paper_2305_18513_amd.profile_counters --trace %s %s \\" % (folder, bench_json))
    print("      %s" % (plain_json or ""))
    print()
    print("1. Kernel trace statistics, library kernels (all launches of the run: warm-up, survey and timed steps of the")
    print("   default workload, its HIP-graph replays, the extras, the brief runs of the other four configurations)")
    print("%-120s %6s %12s %8s" % ("kernel", "calls", "avg ns", "% time"))
    if stats:
        with open(stats[0]) as fh:
            for r in csv.DictReader(fh):
                if "slimfit" in r["Name"]:
                    print("%-120s %6s %12.0f %8s" % (short(r["Name"]), r["Calls"], float(r["AverageNs"]), r["Percentage"]))
    dom = bench["roofline"]["kernel"]
    if traces and dom in KERNELS:
        # the dominant kernel of the default workload, launch by launch, in program order: its launches during the timed
        # steps are the ones bench.py's events bracket
        with open(traces[0]) as fh:
            tr = [r for r in csv.DictReader(fh) if re.search(KERNELS[dom], r["Kernel_Name"])]
        tr.sort(key=lambda r: int(r["Start_Timestamp"]))
        dur = [(int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3 for r in tr]
        per_step = bench["kernels"][dom]["calls"] // max(bench["steps"], 1)
        first_timed = per_step * (bench["warmup"] + 1)
        timed = dur[first_timed:first_timed + per_step * bench["steps"]]
        if timed:
            print()
            print("   %s during the %d timed steps of the default workload (launches %d .. %d of the trace): mean %.1f us,"
                  % (dom, bench["steps"], first_timed, first_timed + len(timed) - 1, sum(timed) / len(timed)))
            print("   min %.1f, max %.1f; bench.py's events around the same launches: %.1f us"
                  % (min(timed), max(timed), 1e3 * bench["kernels"][dom]["avg_ms"]))
    print()
    print("2. The profiled run's own JSON line")
    print("   step: %.3f ms, %.1f GB/s = %.1f %% of 8 TB/s" % (bench["ms_per_step"], bench["value"], 100 * bench["frac_hbm_peak"]))
    for k, v in bench["kernels"].items():
        print("   %-26s calls %4d  avg %.5f ms  %7.1f GB/s  %5.1f %% of 8 TB/s  bound %-6s  %5.1f %% of its streaming probe  [%s]"
              % (k, v["calls"], v["avg_ms"], v["GBps"], 100 * v["frac_hbm_peak"], v["bound"],
                 100 * v.get("frac_of_stream_probe", float("nan")), v["measured_in"]))
    g = bench.get("extras", {}).get("step_as_hip_graph")
    if g:
        print("   the step replayed as a HIP graph: %.3f ms, %.1f GB/s = %.1f %% of 8 TB/s, replays match eager: %s"
              % (g["ms_per_step"], g["GBps"], 100 * g["frac_hbm_peak"], g["replays_match_eager"]))
    cb = bench.get("cpu_baseline")
    if cb and cb.get("value"):
        print("   cpu oracle: %s GB/s on %d threads (box: %s cores), %s s" % (cb["value"], cb["cores"], cb.get("host_cores"), cb.get("seconds")))
    print()
    print("3. The run without the profiler: %.3f ms per step, %.1f GB/s = %.1f %% of 8 TB/s; %s %.5f ms = %.1f %% of 8 TB/s,"
          % (plain["ms_per_step"], plain["value"], 100 * plain["frac_hbm_peak"], dom, plain["roofline"]["avg_ms"],
             100 * plain["roofline"]["frac"]))
    print("   bound %s, %.1f %% of its streaming probe.  All five configurations (the others brief: 2 warm-ups, 1 survey,"
          % (plain["roofline"]["bound"], 100 * plain["roofline"].get("frac_of_stream_probe", float("nan"))))
    print("   5 timed steps each):")
    for c, v in sorted(plain.get("configs", {}).items()):
        if "kernels" not in v:
            continue
        print("   %s: %.3f ms per step, %.1f GB/s = %.1f %% of 8 TB/s" % (v["workload"], v["ms_per_step"], v["GBps"], 100 * v["frac_hbm_peak"]))
        for k, e in v["kernels"].items():
            print("      %-26s avg %.5f ms  %7.1f GB/s  %5.1f %%  bound %s" % (k, e["avg_ms"], e["GBps"], 100 * e["frac_hbm_peak"], e["bound"]))
    print()
    print("4. Extras of the run without the profiler (outside the timed step; HIP events, median of 12; bytes moved are")
    print("   those of profiles/kernel_counters.txt)")
    for k, v in plain.get("extras", {}).items():
        if isinstance(v, dict) and "median_ms" in v:
            line = "   %-44s %.5f ms  %7.1f GB/s  %5.1f %% of 8 TB/s" % (k, v["median_ms"], v["GBps"], 100 * v["frac_hbm_peak"])
            if "frac_of_stream_probe" in v:
                line += "  %5.1f %% of its streaming probe" % (100 * v["frac_of_stream_probe"])
            if "frac_hbm_peak_on_traffic" in v:
                line += "  moved %.2fx the algorithmic bytes: %5.1f %% of 8 TB/s on that basis" % (
                    v["traffic_over_algorithmic"], 100 * v["frac_hbm_peak_on_traffic"])
            print(line)
    return 0


def main(argv):
    if len(argv) in (4, 5) and argv[1] == "--trace":
        return trace_summary(argv[2], argv[3], argv[4] if len(argv) == 5 else None)
    if len(argv) != 2:
        sys.stderr.write(__doc__)
        return 2
    lines, data = summarise(argv[1])
    xlines, xdata = summarise_extras(argv[1])
    print("rocprofv3 counters of the hot-path kernels as bench.py launches them, one MI355X")
    print("=" * 84)
    print()
    out = argv[1].rstrip("/")
    print("Written by `python3 -m paper_2305_18513_amd.profile_counters %s` from three counter runs per" % out)
    print("configuration C (from the repository root, after `cd /tmp && export TMPDIR=/tmp`):")
    print("  rocprofv3 --pmc SQ_INSTS_VALU SQ_INSTS_SALU -d %s/cfgC_insts -o r --output-format csv -- \\" % out)
    print("      python3 bench.py --config C --steps 1 --warmup 0 --no-cpu-baseline --no-extras --no-other-configs")
    print("  rocprofv3 --pmc FETCH_SIZE -d %s/cfgC_fetch -o r --output-format csv -- \\" % out)
    print("      python3 bench.py --config C --steps 1 --warmup 0 --no-cpu-baseline --no-extras --no-other-configs --calibrate-copy")
    print("  rocprofv3 --pmc WRITE_SIZE -d %s/cfgC_write -o r --output-format csv -- \\" % out)
    print("      python3 bench.py --config C --steps 1 --warmup 0 --no-cpu-baseline --no-extras --no-other-configs --calibrate-copy")
    print("and, for the operations outside the timed step, from two runs of the default configuration with its extras:")
    print("  rocprofv3 --pmc FETCH_SIZE -d %s/extras_fetch -o r --output-format csv -- \\" % out)
    print("      python3 bench.py --steps 1 --warmup 0 --no-cpu-baseline --no-other-configs --calibrate-copy")
    print("  rocprofv3 --pmc WRITE_SIZE -d %s/extras_write -o r --output-format csv -- \\" % out)
    print("      python3 bench.py --steps 1 --warmup 0 --no-cpu-baseline --no-other-configs --calibrate-copy")
    print("Counter values are means over the kernel's launches in the run (first, cold launches included), summed over")
    print("the chip as rocprofv3 reports them; byte counters are scaled by the same counter's reading of a 1 GiB copy.")
    print("bench.py reads the DATA lines (roofline.traffic, the issue side of the bound rule).")
    print()
    print("\n".join(lines + xlines))
    print("\n".join(data + xdata))
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
