"""The counter summariser on a hand-made rocprofv3 folder: per-row instruction counts, byte counters scaled by the
copy calibration, and the DATA lines bench.py reads."""
import csv
import os

from paper_2305_18513_amd import profile_counters as pc
from paper_2305_18513_amd import synth


def _write(folder, rows):
    os.makedirs(folder, exist_ok=True)
    with open(os.path.join(folder, "r_counter_collection.csv"), "w", newline="") as fh:
        w = csv.DictWriter(fh, fieldnames=["Kernel_Name", "Grid_Size", "Counter_Name", "Counter_Value"])
        w.writeheader()
        for r in rows:
            w.writerow(dict(zip(w.fieldnames, r)))


def test_summary_of_a_hand_made_run(tmp_path):
    cfg = synth.CONFIGS[3]
    rows = cfg.score_rows
    prune = "void slimfit::(anonymous namespace)::prune_rows_kernel<float, 6, true, true, false>(float const*)"
    quant = "void slimfit::(anonymous namespace)::quant_pack_kernel<float, 4, true, 16, false>(float const*)"
    copy = "__amd_rocclr_copyBuffer"
    root = str(tmp_path)
    _write(os.path.join(root, "cfg3_insts"),
           [(prune, 1024, "SQ_INSTS_VALU", 100.0 * rows), (prune, 1024, "SQ_INSTS_VALU", 120.0 * rows),
            (prune, 1024, "SQ_INSTS_SALU", 130.0 * rows), (prune, 1024, "SQ_INSTS_SALU", 130.0 * rows)])
    # the copy reads half of its bytes on the fetch counter: everything is scaled by 2
    _write(os.path.join(root, "cfg3_fetch"),
           [(copy, 1, "FETCH_SIZE", 524288.0), (prune, 1024, "FETCH_SIZE", 1000.0), (prune, 1024, "FETCH_SIZE", 3000.0),
            (quant, 4096, "FETCH_SIZE", 800.0), (quant, 1024, "FETCH_SIZE", 200.0)])
    _write(os.path.join(root, "cfg3_write"),
           [(copy, 1, "WRITE_SIZE", 1048576.0), (prune, 1024, "WRITE_SIZE", 500.0), (prune, 1024, "WRITE_SIZE", 500.0),
            (quant, 4096, "WRITE_SIZE", 100.0), (quant, 1024, "WRITE_SIZE", 25.0)])
    lines, data = pc.summarise(root)
    table = {}
    for d in data:
        kv = dict(tok.split("=", 1) for tok in d.split()[1:])
        table[(int(kv["config"]), kv["kernel"])] = kv
    p = table[(3, "prune_scores")]
    assert int(p["rows"]) == rows and int(p["launches"]) == 2
    assert abs(float(p["valu_per_row"]) - 110.0) < 1e-3 and abs(float(p["salu_per_row"]) - 130.0) < 1e-3
    assert abs(float(p["fetch_bytes"]) - 2000.0 * 2.0 * 1024) < 1.0          # mean of the launches x the copy's factor
    assert abs(float(p["write_bytes"]) - 500.0 * 1024) < 1.0
    # quantiser launches are told apart by their size: the larger grid is the GELU input
    assert abs(float(table[(3, "quant_pack[gelu_in]")]["fetch_bytes"]) - 800.0 * 2.0 * 1024) < 1.0
    assert abs(float(table[(3, "quant_pack[ln_in]")]["fetch_bytes"]) - 200.0 * 2.0 * 1024) < 1.0
    assert any("config 3" in line for line in lines)


def test_bench_reads_the_tracked_summary():
    """Every DATA line of the tracked file parses, and the default configuration's dominant kernel is there."""
    import importlib.util
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    table = bench.load_counters(os.path.join(root, "profiles", "kernel_counters.txt"))
    cnt = table[(3, "prune_scores")]
    assert cnt["rows"] == synth.CONFIGS[3].score_rows and cnt["fetch_bytes"] > 0 and cnt["valu_per_row"] > 0
    bound, t_issue = bench.classify_bound(0.247, 1387266048, cnt)
    assert bound in ("issue", "hbm") and t_issue is not None
    assert bench.classify_bound(0.01, 1 << 20, {})[0] == "launch"
