#!/usr/bin/env python3
"""Benchmark of the SlimFit hot path on one MI355X.

One "step" is one pass of the whole per-iteration path of a fine-tune step over
one batch of synthetic input of the chosen workload configuration:

  forward,  per encoder block : quant_pack(GELU input), quant_pack(LayerNorm
                                input) x2, prune_scores(attention probabilities)
  backward, per encoder block : dequant_unpack of the three cached tensors
  after the optimizer step    : layer_delta over every weight tensor, copy of
                                the L scores to the host, ils_update +
                                ils_select on the host

The metric is algorithmic bytes of the step / wall time of the step, inputs
resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3]
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2305_18513_amd import binding as sf  # noqa: E402
from paper_2305_18513_amd import synth  # noqa: E402

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published

# Chip constants for the issue-side estimate of a kernel's time: 256 compute units x 4 SIMDs, a wave64 vector or
# scalar instruction occupying its SIMD's issue slot for 4 cycles at 2.4 GHz.
SIMDS = 1024
CLOCK_HZ = 2.4e9
ISSUE_CYCLES = 4

# rocprofv3 counter figures per (config, kernel): HBM bytes per launch (FETCH_SIZE / WRITE_SIZE, scaled by the same
# counters' reading of a device copy of known size) and wave-level instructions issued per row.  Read from the
# tracked summary that `python -m paper_2305_18513_amd.profile_counters` writes from the profiling runs, so that this
# record and the summary cannot disagree; absent file or entry: null.
COUNTERS_FILE = os.path.join(ROOT, "profiles", "kernel_counters.txt")


def load_counters(path=COUNTERS_FILE):
    """{(config, kernel): {field: value}} from the DATA lines of the tracked counter summary."""
    table = {}
    try:
        with open(path) as fh:
            for line in fh:
                if not line.startswith("DATA "):
                    continue
                kv = dict(tok.split("=", 1) for tok in line.split()[1:])
                key = (int(kv.pop("config")), kv.pop("kernel"))
                table[key] = {k: float(v) for k, v in kv.items()}
    except OSError:
        pass
    return table


def classify_bound(avg_ms, nbytes, counters):
    """Which limit a kernel ran against, by a fixed rule:
      launch : its algorithmic bytes would take under 4 us at 8 TB/s (less than 32 MB a launch): start-up, ramp and
               drain of a launch (5 - 10 us) outweigh the streaming;
      issue  : the instructions the counters show (the larger of vector and scalar wave instructions per row x rows,
               4 cycles each, over 1024 SIMDs at 2.4 GHz) account for at least half of the measured time;
      hbm    : otherwise."""
    t = avg_ms * 1e-3
    if nbytes / (HBM_PEAK_GBS * 1e9) < 4e-6:
        return "launch", None
    t_issue = None
    if counters and counters.get("rows") and (counters.get("valu_per_row") or counters.get("salu_per_row")):
        per_row = max(counters.get("valu_per_row", 0.0), counters.get("salu_per_row", 0.0))
        t_issue = per_row * counters["rows"] * ISSUE_CYCLES / (SIMDS * CLOCK_HZ)
        if t_issue >= 0.5 * t:
            return "issue", t_issue
    return "hbm", t_issue


def esize(dt: torch.dtype) -> int:
    return 2 if dt == torch.bfloat16 else 4


class BlockSet:
    """Device tensors of one encoder block: inputs and caller-owned outputs."""

    def __init__(self, cfg: synth.WorkloadConfig, block: int, bits: int):
        dev = "cuda"
        self.gelu = synth.activation(cfg, "gelu_in", dev, block).reshape(-1)
        self.ln = [synth.activation(cfg, "ln_in", dev, block * 2 + i).reshape(-1) for i in range(2)]
        self.scores = synth.attention_scores(cfg, dev, block)
        self.acts = [self.gelu] + self.ln
        self.codes = [torch.empty(sf.packed_bytes(a.numel(), bits), dtype=torch.uint8, device=dev)
                      for a in self.acts]
        self.scales = [torch.empty(sf.num_blocks(a.numel(), cfg.quant_block), dtype=torch.float32, device=dev)
                       for a in self.acts]
        self.deq = [torch.empty_like(a) for a in self.acts]
        rows, k = cfg.score_rows, cfg.keep_k
        self.vals = torch.empty(rows, k, dtype=self.scores.dtype, device=dev)
        self.idx = torch.empty(rows, k, dtype=torch.uint16, device=dev)
        self.counts = torch.empty(rows, dtype=torch.int32, device=dev)


class Timers:
    """Per-kernel device time from events on the stream the kernels run on."""

    def __init__(self):
        self.pending = []
        self.total_ms = {}
        self.calls = {}
        self.bytes = {}

    def launch(self, name, nbytes, fn):
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        # a first marker soaks up the wait for the kernel ahead, so that [a, b] holds this kernel alone
        torch.cuda.Event().record()
        a.record()
        fn()
        b.record()
        self.pending.append((name, nbytes, a, b))

    def collect(self):
        for name, nbytes, a, b in self.pending:
            self.total_ms[name] = self.total_ms.get(name, 0.0) + a.elapsed_time(b)
            self.calls[name] = self.calls.get(name, 0) + 1
            self.bytes[name] = nbytes
        self.pending = []


def quant_bytes(n, in_sz, bits, block):
    return n * in_sz + (n * bits + 7) // 8 + ((n + block - 1) // block) * 4


def prune_bytes(rows, cols, k, in_sz):
    return rows * cols * in_sz + rows * k * (in_sz + 2)


NAMES_Q = ["quant_pack[gelu_in]", "quant_pack[ln_in]", "quant_pack[ln_in]"]
NAMES_D = ["dequant_unpack[gelu_in]", "dequant_unpack[ln_in]", "dequant_unpack[ln_in]"]


class Workload:
    """One configuration resident in HBM: n_sets encoder-block buffer sets, every weight tensor, the plan."""

    def __init__(self, cfg: synth.WorkloadConfig, n_sets: int):
        self.cfg = cfg
        self.bits = cfg.quant_bits[-1]
        self.block = cfg.quant_block
        self.mode = sf.PRUNE_THRESHOLD if cfg.threshold_variant else sf.PRUNE_TOPK
        self.tau = cfg.threshold_tau if cfg.threshold_variant else 0.0
        self.in_sz = esize(cfg.act_dtype)
        self.n_sets = max(1, min(n_sets, cfg.n_blocks))
        self.sets = [BlockSet(cfg, b, self.bits) for b in range(self.n_sets)]
        self.prev, self.cur = synth.weight_units(cfg, "cuda")
        self.numel = [t.numel() for t in self.prev]
        self.L = len(self.numel)
        self.ws = torch.empty(sf.layer_delta_workspace(self.numel), dtype=torch.uint8, device="cuda")
        self.d_dev = torch.empty(self.L, dtype=torch.float32, device="cuda")
        self.d_host_pinned = torch.empty(self.L, dtype=torch.float32, pin_memory=True)
        self.d_vec = synth.initial_distance(cfg).numpy().copy()
        self.n_freeze = sf.freeze_count(self.L, cfg.freeze_rate)
        _, self.mask = sf.ils_select(self.d_vec, self.n_freeze)
        self.pdt = sf.BF16 if cfg.w_dtype == torch.bfloat16 else sf.F32
        sf.layer_delta_plan(self.prev, self.cur, self.ws)           # pointers are stable across steps: planned once
        torch.cuda.synchronize()
        self.w_bytes = sum(self.numel) * (esize(cfg.w_dtype) + 4) + 4 * self.L
        self.b_quant = [quant_bytes(a.numel(), self.in_sz, self.bits, self.block) for a in self.sets[0].acts]
        self.b_prune = prune_bytes(cfg.score_rows, cfg.score_cols, cfg.keep_k, self.in_sz)
        self.step_bytes = cfg.n_blocks * (2 * sum(self.b_quant) + self.b_prune) + self.w_bytes
        # what each kernel reads and writes per launch (for the streaming yardstick of its traffic mix)
        self.read_write = {"prune_scores": (cfg.score_rows * cfg.score_cols * self.in_sz,
                                            self.b_prune - cfg.score_rows * cfg.score_cols * self.in_sz),
                           "layer_delta": (self.w_bytes - 4 * self.L, 4 * self.L)}
        for nq, nd, a, nb in zip(NAMES_Q, NAMES_D, self.sets[0].acts, self.b_quant):
            self.read_write[nq] = (a.numel() * self.in_sz, nb - a.numel() * self.in_sz)
            self.read_write[nd] = (nb - a.numel() * self.in_sz, a.numel() * self.in_sz)
        self.rows_of = {"prune_scores": cfg.score_rows}

    def describe(self):
        cfg = self.cfg
        return "config %d: %s-shaped (%d blocks, hidden %d, %d heads, tokens %d, batch %d)" % (
            cfg.index, cfg.name, cfg.n_blocks, cfg.hidden, cfg.heads, cfg.tokens, cfg.batch)

    def step(self, run):
        """One pass of the hot path; run(name, bytes, fn) launches fn (with or without events around it)."""
        cfg, bits, block = self.cfg, self.bits, self.block
        for b in range(cfg.n_blocks):                     # forward
            s = self.sets[b % self.n_sets]
            for i, a in enumerate(s.acts):
                run(NAMES_Q[i], self.b_quant[i],
                    lambda a=a, i=i, s=s: sf.quant_pack(a, sf.Q_BLOCK, bits, block, 0, s.codes[i], s.scales[i]))
            run("prune_scores", self.b_prune,
                lambda s=s: sf.prune_scores(s.scores, cfg.keep_k, self.mode, self.tau, s.vals, s.idx, s.counts))
        for b in reversed(range(cfg.n_blocks)):           # backward
            s = self.sets[b % self.n_sets]
            for i in reversed(range(3)):
                run(NAMES_D[i], self.b_quant[i],
                    lambda i=i, s=s: sf.dequant_unpack(s.codes[i], s.scales[i], sf.Q_BLOCK, bits, block, 0, s.deq[i]))
        run("layer_delta", self.w_bytes,
            lambda: sf.layer_delta_run(self.numel, self.pdt, sf.F32, cfg.delta_given, 0.0, self.d_dev, self.ws))
        self.d_host_pinned.copy_(self.d_dev, non_blocking=True)
        torch.cuda.current_stream().synchronize()         # the host needs the L scores
        sf.ils_update(self.d_vec, self.d_host_pinned.numpy(), self.mask)
        _, self.mask = sf.ils_select(self.d_vec, self.n_freeze)

    def measure(self, steps, warmup):
        """warm-up steps, one untimed survey step with events around every launch, then `steps` timed steps with
        events around the dominant kernel only.  Returns (wall seconds, survey, timers, dominant kernel)."""
        timers, survey = Timers(), Timers()
        plain = lambda name, nbytes, fn: fn()
        for _ in range(warmup):
            self.step(plain)
        # An event pair costs about 3 us of stream time; around each of the step's launches that is several per
        # cent of the step.  So one untimed step surveys every kernel and names the dominant one, and the timed
        # region carries events around that kernel's launches only.
        self.step(survey.launch)
        torch.cuda.synchronize()
        survey.collect()
        dom = max(survey.total_ms, key=lambda n: survey.total_ms[n])
        only_dom = lambda name, nbytes, fn: timers.launch(name, nbytes, fn) if name == dom else fn()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step(only_dom)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        timers.collect()
        return wall, survey, timers, dom


def kernel_entry(t, name, per_step):
    calls = t.calls[name]
    avg_ms = t.total_ms[name] / calls
    gbs = t.bytes[name] / (avg_ms * 1e-3) / 1e9
    return {"calls": calls, "avg_ms": round(avg_ms, 5), "bytes_per_launch": t.bytes[name],
            "GBps": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
            "total_ms_per_step": round(t.total_ms[name] / per_step, 4)}


def stream_yardstick(read_bytes, write_bytes, cache={}):
    """What a kernel that only streams reaches with this read : write mix and size: the library's diagnostic probe,
    timed the same way (median of 12 launches between events).  The mix is rounded to the probe's nearest shape:
    16 / r bytes written per 16 read (r = 1 .. 16), read-only, or 2 / 4 / 8 vectors written per vector read."""
    if read_bytes <= 0:
        return None
    if write_bytes * 64 < read_bytes:
        ratio = 0
    elif read_bytes >= write_bytes:
        ratio = min((1, 2, 4, 8, 16), key=lambda r: abs(math.log2(r) - math.log2(read_bytes / write_bytes)))
    else:
        ratio = -min((1, 2, 4, 8), key=lambda m: abs(math.log2(m) - math.log2(write_bytes / read_bytes)))
        ratio = 1 if ratio == -1 else ratio
    in_vecs = max(1024, read_bytes // 16 // 1024 * 1024)
    key = (ratio, in_vecs)
    if key not in cache:
        out_bytes = sf.stream_probe_bytes(in_vecs, ratio)
        psrc = torch.empty(in_vecs * 4, dtype=torch.float32, device="cuda").normal_()
        pdst = torch.empty(max(out_bytes, 16), dtype=torch.uint8, device="cuda")
        for _ in range(3):
            sf.stream_probe(psrc, pdst, ratio)
        torch.cuda.synchronize()
        pev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(12)]
        for a, b in pev:
            a.record()
            sf.stream_probe(psrc, pdst, ratio)
            b.record()
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in pev)[len(pev) // 2]
        nbytes = in_vecs * 16 + out_bytes
        cache[key] = {"shape": ratio, "bytes": nbytes, "ms": round(ms, 5), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1)}
        del psrc, pdst
    return dict(cache[key], kernel_read_write_ratio=round(read_bytes / max(write_bytes, 1), 2))


def extra_record(name, ms, nbytes, write_bytes, counters, **more):
    """Record of an operation timed outside the step: its algorithmic bytes against the HBM peak, against the
    streaming probe of the same read : write mix and size, and (when the tracked counter summary has the operation)
    against the HBM bytes its kernels really moved."""
    rec = {"median_ms": round(ms, 5), "bytes_per_launch": nbytes}
    rec.update(more)
    gbps = nbytes / (ms * 1e-3) / 1e9
    rec["GBps"] = round(gbps, 1)
    rec["frac_hbm_peak"] = round(gbps / HBM_PEAK_GBS, 4)
    probe = stream_yardstick(nbytes - write_bytes, write_bytes)
    if probe:
        rec["stream_probe"] = probe
        rec["frac_of_stream_probe"] = round(gbps / probe["GBps"], 4)
    cnt = counters.get((-1, name.replace(" ", "_")))
    if cnt and "fetch_bytes" in cnt:
        moved = cnt["fetch_bytes"] + cnt["write_bytes"]
        rec["traffic"] = int(moved)
        rec["traffic_over_algorithmic"] = round(moved / nbytes, 3)
        rec["frac_hbm_peak_on_traffic"] = round(moved / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    return rec


def kernel_table(wl, survey, timers, dom, steps, counters, with_probe):
    """Per-kernel record of one configuration: every kernel from the survey step, the dominant one from the timed
    region; each with the bound the rule assigns and (with_probe) its streaming yardstick."""
    kernels = {name: dict(kernel_entry(survey, name, 1), measured_in="survey step (untimed)") for name in survey.total_ms}
    kernels[dom] = dict(kernel_entry(timers, dom, steps), measured_in="timed region", survey_avg_ms=kernels[dom]["avg_ms"])
    for name, k in kernels.items():
        cnt = dict(counters.get((wl.cfg.index, name), {}))
        if name in wl.rows_of:
            cnt.setdefault("rows", wl.rows_of[name])
        bound, t_issue = classify_bound(k["avg_ms"], k["bytes_per_launch"], cnt)
        k["bound"] = bound
        if t_issue is not None:
            k["issue_ms_estimate"] = round(t_issue * 1e3, 5)
        if with_probe:
            try:
                rd, wr = wl.read_write[name]
                probe = stream_yardstick(rd, wr)
                if probe:
                    k["stream_probe"] = probe
                    k["frac_of_stream_probe"] = round(k["GBps"] / probe["GBps"], 4)
            except Exception as exc:          # the yardstick is context: it never costs the result its line
                k["stream_probe"] = {"error": repr(exc)}
    return kernels


def sets_for(cfg, requested):
    """Buffer sets to rotate over: at least `requested`, and enough that one pass over them exceeds 1 GB of inputs
    (four times the 256 MB memory-side cache), never more than the configuration has encoder blocks."""
    per_set = (cfg.gelu_in_numel + 2 * cfg.ln_in_numel + cfg.score_rows * cfg.score_cols) * esize(cfg.act_dtype)
    return max(1, min(cfg.n_blocks, max(requested, -(-(1 << 30) // per_set))))


def brief_config(ci, counters):
    """Another configuration, briefly: two warm-up steps, the survey step, five timed steps."""
    cfg = synth.CONFIGS[ci]
    wl = Workload(cfg, sets_for(cfg, 3))
    wall, survey, timers, dom = wl.measure(5, 2)
    kernels = kernel_table(wl, survey, timers, dom, 5, counters, with_probe=False)
    ms = wall * 1e3 / 5
    out = {"workload": wl.describe(), "dtype": "f32" if cfg.act_dtype == torch.float32 else "bf16",
           "quant": "%d-bit block-%d" % (wl.bits, wl.block), "keep_k": cfg.keep_k,
           "prune_mode": "threshold" if cfg.threshold_variant else "topk", "buffer_sets": wl.n_sets,
           "step_bytes": wl.step_bytes, "ms_per_step": round(ms, 4),
           "GBps": round(wl.step_bytes / (ms * 1e-3) / 1e9, 1),
           "frac_hbm_peak": round(wl.step_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
           "dominant_kernel": dom,
           "kernels": {n: {f: k[f] for f in ("calls", "avg_ms", "bytes_per_launch", "GBps", "frac_hbm_peak", "bound",
                                             "measured_in") if f in k} for n, k in kernels.items()}}
    del wl
    torch.cuda.empty_cache()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=3, help="workload index 0..4 (3 = BERT-large-shaped)")
    ap.add_argument("--sets", type=int, default=3, help="distinct encoder-block buffer sets to rotate over (at least)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip kernels outside the timed step (restore_scores, 8-bit scores, whole-tensor pruning)")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the brief runs of the other four configurations")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three 1 GiB device copies (for scaling rocprofv3 byte counters)")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    if not sf.is_built():
        from paper_2305_18513_amd import build
        build.build_library()
    sf.lib()
    torch.cuda.set_device(0)
    counters = load_counters()

    cfg = synth.CONFIGS[args.config]
    wl = Workload(cfg, sets_for(cfg, args.sets))
    # the names the kernels outside the timed step (extras) use
    bits, block, mode, tau, in_sz = wl.bits, wl.block, wl.mode, wl.tau, wl.in_sz
    sets, n_sets, prev, cur, numel, L = wl.sets, wl.n_sets, wl.prev, wl.cur, wl.numel, wl.L
    ws, d_dev, d_host_pinned, d_vec, n_freeze, pdt = wl.ws, wl.d_dev, wl.d_host_pinned, wl.d_vec, wl.n_freeze, wl.pdt
    b_prune, step_bytes = wl.b_prune, wl.step_bytes

    wall, survey, timers, dom = wl.measure(args.steps, args.warmup)
    mask = wl.mask

    extras = {}
    if not args.no_extras:
        try:
            # the same step with its 169 launches captured in one HIP graph (the library allocates nothing and
            # never synchronises, so the calls capture as they are); replays are checked against the eager results
            eager_d = d_dev.clone()
            eager_codes = sets[0].codes[0].clone()
            eager_vals = sets[0].vals.clone()

            def kernels_only():
                for b in range(cfg.n_blocks):
                    s = sets[b % n_sets]
                    for i, a in enumerate(s.acts):
                        sf.quant_pack(a, sf.Q_BLOCK, bits, block, 0, s.codes[i], s.scales[i])
                    sf.prune_scores(s.scores, cfg.keep_k, mode, tau, s.vals, s.idx, s.counts)
                for b in reversed(range(cfg.n_blocks)):
                    s = sets[b % n_sets]
                    for i in reversed(range(3)):
                        sf.dequant_unpack(s.codes[i], s.scales[i], sf.Q_BLOCK, bits, block, 0, s.deq[i])
                sf.layer_delta_run(numel, pdt, sf.F32, cfg.delta_given, 0.0, d_dev, ws)

            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                kernels_only()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):        # (the library skips its pointer look-ups on a capturing stream)
                kernels_only()

            def graph_step():
                nonlocal mask
                graph.replay()
                d_host_pinned.copy_(d_dev, non_blocking=True)
                torch.cuda.current_stream().synchronize()
                sf.ils_update(d_vec, d_host_pinned.numpy(), mask)
                _, mask = sf.ils_select(d_vec, n_freeze)

            same = True
            for _ in range(max(args.warmup, 2)):
                d_dev.zero_()
                sets[0].codes[0].zero_()
                sets[0].vals.zero_()
                torch.cuda.synchronize()
                graph_step()
                same = same and torch.equal(d_dev, eager_d) and torch.equal(sets[0].codes[0], eager_codes) \
                    and torch.equal(sets[0].vals.view(torch.uint8), eager_vals.view(torch.uint8))
            torch.cuda.synchronize()
            tg = time.perf_counter()
            for _ in range(args.steps):
                graph_step()
            torch.cuda.synchronize()
            g_ms = (time.perf_counter() - tg) * 1e3 / args.steps
            extras["step_as_hip_graph"] = {"ms_per_step": round(g_ms, 4), "GBps": round(step_bytes / (g_ms * 1e-3) / 1e9, 1),
                                           "frac_hbm_peak": round(step_bytes / (g_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                           "replays_match_eager": bool(same)}
            del graph, eager_codes, eager_vals
        except Exception as exc:       # an extra must not cost the step its result line
            extras.setdefault("errors", []).append(repr(exc))

    # next rows of the scope table, outside the timed step: the backward half of pruning
    if not args.no_extras:
        try:
            dense = [torch.empty_like(s.scores) for s in sets]
            for i in range(len(sets)):
                sf.restore_scores(sets[i].vals, sets[i].idx, sets[i].counts, dense[i])
            torch.cuda.synchronize()
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(12)]
            for i, (a, b) in enumerate(ev):
                s = sets[i % n_sets]
                a.record()
                sf.restore_scores(s.vals, s.idx, s.counts, dense[i % n_sets])
                b.record()
            torch.cuda.synchronize()
            ms = sorted(a.elapsed_time(b) for a, b in ev)[len(ev) // 2]
            nb = b_prune + 4 * cfg.score_rows
            extras["restore_scores"] = extra_record("restore_scores", ms, nb, cfg.score_rows * cfg.score_cols * in_sz, counters)
            del dense
            # the paper's own placement for the same tensor: 8-bit fixed point, 4 integer + 4 fractional bits
            sc = [s.scores.reshape(-1) for s in sets]
            n_sc = sc[0].numel()
            c8 = [torch.empty(n_sc, dtype=torch.uint8, device="cuda") for _ in sets]
            for i in range(len(sets)):
                sf.quant_pack(sc[i], sf.Q_FIXED, 8, 64, 4, c8[i], None)
            torch.cuda.synchronize()
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(12)]
            for i, (a, b) in enumerate(ev):
                a.record()
                sf.quant_pack(sc[i % n_sets], sf.Q_FIXED, 8, 64, 4, c8[i % n_sets], None)
                b.record()
            torch.cuda.synchronize()
            ms = sorted(a.elapsed_time(b) for a, b in ev)[len(ev) // 2]
            nb = n_sc * (in_sz + 1)
            extras["quant_pack[scores, fixed 4.4]"] = extra_record("quant_pack[scores, fixed 4.4]", ms, nb, n_sc, counters)
            del c8, sc
            # Alg. 5 as printed: the flattened LayerNorm input, int(numel * 0.1) survivors by magnitude, and its restore
            lns = [s.ln[0] for s in sets]
            n_ln = lns[0].numel()
            k_ln = sf.keep_count(n_ln, 100000)
            gv = [torch.empty(k_ln, dtype=lns[0].dtype, device="cuda") for _ in sets]
            gi = [torch.empty(k_ln, dtype=torch.int32, device="cuda") for _ in sets]
            gp = [torch.empty(sf.global_tile_ptr_len(n_ln), dtype=torch.int32, device="cuda") for _ in sets]
            gws = torch.empty(sf.prune_global_workspace(n_ln), dtype=torch.uint8, device="cuda")
            gout = [torch.empty_like(x) for x in lns]
            nb = n_ln * in_sz + k_ln * (in_sz + 4)
            runs = {
                "prune_global[ln_in, 10%]": (k_ln * (in_sz + 4), lambda i: sf.prune_global(lns[i], k_ln, gv[i], gi[i], True, gp[i], gws)),
                "restore_global[ln_in, tile pointers]": (n_ln * in_sz, lambda i: sf.restore_global(gv[i], gi[i], k_ln, gout[i], gp[i])),
                "restore_global[ln_in, zeros+scatter]": (n_ln * in_sz, lambda i: sf.restore_global(gv[i], gi[i], k_ln, gout[i])),
            }
            for name, (wb, fn) in runs.items():
                for i in range(len(sets)):
                    fn(i)
                torch.cuda.synchronize()
                ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(12)]
                for i, (a, b) in enumerate(ev):
                    a.record()
                    fn(i % n_sets)
                    b.record()
                torch.cuda.synchronize()
                ms = sorted(a.elapsed_time(b) for a, b in ev)[len(ev) // 2]
                extras[name] = extra_record(name, ms, nb, wb, counters, numel=n_ln, k=k_ln)
            del gv, gi, gp, gws, gout
            # the caches fused into their producer / consumer (x read once; the dequantised values never stored;
            # softmax and pruning in one pass over the logits)
            n_g = sets[0].gelu.numel()
            nb_g = 2 * n_g * in_sz + sf.packed_bytes(n_g, bits) + 4 * sf.num_blocks(n_g, block)
            rows_s, cols_s = sets[0].scores.shape
            nb_s = 2 * rows_s * cols_s * in_sz + rows_s * cfg.keep_k * (in_sz + 2)
            probs = [torch.empty_like(s.scores) for s in sets]
            fused = {
                "gelu_quant_pack[gelu_in]": (nb_g, nb_g - n_g * in_sz, lambda i: sf.gelu_quant_pack(
                    sets[i].gelu, sf.Q_BLOCK, bits, block, 0, sets[i].deq[0], sets[i].codes[0], sets[i].scales[0])),
                "gelu_backward_dequant[gelu_in]": (nb_g, n_g * in_sz, lambda i: sf.gelu_backward_dequant(
                    sets[i].codes[0], sets[i].scales[0], sf.Q_BLOCK, bits, block, 0, sets[i].gelu, sets[i].deq[0])),
                "softmax_prune[scores as logits]": (nb_s, nb_s - rows_s * cols_s * in_sz, lambda i: sf.softmax_prune(
                    sets[i].scores, cfg.keep_k, probs[i], sets[i].vals, sets[i].idx)),
                # consumes the pairs the line above left; the score tensor stands in for the incoming gradient
                # (only its kept columns are read: k elements per row are the algorithmic bytes, although at
                # 10 % kept nearly every 128-byte line of it is touched)
                "softmax_backward_pruned[scores]": (
                    rows_s * cols_s * in_sz + rows_s * cfg.keep_k * (2 * in_sz + 2), rows_s * cols_s * in_sz,
                    lambda i: sf.softmax_backward_pruned(sets[i].vals, sets[i].idx, None, sets[i].scores, probs[i])),
            }
            for name, (nb, wb, fn) in fused.items():
                for i in range(len(sets)):
                    fn(i)
                torch.cuda.synchronize()
                ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(12)]
                for i, (a, b) in enumerate(ev):
                    a.record()
                    fn(i % n_sets)
                    b.record()
                torch.cuda.synchronize()
                ms = sorted(a.elapsed_time(b) for a, b in ev)[len(ev) // 2]
                extras[name] = extra_record(name, ms, nb, wb, counters)
            del probs
            # LayerNorm around its caches: forward with row statistics; the pruned cache (10 % of the standardised input
            # kept without storing it, input gradient of the frozen layer from the kept pairs); the quantised cache fused
            # into the forward and backward kernels
            H = cfg.hidden
            lnx = [s.ln[0].view(-1, H) for s in sets]
            rows_l = lnx[0].shape[0]
            n_l = rows_l * H
            k_l = sf.keep_count(n_l, 100000)
            gam = torch.rand(H, device="cuda") + 0.5
            bet = torch.rand(H, device="cuda") - 0.5
            lny = [torch.empty_like(x) for x in lnx]
            mu = [torch.empty(rows_l, device="cuda") for _ in sets]
            rs = [torch.empty(rows_l, device="cuda") for _ in sets]
            pv = [torch.empty(k_l, device="cuda") for _ in sets]
            pi = [torch.empty(k_l, dtype=torch.int32, device="cuda") for _ in sets]
            rp = [torch.empty(rows_l + 1, dtype=torch.int32, device="cuda") for _ in sets]
            lws = torch.empty(sf.prune_global_workspace(n_l), dtype=torch.uint8, device="cuda")
            nb_lq = 2 * in_sz * n_l + sf.packed_bytes(n_l, bits) + 4 * sf.num_blocks(n_l, block) + 8 * rows_l
            ln_runs = {
                "layernorm_forward[ln_in]": (2 * in_sz * n_l + 8 * rows_l, in_sz * n_l + 8 * rows_l, lambda i: sf.layernorm_forward(
                    lnx[i], gam, bet, 1e-5, lny[i], mu[i], rs[i])),
                "prune_global_standardized[ln_in, 10%]": (in_sz * n_l + 8 * k_l + 12 * rows_l, 8 * k_l + 4 * rows_l, lambda i:
                    sf.prune_global_standardized(lnx[i], mu[i], rs[i], k_l, pv[i], pi[i], True, None, rp[i], lws)),
                "layernorm_backward_pruned[ln_in]": (2 * in_sz * n_l + 8 * k_l + 8 * rows_l, in_sz * n_l, lambda i:
                    sf.layernorm_backward_pruned(pv[i], pi[i], rp[i], k_l, rs[i], gam, lnx[i], lny[i])),
                # the step's own cache (block-scaled codes of the LayerNorm input) written by the LayerNorm that
                # reads the input anyway, and the input gradient straight from that cache
                "layernorm_forward_quant_pack[ln_in]": (nb_lq, nb_lq - in_sz * n_l, lambda i: sf.layernorm_forward_quant_pack(
                    lnx[i], gam, bet, 1e-5, bits, block, lny[i], mu[i], rs[i], sets[i].codes[1], sets[i].scales[1])),
                "layernorm_backward_dequant[ln_in]": (nb_lq, in_sz * n_l, lambda i: sf.layernorm_backward_dequant(
                    sets[i].codes[1], sets[i].scales[1], bits, block, mu[i], rs[i], gam, lnx[i], lny[i])),
            }
            for name, (nb, wb, fn) in ln_runs.items():
                for i in range(len(sets)):
                    fn(i)
                torch.cuda.synchronize()
                ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(12)]
                for i, (a, b) in enumerate(ev):
                    a.record()
                    fn(i % n_sets)
                    b.record()
                torch.cuda.synchronize()
                ms = sorted(a.elapsed_time(b) for a, b in ev)[len(ev) // 2]
                extras[name] = extra_record(name, ms, nb, wb, counters)
            del lny, mu, rs, pv, pi, rp, lws

            # Eq. 1 taken while the update is applied (weights read, update read, weights written: one pass instead of
            # the optimizer's own apply pass, a kept copy of the old weights and the scoring pass); on copies, so that
            # the step's own tensors stay as generated
            w_tmp = [p.clone() for p in prev]
            upd = [c.clone() for c in cur] if cfg.delta_given else [c - p.float() for p, c in zip(prev, cur)]
            ws_apply = torch.empty_like(ws)
            d_apply = torch.empty_like(d_dev)
            sf.layer_delta_plan(w_tmp, upd, ws_apply)
            for _ in range(2):
                sf.layer_delta_apply_run(numel, pdt, sf.F32, 0.0, d_apply, ws_apply)
            torch.cuda.synchronize()
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(8)]
            for a, b in ev:
                a.record()
                sf.layer_delta_apply_run(numel, pdt, sf.F32, 0.0, d_apply, ws_apply)
                b.record()
            torch.cuda.synchronize()
            ms = sorted(a.elapsed_time(b) for a, b in ev)[len(ev) // 2]
            nb = sum(numel) * (2 * esize(cfg.w_dtype) + 4) + 4 * L
            extras["apply_update_layer_delta[all weight tensors]"] = extra_record(
                "apply_update_layer_delta[all weight tensors]", ms, nb, sum(numel) * esize(cfg.w_dtype) + 4 * L, counters)
            del w_tmp, upd, ws_apply, d_apply

            # one frozen encoder block of this configuration through the autograd wrappers: activation bytes held between
            # forward and backward, against the same block in plain torch ops (the paper's figures are for whole models
            # on its own hardware: context, not a target)
            from paper_2305_18513_amd import autograd as ag
            blk_b = min(cfg.batch, 32)
            xb = torch.randn(blk_b, cfg.tokens, cfg.hidden, device="cuda").to(cfg.act_dtype).requires_grad_(True)
            blk = ag.encoder_block_params(cfg.hidden, seed=cfg.seed, dtype=cfg.act_dtype)
            keep = cfg.keep_ppm
            for wrapped in (False, True):                       # untimed first pass of each
                ag.held_activation_bytes(lambda: ag.frozen_encoder_block(xb, blk, cfg.heads, wrapped, keep, bits, block))
            kept_p, ms_p = ag.held_activation_bytes(lambda: ag.frozen_encoder_block(xb, blk, cfg.heads, False))
            kept_w, ms_w = ag.held_activation_bytes(lambda: ag.frozen_encoder_block(xb, blk, cfg.heads, True, keep, bits, block))
            extras["encoder_block_autograd"] = {
                "shape": {"batch": blk_b, "tokens": cfg.tokens, "hidden": cfg.hidden, "heads": cfg.heads},
                "held_MB_plain_torch": round(kept_p / 1e6, 1), "held_MB_wrapped": round(kept_w / 1e6, 1),
                "reduction": round(kept_p / max(kept_w, 1), 2),
                "fwd_bwd_ms_plain_torch": round(ms_p, 3), "fwd_bwd_ms_wrapped": round(ms_w, 3)}
            del xb, blk
        except Exception as exc:       # an extra must not cost the step its result line
            extras.setdefault("errors", []).append(repr(exc))

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # host side of the step alone: ils_update + ils_select over the L scores
    lat = []
    probe_d, probe_new = d_vec.copy(), d_host_pinned.numpy().copy()
    for _ in range(50):
        th = time.perf_counter()
        sf.ils_update(probe_d, probe_new, mask)
        sf.ils_select(probe_d, n_freeze)
        lat.append((time.perf_counter() - th) * 1e6)
    host_ils_us = sorted(lat)[len(lat) // 2]

    def checksum(t):
        """sum of the tensor's 32-bit words modulo 2^32 (identifies the generated input)"""
        w = t.contiguous().view(-1).view(torch.uint8)
        w = w[: w.numel() // 4 * 4].view(torch.int32)
        return int(w.sum(dtype=torch.int64).item()) & 0xFFFFFFFF

    input_checksum = {"gelu_in": checksum(sets[0].gelu), "ln_in": checksum(sets[0].ln[0]),
                      "scores": checksum(sets[0].scores), "w_prev[0]": checksum(prev[0])}

    ms_per_step = wall * 1e3 / args.steps
    value = step_bytes / (wall / args.steps) / 1e9

    kernels = kernel_table(wl, survey, timers, dom, args.steps, counters, with_probe=True)
    kd = kernels[dom]
    cnt = counters.get((cfg.index, dom), {})
    traffic = None
    if cnt.get("fetch_bytes") is not None and cnt.get("write_bytes") is not None:
        traffic = cnt["fetch_bytes"] + cnt["write_bytes"]
    roofline = {"kernel": dom, "bound": kd["bound"], "achieved": kd["GBps"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": kd["frac_hbm_peak"], "traffic": traffic,
                "traffic_source": "profiles/kernel_counters.txt (rocprofv3 FETCH_SIZE + WRITE_SIZE per launch, from "
                                  "separate profiling runs of this bench; not measured in this run)",
                "algorithmic_bytes": kd["bytes_per_launch"], "avg_ms": kd["avg_ms"],
                "bound_rule": "launch: bytes / 8 TB/s < 4 us; issue: max(VALU, SALU) wave instructions per row "
                              "(profiles/kernel_counters.txt) x rows x 4 cycles / (1024 SIMDs x 2.4 GHz) >= half the "
                              "measured time; hbm: otherwise"}
    if cnt.get("rows") and (cnt.get("valu_per_row") or cnt.get("salu_per_row")):
        # the other roofline of this kernel: wave instructions issued against what the chip can issue (each compute
        # unit starts one vector and one scalar wave instruction a cycle: 256 x 2.4 GHz = 614.4 G/s per pipe)
        per_row = max(cnt.get("valu_per_row", 0.0), cnt.get("salu_per_row", 0.0))
        rate = per_row * cnt["rows"] / (kd["avg_ms"] * 1e-3) / 1e9
        peak = SIMDS * CLOCK_HZ / ISSUE_CYCLES / 1e9
        roofline["issue"] = {"valu_per_row": round(cnt.get("valu_per_row", 0.0), 1),
                             "salu_per_row": round(cnt.get("salu_per_row", 0.0), 1), "rows": int(cnt["rows"]),
                             "achieved": round(rate, 1), "peak": round(peak, 1), "unit": "G wave instructions/s (busier pipe)",
                             "frac": round(rate / peak, 4)}
    if "stream_probe" in kd:
        # a streaming kernel of the same read : write mix and size, timed the same way on this machine
        roofline["stream_probe"] = kd["stream_probe"]
        if "frac_of_stream_probe" in kd:
            roofline["frac_of_stream_probe"] = kd["frac_of_stream_probe"]

    # the other configurations, briefly (per-config throughput and the bound that applies, in this same record)
    configs = {}
    if not args.no_other_configs:
        main_summary = {"workload": wl.describe(), "ms_per_step": round(ms_per_step, 4), "GBps": round(value, 1),
                        "frac_hbm_peak": round(value / HBM_PEAK_GBS, 4), "dominant_kernel": dom,
                        "kernels": {n: {f: k[f] for f in ("calls", "avg_ms", "bytes_per_launch", "GBps", "frac_hbm_peak",
                                                          "bound", "measured_in") if f in k} for n, k in kernels.items()}}
        configs[str(cfg.index)] = main_summary

    out = {
        "metric": "activation-compression + freeze-score GB/s per fine-tune step; % of HBM peak",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if cfg.act_dtype == torch.float32 else "bf16", "data": "synthetic",
        "frac_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "config": {"workload": "config %d: %s-shaped (%d blocks, hidden %d, %d heads, tokens %d, batch %d)"
                               % (cfg.index, cfg.name, cfg.n_blocks, cfg.hidden, cfg.heads, cfg.tokens, cfg.batch),
                   "quant": "%d-bit block-%d" % (bits, block), "keep_k": cfg.keep_k, "score_cols": cfg.score_cols,
                   "prune_mode": "threshold" if cfg.threshold_variant else "topk",
                   "layers_scored": L, "n_freeze": n_freeze, "step_bytes": step_bytes,
                   "buffer_sets": n_sets, "input_checksum": input_checksum},
        "host_ils_us": round(host_ils_us, 1),
        "roofline": roofline,
        "kernels": kernels,
        "extras": extras,
    }
    if not args.no_other_configs:
        for ci in range(len(synth.CONFIGS)):
            if ci == cfg.index:
                continue
            try:
                configs[str(ci)] = brief_config(ci, counters)
            except Exception as exc:       # another configuration must not cost the headline one its line
                configs[str(ci)] = {"error": repr(exc)}
        out["configs"] = dict(sorted(configs.items()))
    if not args.no_cpu_baseline:
        try:
            out["cpu_baseline"] = cpu_baseline(cfg, bits, block, mode, tau, sets, prev, cur)
        except Exception as exc:           # the oracle leg must not cost the GPU result its line
            out["cpu_baseline"] = {"value": None, "unit": "GB/s", "cores": 0, "host_cores": os.cpu_count(), "kind": "oracle",
                                   "sample": "failed: %r" % (exc,)}
    print(json.dumps(out))
    return 0


def cpu_baseline(cfg, bits, block, mode, tau, sets, prev, cur):
    """The CPU oracle, as it stands, on a bounded sample of the same workload:
    the first resident encoder-block sets (full batch, copied back from HBM) and
    every weight tensor."""
    from oracle import ref
    threads = min(ref.host_threads(), 16)
    in_sz = esize(cfg.act_dtype)
    n_blocks = min(2, len(sets))

    def host(t):
        t = t.detach().cpu().contiguous()
        return t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()

    acts = [[host(a) for a in s.acts] for s in sets[:n_blocks]]
    scores = [host(s.scores) for s in sets[:n_blocks]]
    hp, hc = [host(t) for t in prev], [host(t) for t in cur]
    ref.lib()
    nbytes = 0
    t0 = time.perf_counter()
    for b in range(n_blocks):
        packed = []
        for a in acts[b]:
            packed.append(ref.quant_pack(a, mode=ref.Q_BLOCK, bits=bits, block=block, threads=threads))
            nbytes += quant_bytes(a.size, in_sz, bits, block)
        ref.prune_scores(scores[b], cfg.keep_k, mode=mode, tau=tau, threads=threads)
        nbytes += prune_bytes(scores[b].shape[0], scores[b].shape[1], cfg.keep_k, in_sz)
        for a, (c, sc) in zip(acts[b], packed):
            ref.dequant_unpack(c, sc, a.size, mode=ref.Q_BLOCK, bits=bits, block=block,
                               out_dtype=a.dtype, threads=threads)
            nbytes += quant_bytes(a.size, in_sz, bits, block)
    d = ref.layer_delta(hp, hc, cur_is_delta=cfg.delta_given, threads=threads)
    nbytes += sum(p.size for p in hp) * (esize(cfg.w_dtype) + 4)
    ref.ils_select(d, ref.freeze_count(d.size, cfg.freeze_rate))
    dt = time.perf_counter() - t0
    # the same oracle on one thread, on a slice it finishes in a few seconds: 1/16 of the first block's rows
    a0 = acts[0][0][: acts[0][0].size // 16 // block * block]
    s0 = scores[0][: scores[0].shape[0] // 16]
    t1 = time.perf_counter()
    c1, sc1 = ref.quant_pack(a0, mode=ref.Q_BLOCK, bits=bits, block=block, threads=1)
    ref.dequant_unpack(c1, sc1, a0.size, mode=ref.Q_BLOCK, bits=bits, block=block, out_dtype=a0.dtype, threads=1)
    ref.prune_scores(s0, cfg.keep_k, mode=mode, tau=tau, threads=1)
    dt1 = time.perf_counter() - t1
    nb1 = 2 * quant_bytes(a0.size, in_sz, bits, block) + prune_bytes(s0.shape[0], s0.shape[1], cfg.keep_k, in_sz)
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count()
    # cores: the threads the oracle ran on; host_cores: what the box has; usable_cores: what this process may use
    return {"value": round(nbytes / dt / 1e9, 3), "unit": "GB/s", "cores": threads, "host_cores": os.cpu_count(),
            "usable_cores": usable, "kind": "oracle",
            "seconds": round(dt, 2), "bytes": nbytes,
            "single_thread": {"value": round(nb1 / dt1 / 1e9, 3), "unit": "GB/s", "seconds": round(dt1, 2),
                              "sample": "quant + dequant of 1/16 of one GELU input and prune of 1/16 of one score tensor"},
            "sample": "%d of the %d encoder blocks at full batch (quant x3, prune, dequant x3 each) plus "
                      "layer_delta over all %d weight tensors and one ils_select; OpenMP over independent "
                      "blocks/rows/layers" % (n_blocks, cfg.n_blocks, len(hp))}


if __name__ == "__main__":
    sys.exit(main())
