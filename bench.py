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

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by the same counters' reading of
# a 1 GiB device copy; see profiles/bench_config3_bert_large.txt), for the default workload only.
MEASURED_TRAFFIC_BYTES = {
    3: {"quant_pack[gelu_in]": 918.6e6, "dequant_unpack[gelu_in]": 918.8e6,
        "prune_scores": 1399.1e6, "layer_delta": 2417.3e6},
}


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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=3, help="workload index 0..4 (3 = BERT-large-shaped)")
    ap.add_argument("--sets", type=int, default=3, help="distinct encoder-block buffer sets to rotate over")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip kernels outside the timed step (restore_scores, 8-bit scores, whole-tensor pruning)")
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

    cfg = synth.CONFIGS[args.config]
    bits = cfg.quant_bits[-1]
    block = cfg.quant_block
    mode = sf.PRUNE_THRESHOLD if cfg.threshold_variant else sf.PRUNE_TOPK
    tau = cfg.threshold_tau if cfg.threshold_variant else 0.0
    torch.cuda.set_device(0)
    in_sz = esize(cfg.act_dtype)

    n_sets = max(1, min(args.sets, cfg.n_blocks))
    sets = [BlockSet(cfg, b, bits) for b in range(n_sets)]
    prev, cur = synth.weight_units(cfg, "cuda")
    numel = [t.numel() for t in prev]
    L = len(numel)
    ws = torch.empty(sf.layer_delta_workspace(numel), dtype=torch.uint8, device="cuda")
    d_dev = torch.empty(L, dtype=torch.float32, device="cuda")
    d_host_pinned = torch.empty(L, dtype=torch.float32, pin_memory=True)
    d_vec = synth.initial_distance(cfg).numpy().copy()
    n_freeze = sf.freeze_count(L, cfg.freeze_rate)
    _, mask = sf.ils_select(d_vec, n_freeze)
    pdt = sf.BF16 if cfg.w_dtype == torch.bfloat16 else sf.F32
    sf.layer_delta_plan(prev, cur, ws)           # pointers are stable across steps: planned once
    torch.cuda.synchronize()

    w_bytes = sum(numel) * (esize(cfg.w_dtype) + 4) + 4 * L
    b_quant = [quant_bytes(a.numel(), in_sz, bits, block) for a in sets[0].acts]
    b_prune = prune_bytes(cfg.score_rows, cfg.score_cols, cfg.keep_k, in_sz)
    step_bytes = cfg.n_blocks * (2 * sum(b_quant) + b_prune) + w_bytes
    names_q = ["quant_pack[gelu_in]", "quant_pack[ln_in]", "quant_pack[ln_in]"]
    names_d = ["dequant_unpack[gelu_in]", "dequant_unpack[ln_in]", "dequant_unpack[ln_in]"]

    timers = Timers()            # the timed region: events around the dominant kernel only
    survey = Timers()            # one untimed step with events around every kernel

    def step(record):
        """record: None (no events), "all" (survey step) or the name of the one kernel to time."""
        nonlocal mask

        def run(name, nbytes, fn):
            if record == "all":
                survey.launch(name, nbytes, fn)
            elif record == name:
                timers.launch(name, nbytes, fn)
            else:
                fn()
        for b in range(cfg.n_blocks):                     # forward
            s = sets[b % n_sets]
            for i, a in enumerate(s.acts):
                run(names_q[i], b_quant[i],
                    lambda a=a, i=i, s=s: sf.quant_pack(a, sf.Q_BLOCK, bits, block, 0, s.codes[i], s.scales[i]))
            run("prune_scores", b_prune,
                lambda s=s: sf.prune_scores(s.scores, cfg.keep_k, mode, tau, s.vals, s.idx, s.counts))
        for b in reversed(range(cfg.n_blocks)):           # backward
            s = sets[b % n_sets]
            for i in reversed(range(3)):
                run(names_d[i], b_quant[i],
                    lambda i=i, s=s: sf.dequant_unpack(s.codes[i], s.scales[i], sf.Q_BLOCK, bits, block, 0, s.deq[i]))
        run("layer_delta", w_bytes,
            lambda: sf.layer_delta_run(numel, pdt, sf.F32, cfg.delta_given, 0.0, d_dev, ws))
        d_host_pinned.copy_(d_dev, non_blocking=True)
        torch.cuda.current_stream().synchronize()         # the host needs the L scores
        sf.ils_update(d_vec, d_host_pinned.numpy(), mask)
        _, mask = sf.ils_select(d_vec, n_freeze)

    for _ in range(args.warmup):
        step(None)
    # An event pair costs about 3 us of stream time; around each of the step's 169 launches that is 6 % of
    # the step.  So one untimed step surveys every kernel and names the dominant one, and the timed region
    # carries events around that kernel's launches only.
    step("all")
    torch.cuda.synchronize()
    survey.collect()
    dom = max(survey.total_ms, key=lambda n: survey.total_ms[n])
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(dom)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    timers.collect()

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
            extras["restore_scores"] = {"median_ms": round(ms, 5), "bytes_per_launch": nb,
                                        "GBps": round(nb / (ms * 1e-3) / 1e9, 1),
                                        "frac_hbm_peak": round(nb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
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
            extras["quant_pack[scores, fixed 4.4]"] = {"median_ms": round(ms, 5), "bytes_per_launch": nb,
                                                       "GBps": round(nb / (ms * 1e-3) / 1e9, 1),
                                                       "frac_hbm_peak": round(nb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
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
                "prune_global[ln_in, 10%]": lambda i: sf.prune_global(lns[i], k_ln, gv[i], gi[i], True, gp[i], gws),
                "restore_global[ln_in, tile pointers]": lambda i: sf.restore_global(gv[i], gi[i], k_ln, gout[i], gp[i]),
                "restore_global[ln_in, zeros+scatter]": lambda i: sf.restore_global(gv[i], gi[i], k_ln, gout[i]),
            }
            for name, fn in runs.items():
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
                extras[name] = {"median_ms": round(ms, 5), "bytes_per_launch": nb, "numel": n_ln, "k": k_ln,
                                "GBps": round(nb / (ms * 1e-3) / 1e9, 1),
                                "frac_hbm_peak": round(nb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
            del gv, gi, gp, gws, gout
            # the caches fused into their producer / consumer (x read once; the dequantised values never stored;
            # softmax and pruning in one pass over the logits)
            n_g = sets[0].gelu.numel()
            nb_g = 2 * n_g * in_sz + sf.packed_bytes(n_g, bits) + 4 * sf.num_blocks(n_g, block)
            rows_s, cols_s = sets[0].scores.shape
            nb_s = 2 * rows_s * cols_s * in_sz + rows_s * cfg.keep_k * (in_sz + 2)
            probs = [torch.empty_like(s.scores) for s in sets]
            fused = {
                "gelu_quant_pack[gelu_in]": (nb_g, lambda i: sf.gelu_quant_pack(
                    sets[i].gelu, sf.Q_BLOCK, bits, block, 0, sets[i].deq[0], sets[i].codes[0], sets[i].scales[0])),
                "gelu_backward_dequant[gelu_in]": (nb_g, lambda i: sf.gelu_backward_dequant(
                    sets[i].codes[0], sets[i].scales[0], sf.Q_BLOCK, bits, block, 0, sets[i].gelu, sets[i].deq[0])),
                "softmax_prune[scores as logits]": (nb_s, lambda i: sf.softmax_prune(
                    sets[i].scores, cfg.keep_k, probs[i], sets[i].vals, sets[i].idx)),
                # consumes the pairs the line above left; the score tensor stands in for the incoming gradient
                # (only its kept columns are read: k elements per row are the algorithmic bytes, although at
                # 10 % kept nearly every 128-byte line of it is touched)
                "softmax_backward_pruned[scores]": (
                    rows_s * cols_s * in_sz + rows_s * cfg.keep_k * (2 * in_sz + 2),
                    lambda i: sf.softmax_backward_pruned(sets[i].vals, sets[i].idx, None, sets[i].scores, probs[i])),
            }
            for name, (nb, fn) in fused.items():
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
                extras[name] = {"median_ms": round(ms, 5), "bytes_per_launch": nb,
                                "GBps": round(nb / (ms * 1e-3) / 1e9, 1),
                                "frac_hbm_peak": round(nb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
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
                "layernorm_forward[ln_in]": (2 * in_sz * n_l + 8 * rows_l, lambda i: sf.layernorm_forward(
                    lnx[i], gam, bet, 1e-5, lny[i], mu[i], rs[i])),
                "prune_global_standardized[ln_in, 10%]": (in_sz * n_l + 8 * k_l + 12 * rows_l, lambda i:
                    sf.prune_global_standardized(lnx[i], mu[i], rs[i], k_l, pv[i], pi[i], True, None, rp[i], lws)),
                "layernorm_backward_pruned[ln_in]": (2 * in_sz * n_l + 8 * k_l + 8 * rows_l, lambda i:
                    sf.layernorm_backward_pruned(pv[i], pi[i], rp[i], k_l, rs[i], gam, lnx[i], lny[i])),
                # the step's own cache (block-scaled codes of the LayerNorm input) written by the LayerNorm that
                # reads the input anyway, and the input gradient straight from that cache
                "layernorm_forward_quant_pack[ln_in]": (nb_lq, lambda i: sf.layernorm_forward_quant_pack(
                    lnx[i], gam, bet, 1e-5, bits, block, lny[i], mu[i], rs[i], sets[i].codes[1], sets[i].scales[1])),
                "layernorm_backward_dequant[ln_in]": (nb_lq, lambda i: sf.layernorm_backward_dequant(
                    sets[i].codes[1], sets[i].scales[1], bits, block, mu[i], rs[i], gam, lnx[i], lny[i])),
            }
            for name, (nb, fn) in ln_runs.items():
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
                extras[name] = {"median_ms": round(ms, 5), "bytes_per_launch": nb,
                                "GBps": round(nb / (ms * 1e-3) / 1e9, 1),
                                "frac_hbm_peak": round(nb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
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
            extras["apply_update_layer_delta[all weight tensors]"] = {
                "median_ms": round(ms, 5), "bytes_per_launch": nb, "GBps": round(nb / (ms * 1e-3) / 1e9, 1),
                "frac_hbm_peak": round(nb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
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

    # what a plain device copy of 1 GiB reaches on this machine (read + write bytes), for scale
    csrc = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    cdst = torch.empty_like(csrc)
    for _ in range(3):
        cdst.copy_(csrc)
    torch.cuda.synchronize()
    cev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
    for a, b in cev:
        a.record()
        cdst.copy_(csrc)
        b.record()
    torch.cuda.synchronize()
    copy_ms = sorted(a.elapsed_time(b) for a, b in cev)[len(cev) // 2]
    copy_gbs = 2 * csrc.numel() * 4 / (copy_ms * 1e-3) / 1e9
    del csrc, cdst

    # what a kernel that only streams reaches with the dominant kernel's own read : write mix and size
    probe = None
    try:
        reads = {"prune_scores": cfg.score_rows * cfg.score_cols * in_sz}
        for nm, a in zip(names_q, sets[0].acts):
            reads[nm] = a.numel() * in_sz
        dom_read = reads.get(dom, 0)
        dom_write = timers.bytes[dom] - dom_read if dom_read else 0
        if dom_read and dom_write > 0 and dom_read >= dom_write:
            # the probe writes 16 / ratio bytes per 16 bytes read, ratio a power of two: the one nearest the kernel's
            ratio = min((1, 2, 4, 8, 16), key=lambda r: abs(math.log2(r) - math.log2(dom_read / dom_write)))
            in_vecs = max(1024, dom_read // 16 // 1024 * 1024)
            psrc = torch.empty(in_vecs * 4, dtype=torch.float32, device="cuda").normal_()
            pdst = torch.empty(in_vecs * (16 // ratio), dtype=torch.uint8, device="cuda")
            for _ in range(3):
                sf.stream_probe(psrc, pdst, ratio)
            torch.cuda.synchronize()
            pev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(12)]
            for a, b in pev:
                a.record()
                sf.stream_probe(psrc, pdst, ratio)
                b.record()
            torch.cuda.synchronize()
            probe_ms = sorted(a.elapsed_time(b) for a, b in pev)[len(pev) // 2]
            probe_bytes = in_vecs * 16 + in_vecs * (16 // ratio)
            probe = {"read_write_ratio": ratio, "kernel_read_write_ratio": round(dom_read / dom_write, 2),
                     "bytes": probe_bytes, "ms": round(probe_ms, 5),
                     "GBps": round(probe_bytes / (probe_ms * 1e-3) / 1e9, 1)}
            del psrc, pdst
    except Exception as exc:  # the yardstick is context: it never costs the result its line
        probe = {"error": repr(exc)}

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

    def entry(t, name, per_step):
        calls = t.calls[name]
        avg_ms = t.total_ms[name] / calls
        gbs = t.bytes[name] / (avg_ms * 1e-3) / 1e9
        return {"calls": calls, "avg_ms": round(avg_ms, 5), "bytes_per_launch": t.bytes[name],
                "GBps": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                "total_ms_per_step": round(t.total_ms[name] / per_step, 4)}

    # every kernel from the survey step; the dominant one from the timed region
    kernels = {name: dict(entry(survey, name, 1), measured_in="survey step (untimed)") for name in survey.total_ms}
    kernels[dom] = dict(entry(timers, dom, args.steps), measured_in="timed region",
                        survey_avg_ms=kernels[dom]["avg_ms"])
    roofline = {"kernel": dom, "bound": "hbm", "achieved": kernels[dom]["GBps"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": kernels[dom]["frac_hbm_peak"],
                "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.index, {}).get(dom),
                "algorithmic_bytes": kernels[dom]["bytes_per_launch"], "avg_ms": kernels[dom]["avg_ms"],
                "measured_copy_GBps": round(copy_gbs, 1), "frac_of_measured_copy": round(kernels[dom]["GBps"] / copy_gbs, 4)}
    if probe is not None:
        # a streaming kernel of the same read : write mix and size, timed the same way on this machine
        roofline["stream_probe"] = probe
        if probe.get("GBps"):
            roofline["frac_of_stream_probe"] = round(kernels[dom]["GBps"] / probe["GBps"], 4)

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
    if not args.no_cpu_baseline:
        try:
            out["cpu_baseline"] = cpu_baseline(cfg, bits, block, mode, tau, sets, prev, cur)
        except Exception as exc:           # the oracle leg must not cost the GPU result its line
            out["cpu_baseline"] = {"value": None, "unit": "GB/s", "cores": 0, "kind": "oracle", "sample": "failed: %r" % (exc,)}
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
    return {"value": round(nbytes / dt / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "seconds": round(dt, 2), "bytes": nbytes,
            "single_thread": {"value": round(nb1 / dt1 / 1e9, 3), "unit": "GB/s", "seconds": round(dt1, 2),
                              "sample": "quant + dequant of 1/16 of one GELU input and prune of 1/16 of one score tensor"},
            "sample": "%d of the %d encoder blocks at full batch (quant x3, prune, dequant x3 each) plus "
                      "layer_delta over all %d weight tensors and one ils_select; OpenMP over independent "
                      "blocks/rows/layers" % (n_blocks, cfg.n_blocks, len(hp))}


if __name__ == "__main__":
    sys.exit(main())
