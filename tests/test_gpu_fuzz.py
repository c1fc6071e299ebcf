"""Seeded, time-bounded differential tests: random shapes and value grids through the C ABI against the CPU
oracle, stopping at the first mismatch.  The grids are chosen so that ties fall on the cut on both sides of
zero (coarse multiples, constant rows, signed zeros, denormals); sizes stay small enough for the oracle."""
import random
import time

import pytest
import torch

from paper_2305_18513_amd import binding as sf
from tests.gpu_util import require_gpu
from tests.test_gpu_prune import _run_both
from tests.test_gpu_quant import _run_both as _quant_both

pytestmark = pytest.mark.gpu

PRUNE_SECONDS = 30.0
QUANT_SECONDS = 15.0


def _prune_input(rnd, g, rows, cols, dtype):
    kind = rnd.choice(["softmax", "softmax", "grid", "grid_neg", "const", "zeros", "denormal", "mixed"])
    x = torch.randn(rows, cols, generator=g, device="cuda")
    if kind == "softmax":
        p = torch.softmax(x * rnd.choice([0.177, 0.5, 2.0, 8.0]), dim=-1)
    elif kind == "grid":
        step = rnd.choice([0.25, 0.5, 1.0 / 64])
        p = (x / step).round() * step                           # few distinct values, both signs
    elif kind == "grid_neg":
        p = -((x.abs() * 4).round() / 4) - rnd.choice([0.0, 0.25])
        p[:, 0] = 3.0                                           # a positive maximum above tied negative values
    elif kind == "const":
        p = torch.full_like(x, rnd.choice([0.0, -0.0, 0.125, -2.0]))
    elif kind == "zeros":
        p = torch.where(x > 0.5, x, torch.zeros_like(x))
        p = torch.where(x < -1.0, -torch.zeros_like(x), p)      # +0, -0 and a few positive entries
    elif kind == "denormal":
        p = x * 1e-41
    else:
        p = x.clone()
        p[::2] = (p[::2] * 2).round() / 2
        p[1::3] = -p[1::3].abs()
    return p.to(dtype)


def test_prune_scores_random_cases():
    require_gpu()
    rnd = random.Random(20230518)
    t_end = time.time() + PRUNE_SECONDS
    n = 0
    while time.time() < t_end:
        dtype = rnd.choice([torch.float32, torch.bfloat16])
        cols = rnd.choice([rnd.randint(1, 70), rnd.randint(64, 256), rnd.randint(150, 260), rnd.randint(257, 2048)])
        rows = rnd.randint(1, max(2, 40000 // cols))
        k = rnd.choice([1, max(1, cols // 20), max(1, cols // 10), rnd.randint(1, min(cols, 16)), rnd.randint(1, cols), cols])
        mode = rnd.choice([sf.PRUNE_TOPK, sf.PRUNE_THRESHOLD])
        g = torch.Generator(device="cuda").manual_seed(rnd.randrange(1 << 30))
        p = _prune_input(rnd, g, rows, cols, dtype)
        if mode == sf.PRUNE_THRESHOLD:                          # thresholds that sit on entries of the tensor or between them
            flat = p.float().reshape(-1)
            tau = float(rnd.choice([flat[rnd.randrange(flat.numel())].item(), 0.0, -0.0, 1.0 / cols, 0.5, -0.5]))
        else:
            tau = 0.0
        print("prune case %d: rows=%d cols=%d k=%d %s mode=%d tau=%r" % (n, rows, cols, k, dtype, mode, tau), flush=True)
        with_counts = rnd.random() < 0.8
        # (without counts the unused slots of a threshold run cannot be told from pairs: no restore then)
        restore = rnd.random() < 0.3 and (with_counts or mode == sf.PRUNE_TOPK)
        _run_both(p, k, mode=mode, tau=tau, with_counts=with_counts, restore=restore)
        n += 1
    assert n >= 20


def test_quant_dequant_random_cases():
    require_gpu()
    rnd = random.Random(18513)
    t_end = time.time() + QUANT_SECONDS
    n_cases = 0
    while time.time() < t_end:
        dtype = rnd.choice([torch.float32, torch.bfloat16])
        n = rnd.choice([rnd.randint(1, 300), rnd.randint(300, 9000), rnd.randint(9000, 300000)])
        bits, block = rnd.choice([4, 8]), rnd.choice([32, 64, 128, 256])
        mode = rnd.choice([sf.Q_BLOCK, sf.Q_BLOCK, sf.Q_FIXED])
        fb = rnd.randint(0, 6)
        g = torch.Generator(device="cuda").manual_seed(rnd.randrange(1 << 30))
        x = torch.randn(n, generator=g, device="cuda") * rnd.choice([1e-3, 0.1, 1.0, 30.0])
        kind = rnd.choice(["plain", "halfway", "zeros", "outliers"])
        if kind == "halfway":
            x = (x * (1 << fb) * 2).round() / ((1 << fb) * 2)   # multiples of half a step: every .5 product occurs
        elif kind == "zeros":
            x = torch.where(x.abs() < 0.5 * x.abs().mean(), torch.zeros_like(x), x)
        elif kind == "outliers":
            hit = torch.rand(n, generator=g, device="cuda") < 0.01
            x = torch.where(hit, x * 50, x)
        x = x.to(dtype)
        print("quant case %d: n=%d bits=%d block=%d mode=%d fb=%d %s %s" % (n_cases, n, bits, block, mode, fb, dtype, kind), flush=True)
        _quant_both(x, mode, bits, block, fb)
        n_cases += 1
    assert n_cases >= 20
