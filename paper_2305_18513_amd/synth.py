"""Seeded synthetic inputs for the SlimFit hot path.

This module only draws random tensors with the shapes and value distributions
of the five workload configurations; it holds none of the method's arithmetic
and imports neither the HIP binding nor the CPU oracle, so both sides can be
fed the same bytes.  Tensors are produced by torch on the requested device
(``cpu`` for host-only tests, ``cuda`` at full size) from a
``torch.Generator`` seeded per (config seed, tensor kind, encoder block).

Shapes follow the paper's per-block activation counts (Appendix, table of
activations per layer): GELU input B*T*4H, LayerNorm input B*T*H, attention
probabilities B*h*T*T; the freeze-score units follow the per-weight-tensor
layer list of the heat-map appendix: per encoder block four HxH matrices, one
Hx4H, one 4HxH and two LayerNorm weight vectors of length H.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Tuple

import torch


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    index: int
    n_blocks: int          # encoder blocks
    hidden: int
    heads: int
    tokens: int            # sequence length / number of image tokens
    batch: int
    act_dtype: torch.dtype = torch.float32
    w_dtype: torch.dtype = torch.float32
    delta_given: bool = False          # pass fp32 deltas instead of W_t
    outliers: str = "sparse"           # "sparse" (x20 w.p. 0.1%) | "student_t"
    quant_bits: Tuple[int, ...] = (4,)
    quant_block: int = 64
    keep_ppm: int = 100_000            # fraction of scores kept, parts/million
    keep_k: int = 0                    # pairs kept per score row: a stated figure of the workload (6, 12, 9, 38, 9),
                                       # not computed here; both libraries' own count functions are tested against it
    n_freeze: int = 0                  # layers frozen per iteration, likewise stated (15, 91, 91, 182, 182)
    threshold_variant: bool = False
    freeze_rate: float = 0.95
    seed: int = 0
    logit_sigma: float = 1.0 / math.sqrt(32.0)

    @property
    def ffn(self) -> int:
        return 4 * self.hidden

    @property
    def gelu_in_numel(self) -> int:
        return self.batch * self.tokens * self.ffn

    @property
    def ln_in_numel(self) -> int:
        return self.batch * self.tokens * self.hidden

    @property
    def score_rows(self) -> int:
        return self.batch * self.heads * self.tokens

    @property
    def score_cols(self) -> int:
        return self.tokens

    @property
    def unit_numels(self) -> List[int]:
        h, f = self.hidden, self.ffn
        per_block = [h * h, h * h, h * h, h * h, h, h * f, f * h, h]
        return per_block * self.n_blocks

    @property
    def n_units(self) -> int:
        return 8 * self.n_blocks

    @property
    def threshold_tau(self) -> float:
        """Expected 95th percentile of a log-normal softmax row entry."""
        s = self.logit_sigma
        return math.exp(1.645 * s - 0.5 * s * s) / self.score_cols


CONFIGS: Tuple[WorkloadConfig, ...] = (
    WorkloadConfig("tiny", 0, 2, 128, 4, 64, 4, keep_k=6, n_freeze=15, seed=0),
    WorkloadConfig("bert_base", 1, 12, 768, 12, 128, 32, keep_k=12, n_freeze=91, seed=1),
    WorkloadConfig("vit_base", 2, 12, 768, 12, 197, 128, outliers="student_t",
                   quant_bits=(8, 4), keep_ppm=50_000, keep_k=9, n_freeze=91, seed=2),
    WorkloadConfig("bert_large", 3, 24, 1024, 16, 384, 128, keep_k=38, n_freeze=182, seed=3),
    WorkloadConfig("vit_large", 4, 24, 1024, 16, 197, 256,
                   act_dtype=torch.bfloat16, w_dtype=torch.bfloat16,
                   delta_given=True, outliers="student_t", quant_block=32,
                   keep_ppm=50_000, keep_k=9, n_freeze=182, threshold_variant=True, seed=4),
)

_KIND = {"w_prev": 1, "delta": 2, "lr": 3, "gelu_in": 4, "ln_in": 5,
         "scores": 6, "channels": 7}


def _gen(cfg: WorkloadConfig, kind: str, block: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(cfg.seed * 1_000_003 + _KIND[kind] * 10_007 + block)
    return g


def weight_units(cfg: WorkloadConfig, device="cpu", n_blocks=None):
    """Per-unit (w_prev, w_cur_or_delta) lists for Eq. 1.

    w_prev ~ N(0, 0.02); delta = lr_i * N(0,1) with lr_i = 10**U(-6,-3) per
    unit.  fp32 configs return W_t = W_{t-1} + delta; the bf16 config returns
    bf16 W_{t-1} and the fp32 delta itself.
    """
    nb = cfg.n_blocks if n_blocks is None else n_blocks
    numels = cfg.unit_numels[: 8 * nb]
    prev, cur = [], []
    glr = _gen(cfg, "lr", 0, "cpu")
    lrs = 10.0 ** (torch.rand(len(numels), generator=glr, dtype=torch.float64)
                   * 3.0 - 6.0)
    for i, n in enumerate(numels):
        gp = _gen(cfg, "w_prev", i, device)
        gd = _gen(cfg, "delta", i, device)
        wp = torch.randn(n, generator=gp, device=device, dtype=torch.float32) * 0.02
        # the 32-bit uniform source behind randn yields an exact 0.0 about once in 10^7 draws; a
        # continuous N(0, 0.02) never does, and Eq. 1 divides by this tensor
        wp = torch.where(wp == 0, torch.full_like(wp, 0.02), wp)
        dl = torch.randn(n, generator=gd, device=device, dtype=torch.float32) * float(lrs[i])
        if cfg.w_dtype == torch.bfloat16:
            wp = wp.to(torch.bfloat16)
        if cfg.delta_given:
            prev.append(wp)
            cur.append(dl)
        else:
            prev.append(wp)
            cur.append(wp.float() + dl)
    return prev, cur


def activation(cfg: WorkloadConfig, kind: str, device="cpu", block: int = 0,
               batch=None) -> torch.Tensor:
    """GELU-input (B,T,4H) or LayerNorm-input (B,T,H) tensor.

    N(0,1) body.  "sparse": every element independently x20 with probability
    0.001.  "student_t": a seeded 1 % of the channels (last dimension) is
    drawn from Student-t with 3 degrees of freedom instead.
    """
    if kind not in ("gelu_in", "ln_in"):
        raise ValueError("kind must be gelu_in or ln_in")
    b = cfg.batch if batch is None else batch
    width = cfg.ffn if kind == "gelu_in" else cfg.hidden
    g = _gen(cfg, kind, block, device)
    x = torch.randn(b, cfg.tokens, width, generator=g, device=device,
                    dtype=torch.float32)
    if cfg.outliers == "sparse":
        hit = torch.rand(x.shape, generator=g, device=device) < 0.001
        x = torch.where(hit, x * 20.0, x)
    else:
        gc = _gen(cfg, "channels", block * 2 + (kind == "ln_in"), "cpu")
        n_heavy = max(1, width // 100)
        chans = torch.randperm(width, generator=gc)[:n_heavy].to(device)
        z = torch.randn(b, cfg.tokens, n_heavy, generator=g, device=device)
        chi = torch.randn(3, b, cfg.tokens, n_heavy, generator=g,
                          device=device).square().sum(0)
        x[:, :, chans] = z / torch.sqrt(chi / 3.0)
    return x.to(cfg.act_dtype).contiguous()


def attention_scores(cfg: WorkloadConfig, device="cpu", block: int = 0,
                     batch=None) -> torch.Tensor:
    """Attention probabilities as a (B*h*T, T) row-major matrix.

    Logits ~ N(0,1) * logit_sigma, softmax over each row in fp32.
    """
    b = cfg.batch if batch is None else batch
    rows = b * cfg.heads * cfg.tokens
    g = _gen(cfg, "scores", block, device)
    p = torch.empty(rows, cfg.tokens, device=device, dtype=torch.float32)
    step = max(1, (1 << 26) // cfg.tokens)      # bound the temporary
    for lo in range(0, rows, step):
        hi = min(rows, lo + step)
        z = torch.randn(hi - lo, cfg.tokens, generator=g, device=device,
                        dtype=torch.float32) * cfg.logit_sigma
        p[lo:hi] = torch.softmax(z, dim=-1)
    return p.to(cfg.act_dtype).contiguous()


def initial_distance(cfg: WorkloadConfig, n_units=None) -> torch.Tensor:
    """Start-up distance vector: large random values (host, fp32)."""
    n = cfg.n_units if n_units is None else n_units
    g = _gen(cfg, "lr", 1, "cpu")
    return (1e30 * (1.0 + torch.rand(n, generator=g))).float()
