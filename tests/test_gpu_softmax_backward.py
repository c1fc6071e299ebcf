"""GPU parity: slimfit_softmax_backward_pruned vs the CPU oracle.  The pairs both sides consume are the
oracle's own (softmax_prune / prune_scores on the host, uploaded); outside the kept columns the output
must be +0 bit for bit, at the kept columns an fp32 evaluation within the tolerance the header states."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2305_18513_amd import binding as sf
from paper_2305_18513_amd import synth
from tests.gpu_util import Guarded, require_gpu, to_np

pytestmark = pytest.mark.gpu


def _wide32(a):
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32)
    return a.astype(np.float32)


def _dev(a, dtype):
    t = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()
    return t.view(dtype) if a.dtype == np.uint16 else t


def _run_both(vals_h, idx_h, counts_h, dp: torch.Tensor):
    """vals_h / idx_h / counts_h: host arrays from the oracle; dp: device tensor (rows, cols)."""
    rows, cols = dp.shape
    k = vals_h.shape[1]
    bf16 = dp.dtype == torch.bfloat16
    vals = _dev(vals_h, dp.dtype)
    idx = _dev(idx_h, torch.uint16)
    counts = None if counts_h is None else torch.from_numpy(counts_h).cuda()
    ds = Guarded(rows * cols, dp.dtype)
    before = dp.clone()
    sf.softmax_backward_pruned(vals, idx, counts, dp, ds.t.view(rows, cols))
    torch.cuda.synchronize()
    ds.check()
    assert torch.equal(dp.view(torch.uint8), before.view(torch.uint8))

    dph = to_np(dp)
    v32, d32 = _wide32(vals_h), _wide32(dph)
    want = ref.softmax_backward_pruned(v32, idx_h, counts_h, d32, threads=4).astype(np.float64)
    got_raw = to_np(ds.t).reshape(rows, cols)
    got = _wide32(got_raw).astype(np.float64)
    # tolerance per kept element
    kept = np.zeros((rows, cols), bool)
    cnt = np.full(rows, k) if counts_h is None else counts_h
    live = (np.arange(k)[None, :] < np.asarray(cnt)[:, None]) & (idx_h < cols)
    rr = np.broadcast_to(np.arange(rows)[:, None], idx_h.shape)
    kept[rr[live], idx_h[live].astype(np.int64)] = True
    dense = np.zeros((rows, cols))
    dense[rr[live], idx_h[live].astype(np.int64)] = v32[live]
    assert not got_raw.view(np.uint16 if bf16 else np.uint32)[~kept].any()       # +0 outside the kept set
    absdot = (np.abs(dense) * np.abs(d32.astype(np.float64))).sum(axis=1, keepdims=True)
    tol = np.abs(dense) * ((8 + k / 64) * 6e-8 * absdot + 1.2e-7 * np.abs(d32)) + 6e-8 * np.abs(want) + 1.2e-38
    if bf16:
        tol = tol + np.abs(want) * 2.0 ** -8
    bad = np.abs(got - want) > tol
    assert not bad.any(), "%d outside tolerance, worst ratio %.3g" % (
        int(bad.sum()), float((np.abs(got - want) / tol).max()))


SHAPES = [(1, 1, 1), (7, 5, 2), (7, 5, 5), (33, 64, 6), (65, 70, 69), (130, 128, 12), (257, 197, 9),
          (101, 384, 38), (40, 577, 57), (19, 1024, 102), (1001, 256, 32), (130, 16, 3), (9, 17, 17),
          (3, 5000, 500), (2, 4096, 4096), (5000, 3, 1), (11, 8191, 70)]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("rows,cols,k", SHAPES)
def test_pairs_from_softmax_prune(rows, cols, k, dtype):
    require_gpu()
    rng = np.random.default_rng(rows * 13 + cols)
    l = (rng.standard_normal((rows, cols)) * 2).astype(np.float32)
    if dtype == torch.bfloat16:
        lt = torch.from_numpy(l).to(torch.bfloat16)
        l = lt.view(torch.int16).numpy().view(np.uint16)
    vals_h, idx_h = ref.prune_scores(ref.softmax_prune(l, 1)[0], k)[:2]
    g = torch.Generator(device="cuda").manual_seed(rows + cols)
    dp = torch.randn(rows, cols, generator=g, device="cuda").to(dtype)
    _run_both(vals_h, idx_h, None, dp)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_threshold_mode_pairs_with_counts(dtype):
    require_gpu()
    rows, cols, k = 300, 197, 40
    rng = np.random.default_rng(5)
    p = rng.random((rows, cols)).astype(np.float32)
    p /= p.sum(1, keepdims=True)
    if dtype == torch.bfloat16:
        p = torch.from_numpy(p).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    vals_h, idx_h, counts_h = ref.prune_scores(p, k, mode=sf.PRUNE_THRESHOLD, tau=1.8 / cols)
    assert counts_h.min() < k                                   # some rows keep fewer than k: unused slots exist
    g = torch.Generator(device="cuda").manual_seed(6)
    dp = torch.randn(rows, cols, generator=g, device="cuda").to(dtype)
    _run_both(vals_h, idx_h, counts_h, dp)
    _run_both(vals_h, idx_h, None, dp)                          # the 0xFFFF sentinel alone


def test_argument_errors():
    require_gpu()
    dp = torch.randn(8, 64, device="cuda")
    ds = torch.empty_like(dp)
    v = torch.zeros(8, 4, device="cuda")
    i = torch.zeros(8, 4, dtype=torch.int16, device="cuda").view(torch.uint16)
    with pytest.raises(sf.SlimfitError) as e:
        sf.softmax_backward_pruned(v, i, None, dp, dp)                              # in place
    assert e.value.status == sf.ERR_INVALID_ARG
    with pytest.raises(sf.SlimfitError) as e:
        sf.softmax_backward_pruned(v, i, None, dp.view(-1)[1:449].view(7, 64), ds.view(-1)[1:449].view(7, 64))
    assert e.value.status == sf.ERR_ALIGNMENT
    big = torch.zeros(8, 65, device="cuda")
    bigi = torch.zeros(8, 65, dtype=torch.int16, device="cuda").view(torch.uint16)
    with pytest.raises(sf.SlimfitError) as e:
        sf.softmax_backward_pruned(big, bigi, None, dp, ds)                         # k > cols
    assert e.value.status == sf.ERR_INVALID_ARG
    sf.softmax_backward_pruned(v[:0], i[:0], None, dp[:0], ds[:0])                  # no rows: nothing to do


@pytest.mark.parametrize("ci", [1, 3])
def test_attention_scores_at_full_size(ci):
    require_gpu()
    cfg = synth.CONFIGS[ci]
    p = synth.attention_scores(cfg, device="cuda", batch=max(1, 300_000 // (cfg.heads * cfg.tokens)))
    rows = p.shape[0]
    k = cfg.keep_k
    vals_h, idx_h = ref.prune_scores(to_np(p), k, threads=4)[:2]
    g = torch.Generator(device="cuda").manual_seed(ci)
    dp = torch.randn(rows, p.shape[1], generator=g, device="cuda").to(p.dtype)
    _run_both(vals_h, idx_h, None, dp)
