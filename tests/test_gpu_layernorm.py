"""GPU parity: the LayerNorm path around the pruned cache (slimfit_layernorm_forward,
slimfit_prune_global_standardized, slimfit_layernorm_backward_pruned) vs the CPU oracle.
The kept set of the standardised tensor is bit-identical given the same fp32 statistics; the fp32
arithmetic of forward and backward is compared with the fp64 oracle within the header's tolerances."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2305_18513_amd import binding as sf
from paper_2305_18513_amd import synth
from tests.gpu_util import Guarded, require_gpu, to_np

pytestmark = pytest.mark.gpu


def _inputs(seed, rows, H):
    g = torch.Generator(device="cuda").manual_seed(seed)
    x = torch.randn(rows, H, generator=g, device="cuda") * (0.5 + 2.5 * torch.rand(rows, 1, generator=g, device="cuda"))
    x = x + 4 * torch.rand(rows, 1, generator=g, device="cuda") - 2
    gamma = 0.5 + torch.rand(H, generator=g, device="cuda")
    beta = torch.rand(H, generator=g, device="cuda") - 0.5
    dy = torch.randn(rows, H, generator=g, device="cuda")
    return x, gamma, beta, dy


def _f32(t):
    """Device tensor (fp32 or bf16) -> host float32 array; the widening of bf16 is exact."""
    return t.detach().float().cpu().numpy()


def _forward_both(x, gamma, beta, eps=1e-5):
    rows, H = x.shape
    bf16 = x.dtype == torch.bfloat16
    y = Guarded(rows * H, x.dtype)
    mean = Guarded(rows, torch.float32)
    rstd = Guarded(rows, torch.float32)
    sf.layernorm_forward(x, gamma, beta, eps, y.t.view(rows, H), mean.t, rstd.t)
    torch.cuda.synchronize()
    y.check(); mean.check(); rstd.check()
    xh, gh, bh = _f32(x), to_np(gamma), to_np(beta)
    oy, om, orr = ref.layernorm_forward(xh, gh, bh, eps=eps, threads=4)
    xd = xh.astype(np.float64)
    xmax = np.abs(xd).max(axis=1)
    mu = xd.mean(1)
    rs = 1.0 / np.sqrt(xd.var(1) + eps)
    gm, gr = to_np(mean.t).astype(np.float64), to_np(rstd.t).astype(np.float64)
    assert np.all(np.abs(gm - mu) <= 1e-6 * xmax + 1e-30)
    assert np.all(np.abs(gr - rs) <= 2e-6 * rs)
    xt = (xd - mu[:, None]) * rs[:, None]
    tol = np.abs(gh)[None, :] * (4e-6 * np.abs(xt) + 2e-6 * (xmax * rs)[:, None]) + 1e-6 * np.abs(oy.astype(np.float64))
    gy = _f32(y.t).reshape(rows, H).astype(np.float64)
    want = xt * gh.astype(np.float64) + bh.astype(np.float64)
    if bf16:
        tol = tol + np.abs(want) * 2.0 ** -8                                   # the output's own rounding
    bad = np.abs(gy - want) > tol
    assert not bad.any(), "y: %d outside tolerance, worst ratio %.3g" % (int(bad.sum()), float((np.abs(gy - want) / tol).max()))
    # the later stages are fed with the oracle's statistics (fp64 results rounded to fp32), not with the kernel's
    return torch.from_numpy(om).cuda(), torch.from_numpy(orr).cuda()


def _prune_both(x, mean, rstd, k, by_mag=True):
    rows, H = x.shape
    n = rows * H
    vals = Guarded(k, torch.float32)
    idx = Guarded(k, torch.int32)
    ptr = Guarded(sf.global_tile_ptr_len(n), torch.int32)
    rptr = Guarded(rows + 1, torch.int32)
    ws = Guarded(sf.prune_global_workspace(n), torch.uint8)
    sf.prune_global_standardized(x, mean, rstd, k, vals.t, idx.t, by_mag, ptr.t, rptr.t, ws.t)
    torch.cuda.synchronize()
    vals.check(); idx.check(); ptr.check(); rptr.check(); ws.check()
    xs = ref.standardize(_f32(x), to_np(mean), to_np(rstd)).reshape(-1)            # bf16 rows widen exactly
    ov, oi = ref.prune_global(xs, k, by_magnitude=by_mag)
    np.testing.assert_array_equal(to_np(idx.t), oi)
    np.testing.assert_array_equal(to_np(vals.t).view(np.uint32), ov.view(np.uint32))
    edges = np.arange(ptr.t.numel(), dtype=np.int64) * sf.GLOBAL_TILE
    np.testing.assert_array_equal(to_np(ptr.t), np.searchsorted(oi, edges, side="left").astype(np.int32))
    row_edges = np.arange(rows + 1, dtype=np.int64) * H
    np.testing.assert_array_equal(to_np(rptr.t), np.searchsorted(oi, row_edges, side="left").astype(np.int32))
    return vals.t, idx.t, rptr.t


def _backward_both(vals, idx, ptr, k, rstd, gamma, dy):
    rows, H = dy.shape
    bf16 = dy.dtype == torch.bfloat16
    dx = Guarded(rows * H, dy.dtype)
    sf.layernorm_backward_pruned(vals, idx, ptr, k, rstd, gamma, dy, dx.t.view(rows, H))
    torch.cuda.synchronize()
    dx.check()
    vh, ih, rh, gh, dyh = to_np(vals)[:k], to_np(idx)[:k], to_np(rstd), to_np(gamma), _f32(dy)
    want = ref.layernorm_backward_pruned(vh, ih, rh, gh, dyh).astype(np.float64)
    dense = np.zeros(rows * H)
    dense[ih] = vh
    dense = dense.reshape(rows, H)
    g = gh.astype(np.float64) * dyh.astype(np.float64) * rh.astype(np.float64)[:, None] / H
    tol = 4e-6 * (H * np.abs(g) + np.abs(g).sum(1, keepdims=True) + np.abs(dense) * np.abs(g * dense).sum(1, keepdims=True)) + 1e-30
    if bf16:
        tol = tol + np.abs(want) * 2.0 ** -8
    got = _f32(dx.t).reshape(rows, H).astype(np.float64)
    bad = np.abs(got - want) > tol
    assert not bad.any(), "dx: %d outside tolerance, worst ratio %.3g" % (int(bad.sum()), float((np.abs(got - want) / tol).max()))


SHAPES = [(1, 4), (3, 8), (5, 64), (9, 252), (9, 248), (7, 768), (33, 1024), (6, 1000), (4, 2048), (3, 4096), (130, 20),
          (130, 24), (1025, 12), (1025, 16), (300, 512)]


# a bf16 row must be whole 16-byte vectors (8 elements)
CHAIN_CASES = [(r, h, torch.float32) for r, h in SHAPES] + [(r, h, torch.bfloat16) for r, h in SHAPES if h % 8 == 0]


@pytest.mark.parametrize("rows,H,dtype", CHAIN_CASES)
def test_forward_prune_backward_chain(rows, H, dtype):
    require_gpu()
    x, gamma, beta, dy = _inputs(rows * 7 + H, rows, H)
    x, dy = x.to(dtype), dy.to(dtype)
    mean, rstd = _forward_both(x, gamma, beta)
    n = rows * H
    for k in sorted({max(1, n // 10), 1, n}):
        vals, idx, ptr = _prune_both(x, mean, rstd, k)
        _backward_both(vals, idx, ptr, k, rstd, gamma, dy)
    _prune_both(x, mean, rstd, max(1, n // 10), by_mag=False)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("rows,H", [(1, 4), (1, 8), (63, 64), (64, 252), (64, 248), (65, 768), (1000, 1024), (130, 4096),
                                    (257, 20), (257, 24)])
def test_active_layer_gradients(rows, H, dtype):
    require_gpu()
    bf16 = dtype == torch.bfloat16
    x, gamma, beta, dy = _inputs(rows * 3 + H, rows, H)
    x, dy = x.to(dtype), dy.to(dtype)
    if bf16 and H % 8:                                                          # a bf16 row must be whole 16-byte vectors
        with pytest.raises(sf.SlimfitError) as e:
            sf.layernorm_backward(x, torch.zeros(rows, device="cuda"), torch.ones(rows, device="cuda"), gamma, dy,
                                  torch.empty_like(x))
        assert e.value.status == sf.ERR_INVALID_ARG
        return
    if bf16:
        _forward_both(x, gamma, beta)                                           # bf16 rows through the forward kernel too
    xh, dyh = _f32(x), _f32(dy)
    _, om, orr = ref.layernorm_forward(xh, to_np(gamma), to_np(beta), eps=1e-5, threads=4)
    mean, rstd = torch.from_numpy(om).cuda(), torch.from_numpy(orr).cuda()
    dg, db = Guarded(H, torch.float32), Guarded(H, torch.float32)
    sf.layernorm_param_grads(x, mean, rstd, dy, dg.t, db.t)
    torch.cuda.synchronize()
    dg.check(); db.check()
    dx = Guarded(rows * H, dtype)
    sf.layernorm_backward(x, mean, rstd, gamma, dy, dx.t.view(rows, H))
    torch.cuda.synchronize()
    dx.check()
    want = ref.layernorm_backward(xh, om, orr, to_np(gamma), dyh).astype(np.float64)
    xt64 = (xh.astype(np.float64) - om.astype(np.float64)[:, None]) * orr.astype(np.float64)[:, None]
    g64 = to_np(gamma).astype(np.float64) * dyh.astype(np.float64) * orr.astype(np.float64)[:, None] / H
    tol = 4e-6 * (H * np.abs(g64) + np.abs(g64).sum(1, keepdims=True) + np.abs(xt64) * np.abs(g64 * xt64).sum(1, keepdims=True)) + 1e-30
    if bf16:
        tol = tol + np.abs(want) * 2.0 ** -8
    got = _f32(dx.t).reshape(rows, H).astype(np.float64)
    assert np.all(np.abs(got - want) <= tol), "dense dx: worst ratio %.3g" % float((np.abs(got - want) / tol).max())
    wg, wb = ref.layernorm_param_grads(xh, om, orr, dyh)
    xt = (xh.astype(np.float64) - om.astype(np.float64)[:, None]) * orr.astype(np.float64)[:, None]
    tol_g = 4e-6 * np.abs(xt * dyh).sum(0) + 1e-30
    tol_b = 4e-6 * np.abs(dyh.astype(np.float64)).sum(0) + 1e-30
    assert np.all(np.abs(to_np(dg.t).astype(np.float64) - wg) <= tol_g)
    assert np.all(np.abs(to_np(db.t).astype(np.float64) - wb) <= tol_b)


def test_prune_with_arbitrary_statistics_and_ties():
    """The selection only depends on the two fp32 operations, whatever the statistics are."""
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(3)
    rows, H = 300, 768
    x = (torch.randn(rows, H, generator=g, device="cuda") * 4).round() / 4          # many equal x~ within a row
    mean = torch.randn(rows, generator=g, device="cuda")
    rstd = torch.rand(rows, generator=g, device="cuda") + 0.5
    rstd[::7] = 1.0
    mean[::7] = 0.0
    for k in (1, 2000, rows * H // 10, rows * H - 1):
        _prune_both(x, mean, rstd, k)


def test_backward_with_nothing_kept_and_inconsistent_pointers():
    require_gpu()
    rows, H = 17, 256
    x, gamma, beta, dy = _inputs(5, rows, H)
    mean, rstd = _forward_both(x, gamma, beta)
    n = rows * H
    ptr0 = torch.zeros(rows + 1, dtype=torch.int32, device="cuda")
    _backward_both(torch.empty(0, device="cuda"), torch.empty(0, dtype=torch.int32, device="cuda"), ptr0, 0, rstd,
                   gamma, dy)
    # pointers that file the pairs under wrong rows: no fault, pairs outside their row are dropped
    k = n // 10
    vals, idx, ptr = _prune_both(x, mean, rstd, k)
    dx = Guarded(n, torch.float32)
    for bad in (torch.full_like(ptr, k), torch.flip(ptr, [0]).contiguous(), ptr * 0 - 7, ptr * 3):
        sf.layernorm_backward_pruned(vals, idx, bad, k, rstd, gamma, dy, dx.t.view(rows, H))
        torch.cuda.synchronize()
        dx.check()
        assert bool(torch.isfinite(dx.t).all())


def test_argument_errors():
    require_gpu()
    x = torch.randn(8, 64, device="cuda")
    y = torch.empty_like(x)
    ga = torch.ones(64, device="cuda")
    m = torch.empty(8, device="cuda")
    with pytest.raises(sf.SlimfitError) as e:
        sf.layernorm_forward(x, ga, ga, 1e-5, x, m, m.clone())                      # in place
    assert e.value.status == sf.ERR_INVALID_ARG
    big = torch.randn(2, 4100, device="cuda")
    with pytest.raises(sf.SlimfitError) as e:
        sf.layernorm_forward(big, torch.ones(4100, device="cuda"), torch.ones(4100, device="cuda"), 1e-5,
                             torch.empty_like(big), m, m.clone())
    assert e.value.status == sf.ERR_UNSUPPORTED
    odd = torch.randn(4, 6, device="cuda")
    with pytest.raises(sf.SlimfitError) as e:
        sf.prune_global_standardized(odd, m, m, 2, torch.empty(2, device="cuda"),
                                     torch.empty(2, dtype=torch.int32, device="cuda"))
    assert e.value.status == sf.ERR_INVALID_ARG
    xb = x.bfloat16()[:, :60].contiguous()                                         # 60 bf16 elements: not whole vectors
    with pytest.raises(sf.SlimfitError) as e:
        sf.prune_global_standardized(xb, m, m, 2, torch.empty(2, device="cuda"),
                                     torch.empty(2, dtype=torch.int32, device="cuda"))
    assert e.value.status == sf.ERR_INVALID_ARG


@pytest.mark.parametrize("ci", [1, 2, 3, 4])
def test_layernorm_input_at_full_size(ci):
    """The paper's placement end to end on the configuration's LayerNorm input: forward, 10 % of x~ kept, backward."""
    require_gpu()
    cfg = synth.CONFIGS[ci]
    x = synth.activation(cfg, "ln_in", device="cuda").reshape(-1, cfg.hidden)
    rows, H = x.shape
    g = torch.Generator(device="cuda").manual_seed(ci)
    gamma = 0.5 + torch.rand(H, generator=g, device="cuda")
    beta = torch.rand(H, generator=g, device="cuda") - 0.5
    dy = torch.randn(rows, H, generator=g, device="cuda").to(x.dtype)
    mean, rstd = _forward_both(x, gamma, beta)
    k = sf.keep_count(x.numel(), 100000)
    vals, idx, ptr = _prune_both(x, mean, rstd, k)
    _backward_both(vals, idx, ptr, k, rstd, gamma, dy)
