"""GPU parity: slimfit_prune_global / slimfit_restore_global (Alg. 5 on the whole flattened
tensor) vs the CPU oracle.  Values and indices must be bit-identical."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2305_18513_amd import binding as sf
from paper_2305_18513_amd import synth
from tests.gpu_util import Guarded, require_gpu, to_np

pytestmark = pytest.mark.gpu


def _bits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a


def _run_both(x: torch.Tensor, k: int, by_magnitude: bool, restore=True, workspace=None):
    n = x.numel()
    vals = Guarded(k, x.dtype)
    idx = Guarded(k, torch.int32)
    ws = Guarded(sf.prune_global_workspace(n), torch.uint8) if workspace is None else workspace
    ptr = Guarded(sf.global_tile_ptr_len(n), torch.int32)
    sf.prune_global(x, k, vals.t, idx.t, by_magnitude=by_magnitude, tile_ptr=ptr.t, workspace=ws.t)
    torch.cuda.synchronize()
    vals.check(); idx.check(); ws.check(); ptr.check()
    ov, oi = ref.prune_global(to_np(x), k, by_magnitude=by_magnitude)
    np.testing.assert_array_equal(to_np(idx.t), oi)
    np.testing.assert_array_equal(_bits(to_np(vals.t)), _bits(ov))
    # tile pointers: survivors ahead of every 4096 elements, counted on the oracle's index list
    edges = np.arange(ptr.t.numel(), dtype=np.int64) * sf.GLOBAL_TILE
    np.testing.assert_array_equal(to_np(ptr.t), np.searchsorted(oi, edges, side="left").astype(np.int32))
    assert int(ptr.t[-1]) == k
    if restore:
        want = _bits(ref.restore_global(ov, oi, n))
        for tp in (None, ptr.t):                                   # zeros + scatter, and the one-pass form
            out = Guarded(n, x.dtype)
            sf.restore_global(vals.t, idx.t, k, out.t, tile_ptr=tp)
            torch.cuda.synchronize()
            out.check()
            np.testing.assert_array_equal(_bits(to_np(out.t)), want)
    # the pointer list is optional
    vals2 = Guarded(k, x.dtype)
    idx2 = Guarded(k, torch.int32)
    sf.prune_global(x, k, vals2.t, idx2.t, by_magnitude=by_magnitude, workspace=ws.t)
    torch.cuda.synchronize()
    vals2.check(); idx2.check()
    assert torch.equal(idx2.t, idx.t) and torch.equal(vals2.t.view(torch.uint8), vals.t.view(torch.uint8))
    return oi


SIZES = [(1, 1), (5, 2), (63, 63), (64, 6), (4096, 409), (4097, 1), (4097, 4097), (10000, 1000),
         (70001, 7000), (8192 * 3 + 5, 2500), ((1 << 20) + 3, 104857)]


@pytest.mark.parametrize("by_mag", [True, False])
@pytest.mark.parametrize("n,k", SIZES)
def test_fp32_random_ties_and_constant(n, k, by_mag):
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(n * 3 + k)
    x = torch.randn(n, generator=g, device="cuda")
    _run_both(x, k, by_mag)
    _run_both((x * 2).round() / 2, k, by_mag)                       # heavy ties, both signs, +-0
    _run_both(torch.full((n,), -0.75, device="cuda"), k, by_mag)    # every key equal
    z = torch.zeros(n, device="cuda")
    z[::2] = -0.0
    _run_both(z, k, by_mag)


@pytest.mark.parametrize("by_mag", [True, False])
@pytest.mark.parametrize("n,k", SIZES)
def test_bf16_random_ties_and_constant(n, k, by_mag):
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(n * 5 + k)
    x = torch.randn(n, generator=g, device="cuda").bfloat16()
    _run_both(x, k, by_mag)
    _run_both(((x.float() * 2).round() / 2).bfloat16(), k, by_mag)
    _run_both(torch.full((n,), -0.75, device="cuda").bfloat16(), k, by_mag)


def test_wide_dynamic_range_and_infinities():
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(11)
    n = 50000
    x = torch.randn(n, generator=g, device="cuda") * torch.exp2(torch.randint(-120, 120, (n,), generator=g,
                                                                              device="cuda").float())
    x[17] = float("inf")
    x[4099] = float("-inf")
    x[33] = 1e-42                                                     # subnormal
    x[34] = -1e-42
    for k in (1, 2, 3, 5000, n - 1):
        _run_both(x, k, True, restore=False)
        _run_both(x, k, False, restore=False)


def test_bunched_candidates_overflow_a_sub_list():
    """The keys that share the cut's leading digit sit in one tile: the candidate list gives up and the
    digits are counted from the tensor instead."""
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(21)
    n = 1 << 21
    for dtype in (torch.float32, torch.bfloat16):
        x = torch.rand(n, generator=g, device="cuda") * 0.5
        x[1000:4000] = 1.0 + torch.rand(3000, generator=g, device="cuda") * 0.06      # one 1/16-binade bin
        hot = torch.randperm(n, generator=g, device="cuda")[:100]
        hot = hot[(hot < 1000) | (hot >= 4000)]
        x[hot] = 2.0 + torch.rand(hot.numel(), generator=g, device="cuda")
        x = (x * torch.where(torch.rand(n, generator=g, device="cuda") < 0.5, -1.0, 1.0)).to(dtype)
        _run_both(x, int(hot.numel()) + 1500, True)
        # the same keys spread over the tensor take the list
        _run_both(x[torch.randperm(n, generator=g, device="cuda")].contiguous(), int(hot.numel()) + 1500, True)


def test_workspace_is_reusable_and_need_not_be_clean():
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(5)
    ws = Guarded(sf.prune_global_workspace(100000), torch.uint8)     # starts as 0xAB bytes
    for n, k in ((100000, 10000), (9000, 17), (100000, 99999)):
        x = torch.randn(n, generator=g, device="cuda")
        _run_both(x, k, True, workspace=ws)


def test_k_zero_and_empty_are_no_ops():
    require_gpu()
    x = torch.randn(100, device="cuda")
    vals = Guarded(4, torch.float32)
    idx = Guarded(4, torch.int32)
    before = vals.raw.clone()
    sf.prune_global(x, 0, vals.t, idx.t)
    sf.prune_global(x[:0], 0, vals.t, idx.t)
    torch.cuda.synchronize()
    assert torch.equal(before, vals.raw)
    out = Guarded(100, torch.float32)
    sf.restore_global(vals.t, idx.t, 0, out.t)
    torch.cuda.synchronize()
    out.check()
    assert not out.t.any()


def test_restore_skips_bad_indices_and_accepts_any_order():
    require_gpu()
    vals = torch.tensor([1.0, 2.0, 3.0, 4.0], device="cuda")
    idx = torch.tensor([7, -1, 0, 12], dtype=torch.int32, device="cuda")
    out = Guarded(9, torch.float32)
    sf.restore_global(vals, idx, 4, out.t)
    torch.cuda.synchronize()
    out.check()
    assert out.t.tolist() == [3.0, 0, 0, 0, 0, 0, 0, 1.0, 0]


def test_restore_with_inconsistent_tile_pointers_stays_in_bounds():
    require_gpu()
    n, k = 10000, 6
    vals = torch.arange(1, k + 1, device="cuda").float()
    idx = torch.tensor([5, 4095, 4096, 9000, 9999, 123456], dtype=torch.int32, device="cuda")
    out = Guarded(n, torch.float32)
    good = torch.tensor([0, 2, 3, 6], dtype=torch.int32, device="cuda")
    sf.restore_global(vals, idx, k, out.t, tile_ptr=good)
    torch.cuda.synchronize()
    out.check()
    want = torch.zeros(n)
    want[[5, 4095, 4096, 9000, 9999]] = torch.tensor([1.0, 2.0, 3.0, 4.0, 5.0])
    assert torch.equal(out.t.cpu(), want)
    for bad in ([0, 6, 6, 6], [-5, 100, 3, 99], [6, 0, 0, 0], [0, 0, 0, 0]):
        sf.restore_global(vals, idx, k, out.t, tile_ptr=torch.tensor(bad, dtype=torch.int32, device="cuda"))
        torch.cuda.synchronize()
        out.check()
        got = out.t.cpu()
        assert bool(((got == 0) | (got == want)).all())            # misplaced pairs are dropped, nothing else appears


def test_argument_errors():
    require_gpu()
    x = torch.randn(4096, device="cuda")
    vals = torch.empty(16, device="cuda")
    idx = torch.empty(16, dtype=torch.int32, device="cuda")
    ws = torch.empty(sf.prune_global_workspace(4096), dtype=torch.uint8, device="cuda")
    cases = [
        (dict(x=x, k=5000), sf.ERR_INVALID_ARG),                      # k > n
        (dict(x=x, k=-1), sf.ERR_INVALID_ARG),
        (dict(x=x[1:], k=4), sf.ERR_ALIGNMENT),
        (dict(x=x, k=4, workspace=ws[:64]), sf.ERR_WORKSPACE),
    ]
    for kw, want in cases:
        kw.setdefault("workspace", ws)
        xx = kw.pop("x")
        k = kw.pop("k")
        with pytest.raises(sf.SlimfitError) as e:
            sf.prune_global(xx, k, vals if k <= 16 else torch.empty(max(k, 1), device="cuda"),
                            idx if k <= 16 else torch.empty(max(k, 1), dtype=torch.int32, device="cuda"), **kw)
        assert e.value.status == want
    with pytest.raises(sf.SlimfitError):
        sf.prune_global_workspace(1 << 31)


@pytest.mark.parametrize("ci", [1, 2, 3, 4])
def test_layernorm_input_at_full_size(ci):
    """The paper's placement: 10 % of the standardised LayerNorm input, whole batch."""
    require_gpu()
    cfg = synth.CONFIGS[ci]
    x = synth.activation(cfg, "ln_in", device="cuda").reshape(-1)
    k = sf.keep_count(x.numel(), 100000)
    assert k == int(x.numel() * 0.1)
    _run_both(x, k, True)
