"""GPU parity: slimfit_apply_update_layer_delta vs the CPU oracle.  The new weights are one fp32 addition (one more
rounding for bf16 weights) and must match bit for bit; the scores are those of slimfit_layer_delta with the update
given, 1e-6 relative against the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2305_18513_amd import binding as sf
from paper_2305_18513_amd import synth
from tests.gpu_util import Guarded, require_gpu, to_np

pytestmark = pytest.mark.gpu

RTOL = 1e-6


def _bits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a


def _run_both(w, delta, eps=0.0, split=False):
    """w, delta: lists of device tensors; w is updated in place (guard bytes behind every weight tensor)."""
    L = len(w)
    numel = [t.numel() for t in w]
    wh, dh = [to_np(t).copy() for t in w], [to_np(t).copy() for t in delta]
    guards = [Guarded(t.numel(), t.dtype) for t in w]
    for g, t in zip(guards, w):
        g.t.copy_(t)
    wg = [g.t for g in guards]
    ws = torch.empty(sf.layer_delta_workspace(numel), dtype=torch.uint8, device="cuda")
    d = Guarded(L, torch.float32)
    if split:
        sf.layer_delta_plan(wg, delta, ws)
        wdt = sf.BF16 if w[0].dtype == torch.bfloat16 else sf.F32
        ddt = sf.BF16 if delta[0].dtype == torch.bfloat16 else sf.F32
        sf.layer_delta_apply_run(numel, wdt, ddt, eps, d.t, ws)
    else:
        sf.apply_update_layer_delta(wg, delta, eps, d.t, ws)
    torch.cuda.synchronize()
    d.check()
    for g in guards:
        g.check()
    od, ow = ref.apply_update_layer_delta(wh, dh, eps=eps, threads=8)
    for t, before in zip(delta, dh):
        np.testing.assert_array_equal(_bits(to_np(t)), _bits(before))                 # the update is only read
    for g, want in zip(wg, ow):
        np.testing.assert_array_equal(_bits(to_np(g)), _bits(want))
    got = to_np(d.t)
    fin = np.isfinite(od)
    np.testing.assert_array_equal(np.isfinite(got), fin)
    np.testing.assert_allclose(got[fin], od[fin], rtol=RTOL, atol=0)
    np.testing.assert_array_equal(got[~fin], od[~fin])
    return got, wg


def test_ragged_sizes_many_layers():
    require_gpu()
    sizes = [1, 2, 3, 5, 0, 63, 64, 65, 1000, 4095, 8191, 8192, 8193, 0, 16384, 16385,
             3 * 8192 + 4, 100003, 7, 1 << 20] + [16384 * 2 + i for i in range(12)]
    g = torch.Generator(device="cuda").manual_seed(0)
    w = [torch.randn(n, generator=g, device="cuda") * 0.02 for n in sizes]
    dl = [torch.randn(n, generator=g, device="cuda") * 1e-4 for n in sizes]
    got, _ = _run_both(w, dl)
    assert got[4] == 0.0 and got[13] == 0.0
    again, _ = _run_both(w, dl, split=True)
    np.testing.assert_array_equal(got.view(np.uint32), again.view(np.uint32))


@pytest.mark.parametrize("wdt,ddt", [(torch.bfloat16, torch.float32), (torch.bfloat16, torch.bfloat16),
                                     (torch.float32, torch.bfloat16)])
def test_mixed_dtypes(wdt, ddt):
    require_gpu()
    sizes = [5, 4096, 16384, 16385, 70001]
    g = torch.Generator(device="cuda").manual_seed(1)
    w = [(torch.randn(n, generator=g, device="cuda") * 0.02).to(wdt) for n in sizes]
    dl = [(torch.randn(n, generator=g, device="cuda") * 1e-3).to(ddt) for n in sizes]
    _run_both(w, dl)


def test_scores_equal_layer_delta_with_the_update_given_and_eps():
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(2)
    sizes = [33000, 20, 16384]
    w = [torch.randn(n, generator=g, device="cuda") * 0.02 for n in sizes]
    w[1][3] = 0.0                                                        # a zero weight that changes
    dl = [torch.randn(n, generator=g, device="cuda") * 1e-4 for n in sizes]
    numel = [t.numel() for t in w]
    ws = torch.empty(sf.layer_delta_workspace(numel), dtype=torch.uint8, device="cuda")
    for eps in (0.0, 1e-8):
        d0 = torch.empty(3, device="cuda")
        sf.layer_delta(w, dl, True, eps, d0, ws)
        got, _ = _run_both(w, dl, eps=eps)
        # same terms, fp64 sums in a different order (other workgroup shape): equal up to the final fp32 rounding
        fin = np.isfinite(got)
        np.testing.assert_allclose(got[fin], to_np(d0)[fin], rtol=1.2e-7, atol=0)
        np.testing.assert_array_equal(got[~fin], to_np(d0)[~fin])
    assert np.isinf(_run_both(w, dl, eps=0.0)[0][1])


def test_argument_errors_and_missing_plan():
    require_gpu()
    w = [torch.randn(5000, device="cuda")]
    dl = [torch.randn(5000, device="cuda")]
    ws = torch.zeros(sf.layer_delta_workspace([5000]), dtype=torch.uint8, device="cuda")
    d = torch.empty(1, device="cuda")
    with pytest.raises(sf.SlimfitError) as e:
        sf.apply_update_layer_delta(w, w, 0.0, d, ws)                    # update aliases the weights
    assert e.value.status == sf.ERR_INVALID_ARG
    with pytest.raises(sf.SlimfitError) as e:
        sf.apply_update_layer_delta(w, dl, -1.0, d, ws)
    assert e.value.status == sf.ERR_INVALID_ARG
    with pytest.raises(sf.SlimfitError) as e:
        sf.apply_update_layer_delta(w, dl, 0.0, d, ws[:64])
    assert e.value.status == sf.ERR_WORKSPACE
    before = w[0].clone()
    sf.layer_delta_apply_run([5000], sf.F32, sf.F32, 0.0, d, ws)          # zeroed workspace: no plan
    torch.cuda.synchronize()
    assert bool(torch.isnan(d).all()) and torch.equal(w[0], before)


@pytest.mark.parametrize("ci", [0, 4])
def test_config_weights(ci):
    require_gpu()
    cfg = synth.CONFIGS[ci]
    prev, cur = synth.weight_units(cfg, device="cuda", n_blocks=min(cfg.n_blocks, 2))
    delta = cur if cfg.delta_given else [c - p.float() for p, c in zip(prev, cur)]
    _run_both(prev, delta)
