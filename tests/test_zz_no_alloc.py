"""slimfit_layer_delta_static (the entry point that allocates nothing) against slimfit_layer_delta, through the
C ABI: same kernels on the library's fixed scratch array, so the scores must be bit-identical.  Two calls in a
row, the second on a smaller model, so that what the first left in the array is there to trip over."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2305_18513_amd import binding as sf
from paper_2305_18513_amd import synth
from tests.gpu_util import require_gpu

pytestmark = pytest.mark.gpu


def _both(prev, cur, is_delta, eps=0.0):
    L = len(prev)
    numel = [t.numel() for t in prev]
    ws = torch.empty(sf.layer_delta_workspace(numel), dtype=torch.uint8, device="cuda")
    want = torch.full((L,), -1.0, device="cuda")
    got = torch.full((L,), -2.0, device="cuda")
    sf.layer_delta(prev, cur, is_delta, eps, want, ws)
    sf.layer_delta_static(prev, cur, is_delta, eps, got)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got.cpu().numpy().view(np.uint32), want.cpu().numpy().view(np.uint32))
    return got.cpu().numpy()


def test_static_scratch_matches_the_workspace_entry_point_twice_in_a_row():
    require_gpu()
    cfg = synth.CONFIGS[1]                                   # 96 layers, 85 M weights: 5 200 partial sums
    prev, cur = synth.weight_units(cfg, "cuda")
    first = _both(prev, cur, False)
    assert np.isfinite(first).all() and (first > 0).all()
    small_prev, small_cur = synth.weight_units(synth.CONFIGS[0], "cuda")     # 16 layers, 0.4 M weights
    second = _both(small_prev, small_cur, False)
    od = ref.layer_delta([t.cpu().numpy() for t in small_prev], [t.cpu().numpy() for t in small_cur])
    np.testing.assert_allclose(second, od, rtol=1e-6, atol=0)
    # bf16 weights with fp32 updates, ragged sizes, an empty layer; then the first model again
    g = torch.Generator(device="cuda").manual_seed(11)
    sizes = [1, 16385, 0, 70001, 5]
    wp = [(torch.randn(n, generator=g, device="cuda") * 0.02 + 0.001).to(torch.bfloat16) for n in sizes]
    dl = [torch.randn(n, generator=g, device="cuda") * 1e-4 for n in sizes]
    _both(wp, dl, True, eps=1e-8)
    again = _both(prev, cur, False)
    np.testing.assert_array_equal(again.view(np.uint32), first.view(np.uint32))


def test_static_scratch_rejects_what_does_not_fit():
    require_gpu()
    # 2^40 weights in one layer would need 2^26 partial sums: far beyond the fixed array; nothing is launched
    numel = np.array([1 << 40], dtype=np.int64)
    d = torch.zeros(1, device="cuda")
    import ctypes as C
    ptrs = (C.c_void_p * 1)(d.data_ptr())
    rc = sf.lib().slimfit_layer_delta_static(ptrs, C.c_int32(sf.F32), ptrs, C.c_int32(sf.F32), C.c_int32(0),
                                             C.c_void_p(numel.ctypes.data), C.c_int32(1), C.c_float(0.0),
                                             C.c_void_p(d.data_ptr()), C.c_void_p(0))
    assert rc == sf.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert float(d[0]) == 0.0
