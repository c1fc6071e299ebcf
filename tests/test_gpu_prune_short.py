"""GPU parity of slimfit_prune_scores on short rows that keep few entries (the kernel with several rows per
wavefront): every route of it -- keys that carry the column, the exact route for rows whose cut cannot be
told from 24 value bits, signed keys -- against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

from paper_2305_18513_amd import binding as sf
from tests.gpu_util import require_gpu
from tests.test_gpu_prune import _run_both

pytestmark = pytest.mark.gpu

ROWS = [1, 15, 16, 17, 31, 32, 33, 64, 1000, 1037]
COLS_K = [(1, 1), (2, 1), (3, 3), (5, 2), (16, 4), (17, 9), (63, 6), (64, 6), (65, 7), (100, 9), (128, 9),
          (197, 9), (197, 1), (199, 5), (250, 8), (255, 9), (256, 9), (256, 2)]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("cols,k", COLS_K)
def test_shapes_and_ragged_row_counts(cols, k, dtype):
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(cols * 131 + k)
    for rows in ROWS:
        p = torch.softmax(torch.randn(rows, cols, generator=g, device="cuda") * 0.5, dim=-1).to(dtype)
        _run_both(p, k, restore=False)
        _run_both(p, k, mode=sf.PRUNE_THRESHOLD, tau=1.3 / cols, restore=False)


@pytest.mark.parametrize("cols,k", [(197, 9), (128, 12), (250, 16), (64, 13), (33, 16)])
def test_bf16_keeps_up_to_sixteen(cols, k):
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(cols + k)
    p = torch.softmax(torch.randn(333, cols, generator=g, device="cuda") * 0.3, dim=-1).to(torch.bfloat16)   # many ties
    _run_both(p, k)
    _run_both(p, k, mode=sf.PRUNE_THRESHOLD, tau=1.0 / cols)


@pytest.mark.parametrize("k", [1, 4, 9])
def test_fp32_cut_inside_one_bucket_of_24_bits(k):
    """Entries that agree in their upper 24 bits and differ below: only the full 32-bit images order them."""
    require_gpu()
    cols, rows = 197, 70
    g = torch.Generator(device="cuda").manual_seed(k)
    low = torch.randint(0, 256, (rows, cols), generator=g, device="cuda", dtype=torch.int32)
    base = torch.full((rows, cols), 0x3C000000, dtype=torch.int32, device="cuda")       # 2^-7 and the 255 floats above it
    p = (base + low).view(torch.float32).clone()
    p[10:20, ::3] *= 0.5                                            # some entries far below the bucket
    p[20:30, 5] = 1.0                                               # one far above
    p[30:40] = p[30:40, :1]                                         # constant rows
    p[40:50, 100:] = p[40:50, 99:100]                               # long runs of equal entries across lanes
    _run_both(p, k)
    tau = float(torch.tensor(0x3C000080, dtype=torch.int32).view(torch.float32))        # a threshold inside the bucket
    _run_both(p, k, mode=sf.PRUNE_THRESHOLD, tau=tau)
    _run_both(-p, k)                                                # the same among negative entries
    _run_both(-p, k, mode=sf.PRUNE_THRESHOLD, tau=-tau)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("cols,k", [(197, 9), (64, 6), (130, 3)])
def test_signs_zeros_and_ties(cols, k, dtype):
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(cols + 7 * k)
    p = torch.randn(200, cols, generator=g, device="cuda")
    p[0:20] = -p[0:20].abs()                                        # all negative
    p[20:40] = (p[20:40] * 2).round() / 2                           # few distinct values, both signs
    p[40:50] = 0.0
    p[40:50, ::2] = -0.0                                            # +0 and -0 tie; the kept bits must be the entry's own
    p[50:60] = -0.0
    p[60:70, : cols // 2] = 0.0                                     # zeros at the cut below a few positive entries
    p[60:70, 0] = 1.0
    p[70:80] = p[70:80].abs() * 1e-41                               # denormals (fp32); flushed to zero patterns in bf16
    p[80:90] = -1.5
    p[90:100, 3] = float("inf")
    p[100:110, 4] = float("-inf")
    p = p.to(dtype)
    _run_both(p, k)
    _run_both(p, k, mode=sf.PRUNE_THRESHOLD, tau=0.0)
    _run_both(p, k, mode=sf.PRUNE_THRESHOLD, tau=-0.0)
    _run_both(p, k, mode=sf.PRUNE_THRESHOLD, tau=-0.75)
    _run_both(p, k, mode=sf.PRUNE_THRESHOLD, tau=0.5)


def test_misaligned_rows_take_the_other_kernel_and_agree():
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(5)
    base = torch.softmax(torch.randn(77, 197, generator=g, device="cuda"), dim=-1)
    flat = torch.empty(77 * 197 + 1, device="cuda")
    flat[1:] = base.reshape(-1)
    p = flat[1:].view(77, 197)
    assert p.data_ptr() % 16 != 0
    vals = torch.empty(77, 9, device="cuda")
    idx = torch.empty(77, 9, dtype=torch.uint16, device="cuda")
    vals2, idx2 = torch.empty_like(vals), torch.empty_like(idx)
    sf.prune_scores(p, 9, sf.PRUNE_TOPK, 0.0, vals, idx, None)
    sf.prune_scores(base, 9, sf.PRUNE_TOPK, 0.0, vals2, idx2, None)
    torch.cuda.synchronize()
    assert torch.equal(vals, vals2) and torch.equal(idx.view(torch.int16), idx2.view(torch.int16))
