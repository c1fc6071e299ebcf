"""GPU check of the diagnostic streaming kernel: every output vector is the sum, in order, of its ``ratio`` source
vectors (the layout the header states), for full and ragged sizes.  It computes nothing of the method; the expected
values are plain torch additions in the same order, so the comparison is bit for bit."""
import pytest
import torch

from paper_2305_18513_amd import binding as sf
from tests.gpu_util import Guarded, require_gpu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("ratio", [1, 2, 6, 16])
@pytest.mark.parametrize("out_vecs", [1, 255, 256, 1000, 256 * 37 + 3])
def test_sums_of_ratio_vectors(ratio, out_vecs):
    require_gpu()
    blocks = (out_vecs + 255) // 256
    g = torch.Generator(device="cuda").manual_seed(ratio * 1000 + out_vecs)
    src = torch.randn(blocks * 256 * ratio * 4, device="cuda", generator=g)
    dst = Guarded(out_vecs * 4, torch.float32)
    sf.stream_probe(src, dst.t, ratio)
    torch.cuda.synchronize()
    v = src.view(blocks, ratio, 256, 4)
    want = v[:, 0].clone()
    for r in range(1, ratio):
        want += v[:, r]
    want = want.reshape(-1)[: out_vecs * 4]
    assert torch.equal(dst.t, want)
    dst.check()


def test_source_too_short_is_refused():
    require_gpu()
    src = torch.zeros(256 * 4 * 5, device="cuda")
    dst = torch.zeros(256 * 4, device="cuda")
    with pytest.raises(ValueError):
        sf.stream_probe(src, dst, 6)
