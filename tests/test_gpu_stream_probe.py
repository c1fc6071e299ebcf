"""GPU check of the diagnostic streaming kernel: every output element is what the header states for its source
vector (the vector, pair sums, the sum, or the sum's upper bits), for full workgroups and ragged tails.  It computes
nothing of the method; the expected values are plain torch additions in the same order, so the comparison is bit for
bit."""
import pytest
import torch

from paper_2305_18513_amd import binding as sf
from tests.gpu_util import Guarded, require_gpu

pytestmark = pytest.mark.gpu


def _expected(src, ratio):
    v = src.view(-1, 4)
    if ratio == 1:
        return v.reshape(-1).view(torch.uint8)
    if ratio == 2:
        return torch.stack([v[:, 0] + v[:, 1], v[:, 2] + v[:, 3]], dim=1).reshape(-1).view(torch.uint8)
    s = ((v[:, 0] + v[:, 1]) + v[:, 2]) + v[:, 3]
    if ratio == 4:
        return s.contiguous().view(torch.uint8)
    bits = s.contiguous().view(torch.int32)
    if ratio == 8:
        return (bits >> 16).to(torch.int16).view(torch.uint8)
    return (bits >> 24).to(torch.int8).view(torch.uint8)


@pytest.mark.parametrize("ratio", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("in_vecs", [1, 255, 1024, 1000, 1024 * 37 + 3])
def test_every_vector_becomes_its_share_of_bytes(ratio, in_vecs):
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(ratio * 1000 + in_vecs)
    src = torch.randn(in_vecs * 4, device="cuda", generator=g)
    dst = Guarded(in_vecs * (16 // ratio), torch.uint8)
    sf.stream_probe(src, dst.t, ratio)
    torch.cuda.synchronize()
    assert torch.equal(dst.t, _expected(src, ratio))
    dst.check()


def test_destination_too_short_is_refused():
    require_gpu()
    src = torch.zeros(1024 * 4, device="cuda")
    dst = torch.zeros(1024 * 2 - 1, dtype=torch.uint8, device="cuda")
    with pytest.raises(ValueError):
        sf.stream_probe(src, dst, 8)
