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


@pytest.mark.parametrize("in_vecs", [1, 255, 1024, 1000, 1024 * 37 + 3])
def test_read_only_probe_sums_every_wavefront(in_vecs):
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(in_vecs)
    src = torch.randn(in_vecs * 4, device="cuda", generator=g)
    dst = Guarded(sf.stream_probe_bytes(in_vecs, 0) // 4, torch.float32)
    sf.stream_probe(src, dst.t, 0)
    torch.cuda.synchronize()
    dst.check()
    blocks = (in_vecs + 1023) // 1024
    v = torch.zeros(blocks * 1024, 4, device="cuda")
    v[:in_vecs] = src.view(-1, 4)
    s = ((v[:, 0] + v[:, 1]) + v[:, 2]) + v[:, 3]                   # per vector, the header's order
    lanes = torch.zeros(blocks, 256, device="cuda")
    for j in range(4):                                              # thread t of workgroup b: vectors b*1024 + t + 256*j
        lanes = lanes + s.view(blocks, 4, 256)[:, j]
    w = lanes.view(blocks, 4, 64)                                   # wavefront g: threads 64*g .. 64*g + 63
    for off in (32, 16, 8, 4, 2, 1):                                # butterfly: every lane adds its partner's value
        w = w + w[:, :, torch.arange(64, device="cuda") ^ off]
    assert torch.equal(dst.t.view(blocks, 4), w[:, :, 0])


@pytest.mark.parametrize("ratio", [-2, -4, -8])
@pytest.mark.parametrize("in_vecs", [1, 255, 1024, 1000, 1024 * 37 + 3])
def test_growing_probe_writes_m_vectors_per_vector(ratio, in_vecs):
    require_gpu()
    m = -ratio
    g = torch.Generator(device="cuda").manual_seed(in_vecs + m)
    src = torch.randn(in_vecs * 4, device="cuda", generator=g)
    dst = Guarded(sf.stream_probe_bytes(in_vecs, ratio) // 4, torch.float32)
    sf.stream_probe(src, dst.t, ratio)
    torch.cuda.synchronize()
    dst.check()
    words = src.view(torch.int16).to(torch.int32) & 0xFFFF                             # the source as unsigned 16-bit words
    s = words.view(in_vecs * m, 8 // m).sum(dim=1).to(torch.float32)                  # exact: at most 4 * 65535
    want = s.view(-1, 1) + torch.arange(4, device="cuda", dtype=torch.float32).view(1, 4)
    assert torch.equal(dst.t.view(in_vecs * m, 4), want)
