"""Helpers shared by the GPU parity tests (marshalling only)."""
import numpy as np
import pytest
import torch

from paper_2305_18513_amd import binding as sf


def require_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU in this container")
    if not sf.is_built():
        raise RuntimeError("libslimfit.so has not been built; GPU tests never fall back")
    sf.lib()


def to_np(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> host NumPy array; bf16 becomes its uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.uint16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


GUARD = 256          # sentinel bytes after every output


class Guarded:
    """An output buffer followed by sentinel bytes that must stay untouched."""

    def __init__(self, numel, dtype, device="cuda"):
        esz = torch.empty((), dtype=dtype).element_size()
        self.nbytes = numel * esz
        total = (self.nbytes + 15) // 16 * 16 + GUARD
        self.raw = torch.full((total,), 0xAB, dtype=torch.uint8, device=device)
        self.t = self.raw[: self.nbytes].view(dtype) if numel else torch.empty(0, dtype=dtype, device=device)

    def check(self):
        tail = self.raw[self.nbytes:]
        assert bool((tail == 0xAB).all()), "kernel wrote past the end of its output"
