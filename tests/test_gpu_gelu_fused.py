"""GPU parity: slimfit_gelu_quant_pack / slimfit_gelu_backward_dequant vs the CPU oracle.
Codes and scales are bit-identical to the unfused quantiser's; the GELU values and gradients are fp32
evaluations compared with the fp64 oracle within the tolerance the header states."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2305_18513_amd import binding as sf
from paper_2305_18513_amd import synth
from tests.gpu_util import Guarded, require_gpu, to_np

pytestmark = pytest.mark.gpu


def _wide(a):
    """NumPy fp32 or bf16 bit patterns -> float64."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def _wide_exact_gelu(xh):
    """The oracle's GELU of the widened input, before its final rounding matters: for bf16 inputs the
    oracle is asked in fp32 so that only the kernel's own output rounding is inside the tolerance."""
    if xh.dtype == np.uint16:
        return ref.gelu((xh.astype(np.uint32) << 16).view(np.float32)).astype(np.float64)
    return ref.gelu(xh).astype(np.float64)


def _check_close(got, want_f64, scale_abs, rel, bf16):
    """|got - want| <= scale_abs + rel*|want| (fp32); for bf16 one more rounding of 2^-8 relative."""
    g = _wide(got)
    tol = scale_abs + rel * np.abs(want_f64)
    if bf16:
        tol = tol + np.abs(want_f64) * 2.0 ** -8
    bad = np.abs(g - want_f64) > tol
    assert not bad.any(), "max excess %.3g at %d" % (float((np.abs(g - want_f64) - tol).max()), int(np.argmax(bad)))


def _run_both(x: torch.Tensor, dy: torch.Tensor, mode, bits, block, fb):
    n = x.numel()
    bf16 = x.dtype == torch.bfloat16
    blocked = mode == sf.Q_BLOCK
    codes = Guarded(sf.packed_bytes(n, bits), torch.uint8)
    scales = Guarded(sf.num_blocks(n, block) if blocked else 0, torch.float32)
    y = Guarded(n, x.dtype)
    dx = Guarded(n, x.dtype)
    x_before = x.clone()
    sf.gelu_quant_pack(x, mode, bits, block, fb, y.t, codes.t, scales.t if blocked else None)
    sf.gelu_backward_dequant(codes.t, scales.t if blocked else None, mode, bits, block, fb, dy, dx.t)
    torch.cuda.synchronize()
    codes.check(); scales.check(); y.check(); dx.check()
    assert torch.equal(x.view(torch.uint8), x_before.view(torch.uint8))            # the input is only read

    xh, dyh = to_np(x), to_np(dy)
    oc, osc = ref.quant_pack(xh, mode=mode, bits=bits, block=block, frac_bits=fb, threads=4)
    np.testing.assert_array_equal(to_np(codes.t), oc)
    if blocked:
        np.testing.assert_array_equal(to_np(scales.t).view(np.uint32), osc.view(np.uint32))
    xw = _wide(xh)
    _check_close(to_np(y.t), _wide_exact_gelu(xh), 4e-7 * np.abs(xw), 1e-6, bf16)
    xhat = ref.dequant_unpack(oc, osc, n, mode=mode, bits=bits, block=block, frac_bits=fb,
                              out_dtype=np.float32, threads=4)
    want_dx = _wide(ref.gelu_backward(xhat, np.ones(n, np.float32))) * _wide(dyh)
    _check_close(to_np(dx.t), want_dx, 1e-6 * np.abs(_wide(dyh)), 2e-7, bf16)


SIZES = [1, 3, 31, 64, 65, 257, 1023, 4096, 4097, 3 * 8192 + 37, 100003]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("bits,block", [(4, 64), (4, 32), (8, 128), (8, 256)])
def test_block_mode_sizes(dtype, bits, block):
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(bits * 100 + block)
    for n in SIZES:
        x = torch.randn(n, generator=g, device="cuda") * 2
        x = torch.where(torch.rand(n, generator=g, device="cuda") < 0.01, x * 10, x).to(dtype)
        dy = torch.randn(n, generator=g, device="cuda").to(dtype)
        _run_both(x, dy, sf.Q_BLOCK, bits, block, 0)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_fixed_mode_and_special_inputs(dtype):
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(9)
    n = 5000
    x = torch.randn(n, generator=g, device="cuda") * 3
    x[:12] = torch.tensor([0.0, -0.0, 1e-30, -1e-30, 40.0, -40.0, 6.0, -6.0, -0.7517916, 1.0, -1.0, 100.0])
    x = x.to(dtype)
    dy = torch.randn(n, generator=g, device="cuda").to(dtype)
    _run_both(x, dy, sf.Q_FIXED, 8, 64, 4)
    _run_both(x, dy, sf.Q_FIXED, 4, 64, 1)
    _run_both(x, dy, sf.Q_BLOCK, 4, 64, 0)


def test_argument_errors():
    require_gpu()
    x = torch.randn(4096, device="cuda")
    y = torch.empty_like(x)
    codes = torch.empty(2048, dtype=torch.uint8, device="cuda")
    scales = torch.empty(64, device="cuda")
    with pytest.raises(sf.SlimfitError) as e:
        sf.gelu_quant_pack(x, sf.Q_BLOCK, 4, 64, 0, x, codes, scales)                 # in place
    assert e.value.status == sf.ERR_INVALID_ARG
    with pytest.raises(sf.SlimfitError) as e:
        sf.gelu_backward_dequant(codes, scales, sf.Q_BLOCK, 4, 64, 0, y, y)
    assert e.value.status == sf.ERR_INVALID_ARG
    with pytest.raises(sf.SlimfitError) as e:
        sf.gelu_quant_pack(x[1:], sf.Q_BLOCK, 4, 64, 0, y[1:], codes, scales)
    assert e.value.status == sf.ERR_ALIGNMENT
    with pytest.raises(sf.SlimfitError) as e:
        sf.gelu_quant_pack(x, sf.Q_BLOCK, 5, 64, 0, y, codes, scales)
    assert e.value.status == sf.ERR_UNSUPPORTED


@pytest.mark.parametrize("ci", [1, 3, 4])
def test_gelu_input_at_full_size(ci):
    require_gpu()
    cfg = synth.CONFIGS[ci]
    x = synth.activation(cfg, "gelu_in", device="cuda").reshape(-1)
    if x.numel() > 60_000_000:
        x = x[: 60_000_000 + 37 * 64].contiguous()          # the oracle's GELU is scalar C: keep it to seconds
    g = torch.Generator(device="cuda").manual_seed(ci)
    dy = torch.randn(x.numel(), generator=g, device="cuda").to(x.dtype)
    _run_both(x, dy, sf.Q_BLOCK, cfg.quant_bits[-1], cfg.quant_block, 0)
