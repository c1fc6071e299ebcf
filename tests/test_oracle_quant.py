"""Pins for the oracle's quantiser (Alg. 2, Sec. 4/5, App. on conversion) -- CPU only."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2305_18513_amd import synth


def _f32(a):
    return np.asarray(a, dtype=np.float32)


def _unpack(codes, n, bits):
    """Independent decoder used by the pins (byte-level definition)."""
    if bits == 8:
        return codes[:n].view(np.int8).astype(np.int32)
    lo = (codes & 0xF).astype(np.int32)
    hi = (codes >> 4).astype(np.int32)
    both = np.stack([lo, hi], axis=1).reshape(-1)[:n]
    return np.where(both >= 8, both - 16, both)


def _alg2_exact(x, ib, fb):
    """Alg. 2 in exact rational arithmetic; Python rounds halves to even."""
    out = []
    for v in x:
        q = Fraction(float(v)) * Fraction(2) ** fb
        r = round(q)
        out.append(min(max(r, -2 ** (fb + ib - 1)), 2 ** (fb + ib - 1) - 1))
    return np.array(out, dtype=np.int32)


def _grid(fb):
    step = 2.0 ** -fb
    pts = [0.0, -0.0, 1e-45, -1e-45, 1e-39, 3e38, -3e38, 0.03125, 0.09375,
           -0.03125, -0.09375]
    for kk in range(-140, 141):
        base = kk * step
        pts += [base, base + step / 2, base + step / 2 * (1 + 2 ** -20),
                base + step / 2 * (1 - 2 ** -20), base - step / 4]
    return _f32(pts)


@pytest.mark.parametrize("ib,fb", [(4, 4), (8, 0), (1, 7), (2, 2), (3, 1), (4, 0)])
def test_fixed_mode_matches_alg2_in_exact_arithmetic(ib, fb):
    bits = ib + fb
    x = _grid(fb)
    codes, scales = ref.quant_pack(x, mode=ref.Q_FIXED, bits=bits, frac_bits=fb)
    assert scales is None
    np.testing.assert_array_equal(_unpack(codes, x.size, bits), _alg2_exact(x, ib, fb))


def test_fixed_8bit_4p4_format_range_and_step():
    # Sec. 4: 8 bits, 4 integer + 4 fractional  ->  [-8, 7.9375], step 1/16
    x = _f32([-100, -8, -7.97, 0.03, 0.04, 7.9375, 7.97, 100, 0.03125, 0.09375])
    codes, _ = ref.quant_pack(x, mode=ref.Q_FIXED, bits=8, frac_bits=4)
    y = ref.dequant_unpack(codes, None, x.size, mode=ref.Q_FIXED, bits=8, frac_bits=4)
    np.testing.assert_array_equal(
        y, _f32([-8, -8, -8, 0, 0.0625, 7.9375, 7.9375, 7.9375, 0.0, 0.125]))


def test_fixed_half_step_bound_in_range_and_idempotence():
    rng = np.random.default_rng(0)
    for bits, fb in ((8, 4), (4, 2), (4, 0), (8, 7)):
        qmax = 2 ** (bits - 1) - 1
        hi = qmax / 2.0 ** fb
        lo = -(qmax + 1) / 2.0 ** fb
        x = _f32(rng.uniform(lo, hi, 20000))
        c, _ = ref.quant_pack(x, mode=ref.Q_FIXED, bits=bits, frac_bits=fb)
        y = ref.dequant_unpack(c, None, x.size, mode=ref.Q_FIXED, bits=bits, frac_bits=fb)
        assert np.max(np.abs(x.astype(np.float64) - y)) <= 2.0 ** -fb / 2
        c2, _ = ref.quant_pack(y, mode=ref.Q_FIXED, bits=bits, frac_bits=fb)
        np.testing.assert_array_equal(c, c2)


def test_pack_layout_and_all_code_values():
    # 8-bit: byte j is the two's-complement code of element j
    x = _f32(np.arange(-128, 128))
    c, _ = ref.quant_pack(x, mode=ref.Q_FIXED, bits=8, frac_bits=0)
    np.testing.assert_array_equal(c, np.arange(-128, 128).astype(np.int8).view(np.uint8))
    np.testing.assert_array_equal(
        ref.dequant_unpack(c, None, 256, mode=ref.Q_FIXED, bits=8, frac_bits=0), x)
    # 4-bit: two codes per byte by shifts, even element in the low nibble
    c, _ = ref.quant_pack(_f32([1, -1, -8, 7, 3]), mode=ref.Q_FIXED, bits=4, frac_bits=0)
    assert c.tolist() == [0xF1, 0x78, 0x03]          # odd tail: high nibble 0
    # every (low, high) pair round-trips, i.e. all 256 byte values
    lo, hi = np.meshgrid(np.arange(-8, 8), np.arange(-8, 8), indexing="ij")
    x = _f32(np.stack([lo.reshape(-1), hi.reshape(-1)], axis=1).reshape(-1))
    c, _ = ref.quant_pack(x, mode=ref.Q_FIXED, bits=4, frac_bits=0)
    assert sorted(c.tolist()) == list(range(256))
    np.testing.assert_array_equal(
        ref.dequant_unpack(c, None, x.size, mode=ref.Q_FIXED, bits=4, frac_bits=0), x)
    # decoding any byte gives sign-extended nibbles
    allb = np.arange(256, dtype=np.uint8)
    y = ref.dequant_unpack(allb, None, 512, mode=ref.Q_FIXED, bits=4, frac_bits=0)
    np.testing.assert_array_equal(y, _unpack(allb, 512, 4).astype(np.float32))


def test_dequant_is_code_over_two_to_fb():
    allb = np.arange(256, dtype=np.uint8)
    for fb in (0, 1, 4, 7):
        y = ref.dequant_unpack(allb, None, 256, mode=ref.Q_FIXED, bits=8, frac_bits=fb)
        np.testing.assert_array_equal(y, allb.view(np.int8).astype(np.float64) / 2.0 ** fb)


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("block", [32, 64, 128, 256])
def test_block_mode_invariants(bits, block):
    rng = np.random.default_rng(bits * 1000 + block)
    n = 5 * block + 37                                  # ragged last block
    x = _f32(rng.standard_normal(n))
    x[rng.random(n) < 0.01] *= 20
    qmax = 2 ** (bits - 1) - 1
    c, s = ref.quant_pack(x, mode=ref.Q_BLOCK, bits=bits, block=block)
    q = _unpack(c, n, bits)
    y = ref.dequant_unpack(c, s, n, mode=ref.Q_BLOCK, bits=bits, block=block)
    assert s.size == -(-n // block) and c.size == (n * bits + 7) // 8
    assert q.min() >= -qmax and q.max() <= qmax         # -qmax-1 is never produced
    for b in range(s.size):
        sl = slice(b * block, min(n, (b + 1) * block))
        xb, qb, yb = x[sl].astype(np.float64), q[sl], y[sl].astype(np.float64)
        a = np.abs(xb).max()
        assert s[b] == np.float32(a) / np.float32(qmax)   # one fp32 division
        # round-trip error at most half a quantisation step
        # half a step, plus the four fp32 roundings (inv, product, scale, dequantising
        # multiply) acting on a value of at most qmax steps
        assert np.max(np.abs(xb - yb)) <= float(s[b]) * (0.5 + qmax * 2.0 ** -22 * 1.01)
        # the largest-magnitude element maps to +-qmax and back to +-qmax*scale
        j = int(np.argmax(np.abs(xb)))
        assert abs(qb[j]) == qmax and yb[j] == np.float32(qb[j]) * s[b]
        # monotone inside a block
        order = np.argsort(xb, kind="stable")
        assert np.all(np.diff(qb[order]) >= 0)
        # dequantised value is code * scale, one fp32 multiply
        np.testing.assert_array_equal(y[sl], qb.astype(np.float32) * s[b])


def test_block_mode_against_numpy_float32_library_ops():
    rng = np.random.default_rng(11)
    x = _f32(rng.standard_normal(64 * 200) * rng.lognormal(0, 2, 64 * 200))
    for bits in (4, 8):
        qmax = np.float32(2 ** (bits - 1) - 1)
        xb = x.reshape(-1, 64)
        a = np.abs(xb).max(axis=1, keepdims=True)
        inv = qmax / a
        want = np.clip(np.rint(xb * inv), -qmax - 1, qmax).astype(np.int32)
        c, s = ref.quant_pack(x, mode=ref.Q_BLOCK, bits=bits, block=64)
        np.testing.assert_array_equal(_unpack(c, x.size, bits), want.reshape(-1))
        np.testing.assert_array_equal(s, (a / qmax).reshape(-1))


def test_block_mode_reduces_to_alg2_when_absmax_is_qmax_times_power_of_two():
    rng = np.random.default_rng(12)
    for bits, m in ((8, -4), (4, -2), (8, 0), (4, 1)):
        qmax = 2 ** (bits - 1) - 1
        a = qmax * 2.0 ** m
        x = _f32(rng.uniform(-a, a, 64))
        x[17] = a
        cb, s = ref.quant_pack(x, mode=ref.Q_BLOCK, bits=bits, block=64)
        cf, _ = ref.quant_pack(x, mode=ref.Q_FIXED, bits=bits, frac_bits=-m)
        np.testing.assert_array_equal(cb, cf)
        assert s[0] == 2.0 ** m


def test_degenerate_blocks():
    x = np.zeros(130, dtype=np.float32)
    x[64:128] = 1e-39                                   # 127/1e-39 overflows fp32
    x[128:] = [-0.0, 0.0]
    c, s = ref.quant_pack(x, mode=ref.Q_BLOCK, bits=8, block=64)
    assert not c.any() and s.tolist() == [0.0, 0.0, 0.0]
    y = ref.dequant_unpack(c, s, 130, mode=ref.Q_BLOCK, bits=8, block=64)
    assert not y.any()
    # a tiny but representable block still quantises (4-bit: 7/1e-37 is finite)
    x = _f32(np.linspace(-1e-37, 1e-37, 64))
    c, s = ref.quant_pack(x, mode=ref.Q_BLOCK, bits=4, block=64)
    assert s[0] > 0 and _unpack(c, 64, 4).max() == 7


def test_bf16_io():
    rng = np.random.default_rng(13)
    t = torch.from_numpy(_f32(rng.standard_normal(32 * 9 + 5))).to(torch.bfloat16)
    bits16 = t.view(torch.int16).numpy().view(np.uint16)
    wide = t.float().numpy()
    c1, s1 = ref.quant_pack(bits16, mode=ref.Q_BLOCK, bits=4, block=32)
    c2, s2 = ref.quant_pack(wide, mode=ref.Q_BLOCK, bits=4, block=32)
    np.testing.assert_array_equal(c1, c2)
    np.testing.assert_array_equal(s1, s2)
    y32 = ref.dequant_unpack(c1, s1, wide.size, mode=ref.Q_BLOCK, bits=4, block=32)
    y16 = ref.dequant_unpack(c1, s1, wide.size, mode=ref.Q_BLOCK, bits=4, block=32,
                             out_dtype=np.uint16)
    want = torch.from_numpy(y32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(y16, want)           # fp32 -> bf16 nearest-even


def test_empty_and_tiny_sizes():
    for n in (0, 1, 2, 3):
        x = _f32(np.linspace(-1, 1, n))
        for bits in (4, 8):
            c, s = ref.quant_pack(x, mode=ref.Q_BLOCK, bits=bits, block=32)
            assert c.size == (n * bits + 7) // 8 and s.size == (1 if n else 0)
            y = ref.dequant_unpack(c, s, n, mode=ref.Q_BLOCK, bits=bits, block=32)
            assert y.size == n


def test_bad_arguments_rejected():
    x = _f32([1, 2, 3])
    with pytest.raises(ValueError):
        ref.quant_pack(x, bits=5)
    with pytest.raises(ValueError):
        ref.quant_pack(x, block=48)
    with pytest.raises(ValueError):
        ref.quant_pack(x, mode=2)


def test_synthetic_activation_recipe():
    cfg = synth.CONFIGS[0]
    x = synth.activation(cfg, "gelu_in")
    assert tuple(x.shape) == (4, 64, 512) and x.numel() == cfg.gelu_in_numel
    assert abs(float(x.std()) - 1.18) < 0.1            # N(0,1) + 0.1 % x20 outliers
    assert float(x.abs().max()) > 20
    assert torch.equal(x, synth.activation(cfg, "gelu_in"))       # seeded
    assert not torch.equal(x, synth.activation(cfg, "gelu_in", block=1))
    v = synth.CONFIGS[2]
    xt = synth.activation(v, "ln_in", batch=2)
    assert tuple(xt.shape) == (2, 197, 768)
    per_chan = xt.abs().amax(dim=(0, 1))
    assert int((per_chan > 8).sum()) <= 7 + 2          # only the heavy-tailed channels
    b = synth.activation(synth.CONFIGS[4], "ln_in", batch=1)
    assert b.dtype == torch.bfloat16
