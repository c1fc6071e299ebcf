"""Pins for the oracle's Eq. 1 (training-dynamics distance) -- CPU only."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2305_18513_amd import synth


def _f32(a):
    return np.asarray(a, dtype=np.float32)


def test_identical_weights_give_exact_zero_even_at_zero_weight():
    w = _f32([0.0, -0.0, 1.5, -3e-5, 1e-40])
    assert ref.layer_delta([w], [w.copy()])[0] == 0.0


def test_uniform_relative_change_is_recovered_exactly():
    rng = np.random.default_rng(1)
    w = _f32(rng.standard_normal(4099) * 0.02)
    w = (w.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)   # 8-bit mantissa
    for m in (1, 4, 9, 12):
        cur = _f32(w * np.float32(1 + 2.0 ** -m))     # exact in fp32
        assert np.all(cur.astype(np.float64) == w.astype(np.float64) * (1 + 2.0 ** -m))
        assert ref.layer_delta([w], [cur])[0] == np.float32(2.0 ** -m)


def test_denominator_is_previous_weight_not_current():
    w_prev = _f32(np.ones(10))
    w_cur = _f32(np.full(10, 2.0))
    assert ref.layer_delta([w_prev], [w_cur])[0] == 1.0      # 0.5 if divided by W^t
    assert ref.layer_delta([w_cur], [w_prev])[0] == 0.5


def test_unit_previous_weight_reduces_to_mean_abs_delta():
    rng = np.random.default_rng(2)
    delta = _f32(rng.standard_normal(10007) * 1e-3)
    ones = _f32(np.ones_like(delta))
    got = ref.layer_delta([ones], [delta], cur_is_delta=True)[0]
    want = np.linalg.norm(delta.astype(np.float64), 1) / delta.size
    assert abs(got - want) <= 1e-7 * want


def test_against_float64_one_liner_on_small_tensors():
    rng = np.random.default_rng(3)
    for n in (1, 2, 63, 64, 65, 1000):
        wp = _f32(rng.standard_normal(n) * 0.02)
        wc = _f32(wp + rng.standard_normal(n) * 1e-4)
        a, b = wp.astype(np.float64), wc.astype(np.float64)
        want = np.mean(np.abs((b - a) / a))
        got = ref.layer_delta([wp], [wc])[0]
        assert abs(got - want) <= 1e-7 * want


def test_mean_not_sum_and_per_layer_independence():
    rng = np.random.default_rng(4)
    wp = _f32(rng.standard_normal(512) * 0.02)
    wc = _f32(wp * np.float32(1.5))
    d1 = ref.layer_delta([wp], [wc])[0]
    d2 = ref.layer_delta([np.tile(wp, 3)], [np.tile(wc, 3)])[0]
    assert d1 == d2 == 0.5
    # several layers in one call: each equals its own single-layer call
    layers_p = [_f32(rng.standard_normal(n) * 0.02) for n in (5, 300, 1, 77)]
    layers_c = [_f32(p + rng.standard_normal(p.size) * 1e-5) for p in layers_p]
    all_d = ref.layer_delta(layers_p, layers_c, threads=4)
    for i in range(4):
        assert all_d[i] == ref.layer_delta([layers_p[i]], [layers_c[i]])[0]


def test_sign_flip_power_of_two_scaling_and_permutation():
    rng = np.random.default_rng(5)
    wp = _f32(rng.standard_normal(2000) * 0.02)
    wc = _f32(wp + rng.standard_normal(2000) * 1e-4)
    base = ref.layer_delta([wp], [wc])[0]
    assert ref.layer_delta([-wp], [-wc])[0] == base
    assert ref.layer_delta([wp * 8], [wc * 8])[0] == base
    perm = rng.permutation(2000)
    assert abs(ref.layer_delta([wp[perm]], [wc[perm]])[0] - base) <= 2e-7 * base


def test_delta_form_equals_difference_form():
    rng = np.random.default_rng(6)
    # values on a coarse binary grid so that W^t = W^{t-1} + delta is exact
    wp = _f32(rng.integers(1, 4000, 1000) * rng.choice([-1, 1], 1000) / 1024.0)
    delta = _f32(rng.integers(-40, 41, 1000) / 1024.0)
    wc = _f32(wp + delta)
    assert np.all(wc.astype(np.float64) == wp.astype(np.float64) + delta.astype(np.float64))
    assert (ref.layer_delta([wp], [delta], cur_is_delta=True)[0]
            == ref.layer_delta([wp], [wc])[0])


def test_zero_previous_weight_and_eps_floor():
    wp = _f32([0.0, 1.0])
    wc = _f32([0.5, 1.0])
    with np.errstate(all="ignore"):
        assert np.isinf(ref.layer_delta([wp], [wc])[0])
    assert ref.layer_delta([wp], [wc], eps=0.25)[0] == 1.0    # (0.5/0.25 + 0)/2
    # eps never lowers a denominator that is already larger
    assert ref.layer_delta([_f32([2.0])], [_f32([3.0])], eps=0.25)[0] == 0.5


def test_bf16_inputs_are_widened_exactly():
    rng = np.random.default_rng(7)
    t = torch.from_numpy(_f32(rng.standard_normal(777) * 0.02)).to(torch.bfloat16)
    bits = t.view(torch.int16).numpy().view(np.uint16)
    wide = t.float().numpy()
    delta = _f32(rng.standard_normal(777) * 1e-4)
    assert (ref.layer_delta([bits], [delta], cur_is_delta=True)[0]
            == ref.layer_delta([wide], [delta], cur_is_delta=True)[0])


def test_empty_layer_and_no_layers():
    e = np.zeros(0, dtype=np.float32)
    assert ref.layer_delta([e], [e])[0] == 0.0
    assert ref.layer_delta([], []).size == 0


def test_synthetic_units_have_paper_layer_list_shape():
    cfg = synth.CONFIGS[0]
    prev, cur = synth.weight_units(cfg)
    assert len(prev) == cfg.n_units == 16
    assert [p.numel() for p in prev[:8]] == [128 * 128] * 4 + [128, 128 * 512, 512 * 128, 128]
    d = ref.layer_delta([p.numpy() for p in prev], [c.numpy() for c in cur], threads=2)
    assert np.all(np.isfinite(d)) and np.all(d > 0)
    assert [c.n_freeze for c in synth.CONFIGS] == [15, 91, 91, 182, 182]         # stated with the workloads
    assert [ref.freeze_count(c.n_units, c.freeze_rate) for c in synth.CONFIGS] == [c.n_freeze for c in synth.CONFIGS]


def test_negative_eps_rejected():
    w = _f32([1.0])
    with pytest.raises(ValueError):
        ref.layer_delta([w], [w], eps=-1.0)


# ---- the score measured while the update is applied ---------------------------------------------------------------

def test_apply_update_new_weights_are_one_fp32_addition():
    rng = np.random.default_rng(21)
    ws = [_f32(rng.standard_normal(n) * 0.02) for n in (1, 7, 4099)]
    ds = [_f32(rng.standard_normal(w.size) * 1e-4) for w in ws]
    d, new = ref.apply_update_layer_delta(ws, ds)
    for w, dl, nw in zip(ws, ds, new):
        np.testing.assert_array_equal(nw.view(np.uint32), (w + dl).view(np.uint32))        # NumPy float32 addition
    np.testing.assert_array_equal(d, ref.layer_delta(ws, ds, cur_is_delta=True))
    # hand value: |0.5/2| and |-1/4| -> mean 0.25; new weights 2.5 and 3
    d, new = ref.apply_update_layer_delta([_f32([2.0, 4.0])], [_f32([0.5, -1.0])])
    assert d[0] == np.float32(0.25) and new[0].tolist() == [2.5, 3.0]


def test_apply_update_agrees_with_the_two_tensor_form_when_the_addition_is_exact():
    rng = np.random.default_rng(22)
    w = _f32(rng.integers(1, 1000, 5000)) / np.float32(64)          # few mantissa bits: w + delta is exact
    dl = _f32(rng.integers(-50, 50, 5000)) / np.float32(64)
    d, new = ref.apply_update_layer_delta([w], [dl])
    assert np.all(new[0].astype(np.float64) == w.astype(np.float64) + dl.astype(np.float64))
    assert d[0] == ref.layer_delta([w], [new[0]])[0]


def test_apply_update_bf16_weights_round_once_more():
    rng = np.random.default_rng(23)
    w32 = _f32(rng.standard_normal(3000) * 0.02)
    wb = torch.from_numpy(w32).to(torch.bfloat16)
    dl = _f32(rng.standard_normal(3000) * 1e-3)
    wbits = wb.view(torch.int16).numpy().view(np.uint16)
    d, new = ref.apply_update_layer_delta([wbits], [dl])
    want = (wb.float() + torch.from_numpy(dl)).to(torch.bfloat16)                           # library rounding
    np.testing.assert_array_equal(new[0], want.view(torch.int16).numpy().view(np.uint16))
    np.testing.assert_array_equal(d, ref.layer_delta([wbits], [dl], cur_is_delta=True))
    # inputs untouched
    np.testing.assert_array_equal(wbits, wb.view(torch.int16).numpy().view(np.uint16))


def test_apply_update_bad_arguments_and_empty():
    d, new = ref.apply_update_layer_delta([], [])
    assert d.size == 0 and new == []
    d, new = ref.apply_update_layer_delta([_f32([])], [_f32([])])
    assert new[0].size == 0
    with pytest.raises(ValueError):
        ref.apply_update_layer_delta([_f32([1.0])], [_f32([1.0])], eps=-1.0)
