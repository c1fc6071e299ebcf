"""Pins for the oracle's whole-tensor pruner (Alg. 5 as the paper states it) -- CPU only."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2305_18513_amd import synth


def _brute(x, k, by_magnitude):
    key = np.abs(x.astype(np.float64)) if by_magnitude else x.astype(np.float64).copy()
    out = []
    for _ in range(k):
        j = int(np.argmax(key))              # first maximum = lowest index among equals
        out.append(j)
        key[j] = -np.inf
    return sorted(out)


@pytest.mark.parametrize("by_mag", [True, False])
@pytest.mark.parametrize("n,k", [(1, 1), (7, 3), (64, 6), (1000, 100), (1000, 1000), (4097, 409)])
def test_equals_bruteforce_and_library_sort(n, k, by_mag):
    rng = np.random.default_rng(n + k)
    for variant in range(3):
        x = rng.standard_normal(n).astype(np.float32)
        if variant == 1:
            x = np.round(x * 2) / 2                    # heavy ties, both signs
        if variant == 2:
            x[:] = -0.75                               # all equal
        vals, idx = ref.prune_global(x, k, by_magnitude=by_mag)
        assert idx.tolist() == _brute(x, k, by_mag)
        key = np.abs(x) if by_mag else x
        lib = np.sort(np.argsort(-key.astype(np.float64), kind="stable")[:k])
        assert idx.tolist() == lib.tolist()
        np.testing.assert_array_equal(vals.view(np.uint32), x[idx].view(np.uint32))   # signed bit copies
        assert np.all(np.diff(idx) > 0)
        dropped = np.setdiff1d(np.arange(n), idx)
        if dropped.size:
            assert key[idx].min() >= key[dropped].max()


def test_count_is_int_of_ten_percent_and_sorted_prefix_multiset():
    # Alg. 5: y_s = sort(x, descending)[0 : int(numel * 0.1)]
    rng = np.random.default_rng(1)
    x = rng.standard_normal(12345).astype(np.float32)
    k = int(x.size * 0.1)
    assert k == 1234
    vals, idx = ref.prune_global(x, k, by_magnitude=False)
    np.testing.assert_array_equal(-np.sort(-vals), -np.sort(-x)[:k])
    vals_m, _ = ref.prune_global(x, k, by_magnitude=True)
    np.testing.assert_array_equal(-np.sort(-np.abs(vals_m)), -np.sort(-np.abs(x))[:k])


def test_magnitude_and_signed_orders_differ_on_signed_data():
    x = np.array([-3.0, 1.0, 2.0, -0.5, 0.25], dtype=np.float32)
    _, i_mag = ref.prune_global(x, 2, by_magnitude=True)
    _, i_sgn = ref.prune_global(x, 2, by_magnitude=False)
    assert i_mag.tolist() == [0, 2] and i_sgn.tolist() == [1, 2]
    z = np.array([-0.0, 0.0, -0.0, 0.0], dtype=np.float32)
    vals, idx = ref.prune_global(z, 2, by_magnitude=False)
    assert idx.tolist() == [0, 1] and np.signbit(vals[0]) and not np.signbit(vals[1])


def test_restore_is_zeros_plus_scatter():
    rng = np.random.default_rng(2)
    x = rng.standard_normal(5000).astype(np.float32)
    vals, idx = ref.prune_global(x, 500)
    dense = ref.restore_global(vals, idx, x.size)
    want = np.zeros_like(x)
    want[idx] = vals
    np.testing.assert_array_equal(dense, want)
    assert np.count_nonzero(dense) == 500
    np.testing.assert_array_equal(dense[idx], x[idx])
    full_v, full_i = ref.prune_global(x, x.size)
    np.testing.assert_array_equal(ref.restore_global(full_v, full_i, x.size), x)


def test_bf16_layernorm_input_with_ties():
    cfg = synth.CONFIGS[4]
    t = synth.activation(cfg, "ln_in", batch=1).reshape(-1)[:60000]
    bits = t.view(torch.int16).numpy().view(np.uint16)
    wide = t.float().numpy()
    k = int(bits.size * 0.1)
    vals, idx = ref.prune_global(bits, k, by_magnitude=True)
    _, idx32 = ref.prune_global(wide, k, by_magnitude=True)
    np.testing.assert_array_equal(idx, idx32)                  # widening is exact
    np.testing.assert_array_equal(vals, bits[idx])
    cut = np.abs(wide[idx]).min()
    assert (np.abs(wide) == cut).sum() > (np.abs(wide[idx]) == cut).sum()      # ties cross the cut
    eq_kept = idx[np.abs(wide[idx]) == cut]
    eq_all = np.flatnonzero(np.abs(wide) == cut)
    np.testing.assert_array_equal(eq_kept, eq_all[: eq_kept.size])            # lowest indices win


def test_bad_arguments_rejected():
    x = np.zeros(4, dtype=np.float32)
    for k in (0, 5):
        with pytest.raises(ValueError):
            ref.prune_global(x, k)
    with pytest.raises(ValueError):
        ref.restore_global(np.zeros(1, np.float32), np.array([9], np.int32), 4)
