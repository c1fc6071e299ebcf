"""Pins for the oracle's fused softmax + per-row pruning (the attention probabilities that Alg. 5
prunes) -- CPU only."""
import numpy as np
import pytest
from scipy import special

from oracle import ref


def _rows(seed, rows, cols, scale=1.0):
    return (np.random.default_rng(seed).standard_normal((rows, cols)) * scale).astype(np.float32)


@pytest.mark.parametrize("rows,cols,k", [(1, 1, 1), (5, 7, 3), (33, 197, 9), (9, 384, 38), (3, 1025, 100)])
def test_probabilities_match_library_softmax(rows, cols, k):
    l = _rows(rows + cols, rows, cols, 3.0)
    p, vals, idx = ref.softmax_prune(l, k)
    want = special.softmax(l.astype(np.float64), axis=1)
    np.testing.assert_allclose(p.astype(np.float64), want, rtol=1.2e-7, atol=1e-45)      # one rounding to fp32
    np.testing.assert_allclose(p.astype(np.float64).sum(1), 1.0, rtol=0, atol=cols * 6e-8)
    np.testing.assert_array_equal(vals, np.take_along_axis(p, idx.astype(np.int64), axis=1))


def test_shift_invariance_and_uniform_row():
    l = _rows(3, 6, 50)
    p0, v0, i0 = ref.softmax_prune(l, 5)
    p1, v1, i1 = ref.softmax_prune(l + np.float32(8.0), 5)
    np.testing.assert_allclose(p1, p0, rtol=2e-6)               # the shifted logits are re-rounded to fp32, hence loosely
    u, vu, iu = ref.softmax_prune(np.full((2, 40), -3.25, np.float32), 4)
    np.testing.assert_array_equal(u, np.float32(1.0 / 40))
    assert iu.tolist() == [[0, 1, 2, 3]] * 2                    # ties -> lowest columns


def test_kept_set_is_the_pruners_on_the_logits_and_on_the_exact_probabilities():
    l = _rows(5, 40, 197, 2.0)
    l[3] = np.round(l[3])                                       # tied logits
    l[4, ::3] = l[4, 0]
    p, vals, idx = ref.softmax_prune(l, 9)
    _, want_idx, _ = ref.prune_scores(l, 9)
    np.testing.assert_array_equal(idx, want_idx)
    # top-k of the exact probabilities (brute force, repeat-argmax, lowest column among equals)
    exact = special.softmax(l.astype(np.float64), axis=1)
    for r in range(l.shape[0]):
        key = exact[r].copy()
        got = []
        for _ in range(9):
            j = int(np.argmax(key))
            got.append(j)
            key[j] = -1.0
        # equal logits give exactly equal exact probabilities, so the same tie rule applies
        assert sorted(got) == idx[r].tolist()


def test_large_logits_do_not_overflow_and_bf16_rounds_once():
    l = np.array([[1000.0, 999.0, -1000.0, 0.0]], dtype=np.float32)
    p, vals, idx = ref.softmax_prune(l, 2)
    np.testing.assert_allclose(p[0, :2], [0.7310586, 0.26894143], rtol=1e-6)
    assert p[0, 2] == 0.0 and idx.tolist() == [[0, 1]]
    lb = (_rows(8, 4, 64).view(np.uint32) >> 16).astype(np.uint16)
    pb, vb, ib = ref.softmax_prune(lb, 6)
    lw = (lb.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    want = special.softmax(lw, axis=1)
    got = (pb.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.all(np.abs(got - want) <= want * 2.0 ** -8)
    np.testing.assert_array_equal(vb, np.take_along_axis(pb, ib.astype(np.int64), axis=1))


def test_backward_with_everything_kept_is_the_derivative_of_softmax():
    import torch
    rows, cols = 7, 53
    l = _rows(11, rows, cols, 2.0)
    dp = _rows(12, rows, cols)
    lt = torch.from_numpy(l).double().requires_grad_(True)
    torch.softmax(lt, dim=1).backward(torch.from_numpy(dp).double())
    p, vals, idx = ref.softmax_prune(l, cols)                      # nothing pruned
    ds = ref.softmax_backward_pruned(vals, idx, None, dp)
    np.testing.assert_allclose(ds.astype(np.float64), lt.grad.numpy(), rtol=0, atol=3e-7 * np.abs(lt.grad.numpy()).max())


def test_backward_is_the_formula_on_the_restored_rows():
    rows, cols, k = 40, 197, 9
    l = _rows(13, rows, cols, 2.0)
    dp = _rows(14, rows, cols)
    _, vals, idx = ref.softmax_prune(l, k)
    ds = ref.softmax_backward_pruned(vals, idx, None, dp)
    dense = ref.restore_scores(vals, idx, None, cols).astype(np.float64)
    want = dense * (dp.astype(np.float64) - (dense * dp).sum(1, keepdims=True))
    np.testing.assert_allclose(ds.astype(np.float64), want, rtol=2e-7, atol=1e-30)
    assert np.all((ds != 0) <= (dense != 0))                        # zero wherever nothing was kept
    # counts and unused slots (threshold mode leaves value 0 / index 0xFFFF)
    counts = np.full(rows, k, np.int32)
    counts[::3] = 4
    v2, i2 = vals.copy(), idx.copy()
    v2[::3, 4:] = 0
    i2[::3, 4:] = 0xFFFF
    a = ref.softmax_backward_pruned(v2, i2, counts, dp)
    b = ref.softmax_backward_pruned(v2, i2, None, dp)              # the sentinel alone also skips them
    np.testing.assert_array_equal(a, b)
    dense2 = ref.restore_scores(v2, i2, counts, cols).astype(np.float64)
    np.testing.assert_allclose(a.astype(np.float64), dense2 * (dp - (dense2 * dp).sum(1, keepdims=True)), rtol=2e-7,
                               atol=1e-30)


def test_bad_arguments_rejected():
    l = np.zeros((2, 4), np.float32)
    for k in (0, 5):
        with pytest.raises(ValueError):
            ref.softmax_prune(l, k)
