"""Pins for the oracle's LayerNorm pieces (Sec. 4: forward, standardised input, frozen-layer input
gradient from the kept pairs) -- CPU only."""
import numpy as np
import pytest
import torch

from oracle import ref


def _case(seed, rows, H):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((rows, H)) * rng.uniform(0.5, 3.0, (rows, 1)) + rng.uniform(-2, 2, (rows, 1))).astype(np.float32)
    gamma = rng.uniform(0.5, 1.5, H).astype(np.float32)
    beta = rng.uniform(-0.5, 0.5, H).astype(np.float32)
    dy = rng.standard_normal((rows, H)).astype(np.float32)
    return x, gamma, beta, dy


@pytest.mark.parametrize("rows,H", [(1, 4), (5, 64), (7, 768), (3, 1024), (2, 1000)])
def test_forward_matches_library_layer_norm(rows, H):
    x, gamma, beta, _ = _case(rows + H, rows, H)
    y, mean, rstd = ref.layernorm_forward(x, gamma, beta, eps=1e-5)
    want = torch.nn.functional.layer_norm(torch.from_numpy(x).double(), (H,), torch.from_numpy(gamma).double(),
                                          torch.from_numpy(beta).double(), eps=1e-5).numpy()
    np.testing.assert_allclose(y.astype(np.float64), want, rtol=1.5e-7, atol=1e-7)
    xd = x.astype(np.float64)
    np.testing.assert_allclose(mean, xd.mean(1), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(rstd, 1.0 / np.sqrt(xd.var(1) + 1e-5), rtol=1e-6)


def test_forward_invariants():
    x, gamma, beta, _ = _case(3, 6, 256)
    one, zero = np.ones(256, np.float32), np.zeros(256, np.float32)
    xt, _, _ = ref.layernorm_forward(x, one, zero, eps=0.0)
    assert np.all(np.abs(xt.astype(np.float64).mean(1)) < 1e-6)
    np.testing.assert_allclose(xt.astype(np.float64).var(1), 1.0, rtol=1e-5)
    x2, _, _ = ref.layernorm_forward(x * np.float32(4.0) + np.float32(8.0), one, zero, eps=0.0)    # shift and scale
    np.testing.assert_allclose(x2, xt, rtol=0, atol=2e-5)
    y, _, _ = ref.layernorm_forward(x, gamma, beta, eps=0.0)
    np.testing.assert_allclose(y, xt * gamma + beta, rtol=0, atol=1e-6)
    const, m, r = ref.layernorm_forward(np.full((2, 8), 3.5, np.float32), one[:8], zero[:8], eps=1e-5)
    assert np.all(const == 0.0) and np.all(m == 3.5) and np.allclose(r, 1.0 / np.sqrt(1e-5))


def test_standardize_is_two_fp32_operations():
    x, _, _, _ = _case(4, 9, 128)
    _, mean, rstd = ref.layernorm_forward(x, np.ones(128, np.float32), np.zeros(128, np.float32))
    xs = ref.standardize(x, mean, rstd)
    want = ((x - mean[:, None]).astype(np.float32) * rstd[:, None]).astype(np.float32)       # NumPy float32 arithmetic
    np.testing.assert_array_equal(xs.view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("rows,H", [(1, 8), (4, 64), (3, 768), (2, 1024)])
def test_unpruned_backward_is_the_derivative_of_layer_norm(rows, H):
    x, gamma, beta, dy = _case(rows * 3 + H, rows, H)
    xt = torch.from_numpy(x).double().requires_grad_(True)
    out = torch.nn.functional.layer_norm(xt, (H,), torch.from_numpy(gamma).double(), torch.from_numpy(beta).double(),
                                         eps=1e-5)
    out.backward(torch.from_numpy(dy).double())
    want = xt.grad.numpy()
    # everything kept: the exact x~ and rstd in double, handed over as the fp32 arrays the interface takes
    xd = x.astype(np.float64)
    rstd = 1.0 / np.sqrt(xd.var(1) + 1e-5)
    xtil = (xd - xd.mean(1, keepdims=True)) * rstd[:, None]
    n = rows * H
    dx = ref.layernorm_backward_pruned(xtil.reshape(-1).astype(np.float32), np.arange(n, dtype=np.int32),
                                       rstd.astype(np.float32), gamma, dy)
    np.testing.assert_allclose(dx.astype(np.float64), want, rtol=0, atol=2e-6 * np.abs(want).max())


def test_pruned_backward_is_the_formula_on_the_restored_tensor():
    rows, H = 6, 256
    x, gamma, beta, dy = _case(9, rows, H)
    _, mean, rstd = ref.layernorm_forward(x, gamma, beta)
    xs = ref.standardize(x, mean, rstd).reshape(-1)
    k = int(xs.size * 0.1)
    vals, idx = ref.prune_global(xs, k, by_magnitude=True)
    dx = ref.layernorm_backward_pruned(vals, idx, rstd, gamma, dy)
    dense = ref.restore_global(vals, idx, xs.size).reshape(rows, H).astype(np.float64)
    g = gamma.astype(np.float64) * dy.astype(np.float64) * rstd.astype(np.float64)[:, None] / H
    want = H * g - g.sum(1, keepdims=True) - dense * (g * dense).sum(1, keepdims=True)
    np.testing.assert_allclose(dx.astype(np.float64), want, rtol=1e-6, atol=1e-7)
    # shuffled pairs give the same gradient; nothing kept drops the last term
    perm = np.random.default_rng(0).permutation(k)
    np.testing.assert_array_equal(ref.layernorm_backward_pruned(vals[perm], idx[perm], rstd, gamma, dy), dx)
    none = ref.layernorm_backward_pruned(vals[:0], idx[:0], rstd, gamma, dy)
    np.testing.assert_allclose(none.astype(np.float64), H * g - g.sum(1, keepdims=True), rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("rows,H", [(1, 8), (4, 64), (3, 768), (2, 1024)])
def test_dense_backward_is_the_derivative_of_layer_norm(rows, H):
    x, gamma, beta, dy = _case(rows * 5 + H, rows, H)
    xt = torch.from_numpy(x).double().requires_grad_(True)
    out = torch.nn.functional.layer_norm(xt, (H,), torch.from_numpy(gamma).double(), torch.from_numpy(beta).double(),
                                         eps=1e-5)
    out.backward(torch.from_numpy(dy).double())
    want = xt.grad.numpy()
    _, mean, rstd = ref.layernorm_forward(x, gamma, beta, eps=1e-5)
    dx = ref.layernorm_backward(x, mean, rstd, gamma, dy)
    np.testing.assert_allclose(dx.astype(np.float64), want, rtol=0, atol=2e-6 * np.abs(want).max())
    # and it agrees with the pair form when every x~ is handed over
    xs = ((x.astype(np.float64) - mean.astype(np.float64)[:, None]) * rstd.astype(np.float64)[:, None])
    full = ref.layernorm_backward_pruned(xs.reshape(-1).astype(np.float32), np.arange(rows * H, dtype=np.int32), rstd,
                                         gamma, dy)
    np.testing.assert_allclose(dx, full, rtol=0, atol=1e-6 * np.abs(want).max())


@pytest.mark.parametrize("rows,H", [(1, 8), (50, 64), (33, 768)])
def test_parameter_gradients_are_the_derivative_of_layer_norm(rows, H):
    x, gamma, beta, dy = _case(rows + 2 * H, rows, H)
    gt = torch.from_numpy(gamma).double().requires_grad_(True)
    bt = torch.from_numpy(beta).double().requires_grad_(True)
    out = torch.nn.functional.layer_norm(torch.from_numpy(x).double(), (H,), gt, bt, eps=1e-5)
    out.backward(torch.from_numpy(dy).double())
    _, mean, rstd = ref.layernorm_forward(x, gamma, beta, eps=1e-5)
    dg, db = ref.layernorm_param_grads(x, mean, rstd, dy)
    scale = np.abs(dy.astype(np.float64)).sum(0).max() * 4
    np.testing.assert_allclose(dg.astype(np.float64), gt.grad.numpy(), rtol=0, atol=1e-6 * scale)
    np.testing.assert_allclose(db.astype(np.float64), bt.grad.numpy(), rtol=1e-6, atol=1e-6 * scale)
    # column sums written out in NumPy float64 from the same fp32 statistics
    xt = (x.astype(np.float64) - mean.astype(np.float64)[:, None]) * rstd.astype(np.float64)[:, None]
    np.testing.assert_allclose(dg, (xt * dy).sum(0), rtol=2e-7, atol=1e-30)
    np.testing.assert_allclose(db, dy.astype(np.float64).sum(0), rtol=2e-7, atol=1e-30)


def test_bad_arguments_rejected():
    with pytest.raises(ValueError):
        ref.layernorm_backward_pruned(np.ones(1, np.float32), np.array([99], np.int32), np.ones(2, np.float32),
                                      np.ones(4, np.float32), np.ones((2, 4), np.float32))
