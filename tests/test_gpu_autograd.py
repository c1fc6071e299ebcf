"""GPU: the torch.autograd wrappers (Alg. 4) marshal into the library correctly -- each Function's results are
those of the same C-ABI calls made by hand (the kernels themselves are compared with the oracle elsewhere) --
frozen layers return no weight gradient, and the cached activations are the compressed ones."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2305_18513_amd import autograd as ag
from paper_2305_18513_amd import binding as sf
from tests.gpu_util import require_gpu

pytestmark = pytest.mark.gpu


def _saved_bytes(out: torch.Tensor) -> int:
    return sum(t.numel() * t.element_size() for t in out.grad_fn.saved_tensors if not isinstance(t, torch.nn.Parameter))


def test_gelu_function_equals_the_fused_calls_and_caches_four_bits():
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(0)
    x = (torch.randn(6, 50, 300, generator=g, device="cuda") * 2).requires_grad_(True)
    dy = torch.randn(6, 50, 300, generator=g, device="cuda")
    y = ag.GeluFunction.apply(x, 4, 64)
    assert _saved_bytes(y) == sf.packed_bytes(x.numel(), 4) + 4 * sf.num_blocks(x.numel(), 64)
    y.backward(dy)
    n = x.numel()
    y2 = torch.empty(n, device="cuda")
    codes = torch.empty(sf.packed_bytes(n, 4), dtype=torch.uint8, device="cuda")
    scales = torch.empty(sf.num_blocks(n, 64), device="cuda")
    sf.gelu_quant_pack(x.detach().view(-1), sf.Q_BLOCK, 4, 64, 0, y2, codes, scales)
    dx2 = torch.empty(n, device="cuda")
    sf.gelu_backward_dequant(codes, scales, sf.Q_BLOCK, 4, 64, 0, dy.view(-1), dx2)
    assert torch.equal(y.detach().view(-1), y2) and torch.equal(x.grad.view(-1), dx2)
    exact = torch.nn.functional.gelu(x.detach())
    assert torch.allclose(y.detach(), exact, rtol=1e-5, atol=1e-5)


def test_layernorm_function_frozen_and_active():
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(1)
    rows, H = 96, 768
    x = torch.randn(4, 24, H, generator=g, device="cuda").requires_grad_(True)
    gamma = torch.nn.Parameter(torch.rand(H, generator=g, device="cuda") + 0.5)
    beta = torch.nn.Parameter(torch.rand(H, generator=g, device="cuda") - 0.5)
    dy = torch.randn(4, 24, H, generator=g, device="cuda")

    # frozen: 10 % of the standardised input + indices + row pointers + rstd, no gradient for gamma / beta
    y = ag.LayerNormFunction.apply(x, gamma, beta, 1e-5, True, 100000)
    k = sf.keep_count(rows * H, 100000)
    assert _saved_bytes(y) == 8 * k + 4 * (rows + 1) + 4 * rows
    y.backward(dy)
    assert gamma.grad is None and beta.grad is None
    y2 = torch.empty(rows, H, device="cuda")
    mean, rstd = torch.empty(rows, device="cuda"), torch.empty(rows, device="cuda")
    sf.layernorm_forward(x.detach().view(rows, H), gamma.detach(), beta.detach(), 1e-5, y2, mean, rstd)
    vals, idx = torch.empty(k, device="cuda"), torch.empty(k, dtype=torch.int32, device="cuda")
    rp = torch.empty(rows + 1, dtype=torch.int32, device="cuda")
    sf.prune_global_standardized(x.detach().view(rows, H), mean, rstd, k, vals, idx, True, None, rp)
    dx2 = torch.empty(rows, H, device="cuda")
    sf.layernorm_backward_pruned(vals, idx, rp, k, rstd, gamma.detach(), dy.view(rows, H), dx2)
    assert torch.equal(y.detach().view(rows, H), y2) and torch.equal(x.grad.view(rows, H), dx2)
    frozen_grad = x.grad.clone()

    # active: exact gradients, equal to torch's own layer norm within fp32 rounding
    x.grad = None
    y = ag.LayerNormFunction.apply(x, gamma, beta, 1e-5, False, 100000)
    y.backward(dy)
    xr = x.detach().clone().requires_grad_(True)
    gr, br = gamma.detach().clone().requires_grad_(True), beta.detach().clone().requires_grad_(True)
    torch.nn.functional.layer_norm(xr, (H,), gr, br, 1e-5).backward(dy)
    assert torch.allclose(x.grad, xr.grad, rtol=1e-4, atol=1e-5)
    assert torch.allclose(gamma.grad, gr.grad, rtol=1e-4, atol=1e-4) and torch.allclose(beta.grad, br.grad, rtol=1e-4, atol=1e-4)
    # the frozen layer's gradient is the paper's formula on the pairs the oracle keeps (its own statistics, its own
    # pruner), at the backward kernel's stated tolerance
    xh, gh, dyh = x.detach().view(rows, H).cpu().numpy(), gamma.detach().cpu().numpy(), dy.view(rows, H).cpu().numpy()
    _, om, orr = ref.layernorm_forward(xh, gh, beta.detach().cpu().numpy(), eps=1e-5)
    ov, oi = ref.prune_global(ref.standardize(xh, om, orr).reshape(-1), k, by_magnitude=True)
    want = ref.layernorm_backward_pruned(ov, oi, orr, gh, dyh)
    tol = 1e-5 * float(np.abs(want).max())
    np.testing.assert_allclose(frozen_grad.view(rows, H).cpu().numpy(), want, rtol=1e-5, atol=tol)


def test_layernorm_function_on_bf16_activations():
    """bf16 rows, fp32 parameters: the frozen layer keeps fp32 standardised values, the active one returns fp32
    parameter gradients; both equal the same C-ABI calls made by hand."""
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(6)
    rows, H = 64, 512
    x = torch.randn(rows, H, generator=g, device="cuda").bfloat16().requires_grad_(True)
    gamma = torch.nn.Parameter(torch.rand(H, generator=g, device="cuda") + 0.5)
    beta = torch.nn.Parameter(torch.rand(H, generator=g, device="cuda") - 0.5)
    dy = torch.randn(rows, H, generator=g, device="cuda").bfloat16()
    k = sf.keep_count(rows * H, 100000)
    y = ag.LayerNormFunction.apply(x, gamma, beta, 1e-5, True, 100000)
    assert y.dtype == torch.bfloat16 and _saved_bytes(y) == 8 * k + 4 * (rows + 1) + 4 * rows
    y.backward(dy)
    assert gamma.grad is None and x.grad.dtype == torch.bfloat16
    y2 = torch.empty_like(x.detach())
    mean, rstd = torch.empty(rows, device="cuda"), torch.empty(rows, device="cuda")
    sf.layernorm_forward(x.detach(), gamma.detach(), beta.detach(), 1e-5, y2, mean, rstd)
    vals, idx = torch.empty(k, device="cuda"), torch.empty(k, dtype=torch.int32, device="cuda")
    rp = torch.empty(rows + 1, dtype=torch.int32, device="cuda")
    sf.prune_global_standardized(x.detach(), mean, rstd, k, vals, idx, True, None, rp)
    dx2 = torch.empty_like(dy)
    sf.layernorm_backward_pruned(vals, idx, rp, k, rstd, gamma.detach(), dy, dx2)
    assert torch.equal(y.detach(), y2) and torch.equal(x.grad, dx2)
    x.grad = None
    ag.LayerNormFunction.apply(x, gamma, beta, 1e-5, False, 100000).backward(dy)
    xr = x.detach().float().requires_grad_(True)
    gr, br = gamma.detach().clone().requires_grad_(True), beta.detach().clone().requires_grad_(True)
    torch.nn.functional.layer_norm(xr, (H,), gr, br, 1e-5).backward(dy.float())
    assert torch.allclose(x.grad.float(), xr.grad, rtol=2e-2, atol=2e-2)
    assert gamma.grad.dtype == torch.float32
    assert torch.allclose(gamma.grad, gr.grad, rtol=1e-3, atol=1e-3) and torch.allclose(beta.grad, br.grad, rtol=1e-3, atol=1e-3)


def test_layernorm_function_with_the_quantised_cache():
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(4)
    rows, H = 96, 768
    x = torch.randn(4, 24, H, generator=g, device="cuda").requires_grad_(True)
    gamma = torch.nn.Parameter(torch.rand(H, generator=g, device="cuda") + 0.5)
    beta = torch.nn.Parameter(torch.rand(H, generator=g, device="cuda") - 0.5)
    dy = torch.randn(4, 24, H, generator=g, device="cuda")
    n = rows * H
    for frozen in (True, False):
        x.grad = gamma.grad = beta.grad = None
        y = ag.LayerNormFunction.apply(x, gamma, beta, 1e-5, frozen, 100000, 4, 64)
        assert _saved_bytes(y) == sf.packed_bytes(n, 4) + 4 * sf.num_blocks(n, 64) + 8 * rows
        y.backward(dy)
        y2 = torch.empty(rows, H, device="cuda")
        mean, rstd = torch.empty(rows, device="cuda"), torch.empty(rows, device="cuda")
        codes = torch.empty(sf.packed_bytes(n, 4), dtype=torch.uint8, device="cuda")
        scales = torch.empty(sf.num_blocks(n, 64), device="cuda")
        sf.layernorm_forward_quant_pack(x.detach().view(rows, H), gamma.detach(), beta.detach(), 1e-5, 4, 64, y2, mean,
                                        rstd, codes, scales)
        dx2 = torch.empty(rows, H, device="cuda")
        sf.layernorm_backward_dequant(codes, scales, 4, 64, mean, rstd, gamma.detach(), dy.view(rows, H), dx2)
        assert torch.equal(y.detach().view(rows, H), y2) and torch.equal(x.grad.view(rows, H), dx2)
        assert torch.allclose(y.detach(), torch.nn.functional.layer_norm(x.detach(), (H,), gamma, beta, 1e-5), rtol=1e-5, atol=1e-5)
        if frozen:
            assert gamma.grad is None and beta.grad is None
        else:
            xh = torch.empty(rows, H, device="cuda")
            sf.dequant_unpack(codes, scales, sf.Q_BLOCK, 4, 64, 0, xh.view(-1))
            dg, db = torch.empty(H, device="cuda"), torch.empty(H, device="cuda")
            sf.layernorm_param_grads(xh, mean, rstd, dy.view(rows, H), dg, db)
            assert torch.equal(gamma.grad, dg) and torch.equal(beta.grad, db)
            # 4-bit cache: the gradient is close to, not equal to, the exact one
            xe = x.detach().clone().requires_grad_(True)
            torch.nn.functional.layer_norm(xe, (H,), gamma.detach(), beta.detach(), 1e-5).backward(dy)
            rel = (x.grad - xe.grad).norm() / xe.grad.norm()
            assert rel < 0.2, float(rel)


def test_softmax_function_equals_the_fused_calls_and_caches_a_tenth():
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(3)
    B, h, T = 3, 4, 197
    l = (torch.randn(B, h, T, T, generator=g, device="cuda") * 2).requires_grad_(True)
    dp = torch.randn(B, h, T, T, generator=g, device="cuda")
    p = ag.SoftmaxFunction.apply(l, 100000)
    rows, k = B * h * T, sf.keep_count(T, 100000)
    assert _saved_bytes(p) == rows * k * (4 + 2)
    p.backward(dp)
    p2 = torch.empty(rows, T, device="cuda")
    vals, idx = torch.empty(rows, k, device="cuda"), torch.empty(rows, k, dtype=torch.uint16, device="cuda")
    sf.softmax_prune(l.detach().view(rows, T), k, p2, vals, idx)
    ds2 = torch.empty(rows, T, device="cuda")
    sf.softmax_backward_pruned(vals, idx, None, dp.view(rows, T), ds2)
    assert torch.equal(p.detach().view(rows, T), p2) and torch.equal(l.grad.view(rows, T), ds2)
    assert torch.allclose(p.detach(), torch.softmax(l.detach(), dim=-1), rtol=1e-5, atol=1e-8)
    # with every column kept the gradient is the dense one
    l3 = l.detach().clone().requires_grad_(True)
    ag.SoftmaxFunction.apply(l3, 1000000).backward(dp)
    l4 = l.detach().clone().requires_grad_(True)
    torch.softmax(l4, dim=-1).backward(dp)
    assert torch.allclose(l3.grad, l4.grad, rtol=1e-4, atol=1e-6)


def test_linear_function_skips_the_weight_gradient_when_frozen():
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(2)
    x = torch.randn(8, 32, 256, generator=g, device="cuda").requires_grad_(True)
    w = torch.nn.Parameter(torch.randn(512, 256, generator=g, device="cuda") * 0.05)
    b = torch.nn.Parameter(torch.zeros(512, device="cuda"))
    dy = torch.randn(8, 32, 512, generator=g, device="cuda")

    w.requires_grad_(False)                                             # what a scheduler does to a frozen layer
    b.requires_grad_(False)
    out = ag.LinearFunction.apply(x, w, b, 8, 64)
    assert _saved_bytes(out) == 0                                       # only the weight (a Parameter) is kept
    out.backward(dy)
    assert w.grad is None and b.grad is None
    assert torch.allclose(x.grad, dy.matmul(w.detach()), rtol=1e-5, atol=1e-5)

    x.grad = None
    w.requires_grad_(True)
    b.requires_grad_(True)
    out = ag.LinearFunction.apply(x, w, b, 8, 64)
    n = x.numel()
    assert _saved_bytes(out) == sf.packed_bytes(n, 8) + 4 * sf.num_blocks(n, 64)       # 8-bit cache of the input
    out.backward(dy)
    codes = torch.empty(sf.packed_bytes(n, 8), dtype=torch.uint8, device="cuda")
    scales = torch.empty(sf.num_blocks(n, 64), device="cuda")
    sf.quant_pack(x.detach().view(-1), sf.Q_BLOCK, 8, 64, 0, codes, scales)
    xh = torch.empty(n, device="cuda")
    sf.dequant_unpack(codes, scales, sf.Q_BLOCK, 8, 64, 0, xh)
    want = dy.view(-1, 512).t().mm(xh.view(-1, 256))
    assert torch.allclose(w.grad, want, rtol=1e-5, atol=1e-4)
    assert torch.allclose(b.grad, dy.view(-1, 512).sum(0), rtol=1e-5, atol=1e-4)
    exact = dy.view(-1, 512).t().mm(x.detach().view(-1, 256))
    assert float((w.grad - exact).norm() / exact.norm()) < 0.01           # 8-bit cache: below 1 % in norm


def test_feed_forward_block_keeps_less_memory_when_wrapped():
    """x -> Linear(H, 4H) -> GELU -> Linear(4H, H) -> LayerNorm, everything frozen: activation memory held
    between forward and backward, wrapped vs plain torch."""
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(3)
    B, T, H = 16, 128, 512
    x = torch.randn(B, T, H, generator=g, device="cuda").requires_grad_(True)
    w1 = torch.nn.Parameter(torch.randn(4 * H, H, generator=g, device="cuda") * 0.03)
    w2 = torch.nn.Parameter(torch.randn(H, 4 * H, generator=g, device="cuda") * 0.03)
    gamma = torch.nn.Parameter(torch.ones(H, device="cuda"))
    beta = torch.nn.Parameter(torch.zeros(H, device="cuda"))

    def held(fn):
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        before = torch.cuda.memory_allocated()
        out = fn()
        torch.cuda.synchronize()
        kept = torch.cuda.memory_allocated() - before - out.numel() * out.element_size()
        out.sum().backward()
        return kept

    def plain():
        h = torch.nn.functional.linear(x, w1)
        h = torch.nn.functional.gelu(h)
        h = torch.nn.functional.linear(h, w2)
        return torch.nn.functional.layer_norm(h, (H,), gamma, beta, 1e-5)

    def wrapped():
        h = ag.LinearFunction.apply(x, w1.detach(), None, 8, 64)
        h = ag.GeluFunction.apply(h, 4, 64)
        h = ag.LinearFunction.apply(h, w2.detach(), None, 8, 64)
        return ag.LayerNormFunction.apply(h, gamma, beta, 1e-5, True, 100000)

    kept_plain, kept_wrapped = held(plain), held(wrapped)
    assert kept_wrapped < 0.25 * kept_plain, (kept_plain, kept_wrapped)


def test_softmax_matmul_function_shares_the_pruned_probabilities():
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(8)
    B, h, T, D = 2, 4, 197, 64
    logits = (torch.randn(B, h, T, T, generator=g, device="cuda") * 2).requires_grad_(True)
    v = torch.randn(B, h, T, D, generator=g, device="cuda").requires_grad_(True)
    do = torch.randn(B, h, T, D, generator=g, device="cuda")
    rows, k = B * h * T, sf.keep_count(T, 100000)
    out = ag.SoftmaxMatmulFunction.apply(logits, v, 100000)
    assert _saved_bytes(out) == rows * k * 6 + v.numel() * 4            # the pairs and V, not the T x T probabilities
    out.backward(do)
    # forward is exact; with every column kept both gradients are the dense ones
    assert torch.allclose(out.detach(), torch.softmax(logits.detach(), -1) @ v.detach(), rtol=1e-4, atol=1e-5)
    l2, v2 = logits.detach().clone().requires_grad_(True), v.detach().clone().requires_grad_(True)
    ag.SoftmaxMatmulFunction.apply(l2, v2, 1000000).backward(do)
    l3, v3 = logits.detach().clone().requires_grad_(True), v.detach().clone().requires_grad_(True)
    (torch.softmax(l3, -1) @ v3).backward(do)
    assert torch.allclose(l2.grad, l3.grad, rtol=1e-3, atol=1e-5) and torch.allclose(v2.grad, v3.grad, rtol=1e-3, atol=1e-4)
    # pruned: the gradients are those of the same library calls made by hand
    p = torch.empty(rows, T, device="cuda")
    vals, idx = torch.empty(rows, k, device="cuda"), torch.empty(rows, k, dtype=torch.uint16, device="cuda")
    sf.softmax_prune(logits.detach().view(rows, T), k, p, vals, idx)
    p_hat = torch.empty(rows, T, device="cuda")
    sf.restore_scores(vals, idx, None, p_hat)
    dp = (do @ v.detach().transpose(-1, -2)).contiguous().view(rows, T)
    ds = torch.empty(rows, T, device="cuda")
    sf.softmax_backward_pruned(vals, idx, None, dp, ds)
    assert torch.equal(logits.grad.view(rows, T), ds)
    assert torch.equal(v.grad, p_hat.view(B, h, T, T).transpose(-1, -2) @ do)


def test_matmul_function_caches_both_operands_in_eight_bits():
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(10)
    a = torch.randn(3, 4, 50, 64, generator=g, device="cuda").requires_grad_(True)
    b = torch.randn(3, 4, 64, 70, generator=g, device="cuda").requires_grad_(True)
    do = torch.randn(3, 4, 50, 70, generator=g, device="cuda")
    out = ag.MatmulFunction.apply(a, b, 8, 64)
    na, nb = a.numel(), b.numel()
    assert _saved_bytes(out) == na + nb + 4 * (sf.num_blocks(na, 64) + sf.num_blocks(nb, 64))
    assert torch.equal(out.detach(), a.detach() @ b.detach())
    out.backward(do)
    a2, b2 = a.detach().clone().requires_grad_(True), b.detach().clone().requires_grad_(True)
    (a2 @ b2).backward(do)
    assert (a.grad - a2.grad).norm() / a2.grad.norm() < 0.02 and (b.grad - b2.grad).norm() / b2.grad.norm() < 0.02
    # exactly the products with the dequantised operands
    ca = torch.empty(na, dtype=torch.uint8, device="cuda"); sa = torch.empty(sf.num_blocks(na, 64), device="cuda")
    sf.quant_pack(a.detach().view(-1), sf.Q_BLOCK, 8, 64, 0, ca, sa)
    ah = torch.empty_like(a.detach())
    sf.dequant_unpack(ca, sa, sf.Q_BLOCK, 8, 64, 0, ah.view(-1))
    assert torch.equal(b.grad, ah.transpose(-1, -2) @ do)


def test_encoder_block_keeps_less_memory_when_wrapped():
    """A whole frozen encoder block (LayerNorm, QKV, attention with shared pruned probabilities, projection,
    LayerNorm, feed-forward with GELU): activation bytes held between forward and backward, wrapped vs plain torch,
    and the wrapped block's output equals the plain one's (compression only touches what backward reads)."""
    require_gpu()
    B, T, H, heads = 8, 256, 512, 8
    g = torch.Generator(device="cuda").manual_seed(9)
    x = torch.randn(B, T, H, generator=g, device="cuda").requires_grad_(True)
    params = ag.encoder_block_params(H, seed=9)
    kept_plain, _ = ag.held_activation_bytes(lambda: ag.frozen_encoder_block(x, params, heads, wrapped=False))
    grad_plain = x.grad.clone()
    x.grad = None
    for q in params.values():
        q.grad = None
    kept_wrapped, _ = ag.held_activation_bytes(lambda: ag.frozen_encoder_block(x, params, heads, wrapped=True))
    assert kept_wrapped < 0.25 * kept_plain, (kept_plain, kept_wrapped)
    with torch.no_grad():
        y0 = ag.frozen_encoder_block(x, params, heads, wrapped=False)
        y1 = ag.frozen_encoder_block(x, params, heads, wrapped=True)
    assert torch.allclose(y0, y1, rtol=1e-4, atol=1e-4)
    assert grad_plain is not None and x.grad is not None
    assert all(q.grad is None for q in params.values())                   # frozen: no parameter gradients


def test_frozen_feed_forward_block_backward_equals_the_composition_of_oracle_functions():
    """x -> Linear(w1) -> GELU -> Linear(w2) -> LayerNorm, every layer frozen, through the wrappers; the same chain
    written with the oracle's functions (quant_pack -> dequant_unpack -> gelu_backward for GELU's cache; layernorm
    statistics -> standardize -> prune_global -> layernorm_backward_pruned for LayerNorm's) and NumPy float64
    products for the two linear layers.  Inputs and the first weight matrix are multiples of small powers of two, so
    that the first product is exact in fp32 and both sides quantise the very same GELU input."""
    require_gpu()
    g = torch.Generator(device="cuda").manual_seed(21)
    rows, H, F = 64, 64, 256
    x = (torch.randint(-16, 17, (rows, H), generator=g, device="cuda").float() / 8).requires_grad_(True)
    w1 = torch.randint(-16, 17, (F, H), generator=g, device="cuda").float() / 64
    w2 = torch.randn(H, F, generator=g, device="cuda") * 0.1
    gamma = torch.rand(H, generator=g, device="cuda") + 0.5
    beta = torch.rand(H, generator=g, device="cuda") - 0.5
    dy = torch.randn(rows, H, generator=g, device="cuda")

    h1 = ag.LinearFunction.apply(x, w1, None, 8, 64)
    a = ag.GeluFunction.apply(h1, 4, 64)
    h3 = ag.LinearFunction.apply(a, w2, None, 8, 64)
    y = ag.LayerNormFunction.apply(h3, gamma, beta, 1e-5, True, 100000)
    kept_vals, kept_idx = y.grad_fn.saved_tensors[0], y.grad_fn.saved_tensors[1]
    y.backward(dy)

    xh, w1h, w2h = x.detach().cpu().numpy(), w1.cpu().numpy(), w2.cpu().numpy()
    gh, bh, dyh = gamma.cpu().numpy(), beta.cpu().numpy(), dy.cpu().numpy()
    o_h1 = (xh.astype(np.float64) @ w1h.astype(np.float64).T)
    assert np.array_equal(o_h1.astype(np.float32).astype(np.float64), o_h1)         # exact in fp32, as constructed
    o_h1 = o_h1.astype(np.float32)
    assert np.array_equal(h1.detach().cpu().numpy(), o_h1)
    o_a = ref.gelu(o_h1).reshape(rows, F)
    o_h3 = (o_a.astype(np.float64) @ w2h.astype(np.float64).T).astype(np.float32)
    o_y, om, orr = ref.layernorm_forward(o_h3, gh, bh, eps=1e-5)
    k = sf.keep_count(rows * H, 100000)
    ov, oi = ref.prune_global(ref.standardize(o_h3, om, orr).reshape(-1), k, by_magnitude=True)
    assert np.array_equal(kept_idx.cpu().numpy(), oi)                                 # the wrapper cached the oracle's set
    np.testing.assert_allclose(kept_vals.cpu().numpy(), ov, rtol=2e-5, atol=2e-6)
    np.testing.assert_allclose(y.detach().cpu().numpy(), o_y, rtol=1e-5, atol=2e-5)
    o_dh3 = ref.layernorm_backward_pruned(ov, oi, orr, gh, dyh)                        # frozen LayerNorm: the paper's formula
    o_da = (o_dh3.astype(np.float64) @ w2h.astype(np.float64)).astype(np.float32)      # frozen Linear: dx only
    oc, osc = ref.quant_pack(o_h1.reshape(-1), bits=4, block=64)
    o_dh1 = ref.gelu_backward(ref.dequant_unpack(oc, osc, o_h1.size, bits=4, block=64), o_da.reshape(-1)).reshape(rows, F)
    o_dx = (o_dh1.astype(np.float64) @ w1h.astype(np.float64)).astype(np.float32)
    # the kernels' own budgets (LayerNorm backward 4e-6 of its terms, GELU backward 1e-6, two fp32 products) add up
    # to a few 1e-6 of the largest entry
    tol = 2e-5 * float(np.abs(o_dx).max())
    np.testing.assert_allclose(x.grad.cpu().numpy(), o_dx, rtol=2e-5, atol=tol)
