"""torch.autograd wrappers over the C ABI (Alg. 4 and Sec. 4 of the paper).

Each Function runs its forward through the library, keeps only the compressed
form of the activation its backward needs, and skips the weight gradient of a
frozen layer.  Nothing here computes on its own what a kernel of the library
computes; the dense matrix products of the linear layer are torch's.

  GeluFunction       y = GELU(x); caches x in `bits` bits (per-block scales);
                     backward multiplies by GELU'(x^) straight from the cache.
  LayerNormFunction  frozen: caches the `keep_ppm` largest |x~| of the whole
                     tensor with int32 indices, row pointers and rstd; backward
                     is the paper's input-gradient formula on those pairs, and
                     gamma / beta get no gradient.  Active: caches x exactly
                     and returns all three gradients.  With `quant_bits` the
                     cache is instead the block-scaled codes of x written by the
                     forward kernel itself (plus mean and rstd); backward rebuilds
                     x^ in registers, and an active layer's gamma / beta gradients
                     use the dequantised x^.
  SoftmaxFunction    p = softmax(logits) over the last dimension (at most 2048
                     wide); caches the `keep_ppm` largest probabilities of every
                     row with uint16 columns; backward is the derivative of
                     softmax with the restored (sparse) row in place of p.
  SoftmaxMatmulFunction  out = softmax(logits) @ V with the probabilities shared
                     between the two ops as the paper has it: only the kept
                     pairs and V are cached.  Backward: dP = dO @ V^T (dense
                     product, torch's), dV = P^^T @ dO with P^ restored from the
                     pairs, dlogits from the pairs as in SoftmaxFunction.
  MatmulFunction     out = a @ b with both operands cached in 8 bits (the paper's
                     placement for MatMul's activations).
  LinearFunction     the freezing rule of Alg. 4: a layer whose weight does not
                     require a gradient (frozen by the scheduler) keeps nothing of
                     its input and returns no weight gradient; an active one keeps
                     its input in `bits` bits and forms the weight gradient from
                     the dequantised input.

All tensors are CUDA tensors (fp32 or bf16 activations; gamma / beta and the
kept standardised values fp32); the kernels run on torch's current stream.
"""
from __future__ import annotations

import torch

from . import binding as sf


def _flat(t: torch.Tensor) -> torch.Tensor:
    return t.contiguous().view(-1)


def _quantise(t: torch.Tensor, bits: int, block: int):
    """(codes, scales) of the flattened tensor, block-scaled."""
    f = _flat(t)
    n = f.numel()
    codes = torch.empty(sf.packed_bytes(n, bits), dtype=torch.uint8, device=t.device)
    scales = torch.empty(sf.num_blocks(n, block), dtype=torch.float32, device=t.device)
    sf.quant_pack(f, sf.Q_BLOCK, bits, block, 0, codes, scales)
    return codes, scales


def _dequantise(codes, scales, bits: int, block: int, shape, dtype) -> torch.Tensor:
    out = torch.empty(shape, dtype=dtype, device=codes.device)
    sf.dequant_unpack(codes, scales, sf.Q_BLOCK, bits, block, 0, out.view(-1))
    return out


class MatmulFunction(torch.autograd.Function):
    """out = a @ b with both operands cached in `bits` bits (the paper keeps MatMul's activations in 8 bits);
    backward multiplies the incoming gradient with the dequantised operands."""

    @staticmethod
    def forward(ctx, a: torch.Tensor, b: torch.Tensor, bits: int = 8, block: int = 64):
        out = torch.matmul(a, b)
        ca, sa = _quantise(a, bits, block)
        cb, sb = _quantise(b, bits, block)
        ctx.save_for_backward(ca, sa, cb, sb)
        ctx.meta = (bits, block, a.shape, b.shape, a.dtype)
        return out

    @staticmethod
    def backward(ctx, grad_output: torch.Tensor):
        ca, sa, cb, sb = ctx.saved_tensors
        bits, block, sha, shb, dtype = ctx.meta
        b_hat = _dequantise(cb, sb, bits, block, shb, dtype)
        da = torch.matmul(grad_output, b_hat.transpose(-1, -2))
        del b_hat
        a_hat = _dequantise(ca, sa, bits, block, sha, dtype)
        db = torch.matmul(a_hat.transpose(-1, -2), grad_output)
        return da, db, None, None


class GeluFunction(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x: torch.Tensor, bits: int = 4, block: int = 64):
        xf = _flat(x)
        n = xf.numel()
        y = torch.empty_like(xf)
        codes = torch.empty(sf.packed_bytes(n, bits), dtype=torch.uint8, device=x.device)
        scales = torch.empty(sf.num_blocks(n, block), dtype=torch.float32, device=x.device)
        sf.gelu_quant_pack(xf, sf.Q_BLOCK, bits, block, 0, y, codes, scales)
        ctx.save_for_backward(codes, scales)
        ctx.quant = (bits, block)
        return y.view(x.shape)

    @staticmethod
    def backward(ctx, grad_output: torch.Tensor):
        codes, scales = ctx.saved_tensors
        bits, block = ctx.quant
        dy = _flat(grad_output)
        dx = torch.empty_like(dy)
        sf.gelu_backward_dequant(codes, scales, sf.Q_BLOCK, bits, block, 0, dy, dx)
        return dx.view(grad_output.shape), None, None


class LayerNormFunction(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x: torch.Tensor, gamma: torch.Tensor, beta: torch.Tensor, eps: float = 1e-5,
                frozen: bool = False, keep_ppm: int = 100000, quant_bits: int = 0, block: int = 64):
        H = x.shape[-1]
        x2 = x.contiguous().view(-1, H)
        rows = x2.shape[0]
        y = torch.empty_like(x2)
        mean = torch.empty(rows, dtype=torch.float32, device=x.device)
        rstd = torch.empty(rows, dtype=torch.float32, device=x.device)
        ctx.frozen = frozen
        ctx.quant = (quant_bits, block)
        if quant_bits:
            n = x2.numel()
            codes = torch.empty(sf.packed_bytes(n, quant_bits), dtype=torch.uint8, device=x.device)
            scales = torch.empty(sf.num_blocks(n, block), dtype=torch.float32, device=x.device)
            sf.layernorm_forward_quant_pack(x2, gamma, beta, eps, quant_bits, block, y, mean, rstd, codes, scales)
            ctx.save_for_backward(codes, scales, mean, rstd, gamma)
            return y.view(x.shape)
        sf.layernorm_forward(x2, gamma, beta, eps, y, mean, rstd)
        if frozen:
            n = x2.numel()
            k = sf.keep_count(n, keep_ppm)
            vals = torch.empty(k, dtype=torch.float32, device=x.device)
            idx = torch.empty(k, dtype=torch.int32, device=x.device)
            row_ptr = torch.empty(rows + 1, dtype=torch.int32, device=x.device)
            if k > 0:
                sf.prune_global_standardized(x2, mean, rstd, k, vals, idx, True, None, row_ptr)
            else:
                row_ptr.zero_()
            ctx.k = k
            ctx.save_for_backward(vals, idx, row_ptr, rstd, gamma)
        else:
            ctx.save_for_backward(x2, mean, rstd, gamma)
        return y.view(x.shape)

    @staticmethod
    def backward(ctx, grad_output: torch.Tensor):
        H = grad_output.shape[-1]
        dy = grad_output.contiguous().view(-1, H)
        none = (None,) * 5
        bits, block = ctx.quant
        if bits:
            codes, scales, mean, rstd, gamma = ctx.saved_tensors
            dx = torch.empty_like(dy)
            sf.layernorm_backward_dequant(codes, scales, bits, block, mean, rstd, gamma, dy, dx)
            if ctx.frozen:
                return (dx.view(grad_output.shape), None, None) + none
            x_hat = torch.empty_like(dy)
            sf.dequant_unpack(codes, scales, sf.Q_BLOCK, bits, block, 0, x_hat.view(-1))
            dgamma, dbeta = torch.empty_like(gamma), torch.empty_like(gamma)
            sf.layernorm_param_grads(x_hat, mean, rstd, dy, dgamma, dbeta)
            return (dx.view(grad_output.shape), dgamma, dbeta) + none
        if ctx.frozen:
            vals, idx, row_ptr, rstd, gamma = ctx.saved_tensors
            dx = torch.empty_like(dy)
            sf.layernorm_backward_pruned(vals, idx, row_ptr, ctx.k, rstd, gamma, dy, dx)
            return (dx.view(grad_output.shape), None, None) + none
        x2, mean, rstd, gamma = ctx.saved_tensors
        dgamma, dbeta = torch.empty_like(gamma), torch.empty_like(gamma)
        sf.layernorm_param_grads(x2, mean, rstd, dy, dgamma, dbeta)
        dx = torch.empty_like(dy)
        sf.layernorm_backward(x2, mean, rstd, gamma, dy, dx)
        return (dx.view(grad_output.shape), dgamma, dbeta) + none


class SoftmaxFunction(torch.autograd.Function):
    @staticmethod
    def forward(ctx, logits: torch.Tensor, keep_ppm: int = 100000):
        cols = logits.shape[-1]
        l2 = logits.contiguous().view(-1, cols)
        rows = l2.shape[0]
        k = max(1, sf.keep_count(cols, keep_ppm))
        probs = torch.empty_like(l2)
        vals = torch.empty(rows, k, dtype=l2.dtype, device=l2.device)
        idx = torch.empty(rows, k, dtype=torch.uint16, device=l2.device)
        sf.softmax_prune(l2, k, probs, vals, idx)
        ctx.save_for_backward(vals, idx)
        return probs.view(logits.shape)

    @staticmethod
    def backward(ctx, grad_output: torch.Tensor):
        vals, idx = ctx.saved_tensors
        cols = grad_output.shape[-1]
        dp = grad_output.contiguous().view(-1, cols)
        ds = torch.empty_like(dp)
        sf.softmax_backward_pruned(vals, idx, None, dp, ds)
        return ds.view(grad_output.shape), None


class SoftmaxMatmulFunction(torch.autograd.Function):
    @staticmethod
    def forward(ctx, logits: torch.Tensor, v: torch.Tensor, keep_ppm: int = 100000, v_bits: int = 0, block: int = 64):
        # logits (..., Tq, Tk), v (..., Tk, D); v_bits != 0 caches V quantised as well
        cols = logits.shape[-1]
        l2 = logits.contiguous().view(-1, cols)
        rows = l2.shape[0]
        k = max(1, sf.keep_count(cols, keep_ppm))
        probs = torch.empty_like(l2)
        vals = torch.empty(rows, k, dtype=l2.dtype, device=l2.device)
        idx = torch.empty(rows, k, dtype=torch.uint16, device=l2.device)
        sf.softmax_prune(l2, k, probs, vals, idx)
        out = torch.matmul(probs.view(logits.shape), v)
        if v_bits:
            cv, sv = _quantise(v, v_bits, block)
            ctx.save_for_backward(vals, idx, cv, sv)
        else:
            ctx.save_for_backward(vals, idx, v)
        ctx.meta = (logits.shape, v.shape, v.dtype, v_bits, block)
        return out

    @staticmethod
    def backward(ctx, grad_output: torch.Tensor):
        shape, v_shape, v_dtype, v_bits, block = ctx.meta
        if v_bits:
            vals, idx, cv, sv = ctx.saved_tensors
            v = _dequantise(cv, sv, v_bits, block, v_shape, v_dtype)
        else:
            vals, idx, v = ctx.saved_tensors
        cols = shape[-1]
        rows = vals.shape[0]
        dp = torch.matmul(grad_output, v.transpose(-1, -2)).contiguous().view(rows, cols)
        p_hat = torch.empty(rows, cols, dtype=vals.dtype, device=vals.device)
        sf.restore_scores(vals, idx, None, p_hat)
        dv = torch.matmul(p_hat.view(shape).transpose(-1, -2), grad_output)
        ds = torch.empty_like(dp)
        sf.softmax_backward_pruned(vals, idx, None, dp, ds)
        return ds.view(shape), dv, None, None, None


class LinearFunction(torch.autograd.Function):
    """y = x W^T (+ b) under the freezing rule of Alg. 4.  Whether the layer is frozen is read off the weight itself
    (``weight.requires_grad``, which is what an inter-layer scheduler flips between iterations): a frozen layer
    keeps nothing of x and produces no weight gradient; an active one keeps x as ``bits``-bit block-scaled codes
    and forms its weight gradient from the dequantised x^."""

    @staticmethod
    def forward(ctx, x: torch.Tensor, weight: torch.Tensor, bias, bits: int = 8, block: int = 64):
        y = torch.nn.functional.linear(x, weight, bias)
        ctx.cache = None                                   # descriptor of what is kept of x: nothing, or (bits, block, shape, dtype)
        ctx.bias_active = bias is not None and bias.requires_grad
        if weight.requires_grad:
            codes, scales = _quantise(x, bits, block)
            ctx.cache = (bits, block, x.shape, x.dtype)
            ctx.save_for_backward(weight, codes, scales)
        else:
            ctx.save_for_backward(weight)
        return y

    @staticmethod
    def backward(ctx, dy: torch.Tensor):
        weight = ctx.saved_tensors[0]
        dx = dy.matmul(weight) if ctx.needs_input_grad[0] else None
        dy2 = dy.reshape(-1, dy.shape[-1])
        dw = None
        if ctx.cache is not None:
            bits, block, shape, dtype = ctx.cache
            x_hat = _dequantise(ctx.saved_tensors[1], ctx.saved_tensors[2], bits, block, shape, dtype)
            dw = dy2.t().mm(x_hat.view(-1, shape[-1]))
        db = dy2.sum(0) if ctx.bias_active else None
        return dx, dw, db, None, None


def encoder_block_params(hidden: int, device="cuda", seed: int = 0, dtype=torch.float32):
    """Random weights of one encoder block (QKV, projection, two feed-forward matrices, two LayerNorms)."""
    g = torch.Generator(device=device).manual_seed(seed)

    def mat(rows, cols):
        return torch.nn.Parameter((torch.randn(rows, cols, generator=g, device=device) * 0.03).to(dtype))

    def vec(value):
        return torch.nn.Parameter(torch.full((hidden,), value, device=device))

    return {"wqkv": mat(3 * hidden, hidden), "wo": mat(hidden, hidden), "w1": mat(4 * hidden, hidden),
            "w2": mat(hidden, 4 * hidden), "g1": vec(1.0), "b1": vec(0.0), "g2": vec(1.0), "b2": vec(0.0)}


def frozen_encoder_block(x: torch.Tensor, p: dict, heads: int, wrapped: bool, keep_ppm: int = 100000,
                         gelu_bits: int = 4, block: int = 64) -> torch.Tensor:
    """One pre-LN encoder block whose layers are all frozen: with ``wrapped`` the activations kept
    for the backward pass are the compressed ones (pruned LayerNorm input, pruned attention probabilities shared by
    Softmax and MatMul, 4-bit GELU input, nothing for the frozen linear layers); without, plain torch ops."""
    B, T, H = x.shape
    D = H // heads
    F = torch.nn.functional

    def split(t):
        return t.reshape(B, T, heads, D).transpose(1, 2)

    if wrapped:
        w = {name: t.detach() for name, t in p.items()}    # frozen: the scheduler has switched their gradients off
        h = LayerNormFunction.apply(x, p["g1"], p["b1"], 1e-5, True, keep_ppm)
        q, k_, v = LinearFunction.apply(h, w["wqkv"], None, 8, block).chunk(3, dim=-1)
        s = MatmulFunction.apply(split(q).contiguous(), split(k_).transpose(-1, -2).contiguous(), 8, block) / D ** 0.5
        a = SoftmaxMatmulFunction.apply(s, split(v).contiguous(), keep_ppm, 8, block).transpose(1, 2).reshape(B, T, H)
        y = x + LinearFunction.apply(a, w["wo"], None, 8, block)
        h = LayerNormFunction.apply(y, p["g2"], p["b2"], 1e-5, True, keep_ppm)
        h = LinearFunction.apply(h, w["w1"], None, 8, block)
        h = LinearFunction.apply(GeluFunction.apply(h, gelu_bits, block), w["w2"], None, 8, block)
        return y + h
    h = F.layer_norm(x, (H,), p["g1"].to(x.dtype), p["b1"].to(x.dtype), 1e-5)
    q, k_, v = F.linear(h, p["wqkv"]).chunk(3, dim=-1)
    s = torch.matmul(split(q), split(k_).transpose(-1, -2)) / D ** 0.5
    a = torch.matmul(torch.softmax(s, -1), split(v)).transpose(1, 2).reshape(B, T, H)
    y = x + F.linear(a, p["wo"])
    h = F.layer_norm(y, (H,), p["g2"].to(x.dtype), p["b2"].to(x.dtype), 1e-5)
    h = F.linear(F.gelu(F.linear(h, p["w1"])), p["w2"])
    return y + h


def held_activation_bytes(fn) -> tuple:
    """(bytes that stay allocated between the forward pass of ``fn`` and its backward pass, apart from the output;
    milliseconds of forward + backward)."""
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    before = torch.cuda.memory_allocated()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    out = fn()
    torch.cuda.synchronize()
    kept = torch.cuda.memory_allocated() - before - out.numel() * out.element_size()
    out.sum().backward()
    t1.record()
    torch.cuda.synchronize()
    return kept, t0.elapsed_time(t1)
