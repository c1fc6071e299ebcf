"""Thin ctypes binding of ``libslimfit.so`` (see ``include/slimfit.h``).

Argument marshalling only: every step of the hot path runs in the library's
HIP kernels (or, for the ILS pair, in its host C++).  Functions carry the C
names without the ``slimfit_`` prefix and take torch tensors for device
buffers (inputs and caller-allocated outputs) and NumPy arrays / sequences for
host buffers.  Device work is enqueued on torch's current stream unless a
stream handle is given.  A non-zero status raises :class:`SlimfitError`.
There is no fallback: if the library has not been built, loading it raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libslimfit.so")

F32, BF16 = 0, 1
Q_FIXED, Q_BLOCK = 0, 1
PRUNE_TOPK, PRUNE_THRESHOLD = 0, 1
GLOBAL_TILE = 4096                 # SLIMFIT_GLOBAL_TILE: granularity of prune_global's tile pointers

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_ALIGNMENT, ERR_WORKSPACE, ERR_HIP, ERR_POINTER = range(7)

EXPORTS = (
    "slimfit_status_string", "slimfit_version", "slimfit_set_pointer_checks", "slimfit_stream_probe",
    "slimfit_layer_delta_workspace", "slimfit_layer_delta_plan",
    "slimfit_layer_delta_run", "slimfit_layer_delta", "slimfit_layer_delta_static", "slimfit_layer_delta_apply_run", "slimfit_apply_update_layer_delta",
    "slimfit_packed_bytes", "slimfit_num_blocks", "slimfit_quant_pack",
    "slimfit_dequant_unpack", "slimfit_gelu_quant_pack", "slimfit_gelu_backward_dequant", "slimfit_keep_count", "slimfit_prune_scores",
    "slimfit_restore_scores", "slimfit_softmax_prune", "slimfit_softmax_backward_pruned", "slimfit_prune_global_workspace", "slimfit_global_tile_ptr_len", "slimfit_prune_global",
    "slimfit_restore_global", "slimfit_layernorm_forward", "slimfit_prune_global_standardized",
    "slimfit_layernorm_backward_pruned", "slimfit_layernorm_forward_quant_pack", "slimfit_layernorm_backward_dequant", "slimfit_layernorm_backward", "slimfit_layernorm_param_grads_workspace", "slimfit_layernorm_param_grads",
    "slimfit_freeze_count", "slimfit_ils_select", "slimfit_ils_select_blocks",
    "slimfit_ils_update", "slimfit_schedule_random", "slimfit_schedule_progressive",
)


class SlimfitError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, status_string(status), status))


def _require(ok: bool) -> None:
    """Shape, size and dtype agreement of the tensors handed to a wrapper.

    The C side can only check a pointer against its enclosing allocation, which under torch's caching allocator
    is a segment shared by many tensors: an output tensor that is too small has to be caught here."""
    if not ok:
        raise ValueError("tensor arguments do not agree in shape or dtype with what the call expects")


_lib = None


def is_built() -> bool:
    return os.path.exists(LIB_PATH)


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not is_built():
            raise RuntimeError(
                "libslimfit.so is missing: build it with "
                "`python -m paper_2305_18513_amd.build` (there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        L.slimfit_status_string.restype = C.c_char_p
        L.slimfit_status_string.argtypes = [C.c_int32]
        L.slimfit_packed_bytes.restype = C.c_size_t
        L.slimfit_packed_bytes.argtypes = [C.c_int64, C.c_int32]
        L.slimfit_num_blocks.restype = C.c_int64
        L.slimfit_num_blocks.argtypes = [C.c_int64, C.c_int32]
        L.slimfit_freeze_count.argtypes = [C.c_int32, C.c_double]
        for name in EXPORTS:
            fn = getattr(L, name)
            if fn.restype is C.c_int:          # ctypes default
                fn.restype = C.c_int32
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().slimfit_status_string(C.c_int32(status)).decode()


def _check(rc: int, where: str) -> None:
    if rc != OK:
        raise SlimfitError(rc, where)


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("expected float32 or bfloat16, got %s" % t.dtype)


def _dev(t: Optional[torch.Tensor]):
    """Raw device address of a contiguous tensor (None -> NULL)."""
    if t is None:
        return C.c_void_p(0)
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return C.c_void_p(t.data_ptr())


_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream(stream) -> C.c_void_p:
    """The hipStream_t to launch on: the caller's, else torch's current stream on the current device."""
    if stream is None:
        # the raw handle straight from torch (0.3 us) where this torch has the call; building a Stream object
        # to read its handle costs 3 us, a third of a whole call
        if _raw_stream is not None:
            stream = _raw_stream(torch.cuda.current_device())
        else:
            stream = torch.cuda.current_stream().cuda_stream
    return C.c_void_p(int(stream))


def version() -> int:
    return lib().slimfit_version()


def set_pointer_checks(on: bool) -> bool:
    return bool(lib().slimfit_set_pointer_checks(C.c_int32(int(bool(on)))))


# ---------------------------------------------------------------- (a) Eq. 1

def _numel_array(numel: Sequence[int]):
    return np.ascontiguousarray(np.asarray(numel, dtype=np.int64))


def layer_delta_workspace(numel: Sequence[int]) -> int:
    n = _numel_array(numel)
    out = C.c_size_t(0)
    rc = lib().slimfit_layer_delta_workspace(C.c_int32(n.size), C.c_void_p(n.ctypes.data), C.byref(out))
    _check(rc, "layer_delta_workspace")
    return int(out.value)


def _same_dtype(tensors: Sequence[torch.Tensor]) -> bool:
    """The C ABI applies one dtype to every layer of a list."""
    return all(t.dtype == tensors[0].dtype for t in tensors)


def _layer_lists_ok(a: Sequence[torch.Tensor], b: Sequence[torch.Tensor]) -> bool:
    return (len(a) == len(b) and (not a or (_same_dtype(a) and _same_dtype(b)))
            and all(x.numel() == y.numel() for x, y in zip(a, b)))


def _ptr_array(tensors: Sequence[torch.Tensor]):
    for t in tensors:
        if not t.is_contiguous():
            raise ValueError("tensor must be contiguous")
    return (C.c_void_p * max(1, len(tensors)))(*[t.data_ptr() for t in tensors])


def layer_delta_plan(w_prev: Sequence[torch.Tensor], w_cur: Sequence[torch.Tensor],
                     workspace: torch.Tensor, stream=None) -> None:
    L = len(w_prev)
    _require(_layer_lists_ok(w_prev, w_cur))
    numel = _numel_array([t.numel() for t in w_prev])
    pdt = _dt(w_prev[0]) if L else F32
    cdt = _dt(w_cur[0]) if L else F32
    rc = lib().slimfit_layer_delta_plan(
        _ptr_array(w_prev), C.c_int32(pdt), _ptr_array(w_cur), C.c_int32(cdt),
        C.c_void_p(numel.ctypes.data), C.c_int32(L), _dev(workspace),
        C.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream))
    _check(rc, "layer_delta_plan")


def layer_delta_run(numel: Sequence[int], prev_dt: int, cur_dt: int, cur_is_delta: bool,
                    eps: float, d_out: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    n = _numel_array(numel)
    _require(d_out.dtype == torch.float32 and d_out.numel() >= n.size)
    rc = lib().slimfit_layer_delta_run(
        C.c_void_p(n.ctypes.data), C.c_int32(n.size), C.c_int32(prev_dt), C.c_int32(cur_dt),
        C.c_int32(int(bool(cur_is_delta))), C.c_float(eps), _dev(d_out), _dev(workspace),
        C.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream))
    _check(rc, "layer_delta_run")


def layer_delta(w_prev: Sequence[torch.Tensor], w_cur: Sequence[torch.Tensor], cur_is_delta: bool,
                eps: float, d_out: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    L = len(w_prev)
    _require(_layer_lists_ok(w_prev, w_cur))
    numel = _numel_array([t.numel() for t in w_prev])
    pdt = _dt(w_prev[0]) if L else F32
    cdt = _dt(w_cur[0]) if L else F32
    _require(d_out.dtype == torch.float32 and d_out.numel() >= L)
    rc = lib().slimfit_layer_delta(
        _ptr_array(w_prev), C.c_int32(pdt), _ptr_array(w_cur), C.c_int32(cdt),
        C.c_int32(int(bool(cur_is_delta))), C.c_void_p(numel.ctypes.data), C.c_int32(L),
        C.c_float(eps), _dev(d_out), _dev(workspace),
        C.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream))
    _check(rc, "layer_delta")


LAYER_DELTA_STATIC_BYTES = 1 << 20     # SLIMFIT_LAYER_DELTA_STATIC_BYTES


def layer_delta_static(w_prev: Sequence[torch.Tensor], w_cur: Sequence[torch.Tensor], cur_is_delta: bool,
                       eps: float, d_out: torch.Tensor, stream=None) -> None:
    """layer_delta on the library's own fixed scratch array: no workspace, no allocation."""
    L = len(w_prev)
    _require(_layer_lists_ok(w_prev, w_cur))
    numel = _numel_array([t.numel() for t in w_prev])
    pdt = _dt(w_prev[0]) if L else F32
    cdt = _dt(w_cur[0]) if L else F32
    _require(d_out.dtype == torch.float32 and d_out.numel() >= L)
    rc = lib().slimfit_layer_delta_static(
        _ptr_array(w_prev), C.c_int32(pdt), _ptr_array(w_cur), C.c_int32(cdt),
        C.c_int32(int(bool(cur_is_delta))), C.c_void_p(numel.ctypes.data), C.c_int32(L),
        C.c_float(eps), _dev(d_out), _stream(stream))
    _check(rc, "layer_delta_static")


def layer_delta_apply_run(numel: Sequence[int], w_dt: int, delta_dt: int, eps: float, d_out: torch.Tensor,
                          workspace: torch.Tensor, stream=None) -> None:
    """Score + apply on a plan made by layer_delta_plan(weights, updates); overwrites the planned weights."""
    n = _numel_array(numel)
    _require(d_out.dtype == torch.float32 and d_out.numel() >= n.size)
    rc = lib().slimfit_layer_delta_apply_run(
        C.c_void_p(n.ctypes.data), C.c_int32(n.size), C.c_int32(w_dt), C.c_int32(delta_dt), C.c_float(eps),
        _dev(d_out), _dev(workspace), C.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream))
    _check(rc, "layer_delta_apply_run")


def apply_update_layer_delta(w: Sequence[torch.Tensor], delta: Sequence[torch.Tensor], eps: float,
                             d_out: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    """d_out[i] = mean |delta_i / w_i| and w_i += delta_i, one pass over both."""
    L = len(w)
    _require(_layer_lists_ok(w, delta))
    numel = _numel_array([t.numel() for t in w])
    wdt = _dt(w[0]) if L else F32
    ddt = _dt(delta[0]) if L else F32
    _require(d_out.dtype == torch.float32 and d_out.numel() >= L)
    rc = lib().slimfit_apply_update_layer_delta(
        _ptr_array(w), C.c_int32(wdt), _ptr_array(delta), C.c_int32(ddt), C.c_void_p(numel.ctypes.data),
        C.c_int32(L), C.c_float(eps), _dev(d_out), _dev(workspace),
        C.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream))
    _check(rc, "apply_update_layer_delta")


def stream_probe_bytes(in_vecs: int, ratio: int) -> int:
    """Bytes slimfit_stream_probe writes for in_vecs source vectors."""
    if ratio > 0:
        return in_vecs * (16 // ratio)
    if ratio == 0:
        return (in_vecs + 1023) // 1024 * 16
    return in_vecs * (-ratio) * 16


def stream_probe(src: torch.Tensor, dst: torch.Tensor, ratio: int, stream=None) -> None:
    """Diagnostic streaming kernel: shrinking (ratio 1..16), read-only (0) or growing (-2, -4, -8) traffic."""
    in_vecs = src.numel() * src.element_size() // 16
    _require(ratio in (1, 2, 4, 8, 16, 0, -2, -4, -8)
             and dst.numel() * dst.element_size() >= stream_probe_bytes(in_vecs, ratio))
    rc = lib().slimfit_stream_probe(_dev(src), _dev(dst), C.c_int64(in_vecs), C.c_int32(ratio), _stream(stream))
    _check(rc, "stream_probe")


# ---------------------------------------------------------------- (b) Alg. 2

def packed_bytes(n: int, bits: int) -> int:
    return int(lib().slimfit_packed_bytes(C.c_int64(n), C.c_int32(bits)))


def num_blocks(n: int, block: int) -> int:
    return int(lib().slimfit_num_blocks(C.c_int64(n), C.c_int32(block)))


def _cache_fits(n: int, mode: int, bits: int, block: int, codes: torch.Tensor, scales: Optional[torch.Tensor]) -> bool:
    """codes / scales hold what Alg. 2 writes for n elements (the C side rejects bad bits / block values)."""
    if codes.dtype != torch.uint8 or (scales is not None and scales.dtype != torch.float32):
        return False
    if bits in (4, 8) and codes.numel() < (n * bits + 7) // 8:
        return False
    if mode == Q_BLOCK and block in (32, 64, 128, 256) and (scales is None or scales.numel() < (n + block - 1) // block):
        return False
    return True


def quant_pack(x: torch.Tensor, mode: int, bits: int, block: int, frac_bits: int,
               codes: torch.Tensor, scales: Optional[torch.Tensor], stream=None) -> None:
    _require(_cache_fits(x.numel(), mode, bits, block, codes, scales))
    rc = lib().slimfit_quant_pack(
        _dev(x), C.c_int32(_dt(x)), C.c_int64(x.numel()), C.c_int32(mode), C.c_int32(bits),
        C.c_int32(block), C.c_int32(frac_bits), _dev(codes), _dev(scales), _stream(stream))
    _check(rc, "quant_pack")


def dequant_unpack(codes: torch.Tensor, scales: Optional[torch.Tensor], mode: int, bits: int,
                   block: int, frac_bits: int, y: torch.Tensor, stream=None) -> None:
    _require(_cache_fits(y.numel(), mode, bits, block, codes, scales))
    rc = lib().slimfit_dequant_unpack(
        _dev(codes), _dev(scales), C.c_int64(y.numel()), C.c_int32(mode), C.c_int32(bits),
        C.c_int32(block), C.c_int32(frac_bits), _dev(y), C.c_int32(_dt(y)), _stream(stream))
    _check(rc, "dequant_unpack")


# ---------------------------------------------------------------- (b') the cache fused into GELU

def gelu_quant_pack(x: torch.Tensor, mode: int, bits: int, block: int, frac_bits: int, y: torch.Tensor,
                    codes: torch.Tensor, scales: Optional[torch.Tensor], stream=None) -> None:
    """y = GELU(x) and (codes, scales) = quant_pack(x) in one pass over x."""
    _require(x.is_contiguous() and y.is_contiguous() and y.dtype == x.dtype and y.numel() == x.numel())
    _require(_cache_fits(x.numel(), mode, bits, block, codes, scales))
    rc = lib().slimfit_gelu_quant_pack(
        _dev(x), C.c_int32(_dt(x)), C.c_int64(x.numel()), C.c_int32(mode), C.c_int32(bits), C.c_int32(block),
        C.c_int32(frac_bits), _dev(y), _dev(codes), _dev(scales), _stream(stream))
    _check(rc, "gelu_quant_pack")


def gelu_backward_dequant(codes: torch.Tensor, scales: Optional[torch.Tensor], mode: int, bits: int, block: int,
                          frac_bits: int, dy: torch.Tensor, dx: torch.Tensor, stream=None) -> None:
    """dx = dy * GELU'(dequantised cache); the dequantised values stay in registers."""
    _require(dy.is_contiguous() and dx.is_contiguous() and dx.dtype == dy.dtype and dx.numel() == dy.numel())
    _require(_cache_fits(dx.numel(), mode, bits, block, codes, scales))
    rc = lib().slimfit_gelu_backward_dequant(
        _dev(codes), _dev(scales), C.c_int64(dx.numel()), C.c_int32(mode), C.c_int32(bits), C.c_int32(block),
        C.c_int32(frac_bits), _dev(dy), _dev(dx), C.c_int32(_dt(dx)), _stream(stream))
    _check(rc, "gelu_backward_dequant")


# ---------------------------------------------------------------- (c) Alg. 5

def keep_count(cols: int, keep_ppm: int) -> int:
    return int(lib().slimfit_keep_count(C.c_int32(cols), C.c_int32(keep_ppm)))


def prune_scores(p: torch.Tensor, k: int, mode: int, tau: float, vals: torch.Tensor,
                 idx: torch.Tensor, counts: Optional[torch.Tensor], stream=None) -> None:
    _require(p.dim() == 2 and vals.dtype == p.dtype and idx.dtype == torch.uint16)
    rows, cols = p.shape
    _require(k >= 0 and vals.numel() >= rows * k and idx.numel() >= rows * k)
    _require(counts is None or (counts.dtype == torch.int32 and counts.numel() >= rows))
    rc = lib().slimfit_prune_scores(
        _dev(p), C.c_int32(_dt(p)), C.c_int64(rows), C.c_int32(cols), C.c_int32(k),
        C.c_int32(mode), C.c_float(tau), _dev(vals), _dev(idx), _dev(counts), _stream(stream))
    _check(rc, "prune_scores")


def restore_scores(vals: torch.Tensor, idx: torch.Tensor, counts: Optional[torch.Tensor],
                   out: torch.Tensor, stream=None) -> None:
    _require(out.dim() == 2 and vals.dim() == 2 and vals.dtype == out.dtype and idx.dtype == torch.uint16)
    rows, cols = out.shape
    k = vals.shape[1]
    _require(vals.shape[0] >= rows and idx.numel() >= rows * k)
    _require(counts is None or (counts.dtype == torch.int32 and counts.numel() >= rows))
    rc = lib().slimfit_restore_scores(
        _dev(vals), _dev(idx), _dev(counts), C.c_int32(_dt(out)), C.c_int64(rows),
        C.c_int32(cols), C.c_int32(k), _dev(out), _stream(stream))
    _check(rc, "restore_scores")


def softmax_prune(logits: torch.Tensor, k: int, probs: torch.Tensor, vals: torch.Tensor, idx: torch.Tensor,
                  stream=None) -> None:
    """probs = softmax(logits) per row; (vals, idx) = the k largest of every row (decided on the logits)."""
    _require(logits.dim() == 2 and logits.is_contiguous() and probs.is_contiguous())
    _require(probs.shape == logits.shape and probs.dtype == logits.dtype)
    _require(vals.dtype == logits.dtype and idx.dtype == torch.uint16)
    rows, cols = logits.shape
    _require(k >= 0 and vals.numel() >= rows * k and idx.numel() >= rows * k)
    rc = lib().slimfit_softmax_prune(
        _dev(logits), C.c_int32(_dt(logits)), C.c_int64(rows), C.c_int32(cols), C.c_int32(k),
        _dev(probs), _dev(vals), _dev(idx), _stream(stream))
    _check(rc, "softmax_prune")


def softmax_backward_pruned(vals: torch.Tensor, idx: torch.Tensor, counts: Optional[torch.Tensor],
                            dp: torch.Tensor, ds: torch.Tensor, stream=None) -> None:
    """ds = p^ * (dp - sum(p^ * dp)) per row, p^ being the rows that restore_scores would rebuild."""
    _require(dp.dim() == 2 and dp.is_contiguous() and ds.is_contiguous())
    _require(ds.shape == dp.shape and ds.dtype == dp.dtype)
    _require(vals.dim() == 2 and vals.dtype == dp.dtype and idx.dtype == torch.uint16 and vals.shape == idx.shape)
    rows, cols = dp.shape
    k = vals.shape[1]
    _require(vals.shape[0] >= rows and (counts is None or (counts.dtype == torch.int32 and counts.numel() >= rows)))
    rc = lib().slimfit_softmax_backward_pruned(
        _dev(vals), _dev(idx), _dev(counts), _dev(dp), C.c_int32(_dt(dp)), C.c_int64(rows),
        C.c_int32(cols), C.c_int32(k), _dev(ds), _stream(stream))
    _check(rc, "softmax_backward_pruned")


# ---------------------------------------------------------------- (c') Alg. 5, whole tensor

def _own_workspace(workspace: Optional[torch.Tensor], nbytes: int, device, stream) -> torch.Tensor:
    """A workspace the wrapper allocates is only safe on torch's current stream (whose allocator then keeps the
    block until the kernels are through); with an explicit stream the caller has to own it."""
    if workspace is not None:
        _require(workspace.dtype == torch.uint8)        # its size goes to the C side, which compares it with the need
        return workspace
    if stream is not None:
        raise ValueError("pass a workspace tensor when launching on an explicit stream")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def prune_global_workspace(n: int) -> int:
    out = C.c_size_t(0)
    _check(lib().slimfit_prune_global_workspace(C.c_int64(n), C.byref(out)), "prune_global_workspace")
    return int(out.value)


def global_tile_ptr_len(n: int) -> int:
    fn = lib().slimfit_global_tile_ptr_len
    fn.restype = C.c_int64
    return int(fn(C.c_int64(n)))


def prune_global(x: torch.Tensor, k: int, vals: torch.Tensor, idx: torch.Tensor, by_magnitude: bool = True,
                 tile_ptr: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                 stream=None) -> None:
    """Keeps the k largest entries of the flattened ``x``; ``workspace`` is a uint8 device tensor."""
    _require(x.is_contiguous() and vals.dtype == x.dtype and idx.dtype == torch.int32)
    _require(vals.numel() >= k and idx.numel() >= k)
    n = x.numel()
    _require(tile_ptr is None or (tile_ptr.dtype == torch.int32 and tile_ptr.numel() >= global_tile_ptr_len(n)))
    workspace = _own_workspace(workspace, prune_global_workspace(n), x.device, stream)
    rc = lib().slimfit_prune_global(
        _dev(x), C.c_int32(_dt(x)), C.c_int64(n), C.c_int64(k), C.c_int32(int(bool(by_magnitude))),
        _dev(vals), _dev(idx), _dev(tile_ptr), _dev(workspace), C.c_size_t(workspace.numel()), _stream(stream))
    _check(rc, "prune_global")


def restore_global(vals: torch.Tensor, idx: torch.Tensor, k: int, out: torch.Tensor,
                   tile_ptr: Optional[torch.Tensor] = None, stream=None) -> None:
    _require(out.is_contiguous() and vals.dtype == out.dtype and idx.dtype == torch.int32)
    _require(tile_ptr is None or tile_ptr.dtype == torch.int32)
    rc = lib().slimfit_restore_global(
        _dev(vals), _dev(idx), _dev(tile_ptr), C.c_int64(k), C.c_int32(_dt(out)), C.c_int64(out.numel()),
        _dev(out), _stream(stream))
    _check(rc, "restore_global")


# ---------------------------------------------------------------- (c-ln) LayerNorm around the pruned cache

def layernorm_forward(x: torch.Tensor, gamma: torch.Tensor, beta: torch.Tensor, eps: float, y: torch.Tensor,
                      mean: torch.Tensor, rstd: torch.Tensor, stream=None) -> None:
    _require(x.dim() == 2 and x.is_contiguous() and y.is_contiguous() and y.shape == x.shape and y.dtype == x.dtype)
    _require(all(t.dtype == torch.float32 for t in (gamma, beta, mean, rstd)))
    rows, H = x.shape
    _require(gamma.numel() == H and beta.numel() == H and mean.numel() >= rows and rstd.numel() >= rows)
    rc = lib().slimfit_layernorm_forward(_dev(x), C.c_int32(_dt(x)), _dev(gamma), _dev(beta), C.c_int64(rows),
                                         C.c_int64(H), C.c_float(eps), _dev(y), _dev(mean), _dev(rstd),
                                         _stream(stream))
    _check(rc, "layernorm_forward")


def prune_global_standardized(x: torch.Tensor, mean: torch.Tensor, rstd: torch.Tensor, k: int, vals: torch.Tensor,
                              idx: torch.Tensor, by_magnitude: bool = True, tile_ptr: Optional[torch.Tensor] = None,
                              row_ptr: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                              stream=None) -> None:
    """prune_global of the standardised rows of ``x`` (rows, H), formed on the fly from mean / rstd."""
    _require(x.dim() == 2 and x.is_contiguous() and vals.dtype == torch.float32 and idx.dtype == torch.int32)
    _require(mean.dtype == torch.float32 and rstd.dtype == torch.float32)
    rows, H = x.shape
    n = x.numel()
    _require(mean.numel() >= rows and rstd.numel() >= rows and vals.numel() >= k and idx.numel() >= k)
    _require(tile_ptr is None or (tile_ptr.dtype == torch.int32 and tile_ptr.numel() >= global_tile_ptr_len(n)))
    _require(row_ptr is None or (row_ptr.dtype == torch.int32 and row_ptr.numel() >= rows + 1))
    workspace = _own_workspace(workspace, prune_global_workspace(n), x.device, stream)
    rc = lib().slimfit_prune_global_standardized(
        _dev(x), C.c_int32(_dt(x)), C.c_int64(n), C.c_int64(H), _dev(mean), _dev(rstd), C.c_int64(k),
        C.c_int32(int(bool(by_magnitude))), _dev(vals), _dev(idx), _dev(tile_ptr), _dev(row_ptr), _dev(workspace),
        C.c_size_t(workspace.numel()), _stream(stream))
    _check(rc, "prune_global_standardized")


def layernorm_backward(x: torch.Tensor, mean: torch.Tensor, rstd: torch.Tensor, gamma: torch.Tensor,
                       dy: torch.Tensor, dx: torch.Tensor, stream=None) -> None:
    """Input gradient of an active LayerNorm (every standardised input present)."""
    _require(x.dim() == 2 and x.is_contiguous() and dy.is_contiguous() and dx.is_contiguous())
    _require(dy.shape == x.shape and dx.shape == x.shape and dy.dtype == x.dtype and dx.dtype == x.dtype)
    _require(all(t.dtype == torch.float32 for t in (mean, rstd, gamma)))
    rows, H = x.shape
    _require(mean.numel() >= rows and rstd.numel() >= rows and gamma.numel() == H)
    rc = lib().slimfit_layernorm_backward(_dev(x), C.c_int32(_dt(x)), _dev(mean), _dev(rstd), _dev(gamma), _dev(dy),
                                          C.c_int64(rows), C.c_int64(H), _dev(dx), _stream(stream))
    _check(rc, "layernorm_backward")


def layernorm_forward_quant_pack(x: torch.Tensor, gamma: torch.Tensor, beta: torch.Tensor, eps: float, bits: int,
                                 block: int, y: torch.Tensor, mean: torch.Tensor, rstd: torch.Tensor,
                                 codes: torch.Tensor, scales: torch.Tensor, stream=None) -> None:
    """layernorm_forward plus, from the same read of x, the codes and scales of quant_pack(x) in BLOCK mode."""
    _require(x.dim() == 2 and x.is_contiguous() and y.is_contiguous() and y.shape == x.shape)
    _require(all(t.dtype == torch.float32 for t in (gamma, beta, mean, rstd, scales)) and codes.dtype == torch.uint8)
    _require(y.dtype == x.dtype)
    rows, H = x.shape
    _require(gamma.numel() == H and beta.numel() == H and mean.numel() >= rows and rstd.numel() >= rows)
    _require(codes.numel() >= rows * H * bits // 8 and scales.numel() >= rows * H // max(block, 1))
    rc = lib().slimfit_layernorm_forward_quant_pack(
        _dev(x), C.c_int32(_dt(x)), _dev(gamma), _dev(beta), C.c_int64(rows), C.c_int64(H), C.c_float(eps), C.c_int32(bits),
        C.c_int32(block), _dev(y), _dev(mean), _dev(rstd), _dev(codes), _dev(scales), _stream(stream))
    _check(rc, "layernorm_forward_quant_pack")


def layernorm_backward_dequant(codes: torch.Tensor, scales: torch.Tensor, bits: int, block: int, mean: torch.Tensor,
                               rstd: torch.Tensor, gamma: torch.Tensor, dy: torch.Tensor, dx: torch.Tensor,
                               stream=None) -> None:
    """Input gradient of a LayerNorm whose input was cached by layernorm_forward_quant_pack."""
    _require(dy.dim() == 2 and dy.is_contiguous() and dx.is_contiguous() and dx.shape == dy.shape)
    _require(all(t.dtype == torch.float32 for t in (scales, mean, rstd, gamma)) and codes.dtype == torch.uint8)
    _require(dx.dtype == dy.dtype)
    rows, H = dy.shape
    _require(gamma.numel() == H and mean.numel() >= rows and rstd.numel() >= rows)
    _require(codes.numel() >= rows * H * bits // 8 and scales.numel() >= rows * H // max(block, 1))
    rc = lib().slimfit_layernorm_backward_dequant(
        _dev(codes), _dev(scales), C.c_int32(bits), C.c_int32(block), _dev(mean), _dev(rstd), _dev(gamma), _dev(dy),
        C.c_int32(_dt(dy)), C.c_int64(rows), C.c_int64(H), _dev(dx), _stream(stream))
    _check(rc, "layernorm_backward_dequant")


def layernorm_param_grads(x: torch.Tensor, mean: torch.Tensor, rstd: torch.Tensor, dy: torch.Tensor,
                          dgamma: torch.Tensor, dbeta: torch.Tensor, workspace: Optional[torch.Tensor] = None,
                          stream=None) -> None:
    """gamma^ and beta^ of an active LayerNorm: column sums over the rows of ``x`` / ``dy`` (rows, H)."""
    _require(x.dim() == 2 and x.is_contiguous() and dy.is_contiguous() and dy.shape == x.shape and dy.dtype == x.dtype)
    _require(all(t.dtype == torch.float32 for t in (mean, rstd, dgamma, dbeta)))
    rows, H = x.shape
    _require(mean.numel() >= rows and rstd.numel() >= rows and dgamma.numel() == H and dbeta.numel() == H)
    need = C.c_size_t(0)
    _check(lib().slimfit_layernorm_param_grads_workspace(C.c_int64(rows), C.c_int64(H), C.byref(need)),
           "layernorm_param_grads_workspace")
    workspace = _own_workspace(workspace, int(need.value), x.device, stream)
    rc = lib().slimfit_layernorm_param_grads(
        _dev(x), C.c_int32(_dt(x)), _dev(mean), _dev(rstd), _dev(dy), C.c_int64(rows), C.c_int64(H), _dev(dgamma),
        _dev(dbeta),
        _dev(workspace), C.c_size_t(workspace.numel()), _stream(stream))
    _check(rc, "layernorm_param_grads")


def layernorm_backward_pruned(vals: torch.Tensor, idx: torch.Tensor, row_ptr: torch.Tensor, k: int,
                              rstd: torch.Tensor, gamma: torch.Tensor, dy: torch.Tensor, dx: torch.Tensor,
                              stream=None) -> None:
    _require(dy.dim() == 2 and dy.is_contiguous() and dx.is_contiguous() and dx.shape == dy.shape)
    _require(all(t.dtype == torch.float32 for t in (vals, rstd, gamma)) and dx.dtype == dy.dtype)
    _require(idx.dtype == torch.int32 and row_ptr.dtype == torch.int32)
    rows, H = dy.shape
    _require(row_ptr.numel() >= rows + 1)
    rc = lib().slimfit_layernorm_backward_pruned(
        _dev(vals), _dev(idx), _dev(row_ptr), C.c_int64(k), _dev(rstd), _dev(gamma), _dev(dy), C.c_int32(_dt(dy)),
        C.c_int64(rows), C.c_int64(H), _dev(dx), _stream(stream))
    _check(rc, "layernorm_backward_pruned")


# ---------------------------------------------------------------- (d) Alg. 1 (host)

def freeze_count(L: int, F: float) -> int:
    return int(lib().slimfit_freeze_count(C.c_int32(L), C.c_double(F)))


def ils_select(d: np.ndarray, n_freeze: int):
    """Returns (frozen_idx int32[n_freeze], mask uint8[L])."""
    d = np.ascontiguousarray(d, dtype=np.float32)
    frozen = np.zeros(max(n_freeze, 0), dtype=np.int32)
    mask = np.zeros(d.size, dtype=np.uint8)
    rc = lib().slimfit_ils_select(C.c_void_p(d.ctypes.data), C.c_int32(d.size), C.c_int32(n_freeze),
                                  C.c_void_p(frozen.ctypes.data), C.c_void_p(mask.ctypes.data))
    _check(rc, "ils_select")
    return frozen, mask


def ils_select_blocks(d: np.ndarray, group: int, n_freeze: int):
    """ILS over blocks of ``group`` consecutive layers.  Returns (frozen_blocks int32[n_freeze], layer mask uint8[L])."""
    d = np.ascontiguousarray(d, dtype=np.float32)
    frozen = np.zeros(max(n_freeze, 0), dtype=np.int32)
    mask = np.zeros(d.size, dtype=np.uint8)
    rc = lib().slimfit_ils_select_blocks(C.c_void_p(d.ctypes.data), C.c_int32(d.size), C.c_int32(group),
                                         C.c_int32(n_freeze), C.c_void_p(frozen.ctypes.data),
                                         C.c_void_p(mask.ctypes.data))
    _check(rc, "ils_select_blocks")
    return frozen, mask


def ils_update(d: np.ndarray, new_scores: np.ndarray, frozen_mask: np.ndarray) -> np.ndarray:
    """In place on ``d`` (float32, contiguous); returns it."""
    _require(d.dtype == np.float32 and d.flags.c_contiguous)
    new_scores = np.ascontiguousarray(new_scores, dtype=np.float32)
    frozen_mask = np.ascontiguousarray(frozen_mask, dtype=np.uint8)
    _require(d.size == new_scores.size == frozen_mask.size)
    rc = lib().slimfit_ils_update(C.c_void_p(d.ctypes.data), C.c_void_p(new_scores.ctypes.data),
                                  C.c_void_p(frozen_mask.ctypes.data), C.c_int32(d.size))
    _check(rc, "ils_update")
    return d


def schedule_random(L: int, n_freeze: int, seed: int, iteration: int):
    """Random freezing schedule.  Returns (frozen_idx int32[n_freeze] in draw order, mask uint8[L])."""
    frozen = np.zeros(max(n_freeze, 0), dtype=np.int32)
    mask = np.zeros(max(L, 0), dtype=np.uint8)
    rc = lib().slimfit_schedule_random(C.c_int32(L), C.c_int32(n_freeze), C.c_uint64(seed), C.c_uint64(iteration),
                                       C.c_void_p(frozen.ctypes.data), C.c_void_p(mask.ctypes.data))
    _check(rc, "schedule_random")
    return frozen, mask


def schedule_progressive(L: int, n_freeze: int):
    """Progressive freezing schedule: the earliest n_freeze layers."""
    frozen = np.zeros(max(n_freeze, 0), dtype=np.int32)
    mask = np.zeros(max(L, 0), dtype=np.uint8)
    rc = lib().slimfit_schedule_progressive(C.c_int32(L), C.c_int32(n_freeze), C.c_void_p(frozen.ctypes.data),
                                            C.c_void_p(mask.ctypes.data))
    _check(rc, "schedule_progressive")
    return frozen, mask
