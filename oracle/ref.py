"""ctypes loader for the CPU oracle (test infrastructure, not a product path).

Only tests, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg
may import this module.  It compiles ``slimfit_ref.c`` with gcc on first use
and wraps each ``slimfit_ref_*`` function for NumPy arrays.  bf16 tensors are
passed as ``uint16`` arrays of raw bit patterns.  Nothing here imports the HIP
package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "slimfit_ref.c")
_LIB = os.path.join(_HERE, "libslimfit_ref.so")
_lock = threading.Lock()
_lib = None

F32, BF16 = 0, 1
Q_FIXED, Q_BLOCK = 0, 1
PRUNE_TOPK, PRUNE_THRESHOLD = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle.  -O2, no fast-math, no FMA contraction."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    tmp = _LIB + ".tmp.%d" % os.getpid()
    cmd = ["gcc", "-std=c11", "-O2", "-fno-fast-math", "-ffp-contract=off",
           "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", tmp, _SRC,
           "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, _LIB)
    return _LIB


def lib():
    global _lib
    with _lock:
        if _lib is None:
            _lib = C.CDLL(build())
            for name in ("layer_delta", "quant_pack", "dequant_unpack",
                         "prune_scores", "restore_scores", "ils_select", "ils_select_blocks",
                         "ils_update", "freeze_count", "keep_count",
                         "prune_global", "restore_global", "gelu", "gelu_backward", "softmax_prune", "softmax_backward_pruned",
                         "layernorm_forward", "standardize", "layernorm_backward_pruned", "layernorm_param_grads", "layernorm_backward",
                         "splitmix64", "schedule_random", "schedule_progressive"):
                getattr(_lib, "slimfit_ref_" + name).restype = C.c_int
        return _lib


def host_threads() -> int:
    return len(os.sched_getaffinity(0))


def _dt(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError("expected float32 or uint16 (bf16 bits), got %s" % a.dtype)


def _ptr(a):
    return None if a is None else C.c_void_p(a.ctypes.data)


def _check(rc, what):
    if rc != 0:
        raise ValueError("oracle %s rejected its arguments (rc=%d)" % (what, rc))


def layer_delta(w_prev, w_cur, cur_is_delta=False, eps=0.0, threads=1):
    """Eq. 1 for a list of layers.  Returns float32[L]."""
    L = len(w_prev)
    assert len(w_cur) == L
    w_prev = [np.ascontiguousarray(w).reshape(-1) for w in w_prev]
    w_cur = [np.ascontiguousarray(w).reshape(-1) for w in w_cur]
    out = np.zeros(L, dtype=np.float32)
    if L == 0:
        return out
    pdt, cdt = _dt(w_prev[0]), _dt(w_cur[0])
    for a, b in zip(w_prev, w_cur):
        assert _dt(a) == pdt and _dt(b) == cdt and a.size == b.size
    numel = np.array([w.size for w in w_prev], dtype=np.int64)
    pp = (C.c_void_p * L)(*[w.ctypes.data for w in w_prev])
    pc = (C.c_void_p * L)(*[w.ctypes.data for w in w_cur])
    rc = lib().slimfit_ref_layer_delta(
        pp, C.c_int(pdt), pc, C.c_int(cdt), C.c_int(int(bool(cur_is_delta))),
        _ptr(numel), C.c_int(L), C.c_float(eps), _ptr(out), C.c_int(threads))
    _check(rc, "layer_delta")
    return out


def apply_update_layer_delta(w, delta, eps=0.0, threads=1):
    """Eq. 1 from (W^{t-1}, update) while the update is applied.  Returns (d float32[L], list of new weights);
    the inputs are left untouched."""
    L = len(w)
    assert len(delta) == L
    w = [np.array(a, copy=True).reshape(-1) for a in w]
    delta = [np.ascontiguousarray(a).reshape(-1) for a in delta]
    out = np.zeros(L, dtype=np.float32)
    if L == 0:
        return out, w
    wdt, ddt = _dt(w[0]), _dt(delta[0])
    for a, b in zip(w, delta):
        assert _dt(a) == wdt and _dt(b) == ddt and a.size == b.size
    numel = np.array([a.size for a in w], dtype=np.int64)
    pw = (C.c_void_p * L)(*[a.ctypes.data for a in w])
    pd = (C.c_void_p * L)(*[a.ctypes.data for a in delta])
    rc = lib().slimfit_ref_apply_update_layer_delta(
        pw, C.c_int(wdt), pd, C.c_int(ddt), _ptr(numel), C.c_int(L), C.c_float(eps), _ptr(out), C.c_int(threads))
    _check(rc, "apply_update_layer_delta")
    return out, w


def packed_bytes(n, bits):
    return (n * bits + 7) // 8


def num_blocks(n, block):
    return (n + block - 1) // block


def quant_pack(x, mode=Q_BLOCK, bits=4, block=64, frac_bits=0, threads=1):
    """Alg. 2 forward (+ per-block-scale mode).  Returns (codes, scales|None)."""
    x = np.ascontiguousarray(x).reshape(-1)
    n = x.size
    codes = np.zeros(packed_bytes(n, bits), dtype=np.uint8)
    scales = (np.zeros(num_blocks(n, block), dtype=np.float32)
              if mode == Q_BLOCK else None)
    rc = lib().slimfit_ref_quant_pack(
        _ptr(x), C.c_int(_dt(x)), C.c_int64(n), C.c_int(mode), C.c_int(bits),
        C.c_int(block), C.c_int(frac_bits), _ptr(codes), _ptr(scales),
        C.c_int(threads))
    _check(rc, "quant_pack")
    return codes, scales


def dequant_unpack(codes, scales, n, mode=Q_BLOCK, bits=4, block=64,
                   frac_bits=0, out_dtype=np.float32, threads=1):
    """Alg. 2 backward.  Returns float32[n] or uint16[n] (bf16 bits)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    if scales is not None:
        scales = np.ascontiguousarray(scales, dtype=np.float32)
    y = np.zeros(n, dtype=out_dtype)
    rc = lib().slimfit_ref_dequant_unpack(
        _ptr(codes), _ptr(scales), C.c_int64(n), C.c_int(mode), C.c_int(bits),
        C.c_int(block), C.c_int(frac_bits), _ptr(y), C.c_int(_dt(y)),
        C.c_int(threads))
    _check(rc, "dequant_unpack")
    return y


def prune_scores(p, k, mode=PRUNE_TOPK, tau=0.0, threads=1):
    """Alg. 5 pruning per row of a 2-D array.  Returns (vals, idx, counts)."""
    p = np.ascontiguousarray(p)
    assert p.ndim == 2
    rows, cols = p.shape
    vals = np.zeros((rows, k), dtype=p.dtype)
    idx = np.zeros((rows, k), dtype=np.uint16)
    counts = np.zeros(rows, dtype=np.int32)
    rc = lib().slimfit_ref_prune_scores(
        _ptr(p), C.c_int(_dt(p)), C.c_int64(rows), C.c_int(cols), C.c_int(k),
        C.c_int(mode), C.c_float(tau), _ptr(vals), _ptr(idx), _ptr(counts),
        C.c_int(threads))
    _check(rc, "prune_scores")
    return vals, idx, counts


def restore_scores(vals, idx, counts, cols, threads=1):
    """Alg. 5 restoring: zeros + scatter.  Returns a dense (rows, cols) array."""
    vals = np.ascontiguousarray(vals)
    idx = np.ascontiguousarray(idx, dtype=np.uint16)
    rows, k = vals.shape
    if counts is not None:
        counts = np.ascontiguousarray(counts, dtype=np.int32)
    out = np.empty((rows, cols), dtype=vals.dtype)
    rc = lib().slimfit_ref_restore_scores(
        _ptr(vals), _ptr(idx), _ptr(counts), C.c_int(_dt(vals)),
        C.c_int64(rows), C.c_int(cols), C.c_int(k), _ptr(out), C.c_int(threads))
    _check(rc, "restore_scores")
    return out


def prune_global(x, k, by_magnitude=True):
    """Alg. 5 on the flattened tensor.  Returns (vals[k], idx int32[k]) in ascending index order."""
    x = np.ascontiguousarray(x).reshape(-1)
    vals = np.zeros(k, dtype=x.dtype)
    idx = np.zeros(k, dtype=np.int32)
    rc = lib().slimfit_ref_prune_global(_ptr(x), C.c_int(_dt(x)), C.c_int64(x.size), C.c_int64(k),
                                        C.c_int(int(bool(by_magnitude))), _ptr(vals), _ptr(idx))
    _check(rc, "prune_global")
    return vals, idx


def restore_global(vals, idx, n):
    """zeros(n) + scatter.  Returns the dense flat array."""
    vals = np.ascontiguousarray(vals)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    out = np.empty(n, dtype=vals.dtype)
    rc = lib().slimfit_ref_restore_global(_ptr(vals), _ptr(idx), C.c_int64(vals.size), C.c_int(_dt(vals)),
                                          C.c_int64(n), _ptr(out))
    _check(rc, "restore_global")
    return out


def softmax_prune(logits, k, want_probs=True, threads=1):
    """Row softmax (fp64, rounded to the logits' dtype) + Alg. 5 per row, the kept set decided on the
    logits.  Returns (probs | None, vals, idx)."""
    logits = np.ascontiguousarray(logits)
    assert logits.ndim == 2
    rows, cols = logits.shape
    probs = np.empty_like(logits) if want_probs else None
    vals = np.zeros((rows, k), dtype=logits.dtype)
    idx = np.zeros((rows, k), dtype=np.uint16)
    rc = lib().slimfit_ref_softmax_prune(_ptr(logits), C.c_int(_dt(logits)), C.c_int64(rows), C.c_int(cols),
                                         C.c_int(k), _ptr(probs), _ptr(vals), _ptr(idx), C.c_int(threads))
    _check(rc, "softmax_prune")
    return probs, vals, idx


def layernorm_forward(x, gamma, beta, eps=1e-5, threads=1):
    """Row LayerNorm in fp64 -> (y, mean, rstd) as float32; x is (rows, H) float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    rows, H = x.shape
    gamma = np.ascontiguousarray(gamma, dtype=np.float32)
    beta = np.ascontiguousarray(beta, dtype=np.float32)
    assert gamma.size == H and beta.size == H
    y = np.empty_like(x)
    mean = np.empty(rows, dtype=np.float32)
    rstd = np.empty(rows, dtype=np.float32)
    rc = lib().slimfit_ref_layernorm_forward(_ptr(x), _ptr(gamma), _ptr(beta), C.c_int64(rows), C.c_int(H),
                                             C.c_float(eps), _ptr(y), _ptr(mean), _ptr(rstd), C.c_int(threads))
    _check(rc, "layernorm_forward")
    return y, mean, rstd


def standardize(x, mean, rstd):
    """x~ = fl(fl(x - mean_r) * rstd_r) in fp32 (the values the fused pruner orders)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    rows, H = x.shape
    mean = np.ascontiguousarray(mean, dtype=np.float32)
    rstd = np.ascontiguousarray(rstd, dtype=np.float32)
    assert mean.size == rows and rstd.size == rows
    xs = np.empty_like(x)
    _check(lib().slimfit_ref_standardize(_ptr(x), _ptr(mean), _ptr(rstd), C.c_int64(rows), C.c_int(H), _ptr(xs)),
           "standardize")
    return xs


def layernorm_backward_pruned(vals, idx, rstd, gamma, dy):
    """Input gradient of a frozen LayerNorm from the kept (value, flat index) pairs of x~; dy is (rows, H)."""
    dy = np.ascontiguousarray(dy, dtype=np.float32)
    rows, H = dy.shape
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    rstd = np.ascontiguousarray(rstd, dtype=np.float32)
    gamma = np.ascontiguousarray(gamma, dtype=np.float32)
    assert vals.size == idx.size and rstd.size == rows and gamma.size == H
    dx = np.empty_like(dy)
    rc = lib().slimfit_ref_layernorm_backward_pruned(_ptr(vals), _ptr(idx), C.c_int64(vals.size), _ptr(rstd),
                                                     _ptr(gamma), _ptr(dy), C.c_int64(rows), C.c_int(H), _ptr(dx))
    _check(rc, "layernorm_backward_pruned")
    return dx


def layernorm_backward(x, mean, rstd, gamma, dy):
    """Input gradient of an active LayerNorm from x, the fp32 row statistics, gamma and dy; fp64."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    dy = np.ascontiguousarray(dy, dtype=np.float32)
    rows, H = x.shape
    mean = np.ascontiguousarray(mean, dtype=np.float32)
    rstd = np.ascontiguousarray(rstd, dtype=np.float32)
    gamma = np.ascontiguousarray(gamma, dtype=np.float32)
    assert dy.shape == x.shape and mean.size == rows and rstd.size == rows and gamma.size == H
    dx = np.empty_like(x)
    rc = lib().slimfit_ref_layernorm_backward(_ptr(x), _ptr(mean), _ptr(rstd), _ptr(gamma), _ptr(dy), C.c_int64(rows),
                                              C.c_int(H), _ptr(dx))
    _check(rc, "layernorm_backward")
    return dx


def layernorm_param_grads(x, mean, rstd, dy):
    """(dgamma, dbeta) of an active LayerNorm from x, the fp32 row statistics and dy; fp64 sums."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    dy = np.ascontiguousarray(dy, dtype=np.float32)
    rows, H = x.shape
    mean = np.ascontiguousarray(mean, dtype=np.float32)
    rstd = np.ascontiguousarray(rstd, dtype=np.float32)
    assert dy.shape == x.shape and mean.size == rows and rstd.size == rows
    dgamma = np.empty(H, dtype=np.float32)
    dbeta = np.empty(H, dtype=np.float32)
    rc = lib().slimfit_ref_layernorm_param_grads(_ptr(x), _ptr(mean), _ptr(rstd), _ptr(dy), C.c_int64(rows), C.c_int(H),
                                                 _ptr(dgamma), _ptr(dbeta))
    _check(rc, "layernorm_param_grads")
    return dgamma, dbeta


def softmax_backward_pruned(vals, idx, counts, dp, threads=1):
    """Softmax backward from the kept (value, column) pairs of every row; dp is (rows, cols).  Dense result."""
    dp = np.ascontiguousarray(dp)
    rows, cols = dp.shape
    vals = np.ascontiguousarray(vals)
    idx = np.ascontiguousarray(idx, dtype=np.uint16)
    k = vals.shape[1]
    assert vals.shape == (rows, k) and idx.shape == (rows, k) and vals.dtype == dp.dtype
    if counts is not None:
        counts = np.ascontiguousarray(counts, dtype=np.int32)
    ds = np.empty_like(dp)
    rc = lib().slimfit_ref_softmax_backward_pruned(_ptr(vals), _ptr(idx), _ptr(counts), _ptr(dp), C.c_int(_dt(dp)),
                                                   C.c_int64(rows), C.c_int(cols), C.c_int(k), _ptr(ds),
                                                   C.c_int(threads))
    _check(rc, "softmax_backward_pruned")
    return ds


def gelu(x):
    """Exact (erf) GELU in fp64, rounded to x's dtype."""
    x = np.ascontiguousarray(x).reshape(-1)
    y = np.empty_like(x)
    _check(lib().slimfit_ref_gelu(_ptr(x), C.c_int(_dt(x)), C.c_int64(x.size), _ptr(y)), "gelu")
    return y


def gelu_backward(xhat, dy):
    """dy * GELU'(xhat) in fp64; xhat float32 (dequantised cache), dy / result share a dtype."""
    xhat = np.ascontiguousarray(xhat, dtype=np.float32).reshape(-1)
    dy = np.ascontiguousarray(dy).reshape(-1)
    assert xhat.size == dy.size
    dx = np.empty_like(dy)
    rc = lib().slimfit_ref_gelu_backward(_ptr(xhat), _ptr(dy), C.c_int(_dt(dy)), C.c_int64(dy.size), _ptr(dx))
    _check(rc, "gelu_backward")
    return dx


def freeze_count(L, F):
    rc = lib().slimfit_ref_freeze_count(C.c_int(L), C.c_double(F))
    if rc < 0:
        raise ValueError("oracle freeze_count rejected its arguments")
    return rc


def keep_count(cols, keep_ppm):
    rc = lib().slimfit_ref_keep_count(C.c_int(cols), C.c_int(keep_ppm))
    if rc < 0:
        raise ValueError("oracle keep_count rejected its arguments")
    return rc


def ils_select(d, n_freeze):
    """Alg. 1 selection.  Returns (frozen_idx int32[n_freeze], mask uint8[L])."""
    d = np.ascontiguousarray(d, dtype=np.float32)
    L = d.size
    frozen = np.zeros(max(n_freeze, 0), dtype=np.int32)
    mask = np.zeros(L, dtype=np.uint8)
    rc = lib().slimfit_ref_ils_select(_ptr(d), C.c_int(L), C.c_int(n_freeze),
                                      _ptr(frozen), _ptr(mask))
    _check(rc, "ils_select")
    return frozen, mask


def ils_select_blocks(d, group, n_freeze):
    """ILS over blocks of `group` consecutive layers.  Returns (frozen_blocks int32[n_freeze], layer mask uint8[L])."""
    d = np.ascontiguousarray(d, dtype=np.float32)
    L = d.size
    frozen = np.zeros(max(n_freeze, 0), dtype=np.int32)
    mask = np.zeros(L, dtype=np.uint8)
    rc = lib().slimfit_ref_ils_select_blocks(_ptr(d), C.c_int(L), C.c_int(group), C.c_int(n_freeze),
                                             _ptr(frozen), _ptr(mask))
    _check(rc, "ils_select_blocks")
    return frozen, mask


def ils_update(d, new_scores, frozen_mask):
    """Only active layers take their new distance.  Returns the new vector."""
    d = np.array(d, dtype=np.float32)
    new_scores = np.ascontiguousarray(new_scores, dtype=np.float32)
    frozen_mask = np.ascontiguousarray(frozen_mask, dtype=np.uint8)
    assert d.size == new_scores.size == frozen_mask.size
    rc = lib().slimfit_ref_ils_update(_ptr(d), _ptr(new_scores),
                                      _ptr(frozen_mask), C.c_int(d.size))
    _check(rc, "ils_update")
    return d


def splitmix64(state, n):
    """n raw outputs of the SplitMix64 stream started at ``state``."""
    out = np.zeros(n, dtype=np.uint64)
    _check(lib().slimfit_ref_splitmix64(C.c_uint64(state), C.c_int(n), _ptr(out)), "splitmix64")
    return out


def schedule_random(L, n_freeze, seed, iteration):
    """Random freezing schedule.  Returns (frozen_idx int32[n_freeze] in draw order, mask uint8[L])."""
    frozen = np.zeros(max(n_freeze, 0), dtype=np.int32)
    mask = np.zeros(L, dtype=np.uint8)
    rc = lib().slimfit_ref_schedule_random(C.c_int(L), C.c_int(n_freeze), C.c_uint64(seed), C.c_uint64(iteration),
                                           _ptr(frozen), _ptr(mask))
    _check(rc, "schedule_random")
    return frozen, mask


def schedule_progressive(L, n_freeze):
    """Progressive freezing schedule: the earliest n_freeze layers."""
    frozen = np.zeros(max(n_freeze, 0), dtype=np.int32)
    mask = np.zeros(L, dtype=np.uint8)
    rc = lib().slimfit_ref_schedule_progressive(C.c_int(L), C.c_int(n_freeze), _ptr(frozen), _ptr(mask))
    _check(rc, "schedule_progressive")
    return frozen, mask
