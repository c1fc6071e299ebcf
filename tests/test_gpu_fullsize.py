"""GPU parity at the full sizes of workload configurations 1-4, in the launch
configuration bench.py times (same calls, same shapes), one encoder block per
config, every output element compared with the oracle."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2305_18513_amd import binding as sf
from paper_2305_18513_amd import synth
from tests.gpu_util import require_gpu, to_np

pytestmark = pytest.mark.gpu
THREADS = 16


def _eq(a, b):
    assert a.shape == b.shape and a.dtype == b.dtype
    if a.dtype == np.float32:
        a, b = a.view(np.uint32), b.view(np.uint32)
    if not np.array_equal(a, b):
        bad = np.flatnonzero(a.reshape(-1) != b.reshape(-1))
        raise AssertionError("%d of %d elements differ, first at %d" % (bad.size, a.size, bad[0]))


@pytest.mark.parametrize("ci", [1, 2, 3, 4])
@pytest.mark.parametrize("kind", ["gelu_in", "ln_in"])
def test_quant_dequant_full_tensor(ci, kind):
    require_gpu()
    cfg = synth.CONFIGS[ci]
    x = synth.activation(cfg, kind, "cuda", 0).reshape(-1)
    n = x.numel()
    assert n == (cfg.gelu_in_numel if kind == "gelu_in" else cfg.ln_in_numel)
    xh = to_np(x)
    for bits in cfg.quant_bits:
        block = cfg.quant_block
        codes = torch.empty(sf.packed_bytes(n, bits), dtype=torch.uint8, device="cuda")
        scales = torch.empty(sf.num_blocks(n, block), dtype=torch.float32, device="cuda")
        y = torch.empty_like(x)
        sf.quant_pack(x, sf.Q_BLOCK, bits, block, 0, codes, scales)
        sf.dequant_unpack(codes, scales, sf.Q_BLOCK, bits, block, 0, y)
        torch.cuda.synchronize()
        oc, osc = ref.quant_pack(xh, mode=ref.Q_BLOCK, bits=bits, block=block, threads=THREADS)
        _eq(to_np(codes), oc)
        _eq(to_np(scales), osc)
        oy = ref.dequant_unpack(oc, osc, n, mode=ref.Q_BLOCK, bits=bits, block=block,
                                out_dtype=xh.dtype, threads=THREADS)
        _eq(to_np(y), oy)
        # the stated invariant of the path: round-trip error at most half a step per block
        # (plus the fp32 roundings of inv, the product, scale and the dequantising multiply:
        #  four relative errors of 2^-24 on a value of at most qmax steps)
        if xh.dtype == np.float32:
            qmax = 2 ** (bits - 1) - 1
            err = np.abs(xh.astype(np.float64) - oy.astype(np.float64)).reshape(-1, block)
            assert np.all(err.max(axis=1) <= osc.astype(np.float64) * (0.5 + qmax * 2.0 ** -22 * 1.01))
        del codes, scales, y


@pytest.mark.parametrize("ci", [1, 3])
def test_paper_fixed_point_4p4_full_tensor(ci):
    # the paper's own format: 8 bits, 4 integer + 4 fractional (Sec. 4, Alg. 2)
    require_gpu()
    cfg = synth.CONFIGS[ci]
    x = synth.activation(cfg, "gelu_in", "cuda", 1).reshape(-1)
    n = x.numel()
    codes = torch.empty(n, dtype=torch.uint8, device="cuda")
    y = torch.empty_like(x)
    sf.quant_pack(x, sf.Q_FIXED, 8, 64, 4, codes, None)
    sf.dequant_unpack(codes, None, sf.Q_FIXED, 8, 64, 4, y)
    torch.cuda.synchronize()
    xh = to_np(x)
    oc, _ = ref.quant_pack(xh, mode=ref.Q_FIXED, bits=8, frac_bits=4, threads=THREADS)
    _eq(to_np(codes), oc)
    _eq(to_np(y), ref.dequant_unpack(oc, None, n, mode=ref.Q_FIXED, bits=8, frac_bits=4, threads=THREADS))


@pytest.mark.parametrize("ci", [1, 3])
def test_paper_placement_8bit_fixed_point_on_attention_probabilities(ci):
    # the paper caches the Softmax/MatMul operand in 8 bits (Sec. 5); its format is Alg. 2's 4.4
    require_gpu()
    cfg = synth.CONFIGS[ci]
    p = synth.attention_scores(cfg, "cuda", 0).reshape(-1)
    n = p.numel()
    codes = torch.empty(n, dtype=torch.uint8, device="cuda")
    y = torch.empty_like(p)
    sf.quant_pack(p, sf.Q_FIXED, 8, 64, 4, codes, None)
    sf.dequant_unpack(codes, None, sf.Q_FIXED, 8, 64, 4, y)
    torch.cuda.synchronize()
    ph = to_np(p)
    oc, _ = ref.quant_pack(ph, mode=ref.Q_FIXED, bits=8, frac_bits=4, threads=THREADS)
    _eq(to_np(codes), oc)
    oy = ref.dequant_unpack(oc, None, n, mode=ref.Q_FIXED, bits=8, frac_bits=4, threads=THREADS)
    _eq(to_np(y), oy)
    assert np.abs(ph.astype(np.float64) - oy).max() <= 1.0 / 32      # in range: half a step of 1/16


@pytest.mark.parametrize("ci", [1, 2, 3, 4])
def test_prune_full_tensor(ci):
    require_gpu()
    cfg = synth.CONFIGS[ci]
    p = synth.attention_scores(cfg, "cuda", 0)
    rows, cols = p.shape
    assert (rows, cols) == (cfg.score_rows, cfg.score_cols)
    k = cfg.keep_k
    ph = to_np(p)
    modes = [(sf.PRUNE_TOPK, 0.0)]
    if cfg.threshold_variant:
        modes.append((sf.PRUNE_THRESHOLD, cfg.threshold_tau))
    for mode, tau in modes:
        vals = torch.empty(rows, k, dtype=p.dtype, device="cuda")
        idx = torch.empty(rows, k, dtype=torch.uint16, device="cuda")
        counts = torch.empty(rows, dtype=torch.int32, device="cuda")
        sf.prune_scores(p, k, mode, tau, vals, idx, counts)
        torch.cuda.synchronize()
        ov, oi, oc = ref.prune_scores(ph, k, mode=mode, tau=tau, threads=THREADS)
        _eq(to_np(idx), oi)
        _eq(to_np(vals), ov)
        _eq(to_np(counts), oc)
        if mode == sf.PRUNE_THRESHOLD:
            assert (oc < k).any() and (oc == k).any()
        # backward half: zeros + scatter of the kept pairs
        dense = torch.empty_like(p)
        sf.restore_scores(vals, idx, counts, dense)
        torch.cuda.synchronize()
        _eq(to_np(dense), ref.restore_scores(ov, oi, oc, cols, threads=THREADS))
        del vals, idx, counts, dense


@pytest.mark.parametrize("ci", [1, 2, 3, 4])
def test_layer_delta_and_ils_all_units(ci):
    require_gpu()
    cfg = synth.CONFIGS[ci]
    prev, cur = synth.weight_units(cfg, "cuda")
    numel = [t.numel() for t in prev]
    assert len(prev) == cfg.n_units and sum(numel) == sum(cfg.unit_numels)
    ws = torch.empty(sf.layer_delta_workspace(numel), dtype=torch.uint8, device="cuda")
    d = torch.empty(len(prev), device="cuda")
    sf.layer_delta_plan(prev, cur, ws)
    pdt = sf.BF16 if cfg.w_dtype == torch.bfloat16 else sf.F32
    sf.layer_delta_run(numel, pdt, sf.F32, cfg.delta_given, 0.0, d, ws)
    torch.cuda.synchronize()
    got = to_np(d)
    want = ref.layer_delta([to_np(t) for t in prev], [to_np(t) for t in cur],
                           cur_is_delta=cfg.delta_given, threads=THREADS)
    fin = np.isfinite(want)
    assert fin.all()                      # the generator leaves no exact zero in W^{t-1}
    np.testing.assert_array_equal(np.isfinite(got), fin)
    np.testing.assert_array_equal(got[~fin], want[~fin])
    np.testing.assert_allclose(got[fin], want[fin], rtol=1e-6, atol=0)
    n_freeze = sf.freeze_count(cfg.n_units, cfg.freeze_rate)
    assert n_freeze == cfg.n_freeze == ref.freeze_count(cfg.n_units, cfg.freeze_rate)
    gi, gm = sf.ils_select(got, n_freeze)
    oi, om = ref.ils_select(want, n_freeze)
    # the two score vectors agree to 1e-6, so the selections agree unless two layers are closer than that
    gaps = np.diff(np.sort(want[fin].astype(np.float64)))
    if gaps.min() > 4e-6 * want[fin].max():
        np.testing.assert_array_equal(gi, oi)
        np.testing.assert_array_equal(gm, om)
    # selection on identical inputs is bit-exact in any case
    gi2, gm2 = sf.ils_select(want, n_freeze)
    np.testing.assert_array_equal(gi2, oi)
    np.testing.assert_array_equal(gm2, om)


@pytest.mark.parametrize("ci", [1, 4])
def test_layer_delta_with_exact_zeros_among_the_old_weights(ci):
    """Eq. 1 divides by W^{t-1}: an unchanged zero weight contributes 0, a changed one makes its layer's score
    +inf (the layer ranks last), and eps > 0 keeps every score finite -- at full size, planted in every chunk
    position class (first element, chunk interior, chunk edge, last element)."""
    require_gpu()
    cfg = synth.CONFIGS[ci]
    prev, cur = synth.weight_units(cfg, "cuda")
    numel = [t.numel() for t in prev]
    unchanged, changed = [0, 5, 7], [1, 4, 6, len(prev) - 1]     # layers whose zero weights stay / get an update
    for i in unchanged + changed:
        n = numel[i]
        spots = sorted({0, 1, n // 3, min(n - 1, 16383), min(n - 1, 16384), n - 1})
        for j in spots:
            prev[i][j] = 0.0
            if cfg.delta_given:
                cur[i][j] = 0.0 if i in unchanged else 1e-3
            else:
                cur[i][j] = 0.0 if i in unchanged else 1e-3
    ws = torch.empty(sf.layer_delta_workspace(numel), dtype=torch.uint8, device="cuda")
    hp, hc = [to_np(t) for t in prev], [to_np(t) for t in cur]
    for eps in (0.0, 1e-6):
        d = torch.empty(len(prev), device="cuda")
        sf.layer_delta(prev, cur, cfg.delta_given, eps, d, ws)
        torch.cuda.synchronize()
        got = to_np(d)
        want = ref.layer_delta(hp, hc, cur_is_delta=cfg.delta_given, eps=eps, threads=THREADS)
        fin = np.isfinite(want)
        if eps == 0.0:
            assert sorted(np.nonzero(~fin)[0].tolist()) == sorted(changed) and np.all(want[~fin] == np.inf)
        else:
            assert fin.all()
        np.testing.assert_array_equal(np.isfinite(got), fin)
        np.testing.assert_array_equal(got[~fin], want[~fin])
        np.testing.assert_allclose(got[fin], want[fin], rtol=1e-6, atol=0)
        # +inf sorts after every finite score: none of the changed-zero layers is frozen at eps = 0
        n_freeze = sf.freeze_count(cfg.n_units, cfg.freeze_rate)
        gi, gm = sf.ils_select(got, n_freeze)
        if eps == 0.0:
            assert not any(gm[i] for i in changed)
