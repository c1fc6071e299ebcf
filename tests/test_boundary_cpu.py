"""Host-only tests of the C-ABI library: it loads, exports what the header
declares, rejects bad arguments before touching a GPU, and its host-side ILS
routines agree with the oracle and with the paper's Fig. 4."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import ref
from paper_2305_18513_amd import binding as sf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not sf.is_built():
        from paper_2305_18513_amd import build
        build.build_library(verbose=False)
    return sf.lib()


def _declared():
    text = open(os.path.join(ROOT, "include", "slimfit.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(slimfit_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = _declared()
    assert len(names) >= 17
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(sf.EXPORTS) == names


def test_status_strings_and_version(lib):
    assert sf.version() >= 100
    texts = {sf.status_string(s) for s in range(7)}
    assert len(texts) == 7 and "ok" in texts
    assert sf.status_string(99) == "unknown status"


def test_size_helpers(lib):
    assert sf.packed_bytes(0, 4) == 0 and sf.packed_bytes(5, 4) == 3 and sf.packed_bytes(5, 8) == 5
    assert sf.packed_bytes(5, 3) == 0 and sf.packed_bytes(-1, 4) == 0
    assert sf.num_blocks(0, 64) == 0 and sf.num_blocks(65, 64) == 2 and sf.num_blocks(64, 64) == 1
    for cols, ppm in ((64, 100000), (128, 100000), (197, 50000), (384, 100000), (577, 100000)):
        assert sf.keep_count(cols, ppm) == ref.keep_count(cols, ppm) == int(cols * ppm / 1e6)
    assert sf.keep_count(10, 2000000) == -1
    for L in (0, 8, 16, 96, 100, 192):
        for F in (0.0, 0.5, 0.8, 0.9, 0.95, 1.0):
            assert sf.freeze_count(L, F) == int(L * F) == ref.freeze_count(L, F)
    assert sf.freeze_count(8, 1.5) == -1 and sf.freeze_count(-1, 0.5) == -1


def _quant(lib, x=16, dt=0, n=64, mode=1, bits=4, block=64, fb=0, codes=16, scales=16):
    return lib.slimfit_quant_pack(C.c_void_p(x), C.c_int32(dt), C.c_int64(n), C.c_int32(mode),
                                  C.c_int32(bits), C.c_int32(block), C.c_int32(fb),
                                  C.c_void_p(codes), C.c_void_p(scales), C.c_void_p(0))


def test_quant_argument_errors_return_before_any_launch(lib):
    assert _quant(lib, n=0) == sf.OK                          # empty is a no-op
    assert _quant(lib, n=-1) == sf.ERR_INVALID_ARG
    assert _quant(lib, dt=7) == sf.ERR_INVALID_ARG
    assert _quant(lib, mode=2) == sf.ERR_INVALID_ARG
    assert _quant(lib, bits=5) == sf.ERR_UNSUPPORTED
    assert _quant(lib, block=48) == sf.ERR_UNSUPPORTED
    assert _quant(lib, mode=0, fb=40) == sf.ERR_UNSUPPORTED
    assert _quant(lib, x=0) == sf.ERR_INVALID_ARG
    assert _quant(lib, scales=0) == sf.ERR_INVALID_ARG
    assert _quant(lib, x=20) == sf.ERR_ALIGNMENT
    assert _quant(lib, codes=8) == sf.ERR_ALIGNMENT
    rc = lib.slimfit_dequant_unpack(C.c_void_p(16), C.c_void_p(16), C.c_int64(64), C.c_int32(1),
                                    C.c_int32(8), C.c_int32(100), C.c_int32(0), C.c_void_p(16),
                                    C.c_int32(0), C.c_void_p(0))
    assert rc == sf.ERR_UNSUPPORTED
    rc = lib.slimfit_dequant_unpack(C.c_void_p(16), C.c_void_p(16), C.c_int64(64), C.c_int32(1),
                                    C.c_int32(8), C.c_int32(64), C.c_int32(0), C.c_void_p(0),
                                    C.c_int32(0), C.c_void_p(0))
    assert rc == sf.ERR_INVALID_ARG


def _prune(lib, p=16, dt=0, rows=4, cols=64, k=6, mode=0, vals=16, idx=16, counts=0):
    return lib.slimfit_prune_scores(C.c_void_p(p), C.c_int32(dt), C.c_int64(rows), C.c_int32(cols),
                                    C.c_int32(k), C.c_int32(mode), C.c_float(0.0), C.c_void_p(vals),
                                    C.c_void_p(idx), C.c_void_p(counts), C.c_void_p(0))


def test_prune_argument_errors(lib):
    assert _prune(lib, rows=0) == sf.OK
    assert _prune(lib, k=0) == sf.ERR_INVALID_ARG
    assert _prune(lib, k=65) == sf.ERR_INVALID_ARG
    assert _prune(lib, cols=0) == sf.ERR_INVALID_ARG
    assert _prune(lib, cols=65537, k=5) == sf.ERR_UNSUPPORTED
    assert _prune(lib, mode=4) == sf.ERR_INVALID_ARG
    assert _prune(lib, rows=-2) == sf.ERR_INVALID_ARG
    assert _prune(lib, p=0) == sf.ERR_INVALID_ARG
    assert _prune(lib, p=18) == sf.ERR_ALIGNMENT                # fp32 needs 4-byte alignment
    assert _prune(lib, idx=17) == sf.ERR_ALIGNMENT
    rc = lib.slimfit_restore_scores(C.c_void_p(16), C.c_void_p(16), C.c_void_p(0), C.c_int32(0),
                                    C.c_int64(4), C.c_int32(64), C.c_int32(6), C.c_void_p(8),
                                    C.c_void_p(0))
    assert rc == sf.ERR_ALIGNMENT


def test_layer_delta_argument_errors(lib):
    numel = np.array([100, 0, 5000], dtype=np.int64)
    assert sf.layer_delta_workspace(numel) >= 64 + 3 * 32 + 8 * 2
    assert sf.layer_delta_workspace([]) >= 64
    with pytest.raises(sf.SlimfitError) as e:
        sf.layer_delta_workspace([5, -1])
    assert e.value.status == sf.ERR_INVALID_ARG
    ptrs = (C.c_void_p * 3)(256, 0, 512)
    n = C.c_void_p(numel.ctypes.data)

    def plan(ws=256, ws_bytes=1 << 20, prev=ptrs, dt=0, L=3):
        return lib.slimfit_layer_delta_plan(prev, C.c_int32(dt), ptrs, C.c_int32(0), n, C.c_int32(L),
                                            C.c_void_p(ws), C.c_size_t(ws_bytes), C.c_void_p(0))

    assert plan(L=0) == sf.OK
    assert plan(L=-1) == sf.ERR_INVALID_ARG
    assert plan(dt=3) == sf.ERR_INVALID_ARG
    assert plan(ws=0) == sf.ERR_WORKSPACE
    assert plan(ws_bytes=64) == sf.ERR_WORKSPACE
    assert plan(ws=264) == sf.ERR_ALIGNMENT
    assert plan(prev=(C.c_void_p * 3)(0, 0, 512)) == sf.ERR_INVALID_ARG     # non-empty layer, NULL
    assert plan(prev=(C.c_void_p * 3)(260, 0, 512)) == sf.ERR_ALIGNMENT
    rc = lib.slimfit_layer_delta_run(n, C.c_int32(3), C.c_int32(0), C.c_int32(0), C.c_int32(0),
                                     C.c_float(-1.0), C.c_void_p(256), C.c_void_p(256),
                                     C.c_size_t(1 << 20), C.c_void_p(0))
    assert rc == sf.ERR_INVALID_ARG                                         # negative eps
    rc = lib.slimfit_layer_delta_run(n, C.c_int32(3), C.c_int32(0), C.c_int32(0), C.c_int32(0),
                                     C.c_float(0.0), C.c_void_p(0), C.c_void_p(256),
                                     C.c_size_t(1 << 20), C.c_void_p(0))
    assert rc == sf.ERR_INVALID_ARG                                         # d_out NULL


def test_ils_fig4_replay_through_the_library(lib, golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "fig4_ils.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                _, d, frozen = [s.strip() for s in line.split("|")]
                rows.append((np.array(d.split(), dtype=np.float32),
                             sorted(int(s) - 1 for s in frozen.split())))
    d = rows[0][0].copy()
    n_freeze = sf.freeze_count(8, 0.5)
    assert n_freeze == 4
    for step in range(3):
        idx, mask = sf.ils_select(d, n_freeze)
        assert sorted(idx.tolist()) == rows[step][1]
        if step < 2:
            new = np.where(mask == 1, np.float32(1e9), rows[step + 1][0]).astype(np.float32)
            sf.ils_update(d, new, mask)
            np.testing.assert_array_equal(d, rows[step + 1][0])


def test_ils_matches_oracle_bit_exact(lib):
    rng = np.random.default_rng(0)
    for L in (1, 2, 16, 96, 192, 198):
        for trial in range(4):
            d = (rng.integers(0, 20, L) / 8).astype(np.float32)        # many ties
            if trial == 3 and L > 4:
                d[rng.integers(0, L, 3)] = np.nan
                d[rng.integers(0, L)] = np.inf
            for n in {0, 1, L // 2, int(L * 0.95), L}:
                gi, gm = sf.ils_select(d, n)
                oi, om = ref.ils_select(d, n)
                np.testing.assert_array_equal(gi, oi)
                np.testing.assert_array_equal(gm, om)
            mask = (rng.random(L) < 0.5).astype(np.uint8)
            new = rng.random(L).astype(np.float32)
            got = sf.ils_update(d.copy(), new, mask)
            np.testing.assert_array_equal(got, ref.ils_update(d, new, mask))


def test_ils_argument_errors(lib):
    d = np.zeros(4, dtype=np.float32)
    for n in (-1, 5):
        with pytest.raises(sf.SlimfitError) as e:
            sf.ils_select(d, n)
        assert e.value.status == sf.ERR_INVALID_ARG
    rc = lib.slimfit_ils_select(C.c_void_p(0), C.c_int32(4), C.c_int32(2), C.c_void_p(0), C.c_void_p(0))
    assert rc == sf.ERR_INVALID_ARG
    assert lib.slimfit_ils_update(C.c_void_p(0), C.c_void_p(0), C.c_void_p(0), C.c_int32(0)) == sf.OK
    assert lib.slimfit_ils_update(C.c_void_p(0), C.c_void_p(0), C.c_void_p(0), C.c_int32(3)) == sf.ERR_INVALID_ARG


def test_schedule_variants_match_the_oracle():
    """Random and progressive freezing (host code): the library against the oracle, draw for draw."""
    for L, n in ((1, 1), (8, 4), (12, 0), (74, 55), (198, 198), (300, 1), (0, 0)):
        for seed, it in ((0, 0), (7, 1), (2 ** 63 + 5, 10 ** 12), (2 ** 64 - 1, 2 ** 64 - 1)):
            gi, gm = sf.schedule_random(L, n, seed, it)
            oi, om = ref.schedule_random(L, n, seed, it)
            np.testing.assert_array_equal(gi, oi)
            np.testing.assert_array_equal(gm, om)
        gi, gm = sf.schedule_progressive(L, n)
        oi, om = ref.schedule_progressive(L, n)
        np.testing.assert_array_equal(gi, oi)
        np.testing.assert_array_equal(gm, om)
    for bad in ((4, 5), (-1, 0), (4, -1)):
        with pytest.raises(sf.SlimfitError):
            sf.schedule_random(bad[0], bad[1], 0, 0)
        with pytest.raises(sf.SlimfitError):
            sf.schedule_progressive(*bad)


def test_block_ils_matches_the_oracle():
    """ILS over blocks of consecutive layers (host code): the library against the oracle."""
    rng = np.random.default_rng(3)
    for L, group in ((1, 1), (8, 2), (74, 6), (198, 8), (25, 8), (7, 10), (192, 8)):
        for trial in range(3):
            d = (10.0 ** rng.uniform(-6, -2, L)).astype(np.float32)
            if trial == 1:
                d = np.round(d * 1e4).astype(np.float32)                 # many ties
            if trial == 2 and L > 3:
                d[rng.integers(0, L)] = np.nan
                d[rng.integers(0, L)] = np.inf
            nb = -(-L // group)
            for n in sorted({0, 1, nb // 2, nb}):
                gi, gm = sf.ils_select_blocks(d, group, n)
                oi, om = ref.ils_select_blocks(d, group, n)
                np.testing.assert_array_equal(gi, oi)
                np.testing.assert_array_equal(gm, om)
    for group, n in ((0, 1), (3, 5), (3, -1)):
        with pytest.raises(sf.SlimfitError):
            sf.ils_select_blocks(np.ones(10, np.float32), group, n)


def test_fused_and_layernorm_argument_errors_return_before_any_launch(lib):
    """The later entry points reject bad sizes, dtypes, null and misaligned pointers on the host (no GPU needed)."""
    P = C.c_void_p
    # softmax backward from the pairs: (vals, idx, counts, dp, dt, rows, cols, k, ds, stream)
    def smb(vals=16, idx=16, dp=16, dt=0, rows=4, cols=64, k=6, ds=32):
        return lib.slimfit_softmax_backward_pruned(P(vals), P(idx), P(0), P(dp), C.c_int32(dt), C.c_int64(rows),
                                                   C.c_int32(cols), C.c_int32(k), P(ds), P(0))
    assert smb(rows=0) == sf.OK
    assert smb(k=65) == sf.ERR_INVALID_ARG
    assert smb(dt=2) == sf.ERR_INVALID_ARG
    assert smb(vals=0) == sf.ERR_INVALID_ARG
    assert smb(dp=32) == sf.ERR_INVALID_ARG                      # ds must not be dp
    assert smb(ds=40) == sf.ERR_ALIGNMENT                        # ds needs 16-byte alignment
    assert smb(cols=70000, k=6) == sf.ERR_UNSUPPORTED

    # LayerNorm forward: (x, dt, gamma, beta, rows, H, eps, y, mean, rstd, stream)
    def lnf(x=16, dt=0, rows=4, H=64, eps=1e-5, y=32, gamma=16):
        return lib.slimfit_layernorm_forward(P(x), C.c_int32(dt), P(gamma), P(16), C.c_int64(rows), C.c_int64(H),
                                             C.c_float(eps), P(y), P(16), P(16), P(0))
    assert lnf(rows=0) == sf.OK
    assert lnf(H=6) == sf.ERR_INVALID_ARG                        # fp32 rows are whole 16-byte vectors
    assert lnf(dt=1, H=12) == sf.ERR_INVALID_ARG                 # bf16 rows too: multiples of 8
    assert lnf(dt=1, H=16, rows=0) == sf.OK
    assert lnf(H=4100) == sf.ERR_UNSUPPORTED
    assert lnf(eps=-1.0) == sf.ERR_INVALID_ARG
    assert lnf(y=16) == sf.ERR_INVALID_ARG                       # in place
    assert lnf(gamma=20) == sf.ERR_ALIGNMENT
    assert lnf(dt=7) == sf.ERR_INVALID_ARG

    # LayerNorm forward + quantiser: (x, dt, gamma, beta, rows, H, eps, bits, block, y, mean, rstd, codes, scales, stream)
    def lnq(H=64, bits=4, block=64, codes=16):
        return lib.slimfit_layernorm_forward_quant_pack(P(16), C.c_int32(0), P(16), P(16), C.c_int64(4), C.c_int64(H),
                                                        C.c_float(1e-5), C.c_int32(bits), C.c_int32(block), P(32), P(16),
                                                        P(16), P(codes), P(16), P(0))
    assert lnq(bits=5) == sf.ERR_UNSUPPORTED
    assert lnq(block=48) == sf.ERR_UNSUPPORTED
    assert lnq(H=96) == sf.ERR_UNSUPPORTED                       # a block would straddle two rows
    assert lnq(codes=0) == sf.ERR_INVALID_ARG
    assert lnq(codes=24) == sf.ERR_ALIGNMENT

    # score while applying the update: (w, w_dt, delta, delta_dt, numel, L, eps, d_out, workspace, bytes, stream)
    numel = np.array([100, 5000], dtype=np.int64)
    w = (C.c_void_p * 2)(256, 512)
    dl = (C.c_void_p * 2)(1024, 2048)
    def app(w=w, dl=dl, eps=0.0, d_out=256, ws=256, ws_bytes=1 << 20, L=2):      # (sizes are checked after d_out's range)
        return lib.slimfit_apply_update_layer_delta(w, C.c_int32(0), dl, C.c_int32(0), P(numel.ctypes.data), C.c_int32(L),
                                                    C.c_float(eps), P(d_out), P(ws), C.c_size_t(ws_bytes), P(0))
    assert app(L=0) == sf.OK
    assert app(eps=-1.0) == sf.ERR_INVALID_ARG
    assert app(d_out=0) == sf.ERR_INVALID_ARG
    assert app(d_out=258) == sf.ERR_ALIGNMENT
    assert app(dl=w) == sf.ERR_INVALID_ARG                       # the update aliases the weights

    # block-granularity ILS needs a positive group and at most ceil(L / group) blocks
    d = np.ones(10, np.float32)
    out = np.zeros(4, np.int32)
    assert lib.slimfit_ils_select_blocks(P(d.ctypes.data), C.c_int32(10), C.c_int32(0), C.c_int32(1), P(out.ctypes.data),
                                         P(0)) == sf.ERR_INVALID_ARG
    assert lib.slimfit_ils_select_blocks(P(d.ctypes.data), C.c_int32(10), C.c_int32(3), C.c_int32(5), P(out.ctypes.data),
                                         P(0)) == sf.ERR_INVALID_ARG
    assert lib.slimfit_ils_select_blocks(P(d.ctypes.data), C.c_int32(10), C.c_int32(3), C.c_int32(4), P(out.ctypes.data),
                                         P(0)) == sf.OK


def test_stream_probe_argument_errors(lib):
    """The diagnostic streaming kernel checks its arguments like every other entry point."""
    P = C.c_void_p

    def probe(src=16, dst=64, in_vecs=1024, ratio=8):
        return lib.slimfit_stream_probe(P(src), P(dst), C.c_int64(in_vecs), C.c_int32(ratio), P(0))
    assert probe(in_vecs=0) == sf.OK
    assert probe(in_vecs=-1) == sf.ERR_INVALID_ARG
    for ratio in (3, 7, 32, -1, -3, -16):                        # 1 .. 16 (powers of two), 0, -2, -4, -8 only
        assert probe(ratio=ratio) == sf.ERR_INVALID_ARG
    assert probe(src=0) == sf.ERR_INVALID_ARG
    assert probe(dst=16) == sf.ERR_INVALID_ARG                   # in place
    assert probe(dst=72) == sf.ERR_ALIGNMENT


def test_bench_refuses_more_than_one_gpu():
    """bench.py is single-GPU by design: --gpus above 1 ends with a message and a non-zero status, before any GPU use."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "single-GPU" in (r.stdout + r.stderr)


# ---- the binding's own size and dtype checks (host tensors: a bad argument is refused before any C call) ----

def test_binding_rejects_outputs_that_are_too_small():
    import torch
    n = 1000
    x = torch.zeros(n)
    codes = torch.zeros(sf.packed_bytes(n, 4), dtype=torch.uint8)
    scales = torch.zeros(sf.num_blocks(n, 64))
    y = torch.zeros(n)
    with pytest.raises(ValueError):
        sf.quant_pack(x, sf.Q_BLOCK, 4, 64, 0, codes[:-1], scales)
    with pytest.raises(ValueError):
        sf.quant_pack(x, sf.Q_BLOCK, 4, 64, 0, codes, scales[:-1])
    with pytest.raises(ValueError):
        sf.dequant_unpack(codes[:-1], scales, sf.Q_BLOCK, 4, 64, 0, y)
    with pytest.raises(ValueError):
        sf.gelu_quant_pack(x, sf.Q_BLOCK, 4, 64, 0, y, codes[:-1], scales)
    with pytest.raises(ValueError):
        sf.gelu_backward_dequant(codes, scales[:-1], sf.Q_BLOCK, 4, 64, 0, y, torch.zeros(n))
    rows, cols, k = 10, 40, 4
    p = torch.zeros(rows, cols)
    vals = torch.zeros(rows, k)
    idx = torch.zeros(rows, k, dtype=torch.uint16)
    counts = torch.zeros(rows, dtype=torch.int32)
    with pytest.raises(ValueError):
        sf.prune_scores(p, k, sf.PRUNE_TOPK, 0.0, vals[:-1], idx, None)
    with pytest.raises(ValueError):
        sf.prune_scores(p, k, sf.PRUNE_TOPK, 0.0, vals, idx[:-1], None)
    with pytest.raises(ValueError):
        sf.prune_scores(p, k, sf.PRUNE_THRESHOLD, 0.0, vals, idx, counts[:-1])
    with pytest.raises(ValueError):
        sf.softmax_prune(p, k, torch.zeros_like(p), vals[:-1], idx)
    with pytest.raises(ValueError):
        sf.restore_scores(vals[:-1], idx[:-1], None, p)
    with pytest.raises(ValueError):
        sf.softmax_backward_pruned(vals, idx, counts[:-1], p, torch.zeros_like(p))


def test_binding_rejects_layer_lists_of_mixed_dtype_or_size():
    import torch
    a = [torch.zeros(64), torch.zeros(32, dtype=torch.bfloat16)]          # an fp32 vector next to a bf16 matrix
    b = [torch.zeros(64), torch.zeros(32)]
    d = torch.zeros(2)
    ws = torch.zeros(4096, dtype=torch.uint8)
    for call in (lambda: sf.layer_delta(a, b, False, 0.0, d, ws),
                 lambda: sf.layer_delta(b, a, False, 0.0, d, ws),
                 lambda: sf.layer_delta_plan(a, b, ws),
                 lambda: sf.layer_delta_static(a, b, False, 0.0, d),
                 lambda: sf.apply_update_layer_delta(a, b, 0.0, d, ws),
                 lambda: sf.layer_delta(b, [torch.zeros(64), torch.zeros(31)], False, 0.0, d, ws)):
        with pytest.raises(ValueError):
            call()


def test_binding_wants_a_workspace_with_an_explicit_stream():
    import torch
    x = torch.zeros(100)
    with pytest.raises(ValueError):
        sf.prune_global(x, 10, torch.zeros(10), torch.zeros(10, dtype=torch.int32), stream=12345)


def test_library_counts_reproduce_the_workloads_stated_figures():
    from paper_2305_18513_amd import synth
    for c in synth.CONFIGS:
        assert sf.keep_count(c.score_cols, c.keep_ppm) == c.keep_k
        assert sf.freeze_count(c.n_units, c.freeze_rate) == c.n_freeze
