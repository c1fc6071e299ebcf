"""Pins for the oracle's pruner/restorer (Alg. 5, App. on pruning) -- CPU only."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2305_18513_amd import synth


def _brute_topk(row, k):
    """Repeat arg-max (lowest column among equals) k times."""
    left = row.astype(np.float64).copy()
    cols = []
    for _ in range(k):
        j = int(np.argmax(left))          # numpy returns the first maximum
        cols.append(j)
        left[j] = -np.inf
    return sorted(cols)


def _check_row_invariants(row, vals, idx, cnt):
    cols = idx[:cnt].astype(np.int64)
    assert np.all(np.diff(cols) > 0)                      # strictly ascending
    np.testing.assert_array_equal(vals[:cnt].view(np.uint32), row[cols].view(np.uint32))
    dropped = np.setdiff1d(np.arange(row.size), cols)
    if cnt and dropped.size:
        cut = row[cols].min()
        assert cut >= row[dropped].max()
        # among entries equal to the cut value the lowest columns were kept
        eq_kept = cols[row[cols] == cut]
        eq_drop = dropped[row[dropped] == cut]
        if eq_kept.size and eq_drop.size:
            assert eq_kept.max() < eq_drop.min()


@pytest.mark.parametrize("cols,k", [(1, 1), (5, 1), (5, 5), (64, 6), (128, 12),
                                    (197, 9), (384, 38), (70, 69)])
def test_topk_equals_bruteforce_and_library_sort(cols, k):
    rng = np.random.default_rng(cols * 100 + k)
    p = rng.standard_normal((23, cols)).astype(np.float32)
    p[3] = 0.25                                            # all-equal row
    p[4, :] = rng.integers(0, 3, cols)                     # heavy ties across the cut
    p[5, ::2] = p[5, -1]                                   # more ties
    vals, idx, counts = ref.prune_scores(p, k)
    assert np.all(counts == k)
    for r in range(p.shape[0]):
        assert idx[r].tolist() == _brute_topk(p[r], k)
        lib = np.sort(np.argsort(-p[r].astype(np.float64), kind="stable")[:k])
        assert idx[r].tolist() == lib.tolist()
        _check_row_invariants(p[r], vals[r], idx[r], k)


def test_descending_sort_prefix_is_the_kept_multiset():
    # Alg. 5: y_s = sort(x, descending)[:k]
    rng = np.random.default_rng(2)
    p = rng.standard_normal((50, 40)).astype(np.float32)
    vals, _, _ = ref.prune_scores(p, 4)
    want = -np.sort(-p, axis=1)[:, :4]
    np.testing.assert_array_equal(-np.sort(-vals, axis=1), want)


def test_k_equal_cols_is_identity_and_restore_roundtrip():
    rng = np.random.default_rng(3)
    p = rng.standard_normal((7, 33)).astype(np.float32)
    vals, idx, counts = ref.prune_scores(p, 33)
    np.testing.assert_array_equal(vals, p)
    np.testing.assert_array_equal(idx, np.tile(np.arange(33, dtype=np.uint16), (7, 1)))
    np.testing.assert_array_equal(ref.restore_scores(vals, idx, counts, 33), p)
    # general k: restore = zeros + scatter
    vals, idx, counts = ref.prune_scores(p, 5)
    dense = ref.restore_scores(vals, idx, None, 33)
    want = np.zeros_like(p)
    for r in range(7):
        want[r, idx[r]] = vals[r]
    np.testing.assert_array_equal(dense, want)
    assert np.count_nonzero(dense) == 7 * 5
    kept = dense != 0
    np.testing.assert_array_equal(dense[kept], p[kept])


def test_signed_zero_ties_and_negative_values():
    p = np.array([[-0.0, 0.0, -1.0, 0.0, -0.0]], dtype=np.float32)
    vals, idx, _ = ref.prune_scores(p, 2)
    assert idx[0].tolist() == [0, 1]                       # -0 == +0: lower column wins
    assert np.signbit(vals[0, 0]) and not np.signbit(vals[0, 1])   # bit copies
    p = np.array([[-3, -1, -2, -1, -5]], dtype=np.float32)
    vals, idx, _ = ref.prune_scores(p, 3)
    assert idx[0].tolist() == [1, 2, 3]                    # signed order, not magnitude


def test_threshold_mode():
    p = np.array([[0.1, 0.5, 0.3, 0.5, 0.2, 0.5],
                  [0.1, 0.1, 0.1, 0.1, 0.1, 0.1],
                  [0.9, 0.8, 0.7, 0.6, 0.5, 0.4]], dtype=np.float32)
    vals, idx, counts = ref.prune_scores(p, 3, mode=ref.PRUNE_THRESHOLD, tau=0.3)
    assert counts.tolist() == [3, 0, 3]                    # row 0: 4 pass, capped at 3
    assert idx[0].tolist() == [1, 3, 5]                    # the three 0.5s beat 0.3
    assert idx[1].tolist() == [0xFFFF] * 3 and not vals[1].any()
    assert idx[2].tolist() == [0, 1, 2]
    vals, idx, counts = ref.prune_scores(p, 3, mode=ref.PRUNE_THRESHOLD, tau=0.45)
    assert counts.tolist() == [3, 0, 3]
    vals, idx, counts = ref.prune_scores(p, 4, mode=ref.PRUNE_THRESHOLD, tau=0.75)
    assert counts.tolist() == [0, 0, 2]
    assert idx[2].tolist() == [0, 1, 0xFFFF, 0xFFFF] and vals[2].tolist()[2:] == [0, 0]
    # tau is inclusive
    _, _, counts = ref.prune_scores(p, 6, mode=ref.PRUNE_THRESHOLD, tau=0.5)
    assert counts.tolist() == [3, 0, 5]


def test_threshold_random_against_definition():
    rng = np.random.default_rng(4)
    p = rng.random((200, 50)).astype(np.float32)
    k, tau = 6, np.float32(0.9)
    vals, idx, counts = ref.prune_scores(p, k, mode=ref.PRUNE_THRESHOLD, tau=float(tau))
    seen_less, seen_cap = False, False
    for r in range(200):
        n_pass = int((p[r] >= tau).sum())
        cnt = min(k, n_pass)
        assert counts[r] == cnt
        want = _brute_topk(p[r], cnt)
        assert idx[r, :cnt].tolist() == want
        assert np.all(idx[r, cnt:] == 0xFFFF) and not vals[r, cnt:].any()
        seen_less |= n_pass < k
        seen_cap |= n_pass > k
        dense = ref.restore_scores(vals[r:r + 1], idx[r:r + 1], counts[r:r + 1], 50)
        assert np.count_nonzero(dense) == cnt
    assert seen_less and seen_cap


def test_bf16_rows_with_many_ties():
    cfg = synth.CONFIGS[4]
    p = synth.attention_scores(cfg, batch=1)[:64]           # bf16, 197 columns
    bits = p.view(torch.int16).numpy().view(np.uint16)
    wide = p.float().numpy()
    k = cfg.keep_k
    assert k == 9
    vals, idx, _ = ref.prune_scores(bits, k)
    tie_rows = 0
    for r in range(64):
        assert idx[r].tolist() == _brute_topk(wide[r], k)
        np.testing.assert_array_equal(vals[r], bits[r][idx[r].astype(np.int64)])
        cut = wide[r][idx[r].astype(np.int64)].min()
        tie_rows += int((wide[r] == cut).sum() > (wide[r][idx[r].astype(np.int64)] == cut).sum())
    assert tie_rows > 0                                    # the tie-break is exercised


def test_keep_count_matches_python_truncation():
    for cols, keep in ((64, 0.10), (128, 0.10), (197, 0.05), (384, 0.10), (577, 0.10)):
        assert ref.keep_count(cols, int(round(keep * 1e6))) == int(cols * keep)
    # the workloads state their counts as data; the oracle's own arithmetic has to reproduce them
    assert [c.keep_k for c in synth.CONFIGS] == [6, 12, 9, 38, 9]
    assert [ref.keep_count(c.score_cols, c.keep_ppm) for c in synth.CONFIGS] == [c.keep_k for c in synth.CONFIGS]


def test_scores_recipe_and_table_of_activation_counts(golden_dir):
    cfg = synth.CONFIGS[0]
    p = synth.attention_scores(cfg)
    assert tuple(p.shape) == (cfg.score_rows, cfg.score_cols) == (1024, 64)
    assert torch.allclose(p.sum(1), torch.ones(1024), atol=1e-5) and float(p.min()) > 0
    # shape generator against the paper's per-layer activation counts
    bth = tt = 0
    paper_gb = None
    import os
    with open(os.path.join(golden_dir, "tab8_activation_counts.txt")) as f:
        for line in f:
            line = line.strip()
            if line.startswith("paper_activation_GB"):
                paper_gb = float(line.split("=")[1])
            elif line and not line.startswith("#"):
                parts = [s.strip() for s in line.split("|")]
                bth += int(parts[2])
                tt = max(tt, int(parts[3]))     # softmax output is shared with the matmul
    b = synth.CONFIGS[1]
    per_block = bth * b.ln_in_numel + tt * b.score_rows * b.score_cols
    assert bth == 18 and b.gelu_in_numel == 4 * b.ln_in_numel
    total_gb = per_block * 4 * b.n_blocks / 1e9
    assert abs(total_gb - paper_gb) / paper_gb < 0.10       # 3.02 GB vs 3.2 GB printed


def test_bad_arguments_rejected():
    p = np.zeros((2, 4), dtype=np.float32)
    for k in (0, 5):
        with pytest.raises(ValueError):
            ref.prune_scores(p, k)
    with pytest.raises(ValueError):
        ref.prune_scores(p, 2, mode=3)
    bad_idx = np.array([[7]], dtype=np.uint16)
    with pytest.raises(ValueError):
        ref.restore_scores(np.zeros((1, 1), np.float32), bad_idx, None, 4)
