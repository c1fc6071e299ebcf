"""Pins for the oracle's ILS pair (Alg. 1, Sec. 3.2) -- CPU only."""
import os

import numpy as np
import pytest

from oracle import ref


def _read_fig4(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "fig4_ils.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            _, d, frozen = [s.strip() for s in line.split("|")]
            rows.append((np.array(d.split(), dtype=np.float32),
                         sorted(int(s) - 1 for s in frozen.split())))
    assert len(rows) == 3
    return rows


def test_fig4_selection_each_panel(golden_dir):
    # each printed distance vector alone gives the printed frozen set
    for d, frozen in _read_fig4(golden_dir):
        idx, mask = ref.ils_select(d, ref.freeze_count(8, 0.5))
        assert sorted(idx.tolist()) == frozen
        assert np.flatnonzero(mask).tolist() == frozen


def test_fig4_replay_with_update_rule(golden_dir):
    # select -> only the active layers take the next panel's value -> the
    # whole next panel is reproduced, frozen entries untouched
    rows = _read_fig4(golden_dir)
    d = rows[0][0].copy()
    for step in range(3):
        idx, mask = ref.ils_select(d, 4)
        assert sorted(idx.tolist()) == rows[step][1]
        if step == 2:
            break
        nxt = rows[step + 1][0]
        # scores the training step would report; for frozen layers hand in
        # garbage to prove it is ignored
        new = np.where(mask == 1, np.float32(-777.0), nxt).astype(np.float32)
        d = ref.ils_update(d, new, mask)
        np.testing.assert_array_equal(d, nxt)


def test_freeze_count_is_python_int_of_product():
    for L in (0, 1, 8, 16, 96, 100, 102, 192, 198):
        for F in (0.0, 0.5, 0.75, 0.8, 0.9, 0.95, 1.0):
            assert ref.freeze_count(L, F) == int(L * F)
    assert ref.freeze_count(192, 0.95) == 182
    assert ref.freeze_count(16, 0.95) == 15


def test_order_is_ascending_and_stable():
    d = np.array([3, 1, 2, 1, 3, 1], dtype=np.float32)
    idx, mask = ref.ils_select(d, 4)
    assert idx.tolist() == [1, 3, 5, 2]          # lower index first among ties
    assert mask.tolist() == [0, 1, 1, 1, 0, 1]


def test_matches_library_stable_argsort_and_bruteforce():
    rng = np.random.default_rng(5)
    for L in (1, 2, 7, 16, 96, 192):
        d = rng.integers(0, 12, L).astype(np.float32) / 4     # many ties
        for n in {0, 1, L // 2, int(L * 0.95), L}:
            idx, mask = ref.ils_select(d, n)
            want = np.argsort(d, kind="stable")[:n]
            np.testing.assert_array_equal(idx, want)
            # brute force: repeat arg-min with lowest index
            left = d.astype(np.float64).copy()
            bf = []
            for _ in range(n):
                j = int(np.argmin(left))
                bf.append(j)
                left[j] = np.inf
            assert idx.tolist() == bf
            assert mask.sum() == n and len(set(idx.tolist())) == n
            if 0 < n < L:
                assert d[mask == 1].max() <= d[mask == 0].min()


def test_nan_and_inf_order_last():
    d = np.array([np.nan, 2, np.inf, 1, np.nan, -np.inf], dtype=np.float32)
    idx, _ = ref.ils_select(d, 6)
    assert idx.tolist() == [5, 3, 1, 2, 0, 4]


def test_update_only_touches_active():
    d = np.arange(6, dtype=np.float32)
    new = d + 100
    mask = np.array([1, 0, 1, 0, 0, 1], dtype=np.uint8)
    out = ref.ils_update(d, new, mask)
    assert out.tolist() == [0, 101, 2, 103, 104, 5]


def test_large_random_start_trains_every_layer_once():
    # Sec. 3.2: with a start vector of large random values every layer is
    # visited during the first iterations, before any real distance can
    # freeze it again.
    L, n_freeze = 16, 12
    rng = np.random.default_rng(0)
    d = (1e30 * (1 + rng.random(L))).astype(np.float32)
    seen = set()
    for it in range(L // (L - n_freeze)):
        _, mask = ref.ils_select(d, n_freeze)
        active = np.flatnonzero(mask == 0)
        assert not (set(active.tolist()) & seen)
        seen |= set(active.tolist())
        d = ref.ils_update(d, rng.random(L).astype(np.float32), mask)
    assert seen == set(range(L))


def test_bad_arguments_rejected():
    d = np.zeros(4, dtype=np.float32)
    with pytest.raises(ValueError):
        ref.ils_select(d, 5)
    with pytest.raises(ValueError):
        ref.ils_select(d, -1)
    with pytest.raises(ValueError):
        ref.freeze_count(4, 1.5)


# ---- block granularity ------------------------------------------------------------------------------------------

def test_blocks_of_one_layer_are_plain_ils(golden_dir):
    for d, frozen in _read_fig4(golden_dir):
        fb, mb = ref.ils_select_blocks(d, 1, len(frozen))
        f1, m1 = ref.ils_select(d, len(frozen))
        np.testing.assert_array_equal(fb, f1)
        np.testing.assert_array_equal(mb, m1)
        assert sorted(fb.tolist()) == frozen


def test_blocks_match_numpy_means_and_stable_argsort():
    rng = np.random.default_rng(0)
    for L, group in ((8, 2), (74, 6), (198, 8), (25, 8), (7, 10), (64, 64), (65, 64)):
        d = (10.0 ** rng.uniform(-6, -2, L)).astype(np.float32)
        nb = -(-L // group)
        means = np.array([d[b * group:(b + 1) * group].astype(np.float64).mean() for b in range(nb)])
        order = np.argsort(means, kind="stable")
        for n in (0, 1, nb // 2, nb):
            fb, mask = ref.ils_select_blocks(d, group, n)
            np.testing.assert_array_equal(fb, order[:n])
            want = np.zeros(L, np.uint8)
            for b in order[:n]:
                want[b * group:(b + 1) * group] = 1
            np.testing.assert_array_equal(mask, want)


def test_blocks_worked_example_ties_short_last_block_and_nan():
    # blocks of 3: means 2, 2, 1, (9+1)/2 = 5 -> order: block 2, then the tie 0 before 1, then the short block 3
    d = np.array([1, 2, 3, 3, 2, 1, 1, 1, 1, 9, 1], np.float32)
    fb, mask = ref.ils_select_blocks(d, 3, 4)
    assert fb.tolist() == [2, 0, 1, 3]
    fb, mask = ref.ils_select_blocks(d, 3, 2)
    assert fb.tolist() == [2, 0] and mask.tolist() == [1, 1, 1, 0, 0, 0, 1, 1, 1, 0, 0]
    # the short block is judged by its mean, not by its sum: (4+4)/2 = 4 loses against (3+3+3)/3 = 3
    fb, _ = ref.ils_select_blocks(np.array([3, 3, 3, 5, 5, 5, 4, 4], np.float32), 3, 2)
    assert fb.tolist() == [0, 2]
    # a NaN anywhere in a block sends the block behind every other, +inf included
    d = np.array([np.nan, 0, 0, np.inf, np.inf, np.inf, 5, 5, 5], np.float32)
    fb, _ = ref.ils_select_blocks(d, 3, 3)
    assert fb.tolist() == [2, 1, 0]


def test_blocks_bad_arguments_rejected():
    d = np.ones(10, np.float32)
    for group, n in ((0, 1), (-1, 1), (3, 5), (3, -1)):
        with pytest.raises(ValueError):
            ref.ils_select_blocks(d, group, n)
    fb, mask = ref.ils_select_blocks(np.zeros(0, np.float32), 4, 0)
    assert fb.size == 0 and mask.size == 0
