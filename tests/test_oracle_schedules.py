"""Pins for the oracle's random and progressive freezing schedules (the paper's ablation of freezing
schedules) -- CPU only."""
import os

import numpy as np
import pytest

from oracle import ref


def test_splitmix64_known_answers(golden_dir):
    for line in open(os.path.join(golden_dir, "splitmix64_vectors.txt")):
        if line.startswith("#") or not line.strip():
            continue
        nums = [int(t) for t in line.split()]
        got = ref.splitmix64(nums[0], len(nums) - 1)
        assert got.tolist() == nums[1:]


def test_splitmix64_matches_big_integer_arithmetic():
    M = (1 << 64) - 1
    state = 0xDEADBEEFCAFEF00D
    want = []
    s = state
    for _ in range(50):
        s = (s + 0x9E3779B97F4A7C15) & M
        z = s
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
        want.append(z ^ (z >> 31))
    assert ref.splitmix64(state, 50).tolist() == want


def _python_random_schedule(L, n, seed, it):
    M = (1 << 64) - 1
    s = (seed ^ ((it * 0xD6E8FEB86659FD93) & M)) & M
    perm = list(range(L))
    out = []
    for i in range(n):
        s = (s + 0x9E3779B97F4A7C15) & M
        z = s
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
        z ^= z >> 31
        j = i + z % (L - i)
        perm[i], perm[j] = perm[j], perm[i]
        out.append(perm[i])
    return out


@pytest.mark.parametrize("L,n", [(1, 1), (8, 4), (12, 0), (74, 55), (198, 198), (300, 1)])
def test_random_schedule_is_a_partial_shuffle(L, n):
    for seed, it in ((0, 0), (7, 1), (7, 2), (2 ** 63 + 5, 10 ** 12)):
        idx, mask = ref.schedule_random(L, n, seed, it)
        assert idx.tolist() == _python_random_schedule(L, n, seed, it)
        assert len(set(idx.tolist())) == n and all(0 <= i < L for i in idx)
        assert mask.sum() == n and all(mask[i] == 1 for i in idx)
        again, _ = ref.schedule_random(L, n, seed, it)
        assert again.tolist() == idx.tolist()


def test_random_schedule_changes_every_iteration_and_is_uniform():
    L, n, iters = 24, 12, 20000
    counts = np.zeros(L)
    seen = set()
    for it in range(iters):
        idx, mask = ref.schedule_random(L, n, 1234, it)
        counts += mask
        if it < 200:
            seen.add(tuple(sorted(idx.tolist())))
    assert len(seen) > 190                                    # 2.7 M possible sets: repeats are rare
    expect = iters * n / L
    chi2 = float(((counts - expect) ** 2 / (expect * (1 - n / L))).sum())
    assert chi2 < 60.0                                        # 23 degrees of freedom: P(chi2 > 60) < 1e-4
    a, _ = ref.schedule_random(L, n, 1, 5)
    b, _ = ref.schedule_random(L, n, 2, 5)
    assert a.tolist() != b.tolist()


def test_progressive_schedule_freezes_the_earliest_layers():
    idx, mask = ref.schedule_progressive(10, 4)
    assert idx.tolist() == [0, 1, 2, 3] and mask.tolist() == [1, 1, 1, 1, 0, 0, 0, 0, 0, 0]
    idx, mask = ref.schedule_progressive(5, 0)
    assert idx.size == 0 and mask.sum() == 0
    idx, mask = ref.schedule_progressive(3, 3)
    assert mask.tolist() == [1, 1, 1]


def test_bad_arguments_rejected():
    for fn, args in ((ref.schedule_random, (4, 5, 0, 0)), (ref.schedule_random, (-1, 0, 0, 0)),
                     (ref.schedule_progressive, (4, 5)), (ref.schedule_progressive, (4, -1))):
        with pytest.raises(ValueError):
            fn(*args)
