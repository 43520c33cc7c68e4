"""Pins for the oracle's shard assignment (sections 3.1 and 4.3): brute-force
invariants, generator known answers, uniformity (CPU only)."""
import os

import numpy as np
import pytest

from oracle import oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_splitmix64_known_answers():
    want = [int(l, 16) for l in open(os.path.join(GOLD, "splitmix64_seed0.txt")) if not l.startswith("#")]
    assert [O.splitmix64_at(0, j) for j in range(3)] == want
    j = np.arange(3, dtype=np.uint64)
    assert [int(v) for v in O._splitmix64_vec(0, j)] == want


@pytest.mark.parametrize("seed", [0, 1, 12345])
@pytest.mark.parametrize("N,B", [(64, 8), (1024, 64), (2048, 128)])
def test_once_per_epoch_whatever_p_does(seed, N, B):
    rng = np.random.default_rng(seed)
    for epoch in (0, 1):
        seen = []
        sets = []
        for t in range(N // B):
            p = int(rng.choice([1, 2, 4, 8]))
            idx, off = O.shard(seed, N, B, p, epoch, t)
            assert len(idx) == B and list(off) == [k * (B // p) for k in range(p + 1)]
            pieces = [idx[off[k]:off[k + 1]] for k in range(p)]
            assert sum(len(q) for q in pieces) == B
            assert len(set(idx.tolist())) == B                      # workers' shards are disjoint
            # the aggregate batch does not depend on p
            for p2 in (1, 2, 4, 8):
                assert np.array_equal(O.shard(seed, N, B, p2, epoch, t)[0], idx)
            seen += idx.tolist()
            sets.append(frozenset(idx.tolist()))
        assert sorted(seen) == list(range(N))                       # no repetition, no omission
    assert O.epoch_permutation(seed, 0, N) != O.epoch_permutation(seed, 1, N)
    assert O.epoch_permutation(seed, 0, N) == O.epoch_permutation(seed, 0, N)
    assert O.epoch_permutation(seed, 0, N) != O.epoch_permutation(seed + 1, 0, N)


def test_bad_requests_are_rejected():
    for args in [(0, 64, 8, 3, 0, 0), (0, 60, 8, 2, 0, 0), (0, 64, 8, 2, 0, 8), (0, 64, 8, 0, 0, 0)]:
        with pytest.raises(ValueError):
            O.shard(*args)


def test_shuffle_is_uniform():
    N, trials = 8, 4000
    counts = np.zeros((N, N))
    for seed in range(trials):
        perm = O.epoch_permutation(seed, 0, N)
        for pos, v in enumerate(perm):
            counts[pos, v] += 1
    chi2 = ((counts - trials / N) ** 2 / (trials / N)).sum()
    # (N-1)^2 = 49 degrees of freedom; 99.9th percentile is 85.4
    assert chi2 < 85.4, chi2
