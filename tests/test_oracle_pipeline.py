"""Pins of the dynamic-data-pipeline oracle (section 4.3 of the paper) against
what the section and arithmetic fix: the one-sample-partition scheme (the
already pinned shard assignment), brute-force coverage of every epoch under
random scaling, the section's own scaling example, hand-back order, and
checkpoint / restore.  CPU only."""
import random

import numpy as np
import pytest

from oracle import oracle as O
from oracle.pipeline import DataPipeline


def test_one_sample_partitions_are_the_shard_assignment():
    """d = N: whatever p does, batch t of epoch e is the next B entries of the epoch's
    permutation, cut into p equal consecutive pieces."""
    seed, N, B = 5, 96, 24
    pipe = DataPipeline(seed, N, N)
    schedule = [2, 4, 1, 3, 2, 6, 8, 12]                  # two epochs of four batches
    for step, p in enumerate(schedule):
        idx, off = pipe.next_batch(B, range(p))
        ref_idx, ref_off = O.shard(seed, N, B, p, step // 4, step % 4)
        assert idx == ref_idx.tolist()
        assert off == ref_off.tolist()
    assert pipe.epoch == 1 and pipe.consumed == N


def _check_epoch(pipe, N, B, make_workers, steps):
    """Runs `steps` batches; returns per-epoch lists of indices and per-(worker, batch) shards."""
    epochs = {}
    for t in range(steps):
        workers = make_workers(t)
        idx, off = pipe.next_batch(B, workers)
        assert len(idx) == B and off[0] == 0 and off[-1] == B and len(off) == len(workers) + 1
        assert all(off[k] <= off[k + 1] for k in range(len(workers)))
        epochs.setdefault(pipe.epoch, []).extend(idx)
    return epochs


@pytest.mark.parametrize("N,d,B", [(240, 12, 24), (240, 7, 24), (1000, 36, 40), (512, 512, 64), (360, 1, 12)])
def test_every_epoch_visits_every_sample_once_under_random_scaling(N, d, B):
    rng = random.Random(N * 31 + d)
    pipe = DataPipeline(9, N, d)
    divisors = [p for p in range(1, B + 1) if B % p == 0 and p <= 12]
    pool = list(range(100))
    state = {"workers": [0]}

    def make_workers(t):
        if rng.random() < 0.6:                              # an adjustment: some leave, some join
            p = rng.choice(divisors)
            keep = [w for w in state["workers"] if rng.random() < 0.6][:p]
            fresh = [w for w in pool if w not in state["workers"]]
            rng.shuffle(fresh)
            state["workers"] = keep + fresh[:p - len(keep)]
            rng.shuffle(state["workers"])
        return state["workers"]

    epochs = _check_epoch(pipe, N, B, make_workers, 3 * (N // B))
    assert sorted(epochs) == [0, 1, 2]
    for e, seen in epochs.items():
        assert sorted(seen) == list(range(N)), "epoch %d repeats or omits samples" % e


def test_a_worker_reads_its_partition_front_to_back():
    N, d, B = 120, 6, 12
    pipe = DataPipeline(3, N, d)
    s = N // d
    perm = O.epoch_permutation(3, 0, d)
    # two workers, six samples each per batch: worker 0 owns perm[0], worker 1 owns perm[1] for the first
    # three batches (18 of 20 samples), then each finishes its partition and starts the next unassigned one
    for t in range(3):
        idx, off = pipe.next_batch(B, [10, 11])
        assert idx[off[0]:off[1]] == list(range(perm[0] * s + 6 * t, perm[0] * s + 6 * t + 6))
        assert idx[off[1]:off[2]] == list(range(perm[1] * s + 6 * t, perm[1] * s + 6 * t + 6))
    idx, off = pipe.next_batch(B, [10, 11])
    assert idx[off[0]:off[1]] == [perm[0] * s + 18, perm[0] * s + 19] + list(range(perm[2] * s, perm[2] * s + 4))
    assert idx[off[1]:off[2]] == [perm[1] * s + 18, perm[1] * s + 19] + list(range(perm[3] * s, perm[3] * s + 4))


def test_a_leaver_hands_its_remainder_back_and_it_is_served_first():
    N, d, B = 120, 6, 12
    s = N // d
    perm = O.epoch_permutation(4, 0, d)
    pipe = DataPipeline(4, N, d)
    pipe.next_batch(B, ["a", "b"])                          # a: perm[0] to offset 6, b: perm[1] to offset 6
    # a leaves, c joins: c is given the rest of a's partition before any unassigned one
    idx, off = pipe.next_batch(B, ["b", "c"])
    assert idx[off[0]:off[1]] == list(range(perm[1] * s + 6, perm[1] * s + 12))
    assert idx[off[1]:off[2]] == list(range(perm[0] * s + 6, perm[0] * s + 12))
    # both leave, two others join: remainders come back in the leavers' rank order (b then c)
    idx, off = pipe.next_batch(B, ["x", "y"])
    assert idx[off[0]:off[1]] == list(range(perm[1] * s + 12, perm[1] * s + 18))
    assert idx[off[1]:off[2]] == list(range(perm[0] * s + 12, perm[0] * s + 18))


def test_the_sections_scaling_example():
    """Section 4.3's example, with sizes that divide: 1,000 partitions of 1,200 samples, 10 workers;
    5 join in the middle of an epoch and get data at the very next mini-batch; 3 of them leave again
    before the epoch ends.  The epoch still covers the data set exactly once."""
    N, d, B = 1_200_000, 1000, 600
    pipe = DataPipeline(1, N, d)
    counts = np.zeros(N, dtype=np.int32)
    steps = N // B
    for t in range(steps):
        if t < steps // 3:
            workers = list(range(10))
        elif t < steps // 2:
            workers = list(range(15))
        else:
            workers = list(range(10)) + [10, 13]            # 11, 12, 14 left
        idx, off = pipe.next_batch(B, workers)
        if t == steps // 3:                                 # the joiners' first mini-batch is not empty
            assert all(off[k + 1] - off[k] == B // 15 for k in range(15))
        np.add.at(counts, np.asarray(idx), 1)
    assert pipe.epoch == 0 and pipe.consumed == N
    assert counts.min() == 1 and counts.max() == 1


def test_a_tail_mini_batch_is_still_full_when_a_worker_runs_dry():
    """Two partitions of 12, two workers read half of each; then a third worker joins when nothing is
    unassigned any more: what it cannot get goes round to the workers that still hold data, and the
    mini-batch keeps its B samples."""
    N, d, B = 24, 2, 12
    pipe = DataPipeline(2, N, d)
    idx0, off0 = pipe.next_batch(B, [0, 1])                 # 6 + 6: both partitions half read
    idx1, off1 = pipe.next_batch(B, [0, 1, 2])              # 4 each wanted; worker 2 has nothing to get
    assert off1[-1] == B and sorted(idx0 + idx1) == list(range(N))
    sizes = [off1[k + 1] - off1[k] for k in range(3)]
    assert sizes[2] == 0 and sizes[0] + sizes[1] == B       # its share went round to those who hold data


def test_save_and_load_continue_the_same_sequence():
    N, d, B = 240, 16, 24
    a = DataPipeline(8, N, d)
    sched = [[0, 1], [0, 1, 2], [2, 0], [5, 6, 7, 8], [5], [5, 9, 10], [1, 2]]
    for w in sched[:3]:
        a.next_batch(B, w)
    b = DataPipeline.load(a.save())
    for w in sched[3:] * 3:
        assert a.next_batch(B, w) == b.next_batch(B, w)


def test_bad_requests_are_rejected():
    with pytest.raises(ValueError):
        DataPipeline(0, 10, 11)
    with pytest.raises(ValueError):
        DataPipeline(0, 10, 7)                              # ceil(10/7) = 2: partitions 5 and 6 would be empty
    p = DataPipeline(0, 24, 4)
    with pytest.raises(ValueError):
        p.next_batch(12, [0, 0])
    with pytest.raises(ValueError):
        p.next_batch(10, [0, 1])                            # 10 does not divide 24
    with pytest.raises(ValueError):
        p.next_batch(12, [0, 1, 2, 3, 4])                   # 12 % 5
