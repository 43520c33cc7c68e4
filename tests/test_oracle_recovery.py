"""Pins for approximate recovery (section 4.2, failure recovery): the survivors redo the current mini-batch
(CPU, oracle only)."""
import numpy as np
import pytest

from oracle import oracle as O
from test_oracle_nets import make


def test_survivor_cut_is_as_even_as_the_counts_allow():
    assert O.Oracle.survivor_cut(32, 3).tolist() == [0, 11, 22, 32]
    assert O.Oracle.survivor_cut(24, 3).tolist() == [0, 8, 16, 24]
    assert O.Oracle.survivor_cut(8, 3).tolist() == [0, 3, 6, 8]
    assert O.Oracle.survivor_cut(5, 7).tolist() == [0, 1, 2, 3, 4, 5, 5, 5]
    for B in (1, 7, 32, 257):
        for s in (1, 2, 3, 7, 8):
            off = O.Oracle.survivor_cut(B, s)
            sizes = np.diff(off)
            assert off[0] == 0 and off[-1] == B and sizes.max() - sizes.min() <= 1 and np.all(np.diff(sizes) <= 0)


@pytest.mark.parametrize("p,lost", [(4, 0), (4, 2), (2, 1), (8, 7)])
def test_redone_mini_batch_is_the_sgd_equation_of_section_2_1(p, lost):
    """Without momentum and weight decay, on a net without batch norm: after the failure of one of p workers
    the model has moved by -lr/|B| times the sum of the per-sample gradients of the SAME mini-batch (B = 8 is
    not a multiple of 3 or 7, so the survivors' shards are unequal), exactly once."""
    o, x, y = make("mlp", N=16, B=8, lr=0.2, momentum=0.0, wd=0.0)
    o.step(1, x, y)                                        # somewhere inside the epoch
    w0 = o.w.copy()
    idx, _ = O.shard(o.seed, o.N, o.B, 1, o.epoch, o.step_in_epoch)
    per_sample = [o.forward_backward(x[i:i + 1].astype(np.float64), y[i:i + 1]) for i in idx]
    loss, discarded = o.redo_with_survivors(p, lost, x, y)
    np.testing.assert_allclose(o.w, w0 - 0.2 / 8 * sum(g for _, g in per_sample), rtol=1e-11, atol=1e-13)
    assert abs(loss - np.mean([l for l, _ in per_sample])) < 1e-12
    assert len(discarded) == p - 1
    assert (o.step_count, o.epoch, o.step_in_epoch) == (2, 1, 0)      # progress moved on by one mini-batch
    # the plain mean of the survivors' gradients would be something else when their shards are unequal
    if 8 % (p - 1):
        off = O.Oracle.survivor_cut(8, p - 1)
        gs = [o.forward_backward(x[idx[off[k]:off[k + 1]]].astype(np.float64), y[idx[off[k]:off[k + 1]]])[1]
              for k in range(p - 1)]
        o2, _, _ = make("mlp", N=16, B=8, lr=0.2, momentum=0.0, wd=0.0)
        o2.step(1, x, y)
        o2.w = w0.copy()
        gs = [o2.forward_backward(x[idx[off[k]:off[k + 1]]].astype(np.float64), y[idx[off[k]:off[k + 1]]])[1]
              for k in range(p - 1)]
        wrong = w0 - 0.2 * sum(gs) / (p - 1)
        assert np.linalg.norm(wrong - o.w) > 1e-6 * np.linalg.norm(o.w - w0)


def test_recovery_equals_a_job_that_ran_with_the_survivors_all_along():
    """The redone step is an ordinary step of p-1 workers on the survivors' cut: with batch norm the result is
    that of p-1 independent single-worker passes, weighted by their shares; the lost worker leaves no trace."""
    a, x, y = make("resnet20", N=16, B=8)
    b, _, _ = make("resnet20", N=16, B=8)
    a.redo_with_survivors(4, 1, x, y)
    idx, _ = O.shard(b.seed, b.N, b.B, 1, 0, 0)
    b.step(3, x, y, idx, O.Oracle.survivor_cut(8, 3))
    assert np.array_equal(a.w, b.w) and np.array_equal(a.v, b.v) and np.array_equal(a.running, b.running)
    assert (a.step_count, a.epoch, a.step_in_epoch) == (b.step_count, b.epoch, b.step_in_epoch)


def test_joiner_adopts_the_optimizer_coefficients_of_the_job():
    """Section 4.2: the job's meta-data travels with the model.  A joiner created with another learning rate,
    momentum and weight decay continues exactly as the job whose image it received."""
    o, x, y = make("resnet20", N=16, B=8, lr=0.05, momentum=0.8, wd=1e-3)
    o.step(2, x, y)
    blob = o.snapshot()
    j, _, _ = make("resnet20", N=16, B=8, seed=99, lr=0.5, momentum=0.0, wd=0.0)
    j.restore(blob)
    o.restore(blob)
    assert (j.lr, j.momentum, j.wd) == (o.lr, o.momentum, o.wd)
    assert abs(j.lr - 0.05) < 1e-8 and abs(j.momentum - 0.8) < 1e-7
    for p in (4, 1):
        o.step(p, x, y)
        j.step(p, x, y)
    assert np.array_equal(o.w, j.w) and np.array_equal(o.v, j.v)
