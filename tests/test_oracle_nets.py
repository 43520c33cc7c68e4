"""Pins for the oracle's whole iteration: finite-difference gradients on tiny
nets, the elasticity invariant, the SGD equation, snapshots (CPU only)."""
import os

import numpy as np
import pytest

import synth_inputs
from oracle import oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")

TINY = {
    "mlp": dict(model="mlp", kw=dict(H=1, W=1, C=12, hidden=(8, 6), classes=4), hwc=(1, 1, 12), classes=4),
    "resnet20": dict(model="resnet20", kw=dict(H=8, W=8, C=3, classes=4, widths=(4, 8), blocks=1),
                     hwc=(8, 8, 3), classes=4),
    "resnet50": dict(model="resnet50", kw=dict(H=16, W=16, C=3, classes=5, base=4, blocks=(1, 1)),
                     hwc=(16, 16, 3), classes=5),
    "vgg16": dict(model="vgg16", kw=dict(H=32, W=32, C=3, classes=4, base=2, fc=8), hwc=(32, 32, 3), classes=4),
    "vgg19": dict(model="vgg16", kw=dict(H=32, W=32, C=3, classes=4, base=2, fc=8, groups=(2, 2, 4, 4, 4)),
                  hwc=(32, 32, 3), classes=4),
    # 67 -> 16 -> 7 -> 3 -> 1: the smallest side that leaves every pool a full window, plus a ragged edge
    "alexnet": dict(model="alexnet", kw=dict(H=67, W=67, C=3, classes=4, base=2, fc=8), hwc=(67, 67, 3), classes=4),
}


def make(name, N=16, B=8, seed=3, **kw):
    t = TINY[name]
    o = O.Oracle(t["model"], seed, N, B, graph_kwargs=t["kw"], **kw)
    x, y = synth_inputs.dataset(11, N, *t["hwc"], t["classes"])
    return o, x, y


def test_param_counts_match_the_published_architectures():
    for line in open(os.path.join(GOLD, "param_counts.txt")):
        if line.startswith("#"):
            continue
        name, count = line.split()
        builder, kw = O.VARIANTS.get(name, (name, {}))
        assert O.BUILDERS[builder](**kw).P == int(count), name


@pytest.mark.parametrize("name", list(TINY))
def test_gradient_by_central_differences(name):
    o, x, y = make(name)
    rng = np.random.default_rng(5)
    # move biases / beta off zero and gamma off one so every term is exercised
    o.w = o.w + 0.1 * rng.standard_normal(o.w.size)
    xb, yb = x[:6].astype(np.float64), y[:6]
    loss, G = o.forward_backward(xb, yb)
    w0 = o.w.copy()
    h = 1e-6
    picks = []
    for (tname, off, shape, _) in o.graph.tensors:
        n = int(np.prod(shape))
        picks += list(off + rng.choice(n, size=min(3, n), replace=False))
    worst = 0.0
    for i in picks:
        o.w = w0.copy(); o.w[i] += h
        lp, _ = o.forward_backward(xb, yb)
        o.w = w0.copy(); o.w[i] -= h
        lm, _ = o.forward_backward(xb, yb)
        fd = (lp - lm) / (2 * h)
        worst = max(worst, abs(fd - G[i]) / max(abs(fd), abs(G[i]), 1e-3))
    assert worst < 1e-6, worst


@pytest.mark.parametrize("name", ["mlp", "vgg16", "alexnet"])
@pytest.mark.parametrize("p", [1, 2, 4, 8])
def test_elasticity_invariant_without_batchnorm(name, p):
    """Section 3.1 / section 4: with the aggregate batch fixed, the mean of the
    p local gradients is the single worker's gradient on the whole batch."""
    o, x, y = make(name, N=16, B=8)
    idx, off = O.shard(o.seed, o.N, o.B, p, 0, 1)
    _, G_all = o.forward_backward(x[idx].astype(np.float64), y[idx])
    Gs = [o.forward_backward(x[idx[off[k]:off[k + 1]]].astype(np.float64), y[idx[off[k]:off[k + 1]]])[1]
          for k in range(p)]
    gbar = sum(Gs) / p
    assert np.linalg.norm(gbar - G_all) <= 1e-12 * np.linalg.norm(G_all)


def test_step_equals_sgd_equation_of_section_2_1():
    """momentum = wd = 0: w' = w - lr/|B| * sum_i grad f(x_i, w), per-sample gradients."""
    o, x, y = make("mlp", N=16, B=8, lr=0.2, momentum=0.0, wd=0.0)
    w0 = o.w.copy()
    idx, _ = O.shard(o.seed, o.N, o.B, 1, 0, 0)
    per_sample = [o.forward_backward(x[i:i + 1].astype(np.float64), y[i:i + 1])[1] for i in idx]
    o.step(4, x, y)
    np.testing.assert_allclose(o.w, w0 - 0.2 / 8 * sum(per_sample), rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("sizes", [[3, 1, 4], [5, 0, 3], [1, 7], [2, 2, 2, 2]])
def test_unequal_shards_still_give_the_sgd_equation_of_section_2_1(sizes):
    """Shards of unequal size (a tail mini-batch of the data pipeline, a mini-batch redone by the survivors of a
    failure), every worker weighted by its share of the batch: the step is still w - lr/|B| * the sum of the
    per-sample gradients of the whole mini-batch, and the reported loss the mean over the mini-batch."""
    o, x, y = make("mlp", N=16, B=8, lr=0.2, momentum=0.0, wd=0.0)
    w0 = o.w.copy()
    idx, _ = O.shard(o.seed, o.N, o.B, 1, 0, 0)
    per_sample = [o.forward_backward(x[i:i + 1].astype(np.float64), y[i:i + 1]) for i in idx]
    off = np.concatenate([[0], np.cumsum(sizes)])
    loss = o.step(len(sizes), x, y, idx, off)
    np.testing.assert_allclose(o.w, w0 - 0.2 / 8 * sum(g for _, g in per_sample), rtol=1e-11, atol=1e-13)
    assert abs(loss - np.mean([l for l, _ in per_sample])) < 1e-12


def test_weighted_update_by_hand():
    """w = 1, v = 0.5, gradients 2 and -1 with shares 3/4 and 1/4, lr 0.1, momentum 0.9, wd 0.01:
    aggregate 1.25, g = 1.26, v = 0.45 + 1.26 = 1.71, w = 1 - 0.171 = 0.829."""
    w, v = O.sgd_momentum_update(np.array([1.0]), np.array([0.5]), [np.array([2.0]), np.array([-1.0])], 0.1, 0.9, 0.01,
                                 weights=[0.75, 0.25])
    assert abs(v[0] - 1.71) < 1e-15 and abs(w[0] - 0.829) < 1e-15
    # equal shares are the mean
    g = [np.array([0.3, -2.0]), np.array([1.1, 0.5]), np.array([-0.7, 4.0])]
    a = O.sgd_momentum_update(np.array([1.0, 2.0]), np.array([0.1, -0.1]), g, 0.05, 0.9, 5e-4)
    b = O.sgd_momentum_update(np.array([1.0, 2.0]), np.array([0.1, -0.1]), g, 0.05, 0.9, 5e-4, weights=[1 / 3] * 3)
    np.testing.assert_allclose(a[0], b[0], rtol=1e-15)
    np.testing.assert_allclose(a[1], b[1], rtol=1e-15)


def test_trajectory_independent_of_p_schedule_without_batchnorm():
    a, x, y = make("vgg16", N=16, B=8, lr=0.01)
    b, _, _ = make("vgg16", N=16, B=8, lr=0.01)
    for pa, pb in [(1, 2), (1, 4), (1, 8), (1, 4)]:
        a.step(pa, x, y)
        b.step(pb, x, y)
    assert np.linalg.norm(a.w - b.w) <= 1e-11 * np.linalg.norm(a.w)
    assert (a.epoch, a.step_in_epoch) == (2, 0) == (b.epoch, b.step_in_epoch)


def test_batchnorm_shards_are_independent_single_worker_runs():
    o, x, y = make("resnet20", N=16, B=8)
    ref, _, _ = make("resnet20", N=16, B=8)
    idx, off = O.shard(o.seed, o.N, o.B, 2, 0, 0)
    o.step(2, x, y)
    Gs = [ref.forward_backward(x[idx[off[k]:off[k + 1]]].astype(np.float64), y[idx[off[k]:off[k + 1]]])[1]
          for k in range(2)]
    for k in range(2):
        np.testing.assert_array_equal(o.last_grads[k], Gs[k])
    # and per-shard statistics really differ from whole-batch statistics
    _, G_all = ref.forward_backward(x[idx].astype(np.float64), y[idx])
    assert np.linalg.norm(sum(Gs) / 2 - G_all) > 1e-3 * np.linalg.norm(G_all)


def test_running_statistics_follow_worker_zero():
    o, x, y = make("resnet20", N=16, B=8)
    idx, off = O.shard(o.seed, o.N, o.B, 2, 0, 0)
    o.step(2, x, y)
    op = next(op for op in o.graph.ops if op["kind"] == "bn")
    C = op["C"]
    x0 = x[idx[off[0]:off[1]]].astype(np.float64)
    w = o.graph.tensors[0]
    ref, _, _ = make("resnet20", N=16, B=8)
    conv = O.conv2d_forward(x0, ref.w[w[1]:w[1] + int(np.prod(w[2]))].reshape(w[2]), None, 1, 1)
    flat = conv.reshape(-1, C)
    np.testing.assert_allclose(o.running[:C], 0.1 * flat.mean(0), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(o.running[C:2 * C], 0.9 + 0.1 * flat.var(0, ddof=1), rtol=1e-12)


def test_he_init_statistics_and_determinism():
    g = O.build_resnet20()
    w = O.he_init(g, 0)
    assert np.array_equal(w, O.he_init(g, 0)) and not np.array_equal(w, O.he_init(g, 1))
    assert np.array_equal(w, w.astype(np.float32).astype(np.float64))
    for (name, off, shape, fan_in) in g.tensors:
        n = int(np.prod(shape))
        t = w[off:off + n]
        if fan_in == 0:
            assert np.all(t == (1.0 if name.endswith(".g") else 0.0))
        elif n >= 4000:
            assert abs(t.var() / (2.0 / fan_in) - 1) < 0.1
            assert abs(t.mean()) < 4 * np.sqrt(2.0 / fan_in / n)
            z = t / t.std()
            assert abs((z ** 4).mean() - 3.0) < 0.35     # Gaussian kurtosis


def test_snapshot_roundtrip_and_resume():
    o, x, y = make("resnet20", N=16, B=8)
    o.step(2, x, y)
    blob = o.snapshot()
    assert len(blob) == O.SNAPSHOT_HEADER_BYTES + 4 * (2 * o.graph.P + o.graph.R)
    assert np.array_equal(np.frombuffer(blob, np.float32, o.graph.P, O.SNAPSHOT_HEADER_BYTES),
                          o.w.astype(np.float32))
    j, _, _ = make("resnet20", N=16, B=8, seed=99)     # the joiner: different initial model
    j.restore(blob)
    o.restore(blob)                                     # existing worker continues from the same float32 image
    for p in (4, 1):
        o.step(p, x, y)
        j.step(p, x, y)
    assert np.array_equal(o.w, j.w) and np.array_equal(o.v, j.v) and np.array_equal(o.running, j.running)
    assert (j.step_count, j.epoch, j.step_in_epoch) == (3, 1, 1)
