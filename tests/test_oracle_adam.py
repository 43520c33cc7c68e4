"""Pins of the oracle's Adam update (the optimizer of the paper's usage example,
section 3.2 Listing 1; steps of Kingma & Ba's Algorithm 1) against closed forms
and special cases that the algorithm fixes.  CPU only."""
import numpy as np
import pytest

import synth_inputs
from oracle import oracle as O


def _run(w0, grad_seq, lr, b1, b2, eps, wd=0.0):
    w, m, s = w0.copy(), np.zeros_like(w0), np.zeros_like(w0)
    traj = []
    for t, g in enumerate(grad_seq, start=1):
        w, m, s = O.adam_update(w, m, s, [g], t, lr, b1, b2, eps, wd)
        traj.append((w.copy(), m.copy(), s.copy()))
    return traj


def test_first_update_moves_every_weight_by_lr_g_over_abs_g_plus_eps():
    """t = 1 from zero moments: the bias corrections cancel the (1-beta) factors exactly, whatever the betas."""
    rng = np.random.default_rng(0)
    g = rng.standard_normal(50) * np.logspace(-6, 3, 50)
    w0 = rng.standard_normal(50)
    for b1, b2, eps in [(0.9, 0.999, 0.5), (0.5, 0.9, 1e-8), (0.0, 0.99, 0.01)]:
        (w1, m1, s1), = _run(w0, [g], 0.01, b1, b2, eps)
        assert np.allclose(w1, w0 - 0.01 * g / (np.abs(g) + eps), rtol=1e-12, atol=0)
        assert np.allclose(m1, (1 - b1) * g, rtol=1e-14) and np.allclose(s1, (1 - b2) * g * g, rtol=1e-14)


def test_constant_gradient_gives_equal_steps():
    """With the same gradient every time the corrected moments are g and g^2 at every t, so
    w_T = w_0 - T lr g / (|g| + eps), m_T = (1 - beta1^T) g, s_T = (1 - beta2^T) g^2.  An eps as large as the
    gradients separates this from the forms that fold the corrections into the step size or put eps
    under the root."""
    rng = np.random.default_rng(1)
    g = rng.standard_normal(20)
    w0 = rng.standard_normal(20)
    lr, b1, b2, eps, T = 0.003, 0.9, 0.999, 0.7, 25
    traj = _run(w0, [g] * T, lr, b1, b2, eps)
    for t, (w, m, s) in enumerate(traj, start=1):
        assert np.allclose(w, w0 - t * lr * g / (np.abs(g) + eps), rtol=1e-11, atol=1e-14)
        assert np.allclose(m, (1 - b1 ** t) * g, rtol=1e-12)
        assert np.allclose(s, (1 - b2 ** t) * g * g, rtol=1e-12)


def test_zero_betas_reduce_to_sign_descent():
    """beta1 = beta2 = 0, eps = 0: every weight moves by exactly lr against the sign of its gradient."""
    rng = np.random.default_rng(2)
    w0 = rng.standard_normal(30)
    gs = [rng.standard_normal(30) for _ in range(6)]
    traj = _run(w0, gs, 0.05, 0.0, 0.0, 0.0)
    ref = w0.copy()
    for g, (w, _, _) in zip(gs, traj):
        ref = ref - 0.05 * np.sign(g)
        assert np.allclose(w, ref, rtol=0, atol=1e-15)


def test_rescaling_all_gradients_changes_nothing_without_eps():
    rng = np.random.default_rng(3)
    w0 = rng.standard_normal(40)
    gs = [rng.standard_normal(40) for _ in range(12)]
    a = _run(w0, gs, 0.01, 0.9, 0.999, 0.0)
    b = _run(w0, [1e3 * g for g in gs], 0.01, 0.9, 0.999, 0.0)
    assert np.allclose(a[-1][0], b[-1][0], rtol=1e-12, atol=1e-15)
    assert np.allclose(1e3 * a[-1][1], b[-1][1], rtol=1e-12) and np.allclose(1e6 * a[-1][2], b[-1][2], rtol=1e-12)


def test_step_size_bound():
    """Section 2.1 of Kingma & Ba: |delta w| <= lr (1-beta1)/sqrt(1-beta2) when (1-beta1) > sqrt(1-beta2), else <= lr
    (up to the initialisation bias terms, which only shrink it)."""
    rng = np.random.default_rng(4)
    for b1, b2 in [(0.9, 0.999), (0.5, 0.999), (0.9, 0.9)]:
        w0 = np.zeros(200)
        gs = [rng.standard_normal(200) * (10.0 if t % 7 == 0 else 0.01) for t in range(60)]   # sparse large gradients
        traj = _run(w0, gs, 1.0, b1, b2, 0.0)
        bound = max(1.0, (1 - b1) / np.sqrt(1 - b2))
        prev = w0
        for w, _, _ in traj:
            assert np.max(np.abs(w - prev)) <= bound * (1 + 1e-12)
            prev = w


def test_weight_decay_enters_through_the_gradient():
    """Zero loss gradient, wd > 0: the first update shrinks every weight by lr (eps -> 0), as a gradient wd*w does."""
    w0 = np.array([2.0, -3.0, 0.5])
    (w1, m1, _), = [t for t in _run(w0, [np.zeros(3)], 0.1, 0.9, 0.999, 0.0, wd=0.01)]
    assert np.allclose(w1, w0 - 0.1 * np.sign(w0), atol=1e-15)
    assert np.allclose(m1, 0.1 * 0.01 * w0)


def test_aggregation_is_the_mean_and_the_weighted_sum():
    rng = np.random.default_rng(5)
    w0 = rng.standard_normal(10)
    Gs = [rng.standard_normal(10) for _ in range(4)]
    z = np.zeros(10)
    a = O.adam_update(w0, z, z, Gs, 1, 0.01, 0.9, 0.999, 1e-8, 0.0)
    b = O.adam_update(w0, z, z, [sum(Gs) / 4], 1, 0.01, 0.9, 0.999, 1e-8, 0.0)
    c = O.adam_update(w0, z, z, Gs, 1, 0.01, 0.9, 0.999, 1e-8, 0.0, weights=[0.25] * 4)
    d = O.adam_update(w0, z, z, Gs[:2], 1, 0.01, 0.9, 0.999, 1e-8, 0.0, weights=[0.75, 0.25])
    e = O.adam_update(w0, z, z, [0.75 * Gs[0] + 0.25 * Gs[1]], 1, 0.01, 0.9, 0.999, 1e-8, 0.0)
    for x, y in [(a, b), (a, c), (d, e)]:
        assert all(np.allclose(u, v, rtol=1e-13, atol=1e-16) for u, v in zip(x, y))


TINY_MLP = dict(H=1, W=1, C=12, hidden=(8, 6), classes=4)


@pytest.mark.parametrize("p", [2, 4, 8])
def test_elasticity_invariant_of_a_whole_adam_job(p):
    """Sections 3.1 / 4: with the aggregate batch fixed and no batch norm, the trajectory does not depend on p."""
    N, B = 32, 8
    x, y = synth_inputs.dataset(11, N, 1, 1, 12, 4)
    a = O.Oracle("mlp", 3, N, B, lr=0.01, optimizer="adam", graph_kwargs=TINY_MLP)
    b = O.Oracle("mlp", 3, N, B, lr=0.01, optimizer="adam", graph_kwargs=TINY_MLP)
    for _ in range(5):
        la, lb = a.step(1, x, y), b.step(p, x, y)
        assert abs(la - lb) < 1e-12
    assert np.linalg.norm(a.w - b.w) <= 1e-11 * np.linalg.norm(a.w)
    assert np.linalg.norm(a.s - b.s) <= 1e-11 * np.linalg.norm(a.s)
    assert np.linalg.norm(a.w - O.he_init(a.graph, 3)) > 1e-3          # it did move


def test_adam_job_first_step_against_the_closed_form():
    """One whole step of the job: delta w = -lr * G/(|G| + eps) with G the oracle's own (pinned) gradient."""
    N, B = 16, 8
    x, y = synth_inputs.dataset(11, N, 1, 1, 12, 4)
    o = O.Oracle("mlp", 3, N, B, lr=0.01, wd=0.0, optimizer="adam", eps=1e-3, graph_kwargs=TINY_MLP)
    w0 = o.w.copy()
    idx, off = O.shard(3, N, B, 1, 0, 0)
    _, G = o.forward_backward(x[idx].astype(np.float64), y[idx])
    o.step(1, x, y)
    assert np.allclose(o.w, w0 - 0.01 * G / (np.abs(G) + 1e-3), rtol=1e-12, atol=1e-15)


def test_adam_snapshot_carries_both_moments_and_resumes():
    N, B = 32, 8
    x, y = synth_inputs.dataset(11, N, 1, 1, 12, 4)
    a = O.Oracle("mlp", 3, N, B, lr=0.01, optimizer="adam", graph_kwargs=TINY_MLP)
    for _ in range(3):
        a.step(2, x, y)
    blob = a.snapshot()
    P, R = a.graph.P, a.graph.R
    assert len(blob) == O.SNAPSHOT_HEADER_BYTES + 4 * (3 * P + R)
    b = O.Oracle("mlp", 99, N, B, lr=0.01, optimizer="adam", graph_kwargs=TINY_MLP)
    b.restore(blob)
    a32 = O.Oracle("mlp", 3, N, B, lr=0.01, optimizer="adam", graph_kwargs=TINY_MLP)
    a32.restore(blob)                       # the sender continues from the float32 image as well
    for _ in range(3):
        assert a32.step(4, x, y) == b.step(4, x, y)
    assert np.array_equal(a32.w, b.w) and np.array_equal(a32.s, b.s) and b.step_count == 6
    with pytest.raises(AssertionError):
        O.Oracle("mlp", 3, N, B, graph_kwargs=TINY_MLP).restore(blob)      # a momentum job refuses an Adam image
