"""Pins for the oracle's layer arithmetic: library routines on special cases,
closed forms, invariants and finite differences (CPU only)."""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(7)

CONV_CASES = [
    # N H W C K R stride pad
    (2, 8, 8, 3, 4, 3, 1, 1),
    (2, 9, 7, 5, 6, 3, 2, 1),
    (1, 12, 12, 3, 4, 7, 2, 3),
    (3, 6, 6, 8, 5, 1, 1, 0),
    (2, 7, 7, 4, 6, 1, 2, 0),
    (2, 1, 1, 20, 7, 1, 1, 0),
]


def _torch_conv(x, w, b, stride, pad):
    xt = torch.tensor(x).permute(0, 3, 1, 2).requires_grad_(True)
    wt = torch.tensor(w).permute(0, 3, 1, 2).requires_grad_(True)
    bt = torch.tensor(b).requires_grad_(True)
    y = F.conv2d(xt, wt, bt, stride=stride, padding=pad)
    return xt, wt, bt, y


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_matches_library_routine(case):
    N, H, W, C, K, R, st, pad = case
    x = rng.standard_normal((N, H, W, C))
    w = rng.standard_normal((K, R, R, C))
    b = rng.standard_normal(K)
    y = O.conv2d_forward(x, w, b, st, pad)
    xt, wt, bt, yt = _torch_conv(x, w, b, st, pad)
    np.testing.assert_allclose(y, yt.detach().permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)
    dy = rng.standard_normal(y.shape)
    yt.backward(torch.tensor(dy).permute(0, 3, 1, 2))
    dx = O.conv2d_backward_input(dy, w, x.shape, st, pad)
    dw, db = O.conv2d_backward_weight(x, dy, w.shape, st, pad, True)
    np.testing.assert_allclose(dx, xt.grad.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dw, wt.grad.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(db, bt.grad.numpy(), rtol=1e-12, atol=1e-12)


def test_conv_1x1_is_a_matrix_product():
    x = rng.standard_normal((2, 5, 4, 6))
    w = rng.standard_normal((3, 1, 1, 6))
    y = O.conv2d_forward(x, w, None, 1, 0)
    np.testing.assert_allclose(y.reshape(-1, 3), x.reshape(-1, 6) @ w.reshape(3, 6).T, rtol=1e-13)


def test_conv_centred_delta_is_identity():
    C = 4
    x = rng.standard_normal((2, 6, 6, C))
    w = np.zeros((C, 3, 3, C))
    for c in range(C):
        w[c, 1, 1, c] = 1.0
    np.testing.assert_array_equal(O.conv2d_forward(x, w, None, 1, 1), x)


def test_conv_off_centre_delta_shifts():
    # a transposed kernel or a flipped (true convolution) kernel would shift the wrong way
    x = rng.standard_normal((1, 5, 5, 1))
    w = np.zeros((1, 3, 3, 1))
    w[0, 0, 2, 0] = 1.0           # tap at row -1, column +1
    y = O.conv2d_forward(x, w, None, 1, 1)
    assert y[0, 2, 2, 0] == x[0, 1, 3, 0]
    assert y[0, 0, 0, 0] == 0.0   # the tap falls into the zero padding


def test_maxpool_brute_force_and_first_max_rule():
    for (H, W, k, st, pad) in [(7, 7, 3, 2, 1), (6, 6, 2, 2, 0), (5, 4, 3, 2, 1)]:
        x = rng.integers(0, 4, size=(2, H, W, 3)).astype(np.float64)   # many ties
        y, arg = O.maxpool_forward(x, k, st, pad)
        Ho, Wo = y.shape[1:3]
        for n in range(2):
            for ho in range(Ho):
                for wo in range(Wo):
                    for c in range(3):
                        cand = [(x[n, h, w_, c], h * W + w_)
                                for h in range(ho * st - pad, ho * st - pad + k) if 0 <= h < H
                                for w_ in range(wo * st - pad, wo * st - pad + k) if 0 <= w_ < W]
                        best = max(v for v, _ in cand)
                        first = [i for v, i in cand if v == best][0]
                        assert y[n, ho, wo, c] == best and arg[n, ho, wo, c] == first
        dy = rng.standard_normal(y.shape)
        dx = O.maxpool_backward(dy, arg, x.shape)
        assert abs(dx.sum() - dy.sum()) < 1e-12
        ref = np.zeros_like(x)
        for n, ho, wo, c in np.ndindex(*y.shape):
            a = arg[n, ho, wo, c]
            ref[n, a // W, a % W, c] += dy[n, ho, wo, c]
        np.testing.assert_allclose(dx, ref, atol=1e-15)


def test_softmax_ce_closed_forms():
    for C in (10, 1000):
        z = np.zeros((4, C))
        labels = np.array([0, 1, 2, 3])
        loss, prob = O.softmax_ce_forward(z, labels)
        assert abs(loss - math.log(C)) < 1e-12
    z = rng.standard_normal((5, 7)) * 30            # needs the max subtraction
    labels = rng.integers(0, 7, 5)
    loss, prob = O.softmax_ce_forward(z, labels)
    lt = F.cross_entropy(torch.tensor(z), torch.tensor(labels))
    assert abs(loss - lt.item()) < 1e-10
    dz = O.softmax_ce_backward(prob, labels)
    np.testing.assert_allclose(dz.sum(axis=1), 0, atol=1e-15)
    zt = torch.tensor(z, requires_grad=True)
    F.cross_entropy(zt, torch.tensor(labels)).backward()
    np.testing.assert_allclose(dz, zt.grad.numpy(), atol=1e-14)


def test_batchnorm_invariants():
    x = rng.standard_normal((3, 4, 4, 5)) * 3 + 2
    gamma = rng.standard_normal(5)
    beta = rng.standard_normal(5)
    y, xhat, mean, var = O.batchnorm_forward(x, np.ones(5), np.zeros(5))
    np.testing.assert_allclose(y.reshape(-1, 5).mean(0), 0, atol=1e-13)
    np.testing.assert_allclose(y.reshape(-1, 5).var(0), var / (var + O.BN_EPS), rtol=1e-12)
    dy = rng.standard_normal(x.shape)
    y, xhat, mean, var = O.batchnorm_forward(x, gamma, beta)
    dx, dg, db = O.batchnorm_backward(dy, xhat, gamma, var)
    # the batch-norm Jacobian annihilates the constant and the xhat directions
    np.testing.assert_allclose(dx.reshape(-1, 5).sum(0), 0, atol=1e-12)
    # (the xhat direction only up to eps/var, since sum(xhat^2)/M = var/(var+eps))
    resid = gamma / np.sqrt(var + O.BN_EPS) * dg * (O.BN_EPS / (var + O.BN_EPS))
    np.testing.assert_allclose((dx * xhat).reshape(-1, 5).sum(0), resid, atol=1e-12)
    # library routine
    xt = torch.tensor(x).permute(0, 3, 1, 2).requires_grad_(True)
    gt = torch.tensor(gamma, requires_grad=True)
    bt = torch.tensor(beta, requires_grad=True)
    yt = F.batch_norm(xt, None, None, gt, bt, training=True, eps=O.BN_EPS)
    np.testing.assert_allclose(y, yt.detach().permute(0, 2, 3, 1).numpy(), rtol=1e-11, atol=1e-12)
    yt.backward(torch.tensor(dy).permute(0, 3, 1, 2))
    np.testing.assert_allclose(dx, xt.grad.permute(0, 2, 3, 1).numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dg, gt.grad.numpy(), rtol=1e-11)
    np.testing.assert_allclose(db, bt.grad.numpy(), rtol=1e-11)


def test_update_hand_worked_scalar():
    rows = [l.split() for l in open(os.path.join(GOLD, "update_scalar.txt")) if not l.startswith("#")]
    w, v = np.array([1.0]), np.array([0.0])
    for _, gp, vv, ww in rows:
        w, v = O.sgd_momentum_update(w, v, [np.array([0.5])], 0.1, 0.9, 5e-4)
        assert abs(v[0] - float(vv)) < 1e-12 and abs(w[0] - float(ww)) < 1e-12


def test_update_closed_forms():
    P = 50
    w0 = rng.standard_normal(P)
    g = [rng.standard_normal(P) for _ in range(4)]
    # momentum 0, wd 0: the plain SGD equation with the mean of the local gradients
    w1, v1 = O.sgd_momentum_update(w0, np.zeros(P), g, 0.3, 0.0, 0.0)
    np.testing.assert_allclose(w1, w0 - 0.3 * (g[0] + g[1] + g[2] + g[3]) / 4, rtol=1e-14)
    # constant gradient, wd 0: geometric series
    lr, m = 0.05, 0.9
    w, v = w0.copy(), np.zeros(P)
    for t in range(1, 8):
        w, v = O.sgd_momentum_update(w, v, [g[0]], lr, m, 0.0)
        np.testing.assert_allclose(v, g[0] * (1 - m ** t) / (1 - m), rtol=1e-12)
        s = sum((1 - m ** s_) / (1 - m) for s_ in range(1, t + 1))
        np.testing.assert_allclose(w, w0 - lr * g[0] * s, rtol=1e-12, atol=1e-13)
    # zero gradient, momentum 0: pure geometric decay of the weights
    w, v = w0.copy(), np.zeros(P)
    for t in range(1, 5):
        w, v = O.sgd_momentum_update(w, v, [np.zeros(P)], 0.1, 0.0, 0.01)
        np.testing.assert_allclose(w, w0 * (1 - 0.1 * 0.01) ** t, rtol=1e-13)
    # the order of the workers does not matter beyond rounding; a sum instead of a mean would
    wa, _ = O.sgd_momentum_update(w0, np.zeros(P), g, 0.1, 0.9, 5e-4)
    wb, _ = O.sgd_momentum_update(w0, np.zeros(P), g[::-1], 0.1, 0.9, 5e-4)
    np.testing.assert_allclose(wa, wb, rtol=1e-13)


def test_round_bf16_against_integer_reference():
    vals = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 10.0 ** rng.integers(-20, 20, 20000),
                           np.array([0.0, -0.0, 1.0, 1.00390625, 1.0078125, 1.01171875, 3.3895314e38],
                                    dtype=np.float32)]).astype(np.float32)
    got = O.round_bf16(vals).astype(np.float32)
    ref = torch.tensor(vals).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(got.view(np.uint32), ref.view(np.uint32))
    # exact ties go to the even neighbour
    assert O.round_bf16(np.array([1.00390625]))[0] == 1.0           # 1 + 2^-8  -> 1
    assert O.round_bf16(np.array([1.01171875]))[0] == 1.015625      # 1 + 3*2^-8 -> 1 + 2^-6
