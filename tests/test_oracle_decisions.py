"""What a ReLU / max-pool network's gradient does under a perturbation of rounding size (CPU, oracle only).

The backward pass takes discrete decisions from the forward activations (which outputs a ReLU let through,
which element a max pool picked).  Two computations of the same step that differ by rounding - float32
matrix-core sums on the GPU against float64 loops here - agree on almost all of them; where a
pre-activation lies within the rounding error of zero they may not, and then the gradient differs by a
whole term however exact the arithmetic is.  These tests show, inside the oracle, that this is the ONLY
way a small perturbation moves the gradient by more than its own size:
  (a) no decision changed  =>  the gradient moves in proportion to the perturbation;
  (b) some changed         =>  the gradient jumps, and the jump is reproduced by the unperturbed
                               computation with just those decisions swapped.
This is why the GPU parity tests compare free-running gradients "given the same decisions" and pin the
decisions for the layer-by-layer comparisons."""
import numpy as np
import pytest

import synth_inputs
from oracle import oracle as O
from test_oracle_nets import TINY

SMOOTH = 10.0        # measured: the gradient of these nets moves by about 4x a relative parameter perturbation


def _setup(name):
    t = TINY[name]
    o = O.Oracle(t["model"], 3, 16, 8, graph_kwargs=t["kw"])
    x, y = synth_inputs.dataset(11, 16, *t["hwc"], t["classes"])
    rng = np.random.default_rng(5)
    o.w = o.w + 0.1 * rng.standard_normal(o.w.size)        # biases, shifts and scales off their initial values
    return o, x[:8].astype(np.float64), y[:8]


def _flips(d0, d1):
    assert d0.keys() == d1.keys()
    return sum(int(np.sum(d0[k] != d1[k])) for k in d0)


@pytest.mark.parametrize("name", ["resnet50", "resnet20", "vgg16"])
def test_gradient_moves_smoothly_unless_a_decision_flips(name):
    o, xb, yb = _setup(name)
    w0 = o.w.copy()
    _, g0 = o.forward_backward(xb, yb)
    d0 = o.last_decisions
    n0 = np.linalg.norm(g0)
    assert sum(v.size for v in d0.values()) > 1000
    seen_flip = seen_quiet = 0
    biggest_jump = 0.0
    # 2^-24 is float32's rounding, 2^-9 bfloat16's; in between to see both regimes on nets this small
    for delta in (2.0 ** -24, 1e-4, 2.0 ** -9):
        for seed in range(4):
            r = np.random.default_rng(100 + seed)
            o.w = w0 * (1.0 + delta * r.standard_normal(w0.size))
            _, g1 = o.forward_backward(xb, yb)
            d1 = o.last_decisions
            flips = _flips(d0, d1)
            moved = np.linalg.norm(g1 - g0) / n0
            # the unperturbed model with the perturbed run's decisions
            o.w = w0.copy()
            _, g0_swapped = o.forward_backward(xb, yb, decisions=d1)
            rest = np.linalg.norm(g1 - g0_swapped) / n0
            assert rest <= SMOOTH * delta, (delta, seed, flips, rest)        # (b): the swapped bits explain the jump
            if flips == 0:
                seen_quiet += 1
                assert moved <= SMOOTH * delta, (delta, seed, moved)         # (a)
                assert np.array_equal(g0_swapped, g0)
            else:
                seen_flip += 1
                biggest_jump = max(biggest_jump, moved / max(rest, 1e-300))
    assert seen_quiet >= 4, "float32-size perturbations flipped decisions on a net this small?"
    assert seen_flip >= 1, "no perturbation flipped a decision: the test shows nothing"
    assert biggest_jump > 5.0, biggest_jump     # a flip moves the gradient by far more than the perturbation does


def test_float32_rounding_without_a_flip_stays_far_inside_the_float32_bar():
    """At float32's rounding size the smooth part is ~1e-6 of the gradient: two float32-accurate computations
    that take the same decisions agree a hundred times better than the 1e-4 bar."""
    o, xb, yb = _setup("resnet50")
    w0 = o.w.copy()
    _, g0 = o.forward_backward(xb, yb)
    d0 = o.last_decisions
    r = np.random.default_rng(7)
    o.w = w0 * (1.0 + 2.0 ** -24 * r.standard_normal(w0.size))
    _, g1 = o.forward_backward(xb, yb, decisions=d0)
    assert np.linalg.norm(g1 - g0) <= 1e-5 * np.linalg.norm(g0)


def test_one_flipped_relu_changes_the_gradient_by_a_whole_term():
    """Flip the single ReLU decision whose output is closest to zero: forward values are untouched (the
    output is ~0 either way), yet the layer's own gradient changes by about one part in sqrt(elements)."""
    o, xb, yb = _setup("resnet20")
    _, g0 = o.forward_backward(xb, yb)
    d0 = {k: v.copy() for k, v in o.last_decisions.items()}
    act = o.last_act
    # the smallest positive ReLU output of the first batch norm
    i = next(i for i, op in enumerate(o.graph.ops) if op["kind"] == "bn" and op["relu"])
    y_ = act[o.graph.ops[i]["y"]]
    pos = np.where(y_ > 0, y_, np.inf)
    at = np.unravel_index(np.argmin(pos), pos.shape)
    assert d0[i][at]
    d0[i][at] = False
    _, g1 = o.forward_backward(xb, yb, decisions=d0)
    op = o.graph.ops[i]
    C = op["C"]
    sl = slice(op["b_off"], op["b_off"] + C)               # the layer's shift gradient = column sums of the masked dy
    changed = np.abs(g1[sl] - g0[sl]) > 0
    assert changed.sum() == 1 and changed[at[-1]]          # exactly the flipped element's channel
    assert np.linalg.norm(g1 - g0) > 1e-4 * np.linalg.norm(g0)
