"""The comparison criteria of the GPU parity tests, tested by themselves on the CPU: a plausible kernel mistake
planted in a copy of a reference result must fail them."""
import numpy as np

from parity_util import TOL, Modes, Worst, elementwise_excess, layerwise_ok, per_tensor_elementwise, relerr


def _reference(rows=100352, cols=64, seed=0):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((rows, cols))


def test_a_shifted_last_tile_row_passes_the_norm_and_fails_element_wise():
    """An output of 100352 x 64 (a 56x56 layer at a shard of 32) whose very last row holds the row before it - a
    ragged-tile indexing mistake: 64 wrong elements of 6.4 million.  Norm-wise that is 4e-3, inside the bf16
    bar; the element-wise criterion sees it."""
    from oracle.oracle import round_bf16
    b = _reference()
    a = b.copy()
    a[-1, :] = b[-2, :]
    assert relerr(a, b) < TOL["bf16"]                                   # the norm lets it through
    r, i = elementwise_excess(a, b, TOL["bf16"])
    assert r > 10.0 and i // b.shape[1] == b.shape[0] - 1               # ... this does not, and names the row
    w = Worst(TOL["bf16"])
    w.add("conv", a, b)
    assert not w.ok() and "conv[" in w.elem_at
    # the same through the result structure the tests assert on
    for dtype in ("f32", "bf16"):
        m = Modes(dtype, ("fwd",))
        m.add("fwd", "conv", a, b, b)
        ok, text = layerwise_ok(m.result(), dtype)
        assert not ok and "FAILS" in text
        m = Modes(dtype, ("fwd",))
        m.add("fwd", "conv", round_bf16(b) if dtype == "bf16" else b, b, b)     # what a correct kernel stores
        assert layerwise_ok(m.result(), dtype)[0]


def test_rounding_noise_of_the_storage_type_passes_element_wise():
    """bf16 rounding of every element (2^-9 relative at most) is far inside the element-wise bar; a float32-sized
    perturbation far inside the float32 one."""
    from oracle.oracle import round_bf16
    b = _reference(rows=4096)
    assert elementwise_excess(round_bf16(b), b, TOL["bf16"])[0] < 0.2
    assert elementwise_excess(b.astype(np.float32), b, TOL["f32"])[0] < 0.01
    # one element off by 5 % of the tensor's rms, where the reference is ~0: outside
    a = b.copy()
    k = int(np.argmin(np.abs(b)))
    a.flat[k] += 0.05 * np.sqrt(np.mean(b * b))
    r, i = elementwise_excess(a, b, TOL["bf16"])
    assert r > 1.0 and i == k


def test_a_transposed_tile_and_a_dropped_column_fail():
    b = _reference(rows=4096, cols=128, seed=3)
    a = b.copy()
    a[64:96, 32:64] = b[64:96, 32:64].T.copy()                          # one 32x32 tile stored transposed
    assert relerr(a, b) < TOL["bf16"] * 8 and elementwise_excess(a, b, TOL["bf16"])[0] > 10.0
    a = b.copy()
    a[:, -1] = 0.0                                                      # the last column never written
    assert elementwise_excess(a, b, TOL["bf16"])[0] > 10.0


def test_per_tensor_element_wise_holds_zero_tensors_against_the_whole_vector():
    """A parameter tensor whose reference gradient is exactly zero (nothing reaches it) is held against the rms of
    the whole gradient vector, not against zero."""
    rng = np.random.default_rng(1)
    g = rng.standard_normal(300)
    g[100:200] = 0.0
    table = [("a", 0, 100, 0), ("zero", 100, 100, 0), ("c", 200, 100, 0)]
    noisy = g + 1e-9 * rng.standard_normal(300)
    assert per_tensor_elementwise(table, noisy, g, TOL["f32"])[0] < 1.0
    wrong = g.copy()
    wrong[150] = 1.0
    r, where = per_tensor_elementwise(table, wrong, g, TOL["f32"])
    assert r > 1.0 and where.startswith("zero[")
