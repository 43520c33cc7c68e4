"""The entry point that allocates nothing (edl_step_static_scratch): the kernels' scratch lives in the library's
static per-GPU buffer instead of the caller's arena.  Its results must be edl_step's bit for bit, on two calls in a
row (the second with smaller shards, then on a smaller model), and jobs whose kernels need more scratch than the
buffer holds are refused.  Needs an MI355X: run with -m gpu."""
import numpy as np
import pytest

import synth_inputs

pytestmark = pytest.mark.gpu


def _twin_jobs(model, dtype, N, B, p_max, geom, seed=5, lr=0.05):
    import torch
    import paper_1909_11985_amd as E
    from paper_1909_11985_amd.binding import make_config
    assert torch.cuda.is_available(), "these tests need the GPU"
    x, y = synth_inputs.dataset(2, N, geom["H"], geom["W"], geom["C_"], geom["classes"])
    dx, dy = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()
    jobs = []
    for _ in range(2):
        cfg = make_config(model, dtype=dtype, N=N, B=B, p_max=p_max, max_shard=B, lr=lr, **geom)
        job = E.Job(cfg, seed)
        job.bind_dataset(dx, dy)
        jobs.append(job)
    return jobs


def _same_state(a, b, p):
    assert np.array_equal(a.params(), b.params()) and np.array_equal(a.momentum(), b.momentum())
    assert np.array_equal(a.running(), b.running())
    for k in range(p):
        assert np.array_equal(a.grad(k), b.grad(k)), k
    assert a.progress() == b.progress()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_static_scratch_step_equals_the_arena_step_on_two_calls_in_a_row(dtype):
    """ResNet-20 at the shapes of the second configuration (32x32 images, aggregate batch 128): a step at p = 2
    (shards of 64), then one at p = 8 (shards of 16: every partial-sum piece is used at a smaller extent, over what
    the first call left in the buffer), then an unequal cut; each against edl_step on a twin job."""
    geom = dict(H=32, W=32, C_=3, classes=10)
    ref, sta = _twin_jobs("resnet20", dtype, 512, 128, 8, geom)
    for p in (2, 8):
        la, lb = ref.step(p), sta.step_static_scratch(p)
        assert la == lb
        _same_state(ref, sta, p)
    idx, _ = ref.shard(128, 1, *ref.progress()[1:])
    off = np.array([0, 50, 50, 128], dtype=np.int64)
    assert ref.step(3, idx, off) == sta.step_static_scratch(3, idx, off)
    _same_state(ref, sta, 3)
    # a smaller model straight after, on the same buffer
    geom2 = dict(H=1, W=1, C_=24, classes=5, arch=(20, 12))
    ref2, sta2 = _twin_jobs("mlp", dtype, 96, 24, 4, geom2)
    for p in (1, 4):
        assert ref2.step(p) == sta2.step_static_scratch(p)
        _same_state(ref2, sta2, p)
    # and the first pair again: the buffer now holds the small model's leftovers
    assert ref.step(4) == sta.step_static_scratch(4)
    _same_state(ref, sta, 4)


def test_static_scratch_step_refuses_what_does_not_fit():
    """A 16384-wide layer needs 128 MiB of column-sum partials alone: beyond the 64 MiB buffer.  The call says so
    and leaves the job untouched; edl_step on the same job works."""
    import paper_1909_11985_amd as E
    geom = dict(H=1, W=1, C_=64, classes=8, arch=(16384, 32))
    ref, sta = _twin_jobs("mlp", "f32", 32, 16, 2, geom)
    w0 = sta.params()
    with pytest.raises(E.EdlError) as ei:
        sta.step_static_scratch(2)
    assert ei.value.code == -3 and "static buffer" in str(ei.value)
    assert sta.progress() == (0, 0, 0) and np.array_equal(sta.params(), w0)
    assert sta.step(2) == ref.step(2)
    _same_state(ref, sta, 2)
