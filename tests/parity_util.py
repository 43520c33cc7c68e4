"""Helpers for the GPU parity tests: run the HIP path and the oracle on the
same seeded inputs and report norm-wise relative errors per parameter tensor.
"""
import numpy as np

import synth_inputs
from oracle import oracle as O

TOL = {"f32": 1e-4, "bf16": 2e-2}     # the bar stated for this build: fp32 1e-4, bf16 2e-2 (norm-wise)


def relerr(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


def per_tensor_relerr(table, a, b):
    """max over tensors of ||a_t - b_t|| / ||b_t||, and the whole-vector error.
    Tensors whose reference norm is below 1e-12 of the whole vector's are
    compared against the whole-vector norm instead (they are numerically zero)."""
    whole = max(np.linalg.norm(np.asarray(b, dtype=np.float64)), 1e-30)
    worst, worst_name = 0.0, ""
    for name, off, size, _ in table:
        at = np.asarray(a[off:off + size], dtype=np.float64)
        bt = np.asarray(b[off:off + size], dtype=np.float64)
        nb = np.linalg.norm(bt)
        e = np.linalg.norm(at - bt) / (nb if nb > 1e-12 * whole else whole)
        if e > worst:
            worst, worst_name = float(e), name
    return worst, worst_name, relerr(a, b)


def oracle_kwargs(model, H=0, W=0, C=0, classes=0, arch=()):
    """Translate the library's geometry overrides into the oracle's builder arguments."""
    kw = {}
    if H: kw["H"] = H
    if W: kw["W"] = W
    if C: kw["C"] = C
    if classes: kw["classes"] = classes
    arch = list(arch)
    if model == "mlp" and arch:
        kw["hidden"] = tuple(arch[:2])
    elif model == "resnet20" and arch:
        w0, stages, blocks = arch[:3]
        kw["widths"] = tuple(w0 << s for s in range(stages))
        kw["blocks"] = blocks
    elif model == "resnet50" and arch:
        kw["base"] = arch[0]
        kw["blocks"] = tuple(b for b in arch[1:5] if b > 0)
    elif model == "vgg16" and arch:
        kw["base"], kw["fc"] = arch[0], arch[1]
    return kw


DEFAULT_HWC = {"mlp": (1, 1, 784, 10), "resnet20": (32, 32, 3, 10), "resnet50": (224, 224, 3, 1000),
               "vgg16": (224, 224, 3, 1000)}


def run_parity(model, dtype, N, B, schedule, seed=0, data_seed=1, lr=0.1, momentum=0.9, wd=5e-4,
               H=0, W=0, C=0, classes=0, arch=(), emulate=None, check_every_step=True, verbose=True):
    """schedule: list of p, one per step.  Returns dict of worst errors."""
    import torch
    import paper_1909_11985_amd as E
    from paper_1909_11985_amd.binding import make_config

    dH, dW, dC, dK = DEFAULT_HWC[model]
    hh, ww, cc, kk = H or dH, W or dW, C or dC, classes or dK
    x, y = synth_inputs.dataset(data_seed, N, hh, ww, cc, kk)
    p_max = max(schedule)
    cfg = make_config(model, dtype=dtype, N=N, B=B, p_max=p_max, max_shard=B // min(schedule), lr=lr,
                      momentum=momentum, wd=wd, H=H, W=W, C_=C, classes=classes, arch=arch)
    job = E.Job(cfg, seed)
    job.bind_dataset(torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda())
    if emulate is None:
        emulate = dtype == "bf16"
    orc = O.Oracle(model, seed, N, B, lr=lr, momentum=momentum, wd=wd, emulate_bf16=emulate,
                   graph_kwargs=oracle_kwargs(model, H, W, C, classes, arch), dtype_code=E.DTYPES[dtype])
    table = E.edl_tensor_table(cfg)
    assert [(n, o, int(np.prod(s)), f) for n, o, s, f in orc.graph.tensors] == table
    w0 = job.params()
    assert relerr(w0, orc.w) < 3e-7, "initial models differ"
    res = dict(grad=0.0, grad_whole=0.0, param=0.0, param_whole=0.0, loss=0.0, momentum=0.0, running=0.0)
    for t, p in enumerate(schedule):
        idx, off = job.shard(B, p, *job.progress()[1:])
        io, oo = O.shard(seed, N, B, p, orc.epoch, orc.step_in_epoch)
        assert np.array_equal(idx, io) and np.array_equal(off, oo), "shard assignment differs"
        loss = job.step(p, idx, off)
        lo = orc.step(p, x, y)
        last = t == len(schedule) - 1
        if check_every_step or last:
            for k in range(p):
                e, name, whole = per_tensor_relerr(table, job.grad(k), orc.last_grads[k])
                res["grad"] = max(res["grad"], e)
                res["grad_whole"] = max(res["grad_whole"], whole)
                if verbose:
                    print("  step %d p=%d shard %d: grad worst %.3e (%s) whole %.3e" % (t, p, k, e, name, whole), flush=True)
            e, name, whole = per_tensor_relerr(table, job.params(), orc.w)
            res["param"] = max(res["param"], e)
            res["param_whole"] = max(res["param_whole"], whole)
            res["momentum"] = max(res["momentum"], relerr(job.momentum(), orc.v))
            if orc.graph.R:
                res["running"] = max(res["running"], relerr(job.running(), orc.running))
            if verbose:
                print("  step %d: loss gpu %.6f oracle %.6f | param worst %.3e (%s) whole %.3e" %
                      (t, loss, lo, e, name, whole), flush=True)
        res["loss"] = max(res["loss"], abs(loss - lo) / max(abs(lo), 1e-30))
        assert np.isfinite(loss)
    res["job"], res["oracle"], res["table"] = job, orc, table
    return res
