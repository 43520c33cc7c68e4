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
        if len(arch) >= 7 and arch[2] > 0:
            kw["groups"] = tuple(arch[2:7])
    elif model == "alexnet" and arch:
        kw["base"], kw["fc"] = arch[0], arch[1]
    return kw


DEFAULT_HWC = {"mlp": (1, 1, 784, 10), "resnet20": (32, 32, 3, 10), "resnet50": (224, 224, 3, 1000),
               "vgg16": (224, 224, 3, 1000), "alexnet": (224, 224, 3, 1000)}


def run_parity(model, dtype, N, B, schedule, seed=0, data_seed=1, lr=0.1, momentum=0.9, wd=5e-4,
               H=0, W=0, C=0, classes=0, arch=(), emulate=None, check_every_step=True, verbose=True,
               optimizer="momentum", beta2=0.999, eps=1e-8):
    """schedule: list of p, one per step.  Returns dict of worst errors."""
    import torch
    import paper_1909_11985_amd as E
    from paper_1909_11985_amd.binding import make_config

    dH, dW, dC, dK = DEFAULT_HWC[model]
    hh, ww, cc, kk = H or dH, W or dW, C or dC, classes or dK
    x, y = synth_inputs.dataset(data_seed, N, hh, ww, cc, kk)
    p_max = max(schedule)
    cfg = make_config(model, dtype=dtype, N=N, B=B, p_max=p_max, max_shard=B // min(schedule), lr=lr,
                      momentum=momentum, wd=wd, H=H, W=W, C_=C, classes=classes, arch=arch,
                      optimizer=optimizer, beta2=beta2, eps=eps)
    job = E.Job(cfg, seed)
    job.bind_dataset(torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda())
    if emulate is None:
        emulate = dtype == "bf16"
    orc = O.Oracle(model, seed, N, B, lr=lr, momentum=momentum, wd=wd, emulate_bf16=emulate,
                   graph_kwargs=oracle_kwargs(model, H, W, C, classes, arch), dtype_code=E.DTYPES[dtype],
                   optimizer=optimizer, beta2=beta2, eps=eps)
    table = E.edl_tensor_table(cfg)
    assert [(n, o, int(np.prod(s)), f) for n, o, s, f in orc.graph.tensors] == table
    w0 = job.params()
    assert relerr(w0, orc.w) < 3e-7, "initial models differ"
    res = dict(grad=0.0, grad_whole=0.0, param=0.0, param_whole=0.0, loss=0.0, momentum=0.0, second=0.0, running=0.0)
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
            if optimizer == "adam":
                res["second"] = max(res["second"], relerr(job.second_moment(), orc.s))
            if orc.graph.R:
                res["running"] = max(res["running"], relerr(job.running(), orc.running))
            if verbose:
                print("  step %d: loss gpu %.6f oracle %.6f | param worst %.3e (%s) whole %.3e" %
                      (t, loss, lo, e, name, whole), flush=True)
        elif verbose:
            print("  step %d p=%d: loss gpu %.6f oracle %.6f" % (t, p, loss, lo), flush=True)
        res["loss"] = max(res["loss"], abs(loss - lo) / max(abs(lo), 1e-30))
        res.setdefault("loss_steps", []).append(abs(loss - lo) / max(abs(lo), 1e-30))
        assert np.isfinite(loss)
    res["job"], res["oracle"], res["table"] = job, orc, table
    return res


def forced_parity(model, dtype, n, N=None, seed=0, data_seed=1, H=0, W=0, C=0, classes=0, arch=(), emulate=None,
                  perturb=0.05, verbose=True):
    """One worker's whole backward pass with the decisions pinned: every layer's
    forward is run on the oracle's inputs (which also refreshes the batch
    statistics and arg-max positions the layer keeps), its output is then
    replaced by the oracle's, and finally the HIP backward runs through the
    whole layer list in one go.  Its flat gradient is compared with the oracle's.
    Returns dict(fwd=worst layer-output error, loss=..., grad=worst per-tensor, grad_whole=...)."""
    import torch
    import paper_1909_11985_amd as E
    from paper_1909_11985_amd.binding import make_config

    N = N or n
    dH, dW, dC, dK = DEFAULT_HWC[model]
    hh, ww, cc, kk = H or dH, W or dW, C or dC, classes or dK
    x, y = synth_inputs.dataset(data_seed, N, hh, ww, cc, kk)
    cfg = make_config(model, dtype=dtype, N=N, B=n, p_max=1, max_shard=n, H=H, W=W, C_=C, classes=classes, arch=arch)
    job = E.Job(cfg, seed)
    job.bind_dataset(torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda())
    if emulate is None:
        emulate = dtype == "bf16"
    orc = O.Oracle(model, seed, N, n, emulate_bf16=emulate, graph_kwargs=oracle_kwargs(model, H, W, C, classes, arch))
    table = E.edl_tensor_table(cfg)
    if perturb:
        rng = np.random.default_rng(seed + 100)
        orc.w = (orc.w + perturb * rng.standard_normal(orc.w.size) * (np.abs(orc.w) + 0.1)).astype(np.float32).astype(np.float64)
        job.set_params(orc.w)
    idx = np.arange(n, dtype=np.int64)
    loss_o, G = orc.forward_backward(x[idx].astype(np.float64), y[idx])
    job.debug_forward(idx)
    tensors = job.debug_tensors()

    def tid(name):
        return 0 if name == "x" else int(name[1:])

    def shaped(name):
        th, tw, tc, _ = tensors[tid(name)]
        return orc.last_act[name].reshape(n, th, tw, tc)

    ops = [op for op in orc.graph.ops if op["kind"] != "flatten"]
    fwd, fwd_name, loss_g = 0.0, "", None
    for gi, op in enumerate(ops):
        if tid(op["x"]) != 0:                    # the input batch itself was gathered by debug_forward
            job.debug_set(tid(op["x"]), shaped(op["x"]))
        job.debug_forward_op(gi, n)
        if op["kind"] == "loss":
            loss_g = float(job.losses(1)[0])
            continue
        e = relerr(job.debug_get(tid(op["y"]), n), shaped(op["y"]))
        if e > fwd:
            fwd, fwd_name = e, op.get("name", op["kind"])
        job.debug_set(tid(op["y"]), shaped(op["y"]))
    job.debug_backward(n, 0)
    g = job.grad(0)
    worst, worst_name, whole = per_tensor_relerr(table, g, G)
    res = dict(fwd=fwd, fwd_name=fwd_name, loss=abs(loss_g - loss_o) / abs(loss_o), grad=worst, grad_name=worst_name,
               grad_whole=whole)
    if verbose:
        print("  %s %s n=%d: layer outputs worst %.3e (%s) loss %.3e | pinned backward grad worst %.3e (%s) whole %.3e"
              % (model, dtype, n, fwd, fwd_name, res["loss"], worst, worst_name, whole), flush=True)
    job.shutdown()
    return res


def layerwise_parity(model, dtype, n, N=None, seed=0, data_seed=1, H=0, W=0, C=0, classes=0, arch=(), emulate=None,
                     perturb=0.05, verbose=True):
    """Every layer of the model on its own, at the shapes it has inside the
    network: the layer's inputs (and, for the backward, its output and the
    gradient of its output) are the oracle's tensors written into the HIP
    buffers, so each HIP kernel is compared with the oracle's layer on equal
    inputs and no error of an earlier layer is carried along.
    Returns dict(fwd=worst output error, dx=worst input-gradient error, dw=worst parameter-gradient error)."""
    import torch
    import paper_1909_11985_amd as E
    from paper_1909_11985_amd.binding import make_config

    N = N or n
    dH, dW, dC, dK = DEFAULT_HWC[model]
    hh, ww, cc, kk = H or dH, W or dW, C or dC, classes or dK
    x, y = synth_inputs.dataset(data_seed, N, hh, ww, cc, kk)
    cfg = make_config(model, dtype=dtype, N=N, B=n, p_max=1, max_shard=n, H=H, W=W, C_=C, classes=classes, arch=arch)
    job = E.Job(cfg, seed)
    job.bind_dataset(torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda())
    if emulate is None:
        emulate = dtype == "bf16"
    orc = O.Oracle(model, seed, N, n, emulate_bf16=emulate, graph_kwargs=oracle_kwargs(model, H, W, C, classes, arch))
    if perturb:
        rng = np.random.default_rng(seed + 100)
        orc.w = (orc.w + perturb * rng.standard_normal(orc.w.size) * (np.abs(orc.w) + 0.1)).astype(np.float32).astype(np.float64)
        job.set_params(orc.w)
    idx = np.arange(n, dtype=np.int64)
    loss_o, G = orc.forward_backward(x[idx].astype(np.float64), y[idx])
    job.debug_forward(idx)                     # gathers the input batch and the labels
    tensors = job.debug_tensors()

    def tid(name):
        return 0 if name == "x" else int(name[1:])

    def shaped(name, a):
        th, tw, tc, _ = tensors[tid(name)]
        return np.asarray(a).reshape(n, th, tw, tc)

    ops = [(oi, op) for oi, op in enumerate(orc.graph.ops) if op["kind"] != "flatten"]
    assert len(ops) == job.debug_op_count()
    res = dict(fwd=0.0, dx=0.0, dw=0.0, worst="")

    def note(key, e, what):
        if e > res[key]:
            res[key] = e
            res["worst_" + key] = what

    for gi, (oi, op) in enumerate(ops):
        kind = op["kind"]
        label = op.get("name", kind)
        if tid(op["x"]) != 0:                    # the input batch itself was gathered by debug_forward
            job.debug_set(tid(op["x"]), shaped(op["x"], orc.last_act[op["x"]]))
        if kind == "bn" and op["res"] is not None:
            job.debug_set(tid(op["res"]), shaped(op["res"], orc.last_act[op["res"]]))
        job.debug_forward_op(gi, n)
        if kind == "loss":
            note("fwd", abs(float(job.losses(1)[0]) - loss_o) / abs(loss_o), "loss")
            dz = job.debug_get(tid(op["x"]), n, which=1)
            note("dx", relerr(dz, shaped(op["x"], orc.last_dx[oi][op["x"]])), "loss")
            continue
        out = job.debug_get(tid(op["y"]), n)
        e_f = relerr(out, shaped(op["y"], orc.last_act[op["y"]]))
        note("fwd", e_f, label)
        # backward: decisions (ReLU sign) from the oracle's output, upstream gradient from the oracle
        job.debug_set(tid(op["y"]), shaped(op["y"], orc.last_act[op["y"]]))
        job.debug_set(tid(op["y"]), shaped(op["y"], orc.last_dy[oi]), which=1)
        job.debug_backward_op(gi, n, 0)
        e_x = 0.0
        for name, contrib in orc.last_dx.get(oi, {}).items():
            if tid(name) == 0 or tensors[tid(name)][3] == 0:
                continue                      # the input batch has no gradient buffer
            got = job.debug_get(tid(name), n, which=1)
            e_x = max(e_x, relerr(got, shaped(name, contrib)))
        note("dx", e_x, label)
        e_w = 0.0
        if kind == "conv":
            wsize = op["K"] * op["R"] * op["S"] * orc.last_act[op["x"]].shape[-1]
            e_w = relerr(job.grad_slice(0, op["w_off"], wsize), G[op["w_off"]:op["w_off"] + wsize])
            if op["b_off"] is not None:
                e_w = max(e_w, relerr(job.grad_slice(0, op["b_off"], op["K"]), G[op["b_off"]:op["b_off"] + op["K"]]))
        elif kind == "bn":
            cch = op["C"]
            e_w = max(relerr(job.grad_slice(0, op["g_off"], cch), G[op["g_off"]:op["g_off"] + cch]),
                      relerr(job.grad_slice(0, op["b_off"], cch), G[op["b_off"]:op["b_off"] + cch]))
        note("dw", e_w, label)
        if verbose:
            print("    %-16s %-8s fwd %.2e  dx %.2e  dw %.2e" % (label, kind, e_f, e_x, e_w), flush=True)
    if verbose:
        print("  %s %s n=%d layerwise: fwd %.3e (%s) dx %.3e (%s) dw %.3e (%s)" %
              (model, dtype, n, res["fwd"], res.get("worst_fwd"), res["dx"], res.get("worst_dx"), res["dw"],
               res.get("worst_dw")), flush=True)
    job.shutdown()
    return res


def conv_bn_pair_parity(model, dtype, n, N=None, seed=0, data_seed=1, H=0, W=0, C=0, classes=0, arch=(), emulate=None,
                        perturb=0.05):
    """Every convolution that a batch norm follows, run together with that batch
    norm the way a step runs them (the batch statistics come out of the
    convolution's own pass over its output), on the oracle's input of the
    convolution.  Returns the worst error of the batch norms' outputs and the
    number of pairs."""
    import torch
    import paper_1909_11985_amd as E
    from paper_1909_11985_amd.binding import make_config

    N = N or n
    dH, dW, dC, dK = DEFAULT_HWC[model]
    hh, ww, cc, kk = H or dH, W or dW, C or dC, classes or dK
    x, y = synth_inputs.dataset(data_seed, N, hh, ww, cc, kk)
    cfg = make_config(model, dtype=dtype, N=N, B=n, p_max=1, max_shard=n, H=H, W=W, C_=C, classes=classes, arch=arch)
    job = E.Job(cfg, seed)
    job.bind_dataset(torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda())
    if emulate is None:
        emulate = dtype == "bf16"
    orc = O.Oracle(model, seed, N, n, emulate_bf16=emulate, graph_kwargs=oracle_kwargs(model, H, W, C, classes, arch))
    if perturb:
        rng = np.random.default_rng(seed + 100)
        orc.w = (orc.w + perturb * rng.standard_normal(orc.w.size) * (np.abs(orc.w) + 0.1)).astype(np.float32).astype(np.float64)
        job.set_params(orc.w)
    idx = np.arange(n, dtype=np.int64)
    orc.forward_backward(x[idx].astype(np.float64), y[idx])
    job.debug_forward(idx)
    tensors = job.debug_tensors()

    def tid(name):
        return 0 if name == "x" else int(name[1:])

    def shaped(name, a):
        th, tw, tc, _ = tensors[tid(name)]
        return np.asarray(a).reshape(n, th, tw, tc)

    ops = [op for op in orc.graph.ops if op["kind"] != "flatten"]
    worst, pairs, where = 0.0, 0, ""
    for gi in range(len(ops) - 1):
        conv, bn = ops[gi], ops[gi + 1]
        if conv["kind"] != "conv" or bn["kind"] != "bn" or bn["x"] != conv["y"]:
            continue
        if tid(conv["x"]) != 0:
            job.debug_set(tid(conv["x"]), shaped(conv["x"], orc.last_act[conv["x"]]))
        if bn["res"] is not None:
            job.debug_set(tid(bn["res"]), shaped(bn["res"], orc.last_act[bn["res"]]))
        job.debug_forward_range(gi, gi + 2, n)
        e = relerr(job.debug_get(tid(bn["y"]), n), shaped(bn["y"], orc.last_act[bn["y"]]))
        pairs += 1
        if e > worst:
            worst, where = e, bn.get("name", "bn")
    job.shutdown()
    return dict(fwd=worst, pairs=pairs, worst=where)


def relu_producer_pair_parity(model, dtype, n, N=None, seed=0, data_seed=1, H=0, W=0, C=0, classes=0, arch=(), emulate=None,
                              perturb=0.05):
    """Every convolution whose input comes from the layer listed just before it, ending in a ReLU and read by
    nobody else (a batch norm or a convolution with bias and ReLU), run backward together with that layer the
    way a step runs them: the convolution's input-gradient pass stores the gradient masked and leaves the
    producer's column sums.  Inputs are the oracle's; compared are the producer's input gradient and parameter
    gradients.  Returns the worst errors and the number of pairs."""
    import torch
    import paper_1909_11985_amd as E
    from paper_1909_11985_amd.binding import make_config

    N = N or n
    dH, dW, dC, dK = DEFAULT_HWC[model]
    hh, ww, cc, kk = H or dH, W or dW, C or dC, classes or dK
    x, y = synth_inputs.dataset(data_seed, N, hh, ww, cc, kk)
    cfg = make_config(model, dtype=dtype, N=N, B=n, p_max=1, max_shard=n, H=H, W=W, C_=C, classes=classes, arch=arch)
    job = E.Job(cfg, seed)
    job.bind_dataset(torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda())
    if emulate is None:
        emulate = dtype == "bf16"
    orc = O.Oracle(model, seed, N, n, emulate_bf16=emulate, graph_kwargs=oracle_kwargs(model, H, W, C, classes, arch))
    if perturb:
        rng = np.random.default_rng(seed + 100)
        orc.w = (orc.w + perturb * rng.standard_normal(orc.w.size) * (np.abs(orc.w) + 0.1)).astype(np.float32).astype(np.float64)
        job.set_params(orc.w)
    idx = np.arange(n, dtype=np.int64)
    _, G = orc.forward_backward(x[idx].astype(np.float64), y[idx])
    job.debug_forward(idx)
    tensors = job.debug_tensors()

    def tid(name):
        return 0 if name == "x" else int(name[1:])

    def shaped(name, a):
        th, tw, tc, _ = tensors[tid(name)]
        return np.asarray(a).reshape(n, th, tw, tc)

    ops = [(oi, op) for oi, op in enumerate(orc.graph.ops) if op["kind"] != "flatten"]
    readers = {}
    for _, op in ops:
        readers[op["x"]] = readers.get(op["x"], 0) + 1
        if op["kind"] == "bn" and op["res"] is not None:
            readers[op["res"]] = readers.get(op["res"], 0) + 1
    res = dict(dx=0.0, dw=0.0, pairs=0, worst="")
    for gi in range(1, len(ops)):
        (poi, prod), (coi, cons) = ops[gi - 1], ops[gi]
        if cons["kind"] != "conv" or prod["kind"] not in ("bn", "conv") or not prod.get("relu"):
            continue
        if prod["y"] != cons["x"] or readers.get(cons["x"], 0) != 1 or tid(prod["x"]) == 0:
            continue
        # the producer's forward on the oracle's inputs (refreshes the statistics it keeps), then the oracle's output
        job.debug_set(tid(prod["x"]), shaped(prod["x"], orc.last_act[prod["x"]]))
        if prod["kind"] == "bn" and prod["res"] is not None:
            job.debug_set(tid(prod["res"]), shaped(prod["res"], orc.last_act[prod["res"]]))
        job.debug_forward_op(gi - 1, n)
        job.debug_set(tid(prod["y"]), shaped(prod["y"], orc.last_act[prod["y"]]))
        job.debug_set(tid(cons["y"]), shaped(cons["y"], orc.last_act[cons["y"]]))
        job.debug_set(tid(cons["y"]), shaped(cons["y"], orc.last_dy[coi]), which=1)
        job.debug_backward_range(gi - 1, gi + 1, n, 0)
        e_x = 0.0
        for name, contrib in orc.last_dx.get(poi, {}).items():
            if tid(name) == 0 or tensors[tid(name)][3] == 0:
                continue
            e_x = max(e_x, relerr(job.debug_get(tid(name), n, which=1), shaped(name, contrib)))
        if prod["kind"] == "bn":
            cch = prod["C"]
            e_w = max(relerr(job.grad_slice(0, prod["g_off"], cch), G[prod["g_off"]:prod["g_off"] + cch]),
                      relerr(job.grad_slice(0, prod["b_off"], cch), G[prod["b_off"]:prod["b_off"] + cch]))
        else:
            wsize = prod["K"] * prod["R"] * prod["S"] * orc.last_act[prod["x"]].shape[-1]
            e_w = relerr(job.grad_slice(0, prod["w_off"], wsize), G[prod["w_off"]:prod["w_off"] + wsize])
            if prod["b_off"] is not None:
                e_w = max(e_w, relerr(job.grad_slice(0, prod["b_off"], prod["K"]), G[prod["b_off"]:prod["b_off"] + prod["K"]]))
        res["pairs"] += 1
        if e_x > res["dx"] or e_w > res["dw"]:
            res["worst"] = prod.get("name", prod["kind"])
        res["dx"], res["dw"] = max(res["dx"], e_x), max(res["dw"], e_w)
    job.shutdown()
    return res
