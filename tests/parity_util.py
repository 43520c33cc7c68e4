"""Helpers for the GPU parity tests: run the HIP path and the oracle on the same seeded inputs and compare.

Two criteria per compared tensor, both against the stated bar (float32 1e-4, bf16 2e-2):
  norm-wise      ||a - b|| / ||b||  <  tol
  element-wise   max |a - b|  <=  tol * (|b| + rms(b))      (reported as the worst ratio, with its index)
The element-wise one is what catches a wrong ragged tile or last row that the norm lets through.

bf16 jobs are compared twice: with the plain float64 oracle (mode "plain": the stated bar) and with the
oracle that rounds to bf16 where the HIP path stores bf16 (mode "emulated": a tight regression bound,
since the two then differ by summation order only).  float32 jobs have one mode and carry the tight
bound on it.
"""
import numpy as np

import synth_inputs
from oracle import oracle as O

TOL = {"f32": 1e-4, "bf16": 2e-2}       # the bar stated for this build (norm-wise and element-wise)
TIGHT = {"f32": 5e-5, "bf16": 5e-4}     # regression bounds of the per-layer comparisons (measured: 5e-6 / 7e-5)


def relerr(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


def elementwise_excess(a, b, tol, floor=0.0):
    """max over elements of |a-b| / (tol * (|b| + max(rms(b), floor))) and the flat index where it is
    reached.  <= 1 passes.  `floor` stands in for rms(b) where the reference tensor is numerically zero."""
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    if b.size == 0:
        return 0.0, -1
    rms = max(float(np.sqrt(np.mean(b * b))), floor, 1e-300)
    ratio = np.abs(a - b) / (tol * (np.abs(b) + rms))
    i = int(np.argmax(ratio))
    return float(ratio[i]), i


class Worst:
    """Collects comparisons of one kind and keeps the worst of each criterion and where it was."""

    def __init__(self, tol):
        self.tol = tol
        self.norm, self.norm_at = 0.0, ""
        self.elem, self.elem_at = 0.0, ""

    def add(self, what, a, b, floor=0.0):
        e = relerr(a, b)
        r, i = elementwise_excess(a, b, self.tol, floor)
        if e > self.norm:
            self.norm, self.norm_at = e, what
        if r > self.elem:
            self.elem, self.elem_at = r, "%s[%d]" % (what, i)
        return e

    def ok(self, norm_bound=None):
        return self.norm < (self.tol if norm_bound is None else norm_bound) and self.elem <= 1.0

    def __repr__(self):
        return "norm %.3e (%s) elem %.3f (%s)" % (self.norm, self.norm_at, self.elem, self.elem_at)


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


def per_tensor_elementwise(table, a, b, tol):
    """Worst element-wise ratio over the parameter tensors of a flat vector (a tensor whose reference is
    numerically zero is held against the whole vector's rms), and where."""
    b = np.asarray(b, dtype=np.float64)
    whole_rms = float(np.sqrt(np.mean(b * b))) if b.size else 0.0
    worst, where = 0.0, ""
    for name, off, size, _ in table:
        bt = b[off:off + size]
        zero = bt.size == 0 or float(np.sqrt(np.mean(bt * bt))) <= 1e-12 * whole_rms
        r, i = elementwise_excess(a[off:off + size], bt, tol, floor=whole_rms if zero else 0.0)
        if r > worst:
            worst, where = r, "%s[%d]" % (name, i)
    return worst, where


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


def modes_of(dtype):
    """(label, oracle rounds like the HIP path's storage?) for each comparison a job of this dtype gets."""
    return [("plain", False), ("emulated", True)] if dtype == "bf16" else [("plain", False)]


def tid(name):
    """Oracle tensor name -> library tensor number."""
    return 0 if name == "x" else int(name[1:])


class Case:
    """One job on the GPU plus what the helpers need to build oracles for it: the data set, the geometry,
    the parameter table and the activation-tensor shapes."""

    def __init__(self, model, dtype, n, N=None, B=None, seed=0, data_seed=1, H=0, W=0, C=0, classes=0, arch=(),
                 perturb=0.0, p_max=1, lr=0.1, momentum=0.9, wd=5e-4, optimizer="momentum", beta2=0.999, eps=1e-8,
                 side_streams="library"):
        import torch
        import paper_1909_11985_amd as E
        from paper_1909_11985_amd.binding import make_config
        self.E, self.model, self.dtype, self.n, self.seed = E, model, dtype, n, seed
        self.N, self.B = N or n, B or n
        dH, dW, dC, dK = DEFAULT_HWC[model]
        hh, ww, cc, kk = H or dH, W or dW, C or dC, classes or dK
        self.x, self.y = synth_inputs.dataset(data_seed, self.N, hh, ww, cc, kk)
        self.hyper = dict(lr=lr, momentum=momentum, wd=wd, optimizer=optimizer, beta2=beta2, eps=eps)
        self.cfg = make_config(model, dtype=dtype, N=self.N, B=self.B, p_max=p_max, max_shard=n, H=H, W=W, C_=C,
                               classes=classes, arch=arch, **self.hyper)
        self.job = E.Job(self.cfg, seed, side_streams=side_streams)
        self.job.bind_dataset(torch.from_numpy(self.x).cuda(), torch.from_numpy(self.y).cuda())
        self.gkw = oracle_kwargs(model, H, W, C, classes, arch)
        self.table = E.edl_tensor_table(self.cfg)
        self.tensors = self.job.debug_tensors()
        self.w = None
        if perturb:
            # scales, shifts and biases off their initial 1 / 0 so that every term of every layer is exercised
            w0 = self.job.params().astype(np.float64)
            rng = np.random.default_rng(seed + 100)
            self.w = (w0 + perturb * rng.standard_normal(w0.size) * (np.abs(w0) + 0.1)).astype(np.float32)
            self.job.set_params(self.w)

    def oracle(self, emulate):
        orc = O.Oracle(self.model, self.seed, self.N, self.B, emulate_bf16=emulate, graph_kwargs=self.gkw,
                       dtype_code=self.E.DTYPES[self.dtype], **self.hyper)
        assert [(nm, o, int(np.prod(s)), f) for nm, o, s, f in orc.graph.tensors] == self.table
        if self.w is not None:
            orc.w = self.w.astype(np.float64)
        # a bf16 job's max pools decide on bf16 values: the unrounded computation decides in the same precision
        orc.pool_picks_in_bf16 = self.dtype == "bf16"
        return orc

    def shaped(self, name, a, n=None):
        th, tw, tc, _ = self.tensors[tid(name)]
        return np.asarray(a).reshape(n or self.n, th, tw, tc)

    def storage(self, t):
        return self.tensors[t][3] if self.tensors[t][3] >= 0 else t

    def close(self):
        self.job.shutdown()


# ---------------------------------------------------------------------------------------------------------
# free running: edl_step against oracle.step
# ---------------------------------------------------------------------------------------------------------
def run_parity(model, dtype, N, B, schedule, seed=0, data_seed=1, lr=0.1, momentum=0.9, wd=5e-4,
               H=0, W=0, C=0, classes=0, arch=(), emulate=None, check_every_step=True, verbose=True,
               optimizer="momentum", beta2=0.999, eps=1e-8):
    """schedule: list of p, one per step.  Both sides run freely from the same initial model.
    Returns dict of worst errors."""
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
    res = dict(grad=0.0, grad_whole=0.0, grad_elem=0.0, param=0.0, param_whole=0.0, param_elem=0.0, loss=0.0,
               momentum=0.0, second=0.0, running=0.0)
    for t, p in enumerate(schedule):
        idx, off = job.shard(B, p, *job.progress()[1:])
        io, oo = O.shard(seed, N, B, p, orc.epoch, orc.step_in_epoch)
        assert np.array_equal(idx, io) and np.array_equal(off, oo), "shard assignment differs"
        loss = job.step(p, idx, off)
        lo = orc.step(p, x, y)
        last = t == len(schedule) - 1
        if check_every_step or last:
            for k in range(p):
                gk = job.grad(k)
                e, name, whole = per_tensor_relerr(table, gk, orc.last_grads[k])
                res["grad"] = max(res["grad"], e)
                res["grad_whole"] = max(res["grad_whole"], whole)
                res["grad_elem"] = max(res["grad_elem"], per_tensor_elementwise(table, gk, orc.last_grads[k], TOL[dtype])[0])
                if verbose:
                    print("  step %d p=%d shard %d: grad worst %.3e (%s) whole %.3e" % (t, p, k, e, name, whole), flush=True)
            wj = job.params()
            e, name, whole = per_tensor_relerr(table, wj, orc.w)
            res["param"] = max(res["param"], e)
            res["param_whole"] = max(res["param_whole"], whole)
            res["param_elem"] = max(res["param_elem"], per_tensor_elementwise(table, wj, orc.w, TOL[dtype])[0])
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


# ---------------------------------------------------------------------------------------------------------
# the backward pass with the decisions pinned
# ---------------------------------------------------------------------------------------------------------
def pinned_chain(case, orc, sel, update_running=False, check_fwd=True):
    """One worker's whole backward pass on the samples `sel` with every decision taken from the oracle:
    the oracle's activations are written into the HIP buffers layer by layer (layers that keep something for
    their backward - batch statistics, arg-max positions - run their forward on the oracle's input first),
    then the HIP backward runs through the whole layer list in one go into gradient buffer 0.
    Returns dict(loss_o, loss_g, G = oracle's flat gradient, g = the HIP path's, fwd = Worst of the layer
    outputs if check_fwd).  The job's model, optimizer state, running statistics and progress are untouched."""
    job, n = case.job, len(sel)
    tol = TOL[case.dtype]
    xs, ys = case.x[sel].astype(np.float64), case.y[sel]
    loss_o, G = orc.forward_backward(xs, ys, update_running=update_running)
    job.debug_forward(np.asarray(sel, dtype=np.int64))           # gathers the input batch and the labels
    ops = [op for op in orc.graph.ops if op["kind"] != "flatten"]
    holds = {0}                                                  # storages that hold the oracle's values
    fwd = Worst(tol)
    loss_g = None
    for gi, op in enumerate(ops):
        kind = op["kind"]
        keeps_state = kind in ("bn", "maxpool", "loss")
        if check_fwd or keeps_state:
            for name in [op["x"]] + ([op["res"]] if kind == "bn" and op["res"] is not None else []):
                if case.storage(tid(name)) not in holds:
                    job.debug_set(tid(name), case.shaped(name, orc.last_act[name], n))
                    holds.add(case.storage(tid(name)))
            job.debug_forward_op(gi, n)
        if kind == "loss":
            loss_g = float(job.losses(1)[0])
            continue
        want = case.shaped(op["y"], orc.last_act[op["y"]], n)
        if check_fwd:
            fwd.add(op.get("name", kind), job.debug_get(tid(op["y"]), n), want)
        job.debug_set(tid(op["y"]), want)
        holds.add(case.storage(tid(op["y"])))
    job.debug_backward(n, 0)
    return dict(loss_o=loss_o, loss_g=loss_g, G=G, g=job.grad(0), fwd=fwd)


def forced_parity(model, dtype, n, N=None, seed=0, data_seed=1, H=0, W=0, C=0, classes=0, arch=(), perturb=0.05,
                  verbose=True):
    """pinned_chain on the first n samples, per comparison mode of the dtype.  Returns {mode: dict(fwd, fwd_elem,
    loss, grad = worst per tensor, grad_name, grad_whole, grad_elem)}."""
    case = Case(model, dtype, n, N=N, seed=seed, data_seed=data_seed, H=H, W=W, C=C, classes=classes, arch=arch,
                perturb=perturb)
    out = {}
    sel = np.arange(n, dtype=np.int64)
    for mode, emulate in modes_of(dtype):
        r = pinned_chain(case, case.oracle(emulate), sel)
        worst, worst_name, whole = per_tensor_relerr(case.table, r["g"], r["G"])
        elem, elem_at = per_tensor_elementwise(case.table, r["g"], r["G"], TOL[dtype])
        out[mode] = dict(fwd=r["fwd"].norm, fwd_name=r["fwd"].norm_at, fwd_elem=r["fwd"].elem, fwd_elem_at=r["fwd"].elem_at,
                         loss=abs(r["loss_g"] - r["loss_o"]) / abs(r["loss_o"]), grad=worst, grad_name=worst_name,
                         grad_whole=whole, grad_elem=elem, grad_elem_at=elem_at)
        if verbose:
            print("  %s %s n=%d [%s]: layer outputs %r loss %.3e | pinned backward grad worst %.3e (%s) whole %.3e "
                  "elem %.3f (%s)" % (model, dtype, n, mode, r["fwd"], out[mode]["loss"], worst, worst_name, whole, elem,
                                      elem_at), flush=True)
    case.close()
    return out


# ---------------------------------------------------------------------------------------------------------
# every layer alone
# ---------------------------------------------------------------------------------------------------------
class Modes:
    """The comparisons one HIP result gets.
      plain        the oracle's float64 chain, nothing rounded (bf16 jobs: max pools pick in bf16) - what the
                   stated bar is held against;
      same_inputs  (bf16 jobs) the oracle's float64 layer evaluated on exactly the bf16 tensors the HIP layer was
                   given, nothing rounded inside or after: what is left is the kernel's own arithmetic and the
                   rounding of its output;
      emulated     (bf16 jobs) that reference rounded to bf16 where the HIP path stores bf16: the two then
                   differ by summation order only (tight regression bound)."""

    def __init__(self, dtype, keys):
        self.dtype, self.bf = dtype, dtype == "bf16"
        names = ["plain", "same_inputs", "emulated"] if self.bf else ["plain"]
        self.res = {m: {k: Worst(TOL[dtype]) for k in keys} for m in names}
        self.parts = {m: ([], []) for m in names}          # parameter gradients, concatenated at the end

    def add(self, key, what, got, plain, same=None, stored_bf16=True, floor=0.0):
        e = self.res["plain"][key].add(what, got, plain, floor)
        if self.bf:
            same = plain if same is None else same
            self.res["same_inputs"][key].add(what, got, same, floor)
            self.res["emulated"][key].add(what, got, O.round_bf16(same) if stored_bf16 else same, floor)
        return e

    def add_param_grad(self, what, got, plain, same=None, floor=0.0):
        e = self.add("dw", what, got, plain, same, stored_bf16=False, floor=floor)
        for m in self.res:
            ref = plain if (m == "plain" or same is None) else same
            self.parts[m][0].append(np.asarray(got, dtype=np.float64).ravel())
            self.parts[m][1].append(np.asarray(ref, dtype=np.float64).ravel())
        return e

    def result(self, **extra):
        out = {}
        for m, r in self.res.items():
            d = dict(r)
            if self.parts[m][0]:
                d["dw_whole"] = relerr(np.concatenate(self.parts[m][0]), np.concatenate(self.parts[m][1]))
            d.update(extra)
            out[m] = d
        return out


SAME_INPUTS_BOUND = 4e-3        # bf16 output rounding is 2^-9 per element at most, ~1.1e-3 in the norm


def layerwise_ok(res, dtype):
    """The assertion every layerwise / pair result carries.  Returns (passed, text).
    float32: norm-wise below the tight bound and element-wise within the stated bar, against the plain oracle.
    bf16: against the plain chain norm-wise at the stated bar for outputs and input gradients per tensor and for
    the parameter gradients as one vector (a single batch-norm shift whose terms cancel is not a per-tensor
    statement bf16 inputs can carry; element-wise values are reported); on the same inputs both criteria at the
    stated bar and the norm below the output rounding's size; against the rounded reference the tight bound."""
    ok, lines = True, []
    for mode, r in res.items():
        for key, w in r.items():
            if isinstance(w, Worst):
                if dtype == "f32":
                    bound, elem = TIGHT["f32"], True
                elif mode == "plain":
                    bound, elem = (None if key == "dw" else TOL["bf16"]), False
                elif mode == "same_inputs":
                    bound, elem = SAME_INPUTS_BOUND, True
                else:
                    bound, elem = TIGHT["bf16"], True
                good = (bound is None or w.norm < bound) and (not elem or w.elem <= 1.0)
                note = "reported" if bound is None else "norm bound %.0e%s" % (bound, "" if elem else ", elem reported")
                lines.append("%-11s %-3s: %r (%s)%s" % (mode, key, w, note, "" if good else "  <-- FAILS"))
            elif key == "dw_whole":
                bound = TIGHT["f32"] if dtype == "f32" else {"plain": TOL["bf16"], "same_inputs": SAME_INPUTS_BOUND,
                                                             "emulated": TIGHT["bf16"]}[mode]
                good = w < bound
                lines.append("%-11s dw as one vector: %.3e (bound %.0e)%s" % (mode, w, bound, "" if good else "  <-- FAILS"))
            else:
                continue
            ok = ok and good
    return ok, "\n".join(lines)


def _qin(case, a):
    """A tensor as the HIP path holds it once written into one of its activation / gradient buffers."""
    return O.round_bf16(a) if case.dtype == "bf16" else np.asarray(a, dtype=np.float32).astype(np.float64)


def _conv_weights(case, orc, op, C):
    """The weights a convolution of the HIP path contracts with: the bf16 copies in a bf16 job."""
    w = orc._param(op["w_off"], (op["K"], op["R"], op["S"], C))
    return O.round_bf16(w) if case.dtype == "bf16" else w


def layerwise_parity(model, dtype, n, N=None, seed=0, data_seed=1, H=0, W=0, C=0, classes=0, arch=(), perturb=0.05,
                     verbose=True):
    """Every layer of the model on its own, at the shapes it has inside the network: the layer's inputs (and,
    for the backward, its output and the gradient of its output) are the oracle's tensors written into the HIP
    buffers, so each HIP kernel is compared with the oracle's layer on equal inputs and no error of an earlier
    layer is carried along.  Returns {mode: dict(fwd, dx, dw = Worst of outputs, input gradients, parameter
    gradients; dw_whole)} for the modes of class Modes."""
    case = Case(model, dtype, n, N=N, seed=seed, data_seed=data_seed, H=H, W=W, C=C, classes=classes, arch=arch,
                perturb=perturb)
    job, tensors = case.job, case.tensors
    idx = np.arange(n, dtype=np.int64)
    orc = case.oracle(False)
    xs, ys = case.x[idx].astype(np.float64), case.y[idx]
    loss_o, G = orc.forward_backward(xs, ys)
    g_rms = float(np.sqrt(np.mean(G * G)))
    job.debug_forward(idx)                     # gathers the input batch and the labels
    ops = [(oi, op) for oi, op in enumerate(orc.graph.ops) if op["kind"] != "flatten"]
    assert len(ops) == job.debug_op_count()
    modes = Modes(dtype, ("fwd", "dx", "dw"))
    bf = dtype == "bf16"
    act = orc.last_act
    for gi, (oi, op) in enumerate(ops):
        kind = op["kind"]
        label = op.get("name", kind)
        if tid(op["x"]) != 0:                    # the input batch itself was gathered by debug_forward
            job.debug_set(tid(op["x"]), case.shaped(op["x"], act[op["x"]]))
        has_res = kind == "bn" and op["res"] is not None
        if has_res:
            job.debug_set(tid(op["res"]), case.shaped(op["res"], act[op["res"]]))
        job.debug_forward_op(gi, n)
        # the same layer in float64 on the tensors as the HIP buffers hold them
        x_q = _qin(case, act[op["x"]]) if (bf and op["x"] != orc.graph.logits) else act[op["x"]]   # logits stay float32
        same_y = same_saved = None
        if bf:
            same_y, same_saved = orc.op_forward(oi, x_q, res=_qin(case, act[op["res"]]) if has_res else None,
                                                w=_conv_weights(case, orc, op, x_q.shape[-1]) if kind == "conv" else None,
                                                labels=ys)
        if kind == "loss":
            modes.add("fwd", "loss", [float(job.losses(1)[0])], [loss_o], [same_y] if bf else None, stored_bf16=False)
            dz = job.debug_get(tid(op["x"]), n, which=1)
            same_dz = orc.op_backward(oi, None, x_q, None, same_saved, labels=ys)[0][op["x"]] if bf else None
            modes.add("dx", "loss", dz, case.shaped(op["x"], orc.last_dx[oi][op["x"]]),
                      case.shaped(op["x"], same_dz) if bf else None)
            continue
        logits = op["y"] == orc.graph.logits
        e_f = modes.add("fwd", label, job.debug_get(tid(op["y"]), n), case.shaped(op["y"], act[op["y"]]),
                        case.shaped(op["y"], same_y) if bf else None, stored_bf16=not logits)
        # backward: decisions (ReLU sign) from the oracle's output, upstream gradient from the oracle
        job.debug_set(tid(op["y"]), case.shaped(op["y"], act[op["y"]]))
        job.debug_set(tid(op["y"]), case.shaped(op["y"], orc.last_dy[oi]), which=1)
        job.debug_backward_op(gi, n, 0)
        same_dx, same_dp = {}, {}
        if bf:
            y_q = act[op["y"]] if logits else _qin(case, act[op["y"]])
            same_dx, same_dp, _ = orc.op_backward(oi, _qin(case, orc.last_dy[oi]), x_q, y_q, same_saved, labels=ys)
        e_x = 0.0
        for name, contrib in orc.last_dx.get(oi, {}).items():
            if tid(name) == 0 or tensors[tid(name)][3] == 0:
                continue                      # the input batch has no gradient buffer
            e_x = max(e_x, modes.add("dx", label, job.debug_get(tid(name), n, which=1), case.shaped(name, contrib),
                                     case.shaped(name, same_dx[name]) if bf else None))
        e_w = 0.0
        slices = []
        if kind == "conv":
            slices.append((label + ".w", op["w_off"], op["K"] * op["R"] * op["S"] * act[op["x"]].shape[-1]))
            if op["b_off"] is not None:
                slices.append((label + ".b", op["b_off"], op["K"]))
        elif kind == "bn":
            slices += [(label + ".g", op["g_off"], op["C"]), (label + ".b", op["b_off"], op["C"])]
        for what, off, size in slices:
            e_w = max(e_w, modes.add_param_grad(what, job.grad_slice(0, off, size), G[off:off + size],
                                                same_dp[off] if bf else None, floor=1e-6 * g_rms))
        if verbose:
            print("    %-16s %-8s fwd %.2e  dx %.2e  dw %.2e  (against the plain chain)" % (label, kind, e_f, e_x, e_w),
                  flush=True)
    case.close()
    out = modes.result()
    if verbose:
        print("  %s %s n=%d layerwise:\n%s" % (model, dtype, n, layerwise_ok(out, dtype)[1]), flush=True)
    return out


# ---------------------------------------------------------------------------------------------------------
# layers that hand something to their neighbour inside a step
# ---------------------------------------------------------------------------------------------------------
def conv_bn_pair_parity(model, dtype, n, N=None, seed=0, data_seed=1, H=0, W=0, C=0, classes=0, arch=(), perturb=0.05):
    """Every convolution that a batch norm follows, run together with that batch norm the way a step runs them
    (the batch statistics come out of the convolution's own pass over its output), on the oracle's input of the
    convolution.  Returns {mode: dict(fwd = Worst of the batch norms' outputs, pairs)}."""
    case = Case(model, dtype, n, N=N, seed=seed, data_seed=data_seed, H=H, W=W, C=C, classes=classes, arch=arch,
                perturb=perturb)
    job = case.job
    idx = np.arange(n, dtype=np.int64)
    orc = case.oracle(False)
    orc.forward_backward(case.x[idx].astype(np.float64), case.y[idx])
    act = orc.last_act
    job.debug_forward(idx)
    ops = [(oi, op) for oi, op in enumerate(orc.graph.ops) if op["kind"] != "flatten"]
    modes, pairs, bf = Modes(dtype, ("mid", "fwd")), 0, dtype == "bf16"
    for gi in range(len(ops) - 1):
        (ci, conv), (bi, bn) = ops[gi], ops[gi + 1]
        if conv["kind"] != "conv" or bn["kind"] != "bn" or bn["x"] != conv["y"]:
            continue
        if tid(conv["x"]) != 0:
            job.debug_set(tid(conv["x"]), case.shaped(conv["x"], act[conv["x"]]))
        if bn["res"] is not None:
            job.debug_set(tid(bn["res"]), case.shaped(bn["res"], act[bn["res"]]))
        job.debug_forward_range(gi, gi + 2, n)
        got_mid = job.debug_get(tid(conv["y"]), n)
        same = same_mid = None
        if bf:
            # float64 on the same bf16 input.  The tensor between the two layers is a bf16 activation like any
            # other, and a batch norm turns one last-place difference in it into (|x| / sigma) last places of its
            # output: the batch norm's reference is therefore evaluated on the convolution output the HIP path
            # stored (which is itself compared), so that what is checked is the statistics the convolution handed
            # over and the normalisation, not the conditioning of the data.
            x_q = _qin(case, act[conv["x"]])
            same_mid = case.shaped(conv["y"], orc.op_forward(ci, x_q, w=_conv_weights(case, orc, conv, x_q.shape[-1]))[0])
            same = case.shaped(bn["y"], orc.op_forward(bi, got_mid.astype(np.float64),
                                                       res=_qin(case, act[bn["res"]]) if bn["res"] is not None else None)[0])
        modes.add("mid", conv.get("name", "conv"), got_mid, case.shaped(conv["y"], act[conv["y"]]), same_mid)
        modes.add("fwd", bn.get("name", "bn"), job.debug_get(tid(bn["y"]), n), case.shaped(bn["y"], act[bn["y"]]), same)
        pairs += 1
    case.close()
    return modes.result(pairs=pairs)


def relu_producer_pair_parity(model, dtype, n, N=None, seed=0, data_seed=1, H=0, W=0, C=0, classes=0, arch=(),
                              perturb=0.05, joins=True, only_joins=False):
    """Every convolution whose input comes from the layer listed just before it, ending in a ReLU (a batch norm or
    a convolution with bias and ReLU), and which is the first reader of that tensor in the layer list, run
    backward together with that layer the way a step runs them: the convolution's input-gradient pass stores
    the gradient masked and leaves the producer's column sums.  If the tensor has other readers (a residual
    join: the shortcut of the next block), their contribution - the oracle's - is put into the gradient buffer
    first and the pass adds to it, masks the total and sums it, as inside a step.  Inputs are the oracle's;
    compared are the producer's input gradients and parameter gradients.
    Returns {mode: dict(dx, dw = Worst, dw_whole, pairs, join_pairs)}."""
    case = Case(model, dtype, n, N=N, seed=seed, data_seed=data_seed, H=H, W=W, C=C, classes=classes, arch=arch,
                perturb=perturb)
    job, tensors = case.job, case.tensors
    idx = np.arange(n, dtype=np.int64)
    orc = case.oracle(False)
    ys = case.y[idx]
    _, G = orc.forward_backward(case.x[idx].astype(np.float64), ys)
    act = orc.last_act
    g_rms = float(np.sqrt(np.mean(G * G)))
    job.debug_forward(idx)
    ops = [(oi, op) for oi, op in enumerate(orc.graph.ops) if op["kind"] != "flatten"]
    readers = {}
    for oi, op in ops:
        readers.setdefault(op["x"], []).append(oi)
        if op["kind"] == "bn" and op["res"] is not None:
            readers.setdefault(op["res"], []).append(oi)
    modes, bf = Modes(dtype, ("dx", "dw")), dtype == "bf16"
    pairs = join_pairs = 0
    for gi in range(1, len(ops)):
        (poi, prod), (coi, cons) = ops[gi - 1], ops[gi]
        if cons["kind"] != "conv" or prod["kind"] not in ("bn", "conv") or not prod.get("relu"):
            continue
        if prod["y"] != cons["x"] or tid(prod["x"]) == 0:
            continue
        others = [oi for oi in readers[cons["x"]] if oi != coi]
        if min(readers[cons["x"]]) != coi or (others and not joins) or (only_joins and not others):
            continue
        label = prod.get("name", prod["kind"])
        has_res = prod["kind"] == "bn" and prod["res"] is not None
        # the producer's forward on the oracle's inputs (refreshes the statistics it keeps), then the oracle's output
        job.debug_set(tid(prod["x"]), case.shaped(prod["x"], act[prod["x"]]))
        if has_res:
            job.debug_set(tid(prod["res"]), case.shaped(prod["res"], act[prod["res"]]))
        job.debug_forward_op(gi - 1, n)
        job.debug_set(tid(prod["y"]), case.shaped(prod["y"], act[prod["y"]]))
        job.debug_set(tid(cons["y"]), case.shaped(cons["y"], act[cons["y"]]))
        job.debug_set(tid(cons["y"]), case.shaped(cons["y"], orc.last_dy[coi]), which=1)
        held, acc = [], None
        if others:
            # what the other readers have left in the gradient buffer by the time this convolution runs
            # backward (they come later in the list, so earlier in the backward pass), added in that order
            for oi in sorted(others, reverse=True):
                part = orc.last_dx[oi][cons["x"]]
                acc = part if acc is None else acc + part
            job.debug_set(tid(cons["x"]), case.shaped(cons["x"], acc), which=1)
            held = [tid(cons["x"])]
            join_pairs += 1
        job.debug_backward_range_from(gi - 1, gi + 1, n, held)
        same_dx, same_dp = {}, {}
        if bf:
            # float64 on the same bf16 tensors; the gradient between the two layers is a bf16 tensor like any other
            px_q, py_q = _qin(case, act[prod["x"]]), _qin(case, act[prod["y"]])
            cy_q = act[cons["y"]] if cons["y"] == orc.graph.logits else _qin(case, act[cons["y"]])
            w_c = _conv_weights(case, orc, cons, py_q.shape[-1])
            part = orc.op_backward(coi, _qin(case, orc.last_dy[coi]), py_q, cy_q, w_c, labels=ys)[0][cons["x"]]
            total = part if acc is None else _qin(case, acc) + part
            saved = orc.op_forward(poi, px_q, res=_qin(case, act[prod["res"]]) if has_res else None,
                                   w=_conv_weights(case, orc, prod, px_q.shape[-1]) if prod["kind"] == "conv" else None)[1]
            # the stored gradient is masked already; masking is idempotent, so the producer's backward takes it as it is
            same_dx, same_dp, _ = orc.op_backward(poi, _qin(case, total * (py_q > 0)), px_q, py_q, saved, labels=ys)
        for name, contrib in orc.last_dx.get(poi, {}).items():
            if tid(name) == 0 or tensors[tid(name)][3] == 0:
                continue
            modes.add("dx", label, job.debug_get(tid(name), n, which=1), case.shaped(name, contrib),
                      case.shaped(name, same_dx[name]) if bf else None)
        slices = []
        if prod["kind"] == "bn":
            slices += [(label + ".g", prod["g_off"], prod["C"]), (label + ".b", prod["b_off"], prod["C"])]
        else:
            slices.append((label + ".w", prod["w_off"], prod["K"] * prod["R"] * prod["S"] * act[prod["x"]].shape[-1]))
            if prod["b_off"] is not None:
                slices.append((label + ".b", prod["b_off"], prod["K"]))
        for what, off, size in slices:
            modes.add_param_grad(what, job.grad_slice(0, off, size), G[off:off + size], same_dp[off] if bf else None,
                                 floor=1e-6 * g_rms)
        pairs += 1
    case.close()
    return modes.result(pairs=pairs, join_pairs=join_pairs)


# ---------------------------------------------------------------------------------------------------------
# step by step along a real trajectory
# ---------------------------------------------------------------------------------------------------------
def gpu_decisions(case, orc, n):
    """The decisions the HIP path's own forward pass has just taken (edl_debug_forward must have run on the
    shard): ReLU masks from its stored outputs, max-pool picks recomputed from its stored inputs with the
    first-maximum rule both sides follow.  Keys are the oracle's op indices."""
    job = case.job
    dec = {}
    for oi, op in enumerate(orc.graph.ops):
        if op["kind"] in ("conv", "bn") and op.get("relu"):
            dec[oi] = job.debug_get(tid(op["y"]), n).reshape(orc.last_act[op["y"]].shape) > 0
        elif op["kind"] == "maxpool":
            xg = job.debug_get(tid(op["x"]), n).astype(np.float64)
            dec[oi] = O.maxpool_forward(np.ascontiguousarray(xg), op["k"], op["stride"], op["pad"])[1]
    return dec


def stepwise_parity(model, dtype, N, B, schedule, check=None, shards_of=None, seed=0, data_seed=1, lr=0.1, momentum=0.9,
                    wd=5e-4, H=0, W=0, C=0, classes=0, arch=(), free_given_decisions=None, check_fwd=False, verbose=True,
                    max_shard=None):
    """A job runs `schedule` (one p per step) freely on the GPU.  At every step in `check` (default: all) the
    oracle is given the job's own parameters and momentum (exact float32) and, for each shard in
    shards_of(t, p) (default: all), on that step's real shard indices:
      * the pinned chain: gradients with the oracle's decisions, held to the stated bar (pinned_*);
      * float32 jobs (free_given_decisions): the job's own free-running gradient of that shard against the
        oracle's gradient computed with the decisions the HIP forward pass took (free_*), and how many
        decisions differed from the oracle's own (flips);
      * each worker's free-running loss against the oracle's (a forward pass on equal weights);
    then the step runs as edl_gradients + edl_apply, and
      * the oracle's update formula on the job's own gradient buffers must give the job's new parameters and
        momentum to 1e-6 (update), and the running statistics must follow worker 0 (running).
    Shard index sets are the oracle's bit for bit at every step (asserted).  Returns dict of worst values."""
    p_max = max(schedule)
    case = Case(model, dtype, max_shard or B // min(schedule), N=N, B=B, seed=seed, data_seed=data_seed, H=H, W=W, C=C,
                classes=classes, arch=arch, p_max=p_max, lr=lr, momentum=momentum, wd=wd)
    job, table, tol = case.job, case.table, TOL[dtype]
    if free_given_decisions is None:
        free_given_decisions = dtype == "f32"
    orc = case.oracle(False)
    f32 = lambda v: float(np.float32(v))
    res = dict(pinned=0.0, pinned_whole=0.0, pinned_elem=0.0, free=0.0, free_whole=0.0, free_elem=0.0, flips=0,
               decisions=0, loss=0.0, update=0.0, running=0.0, checked_steps=0, checked_shards=0, losses=[])
    epoch = sie = 0
    for t, p in enumerate(schedule):
        assert job.progress() == (t, epoch, sie)
        idx, off = job.shard(B, p, epoch, sie)
        io, oo = O.shard(seed, N, B, p, epoch, sie)
        assert np.array_equal(idx, io) and np.array_equal(off, oo), "shard assignment differs"
        if check is not None and t not in check:
            res["losses"].append(job.step(p, idx, off))
            assert np.isfinite(res["losses"][-1])
        else:
            w0, v0 = job.params().astype(np.float64), job.momentum().astype(np.float64)
            r0 = job.running().astype(np.float64) if job.R else None
            orc.w, orc.v = w0.copy(), v0.copy()
            ks = list(range(p)) if shards_of is None else sorted(set(shards_of(t, p)))
            want_free, want_loss = {}, {}
            for k in ks:
                sel = idx[off[k]:off[k + 1]]
                n = len(sel)
                if r0 is not None and k == 0:
                    orc.running = r0.copy()
                pc = pinned_chain(case, orc, sel, update_running=(k == 0), check_fwd=check_fwd)
                running_after = orc.running.copy() if (r0 is not None and k == 0) else None
                e, name, whole = per_tensor_relerr(table, pc["g"], pc["G"])
                elem, elem_at = per_tensor_elementwise(table, pc["g"], pc["G"], tol)
                res["pinned"], res["pinned_whole"] = max(res["pinned"], e), max(res["pinned_whole"], whole)
                res["pinned_elem"] = max(res["pinned_elem"], elem)
                want_loss[k] = pc["loss_o"]
                msg = "  step %d p=%d shard %d (n=%d): pinned grad worst %.3e (%s) whole %.3e elem %.3f (%s)" % (
                    t, p, k, n, e, name, whole, elem, elem_at)
                if free_given_decisions:
                    own = orc.last_decisions
                    job.debug_forward(np.asarray(sel, dtype=np.int64))          # the HIP path's own forward pass
                    dec = gpu_decisions(case, orc, n)
                    flips = sum(int(np.sum(own[i] != dec[i])) for i in own)
                    res["flips"] += flips
                    res["decisions"] += sum(v.size for v in own.values())
                    want_free[k] = orc.forward_backward(case.x[sel].astype(np.float64), case.y[sel], decisions=dec)[1] \
                        if flips else pc["G"]
                    msg += " | %d decisions differ" % flips
                if running_after is not None:
                    orc.running = running_after
                if verbose:
                    print(msg, flush=True)
                res["checked_shards"] += 1
            loss = job.gradients(p, idx, off)
            G = [job.grad(k).astype(np.float64) for k in range(p)]
            lk = job.losses(p)
            for k in ks:
                res["loss"] = max(res["loss"], abs(float(lk[k]) - want_loss[k]) / abs(want_loss[k]))
                if k in want_free:
                    e, name, whole = per_tensor_relerr(table, G[k], want_free[k])
                    elem, elem_at = per_tensor_elementwise(table, G[k], want_free[k], tol)
                    res["free"], res["free_whole"] = max(res["free"], e), max(res["free_whole"], whole)
                    res["free_elem"] = max(res["free_elem"], elem)
                    if verbose:
                        print("  step %d shard %d: free-running grad given its decisions: worst %.3e (%s) whole %.3e "
                              "elem %.3f (%s)" % (t, k, e, name, whole, elem, elem_at), flush=True)
            job.apply(p)
            w1, v1 = O.sgd_momentum_update(w0, v0, G, f32(lr), f32(momentum), f32(wd))
            res["update"] = max(res["update"], relerr(job.params(), w1), relerr(job.momentum(), v1))
            if r0 is not None and 0 in ks:
                res["running"] = max(res["running"], relerr(job.running(), orc.running))
            res["losses"].append(loss)
            res["checked_steps"] += 1
            assert np.isfinite(loss)
            if verbose:
                print("  step %d p=%d: loss %.6f | update %.2e running %.2e" % (t, p, loss, res["update"], res["running"]),
                      flush=True)
        sie += 1
        if sie == N // B:
            sie, epoch = 0, epoch + 1
    res["job"], res["case"], res["table"] = job, case, table
    return res
