"""CPU oracle for one worker's synchronous-SGD iteration of an elastic job.

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the bench's cpu_baseline
leg may import this; the product path never does.  It shares no code with the
HIP path.  Everything is float64 unless a function says otherwise.

What it computes, in the paper's terms:

* section 2.1, the mini-batch SGD equation: the model moves by minus the
  learning rate times the mean of the per-sample gradients of the mini-batch;
* section 2.1, synchronous data parallelism: each of the p workers computes
  the gradient of its own samples, the local gradients are aggregated, and
  the aggregate is applied before the next mini-batch;
* section 3.1: the aggregate batch size B is constant, a worker's batch is
  B/p, and an epoch visits every sample exactly once whatever p does;
* section 4.3: the leader holds a random permutation and hands out the next
  unassigned piece on request (here: one-sample pieces, requests served in
  worker-rank order);
* section 4.2: a joining worker receives the model of ONE existing worker
  (here: parameters, momentum, running statistics of worker 0, progress).

* section 3.2, Listing 1: the optimizer the elastic optimizer wraps may be a
  variant of SGD such as Adam (adam_update: Algorithm 1 of Kingma & Ba).

Readings the paper leaves open (default optimizer = momentum SGD with weight decay,
mean aggregation, per-worker batch-norm statistics, generator constants) are
listed in the design notes of this repository.

Parity pins: tests/test_oracle_*.py (finite differences, library routines on
special cases, closed forms of both updates, brute-force shard invariants).
Unpinned: the specific permutation constants (any permutation satisfies the
paper) and the bf16 rounding points of emulate_bf16 mode.
"""
import ctypes
import math
import struct

import numpy as np

from . import build as _build

_lib = ctypes.CDLL(_build.build())
_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int32)


def _d(a):
    return None if a is None else a.ctypes.data_as(_dp)


MASK64 = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15
INIT_KEY = 0xD1B54A32D192ED03


# ----------------------------------------------------------------------------
# counter-based generator (SplitMix64 finaliser applied to key + (j+1)*GOLDEN)
# ----------------------------------------------------------------------------
def splitmix64_at(key: int, j: int) -> int:
    z = (key + (j + 1) * GOLDEN) & MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
    return z ^ (z >> 31)


def _splitmix64_vec(key: int, j: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = np.uint64(key) + (j.astype(np.uint64) + np.uint64(1)) * np.uint64(GOLDEN)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


# ----------------------------------------------------------------------------
# shard assignment (sections 3.1 and 4.3)
# ----------------------------------------------------------------------------
def epoch_permutation(seed: int, epoch: int, N: int) -> list:
    """Leader's random permutation for one epoch: Fisher-Yates from the top
    with j = floor(r * (i+1) / 2^64), r the next 64-bit draw."""
    key = (seed ^ ((GOLDEN * (epoch + 1)) & MASK64)) & MASK64
    perm = list(range(N))
    draw = 0
    for i in range(N - 1, 0, -1):
        r = splitmix64_at(key, draw)
        draw += 1
        j = (r * (i + 1)) >> 64
        perm[i], perm[j] = perm[j], perm[i]
    return perm


def shard(seed: int, N: int, B: int, p: int, epoch: int, step_in_epoch: int):
    """Global batch `step_in_epoch` of `epoch`, cut into p consecutive pieces
    of B/p samples (worker k gets piece k).  Returns (idx[B], off[p+1])."""
    if p <= 0 or B <= 0 or B % p or N % B or not 0 <= step_in_epoch < N // B:
        raise ValueError("bad shard request")
    perm = epoch_permutation(seed, epoch, N)
    idx = perm[step_in_epoch * B:(step_in_epoch + 1) * B]
    n = B // p
    return np.array(idx, dtype=np.int64), np.arange(p + 1, dtype=np.int64) * n


# ----------------------------------------------------------------------------
# bf16 rounding used by emulate_bf16 mode only (round to nearest even)
# ----------------------------------------------------------------------------
def round_bf16(a: np.ndarray) -> np.ndarray:
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    r = ((u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16)) << np.uint64(16)
    out = r.astype(np.uint32).view(np.float32).astype(np.float64)
    nan = np.isnan(f)
    if nan.any():
        out[nan] = np.nan
    return out.reshape(a.shape)


# ----------------------------------------------------------------------------
# layer primitives
# ----------------------------------------------------------------------------
def conv_out(n, k, stride, pad):
    return (n + 2 * pad - k) // stride + 1


def conv2d_forward(x, w, b, stride, pad):
    N, H, W, C = x.shape
    K, R, S, C2 = w.shape
    assert C == C2
    y = np.empty((N, conv_out(H, R, stride, pad), conv_out(W, S, stride, pad), K))
    _lib.oracle_conv2d_forward(_d(x), _d(w), _d(b), _d(y), N, H, W, C, K, R, S, stride, pad)
    return y


def conv2d_backward_input(dy, w, xshape, stride, pad):
    N, H, W, C = xshape
    K, R, S, _ = w.shape
    dx = np.empty(xshape)
    _lib.oracle_conv2d_backward_input(_d(dy), _d(w), _d(dx), N, H, W, C, K, R, S, stride, pad)
    return dx


def conv2d_backward_weight(x, dy, wshape, stride, pad, want_bias):
    N, H, W, C = x.shape
    K, R, S, _ = wshape
    dw = np.empty(wshape)
    db = np.empty(K) if want_bias else None
    _lib.oracle_conv2d_backward_weight(_d(x), _d(dy), _d(dw), _d(db), N, H, W, C, K, R, S, stride, pad)
    return dw, db


def maxpool_forward(x, k, stride, pad):
    N, H, W, C = x.shape
    Ho, Wo = conv_out(H, k, stride, pad), conv_out(W, k, stride, pad)
    y = np.empty((N, Ho, Wo, C))
    arg = np.empty((N, Ho, Wo, C), dtype=np.int32)
    _lib.oracle_maxpool_forward(_d(x), _d(y), arg.ctypes.data_as(_ip), N, H, W, C, k, stride, pad)
    return y, arg


def maxpool_backward(dy, arg, xshape):
    N, H, W, C = xshape
    dx = np.empty(xshape)
    _lib.oracle_maxpool_backward(_d(dy), arg.ctypes.data_as(_ip), _d(dx), N, H, W, C,
                                 dy.shape[1], dy.shape[2])
    return dx


BN_EPS = 1e-5
BN_RUNNING_MOMENTUM = 0.1


def batchnorm_forward(x, gamma, beta):
    """Training-mode batch norm over all rows of x[..., C]; returns
    (y, xhat, mean, biased variance)."""
    x2 = x.reshape(-1, x.shape[-1])
    mean = x2.mean(axis=0)
    var = ((x2 - mean) ** 2).mean(axis=0)
    xhat = (x - mean) / np.sqrt(var + BN_EPS)
    return gamma * xhat + beta, xhat, mean, var


def batchnorm_backward(dy, xhat, gamma, var):
    M = dy.size // dy.shape[-1]
    dy2 = dy.reshape(M, -1)
    xh2 = xhat.reshape(M, -1)
    dbeta = dy2.sum(axis=0)
    dgamma = (dy2 * xh2).sum(axis=0)
    dx = (gamma / np.sqrt(var + BN_EPS)) * (dy - dbeta / M - xhat * (dgamma / M))
    return dx, dgamma, dbeta


def softmax_ce_forward(z, labels):
    """Mean over rows of -log softmax(z)[label], with max subtraction."""
    zs = z - z.max(axis=1, keepdims=True)
    e = np.exp(zs)
    prob = e / e.sum(axis=1, keepdims=True)
    n = z.shape[0]
    loss = -np.log(prob[np.arange(n), labels]).mean()
    return loss, prob


def softmax_ce_backward(prob, labels):
    n = prob.shape[0]
    dz = prob.copy()
    dz[np.arange(n), labels] -= 1.0
    return dz / n


def aggregate_gradients(grads, weights=None):
    """The p local gradients added in rank order.  weights None: their mean
    (equal shards, the SGD equation of section 2.1).  weights given (shard sizes
    over the batch size, for shards of unequal size): the sum of
    weights[k]*grads[k], which is again the mean of the per-sample gradients of
    the whole batch."""
    acc = np.zeros_like(grads[0])
    if weights is None:
        for g in grads:
            acc = acc + g
        return acc / len(grads)
    for wk, g in zip(weights, grads):
        acc = acc + wk * g
    return acc


def sgd_momentum_update(w, v, grads, lr, momentum, wd, weights=None):
    """Aggregate the p local gradients (in rank order), then
    g = aggregate + wd*w ; v = momentum*v + g ; w = w - lr*v.
    With momentum = wd = 0 this is the paper's SGD equation."""
    g = aggregate_gradients(grads, weights) + wd * w
    v_new = momentum * v + g
    w_new = w - lr * v_new
    return w_new, v_new


def adam_update(w, m, s, grads, t, lr, beta1, beta2, eps, wd, weights=None):
    """The variant of SGD that the paper's usage example wraps (section 3.2,
    Listing 1: an Adam optimizer inside the elastic optimizer), applied to the
    aggregated gradient.  The steps are those of Algorithm 1 of Kingma & Ba,
    "Adam: a method for stochastic optimization"; t counts updates from 1:
        g = aggregate + wd*w
        m = beta1*m + (1-beta1)*g          s = beta2*s + (1-beta2)*g*g
        mhat = m / (1 - beta1**t)          shat = s / (1 - beta2**t)
        w = w - lr * mhat / (sqrt(shat) + eps)
    Weight decay enters as in the momentum update (an L2 term in the gradient);
    the paper does not say.  Returns (w, m, s)."""
    g = aggregate_gradients(grads, weights) + wd * w
    m_new = beta1 * m + (1.0 - beta1) * g
    s_new = beta2 * s + (1.0 - beta2) * g * g
    mhat = m_new / (1.0 - beta1 ** t)
    shat = s_new / (1.0 - beta2 ** t)
    w_new = w - lr * mhat / (np.sqrt(shat) + eps)
    return w_new, m_new, s_new


# ----------------------------------------------------------------------------
# model tables.  An op list over named tensors; parameters live in one flat
# vector in op order: conv -> weight[K,R,S,C] then bias[K] (if any);
# bn -> gamma[C] then beta[C].  Running statistics: per bn op mean[C], var[C].
# ----------------------------------------------------------------------------
class Graph:
    def __init__(self, H, W, C):
        self.ops = []
        self.shape = {"x": (H, W, C)}
        self.P = 0
        self.R = 0
        self.tensors = []     # (name, offset, shape, fan_in or 0)
        self._n = 0

    def _name(self):
        self._n += 1
        return "t%d" % self._n

    def conv(self, x, K, R, stride, pad, bias, relu, name):
        H, W, C = self.shape[x]
        y = self._name()
        op = dict(kind="conv", x=x, y=y, K=K, R=R, S=R, stride=stride, pad=pad, relu=relu,
                  w_off=self.P, b_off=None, name=name)
        self.tensors.append((name + ".w", self.P, (K, R, R, C), C * R * R))
        self.P += K * R * R * C
        if bias:
            op["b_off"] = self.P
            self.tensors.append((name + ".b", self.P, (K,), 0))
            self.P += K
        self.shape[y] = (conv_out(H, R, stride, pad), conv_out(W, R, stride, pad), K)
        self.ops.append(op)
        return y

    def bn(self, x, relu, res, name):
        H, W, C = self.shape[x]
        y = self._name()
        op = dict(kind="bn", x=x, y=y, C=C, relu=relu, res=res, g_off=self.P, b_off=self.P + C,
                  run_off=self.R, name=name)
        self.tensors.append((name + ".g", self.P, (C,), 0))
        self.tensors.append((name + ".b", self.P + C, (C,), 0))
        self.P += 2 * C
        self.R += 2 * C
        self.shape[y] = (H, W, C)
        self.ops.append(op)
        return y

    def maxpool(self, x, k, stride, pad):
        H, W, C = self.shape[x]
        y = self._name()
        self.ops.append(dict(kind="maxpool", x=x, y=y, k=k, stride=stride, pad=pad))
        self.shape[y] = (conv_out(H, k, stride, pad), conv_out(W, k, stride, pad), C)
        return y

    def gavgpool(self, x):
        H, W, C = self.shape[x]
        y = self._name()
        self.ops.append(dict(kind="gavgpool", x=x, y=y))
        self.shape[y] = (1, 1, C)
        return y

    def flatten(self, x):
        H, W, C = self.shape[x]
        y = self._name()
        self.ops.append(dict(kind="flatten", x=x, y=y))
        self.shape[y] = (1, 1, H * W * C)
        return y

    def loss(self, x):
        self.ops.append(dict(kind="loss", x=x))
        self.logits = x


def build_mlp(H=1, W=1, C=784, hidden=(256, 256), classes=10):
    g = Graph(H, W, C)
    t = g.flatten("x")
    for i, h in enumerate(hidden):
        t = g.conv(t, h, 1, 1, 0, True, True, "fc%d" % (i + 1))
    t = g.conv(t, classes, 1, 1, 0, True, False, "fc%d" % (len(hidden) + 1))
    g.loss(t)
    return g


def build_resnet20(H=32, W=32, C=3, classes=10, widths=(16, 32, 64), blocks=3):
    g = Graph(H, W, C)
    t = g.conv("x", widths[0], 3, 1, 1, False, False, "stem.conv")
    t = g.bn(t, True, None, "stem.bn")
    cin = widths[0]
    for si, wd in enumerate(widths):
        for bi in range(blocks):
            stride = 2 if (si > 0 and bi == 0) else 1
            nm = "s%d.b%d" % (si + 1, bi + 1)
            u = g.conv(t, wd, 3, stride, 1, False, False, nm + ".conv1")
            u = g.bn(u, True, None, nm + ".bn1")
            u = g.conv(u, wd, 3, 1, 1, False, False, nm + ".conv2")
            sc = t
            if stride != 1 or cin != wd:
                sc = g.conv(t, wd, 1, stride, 0, False, False, nm + ".proj")
                sc = g.bn(sc, False, None, nm + ".projbn")
            t = g.bn(u, True, sc, nm + ".bn2")
            cin = wd
    t = g.gavgpool(t)
    t = g.conv(t, classes, 1, 1, 0, True, False, "fc")
    g.loss(t)
    return g


def build_resnet50(H=224, W=224, C=3, classes=1000, base=64, blocks=(3, 4, 6, 3)):
    g = Graph(H, W, C)
    t = g.conv("x", base, 7, 2, 3, False, False, "stem.conv")
    t = g.bn(t, True, None, "stem.bn")
    t = g.maxpool(t, 3, 2, 1)
    cin = base
    for si, nb in enumerate(blocks):
        width = base * (2 ** si)
        for bi in range(nb):
            stride = 2 if (si > 0 and bi == 0) else 1
            nm = "s%d.b%d" % (si + 1, bi + 1)
            u = g.conv(t, width, 1, 1, 0, False, False, nm + ".conv1")
            u = g.bn(u, True, None, nm + ".bn1")
            u = g.conv(u, width, 3, stride, 1, False, False, nm + ".conv2")
            u = g.bn(u, True, None, nm + ".bn2")
            u = g.conv(u, 4 * width, 1, 1, 0, False, False, nm + ".conv3")
            sc = t
            if bi == 0:
                sc = g.conv(t, 4 * width, 1, stride, 0, False, False, nm + ".proj")
                sc = g.bn(sc, False, None, nm + ".projbn")
            t = g.bn(u, True, sc, nm + ".bn3")
            cin = 4 * width
    t = g.gavgpool(t)
    t = g.conv(t, classes, 1, 1, 0, True, False, "fc")
    g.loss(t)
    return g


def build_vgg16(H=224, W=224, C=3, classes=1000, base=64, fc=4096, groups=(2, 2, 3, 3, 3)):
    """VGG: groups (2,2,3,3,3) is the 16-layer net, (2,2,4,4,4) the 19-layer one (both appear in the
    tables of section 6)."""
    g = Graph(H, W, C)
    t = "x"
    plan = list(zip([base, 2 * base, 4 * base, 8 * base, 8 * base], groups))
    i = 0
    for width, reps in plan:
        for _ in range(reps):
            i += 1
            t = g.conv(t, width, 3, 1, 1, True, True, "conv%d" % i)
        t = g.maxpool(t, 2, 2, 0)
    t = g.flatten(t)
    t = g.conv(t, fc, 1, 1, 0, True, True, "fc1")
    t = g.conv(t, fc, 1, 1, 0, True, True, "fc2")
    t = g.conv(t, classes, 1, 1, 0, True, False, "fc3")
    g.loss(t)
    return g


def build_alexnet(H=224, W=224, C=3, classes=1000, base=64, fc=4096):
    """AlexNet (a row of the tables of section 6) in its single-tower form: five biased convolutions
    with ReLU, 3x3/2 max pools after the 1st, 2nd and 5th, three fully connected layers; no response
    normalisation, no dropout."""
    g = Graph(H, W, C)
    t = g.conv("x", base, 11, 4, 2, True, True, "conv1")
    t = g.maxpool(t, 3, 2, 0)
    t = g.conv(t, 3 * base, 5, 1, 2, True, True, "conv2")
    t = g.maxpool(t, 3, 2, 0)
    t = g.conv(t, 6 * base, 3, 1, 1, True, True, "conv3")
    t = g.conv(t, 4 * base, 3, 1, 1, True, True, "conv4")
    t = g.conv(t, 4 * base, 3, 1, 1, True, True, "conv5")
    t = g.maxpool(t, 3, 2, 0)
    t = g.flatten(t)
    t = g.conv(t, fc, 1, 1, 0, True, True, "fc1")
    t = g.conv(t, fc, 1, 1, 0, True, True, "fc2")
    t = g.conv(t, classes, 1, 1, 0, True, False, "fc3")
    g.loss(t)
    return g


MODEL_IDS = {"mlp": 0, "resnet20": 1, "resnet50": 2, "vgg16": 3, "alexnet": 4}
BUILDERS = {"mlp": build_mlp, "resnet20": build_resnet20, "resnet50": build_resnet50,
            "vgg16": build_vgg16, "alexnet": build_alexnet}
# the deeper members of the two families named in section 6, as (builder, keyword arguments)
VARIANTS = {"resnet101": ("resnet50", dict(blocks=(3, 4, 23, 3))),
            "resnet152": ("resnet50", dict(blocks=(3, 8, 36, 3))),
            "vgg19": ("vgg16", dict(groups=(2, 2, 4, 4, 4)))}


# ----------------------------------------------------------------------------
# He initialisation from the seed
# ----------------------------------------------------------------------------
def he_init(graph: Graph, seed: int) -> np.ndarray:
    """Weights ~ N(0, 2/fan_in) by Box-Muller on counter-based draws, one
    stream per parameter tensor; biases 0, gamma 1, beta 0.  Values are
    rounded to float32 (the storage type of the master weights)."""
    w = np.zeros(graph.P, dtype=np.float64)
    for t, (name, off, shape, fan_in) in enumerate(graph.tensors):
        n = int(np.prod(shape))
        if name.endswith(".g"):
            w[off:off + n] = 1.0
        if fan_in == 0:
            continue
        key = (seed ^ ((INIT_KEY * (t + 1)) & MASK64)) & MASK64
        npair = (n + 1) // 2
        q = np.arange(npair, dtype=np.uint64)
        r1 = _splitmix64_vec(key, q * np.uint64(2))
        r2 = _splitmix64_vec(key, q * np.uint64(2) + np.uint64(1))
        u1 = ((r1 >> np.uint64(11)).astype(np.float64) + 1.0) * 2.0 ** -53
        u2 = (r2 >> np.uint64(11)).astype(np.float64) * 2.0 ** -53
        rad = np.sqrt(-2.0 * np.log(u1))
        ang = 2.0 * math.pi * u2
        z = np.empty(2 * npair)
        z[0::2] = rad * np.cos(ang)
        z[1::2] = rad * np.sin(ang)
        std = math.sqrt(2.0 / fan_in)
        w[off:off + n] = (z[:n] * std).astype(np.float32).astype(np.float64)
    return w


# ----------------------------------------------------------------------------
# the worker state and its iteration
# ----------------------------------------------------------------------------
SNAPSHOT_MAGIC = 0x314C4445      # "EDL1"
SNAPSHOT_HEADER_BYTES = 256


OPTIMIZER_IDS = {"momentum": 0, "adam": 1}


class Oracle:
    def __init__(self, model: str, seed: int, N: int, B: int, lr=0.1, momentum=0.9, wd=5e-4,
                 emulate_bf16=False, graph_kwargs=None, dtype_code=0, optimizer="momentum",
                 beta2=0.999, eps=1e-8):
        """optimizer "momentum": momentum-SGD with `momentum`; "adam": Adam, whose beta1 is `momentum`."""
        self.model = model
        self.optimizer, self.beta2, self.eps = optimizer, beta2, eps
        assert optimizer in OPTIMIZER_IDS
        self.graph = BUILDERS[model](**(graph_kwargs or {}))
        self.seed, self.N, self.B = seed, N, B
        self.lr, self.momentum, self.wd = lr, momentum, wd
        self.emulate_bf16 = emulate_bf16
        # Max pools pick their element after rounding the input to bf16 (the precision a bf16 job holds it in);
        # the pooled values themselves are not rounded.  Off by default; tests that compare a bf16 job with the
        # unrounded float64 computation switch it on so that both sides decide in the same precision.
        self.pool_picks_in_bf16 = False
        self.dtype_code = dtype_code
        self.w = he_init(self.graph, seed)
        self.v = np.zeros_like(self.w)          # momentum, or Adam's first moment
        self.s = np.zeros_like(self.w)          # Adam's second moment (unused otherwise)
        self.running = np.zeros(self.graph.R)
        for op in self.graph.ops:
            if op["kind"] == "bn":
                C = op["C"]
                self.running[op["run_off"] + C:op["run_off"] + 2 * C] = 1.0
        self.step_count = 0
        self.epoch = 0
        self.step_in_epoch = 0
        self.last_grads = None
        self.last_losses = None

    # -- helpers ---------------------------------------------------------
    def _q(self, a):
        return round_bf16(a) if self.emulate_bf16 else a

    def _param(self, off, shape):
        n = int(np.prod(shape))
        return self.w[off:off + n].reshape(shape)

    # -- one layer on given tensors ----------------------------------------
    def op_forward(self, i, xin, res=None, w=None, labels=None):
        """Layer i of the model on the given input (and residual input), in
        float64 with no rounding anywhere.  `w` replaces a convolution's
        weights (the bf16 copies a bf16 job contracts with).  Returns
        (output, what the layer's backward needs besides its input and output);
        the loss layer returns (mean loss, softmax probabilities)."""
        op = self.graph.ops[i]
        kind = op["kind"]
        if kind == "conv":
            C = xin.shape[-1]
            if w is None:
                w = self._param(op["w_off"], (op["K"], op["R"], op["S"], C))
            b = self._param(op["b_off"], (op["K"],)) if op["b_off"] is not None else None
            y = conv2d_forward(xin, np.ascontiguousarray(w), b, op["stride"], op["pad"])
            if op["relu"]:
                y = np.maximum(y, 0.0)
            return y, w
        if kind == "bn":
            C = op["C"]
            y, xhat, mean, var = batchnorm_forward(xin, self._param(op["g_off"], (C,)), self._param(op["b_off"], (C,)))
            if res is not None:
                y = y + res
            if op["relu"]:
                y = np.maximum(y, 0.0)
            return y, (xhat, var, mean)
        if kind == "maxpool":
            y, arg = maxpool_forward(xin, op["k"], op["stride"], op["pad"])
            if self.pool_picks_in_bf16:
                # the decision (which element of the window) taken in the precision a bf16 job holds the tensor
                # in: values that round to the same bf16 tie, and ties go to the first in window order
                arg = maxpool_forward(round_bf16(xin), op["k"], op["stride"], op["pad"])[1]
            return y, arg
        if kind == "gavgpool":
            return xin.mean(axis=(1, 2), keepdims=True), None
        if kind == "flatten":
            return xin.reshape(xin.shape[0], 1, 1, -1), None
        if kind == "loss":
            return softmax_ce_forward(xin.reshape(xin.shape[0], -1), labels)
        raise ValueError(kind)

    def op_backward(self, i, dy, xin, y, saved, labels=None, decision=None):
        """Backward of layer i: dy is the gradient of its output (ignored by the
        loss layer), xin / y its forward input / output, saved what op_forward
        returned.  decision replaces the layer's own (ReLU: output > 0; max
        pool: saved positions).  Returns ({input: gradient contribution},
        {offset in the flat vector: parameter gradient}, decision used)."""
        op = self.graph.ops[i]
        kind = op["kind"]
        dxs, dps, used = {}, {}, None
        if kind == "loss":
            dxs[op["x"]] = softmax_ce_backward(saved, labels).reshape(xin.shape)
        elif kind == "conv":
            if op["relu"]:
                used = (y > 0) if decision is None else decision
                dy = dy * used
            w = saved
            dw, db = conv2d_backward_weight(xin, np.ascontiguousarray(dy), w.shape, op["stride"], op["pad"],
                                            op["b_off"] is not None)
            dps[op["w_off"]] = dw.ravel()
            if db is not None:
                dps[op["b_off"]] = db
            if op["x"] != "x":
                dxs[op["x"]] = conv2d_backward_input(np.ascontiguousarray(dy), np.ascontiguousarray(w), xin.shape,
                                                     op["stride"], op["pad"])
        elif kind == "bn":
            if op["relu"]:
                used = (y > 0) if decision is None else decision
                dy = dy * used
            if op["res"] is not None:
                dxs[op["res"]] = dy
            xhat, var = saved[0], saved[1]
            C = op["C"]
            dx, dgamma, dbeta = batchnorm_backward(dy, xhat, self._param(op["g_off"], (C,)), var)
            dps[op["g_off"]] = dgamma
            dps[op["b_off"]] = dbeta
            dxs[op["x"]] = dx
        elif kind == "maxpool":
            used = np.ascontiguousarray(saved if decision is None else decision, dtype=np.int32)
            dxs[op["x"]] = maxpool_backward(np.ascontiguousarray(dy), used, xin.shape)
        elif kind == "gavgpool":
            dxs[op["x"]] = np.broadcast_to(dy / (xin.shape[1] * xin.shape[2]), xin.shape).copy()
        elif kind == "flatten":
            dxs[op["x"]] = dy.reshape(xin.shape)
        return dxs, dps, used

    # -- forward + backward on one worker's samples ------------------------
    def forward_backward(self, x, labels, update_running=False, decisions=None):
        """x: [n,H,W,C] float64, labels: [n] ints.  Returns (mean loss over
        the n samples, flat gradient of that mean loss w.r.t. all parameters).

        The backward pass takes two kinds of discrete decision from the forward
        activations: which outputs a ReLU let through (output > 0) and which
        element of its window a max pool picked.  They are kept in
        self.last_decisions {op index: boolean mask | int32 positions}.
        `decisions` (test hook; same keys) replaces any of them by given ones,
        so that a test can ask what the gradient would be had a neighbouring
        computation decided differently; the forward values are not changed."""
        g = self.graph
        q = self._q
        decisions = decisions or {}
        self.last_decisions = {}
        act = {"x": q(np.ascontiguousarray(x, dtype=np.float64))}
        saved = {}
        loss = None
        for i, op in enumerate(g.ops):
            kind = op["kind"]
            xin = act[op["x"]]
            if kind == "conv":
                w = q(self._param(op["w_off"], (op["K"], op["R"], op["S"], xin.shape[-1])))
                y, saved[i] = self.op_forward(i, xin, w=w)
                act[op["y"]] = q(y) if op["y"] != g.logits else y
            elif kind == "bn":
                y, saved[i] = self.op_forward(i, xin, res=act[op["res"]] if op["res"] is not None else None)
                act[op["y"]] = q(y)
                if update_running:
                    C = op["C"]
                    M = xin.size // C
                    mean, var = saved[i][2], saved[i][1]
                    ro = op["run_off"]
                    m = BN_RUNNING_MOMENTUM
                    self.running[ro:ro + C] = (1 - m) * self.running[ro:ro + C] + m * mean
                    self.running[ro + C:ro + 2 * C] = ((1 - m) * self.running[ro + C:ro + 2 * C]
                                                       + m * var * M / (M - 1))
            elif kind == "maxpool":
                act[op["y"]], saved[i] = self.op_forward(i, xin)
            elif kind == "gavgpool":
                act[op["y"]] = q(self.op_forward(i, xin)[0])
            elif kind == "flatten":
                act[op["y"]] = self.op_forward(i, xin)[0]
            elif kind == "loss":
                loss, saved[i] = self.op_forward(i, xin, labels=labels)
        self.last_act = act            # name -> activation, "x", "t1", "t2", ... in creation order
        self.last_saved = saved
        # backward
        G = np.zeros(g.P)
        grad = {}
        self.last_dy, self.last_dx = {}, {}     # per op: gradient of its output as used; {input: its contribution}
        for i in range(len(g.ops) - 1, -1, -1):
            op = g.ops[i]
            kind = op["kind"]
            dy = None
            if kind != "loss":
                self.last_dy[i] = grad[op["y"]]
                dy = grad.pop(op["y"])
            dxs, dps, used = self.op_backward(i, dy, act[op["x"]], act.get(op.get("y")), saved.get(i), labels=labels,
                                              decision=decisions.get(i))
            if used is not None:
                self.last_decisions[i] = used
            for off, val in dps.items():
                G[off:off + val.size] = val
            for name, val in dxs.items():
                if name == "x":
                    continue
                self.last_dx.setdefault(i, {})[name] = q(val)
                grad[name] = q(grad[name] + val) if name in grad else q(val)
        return loss, G

    # -- one synchronous iteration at parallelism p ----------------------
    def step(self, p, data_x, data_y, idx=None, off=None):
        """One mini-batch: every worker k computes the gradient on its shard,
        the p gradients are averaged and applied.  Returns the mean of the
        workers' losses.  Worker 0 (the one that would broadcast its model to
        a joiner) is the one whose batch-norm running statistics are kept."""
        if idx is None:
            idx, off = shard(self.seed, self.N, self.B, p, self.epoch, self.step_in_epoch)
        sizes = [int(off[k + 1] - off[k]) for k in range(p)]
        grads, losses, live = [], [], []
        for k in range(p):
            if sizes[k] == 0:
                continue                      # a worker the data pipeline could give nothing
            sel = idx[off[k]:off[k + 1]]
            x = np.asarray(data_x[sel], dtype=np.float64)
            loss, G = self.forward_backward(x, np.asarray(data_y[sel]), update_running=(not live))
            live.append(k)
            grads.append(G)
            losses.append(loss)
        if all(n == sizes[0] for n in sizes):
            wts = None
            mean_loss = float(np.mean(losses))
        else:
            # shards of unequal size (a tail batch of the data pipeline, a mini-batch redone by the
            # survivors of a failure): every worker weighs in with its share of the batch
            wts = [sizes[k] / float(self.B) for k in live]
            mean_loss = float(sum(wk * lk for wk, lk in zip(wts, losses)))
        if self.optimizer == "adam":
            self.w, self.v, self.s = adam_update(self.w, self.v, self.s, grads, self.step_count + 1, self.lr,
                                                 self.momentum, self.beta2, self.eps, self.wd, weights=wts)
        else:
            self.w, self.v = sgd_momentum_update(self.w, self.v, grads, self.lr, self.momentum, self.wd, weights=wts)
        self.last_grads, self.last_losses = grads, losses
        self.step_count += 1
        self.step_in_epoch += 1
        if self.step_in_epoch == self.N // self.B:
            self.step_in_epoch = 0
            self.epoch += 1
        return mean_loss

    # -- approximate recovery (section 4.2, failure recovery) ---------------
    @staticmethod
    def survivor_cut(B, survivors):
        """The mini-batch of B samples re-cut over `survivors` workers, as evenly
        as the counts allow: the first B mod survivors workers take one sample
        more (the paper only says that a worker's batch follows from the
        parallelism; the aggregate batch stays B).  Returns off[survivors+1]."""
        base, extra = divmod(B, survivors)
        sizes = [base + (1 if k < extra else 0) for k in range(survivors)]
        return np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)

    def redo_with_survivors(self, p, lost_k, data_x, data_y):
        """Worker lost_k of p fails during the current mini-batch (its gradient
        never arrives, so the aggregation of that attempt cannot complete and
        nothing of it is applied).  Approximate recovery: the p-1 survivors form
        a new group and redo the CURRENT mini-batch - the same B samples at the
        same cursor, re-cut over p-1 workers, every worker weighing in with its
        share n_k/B - and the job moves on by one mini-batch.  Returns
        (loss of the redone mini-batch, gradients of the discarded attempt's
        surviving workers)."""
        assert p >= 2 and 0 <= lost_k < p
        idx, off = shard(self.seed, self.N, self.B, p, self.epoch, self.step_in_epoch)
        before = (self.w.copy(), self.v.copy(), self.s.copy(), self.running.copy(), self.step_count)
        discarded = []
        for k in range(p):
            if k == lost_k:
                continue
            sel = idx[off[k]:off[k + 1]]
            _, G = self.forward_backward(np.asarray(data_x[sel], dtype=np.float64), np.asarray(data_y[sel]))
            discarded.append(G)
        # nothing of the failed attempt may have touched the job
        assert all(np.array_equal(a, b) for a, b in zip(before[:4], (self.w, self.v, self.s, self.running)))
        loss = self.step(p - 1, data_x, data_y, idx, self.survivor_cut(self.B, p - 1))
        assert self.step_count == before[4] + 1
        return loss, discarded

    # -- what a joining worker receives ------------------------------------
    def snapshot(self) -> bytes:
        """Header (job meta-data and progress), then parameters, the optimizer's
        state (momentum; for Adam the first and then the second moment) and
        running statistics as float32.  Little endian."""
        adam = self.optimizer == "adam"
        hdr = struct.pack("<IIIIQqqqqqfffIqqff", SNAPSHOT_MAGIC, 1, MODEL_IDS[self.model], self.dtype_code,
                          self.seed, self.N, self.B, self.step_count, self.epoch, self.step_in_epoch,
                          self.lr, self.momentum, self.wd, OPTIMIZER_IDS[self.optimizer], self.graph.P, self.graph.R,
                          self.beta2 if adam else 0.0, self.eps if adam else 0.0)
        hdr = hdr + b"\0" * (SNAPSHOT_HEADER_BYTES - len(hdr))
        return (hdr + self.w.astype(np.float32).tobytes() + self.v.astype(np.float32).tobytes()
                + (self.s.astype(np.float32).tobytes() if adam else b"")
                + self.running.astype(np.float32).tobytes())

    def restore(self, blob: bytes):
        P, R = self.graph.P, self.graph.R
        f = struct.unpack_from("<IIIIQqqqqqfffIqq", blob, 0)
        assert f[0] == SNAPSHOT_MAGIC and f[14] == P and f[15] == R and f[13] == OPTIMIZER_IDS[self.optimizer]
        # job meta-data travels with the model (section 4.2): seed, sizes, progress and the optimizer's
        # coefficients of the job replace whatever this worker was created with
        self.seed, self.N, self.B = f[4], f[5], f[6]
        self.step_count, self.epoch, self.step_in_epoch = f[7], f[8], f[9]
        self.lr, self.momentum, self.wd = f[10], f[11], f[12]
        if self.optimizer == "adam":
            self.beta2, self.eps = struct.unpack_from("<ff", blob, 96)
        o = SNAPSHOT_HEADER_BYTES
        self.w = np.frombuffer(blob, np.float32, P, o).astype(np.float64)
        self.v = np.frombuffer(blob, np.float32, P, o + 4 * P).astype(np.float64)
        o += 8 * P
        if self.optimizer == "adam":
            self.s = np.frombuffer(blob, np.float32, P, o).astype(np.float64)
            o += 4 * P
        self.running = np.frombuffer(blob, np.float32, R, o).astype(np.float64)
