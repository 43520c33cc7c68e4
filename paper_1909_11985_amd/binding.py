"""ctypes binding of libedl.so: argument marshalling only.

Names follow include/edl.h.  The library is loaded from this directory and is
never replaced by a fallback: if it is missing, build it with
`python -m paper_1909_11985_amd.build` (needs hipcc); if that is impossible the
import fails.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("EDL_LIBRARY") or os.path.join(_HERE, "libedl.so")   # EDL_LIBRARY: another build of the same library

MODELS = {"mlp": 0, "resnet20": 1, "resnet50": 2, "vgg16": 3, "alexnet": 4}
DTYPES = {"f32": 0, "bf16": 1}


class EdlError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("edl error %d: %s" % (code, msg))
        self.code = code


class Config(C.Structure):
    _fields_ = [("model", C.c_int32), ("dtype", C.c_int32), ("N", C.c_int64), ("B", C.c_int64),
                ("p_max", C.c_int32), ("max_shard", C.c_int32),
                ("lr", C.c_float), ("momentum", C.c_float), ("wd", C.c_float),
                ("H", C.c_int32), ("W", C.c_int32), ("C", C.c_int32), ("classes", C.c_int32),
                ("arch", C.c_int32 * 8), ("optimizer", C.c_int32), ("beta2", C.c_float), ("eps", C.c_float)]


class Sizes(C.Structure):
    _fields_ = [("P", C.c_int64), ("R", C.c_int64), ("params_off", C.c_int64), ("momentum_off", C.c_int64),
                ("running_off", C.c_int64), ("grads_off", C.c_int64), ("grad_stride", C.c_int64),
                ("arena_bytes", C.c_int64), ("snapshot_bytes", C.c_int64), ("flops_per_sample", C.c_double),
                ("second_off", C.c_int64), ("scratch_bytes", C.c_int64), ("shadow_off", C.c_int64)]


class Progress(C.Structure):
    _fields_ = [("step", C.c_int64), ("epoch", C.c_int64), ("step_in_epoch", C.c_int64)]


def _load():
    if not os.path.exists(_LIB_PATH):
        from . import build as _b
        _b.build()
    # The caller's device memory and streams come from PyTorch, which ships a HIP runtime of its own.  It has to
    # be the one already in the process when this library is mapped, so that both see the same runtime (a
    # second copy finds no device): torch first, whatever order the caller imports things in.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    return C.CDLL(_LIB_PATH)


lib = _load()
lib.edl_last_error.restype = C.c_char_p
_i64p = C.POINTER(C.c_int64)
_f32p = C.POINTER(C.c_float)

_SIGS = {
    "edl_query": [C.POINTER(Config), C.POINTER(Sizes)],
    "edl_tensor_count": [C.POINTER(Config), C.POINTER(C.c_int32)],
    "edl_tensor_info": [C.POINTER(Config), C.c_int32, C.c_char_p, C.c_size_t, _i64p, _i64p, _i64p],
    "edl_init_params_host": [C.POINTER(Config), C.c_uint64, _f32p],
    "edl_shard_host": [C.c_uint64, C.c_int64, C.c_int64, C.c_int32, C.c_int64, C.c_int64, _i64p, _i64p],
    "edl_init": [C.POINTER(C.c_void_p), C.POINTER(Config), C.c_uint64, C.c_void_p, C.c_size_t, C.c_void_p],
    "edl_bind_dataset": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64],
    "edl_shard": [C.c_void_p, C.c_int64, C.c_int32, C.c_int64, C.c_int64, _i64p, _i64p],
    "edl_step": [C.c_void_p, C.c_int32, _i64p, _i64p, _f32p],
    "edl_step_static_scratch": [C.c_void_p, C.c_int32, _i64p, _i64p, _f32p],
    "edl_gradients": [C.c_void_p, C.c_int32, _i64p, _i64p, _f32p],
    "edl_apply": [C.c_void_p, C.c_int32],
    "edl_snapshot": [C.c_void_p, C.c_void_p, C.c_size_t, C.POINTER(C.c_size_t)],
    "edl_restore": [C.c_void_p, C.c_void_p, C.c_size_t],
    "edl_get_progress": [C.c_void_p, C.POINTER(Progress)],
    "edl_get_params": [C.c_void_p, _f32p],
    "edl_get_momentum": [C.c_void_p, _f32p],
    "edl_get_running": [C.c_void_p, _f32p],
    "edl_get_grad": [C.c_void_p, C.c_int32, _f32p],
    "edl_get_losses": [C.c_void_p, C.c_int32, _f32p],
    "edl_set_params": [C.c_void_p, _f32p],
    "edl_set_momentum": [C.c_void_p, _f32p],
    "edl_get_second_moment": [C.c_void_p, _f32p],
    "edl_set_second_moment": [C.c_void_p, _f32p],
    "edl_debug_tensor_count": [C.c_void_p, C.POINTER(C.c_int32)],
    "edl_debug_tensor_shape": [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                               C.POINTER(C.c_int32), C.POINTER(C.c_int32)],
    "edl_debug_forward": [C.c_void_p, _i64p, C.c_int32],
    "edl_debug_backward": [C.c_void_p, C.c_int32, C.c_int32],
    "edl_debug_get_tensor": [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, _f32p],
    "edl_debug_set_tensor": [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, _f32p],
    "edl_debug_op_count": [C.c_void_p, C.POINTER(C.c_int32)],
    "edl_debug_forward_op": [C.c_void_p, C.c_int32, C.c_int32],
    "edl_debug_forward_range": [C.c_void_p, C.c_int32, C.c_int32, C.c_int32],
    "edl_debug_backward_op": [C.c_void_p, C.c_int32, C.c_int32, C.c_int32],
    "edl_debug_backward_range": [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32],
    "edl_debug_backward_range_from": [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.c_int32],
    "edl_debug_set_labels": [C.c_void_p, C.POINTER(C.c_int32), C.c_int32],
    "edl_set_side_streams": [C.c_void_p, C.c_void_p, C.c_void_p],
    "edl_set_option": [C.c_char_p, C.c_int64],
    "edl_get_option": [C.c_char_p, _i64p],
    "edl_shutdown": [C.c_void_p],
    "edl_average_update": [C.c_int32, C.POINTER(C.c_void_p), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                           C.c_float, C.c_float, C.c_float, C.c_void_p],
    "edl_adam_update": [C.c_int32, C.POINTER(C.c_void_p), C.POINTER(C.c_float), C.c_void_p, C.c_void_p, C.c_void_p,
                        C.c_void_p, C.c_int64, C.c_float, C.c_float, C.c_float, C.c_float, C.c_float, C.c_int64, C.c_void_p],
    "edl_copy": [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p],
    "edl_profile_parallelism": [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.POINTER(C.c_int32)],
    "edl_pipeline_create": [C.c_uint64, C.c_int64, C.c_int64, C.POINTER(C.c_void_p)],
    "edl_pipeline_next_batch": [C.c_void_p, C.c_int64, C.c_int32, _i64p, _i64p, _i64p],
    "edl_pipeline_progress": [C.c_void_p, _i64p, _i64p],
    "edl_pipeline_save": [C.c_void_p, _i64p, C.c_size_t, C.POINTER(C.c_size_t)],
    "edl_pipeline_load": [_i64p, C.c_size_t, C.POINTER(C.c_void_p)],
    "edl_pipeline_destroy": [C.c_void_p],
    "edl_mfma_rate": [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.POINTER(C.c_double)],
    "edl_profile": [C.c_int32],
    "edl_profile_report": [C.c_char_p, C.c_size_t, C.POINTER(C.c_size_t)],
}
for _name, _args in _SIGS.items():
    try:
        _fn = getattr(lib, _name)
    except AttributeError:
        raise ImportError("%s lacks %s: it is older than include/edl.h; rebuild it with "
                          "`python paper_1909_11985_amd/build.py`" % (_LIB_PATH, _name)) from None
    _fn.argtypes = _args
    _fn.restype = C.c_int32
EXPORTS = ["edl_last_error"] + list(_SIGS)


def _check(rc):
    if rc != 0:
        raise EdlError(rc, lib.edl_last_error().decode())


OPTIMIZERS = {"momentum": 0, "adam": 1}


def make_config(model, dtype="f32", N=1024, B=64, p_max=8, max_shard=None, lr=0.1, momentum=0.9, wd=5e-4,
                H=0, W=0, C_=0, classes=0, arch=(), optimizer="momentum", beta2=0.999, eps=1e-8):
    """optimizer "adam": `momentum` is its beta1."""
    cfg = Config()
    cfg.model = MODELS[model] if isinstance(model, str) else model
    cfg.dtype = DTYPES[dtype] if isinstance(dtype, str) else dtype
    cfg.N, cfg.B, cfg.p_max = N, B, p_max
    cfg.max_shard = B if max_shard is None else max_shard
    cfg.lr, cfg.momentum, cfg.wd = lr, momentum, wd
    cfg.H, cfg.W, cfg.C, cfg.classes = H, W, C_, classes
    for i, a in enumerate(arch):
        cfg.arch[i] = a
    cfg.optimizer = OPTIMIZERS[optimizer] if isinstance(optimizer, str) else optimizer
    cfg.beta2, cfg.eps = beta2, eps
    return cfg


def edl_query(cfg):
    s = Sizes()
    _check(lib.edl_query(C.byref(cfg), C.byref(s)))
    return s


def edl_tensor_table(cfg):
    """[(name, offset, size, fan_in)] of the flat parameter vector."""
    n = C.c_int32()
    _check(lib.edl_tensor_count(C.byref(cfg), C.byref(n)))
    out = []
    buf = C.create_string_buffer(64)
    off, size, fan = C.c_int64(), C.c_int64(), C.c_int64()
    for i in range(n.value):
        _check(lib.edl_tensor_info(C.byref(cfg), i, buf, 64, C.byref(off), C.byref(size), C.byref(fan)))
        out.append((buf.value.decode(), off.value, size.value, fan.value))
    return out


def edl_init_params_host(cfg, seed):
    P = edl_query(cfg).P
    out = np.empty(P, dtype=np.float32)
    _check(lib.edl_init_params_host(C.byref(cfg), seed, out.ctypes.data_as(_f32p)))
    return out


def edl_shard_host(seed, N, B, p, epoch, step_in_epoch):
    idx = np.empty(max(B, 1), dtype=np.int64)
    off = np.empty(max(p, 0) + 1, dtype=np.int64)
    _check(lib.edl_shard_host(seed, N, B, p, epoch, step_in_epoch, idx.ctypes.data_as(_i64p), off.ctypes.data_as(_i64p)))
    return idx, off


def edl_average_update(grads, w, v, w16, lr, momentum, wd, stream=0):
    """grads: list of float32 device tensors; w, v: float32 device tensors;
    w16: bfloat16 device tensor or None."""
    p = len(grads)
    ptrs = (C.c_void_p * p)(*[g.data_ptr() for g in grads])
    _check(lib.edl_average_update(p, ptrs, w.data_ptr(), v.data_ptr(), w16.data_ptr() if w16 is not None else None,
                                  w.numel(), lr, momentum, wd, stream))


def edl_adam_update(grads, w, m, s, w16, lr, beta1, beta2, eps, wd, t, shares=None, stream=0):
    """grads: list of float32 device tensors; w, m, s: float32 device tensors; w16: bfloat16 device tensor or
    None; t: number of this update (from 1); shares: optional weights of the gradients (else their mean)."""
    p = len(grads)
    ptrs = (C.c_void_p * p)(*[g.data_ptr() for g in grads])
    sh = None if shares is None else (C.c_float * p)(*[float(x) for x in shares])
    _check(lib.edl_adam_update(p, ptrs, sh, w.data_ptr(), m.data_ptr(), s.data_ptr(),
                               w16.data_ptr() if w16 is not None else None, w.numel(), lr, beta1, beta2, eps, wd, t, stream))


def edl_mfma_rate(dtype, blocks, iters, sink, stream=0):
    """Launches the register-resident MFMA loop; returns the flops it issues (time it with edl_profile)."""
    f = C.c_double(0)
    _check(lib.edl_mfma_rate(DTYPES[dtype], blocks, iters, sink.data_ptr(), stream, C.byref(f)))
    return f.value


def edl_copy(dst, src, nbytes, stream=0):
    _check(lib.edl_copy(dst.data_ptr(), src.data_ptr(), nbytes, stream))


def edl_set_option(name, value):
    _check(lib.edl_set_option(name.encode(), int(value)))


def edl_get_option(name):
    v = C.c_int64()
    _check(lib.edl_get_option(name.encode(), C.byref(v)))
    return v.value


class options:
    """with options(force_tile=2, ...): the named options hold inside the block and are put back after it."""

    def __init__(self, **kw):
        self.kw = kw

    def __enter__(self):
        self.old = {k: edl_get_option(k) for k in self.kw}
        for k, v in self.kw.items():
            edl_set_option(k, v)
        return self

    def __exit__(self, *exc):
        for k, v in self.old.items():
            edl_set_option(k, v)
        return False


def edl_profile(enable):
    _check(lib.edl_profile(1 if enable else 0))


def edl_profile_report():
    """List of dicts {name, launches, ms, flops, bytes}: totals since profiling was switched on
    (or since the last report)."""
    import json
    buf = C.create_string_buffer(1 << 18)
    need = C.c_size_t()
    _check(lib.edl_profile_report(buf, len(buf), C.byref(need)))
    return json.loads(buf.value.decode())


class ParallelismPoint(C.Structure):
    _fields_ = [("p", C.c_int32), ("shard", C.c_int32), ("ms_per_step", C.c_double), ("samples_per_s", C.c_double),
                ("worker_samples_per_s", C.c_double), ("efficiency", C.c_double)]


class Pipeline:
    """The dynamic data pipeline of include/edl.h (edl_pipeline_*): host bookkeeping only."""

    def __init__(self, seed=0, N=0, d=0, _handle=None):
        if _handle is not None:
            self._h = _handle
            return
        h = C.c_void_p()
        _check(lib.edl_pipeline_create(seed, N, d, C.byref(h)))
        self._h = h

    def next_batch(self, B, worker_ids):
        ids = np.ascontiguousarray(worker_ids, dtype=np.int64)
        idx = np.empty(B, dtype=np.int64)
        off = np.empty(len(ids) + 1, dtype=np.int64)
        _check(lib.edl_pipeline_next_batch(self._h, B, len(ids), ids.ctypes.data_as(_i64p), idx.ctypes.data_as(_i64p),
                                           off.ctypes.data_as(_i64p)))
        return idx, off

    def progress(self):
        e, c = C.c_int64(), C.c_int64()
        _check(lib.edl_pipeline_progress(self._h, C.byref(e), C.byref(c)))
        return e.value, c.value

    def save(self):
        n = C.c_size_t(0)
        lib.edl_pipeline_save(self._h, None, 0, C.byref(n))      # asks for the size
        buf = np.empty(n.value, dtype=np.int64)
        _check(lib.edl_pipeline_save(self._h, buf.ctypes.data_as(_i64p), buf.size, C.byref(n)))
        return buf

    @classmethod
    def load(cls, image):
        image = np.ascontiguousarray(image, dtype=np.int64)
        h = C.c_void_p()
        _check(lib.edl_pipeline_load(image.ctypes.data_as(_i64p), image.size, C.byref(h)))
        return cls(_handle=h)

    def close(self):
        if self._h is not None:
            lib.edl_pipeline_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Job:
    """One elastic job on one GPU.  Allocates the arena with torch and hands
    raw pointers to the library."""

    def __init__(self, cfg, seed, device="cuda:0", stream=None, side_streams="library"):
        """side_streams: "library" (the handle makes its own two side streams, unless the option wgrad_stream
        is 0), "torch" (two torch.cuda.Stream objects of default priority made here and handed over), or None
        (everything on the job's stream)."""
        import torch
        self.torch = torch
        self.cfg = cfg
        self.sizes = edl_query(cfg)
        self.device = torch.device(device)
        self.arena = torch.empty(self.sizes.arena_bytes, dtype=torch.uint8, device=self.device)
        self.stream = stream
        sp = stream.cuda_stream if stream is not None else 0
        self._h = C.c_void_p()
        _check(lib.edl_init(C.byref(self._h), C.byref(cfg), seed, self.arena.data_ptr(), self.arena.numel(), sp))
        self.P, self.R = self.sizes.P, self.sizes.R
        self._data = None
        self._side = None
        if side_streams == "torch":
            self._side = (torch.cuda.Stream(device=self.device), torch.cuda.Stream(device=self.device))
            _check(lib.edl_set_side_streams(self._h, self._side[0].cuda_stream, self._side[1].cuda_stream))
        elif side_streams is None:
            _check(lib.edl_set_side_streams(self._h, None, None))

    def bind_dataset(self, x, y):
        """x: float32 [N,H,W,C] device tensor, y: int32 [N] device tensor."""
        assert x.is_contiguous() and y.is_contiguous()
        self._data = (x, y)
        _check(lib.edl_bind_dataset(self._h, x.data_ptr(), y.data_ptr(), x.shape[0]))

    def shard(self, B, p, epoch, step_in_epoch):
        idx = np.empty(B, dtype=np.int64)
        off = np.empty(p + 1, dtype=np.int64)
        _check(lib.edl_shard(self._h, B, p, epoch, step_in_epoch, idx.ctypes.data_as(_i64p), off.ctypes.data_as(_i64p)))
        return idx, off

    def _call_step(self, fn, p, idx, off, want_loss):
        loss = C.c_float()
        ip = idx.ctypes.data_as(_i64p) if idx is not None else None
        op = off.ctypes.data_as(_i64p) if off is not None else None
        _check(fn(self._h, p, ip, op, C.byref(loss) if want_loss else None))
        return loss.value if want_loss else None

    def step(self, p, idx=None, off=None, want_loss=True):
        return self._call_step(lib.edl_step, p, idx, off, want_loss)

    def step_static_scratch(self, p, idx=None, off=None, want_loss=True):
        return self._call_step(lib.edl_step_static_scratch, p, idx, off, want_loss)

    def gradients(self, p, idx=None, off=None, want_loss=True):
        return self._call_step(lib.edl_gradients, p, idx, off, want_loss)

    def apply(self, p):
        _check(lib.edl_apply(self._h, p))

    def snapshot(self, dst=None):
        if dst is None:
            dst = self.torch.empty(self.sizes.snapshot_bytes, dtype=self.torch.uint8, device=self.device)
        n = C.c_size_t()
        _check(lib.edl_snapshot(self._h, dst.data_ptr(), dst.numel(), C.byref(n)))
        return dst

    def restore(self, src):
        _check(lib.edl_restore(self._h, src.data_ptr(), src.numel()))

    def progress(self):
        pr = Progress()
        _check(lib.edl_get_progress(self._h, C.byref(pr)))
        return pr.step, pr.epoch, pr.step_in_epoch

    def _get(self, fn, n, *pre):
        out = np.empty(n, dtype=np.float32)
        _check(fn(self._h, *pre, out.ctypes.data_as(_f32p)))
        return out

    def params(self):
        return self._get(lib.edl_get_params, self.P)

    def momentum(self):
        return self._get(lib.edl_get_momentum, self.P)

    def second_moment(self):
        return self._get(lib.edl_get_second_moment, self.P)

    def running(self):
        return self._get(lib.edl_get_running, self.R)

    def grad(self, k):
        return self._get(lib.edl_get_grad, self.P, k)

    def grad_slice(self, k, off, size):
        """float32 host copy of G_k[off:off+size] (a view of the arena, no library call)."""
        self.sync()
        base = self.sizes.grads_off + 4 * (k * self.sizes.grad_stride + off)
        return self.arena[base:base + 4 * size].view(self.torch.float32).cpu().numpy()

    def losses(self, p):
        return self._get(lib.edl_get_losses, p, p)

    def set_params(self, w):
        w = np.ascontiguousarray(w, dtype=np.float32)
        _check(lib.edl_set_params(self._h, w.ctypes.data_as(_f32p)))

    def set_momentum(self, v):
        v = np.ascontiguousarray(v, dtype=np.float32)
        _check(lib.edl_set_momentum(self._h, v.ctypes.data_as(_f32p)))

    def set_second_moment(self, s):
        s = np.ascontiguousarray(s, dtype=np.float32)
        _check(lib.edl_set_second_moment(self._h, s.ctypes.data_as(_f32p)))

    # -- debugging hooks ---------------------------------------------------
    def debug_tensors(self):
        """[(H, W, C, alias_of)] for every activation tensor."""
        n = C.c_int32()
        _check(lib.edl_debug_tensor_count(self._h, C.byref(n)))
        out = []
        for t in range(n.value):
            H, W, Cc, al = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32()
            _check(lib.edl_debug_tensor_shape(self._h, t, C.byref(H), C.byref(W), C.byref(Cc), C.byref(al)))
            out.append((H.value, W.value, Cc.value, al.value))
        return out

    def debug_forward(self, idx):
        idx = np.ascontiguousarray(idx, dtype=np.int64)
        _check(lib.edl_debug_forward(self._h, idx.ctypes.data_as(_i64p), len(idx)))

    def debug_backward(self, n, k=0):
        _check(lib.edl_debug_backward(self._h, n, k))

    def debug_get(self, t, n, which=0):
        H, W, Cc, _ = self.debug_tensors()[t]
        out = np.empty((n, H, W, Cc), dtype=np.float32)
        _check(lib.edl_debug_get_tensor(self._h, t, which, n, out.ctypes.data_as(_f32p)))
        return out

    def debug_set(self, t, a, which=0):
        a = np.ascontiguousarray(a, dtype=np.float32)
        _check(lib.edl_debug_set_tensor(self._h, t, which, a.shape[0], a.ctypes.data_as(_f32p)))

    def debug_op_count(self):
        n = C.c_int32()
        _check(lib.edl_debug_op_count(self._h, C.byref(n)))
        return n.value

    def debug_forward_op(self, op, n):
        _check(lib.edl_debug_forward_op(self._h, op, n))

    def profile_parallelism(self, min_p, max_p, steps):
        """The scheduler's profile(min_p, max_p): list of dicts, largest parallelism first."""
        out = (ParallelismPoint * 64)()
        n = C.c_int32(0)
        _check(lib.edl_profile_parallelism(self._h, min_p, max_p, steps, C.cast(out, C.c_void_p), 64, C.byref(n)))
        return [dict(p=o.p, shard=o.shard, ms_per_step=o.ms_per_step, samples_per_s=o.samples_per_s,
                     worker_samples_per_s=o.worker_samples_per_s, efficiency=o.efficiency) for o in out[:n.value]]

    def debug_forward_range(self, op_lo, op_hi, n):
        _check(lib.edl_debug_forward_range(self._h, op_lo, op_hi, n))

    def debug_backward_op(self, op, n, k=0):
        _check(lib.edl_debug_backward_op(self._h, op, n, k))

    def debug_backward_range(self, op_lo, op_hi, n, k=0):
        _check(lib.edl_debug_backward_range(self._h, op_lo, op_hi, n, k))

    def debug_backward_range_from(self, op_lo, op_hi, n, held, k=0):
        arr = (C.c_int32 * len(held))(*held)
        _check(lib.edl_debug_backward_range_from(self._h, op_lo, op_hi, n, k, arr, len(held)))

    def debug_set_labels(self, labels):
        labels = np.ascontiguousarray(labels, dtype=np.int32)
        _check(lib.edl_debug_set_labels(self._h, labels.ctypes.data_as(C.POINTER(C.c_int32)), len(labels)))

    def sync(self):
        if self.stream is not None:
            self.stream.synchronize()
        else:
            self.torch.cuda.synchronize(self.device)

    def shutdown(self):
        if self._h:
            _check(lib.edl_shutdown(self._h))
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.shutdown()
        except Exception:
            pass
