#!/usr/bin/env python3
"""Benchmark of the elastic data-parallel training step on one MI355X.

    python bench.py --gpus 1 --steps 20 --warmup 3

A "step" is one pass of the whole hot path: shard assignment, gather + cast,
forward and backward of every worker's shard, aggregation of the p gradient
buffers fused with the momentum-SGD update.  The default workload is the one
the headline metric is quoted on: ResNet-50, bf16 activations with float32
master weights and momentum, one worker's shard of 32 samples of 224x224x3
synthetic N(0,1) images with 1000 uniform labels.  Inputs are resident in HBM
before the timed region.

Prints ONE JSON line.  Besides the contract fields it carries
  roofline      the kernel family that takes the most time in the step, timed with HIP
                events on the launch stream (the library's own profiling hooks)
  cpu_baseline  the CPU oracle, as it stands, timed on a bounded sample of the same workload
  update, snapshot   the HBM-bound parts of the metric on the VGG-16-sized state
                (138,357,544 parameters): achieved GB/s against the 8 TB/s peak; the update
                kernel is timed where it runs in use, at the end of VGG-16 training steps over
                p shards (`gbs`), and launched back to back on its own (`back_to_back_gbs`)
  kernels       per-family time, launches and achieved rate of one step
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
VGG16_P = 138357544

WORKLOADS = {
    # name: (model, dtype, N, B, p, geometry overrides, lr)
    "resnet50_bf16_b32": ("resnet50", "bf16", 1024, 32, 1, {}, 0.1),
    "vgg16_bf16_b32": ("vgg16", "bf16", 256, 32, 1, {}, 0.001),
    # the other networks of the paper's section 6
    "resnet101_bf16_b32": ("resnet50", "bf16", 256, 32, 1, dict(arch=(64, 3, 4, 23, 3)), 0.1),
    "resnet152_bf16_b32": ("resnet50", "bf16", 256, 32, 1, dict(arch=(64, 3, 8, 36, 3)), 0.1),
    "vgg19_bf16_b32": ("vgg16", "bf16", 256, 32, 1, dict(arch=(64, 4096, 2, 2, 4, 4, 4)), 0.001),
    "alexnet_bf16_b128": ("alexnet", "bf16", 512, 128, 1, {}, 0.001),
    "resnet20_f32_b128_p2": ("resnet20", "f32", 2048, 128, 2, {}, 0.1),
    "mlp_f32_b64_p4": ("mlp", "f32", 1024, 64, 4, {}, 0.1),
}
DEFAULT_HWC = {"mlp": (1, 1, 784, 10), "resnet20": (32, 32, 3, 10), "resnet50": (224, 224, 3, 1000),
               "vgg16": (224, 224, 3, 1000), "alexnet": (224, 224, 3, 1000)}


def kernel_sources_digest():
    """sha256 (first 16 hex digits) over the library's kernel and host sources: what a committed counter summary
    was taken from can be told apart from what is being timed now."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_1909_11985_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".cpp", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def committed_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of this workload
    (FETCH_SIZE and WRITE_SIZE scaled by the copy-kernel calibration), and where the figure comes from:
    (bytes or None, dict(file, kernel_sources_at_profile, kernel_sources_now, stale)).  The counters need
    rocprofv3 around the process, so they are not taken in this run; `stale` says whether the sources have
    changed since the summary was written."""
    rel = os.path.join("profiles", "%s_hbm_traffic.txt" % workload)
    value, at = None, None
    try:
        for line in open(os.path.join(ROOT, rel)):
            f = line.split()
            if len(f) >= 3 and f[0] == "traffic_bytes_per_launch" and f[1] == kernel:
                value = float(f[2])
            if len(f) >= 2 and f[0] == "kernel_sources_sha16":
                at = f[1]
    except OSError:
        return None, None
    now = kernel_sources_digest()
    return value, dict(file=rel, kernel_sources_at_profile=at, kernel_sources_now=now, stale=(at != now))


def run_elastic(args, np, torch, synth_inputs, E, make_config):
    """The elastic schedule of the fifth configuration: the aggregate batch stays 256 while the parallelism goes
    1 -> 2 -> 4 -> 8 -> 4; at every adjustment the state image a joining worker receives is taken and restored
    into a second job object (the joiner), which then takes the same step as the job it joined."""
    B, N = 256, 1024
    steps = args.steps if "--steps" in sys.argv else 10
    schedule = [1, 2, 4, 8, 4]
    x, y = synth_inputs.dataset(1, N, 224, 224, 3, 1000)
    cfg = make_config("resnet50", dtype="bf16", N=N, B=B, p_max=8, max_shard=B, lr=0.1)
    job = E.Job(cfg, 0)
    joiner = E.Job(cfg, 7)
    dx, dy = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()
    job.bind_dataset(dx, dy)
    joiner.bind_dataset(dx, dy)
    for _ in range(args.warmup):
        job.step(schedule[0], want_loss=False)
    job.sync()
    snap = torch.empty(job.sizes.snapshot_bytes, dtype=torch.uint8, device="cuda")
    phases = []
    t_all0 = time.perf_counter()
    for i, p in enumerate(schedule):
        snapshot_us = restore_us = None
        if i > 0:      # an adjustment: the joiner receives the model of one existing worker
            job.sync()
            t0 = time.perf_counter()
            job.snapshot(snap)
            job.sync()
            t1 = time.perf_counter()
            joiner.restore(snap)
            joiner.sync()
            t2 = time.perf_counter()
            snapshot_us, restore_us = (t1 - t0) * 1e6, (t2 - t1) * 1e6
            la, lb = job.step(p), joiner.step(p)          # both continue from the same state
            assert la == lb and joiner.progress() == job.progress(), "the joiner did not continue as the job it joined"
        t0 = time.perf_counter()
        for _ in range(steps):
            job.step(p, want_loss=False)
        job.sync()
        t1 = time.perf_counter()
        phases.append(dict(p=p, shard=B // p, steps=steps, ms_per_step=round((t1 - t0) * 1e3 / steps, 3),
                           samples_per_s=round(B * steps / (t1 - t0), 1),
                           snapshot_us=None if snapshot_us is None else round(snapshot_us, 1),
                           restore_us=None if restore_us is None else round(restore_us, 1)))
    job.sync()
    t_all1 = time.perf_counter()
    loss = job.step(schedule[-1])
    assert np.isfinite(loss), "training diverged"
    total_steps = steps * len(schedule) + (len(schedule) - 1)
    out = {
        "metric": "training samples/s per MI355X (ResNet-50 bf16); grad-avg+update HBM GB/s",
        "value": round(B * total_steps / (t_all1 - t_all0), 2), "unit": "samples/s", "n_gpus": 1, "steps": total_steps,
        "warmup": args.warmup, "ms_per_step": round((t_all1 - t_all0) * 1e3 / total_steps, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "resnet50_bf16_b256_elastic", "global_batch": B, "schedule": schedule, "steps_per_phase": steps,
                   "image": [224, 224, 3], "classes": 1000, "parameters": int(job.sizes.P), "dataset_samples": N,
                   "snapshot_bytes": int(job.sizes.snapshot_bytes)},
        "phases": phases,
    }
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="resnet50_bf16_b32", choices=sorted(WORKLOADS))
    ap.add_argument("--p", type=int, default=0, help="override the parallelism (shards of the global batch)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-state-bench", action="store_true", help="skip the VGG-16-sized update / snapshot timing")
    ap.add_argument("--no-in-step-update", action="store_true",
                    help="time the update kernel back to back only, not inside VGG-16 training steps (the counter "
                         "passes of the profiler use this: those steps add some 30,000 dispatches)")
    ap.add_argument("--elastic", action="store_true",
                    help="the elastic schedule instead: ResNet-50 bf16, global batch 256 as p = 1, 2, 4, 8, 4 shards, "
                         "--steps mini-batches per phase (10 if not given), a snapshot and a joiner's restore at every adjustment")
    ap.add_argument("--by-layer-shape", action="store_true",
                    help="name every contraction in the kernel list by its layer shape (one line per distinct shape, "
                         "none cut off) instead of by tile family; the roofline object then names the slowest shape")
    args = ap.parse_args()
    if args.by_layer_shape:
        os.environ["EDL_PROFILE_BY_SHAPE"] = "1"      # read by the library at its first contraction launch
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the p workers are shards of the batch on that GPU); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth_inputs
    import paper_1909_11985_amd as E
    from paper_1909_11985_amd.binding import make_config

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.elastic:
        run_elastic(args, np, torch, synth_inputs, E, make_config)
        return
    model, dtype, N, B, p, geom, lr = WORKLOADS[args.workload]
    if args.p:
        p = args.p
    H, W, C, classes = DEFAULT_HWC[model]
    x, y = synth_inputs.dataset(1, N, H, W, C, classes)
    cfg = make_config(model, dtype=dtype, N=N, B=B, p_max=max(p, 1), max_shard=B // p, lr=lr, **geom)
    job = E.Job(cfg, 0)
    dx, dy = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()
    job.bind_dataset(dx, dy)
    sizes = job.sizes

    for _ in range(args.warmup):
        job.step(p, want_loss=False)
    job.sync()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        job.step(p, want_loss=False)
    job.sync()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = B * args.steps / (t1 - t0)
    loss = job.step(p, want_loss=True)
    assert np.isfinite(loss), "training diverged"

    # ---- per-kernel timing (HIP events on the launch stream) ----
    # The timed steps above run the weight gradients on a second stream beside the
    # rest of the backward pass.  Per-kernel durations are taken with one kernel at
    # a time: a second job whose library keeps everything on one stream, timed
    # plainly first (one_stream_ms_per_step) and then with an event pair per launch.
    job.shutdown()
    del job
    job = E.Job(cfg, 0, side_streams=None)
    job.bind_dataset(dx, dy)
    for _ in range(2):
        job.step(p, want_loss=False)
    job.sync()
    cal_steps = max(3, args.steps // 2)
    tc0 = time.perf_counter()
    for _ in range(cal_steps):
        job.step(p, want_loss=False)
    job.sync()
    one_stream_ms = (time.perf_counter() - tc0) * 1e3 / cal_steps
    prof_steps = 3
    E.edl_profile(True)
    for _ in range(prof_steps):
        job.step(p, want_loss=False)
    job.sync()
    rep = E.edl_profile_report()
    E.edl_profile(False)
    # An event pair reads longer than the kernel it brackets (the events' own
    # dispatch).  The plain one-stream steps keep the stream saturated (rocprofv3's
    # kernel durations add up to the same step time), so what the pairs add is the
    # bracketed total minus the plain step time, shared equally over the launches.
    rep = [r for r in rep if not r["name"].startswith("_")]
    launches = sum(r["launches"] for r in rep)
    raw_ms = sum(r["ms"] for r in rep)
    overhead_ms = max(0.0, (raw_ms / prof_steps - one_stream_ms) * prof_steps / max(launches, 1))
    for r in rep:
        r["ms_raw"] = r["ms"]
        r["ms"] = max(r["ms"] - overhead_ms * r["launches"], 0.05 * r["ms"])
    kernels = []
    for r in rep:
        ms = r["ms"] / prof_steps
        k = dict(name=r["name"], launches_per_step=r["launches"] / prof_steps, ms_per_step=round(ms, 4),
                 avg_launch_us=round(1e3 * r["ms"] / max(r["launches"], 1), 2))
        if r["flops"] > 0:
            k["tflops"] = round(r["flops"] / r["ms"] / 1e9, 2)
        k["gbs"] = round(r["bytes"] / r["ms"] / 1e6, 1)
        kernels.append(k)
    kernels.sort(key=lambda k: -k["ms_per_step"])
    dom = max(rep, key=lambda r: r["ms"])
    if dom["flops"] > 0:
        achieved = dom["flops"] / dom["ms"] / 1e9
        peak = MFMA_PEAK_TFLOPS[dtype]
        roofline = dict(bound="mfma", kernel=dom["name"], achieved=round(achieved, 2), peak=peak, unit="TFLOP/s",
                        frac=round(achieved / peak, 4), traffic=None,
                        avg_launch_us=round(1e3 * dom["ms"] / dom["launches"], 2),
                        launches_per_step=dom["launches"] / prof_steps)
    else:
        achieved = dom["bytes"] / dom["ms"] / 1e6
        roofline = dict(bound="hbm", kernel=dom["name"], achieved=round(achieved, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=round(achieved / HBM_PEAK_GBS, 4), traffic=None,
                        avg_launch_us=round(1e3 * dom["ms"] / dom["launches"], 2),
                        launches_per_step=dom["launches"] / prof_steps)
    roofline["event_pair_overhead_us"] = round(1e3 * overhead_ms, 2)
    roofline["traffic"], roofline["traffic_source"] = committed_traffic(args.workload, roofline["kernel"])
    conv_ms = sum(r["ms"] for r in rep if r["flops"] > 0) / prof_steps
    conv_flops = sum(r["flops"] for r in rep if r["flops"] > 0) / prof_steps
    step_summary = dict(
        flops_per_sample=sizes.flops_per_sample,
        step_tflops=round(sizes.flops_per_sample * B / (ms_per_step * 1e-3) / 1e12, 2),
        step_frac_of_mfma_peak=round(sizes.flops_per_sample * B / (ms_per_step * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS[dtype], 4),
        contraction_ms_per_step=round(conv_ms, 3),
        contraction_tflops=round(conv_flops / max(conv_ms, 1e-9) / 1e9, 2),
        kernel_ms_per_step=round(sum(r["ms"] for r in rep) / prof_steps, 3),
        one_stream_ms_per_step=round(one_stream_ms, 4))

    # ---- the HBM-bound half of the metric on the VGG-16-sized state ----
    update, snapshot, attainable = None, None, None
    job_P = sizes.P
    job.shutdown()
    del job
    if not args.no_state_bench:
        P = VGG16_P
        update = []
        # the state arrays lie where a VGG-16 job of up to 8 shards has them in its arena (edl_query's offsets)
        lays = {opt: E.edl_query(make_config("vgg16", dtype="bf16", N=8, B=8, p_max=8, max_shard=1, optimizer=opt))
                for opt in ("momentum", "adam")}
        state_end = max(max(l.params_off, l.momentum_off, l.second_off, l.shadow_off, l.grads_off + 4 * l.grad_stride * 7)
                        for l in lays.values()) + 4 * P
        pool = torch.empty(state_end + 8192, dtype=torch.uint8, device="cuda")
        pool0 = (-pool.data_ptr()) % 8192              # the arena starts on an 8 KB boundary
        w0 = torch.from_numpy(synth_inputs.vector(4, P))
        g0 = torch.from_numpy(synth_inputs.gradient_buffers(3, 1, P)[0])

        def state_views(lay):
            assert lay.P == P

            def view(off, dtype):
                return pool[pool0 + off: pool0 + off + P * dtype.itemsize].view(dtype)

            w, v, w16 = view(lay.params_off, torch.float32), view(lay.momentum_off, torch.float32), view(lay.shadow_off, torch.bfloat16)
            s2 = view(lay.second_off, torch.float32) if lay.second_off >= 0 else None
            grads = [view(lay.grads_off + 4 * lay.grad_stride * k, torch.float32) for k in range(8)]
            w.copy_(w0)
            v.zero_()
            if s2 is not None:
                s2.zero_()
            for g in grads:
                g.copy_(g0)
            return w, v, s2, w16, grads

        def timed(name, launch, reps=10):
            """GB/s of the kernel `name` over `reps` launches (HIP events on the launch stream, pair overhead taken off)"""
            torch.cuda.synchronize()
            E.edl_profile(True)
            for i in range(reps):
                launch(i)
            torch.cuda.synchronize()
            rr = E.edl_profile_report()
            E.edl_profile(False)
            r = [q for q in rr if q["name"] == name][0]
            ms = r["ms"] - overhead_ms * r["launches"]
            return r["bytes"] / ms / 1e6, 1e3 * ms / r["launches"]

        # launched back to back on their own (every launch starts while the previous one's stores are still on
        # their way to memory: the lower of the two figures) ...
        alone = {}
        w, v, _, w16, grads = state_views(lays["momentum"])
        for pp in (1, 2, 4, 8):
            for _ in range(2):
                E.edl_average_update(grads[:pp], w, v, w16, 0.01, 0.9, 5e-4)
            alone[("momentum", pp)] = timed("average_update", lambda i: E.edl_average_update(grads[:pp], w, v, w16, 0.01, 0.9, 5e-4))[0]
        w, v, s2, w16, grads = state_views(lays["adam"])
        for pp in (1, 8):
            for t in (1, 2):
                E.edl_adam_update(grads[:pp], w, v, s2, w16, 0.001, 0.9, 0.999, 1e-8, 5e-4, t)
            alone[("adam", pp)] = timed("adam_update", lambda i: E.edl_adam_update(grads[:pp], w, v, s2, w16, 0.001, 0.9, 0.999, 1e-8, 5e-4, 3 + i))[0]
        del grads, s2, w, v, w16, pool
        # ... and where the kernel runs in use: at the end of VGG-16 training steps over p shards of 32 / p samples
        # (one stream, so that an event pair brackets one kernel)
        vx, vy = synth_inputs.dataset(1, 64, 224, 224, 3, 1000)
        vdx, vdy = torch.from_numpy(vx).cuda(), torch.from_numpy(vy).cuda()
        legs = (("momentum", "average_update", (1, 2, 4, 8), 18), ("adam", "adam_update", (1, 8), 26))
        if args.no_in_step_update:
            for opt, kernel, ps, extra in legs:
                for pp in ps:
                    gbs = alone[(opt, pp)]
                    row = dict(p=pp, P=P, bytes_per_param=4 * pp + extra, us=round((4 * pp + extra) * P / gbs / 1e3, 1),
                               gbs=round(gbs, 1), frac_of_hbm_peak=round(gbs / HBM_PEAK_GBS, 4), where="back to back, on its own")
                    update.append(dict(optimizer="adam", **row) if opt == "adam" else row)
            legs = ()
        for opt, kernel, ps, extra in legs:
            vjob = E.Job(make_config("vgg16", dtype="bf16", N=64, B=32, p_max=8, max_shard=32, lr=0.001, optimizer=opt), 0,
                         side_streams=None)
            vjob.bind_dataset(vdx, vdy)
            for pp in ps:
                for _ in range(2):
                    vjob.step(pp, want_loss=False)
                gbs, us = timed(kernel, lambda i: vjob.step(pp, want_loss=False), reps=6)
                row = dict(p=pp, P=P, bytes_per_param=4 * pp + extra, us=round(us, 1), gbs=round(gbs, 1),
                           frac_of_hbm_peak=round(gbs / HBM_PEAK_GBS, 4), where="end of a VGG-16 step, shards of %d" % (32 // pp),
                           back_to_back_gbs=round(alone[(opt, pp)], 1))
                if opt == "adam":
                    row = dict(optimizer="adam", **row)
                update.append(row)
            vjob.shutdown()
            del vjob
        del vdx, vdy
        nbytes = 8 * P
        src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        for _ in range(2):
            E.edl_copy(dst, src, nbytes)
        torch.cuda.synchronize()
        E.edl_profile(True)
        for _ in range(10):
            E.edl_copy(dst, src, nbytes)
        torch.cuda.synchronize()
        rr = E.edl_profile_report()
        r = [q for q in rr if q["name"] == "copy"][0]
        r["ms"] -= overhead_ms * r["launches"]
        E.edl_profile(False)
        gbs = r["bytes"] / r["ms"] / 1e6
        snapshot = dict(state_bytes=nbytes, us=round(1e3 * r["ms"] / r["launches"], 1), gbs=round(gbs, 1),
                        frac_of_hbm_peak=round(gbs / HBM_PEAK_GBS, 4))
        del src, dst
        # attainable matrix rate: register-resident MFMA loop in the workload's matrix instruction
        sink = torch.zeros(1, device="cuda")
        E.edl_mfma_rate(dtype, 256 * 8, 2000, sink)
        torch.cuda.synchronize()
        E.edl_profile(True)
        for _ in range(3):
            E.edl_mfma_rate(dtype, 256 * 8, 20000, sink)
        torch.cuda.synchronize()
        rr = E.edl_profile_report()
        E.edl_profile(False)
        r = [q for q in rr if q["name"].startswith("mfma_rate")][0]
        attainable = dict(mfma_tflops=round(r["flops"] / (r["ms"] - overhead_ms * r["launches"]) / 1e9, 1),
                          mfma_peak_tflops=MFMA_PEAK_TFLOPS[dtype], copy_gbs=snapshot["gbs"], hbm_peak_gbs=HBM_PEAK_GBS)

    # ---- the oracle on the host cores, on a bounded sample of the same workload ----
    # The same unit of work as `value`: whole steps (shard assignment, forward and backward of every shard,
    # aggregation + update) of the oracle as it stands.  One small warm-up pass (pages the data in), then
    # `cpu_steps` timed steps on shards of n_cpu samples; for the default workload n_cpu is the benchmark's
    # own shard of 32, for the heavier or lighter ones a size that keeps this leg to about half a minute.
    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import oracle as O
        n_cpu = {"resnet50": 32, "vgg16": 8, "alexnet": 32, "resnet20": B // p, "mlp": B // p}[model]
        cpu_steps = 2
        gkw = {}
        if model == "resnet50" and "arch" in geom:
            gkw = dict(blocks=tuple(geom["arch"][1:5]))
            n_cpu = 8
        if model == "vgg16" and "arch" in geom:
            gkw = dict(groups=tuple(geom["arch"][2:7]))
        p_cpu = p if n_cpu == B // p else 1
        B_cpu = n_cpu * p_cpu
        orc = O.Oracle(model, 0, N - N % B_cpu, B_cpu, lr=lr, graph_kwargs=gkw)
        orc.forward_backward(x[:2].astype(np.float64), y[:2])
        tc0 = time.perf_counter()
        for _ in range(cpu_steps):
            cl = orc.step(p_cpu, x, y)
        tc1 = time.perf_counter()
        assert np.isfinite(cl)
        threads = os.environ.get("OMP_NUM_THREADS")
        cores = int(threads) if threads else (os.cpu_count() or 1)
        cpu_baseline = dict(value=round(B_cpu * cpu_steps / (tc1 - tc0), 3), unit="samples/s", cores=cores, kind="oracle",
                            omp_num_threads=threads, host_cpus=os.cpu_count(),
                            sample="%d whole steps (forward, backward, aggregation + update) at p = %d on shards of %d samples "
                                   "of the same workload, after a 2-sample warm-up pass (%.1f s)"
                                   % (cpu_steps, p_cpu, n_cpu, tc1 - tc0))

    out = {
        "metric": "training samples/s per MI355X (ResNet-50 bf16); grad-avg+update HBM GB/s",
        "value": round(value, 2), "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": args.workload, "global_batch": B, "p": p, "shard": B // p, "image": [H, W, C],
                   "classes": classes, "parameters": job_P, "dataset_samples": N},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "step": step_summary,
        "update": update, "snapshot": snapshot, "attainable": attainable, "kernels": kernels if args.by_layer_shape else kernels[:24],
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
