"""Benchmark of the DSSP hot path on one MI355X.

Workload (default): ResNet-110 for CIFAR-shaped synthetic data, batch 128, 8 virtual workers dealt onto one
HIP stream per hardware queue (by their push rates, so that every stream carries the same share), DSSP s_L = 3,
r_max = 12, lr 0.05, heterogeneous seeded iteration times.
One "step" = one push travelling the whole path: pull -> forward/backward -> push -> apply ->
decision.  Order of a run: untimed set-up (buffers, and every worker step's HIP graph built, so that the run does not
depend on how long the warm-up is), --warmup untimed pushes of the schedule, then --windows (3) consecutive windows of
exactly --steps pushes each; `value` is the median window, `windows_pushes_per_s` lists all of them.
Prints one JSON line: metric, value (pushes/s), ms_per_step, config, roofline (dominant kernel),
roofline_others, one_stream_per_worker (the same run with K streams instead of one per hardware queue),
cpu_baseline (the CPU oracle on the first pushes of the same schedule).

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet110|resnet50|alexnet_ds|alexnet_3c|mlp|stress]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

WORKER_STREAMS = 0      # HIP streams the virtual workers are dealt onto; 0: one per hardware queue, each on a queue
                        # of its own (measured: 327 pushes/s, as with two streams per queue; 291 with eight
                        # streams as the runtime happens to deal them, 1, 2, 2 and 3 to a queue)


def workload(name):
    """-> dict(model, config, K, s_L, r_max, lr, batch, n_classes, pool)"""
    if name == "resnet110":
        return dict(model="resnet110", config=4, K=8, s_L=3, r_max=12, lr=0.05, batch=128, n_classes=100, pool=8)
    if name == "resnet50":       # the paper's other residual network (Sec. V-A3), same 6n+2 family
        return dict(model="resnet50", config=4, K=8, s_L=3, r_max=12, lr=0.05, batch=128, n_classes=100, pool=8)
    if name == "alexnet_ds":
        return dict(model="alexnet_ds", config=2, K=4, s_L=3, r_max=12, lr=0.001, batch=128, n_classes=10, pool=16)
    if name == "alexnet_3c":     # Sec. V-A3's reduced AlexNet with three convolutional and two fully connected layers
        return dict(model="alexnet_3c", config=2, K=4, s_L=3, r_max=12, lr=0.001, batch=128, n_classes=10, pool=16)
    if name == "mlp":
        return dict(model="mlp", config=1, K=4, s_L=3, r_max=4, lr=0.01, batch=32, n_classes=10, pool=50)
    if name == "stress":
        return dict(model="none", config=5, K=16, s_L=3, r_max=15, lr=0.01, batch=0, n_classes=0, pool=0, n=25_000_000)
    raise SystemExit("unknown workload " + name)


EXPECTED_QUEUES = int(os.environ.get("GPU_MAX_HW_QUEUES", "4"))    # hardware queues of a process (HIP's default: 4)


def build_emulation(wl, d, worker_streams, by_rate=True):
    from paper_1908_11848_amd import binding as B, inputs
    from paper_1908_11848_amd.emulation import Emulation
    K = wl["K"]
    if wl["model"] == "none":
        n = wl["n"]
        return Emulation("none", K, wl["s_L"], wl["r_max"], wl["lr"], inputs.stress_weights(n),
                         grads=inputs.stress_grads(K, n)), n
    segs = B.dssp_model_segments(B.model_id(wl["model"]), wl["n_classes"])
    w0 = inputs.init_weights(segs, wl["config"])
    xs, ys = inputs.batches(wl["config"], K, wl["pool"], wl["batch"], wl["n_classes"])
    rates = [1.0 / float(np.mean(row)) for row in d]         # a worker that iterates twice as fast pushes twice as often
    em = Emulation(wl["model"], K, wl["s_L"], wl["r_max"], wl["lr"], w0, wl["batch"], wl["n_classes"], xs, ys,
                   worker_streams=worker_streams, rates=rates if by_rate else None)
    return em, int(w0.size)


def prepare_graphs(em, wl):
    """Untimed set-up: every (worker, mini-batch buffer) pair is stepped twice, so that its launch sequence has run
    once as individual launches and once as the capture of its HIP graph; every step of the run itself, warm-up
    included, is then a graph replay - the path the library takes in steady state."""
    from paper_1908_11848_amd import binding as B
    if wl["model"] == "none":
        return 0
    for p in range(wl["K"]):
        B.dssp_pull(em.ctx, p, em.w_local[p])
    for rep in range(2):
        for j in range(wl["pool"]):
            for p in range(wl["K"]):
                em.step(p, j)
    em.synchronize()
    return 2 * wl["pool"] * wl["K"]


def timed_windows(em, d, warmup, steps, n_windows):
    """warmup untimed pushes of the schedule, then n_windows consecutive windows of exactly `steps` pushes each, every
    window bracketed by a synchronisation of all streams.  -> seconds per window."""
    import torch
    sched = em.schedule(d, log=False, fused_pull=True)   # the pull of a worker granted OK by its own push rides in the apply kernel
    sched.advance(warmup)
    times = []
    for _ in range(n_windows):
        em.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        done = sched.advance(steps)
        em.synchronize()
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t0)
        assert done == steps
    return times


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="resnet110")
    ap.add_argument("--windows", type=int, default=3, help="consecutive timed windows of --steps pushes; the median is reported")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-roofline", action="store_true")
    ap.add_argument("--no-placement-comparison", action="store_true")
    ap.add_argument("--worker-streams", type=int, default=WORKER_STREAMS)
    ap.add_argument("--allow-queue-mismatch", action="store_true",
                    help="go on when the stream probe does not find the expected number of hardware queues")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        raise SystemExit("bench.py: the K workers are emulated on ONE GPU; run it with --gpus 1 "
                         "(no multi-GPU figure exists)")
    import torch
    from paper_1908_11848_amd.emulation import Emulation
    from paper_1908_11848_amd import roofline

    wl = workload(a.workload)
    K = wl["K"]
    total = a.warmup + a.windows * a.steps
    from paper_1908_11848_amd import inputs
    d = inputs.durations(wl["config"], K, total + 8)
    em, n = build_emulation(wl, d, a.worker_streams)
    if em.hardware_queues != EXPECTED_QUEUES and not a.allow_queue_mismatch:
        # the placement (one stream per hardware queue, the same number of workers on each) rests on this probe: a wrong
        # grouping would cost about a tenth of the throughput without any other sign
        Emulation._spread.clear()
        em.close()
        em, n = build_emulation(wl, d, a.worker_streams)
        if em.hardware_queues != EXPECTED_QUEUES:
            raise SystemExit("bench.py: the stream probe found %d hardware queues twice, %d expected (GPU_MAX_HW_QUEUES or "
                             "HIP's default); the worker placement would not be the measured one.  Re-run, or pass "
                             "--allow-queue-mismatch to time whatever placement results." % (em.hardware_queues, EXPECTED_QUEUES))
    prepared = prepare_graphs(em, wl)
    times = timed_windows(em, d, a.warmup, a.steps, a.windows)
    dt = float(np.median(times))
    pushes_per_s = a.steps / dt
    finite = bool(np.isfinite(em.weights()).all())

    out = {
        "metric": "server pushes/s + train img/s (ResNet-110, 8 virtual workers, DSSP)" if a.workload == "resnet110"
                  else "server pushes/s (%s)" % a.workload,
        "value": round(pushes_per_s, 2), "unit": "pushes/s",
        "train_img_per_s": round(pushes_per_s * wl["batch"], 1),
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(1e3 * dt / a.steps, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s, batch %d, %d virtual workers, DSSP s_L=%d r_max=%d, %d params"
                               % (wl["model"], wl["batch"], K, wl["s_L"], wl["r_max"], n),
                   "worker_streams": len(set(em.streams[:K])), "hardware_queues": em.hardware_queues},
        "windows_pushes_per_s": [round(a.steps / t, 2) for t in times],      # value = their median
        "graph_steps_prepared_untimed": prepared,
        "weights_finite": finite,
    }
    if not a.no_roofline:
        out["roofline"], out["roofline_others"] = roofline.measure(a.workload, em)
    em.close()
    del em
    if wl["model"] != "none" and not a.no_placement_comparison and not a.worker_streams:
        # the same run with every virtual worker on a HIP stream of its own (K streams dealt onto the hardware queues by
        # the runtime), for comparison with the default placement above
        em2, _ = build_emulation(wl, d, K, by_rate=False)
        prepare_graphs(em2, wl)
        t2 = timed_windows(em2, d, a.warmup, a.steps, 1)[0]
        out["one_stream_per_worker"] = {"value": round(a.steps / t2, 2), "unit": "pushes/s", "worker_streams": len(set(em2.streams[:K]))}
        em2.close()
        del em2
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(a.workload, wl)
    print(json.dumps(out), flush=True)


def cpu_baseline(name, wl):
    """The oracle, as it stands, on this machine's host cores, on a bounded sample of the workload."""
    from oracle import build, nn, ps
    from paper_1908_11848_amd import binding as B, inputs
    if not os.path.exists(os.path.join(ROOT, "oracle", "liboracle_nn.so")):
        build.build()
    K = wl["K"]
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    if wl["model"] == "none":
        n, sample = wl["n"], 40
        d = inputs.durations(5, K, sample + 8)
        g = inputs.stress_grads(K, n)
        t0 = time.perf_counter()
        ps.run(K, wl["s_L"], wl["r_max"], wl["lr"], inputs.stress_weights(n), d, lambda p, i, w: (0.0, g[p]), total=sample)
        dt = time.perf_counter() - t0
        return {"value": round(sample / dt, 3), "unit": "pushes/s", "cores": 1, "kind": "oracle",
                "sample": "first %d pushes of the same schedule (numpy fp64 apply + snapshot copies)" % sample}
    sample = {"resnet110": 8, "resnet50": 16, "alexnet_ds": 48, "alexnet_3c": 48, "mlp": 200}[name]
    net = nn.make_net(wl["model"], wl["n_classes"])
    w0 = inputs.init_weights(B.dssp_model_segments(B.model_id(wl["model"]), wl["n_classes"]), wl["config"])
    xs, ys = inputs.batches(wl["config"], K, 1, wl["batch"], wl["n_classes"])
    d = inputs.durations(wl["config"], K, sample + 8)
    t0 = time.perf_counter()
    ps.run(K, wl["s_L"], wl["r_max"], wl["lr"], w0, d, ps.model_grad_fn(net, xs, ys), total=sample)
    dt = time.perf_counter() - t0
    return {"value": round(sample / dt, 4), "unit": "pushes/s", "img_per_s": round(sample * wl["batch"] / dt, 2),
            "cores": cores, "kind": "oracle",
            "sample": "first %d pushes of the same schedule (fp64 direct-loop forward/backward, OpenMP)" % sample}


if __name__ == "__main__":
    main()
