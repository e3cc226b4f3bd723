"""Benchmark of the DSSP hot path on one MI355X.

Workload (default): ResNet-110 for CIFAR-shaped synthetic data, batch 128, 8 virtual workers dealt onto one
HIP stream per hardware queue (by their push rates, so that every stream carries the same share), DSSP s_L = 3,
r_max = 12, lr 0.05, heterogeneous seeded iteration times.
One "step" = one push travelling the whole path: pull -> forward/backward -> push -> apply ->
decision.  Prints one JSON line: metric, value (pushes/s), ms_per_step, config, roofline (dominant kernel),
roofline_others, cpu_baseline (the CPU oracle on the first pushes of the same schedule).

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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=160)
    ap.add_argument("--workload", default="resnet110")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-roofline", action="store_true")
    ap.add_argument("--worker-streams", type=int, default=WORKER_STREAMS)
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        raise SystemExit("bench.py: the K workers are emulated on ONE GPU; run it with --gpus 1 "
                         "(no multi-GPU figure exists)")
    import torch
    from paper_1908_11848_amd import binding as B, inputs
    from paper_1908_11848_amd.emulation import Emulation
    from paper_1908_11848_amd import roofline

    wl = workload(a.workload)
    K = wl["K"]
    total = a.steps + a.warmup
    d = inputs.durations(wl["config"], K, total + 8)
    if wl["model"] == "none":
        n = wl["n"]
        em = Emulation("none", K, wl["s_L"], wl["r_max"], wl["lr"], inputs.stress_weights(n),
                       grads=inputs.stress_grads(K, n))
    else:
        segs = B.dssp_model_segments(B.model_id(wl["model"]), wl["n_classes"])
        w0 = inputs.init_weights(segs, wl["config"])
        xs, ys = inputs.batches(wl["config"], K, wl["pool"], wl["batch"], wl["n_classes"])
        rates = [1.0 / float(np.mean(row)) for row in d]         # a worker that iterates twice as fast pushes twice as often
        em = Emulation(wl["model"], K, wl["s_L"], wl["r_max"], wl["lr"], w0, wl["batch"], wl["n_classes"], xs, ys,
                       worker_streams=a.worker_streams, rates=rates)
        n = int(w0.size)
    sched = em.schedule(d, log=False, fused_pull=True)       # the pull of a worker granted OK by its own push rides in the apply kernel
    sched.advance(a.warmup)
    em.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    done = sched.advance(a.steps)
    em.synchronize()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    assert done == a.steps
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
        "weights_finite": finite,
    }
    if not a.no_roofline:
        out["roofline"], out["roofline_others"] = roofline.measure(a.workload, em)
    em.close()
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
    sample = {"resnet110": 3, "resnet50": 6, "alexnet_ds": 16, "alexnet_3c": 16, "mlp": 200}[name]
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
