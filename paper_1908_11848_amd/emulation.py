"""One emulated DSSP cluster on one GPU: device buffers and streams (through torch, which is
used for nothing else), the library context, and the virtual-time schedule.

Every arithmetic step runs inside libdssp (pull, worker gradient, apply, decisions); this class
only owns memory and calls the C ABI through `binding`.
"""
import numpy as np
import torch

from . import binding as B
from . import driver


def deal(rates, n_lanes):
    """Lane of each worker such that the lanes' sums of rates are about equal (longest processing time first)."""
    load = [0.0] * n_lanes
    lane_of = [0] * len(rates)
    for p in sorted(range(len(rates)), key=lambda p: (-rates[p], p)):
        lane = min(range(n_lanes), key=lambda l: (load[l], l))
        lane_of[p] = lane
        load[lane] += rates[p]
    return lane_of


class Emulation:
    def __init__(self, model, K, s_L, r_max, lr, w0, batch=0, n_classes=0, xs=None, ys=None, grads=None,
                 device="cuda:0", worker_streams=None, server_stream=False, rates=None):
        """model: 'mlp' | 'alexnet_ds' | 'resnet<d>' | 'none'.
        w0: float32 initial weights.  xs[p][j] / ys[p][j]: pool of mini-batches of worker p
        (cycled); grads[p]: fixed gradient buffers for model 'none' (server stress).
        worker_streams: number of HIP streams the K workers are dealt onto (worker p -> stream p mod
        that number).  Default: one stream per hardware queue, each on a queue of its own (found with
        dssp_stream_queues), since streams that share a queue run one after the other anyway and an
        uneven spread of the workers over the queues costs throughput.  A given number of streams is
        spread over the queues as evenly as they allow.  Ordering between workers goes through the
        library's events either way, so results do not depend on it.
        rates: expected pushes per unit time of each worker (any scale).  Given them, the workers are dealt onto
        the streams so that every stream gets about the same share of the work (greedily, fastest worker first,
        each to the stream with the smallest sum so far) instead of round-robin.
        server_stream: give the server's applies a stream of their own instead of the pusher's (same results;
        slower when that stream shares a hardware queue with a worker's)."""
        if not torch.cuda.is_available():
            raise RuntimeError("a GPU is required")
        B.lib()
        self.dev = torch.device(device)
        torch.cuda.set_device(self.dev)
        self.model, self.mid = model, B.model_id(model)
        self.K, self.batch, self.n_classes = K, batch, n_classes
        n = int(np.asarray(w0).size)
        self.n = n
        self.w = torch.from_numpy(np.ascontiguousarray(w0, dtype=np.float32)).to(self.dev)
        # one row per worker; rows start 256-byte aligned (the library moves 16-byte vectors)
        pitch = (n + 63) // 64 * 64
        self.w_local = torch.empty((K, pitch), dtype=torch.float32, device=self.dev)[:, :n]
        self.grad = torch.zeros((K, pitch), dtype=torch.float32, device=self.dev)[:, :n]
        if grads is not None:
            for p in range(K):
                self.grad[p].copy_(torch.from_numpy(np.ascontiguousarray(grads[p], dtype=np.float32)))
        self.loss = torch.zeros(K, dtype=torch.float32, device=self.dev)
        lanes, self.hardware_queues = self._lanes(K, worker_streams)
        self.lane_of = deal(rates, len(lanes)) if rates is not None else [p % len(lanes) for p in range(K)]
        self.streams = [lanes[self.lane_of[p]] for p in range(K)]
        self.ctx = B.dssp_create(self.w, n, K, s_L, r_max, lr)
        if server_stream:
            self.streams.append(torch.cuda.Stream(device=self.dev))
            B.dssp_set_stream(self.ctx, -1, self.streams[K])
        for p in range(K):
            B.dssp_set_stream(self.ctx, p, self.streams[p])
        self.ws = None
        if self.mid != B.DSSP_MODEL_NONE:
            nbytes = B.dssp_workspace_bytes(self.mid, batch, n_classes, K)
            self.ws = torch.empty(nbytes, dtype=torch.uint8, device=self.dev)
            B.dssp_set_model(self.ctx, self.mid, batch, n_classes, self.ws, nbytes)
            self.xs = [[torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(self.dev) for x in row] for row in xs]
            self.ys = [[torch.from_numpy(np.ascontiguousarray(y, dtype=np.int32)).to(self.dev) for y in row] for row in ys]
        torch.cuda.synchronize()
        self.on_step = None            # test hook: called after a worker step was enqueued
        self.before_step = None        # test hook: called after the pull, before the step is enqueued

    _spread = {}        # device index -> (streams ordered so that any prefix is spread evenly over the queues, queues)

    def _lanes(self, K, worker_streams):
        """Streams for the workers, out of torch's pool.  The pool lives as long as the process, so it is probed once."""
        key = self.dev.index or 0
        if key not in Emulation._spread:
            cand = [torch.cuda.Stream(device=self.dev) for _ in range(16)]
            queue, nq = B.dssp_stream_queues(cand)
            by_queue = [[s for s, q in zip(cand, queue) if q == g] for g in range(nq)]
            order = [row[depth] for depth in range(len(cand)) for row in by_queue if depth < len(row)]
            Emulation._spread[key] = (order, nq)
        order, nq = Emulation._spread[key]
        want = min(K, nq) if not worker_streams else max(1, min(K, len(order), int(worker_streams)))
        return order[:want], nq

    # ------------------------------------------------------------------ pieces
    def step(self, p, n):
        """Enqueue worker p's n-th iteration (n from 0) on its stream."""
        if self.mid == B.DSSP_MODEL_NONE:
            return
        j = n % len(self.xs[p])
        if self.before_step:
            self.before_step(p, n)
        B.dssp_worker_step(self.ctx, p, self.xs[p][j], self.ys[p][j], self.w_local[p], self.grad[p],
                           self.loss[p:p + 1])
        if self.on_step:
            self.on_step(p, n)

    def run(self, durations, quota=None, total=None, log=True, fused_pull=False, aggregate=False):
        """fused_pull: a worker granted OK by its own push takes its snapshot from the apply kernel (dssp_push_pull).
        aggregate: pushes that share a timestamp are applied by one kernel (dssp_push_many)."""
        out = driver.run_schedule(self.ctx, self.K, durations, quota=quota, total=total,
                                  grad_ptr=lambda p: self.grad[p], pull_dst=lambda p: self.w_local[p],
                                  step=self.step, log=log, fused_pull=fused_pull, aggregate=aggregate)
        return out

    def schedule(self, durations, quota=None, log=True, fused_pull=False, aggregate=False):
        """Resumable form of run(): returns a driver.Schedule (all workers pulled and started)."""
        return driver.Schedule(self.ctx, self.K, durations, quota=quota, grad_ptr=lambda p: self.grad[p],
                               pull_dst=lambda p: self.w_local[p], step=self.step, log=log, fused_pull=fused_pull,
                               aggregate=aggregate)

    def run_wallclock_device(self, total, slowdown=None):
        """Runs `total` pushes with the controller fed by the DEVICE's clock (driver.run_wallclock_device): every
        iteration is timed on its stream, and worker p's stream is held until the iteration has lasted slowdown[p]
        times its real duration (1.0: not at all), which makes the emulated cluster heterogeneous (Sec. V-C).
        Returns (log, stats)."""
        permille = [int(round(1000 * f)) for f in (slowdown or [1.0] * self.K)]

        def step_timed(p, n):
            j = n % len(self.xs[p])
            if self.before_step:
                self.before_step(p, n)
            B.dssp_worker_step_timed(self.ctx, p, self.xs[p][j], self.ys[p][j], self.w_local[p], self.grad[p],
                                     self.loss[p:p + 1], permille[p])
            if self.on_step:
                self.on_step(p, n)

        return driver.run_wallclock_device(self.ctx, self.K, total, grad_ptr=lambda p: self.grad[p],
                                           pull_dst=lambda p: self.w_local[p], step_timed=step_timed)

    def run_wallclock(self, total, min_iteration_us=None):
        """Runs `total` pushes with the controller fed by real completion times (driver.run_wallclock).
        min_iteration_us[p]: an iteration of worker p counts as finished only once the device is done with it AND
        that many microseconds have passed since it started, which makes the emulated cluster heterogeneous without
        occupying a hardware queue (streams that share one would slow each other down).  Returns (log, stats)."""
        import time
        evs = [torch.cuda.Event() for _ in range(self.K)]
        t_start = [0] * self.K
        floor_ns = [int(1000 * u) for u in (min_iteration_us or [0] * self.K)]

        def step(p, n):
            t_start[p] = time.perf_counter_ns()
            self.step(p, n)
            evs[p].record(self.streams[p])

        def done(p):
            return time.perf_counter_ns() - t_start[p] >= floor_ns[p] and evs[p].query()

        return driver.run_wallclock(self.ctx, self.K, total, grad_ptr=lambda p: self.grad[p], pull_dst=lambda p: self.w_local[p],
                                    step=step, done=done, clock_ns=time.perf_counter_ns)

    def synchronize(self):
        B.dssp_synchronize(self.ctx)

    def weights(self):
        self.synchronize()
        return self.w.cpu().numpy()

    def worker_grad(self, p):
        torch.cuda.current_stream().synchronize()
        self.streams[p].synchronize()
        return self.grad[p].cpu().numpy(), float(self.loss[p].item())

    def workspace_tensor(self, p, what, index):
        """Saved tensor of worker p's last step (see dssp_workspace_tensor) as numpy, or None."""
        loc = B.dssp_workspace_tensor(self.mid, self.batch, self.n_classes, self.K, p, what, index)
        if loc is None:
            return None
        off, cnt = loc
        self.streams[p].synchronize()
        if what == 1:
            return self.ws[off:off + cnt].cpu().numpy()
        return self.ws[off:off + 4 * cnt].view(torch.float32).cpu().numpy()

    def close(self):
        if self.ctx is not None:
            B.dssp_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
