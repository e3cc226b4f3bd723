"""Emulation driver: K virtual workers in virtual time, through the C ABI.

A min-heap of (push time, worker) in integer ticks; each popped push goes to dssp_push, and
every worker that thereby holds an OK pulls, has its next iteration enqueued on its stream and
is re-inserted at push time + its next iteration time.  The server's decisions depend only on
the virtual timestamps, never on tensor values, so the host runs ahead of the device and only
stream / event ordering inside the library keeps the device consistent with the schedule.

The integer log has the record format (kind, worker, T, t[worker], r[worker], version, a0, a1):
PUSH a0 = version the gradient was computed on; CTRL a0 = r*, a1 = grant; PULL a0 = version
pulled.
"""
import heapq

from . import binding as B

PUSH, CTRL, OK, BLOCK, RELEASE, PULL = 0, 1, 2, 3, 4, 5


class Schedule:
    """Resumable schedule: advance(n) processes the next n pushes."""

    def __init__(self, ctx, K, durations, quota=None, grad_ptr=None, pull_dst=None, step=None, log=True, fused_pull=False,
                 aggregate=False):
        """grad_ptr(p) -> device pointer of worker p's gradient (None for a host-only context);
        pull_dst(p) -> device pointer of its local weights; step(p, n) enqueues worker p's n-th
        iteration (dssp_worker_step) or is None.  fused_pull: pushes go through dssp_push_pull, i.e. a worker
        that is granted OK by its own push gets its snapshot from the apply kernel (same log, same results).
        aggregate: pushes that share a timestamp go to the server together (dssp_push_many: decided one by one in
        worker order, applied by one kernel that also writes the snapshots; same log, same results)."""
        self.ctx, self.K, self.d, self.quota = ctx, K, durations, quota
        self.fused_pull = fused_pull
        self.aggregate = aggregate
        self.aggregated = 0             # pushes that went through dssp_push_many
        self.gp = grad_ptr or (lambda p: None)
        self.pd = pull_dst or (lambda p: None)
        self.step = step
        self.log = [] if log else None
        self.heap = []
        self.pulled = [0] * K
        self.count = [0] * K            # pushes so far per worker (mirror of the server's t)
        self.version = 0
        self.T_end = 0
        for p in range(K):
            v = B.dssp_pull(ctx, p, self.pd(p))
            if log:
                self.log.append((PULL, p, 0, 0, 0, 0, v, 0))
            if step:
                step(p, 0)
            heapq.heappush(self.heap, (int(durations[p][0]), p))

    def _start_next(self, q, T, tq, rq, pulled_version=None):
        if self.quota is not None and tq >= self.quota:
            return
        v = pulled_version if pulled_version is not None else B.dssp_pull(self.ctx, q, self.pd(q))
        self.pulled[q] = v
        if self.log is not None:
            self.log.append((PULL, q, T, tq, rq, v, v, 0))
        if self.step:
            self.step(q, tq)
        heapq.heappush(self.heap, (T + int(self.d[q][tq]), q))

    def advance(self, n_pushes):
        """Processes up to n_pushes pushes (fewer if every worker reached its quota).  Returns
        the number processed."""
        done = 0
        K, log = self.K, self.log
        while self.heap and done < n_pushes:
            if self.aggregate:
                group = self._same_time_group(n_pushes - done)
                if group is not None:
                    done += self._push_group(*group)
                    continue
            T, p = heapq.heappop(self.heap)
            self.T_end = T
            pulled_version = None
            if self.fused_pull and not (self.quota is not None and self.count[p] + 1 >= self.quota):
                ok, released, rstar, grant, pulled, v_now = B.dssp_push_pull(self.ctx, p, self.gp(p), T, K, self.pd(p))
                if pulled:
                    pulled_version = v_now
            else:
                ok, released, rstar, grant = B.dssp_push(self.ctx, p, self.gp(p), T, K)
            self.version += 1
            self.count[p] += 1
            done += 1
            if log is not None:
                t, r, _, v = B.dssp_clock(self.ctx, K)
                log.append((PUSH, p, T, t[p], r[p], v, self.pulled[p], 0))
                if rstar >= 0:
                    log.append((CTRL, p, T, t[p], r[p], v, rstar, grant))
                log.append((OK if ok else BLOCK, p, T, t[p], r[p], v, 0, 0))
            else:
                t, r = self.count, [0] * K
            if ok:
                self._start_next(p, T, t[p], r[p], pulled_version)
            for q in released:
                if log is not None:
                    log.append((RELEASE, q, T, t[q], r[q], self.version, 0, 0))
                self._start_next(q, T, t[q], r[q])
        return done


    MAX_GROUP = 16                      # DSSPK_APPLY_MANY_MAX

    def _same_time_group(self, room):
        """The pushes at the head of the heap that share its smallest timestamp, if there are at least two (at most
        `room`, at most MAX_GROUP; the rest of a larger group follows in the next call)."""
        T = self.heap[0][0]
        if room < 2 or sum(1 for e in self.heap if e[0] == T) < 2:
            return None
        workers = []
        while self.heap and self.heap[0][0] == T and len(workers) < min(room, self.MAX_GROUP):
            workers.append(heapq.heappop(self.heap)[1])
        return T, workers

    def _push_group(self, T, workers):
        K, log = self.K, self.log
        t0 = list(self.count)
        ok, released, rstar, grant, pv = B.dssp_push_many(self.ctx, workers, [self.gp(p) for p in workers], T, K,
                                                          [self.pd(q) for q in range(K)])
        self.T_end = T
        self.aggregated += len(workers)
        t, r, _, v_end = B.dssp_clock(self.ctx, K) if log is not None else (None, None, None, None)
        for j, p in enumerate(workers):
            self.version += 1
            self.count[p] += 1
            v = self.version
            # worker p pushes once in the group and nobody else changes t[p] or r[p], so the final counters are those
            # right after its push; a worker released here was waiting, so its counters did not move either
            tp, rp = (t[p], r[p]) if log is not None else (self.count[p], 0)
            if log is not None:
                log.append((PUSH, p, T, tp, rp, v, self.pulled[p], 0))
                if rstar[j] >= 0:
                    log.append((CTRL, p, T, tp, rp, v, rstar[j], grant[j]))
                log.append((OK if ok[j] else BLOCK, p, T, tp, rp, v, 0, 0))
            if ok[j]:
                self._start_next(p, T, tp, rp, pv[p] if pv[p] else None)
            for q in released[j]:
                tq, rq = (t[q], r[q]) if log is not None else (self.count[q], 0)
                if log is not None:
                    log.append((RELEASE, q, T, tq, rq, v, 0, 0))
                self._start_next(q, T, tq, rq, pv[q] if pv[q] else None)
        return len(workers)


def run_schedule(ctx, K, durations, quota=None, total=None, grad_ptr=None, pull_dst=None, step=None, log=True, fused_pull=False,
                 aggregate=False):
    """Runs a whole schedule: until `total` pushes were applied and / or every worker made
    `quota` pushes.  Returns (log, stats)."""
    if quota is None and total is None:
        raise ValueError("need quota or total")
    s = Schedule(ctx, K, durations, quota=quota, grad_ptr=grad_ptr, pull_dst=pull_dst, step=step, log=log, fused_pull=fused_pull,
                 aggregate=aggregate)
    s.advance(total if total is not None else K * quota)
    return s.log, dict(T_end=s.T_end, pushes=s.version, aggregated=s.aggregated)


def run_wallclock(ctx, K, total, grad_ptr, pull_dst, step, done, clock_ns, poll_sleep=None):
    """The controller fed with REAL push times instead of a table (how the paper's server runs): a worker's push
    reaches the server when its gradient is actually finished on the device.

    step(p, n) enqueues worker p's n-th iteration and arranges for done(p) to turn true once the device has
    finished it; clock_ns() is a monotonic clock.  The loop polls the running workers in index order; the first one
    found finished pushes with T = elapsed microseconds (integer ticks, strictly increasing so that two pushes never
    share a timestamp), and every worker that thereby holds an OK pulls and starts its next iteration.  Runs until
    `total` pushes.  Returns the same integer log as Schedule (PUSH / CTRL / OK / BLOCK / RELEASE / PULL records);
    replaying its (T, worker) sequence through any implementation of the rules must give the same decisions.
    """
    log = []
    running = [False] * K
    count = [0] * K
    pulled = [0] * K
    t0 = clock_ns()
    last_T = 0

    def start(q, T, tq, rq):
        v = B.dssp_pull(ctx, q, pull_dst(q))
        pulled[q] = v
        log.append((PULL, q, T, tq, rq, v, v, 0))
        step(q, tq)
        running[q] = True

    for p in range(K):
        start(p, 0, 0, 0)
    pushes = 0
    while pushes < total:
        if not any(running):
            raise RuntimeError("no worker is running: the schedule is stuck")
        progressed = False
        for p in range(K):
            if pushes >= total or not running[p] or not done(p):
                continue
            progressed = True
            running[p] = False
            T = max(last_T + 1, (clock_ns() - t0) // 1000)
            last_T = T
            ok, released, rstar, grant = B.dssp_push(ctx, p, grad_ptr(p), T, K)
            pushes += 1
            count[p] += 1
            t, r, _, v = B.dssp_clock(ctx, K)
            log.append((PUSH, p, T, t[p], r[p], v, pulled[p], 0))
            if rstar >= 0:
                log.append((CTRL, p, T, t[p], r[p], v, rstar, grant))
            log.append((OK if ok else BLOCK, p, T, t[p], r[p], v, 0, 0))
            if ok:
                start(p, T, t[p], r[p])
            for q in released:
                log.append((RELEASE, q, T, t[q], r[q], v, 0, 0))
                start(q, T, t[q], r[q])
        if not progressed and poll_sleep:
            poll_sleep()
    return log, dict(T_end=last_T, pushes=pushes)


def run_wallclock_device(ctx, K, total, grad_ptr, pull_dst, step_timed, poll_sleep=None):
    """The controller fed with DEVICE times: every iteration is a dssp_worker_step_timed (step_timed(p, n) enqueues worker
    p's n-th one, with whatever slowdown emulates that worker's GPU), and a push reaches the server with the device-clock
    microsecond at which the worker's stream was done with the iteration, as reported by dssp_step_done.

    The loop sweeps over the running workers; those found finished in one sweep push in the order of their device times
    (ties: lower index).  Timestamps handed to the server are kept strictly increasing (T = max(device time, last T + 1)):
    a completion noticed a sweep late keeps its place in the order of arrival, as at a real server.  Runs until `total`
    pushes.  Returns (log, stats) with the same integer log as Schedule; stats['times'][p] lists (start, gradient
    finished, done) of worker p's iterations in device microseconds.  Replaying the log's (T, worker) sequence through
    any implementation of the rules must give the same decisions."""
    log = []
    running = [False] * K
    pulled = [0] * K
    times = [[] for _ in range(K)]
    last_T = 0

    def start(q, T, tq, rq):
        v = B.dssp_pull(ctx, q, pull_dst(q))
        pulled[q] = v
        log.append((PULL, q, T, tq, rq, v, v, 0))
        step_timed(q, tq)
        running[q] = True

    for p in range(K):
        start(p, 0, 0, 0)
    pushes = 0
    while pushes < total:
        if not any(running):
            raise RuntimeError("no worker is running: the schedule is stuck")
        finished = []
        for p in range(K):
            if running[p]:
                t = B.dssp_step_done(ctx, p)
                if t is not None:
                    running[p] = False
                    times[p].append(t)
                    finished.append((t[2], p))
        if not finished:
            if poll_sleep:
                poll_sleep()
            continue
        for t_done, p in sorted(finished):
            if pushes >= total:
                break
            T = max(last_T + 1, t_done)
            last_T = T
            ok, released, rstar, grant = B.dssp_push(ctx, p, grad_ptr(p), T, K)
            pushes += 1
            t, r, _, v = B.dssp_clock(ctx, K)
            log.append((PUSH, p, T, t[p], r[p], v, pulled[p], 0))
            if rstar >= 0:
                log.append((CTRL, p, T, t[p], r[p], v, rstar, grant))
            log.append((OK if ok else BLOCK, p, T, t[p], r[p], v, 0, 0))
            if ok:
                start(p, T, t[p], r[p])
            for q in released:
                log.append((RELEASE, q, T, t[q], r[q], v, 0, 0))
                start(q, T, t[q], r[q])
    return log, dict(T_end=last_T, pushes=pushes, times=times)
