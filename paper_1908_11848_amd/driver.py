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


def run_schedule(ctx, K, durations, quota=None, total=None, grad_ptr=None, pull_dst=None, step=None, log=True):
    """Runs the schedule.  grad_ptr(p) -> device pointer of worker p's gradient (None for a
    host-only context); pull_dst(p) -> device pointer of its local weights; step(p, n) enqueues
    worker p's n-th iteration (dssp_worker_step) or None.  Returns (log, stats)."""
    if quota is None and total is None:
        raise ValueError("need quota or total")
    gp = grad_ptr or (lambda p: None)
    pd = pull_dst or (lambda p: None)
    out = [] if log else None
    heap = []
    pulled = [0] * K
    count = [0] * K             # pushes so far per worker (mirror of the server's t)
    version = 0
    T_end = 0
    for p in range(K):
        v = B.dssp_pull(ctx, p, pd(p))
        if log:
            out.append((PULL, p, 0, 0, 0, 0, v, 0))
        if step:
            step(p, 0)
        heapq.heappush(heap, (int(durations[p][0]), p))

    def start_next(q, T, tq, rq):
        if quota is not None and tq >= quota:
            return
        v = B.dssp_pull(ctx, q, pd(q))
        pulled[q] = v
        if log:
            out.append((PULL, q, T, tq, rq, v, v, 0))
        if step:
            step(q, tq)
        heapq.heappush(heap, (T + int(durations[q][tq]), q))

    while heap and (total is None or version < total):
        T, p = heapq.heappop(heap)
        T_end = T
        ok, released, rstar, grant = B.dssp_push(ctx, p, gp(p), T, K)
        version += 1
        count[p] += 1
        if log:
            t, r, _, v = B.dssp_clock(ctx, K)
            out.append((PUSH, p, T, t[p], r[p], v, pulled[p], 0))
            if rstar >= 0:
                out.append((CTRL, p, T, t[p], r[p], v, rstar, grant))
            out.append((OK if ok else BLOCK, p, T, t[p], r[p], v, 0, 0))
        else:
            t, r = count, [0] * K
        if ok:
            start_next(p, T, t[p], r[p])
        for q in released:
            if log:
                out.append((RELEASE, q, T, t[q], r[q], version, 0, 0))
            start_next(q, T, t[q], r[q])
    return out, dict(T_end=T_end, pushes=version)
