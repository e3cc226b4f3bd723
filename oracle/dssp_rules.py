"""Oracle, part 1: the server's decision rules and the event simulator.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Pure Python integers; no
floating point anywhere, so every value in the event log is exact.

What is followed:
  * Alg. 1, server part: count the push, apply the gradient, then decide
    whether worker p gets its OK now or must wait for the slowest worker.
  * Alg. 2 (synchronization_controller): from the two latest push timestamps
    of p and of the slowest worker, extrapolate r_max+1 future push times of
    each and return the index r on p's timeline whose extrapolated time is
    closest to any extrapolated push of the slowest worker.
  * Sec. I-A: BSP, ASP, SSP as special cases (BSP = (s_L, r_max) = (0, 0),
    SSP(s) = (s, 0), ASP = never wait).

Readings taken where the paper is silent or inconsistent (each is listed with
its reason in the design notes of the repository):
  R1  Table A is shifted on every push, before the decision, not only inside
      the controller (Alg. 2's caption says A holds the two latest pushes of
      all workers, and the slowest worker's interval is read from it).
  R2  The OK sent right after the controller call is the first of the r*
      extra iterations (Sec. III-C prose and Fig. 2: r* = 3 means three more
      iterations), so r_p <- grant - 1 after that OK.
  R3  slowest = argmin t, ties broken by the oldest latest push A[i][0], then
      by the smallest index.  "p is the fastest" iff t_p = max t (ties count).
  R4  Hard cap so that the gap at every OK stays within s_L + r_max (problem
      statement, Sec. III-A, and the proof of Theorem 2):
      grant = min(r*, s_L + r_max - gap + 1).
  R5  argmin ties in Alg. 2: smallest r.
  R6  Sim arrays have r_max+1 entries; p's starts at its current push, the
      slowest worker's one interval after its latest push (Alg. 2 steps 6-7).
  R7  A starts at 0 (the common start time); a slowest worker without any push
      has interval 0, which makes every extrapolated time 0 and r* = 0.
  R8  "Wait until the slowest catches up" applies only if no OK was sent by
      the controller branch.
  R9  Pushes are handled strictly one by one in (timestamp, worker) order.
  R10 Released workers have r = 0 and are released in ascending index order,
      after the pusher's own pull; release condition is t_q - min t <= s_L.
"""

import heapq

# event kinds of the integer log
PUSH, CTRL, OK, BLOCK, RELEASE, PULL = 0, 1, 2, 3, 4, 5
KIND_NAMES = ("PUSH", "CTRL", "OK", "BLOCK", "RELEASE", "PULL")

ASP_S_L = 2**31 - 1   # a lower bound no gap can exceed: the server never makes anyone wait


class ServerState:
    """Integer state the server keeps (Alg. 1 preamble, Alg. 2 table A)."""

    def __init__(self, K, s_L, r_max):
        if K < 1 or s_L < 0 or r_max < 0:
            raise ValueError("K >= 1, s_L >= 0, r_max >= 0 required")
        self.K, self.s_L, self.r_max = K, s_L, r_max
        self.t = [0] * K                      # pushes received per worker
        self.r = [0] * K                      # extra-iteration credit per worker
        self.A = [[0, 0] for _ in range(K)]   # [latest, second latest] push time
        self.blocked = [False] * K
        self.version = 0                      # number of applies so far


def slowest_worker(t, A):
    """R3: fewest pushes; ties -> oldest latest push; then smallest index."""
    best = 0
    for i in range(1, len(t)):
        if (t[i], A[i][0], i) < (t[best], A[best][0], best):
            best = i
    return best


def synchronization_controller(A, t, p, r_max):
    """Alg. 2 after its first two steps (the shift of A[p] was done by the caller, R1)."""
    slow = slowest_worker(t, A)
    I_p = A[p][0] - A[p][1]
    I_s = A[slow][0] - A[slow][1]
    sim_p = [A[p][0] + i * I_p for i in range(r_max + 1)]
    sim_s = [A[slow][0] + I_s + k * I_s for k in range(r_max + 1)]
    r_star, best = 0, None
    for r in range(r_max + 1):
        for k in range(r_max + 1):
            d = abs(sim_s[k] - sim_p[r])
            if best is None or d < best:      # strict: ties keep the smaller r (R5)
                best, r_star = d, r
    return r_star


def server_on_push(st, p, T):
    """Alg. 1, server part, for one push.  Returns (ok, r_star, grant, released).

    r_star = grant = -1 when the controller was not called.  The caller is
    responsible for the weight update itself; here `version` counts it.
    """
    if st.blocked[p]:
        raise RuntimeError("push from a worker that is waiting for OK")
    st.A[p][1] = st.A[p][0]
    st.A[p][0] = T
    st.t[p] += 1
    st.version += 1
    r_star = grant = -1
    if st.r[p] > 0:
        st.r[p] -= 1
        ok = True
    else:
        gap = st.t[p] - min(st.t)
        if gap <= st.s_L:
            ok = True
        elif st.t[p] == max(st.t):
            r_star = synchronization_controller(st.A, st.t, p, st.r_max)
            grant = min(r_star, st.s_L + st.r_max - gap + 1)      # R4
            if grant >= 1:
                st.r[p] = grant - 1                                # R2
                ok = True
            else:
                ok = False
        else:
            ok = False
    if not ok:
        st.blocked[p] = True
    released = []
    t_min = min(st.t)
    for q in range(st.K):
        if st.blocked[q] and q != p and st.t[q] - t_min <= st.s_L:
            st.blocked[q] = False
            released.append(q)
    return ok, r_star, grant, released


def simulate(K, s_L, r_max, durations, quota=None, total=None, on_pull=None, on_push=None):
    """Run the emulated cluster in virtual time and return (log, state, stats).

    durations[p][n]  int ticks worker p needs for its n-th iteration (n from 0),
                     i.e. from the moment it is allowed to start until its push
                     reaches the server.
    quota            each worker stops after this many pushes (or None)
    total            the run stops once this many pushes were applied (or None)
    on_pull(p, version), on_push(p, n, version_before)
                     numerics hooks, called in log order (used by oracle/ps.py)

    Log records are 8-tuples of ints:
      (kind, worker, T, t[worker], r[worker], version, a0, a1)
      PUSH    a0 = version the pushed gradient was computed on
      CTRL    a0 = r*, a1 = grant
      PULL    a0 = version pulled
    """
    if quota is None and total is None:
        raise ValueError("need quota or total")
    st = ServerState(K, s_L, r_max)
    pulled = [0] * K
    log = []
    heap = []
    wait_ticks = [0] * K
    blocked_since = [0] * K
    for p in range(K):
        if on_pull:
            on_pull(p, 0)
        log.append((PULL, p, 0, 0, 0, 0, 0, 0))
        heapq.heappush(heap, (int(durations[p][0]), p))
    T_end = 0

    def start_next(q, T):
        if quota is not None and st.t[q] >= quota:
            return
        pulled[q] = st.version
        if on_pull:
            on_pull(q, st.version)
        log.append((PULL, q, T, st.t[q], st.r[q], st.version, st.version, 0))
        heapq.heappush(heap, (T + int(durations[q][st.t[q]]), q))

    while heap and (total is None or st.version < total):
        T, p = heapq.heappop(heap)
        T_end = T
        if on_push:
            on_push(p, st.t[p], pulled[p])
        ok, r_star, grant, released = server_on_push(st, p, T)
        log.append((PUSH, p, T, st.t[p], st.r[p], st.version, pulled[p], 0))
        if r_star >= 0:
            log.append((CTRL, p, T, st.t[p], st.r[p], st.version, r_star, grant))
        if ok:
            log.append((OK, p, T, st.t[p], st.r[p], st.version, 0, 0))
            start_next(p, T)
        else:
            log.append((BLOCK, p, T, st.t[p], st.r[p], st.version, 0, 0))
            blocked_since[p] = T
        for q in released:
            wait_ticks[q] += T - blocked_since[q]
            log.append((RELEASE, q, T, st.t[q], st.r[q], st.version, 0, 0))
            start_next(q, T)
    stats = {
        "T_end": T_end,
        "pushes": st.version,
        "wait_ticks": wait_ticks,
        "pushes_per_Mtick": (st.version * 1e6 / T_end) if T_end else 0.0,
    }
    return log, st, stats
