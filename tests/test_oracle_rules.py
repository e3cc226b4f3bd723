"""Pins of the oracle's decision rules against what the paper fixes.

Every check here compares oracle/dssp_rules.py with something that is not
itself: hand-computed controller tables, separately written BSP / SSP / ASP
rules (Sec. I-A), the staleness bound of the problem statement (Sec. III-A)
and the throughput ordering the paper reports (Sec. V-B).
"""
import heapq
import random

import numpy as np
import pytest

from oracle import dssp_rules as R


# ---------------------------------------------------------------- Alg. 2
def brute_controller(A, slow, p, r_max):
    """Alg. 2 steps 4-8 with a full table of absolute differences."""
    Ip, Is = A[p][0] - A[p][1], A[slow][0] - A[slow][1]
    sp = np.array([A[p][0] + i * Ip for i in range(r_max + 1)], dtype=object)
    ss = np.array([A[slow][0] + Is * (k + 1) for k in range(r_max + 1)], dtype=object)
    D = np.abs(ss[:, None] - sp[None, :])            # [k][r]
    best = D.min()
    return min(r for r in range(r_max + 1) if (D[:, r] == best).any())


def test_controller_constructed_example_like_fig2():
    # fast worker p=0: pushes at 90, 100 (interval 10); slowest p=1: pushes at 61, 96
    # (interval 35, next push expected at 131).  With R=[0,4] p's simulated pushes are
    # 100,110,120,130,140; 130 is closest to 131 -> r* = 3 (the shape of Fig. 2).
    A = [[100, 90], [96, 61]]
    t = [9, 2]
    assert R.synchronization_controller(A, t, 0, 4) == 3


def test_controller_golden_table():
    rows = [l.split() for l in open(__file__.replace("test_oracle_rules.py", "golden/controller_cases.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) >= 8
    for row in rows:
        ap0, ap1, as0, as1, r_max, want = map(int, row)
        A = [[ap0, ap1], [as0, as1]]
        assert R.synchronization_controller(A, [10, 1], 0, r_max) == want, row


def test_controller_special_cases():
    # r_max = 0: only r = 0 exists
    assert R.synchronization_controller([[50, 40], [30, 10]], [5, 1], 0, 0) == 0
    # slowest has never pushed: interval 0, all simulated times 0 -> closest is p's current push
    assert R.synchronization_controller([[50, 40], [0, 0]], [5, 0], 0, 6) == 0
    # slowest's next push is exactly j fast intervals after p's current push -> j
    for j in range(0, 6):
        A = [[1000, 990], [1000 + 10 * j - 400, 1000 + 10 * j - 800]]
        assert R.synchronization_controller(A, [9, 1], 0, 5) == j
    # ... and beyond the range the last index is the closest
    A = [[1000, 990], [1000 + 10 * 9 - 400, 1000 + 10 * 9 - 800]]
    assert R.synchronization_controller(A, [9, 1], 0, 5) == 5


def test_controller_matches_brute_force_table():
    rnd = random.Random(7)
    for _ in range(3000):
        K = rnd.randint(2, 6)
        r_max = rnd.randint(0, 15)
        A = [[0, 0] for _ in range(K)]
        t = [rnd.randint(0, 20) for _ in range(K)]
        for i in range(K):
            a1 = rnd.randint(0, 10**6)
            A[i] = [a1 + rnd.randint(0, 10**5), a1]
        p = max(range(K), key=lambda i: t[i])
        slow = min(range(K), key=lambda i: (t[i], A[i][0], i))
        assert R.slowest_worker(t, A) == slow
        assert R.synchronization_controller(A, t, p, r_max) == brute_controller(A, slow, p, r_max)


def test_slowest_tie_breaks():
    assert R.slowest_worker([3, 3, 3], [[50, 0], [40, 0], [40, 0]]) == 1
    assert R.slowest_worker([4, 3, 3], [[1, 0], [40, 0], [39, 0]]) == 2


# ---------------------------------------------------------------- Alg. 1 server part
def test_credit_is_consumed_even_when_not_fastest():
    st = R.ServerState(3, 1, 4)
    st.t = [5, 9, 2]
    st.r = [2, 0, 0]
    ok, r_star, grant, rel = R.server_on_push(st, 0, 100)
    assert ok and r_star == -1 and st.r[0] == 1 and st.t[0] == 6     # 6-2 > s_L, not fastest, still OK


def test_controller_zero_means_wait_now():
    st = R.ServerState(2, 1, 4)
    st.t = [2, 1]
    st.A = [[100, 50], [80, 0]]        # slow interval 80 -> next at 160; p interval 50: 150 closest? no:
    # p pushes at 151 -> interval 51, Sim_p = 151, 202, ...; Sim_s = 160, 240, ... -> |160-151| = 9 minimal -> r* = 0
    ok, r_star, grant, rel = R.server_on_push(st, 0, 151)
    assert (ok, r_star, grant) == (False, 0, 0) and st.blocked[0]


def test_rstar_grants_exactly_rstar_more_iterations():
    # Sec. III-C / Fig. 2: r* = 3 -> three more iterations, then the worker waits.
    st = R.ServerState(2, 1, 4)
    st.t = [2, 1]
    st.A = [[100, 90], [96, 61]]
    oks = 0
    T = 110
    # push at 110: interval 10, Sim_p = 110..150 ; Sim_s = 131,... -> r* = 2 (130)
    ok, r_star, grant, _ = R.server_on_push(st, 0, T)
    assert ok and r_star == 2 and grant == 2 and st.r[0] == 1
    oks += 1
    while True:
        T += 10
        ok, r_star, grant, _ = R.server_on_push(st, 0, T)
        if not ok:
            break
        oks += 1
        assert oks < 10
    # 2 granted iterations in total before the wait: the OK of the controller call + 1 credit
    assert oks == 2 and st.blocked[0]


def test_cap_at_upper_bound_on_reentry():
    st = R.ServerState(2, 1, 2)            # s_U = 3
    st.t = [3, 0]                          # gap will be 4 > s_U
    st.A = [[30, 20], [0, 0]]
    st.A[1] = [1000, 0]                    # slowest far in the future -> controller wants the maximum
    ok, r_star, grant, _ = R.server_on_push(st, 0, 40)
    assert r_star == 2 and grant == 0 and not ok


# ---------------------------------------------------------------- independent paradigms (Sec. I-A)
def simulate_ssp_independent(K, s, d, quota):
    """SSP as in Sec. I-A: a worker that is more than s iterations ahead of the
    slowest waits; nobody else waits.  Written without dssp_rules."""
    clock = [0] * K
    waiting = {}
    events = []
    version = 0
    heap = [(int(d[p][0]), p) for p in range(K)]
    heapq.heapify(heap)
    starts = [[0] for _ in range(K)]
    pushes = [[] for _ in range(K)]
    while heap:
        T, p = heapq.heappop(heap)
        clock[p] += 1
        version += 1
        pushes[p].append(T)
        go = []
        if clock[p] - min(clock) <= s:
            go.append(p)
        else:
            waiting[p] = T
        for q in sorted(waiting):
            if q != p and clock[q] - min(clock) <= s:
                go.append(q)
        for q in go:
            waiting.pop(q, None)
            events.append((q, T, version))
            if clock[q] < quota:
                starts[q].append(T)
                heapq.heappush(heap, (T + int(d[q][clock[q]]), q))
    return pushes, events


def simulate_bsp_independent(K, d, quota):
    """Barrier: round n starts for everyone when the last push of round n-1 arrived."""
    start = 0
    pushes = [[] for _ in range(K)]
    for n in range(quota):
        ts = [start + int(d[p][n]) for p in range(K)]
        for p in range(K):
            pushes[p].append(ts[p])
        start = max(ts)
    return pushes


def push_times(log, K):
    out = [[] for _ in range(K)]
    for kind, p, T, *_ in log:
        if kind == R.PUSH:
            out[p].append(T)
    return out


def rand_durations(seed, K, n, hetero=True):
    g = np.random.default_rng(seed)
    m = g.uniform(1.0, 4.0, K) if hetero else np.ones(K)
    return np.maximum((m[:, None] * np.exp(0.2 * g.standard_normal((K, n))) * 1000).astype(np.int64), 1)


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("s", [0, 1, 3, 6])
def test_rmax0_is_ssp(seed, s):
    K, quota = 5, 40
    d = rand_durations(seed, K, quota + 1)
    log, st, _ = R.simulate(K, s, 0, d, quota=quota)
    pushes, events = simulate_ssp_independent(K, s, d, quota)
    assert push_times(log, K) == pushes
    go = [(p, T, v) for kind, p, T, tp, rp, v, *_ in log if kind in (R.OK, R.RELEASE)]
    assert go == events


@pytest.mark.parametrize("seed", range(6))
def test_zero_zero_is_bsp(seed):
    K, quota = 4, 30
    d = rand_durations(seed, K, quota + 1)
    log, st, _ = R.simulate(K, 0, 0, d, quota=quota)
    assert push_times(log, K) == simulate_bsp_independent(K, d, quota)
    # every worker starts a round from the same version: pulls see multiples of K
    for kind, p, T, tp, rp, v, a0, a1 in log:
        if kind == R.PULL:
            assert a0 % K == 0 and a0 == K * tp
        if kind == R.PUSH:
            assert a0 == K * (tp - 1)


@pytest.mark.parametrize("seed", range(4))
def test_asp_never_waits(seed):
    K, quota = 6, 50
    d = rand_durations(seed, K, quota + 1)
    log, st, _ = R.simulate(K, R.ASP_S_L, 0, d, quota=quota)
    assert not any(rec[0] in (R.BLOCK, R.RELEASE, R.CTRL) for rec in log)
    want = [list(np.cumsum(d[p][:quota])) for p in range(K)]
    assert push_times(log, K) == want


def check_invariants(log, K, s_L, r_max):
    t = [0] * K
    for kind, p, T, tp, rp, v, a0, a1 in log:
        if kind == R.PUSH:
            t[p] += 1
            assert tp == t[p] and v == sum(t)
            assert max(t) - min(t) <= s_L + r_max + 1
            assert v - a0 >= 1                       # a gradient is at least one version stale-free
        elif kind in (R.OK, R.RELEASE):
            assert t[p] - min(t) <= s_L + r_max      # Sec. III-A: threshold within [s_L, s_U]
            if kind == R.RELEASE:
                assert t[p] - min(t) <= s_L and rp == 0
        elif kind == R.BLOCK:
            assert t[p] - min(t) > s_L               # only workers beyond s_L ever wait
        elif kind == R.CTRL:
            assert t[p] == max(t) and 0 <= a0 <= r_max and a1 <= a0


@pytest.mark.parametrize("seed", range(25))
def test_staleness_bound_random_schedules(seed):
    rnd = random.Random(seed)
    K = rnd.randint(2, 9)
    s_L, r_max = rnd.randint(0, 4), rnd.randint(0, 15)
    quota = 60
    d = rand_durations(100 + seed, K, quota + 1)
    if seed % 3 == 0:                  # a straggler appears: one worker turns 10x slower half way
        d[rnd.randrange(K), quota // 2:] *= 10
    log, st, _ = R.simulate(K, s_L, r_max, d, quota=quota)
    check_invariants(log, K, s_L, r_max)
    assert st.t == [quota] * K and not any(st.blocked)        # everyone finishes, nobody is left waiting


@pytest.mark.parametrize("seed", range(8))
def test_paradigm_ordering_per_push(seed):
    # Sec. V-B: ASP has the largest iteration throughput, BSP the smallest; on a shared
    # duration table this holds push by push.
    K, quota, s_L, r_max = 5, 50, 3, 12
    d = rand_durations(200 + seed, K, quota + 1)
    runs = [R.simulate(K, *cfg, d, quota=quota)[0] for cfg in
            [(R.ASP_S_L, 0), (s_L + r_max, 0), (s_L, r_max), (s_L, 0), (0, 0)]]
    T = [push_times(l, K) for l in runs]
    for a, b in zip(T[:-1], T[1:]):
        for p in range(K):
            assert all(x <= y for x, y in zip(a[p], b[p]))


def test_total_limit_and_log_shape():
    K = 16
    d = rand_durations(5, K, 2000)
    log, st, stats = R.simulate(K, 3, 15, d, total=1000)
    assert st.version == 1000 and stats["pushes"] == 1000
    assert all(len(rec) == 8 and all(isinstance(v, (int, np.integer)) for v in rec) for rec in log)
    check_invariants(log, K, 3, 15)


def test_dssp_beats_ssp_low_on_heterogeneous_table():
    # the point of the method (Sec. I-B): fewer waits than SSP at the lower bound
    K, quota = 4, 200
    d = rand_durations(11, K, quota + 1)
    _, _, ssp = R.simulate(K, 3, 0, d, quota=quota)
    _, _, dssp = R.simulate(K, 3, 12, d, quota=quota)
    assert sum(dssp["wait_ticks"]) <= sum(ssp["wait_ticks"])
