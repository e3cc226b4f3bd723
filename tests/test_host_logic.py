"""CPU-side checks of the library: it loads, exports every symbol the headers declare, its host
controller (Alg. 1 server part + Alg. 2) makes the oracle's decisions, and its parameter layout is
the documented one.  No compute call is made (host-only contexts enqueue nothing)."""
import os
import random
import re
import subprocess
import sys

import numpy as np
import pytest

from paper_1908_11848_amd import binding as B, driver, inputs
from oracle import dssp_rules as R

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for h in ("dssp.h", "dssp_kernels.h"):
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(dsspk?_[a-z0-9_]+)\s*\(", text))
    return names


def test_library_loads_and_exports_every_declared_symbol():
    lib = B.lib()
    names = declared_symbols()
    assert len(names) >= 30
    for n in names:
        assert hasattr(lib, n), n
    assert names == set(B._SIGNATURES), names ^ set(B._SIGNATURES)      # binding and headers list the same calls


def host_log(K, s_L, r_max, d, quota=None, total=None, fused_pull=False, aggregate=False, stats=None):
    ctx = B.dssp_create(None, 0, K, s_L, r_max, 0.1)
    try:
        log, st = driver.run_schedule(ctx, K, d, quota=quota, total=total, fused_pull=fused_pull, aggregate=aggregate)
        if stats is not None:
            stats.update(st)
        return log
    finally:
        B.dssp_destroy(ctx)


def tie_table(kind, K, n, seed=0):
    """Iteration-time tables in which pushes of different workers coincide."""
    if kind == "rounded":            # the homogeneous cluster's +-5 % jitter on a grid of 0.05
        return np.maximum(np.rint(inputs.durations(2, K, n) / 50_000).astype(np.int64) * 50_000, 50_000)
    if kind == "equal":              # identical workers: every push of a round arrives together
        return np.full((K, n), 1_000_000, dtype=np.int64)
    g = np.random.default_rng(seed)  # small integers: ties of every size, stragglers included
    return g.integers(1, 5, (K, n)).astype(np.int64) * np.where(g.random((K, 1)) < 0.3, 3, 1)


@pytest.mark.parametrize("kind,K,s_L,r_max", [("rounded", 4, 3, 12), ("equal", 8, 0, 0), ("equal", 16, 3, 15), ("equal", 5, 1, 0),
                                              ("small", 8, 3, 12), ("small", 16, 0, 0), ("small", 3, 2, 4), ("small", 20, 1, 2)])
def test_same_timestamp_pushes_aggregated_take_the_oracles_decisions(kind, K, s_L, r_max):
    """Alg. 1 server step 2: simultaneous pushes are aggregated.  Handing them to the server together (dssp_push_many)
    must leave every decision, clock, version and pull as the oracle's one-by-one processing has them."""
    for seed in range(3):
        d = tie_table(kind, K, 80, seed)
        for total, quota in ((None, 60), (157, None)):
            olog, st, _ = R.simulate(K, s_L, r_max, d, quota=quota, total=total)
            stats = {}
            assert host_log(K, s_L, r_max, d, quota=quota, total=total, aggregate=True, stats=stats) == olog
            assert stats["aggregated"] > 0 and stats["pushes"] == st.version
            assert host_log(K, s_L, r_max, d, quota=quota, total=total, fused_pull=True, aggregate=True) == olog


def test_controller_search_equals_the_double_loop_of_alg2():
    """The library finds the closest pair of extrapolated push times by one division per candidate; the oracle scans all
    pairs as Alg. 2 prints it.  Same r* on random tables: long and short intervals, exact ties, zero and negative
    intervals (timestamps are the caller's), r_max up to 300."""
    rnd = random.Random(5)
    for case in range(300):
        r_max = rnd.choice([0, 1, 2, 5, 12, 15, 40, 300])
        scale = rnd.choice([1, 10, 1000, 10**9, 10**15])
        a1, b1 = rnd.randrange(0, 50) * scale, rnd.randrange(0, 50) * scale
        ip, isl = rnd.randrange(-3, 40) * scale // rnd.choice([1, 1, 7]), rnd.randrange(-3, 40) * scale // rnd.choice([1, 1, 3])
        # worker 0 = p pushes twice (at a1 - ip... then a1), worker 1 = the slowest pushes at b1 - isl, then b1, in a
        # 2-worker context with s_L = 0 where worker 0 is made the fastest by one more push
        ctx = B.dssp_create(None, 0, 2, 0, r_max, 0.1)
        seq = [(1, b1 - isl), (0, a1 - 2 * ip)]
        st = R.ServerState(2, 0, r_max)
        ok_all = True
        for p, T in seq + [(1, b1), (0, a1 - ip), (0, a1)]:
            if st.blocked[p]:
                ok_all = False
                break
            want = R.server_on_push(st, p, T)
            ok, rel, rstar, grant = B.dssp_push(ctx, p, None, T, 2)
            assert (ok, rstar, grant, rel) == want, (case, p, T, want, (ok, rstar, grant, rel))
        B.dssp_destroy(ctx)
    # and directly against the definition on the controller's own inputs
    for case in range(200):
        r_max = rnd.choice([0, 3, 12, 100])
        A = [[rnd.randrange(-10**6, 10**6), rnd.randrange(-10**6, 10**6)] for _ in range(2)]
        t = [5, 2]
        want = R.synchronization_controller(A, t, 0, r_max)
        sim_p = [A[0][0] + i * (A[0][0] - A[0][1]) for i in range(r_max + 1)]
        sim_s = [A[1][0] + (k + 1) * (A[1][0] - A[1][1]) for k in range(r_max + 1)]
        best = min(abs(a - b) for a in sim_p for b in sim_s)
        assert want == min(i for i, a in enumerate(sim_p) if min(abs(a - b) for b in sim_s) == best)


@pytest.mark.parametrize("seed", range(20))
def test_host_controller_matches_oracle_random(seed):
    rnd = random.Random(seed)
    K = rnd.randint(1, 12)
    s_L, r_max = rnd.choice([0, 1, 2, 3, 5]), rnd.choice([0, 1, 4, 12, 15])
    g = np.random.default_rng(seed)
    m = g.uniform(1.0, 4.0, K)
    d = np.maximum((m[:, None] * np.exp(0.3 * g.standard_normal((K, 130))) * 1000).astype(np.int64), 1)
    if seed % 4 == 0:
        d[:, :] = d[:, :1]                       # constant intervals: many exact ties in Alg. 2
    if seed % 5 == 0:
        d[rnd.randrange(K), 40:] *= 12           # a straggler appears
    quota = 120
    olog, st, _ = R.simulate(K, s_L, r_max, d, quota=quota)
    assert host_log(K, s_L, r_max, d, quota=quota) == olog
    # pushes through dssp_push_pull (the pusher's pull folded into the apply when it is granted OK): same schedule
    assert host_log(K, s_L, r_max, d, quota=quota, fused_pull=True) == olog


@pytest.mark.parametrize("cfg,K,s_L,r_max,total", [(1, 4, 3, 4, 200), (2, 4, 3, 12, 400), (3, 4, 3, 12, 400),
                                                   (3, 4, 0, 0, 400), (3, 4, 3, 0, 400), (3, 4, B.DSSP_S_L_NEVER_WAIT, 0, 400),
                                                   (4, 8, 3, 12, 200), (5, 16, 3, 15, 10000)])
def test_host_controller_matches_oracle_on_workload_schedules(cfg, K, s_L, r_max, total):
    d = inputs.durations(cfg, K, total)
    olog, _, _ = R.simulate(K, s_L, r_max, d, total=total)
    assert host_log(K, s_L, r_max, d, total=total) == olog
    assert host_log(K, s_L, r_max, d, total=total, fused_pull=True) == olog


def test_clock_and_state_errors_host_only():
    ctx = B.dssp_create(None, 0, 3, 1, 0, 0.1)
    t, r, blocked, v = B.dssp_clock(ctx, 3)
    assert (t, r, blocked, v) == ([0, 0, 0], [0, 0, 0], [False] * 3, 0)
    for T in (10, 20):
        ok, rel, rs, gr = B.dssp_push(ctx, 0, None, T, 3)
        assert B.dssp_pull(ctx, 0, None) == (1 if T == 10 else 2) if ok else True
    # t = [2,0,0], s_L = 1: worker 0 is 2 ahead -> it waits, the controller (r_max = 0) returned 0
    t, r, blocked, v = B.dssp_clock(ctx, 3)
    assert t == [2, 0, 0] and blocked == [True, False, False] and v == 2
    with pytest.raises(B.DsspError) as e:
        B.dssp_push(ctx, 0, None, 30, 3)
    assert e.value.code == B.DSSP_ESTATE
    with pytest.raises(B.DsspError) as e:
        B.dssp_pull(ctx, 0, None)
    assert e.value.code == B.DSSP_ESTATE
    with pytest.raises(B.DsspError) as e:
        B.dssp_pull(ctx, 3, None)
    assert e.value.code == B.DSSP_EINVAL
    ok, rel, _, _ = B.dssp_push(ctx, 1, None, 40, 3)
    assert ok and rel == []
    ok, rel, _, _ = B.dssp_push(ctx, 2, None, 41, 3)
    assert ok and rel == [0]                     # slowest caught up to within s_L
    B.dssp_destroy(ctx)
    for bad in [(0, 0, 0), (2, -1, 0), (2, 0, -1)]:
        with pytest.raises(B.DsspError):
            B.dssp_create(None, 0, *bad, 0.1)


def test_push_many_argument_and_state_errors_leave_the_clocks_untouched():
    K = 4
    ctx = B.dssp_create(None, 0, K, 0, 0, 0.1)                  # BSP: whoever pushes first waits
    none = [None] * K
    for bad in ([1, 0], [2, 2], [0, 4], [-1, 2]):               # not ascending, repeated, out of range
        with pytest.raises(B.DsspError) as e:
            B.dssp_push_many(ctx, bad, [None] * len(bad), 10, K, none)
        assert e.value.code == B.DSSP_EINVAL
    with pytest.raises(B.DsspError) as e:
        B.dssp_push_many(ctx, list(range(17)), [None] * 17, 10, K, none)
    assert e.value.code == B.DSSP_EINVAL                        # more than 16 pushes in one call
    assert B.dssp_clock(ctx, K) == ([0] * K, [0] * K, [False] * K, 0)
    ok, rel, rstar, grant, pv = B.dssp_push_many(ctx, [0, 2], none[:2], 10, K, none)
    assert ok == [False, False] and rel == [[], []] and pv == [0] * K
    t, r, blocked, v = B.dssp_clock(ctx, K)
    assert t == [1, 0, 1, 0] and blocked == [True, False, True, False] and v == 2
    with pytest.raises(B.DsspError) as e:                       # worker 2 is waiting: nothing of the group may count
        B.dssp_push_many(ctx, [1, 2], none[:2], 11, K, none)
    assert e.value.code == B.DSSP_ESTATE
    assert B.dssp_clock(ctx, K) == (t, r, blocked, v)
    ok, rel, rstar, grant, pv = B.dssp_push_many(ctx, [1, 3], none[:2], 12, K, none)
    assert ok == [False, True] and rel == [[], [0, 1, 2]]       # the last push of the round releases the three that waited
    assert pv == [4, 4, 4, 4]                                   # everybody goes on with the weights after all four pushes
    assert B.dssp_clock(ctx, K) == ([1] * K, [0] * K, [False] * K, 4)
    B.dssp_destroy(ctx)


def test_parameter_layout_matches_documented_one(oracle_nn):
    for model, ncls, want in [("mlp", 10, 789_258), ("alexnet_ds", 10, 1_387_786), ("alexnet_3c", 10, 1_352_714), ("resnet110", 100, 1_733_812),
                              ("resnet20", 100, None), ("resnet8", 7, None)]:
        mid = B.model_id(model)
        segs = B.dssp_model_segments(mid, ncls)
        net = oracle_nn.make_net(model, ncls)
        osegs = net.segments()
        assert [s[1] for s in segs] == [int(np.prod(shape)) for _, shape in osegs]
        for (kind, size, fan), (name, shape) in zip(segs, osegs):
            suffix = name.rsplit(".", 1)[1]
            assert kind == {"w": 0, "g": 2, "b": 3 if ".bn" in name else 1}[suffix]
            if kind == 0:
                assert fan == int(np.prod(shape[:-1]))
        n = B.dssp_model_param_count(mid, ncls)
        assert n == net.n_params() and (want is None or n == want)
        assert B.dssp_workspace_bytes(mid, 8, ncls, 2) == 2 * B.dssp_workspace_bytes(mid, 8, ncls, 1) > 0
    assert B.dssp_model_param_count(7, 10) < 0 and B.dssp_workspace_bytes(0, 8, 10, 2) == 0


def test_bench_refuses_more_than_one_gpu():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and "ONE GPU" in (p.stderr + p.stdout)


def test_oracle_is_not_imported_by_the_product():
    pkg = os.path.join(ROOT, "paper_1908_11848_amd")
    for fn in os.listdir(pkg):
        if fn.endswith(".py"):
            assert "oracle" not in open(os.path.join(pkg, fn)).read(), fn
    for fn in os.listdir(os.path.join(pkg, "csrc")):
        assert "oracle" not in open(os.path.join(pkg, "csrc", fn)).read(), fn


def test_paradigm_sweep_in_virtual_time():
    """The library's controller alone on the heterogeneous tables: the looser the paradigm, the sooner the server has
    its pushes (Sec. V-B: ASP fastest, BSP slowest, DSSP between SSP at its two bounds), workers never wait under ASP,
    and the staleness a worker is allowed to go on with respects each paradigm's bound."""
    from paper_1908_11848_amd import paradigms
    for config, K in ((3, 4), (4, 8)):
        res = dict(paradigms.sweep(config, K, 100 * K))
        rate = {k: v["pushes_per_unit_time"] for k, v in res.items()}
        assert rate["ASP"] >= rate["SSP s=15"] >= rate["DSSP (3,12)"] >= rate["SSP s=3"] >= rate["BSP"] > 0
        assert res["ASP"]["wait_fraction"] == 0 and res["BSP"]["wait_fraction"] > res["DSSP (3,12)"]["wait_fraction"] > 0
        assert res["BSP"]["staleness_max"] == 0 and res["SSP s=3"]["staleness_max"] <= 3
        assert res["SSP s=15"]["staleness_max"] <= 15 and res["DSSP (3,12)"]["staleness_max"] <= 15
        assert all(v["pushes"] == 100 * K for v in res.values())
        # staleness histograms: one entry per OK; nothing beyond the paradigm's bound; the averaged SSP of DSSP's
        # range (Sec. V-B) lies between SSP at the two ends, and DSSP keeps most OKs at or below its lower bound
        for name, v in res.items():
            h = v["staleness_hist"]
            assert len(h) == v["staleness_max"] + 1 and h[-1] > 0
            if name != "SSP s=3..15":            # (a mean of thirteen means, not the mean of the summed histogram)
                assert abs(sum(k * c for k, c in enumerate(h)) / sum(h) - v["staleness_mean"]) < 1e-9
        avg = res["SSP s=3..15"]
        assert rate["SSP s=15"] >= avg["pushes_per_unit_time"] >= rate["SSP s=3"]
        assert res["SSP s=3"]["staleness_mean"] <= avg["staleness_mean"] <= res["SSP s=15"]["staleness_mean"]
        hd = res["DSSP (3,12)"]["staleness_hist"]
        assert sum(hd[:4]) > 0.6 * sum(hd) and res["DSSP (3,12)"]["staleness_mean"] < avg["staleness_mean"]


def test_workers_are_dealt_onto_streams_by_their_rates():
    from paper_1908_11848_amd.emulation import deal
    rates = [1.0, 0.4, 0.9, 0.5, 0.8, 0.6, 0.7, 0.45]
    lane_of = deal(rates, 4)
    assert sorted(set(lane_of)) == [0, 1, 2, 3]
    load = [sum(r for r, l in zip(rates, lane_of) if l == lane) for lane in range(4)]
    assert max(load) - min(load) <= 0.11 and lane_of[0] == lane_of[1]          # fastest shares with slowest
    assert deal(rates, 4) == lane_of                                          # deterministic
    assert deal([1.0] * 8, 4) == [0, 1, 2, 3, 0, 1, 2, 3]                     # equal workers: round-robin
    assert deal([3.0, 1.0], 4) == [0, 1] and deal([1.0, 2.0, 3.0], 1) == [0, 0, 0]
