"""Paradigm sweep in virtual time: what the controller alone decides (Sec. V-B of the paper compares BSP, ASP,
SSP and DSSP by how fast the server receives pushes and how long workers wait).

Runs the library's host-side controller (a context without device memory, so no GPU is needed) on the seeded
iteration-time tables of the workloads, and reports per paradigm

    pushes per unit of virtual time   (1 unit = 1e6 ticks = one nominal iteration)
    wait fraction                     blocked time summed over the workers / (K x run time)
    staleness at OK                   t_p - min t when a worker is allowed to go on: mean, maximum and histogram

"SSP s=3..15" is the mean over the thirteen SSP thresholds of DSSP's range, the "averaged SSP" Sec. V-B sets
against DSSP (3,12).

    python -m paper_1908_11848_amd.paradigms [--pushes N] [--hist]
"""
import argparse

from . import binding as B, driver, inputs

PARADIGMS = (("BSP", 0, 0), ("SSP s=3", 3, 0), ("SSP s=15", 15, 0), ("DSSP (3,12)", 3, 12), ("ASP", B.DSSP_S_L_NEVER_WAIT, 0))


def run(K, s_L, r_max, durations, total):
    """One schedule of `total` pushes through the C ABI; returns a dict of the figures above."""
    ctx = B.dssp_create(None, 0, K, s_L, r_max, 0.01)
    try:
        log, st = driver.run_schedule(ctx, K, durations, total=total)
    finally:
        B.dssp_destroy(ctx)
    blocked_at, waited = {}, 0
    t = [0] * K
    stale = []
    for kind, p, T, tp, rp, v, a0, a1 in log:
        if kind == driver.PUSH:
            t[p] = tp
        elif kind == driver.BLOCK:
            blocked_at[p] = T
        elif kind == driver.RELEASE:
            waited += T - blocked_at.pop(p)
            stale.append(tp - min(t))
        elif kind == driver.OK:
            stale.append(tp - min(t))
    T_end = st["T_end"]
    hist = [0] * (max(stale) + 1 if stale else 1)
    for v in stale:
        hist[v] += 1
    return {"pushes": st["pushes"], "T_end": T_end, "pushes_per_unit_time": st["pushes"] / (T_end / 1e6),
            "wait_fraction": waited / (K * T_end), "staleness_mean": sum(stale) / max(1, len(stale)),
            "staleness_max": max(stale) if stale else 0, "staleness_hist": hist}


def averaged_ssp(K, durations, total, s_from=3, s_to=15):
    """Mean of the figures over SSP with every threshold in [s_from, s_to]; the histogram is the sum of theirs."""
    runs = [run(K, s, 0, durations, total) for s in range(s_from, s_to + 1)]
    out = {k: sum(r[k] for r in runs) / len(runs) for k in ("pushes", "T_end", "pushes_per_unit_time", "wait_fraction", "staleness_mean")}
    out["staleness_max"] = max(r["staleness_max"] for r in runs)
    hist = [0] * (out["staleness_max"] + 1)
    for r in runs:
        for v, c in enumerate(r["staleness_hist"]):
            hist[v] += c
    out["staleness_hist"] = hist
    return out


def sweep(config, K, total):
    """Every paradigm on the same table, until the server has received `total` pushes (fast workers push more often
    under the looser paradigms, so the same number of pushes takes less time)."""
    d = inputs.durations(config, K, total + 1)
    out = [(name, run(K, s_L, r_max, d, total)) for name, s_L, r_max in PARADIGMS]
    out.insert(3, ("SSP s=3..15", averaged_ssp(K, d, total)))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--pushes", type=int, default=200, help="pushes per worker on average (total = K x this)")
    ap.add_argument("--hist", action="store_true", help="also print the staleness histograms (share of the OKs per staleness)")
    a = ap.parse_args()
    for config, K, what in ((3, 4, "4 workers, iteration times (1, 1, 2, 3.5) x exp(0.1 z)"),
                            (4, 8, "8 workers, iteration times U[1, 2.5] drawn once per worker")):
        print("configuration %d: %s; %d pushes in all" % (config, what, K * a.pushes))
        print("  %-12s %22s %14s %22s" % ("paradigm", "pushes / unit time", "wait fraction", "staleness mean / max"))
        for name, r in sweep(config, K, K * a.pushes):
            print("  %-12s %22.3f %14.3f %15.2f / %d" % (name, r["pushes_per_unit_time"], r["wait_fraction"],
                                                        r["staleness_mean"], r["staleness_max"]))
            if a.hist and name != "ASP":
                n = sum(r["staleness_hist"])
                print("      " + " ".join("%d:%.2f" % (v, c / n) for v, c in enumerate(r["staleness_hist"]) if c))


if __name__ == "__main__":
    main()
