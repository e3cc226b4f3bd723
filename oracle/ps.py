"""Oracle, part 3: the whole emulated parameter-server run, numerics included.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Worker side (Alg. 1, worker part): after OK, pull the global weights, replace
the local weights, compute the mini-batch gradient on them, push it.
Server side (Alg. 1, server part, step 2): w <- w - scale * g per push, one
push at a time in (timestamp, worker) order.  scale = lr / K, the reading
under which s_L = r_max = 0 is synchronous SGD on the gradient averaged over
the K workers (Sec. I-A: BSP equals single-machine training).

Weights, gradients and the update are fp64 here.  The order of everything is
dictated by the integer simulator of dssp_rules.py.
"""

import numpy as np

from . import dssp_rules


def run(K, s_L, r_max, lr, w0, durations, grad_fn, quota=None, total=None, keep_grads=False,
        keep_snapshots=False):
    """grad_fn(p, n, w_local) -> (loss, g): gradient of worker p's n-th iteration
    (n from 0) on its local weights.  Returns dict(log, w, state, stats, pushes)
    where pushes[i] = dict(worker, n, pulled_version, loss[, g][, w_local]) in apply order
    (w_local: the snapshot the gradient was computed on, narrowed to float32)."""
    w = np.array(w0, dtype=np.float64)
    scale = float(lr) / float(K)
    w_local = [None] * K
    pushes = []

    def on_pull(p, version):
        w_local[p] = w.copy()

    def on_push(p, n, pulled_version):
        loss, g = grad_fn(p, n, w_local[p])
        rec = dict(worker=p, n=n, pulled_version=pulled_version, loss=loss)
        if keep_grads:
            rec["g"] = np.array(g, dtype=np.float64)
        if keep_snapshots:
            rec["w_local"] = w_local[p].astype(np.float32)
        pushes.append(rec)
        np.subtract(w, scale * np.asarray(g, dtype=np.float64), out=w)

    log, st, stats = dssp_rules.simulate(K, s_L, r_max, durations, quota=quota, total=total,
                                         on_pull=on_pull, on_push=on_push)
    return dict(log=log, w=w, state=st, stats=stats, pushes=pushes)


def model_grad_fn(net, xs, ys):
    """xs[p][j], ys[p][j]: pool of mini-batches of worker p, cycled over iterations."""
    def fn(p, n, w_local):
        j = n % len(xs[p])
        loss, g, _ = net.loss_and_grad(w_local, xs[p][j], ys[p][j])
        return loss, g
    return fn
