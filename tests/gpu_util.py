"""Helpers for the GPU parity tests: device buffers through torch, and the gradient parity protocol."""
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def dev(a):
    """numpy -> device tensor (same dtype; float64 is narrowed to float32)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float64:
        a = a.astype(np.float32)
    return torch.from_numpy(a).cuda()


def empty(shape, dtype=torch.float32):
    # filled with NaN so that an element a kernel forgets to write is noticed
    t = torch.empty(shape, dtype=dtype, device="cuda")
    if dtype.is_floating_point:
        t.fill_(float("nan"))
    else:
        t.fill_(113)
    return t


def host(t):
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def max_abs(a, b):
    """Largest element-wise difference, relative to the largest magnitude of the expected values."""
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    if a.size == 0:
        return 0.0
    return float(np.max(np.abs(a - b)) / max(float(np.max(np.abs(b))), 1e-300))


def stream_ptr():
    return torch.cuda.current_stream().cuda_stream


_T0 = time.time()
PYTEST_CONFIG = None        # set by conftest.pytest_configure


def progress(msg):
    """One line that reaches the terminal even while pytest captures output (a long oracle run must not look hung)."""
    line = "[%6.0fs] %s" % (time.time() - _T0, msg)
    capman = PYTEST_CONFIG.pluginmanager.getplugin("capturemanager") if PYTEST_CONFIG is not None else None
    if capman is not None:
        with capman.global_and_fixture_disabled():
            print(line, file=sys.stderr, flush=True)
    else:
        print(line, file=sys.stderr, flush=True)
    d = os.environ.get("DSSP_TEST_PROGRESS_DIR")        # optionally also into a file of the caller's choosing
    if d:
        try:
            os.makedirs(d, exist_ok=True)
            with open(os.path.join(d, "test_progress.log"), "a") as f:
                f.write(line + "\n")
        except OSError:
            pass


MARGIN_FACTOR = 8.0         # a decision may differ only where the oracle's margin is within this many forward errors
MARGIN_CEILING = 1e-4       # ... and never beyond this (the oracle refuses to force anything farther from a tie)


def gradient_parity(net, em, p, w_local, x, y, stats=None):
    """Gradient of worker p's last step against the oracle's for the same snapshot and batch.  ReLU's derivative and
    max-pool routing are decided by comparing floats, fp32 here and fp64 there, so a comparison whose margin is
    below the fp32 forward error may fall either way, and both outcomes are valid.  Hence:
      (1) every saved activation of the GPU matches the oracle's forward to fp32 accuracy; the largest error of a
          layer over the elements decided alike is that layer's measured forward error e_i;
      (2) where the GPU decided differently, the oracle's own margin (|z| of a ReLU, max minus the chosen value of a
          pool window) must be <= 8 e_i (and <= 1e-4), and no more decisions may differ than ten times the number the
          oracle has within e_i of a tie (a kernel that dropped small activations would fail both);
      (3) the oracle re-runs with those decisions forced (it refuses any that is farther than 1e-4 from a tie) and
          the gradients are compared.
    Returns (relative L2 error, number of near-ties resolved); stats (a dict) receives the largest differing margin,
    the largest forward error and the largest element-wise gradient error."""
    loss_o, g_o, trace = net.loss_and_grad(w_local, x, y)
    g_gpu, loss_gpu = em.worker_grad(p)
    tie, nflip = {}, 0
    worst_margin, worst_err = 0.0, 0.0
    relu_err = {}
    i = 0
    while ("relu", i) in trace:
        z, act = trace[("relu", i)]["z"], trace[("relu", i)]["active"].astype(bool)
        a_gpu = em.workspace_tensor(p, 0, i).reshape(z.shape)
        assert np.isfinite(a_gpu).all(), ("forward activation not finite", i)
        err = np.abs(a_gpu - np.maximum(z, 0))
        diff = (a_gpu > 0) != act
        e_i = float(err[~diff].max()) if (~diff).any() else 0.0
        assert e_i <= 2e-5 * (1 + np.abs(z).max()), ("forward activation", i, e_i)
        relu_err[i] = e_i
        worst_err = max(worst_err, e_i)
        if diff.any():
            margin = float(np.abs(z[diff]).max())
            allowed = min(MARGIN_FACTOR * e_i, MARGIN_CEILING)
            assert margin <= allowed, ("ReLU decided differently away from a tie", i, margin, allowed, e_i, float(np.abs(z).max()))
            n_i = int(diff.sum())
            near = int((np.abs(z) <= e_i).sum())
            assert n_i <= 10 * max(near, 1), ("too many differing ReLU decisions", i, n_i, near)
            worst_margin = max(worst_margin, margin)
            forced = np.full(z.shape, -1, dtype=np.int8)
            forced[diff] = (a_gpu > 0)[diff]
            tie[("relu", i)] = forced
            nflip += n_i
        i += 1
    i = 0
    while ("pool", i) in trace:
        arg, xin = trace[("pool", i)]["arg"], trace[("pool", i)]["x"]
        arg_gpu = em.workspace_tensor(p, 1, i).reshape(arg.shape).astype(np.int32)
        diff = arg_gpu != arg
        if diff.any():
            n, ho, wo, c = np.nonzero(diff)
            v_o = xin[n, 2 * ho + arg[diff] // 3, 2 * wo + arg[diff] % 3, c]
            v_g = xin[n, 2 * ho + arg_gpu[diff] // 3, 2 * wo + arg_gpu[diff] % 3, c]
            margin = float(np.max(v_o - v_g))
            e_i = relu_err.get(i, worst_err)            # pool i reads the output of ReLU i in these networks
            allowed = min(MARGIN_FACTOR * e_i, MARGIN_CEILING)
            assert margin <= allowed, ("max-pool chose differently away from a tie", i, margin, allowed)
            near = int((trace[("pool", i)]["gap"] <= e_i).sum())
            assert int(diff.sum()) <= 10 * max(near, 1), ("too many differing max-pool choices", i, int(diff.sum()), near)
            worst_margin = max(worst_margin, margin)
            forced = np.full(arg.shape, -1, dtype=np.int32)
            forced[diff] = arg_gpu[diff]
            tie[("pool", i)] = forced
            nflip += int(diff.sum())
        i += 1
    logits_gpu = em.workspace_tensor(p, 2, 0).reshape(trace["logits"].shape)
    assert rel_l2(logits_gpu, trace["logits"]) < 2e-5
    assert abs(loss_gpu - loss_o) < 2e-5 * max(1.0, abs(loss_o))
    if tie:
        _, g_o, _ = net.loss_and_grad(w_local, x, y, tie_break=tie)     # raises unless every forced decision is a near-tie
    if stats is not None:
        stats["margin"] = max(stats.get("margin", 0.0), worst_margin)
        stats["forward_err"] = max(stats.get("forward_err", 0.0), worst_err)
        stats["layer_forward_err"] = relu_err
        stats["grad_max_abs"] = max(stats.get("grad_max_abs", 0.0), max_abs(g_gpu, g_o))
    return rel_l2(g_gpu, g_o), nflip
