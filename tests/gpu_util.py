"""Helpers for the GPU parity tests: device buffers through torch, and the gradient parity protocol."""
import numpy as np
import torch


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


def stream_ptr():
    return torch.cuda.current_stream().cuda_stream


def gradient_parity(net, em, p, w_local, x, y):
    """Gradient of worker p's last step against the oracle's for the same snapshot and batch.  ReLU's derivative and
    max-pool routing are decided by comparing floats, fp32 here and fp64 there, so a comparison whose margin is
    below the fp32 forward error may fall either way, and both outcomes are valid.  Hence: (1) every saved
    activation of the GPU matches the oracle's forward to fp32 accuracy; (2) wherever the GPU decided differently,
    the oracle re-runs with that decision forced - and refuses unless its own margin is a near-tie (<= 1e-4);
    (3) the gradients are then compared.  Returns (relative L2 error, number of near-ties resolved)."""
    loss_o, g_o, trace = net.loss_and_grad(w_local, x, y)
    g_gpu, loss_gpu = em.worker_grad(p)
    tie, nflip = {}, 0
    i = 0
    while ("relu", i) in trace:
        z, act = trace[("relu", i)]["z"], trace[("relu", i)]["active"].astype(bool)
        a_gpu = em.workspace_tensor(p, 0, i).reshape(z.shape)
        err = np.abs(a_gpu - np.maximum(z, 0))
        assert err.max() <= 2e-5 * (1 + np.abs(z).max()), ("forward activation", i, err.max())
        diff = (a_gpu > 0) != act
        if diff.any():
            forced = np.full(z.shape, -1, dtype=np.int8)
            forced[diff] = (a_gpu > 0)[diff]
            tie[("relu", i)] = forced
            nflip += int(diff.sum())
        i += 1
    i = 0
    while ("pool", i) in trace:
        arg = trace[("pool", i)]["arg"]
        arg_gpu = em.workspace_tensor(p, 1, i).reshape(arg.shape).astype(np.int32)
        diff = arg_gpu != arg
        if diff.any():
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
    return rel_l2(g_gpu, g_o), nflip
