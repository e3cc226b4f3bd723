"""Helpers for the GPU parity tests: device buffers through torch, nothing else."""
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
