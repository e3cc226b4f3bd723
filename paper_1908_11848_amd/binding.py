"""ctypes binding of libdssp.so: the same names as include/dssp.h, argument marshalling only.

Device pointers may be given as ints or as anything with .data_ptr() (torch tensors); streams
as ints or objects with .cuda_stream.  Every wrapper raises DsspError on a negative return code.
There is no fallback: if the library is not built, loading raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdssp.so")

DSSP_OK, DSSP_EINVAL, DSSP_ESTATE, DSSP_EHIP, DSSP_ENOMEM = 0, -1, -2, -3, -4
DSSP_MODEL_NONE, DSSP_MODEL_MLP, DSSP_MODEL_ALEXNET_DS, DSSP_MODEL_RESNET110 = 0, 1, 2, 110
DSSP_S_L_NEVER_WAIT = 2**31 - 1

MODEL_IDS = {"none": 0, "mlp": 1, "alexnet_ds": 2, "alexnet_3c": 3}


def model_id(name):
    """'mlp' | 'alexnet_ds' | 'alexnet_3c' | 'resnet<6n+2>' | 'none' -> model id of the C ABI."""
    if name in MODEL_IDS:
        return MODEL_IDS[name]
    if name.startswith("resnet"):
        return int(name[len("resnet"):])
    raise ValueError(name)


class DsspError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("libdssp error %d: %s" % (code, msg))
        self.code = code


_lib = None
c_void_p, c_int, c_int64, c_float, c_size_t = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
c_long = ctypes.c_long
P = ctypes.POINTER

_SIGNATURES = {
    # include/dssp.h
    "dssp_create": (c_int, [P(c_void_p), c_void_p, c_int64, c_int, c_int, c_int, c_float]),
    "dssp_set_stream": (c_int, [c_void_p, c_int, c_void_p]),
    "dssp_set_model": (c_int, [c_void_p, c_int, c_int, c_int, c_void_p, c_size_t]),
    "dssp_pull": (c_int, [c_void_p, c_int, c_void_p, P(ctypes.c_uint64)]),
    "dssp_worker_step": (c_int, [c_void_p, c_int, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
    "dssp_push": (c_int, [c_void_p, c_int, c_void_p, c_int64, P(c_int), P(c_int), P(c_int), P(c_int), P(c_int)]),
    "dssp_push_pull": (c_int, [c_void_p, c_int, c_void_p, c_int64, c_void_p, P(c_int), P(c_int), P(c_int), P(c_int), P(c_int),
                               P(c_int), P(ctypes.c_uint64)]),
    "dssp_push_many": (c_int, [c_void_p, c_int, P(c_int), P(c_void_p), c_int64, P(c_void_p), P(c_int), P(c_int), P(c_int), P(c_int),
                               P(c_int), P(ctypes.c_uint64)]),
    "dssp_worker_step_timed": (c_int, [c_void_p, c_int, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int]),
    "dssp_step_done": (c_int, [c_void_p, c_int, P(c_int), P(c_int64), P(c_int64), P(c_int64)]),
    "dssp_clock": (c_int, [c_void_p, P(c_int64), P(ctypes.c_int32), P(ctypes.c_uint8), P(ctypes.c_uint64)]),
    "dssp_device_stamps": (c_int, [c_void_p, P(ctypes.c_uint64)]),
    "dssp_synchronize": (c_int, [c_void_p]),
    "dssp_stream_queues": (c_int, [P(c_void_p), c_int, P(c_int), P(c_int)]),
    "dssp_last_error": (ctypes.c_char_p, [c_void_p]),
    "dssp_destroy": (c_int, [c_void_p]),
    "dssp_model_param_count": (c_int64, [c_int, c_int]),
    "dssp_model_segments": (c_int, [c_int, c_int, P(ctypes.c_int32), P(c_int64), P(c_int64), c_int]),
    "dssp_workspace_bytes": (c_size_t, [c_int, c_int, c_int, c_int]),
    "dssp_workspace_tensor": (c_int, [c_int, c_int, c_int, c_int, c_int, c_int, c_int, P(c_size_t), P(c_int64)]),
    # include/dssp_kernels.h
    "dsspk_apply": (c_int, [c_void_p, c_void_p, c_void_p, c_int64, c_float, c_void_p, ctypes.c_uint64]),
    "dsspk_pull": (c_int, [c_void_p, c_void_p, c_void_p, c_int64, c_void_p, c_void_p]),
    "dsspk_apply_pull": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, ctypes.c_float, c_void_p, c_void_p, ctypes.c_uint64]),
    "dsspk_apply_many": (c_int, [c_void_p, c_void_p, c_int, P(c_void_p), c_int64, c_float, c_int, P(c_void_p), P(c_int), P(c_void_p),
                                 c_void_p, ctypes.c_uint64]),
    "dsspk_clock_khz": (c_int, []),
    "dsspk_clock_stamp": (c_int, [c_void_p, c_void_p, c_void_p]),
    "dsspk_clock_stretch": (c_int, [c_void_p, c_void_p, c_int, ctypes.c_uint64, c_void_p, c_void_p]),
    "dsspk_gemm": (c_int, [c_void_p, c_void_p, c_long, c_long, c_void_p, c_long, c_long, c_void_p, c_long,
                           c_int, c_int, c_int, c_void_p, c_int]),
    "dsspk_gemm_splitk_layers": (c_int, [c_int, c_int, c_int]),
    "dsspk_gemm_splitk": (c_int, [c_void_p, c_void_p, c_long, c_long, c_void_p, c_long, c_long, c_void_p, c_long,
                                  c_int, c_int, c_int, c_void_p, c_int, c_void_p, c_int]),
    "dsspk_colsum": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_long, c_int]),
    "dsspk_colsum_scratch_floats": (c_size_t, [c_long, c_int]),
    "dsspk_colsum_noalloc": (c_int, [c_void_p, c_void_p, c_void_p, c_long, c_int]),
    "dsspk_conv_fwd": (c_int, [c_void_p] * 5 + [c_int] * 10 + [c_void_p]),
    "dsspk_conv_fwd_stat_parts": (c_int, [c_int] * 9),
    "dsspk_conv_fwd_prebn": (c_int, [c_void_p, c_void_p, c_void_p, c_int, c_void_p, c_void_p, c_float, c_void_p, c_void_p,
                                     c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int]),
    "dsspk_conv_bwd_data": (c_int, [c_void_p] * 5 + [c_int] * 9),
    "dsspk_conv_bwd_weight": (c_int, [c_void_p] * 5 + [c_int] * 9),
    "dsspk_conv_wgrad_scratch_floats": (c_size_t, [c_int] * 9),
    "dsspk_relu_bwd": (c_int, [c_void_p, c_void_p, c_void_p, c_long]),
    "dsspk_add": (c_int, [c_void_p, c_void_p, c_void_p, c_long]),
    "dsspk_maxpool_fwd": (c_int, [c_void_p] * 4 + [c_int] * 4),
    "dsspk_maxpool_bwd": (c_int, [c_void_p] * 4 + [c_int] * 4),
    "dsspk_maxpool_bwd_relu": (c_int, [c_void_p] * 5 + [c_int] * 4),
    "dsspk_bn_fwd": (c_int, [c_void_p] * 7 + [c_long, c_int, c_float, c_int, c_int, c_void_p, c_int, c_int, c_int, c_int]),
    "dsspk_bn_bwd": (c_int, [c_void_p] * 10 + [c_long, c_int]),
    "dsspk_bn_bwd_reduce": (c_int, [c_void_p] * 6 + [c_long, c_int]),
    "dsspk_bn_bwd_dx": (c_int, [c_void_p] * 9 + [c_long, c_int, c_int]),
    "dsspk_conv_bwd_data_post": (c_int, [c_void_p] * 9 + [c_int] * 3),
    "dsspk_conv_bwd_data_bn": (c_int, [c_void_p] * 16 + [c_int] * 5),
    "dsspk_conv_bwd_data_bn_wgrad": (c_int, [c_void_p] * 16 + [c_int] * 5),
    "dsspk_conv_bwd_fused_chunks": (c_int, [c_int] * 3),
    "dsspk_conv_bwd_weight_parts": (c_int, [c_void_p] * 4 + [c_int] * 9 + [c_void_p, c_int, c_int] + [c_void_p] * 4),
    "dsspk_wgrad_reduce": (c_int, [c_void_p] * 3 + [c_int] * 2),
    "dsspk_bn_bwd_totals": (c_int, [c_void_p, c_void_p, c_int, c_int] + [c_void_p] * 3),
    "dsspk_bn_scratch_floats": (c_size_t, [c_long, c_int]),
    "dsspk_shortcut_bwd_acc": (c_int, [c_void_p] * 3 + [c_int] * 4),
    "dsspk_gap_fwd": (c_int, [c_void_p] * 3 + [c_int] * 3),
    "dsspk_gap_bwd": (c_int, [c_void_p] * 3 + [c_int] * 3),
    "dsspk_softmax_xent": (c_int, [c_void_p] * 5 + [c_int] * 2),
}


def lib():
    """Loads libdssp.so (once).  Raises if it has not been built: there is no other path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s not found: build it with `python -m paper_1908_11848_amd.buildlib`" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(L, name)          # AttributeError if a declared symbol is not exported
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def ptr(x):
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


def stream_handle(s):
    if s is None:
        return None
    return s.cuda_stream if hasattr(s, "cuda_stream") else int(s)


def _check(ctx, rc):
    if rc < 0:
        msg = lib().dssp_last_error(ctx).decode() if ctx else ""
        raise DsspError(rc, msg)
    return rc


def dssp_create(params_dev, n_params, K, s_L, r_max, lr):
    ctx = c_void_p()
    rc = lib().dssp_create(ctypes.byref(ctx), ptr(params_dev), n_params, K, s_L, r_max, lr)
    if rc < 0:
        raise DsspError(rc, "dssp_create")
    return ctx


def dssp_set_stream(ctx, worker, stream):
    _check(ctx, lib().dssp_set_stream(ctx, worker, stream_handle(stream)))


def dssp_set_model(ctx, model, batch, n_classes, workspace_dev, workspace_bytes):
    _check(ctx, lib().dssp_set_model(ctx, model, batch, n_classes, ptr(workspace_dev), workspace_bytes))


def dssp_pull(ctx, worker, dst_dev):
    v = ctypes.c_uint64()
    _check(ctx, lib().dssp_pull(ctx, worker, ptr(dst_dev), ctypes.byref(v)))
    return v.value


def dssp_worker_step(ctx, worker, x_dev, y_dev, w_local_dev, grad_dev, loss_dev=None):
    _check(ctx, lib().dssp_worker_step(ctx, worker, ptr(x_dev), ptr(y_dev), ptr(w_local_dev), ptr(grad_dev), ptr(loss_dev)))


def dssp_push(ctx, worker, grad_dev, t_push_ticks, K):
    """-> (ok, released list, r*, grant)"""
    ok, n_rel, rstar, grant = c_int(), c_int(), c_int(), c_int()
    rel = (c_int * K)()
    _check(ctx, lib().dssp_push(ctx, worker, ptr(grad_dev), int(t_push_ticks), ctypes.byref(ok), rel,
                                ctypes.byref(n_rel), ctypes.byref(rstar), ctypes.byref(grant)))
    return bool(ok.value), list(rel[:n_rel.value]), rstar.value, grant.value


def dssp_push_pull(ctx, worker, grad_dev, t_push_ticks, K, pull_dst_dev):
    """-> (ok, released list, r*, grant, pulled, version): as dssp_push; pulled = the pusher's snapshot of the new
    weights was written to pull_dst_dev by the same kernel (it was granted OK), so it must not call dssp_pull."""
    ok, n_rel, rstar, grant, pulled = c_int(), c_int(), c_int(), c_int(), c_int()
    v = ctypes.c_uint64()
    rel = (c_int * K)()
    _check(ctx, lib().dssp_push_pull(ctx, worker, ptr(grad_dev), int(t_push_ticks), ptr(pull_dst_dev), ctypes.byref(ok), rel,
                                     ctypes.byref(n_rel), ctypes.byref(rstar), ctypes.byref(grant), ctypes.byref(pulled),
                                     ctypes.byref(v)))
    return bool(ok.value), list(rel[:n_rel.value]), rstar.value, grant.value, bool(pulled.value), v.value


def dssp_push_many(ctx, workers, grads_dev, t_push_ticks, K, pull_dst_dev):
    """workers: ascending indices; grads_dev[j]: gradient of workers[j]; pull_dst_dev[q]: snapshot buffer of worker q (all K).
    -> (ok list, released lists (one per push), r* list, grant list, pulled_version list [K] (0 = no snapshot))"""
    m = len(workers)
    wk = (c_int * m)(*workers)
    g = (c_void_p * m)(*[ptr(x) for x in grads_dev])
    dst = (c_void_p * K)(*[ptr(x) for x in pull_dst_dev])
    ok, rstar, grant, n_rel = (c_int * m)(), (c_int * m)(), (c_int * m)(), (c_int * m)()
    rel = (c_int * K)()
    pv = (ctypes.c_uint64 * K)()
    _check(ctx, lib().dssp_push_many(ctx, m, wk, g, int(t_push_ticks), dst, ok, rstar, grant, n_rel, rel, pv))
    released, at = [], 0
    for j in range(m):
        released.append(list(rel[at:at + n_rel[j]]))
        at += n_rel[j]
    return [bool(x) for x in ok], released, list(rstar), list(grant), list(pv)


def dssp_worker_step_timed(ctx, worker, x_dev, y_dev, w_local_dev, grad_dev, loss_dev=None, slowdown_permille=1000):
    _check(ctx, lib().dssp_worker_step_timed(ctx, worker, ptr(x_dev), ptr(y_dev), ptr(w_local_dev), ptr(grad_dev), ptr(loss_dev),
                                             int(slowdown_permille)))


def dssp_step_done(ctx, worker):
    """-> None while the worker's timed step is still on its stream, else (t_start, t_gradient, t_done) in microseconds"""
    done = c_int()
    a, b, c = c_int64(), c_int64(), c_int64()
    _check(ctx, lib().dssp_step_done(ctx, worker, ctypes.byref(done), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
    return (a.value, b.value, c.value) if done.value else None


def dssp_clock(ctx, K):
    """-> (t list, r list, blocked list, version)"""
    t = (c_int64 * K)()
    r = (ctypes.c_int32 * K)()
    b = (ctypes.c_uint8 * K)()
    v = ctypes.c_uint64()
    _check(ctx, lib().dssp_clock(ctx, t, r, b, ctypes.byref(v)))
    return list(t), list(r), [bool(x) for x in b], v.value


def dssp_device_stamps(ctx, K):
    s = (ctypes.c_uint64 * (K + 1))()
    _check(ctx, lib().dssp_device_stamps(ctx, s))
    return list(s)


def dssp_synchronize(ctx):
    _check(ctx, lib().dssp_synchronize(ctx))


def dssp_stream_queues(streams):
    """-> (queue number of each stream, number of hardware queues seen)"""
    n = len(streams)
    h = (c_void_p * n)(*[stream_handle(s) for s in streams])
    q = (c_int * n)()
    nq = c_int()
    rc = lib().dssp_stream_queues(h, n, q, ctypes.byref(nq))
    if rc < 0:
        raise DsspError(rc, "dssp_stream_queues")
    return list(q), nq.value


def dssp_destroy(ctx):
    lib().dssp_destroy(ctx)


def dssp_model_param_count(model, n_classes):
    return lib().dssp_model_param_count(model, n_classes)


def dssp_model_segments(model, n_classes):
    """-> [(kind, size, fan_in)] in flat-vector order"""
    n = lib().dssp_model_segments(model, n_classes, None, None, None, 0)
    if n < 0:
        raise DsspError(n, "unknown model")
    kind = (ctypes.c_int32 * n)()
    size = (c_int64 * n)()
    fan = (c_int64 * n)()
    lib().dssp_model_segments(model, n_classes, kind, size, fan, n)
    return [(kind[i], size[i], fan[i]) for i in range(n)]


def dssp_workspace_bytes(model, batch, n_classes, K):
    return lib().dssp_workspace_bytes(model, batch, n_classes, K)


def dssp_workspace_tensor(model, batch, n_classes, K, worker, what, index):
    """-> (byte offset, count) or None past the last tensor of that kind"""
    off, cnt = c_size_t(), c_int64()
    rc = lib().dssp_workspace_tensor(model, batch, n_classes, K, worker, what, index, ctypes.byref(off), ctypes.byref(cnt))
    return None if rc < 0 else (off.value, cnt.value)
