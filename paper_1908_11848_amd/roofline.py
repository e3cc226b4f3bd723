"""Live per-kernel timing for the benchmark's roofline fields.

Each measurement launches one kernel of the worker step, at the shape and launch configuration
the benchmark's workload uses, `reps` times back to back on one stream, bracketed by HIP events
recorded on that same stream.  Algorithmic work per launch is stated next to each entry.
Peaks: fp32 matrix cores 157.3 TFLOP/s (256 CUs x 4 SIMDs x 64 FLOP/cycle x 2.4 GHz), HBM 8 TB/s.
"""
import torch

from . import binding as B

PEAK_MFMA_F32 = 157.3e12
PEAK_HBM = 8.0e12


def _time(fn, stream, reps=50, warm=5):
    with torch.cuda.stream(stream):
        for _ in range(warm):
            fn(stream.cuda_stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn(stream.cuda_stream)
        e1.record(stream)
    e1.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / reps


def _conv_case(N, H, Cin, Cout, k, s, p, which, dev):
    L = B.lib()
    Ho = (H + 2 * p - k) // s + 1
    x = torch.randn(N, H, H, Cin, device=dev)
    w = torch.randn(k, k, Cin, Cout, device=dev) * 0.1
    y = torch.empty(N, Ho, Ho, Cout, device=dev)
    dy = torch.randn(N, Ho, Ho, Cout, device=dev)
    dx = torch.empty_like(x)
    dw = torch.empty_like(w)
    scr = torch.empty(max(1, L.dsspk_conv_wgrad_scratch_floats(N, H, H, Cin, Cout, k, k, s, p)), device=dev)
    flops = 2.0 * N * Ho * Ho * Cout * k * k * Cin
    if which == "fwd":
        fn = lambda st: L.dsspk_conv_fwd(st, x.data_ptr(), w.data_ptr(), None, y.data_ptr(), N, H, H, Cin, Cout, k, k, s, p, 0)
    elif which == "dgrad":
        fn = lambda st: L.dsspk_conv_bwd_data(st, dy.data_ptr(), w.data_ptr(), None, dx.data_ptr(), N, H, H, Cin, Cout, k, k, s, p)
    else:
        fn = lambda st: L.dsspk_conv_bwd_weight(st, x.data_ptr(), dy.data_ptr(), dw.data_ptr(), scr.data_ptr(), N, H, H, Cin, Cout, k, k, s, p)
    keep = (x, w, y, dy, dx, dw, scr)
    return fn, flops, keep


def _entry(bound, achieved, peak, unit, name, work):
    return {"kernel": name, "bound": bound, "achieved": round(achieved, 3), "peak": peak, "unit": unit,
            "frac": round(achieved / peak, 5), "traffic": None, "work_per_launch": work}


def conv_entry(N, H, Cin, Cout, k, s, p, which, stream, dev, name):
    fn, flops, keep = _conv_case(N, H, Cin, Cout, k, s, p, which, dev)
    t = _time(fn, stream)
    e = _entry("mfma", flops / t / 1e12, PEAK_MFMA_F32 / 1e12, "TFLOP/s", name, "%.1f MFLOP" % (flops / 1e6))
    e["avg_us"] = round(t * 1e6, 2)
    return e


def server_entries(n, stream, dev):
    L = B.lib()
    w = torch.randn(n, device=dev)
    g = torch.randn(n, device=dev) * 1e-3
    dst = torch.empty(n, device=dev)
    st = torch.zeros(2, dtype=torch.int64, device=dev)
    ta = _time(lambda s: L.dsspk_apply(s, w.data_ptr(), g.data_ptr(), n, 1e-3, st.data_ptr(), 1), stream)
    tp = _time(lambda s: L.dsspk_pull(s, dst.data_ptr(), w.data_ptr(), n, st[1:].data_ptr(), st.data_ptr()), stream)
    ea = _entry("hbm", 12.0 * n / ta / 1e9, PEAK_HBM / 1e9, "GB/s", "apply_kernel (%d params)" % n, "%.1f MB" % (12.0 * n / 1e6))
    ep = _entry("hbm", 8.0 * n / tp / 1e9, PEAK_HBM / 1e9, "GB/s", "pull_kernel (%d params)" % n, "%.1f MB" % (8.0 * n / 1e6))
    ea["avg_us"], ep["avg_us"] = round(ta * 1e6, 2), round(tp * 1e6, 2)
    return ea, ep


def measure(workload, em):
    """The dominant kernel of the workload."""
    dev, stream = em.dev, em.streams[0]
    if workload == "stress":
        return server_entries(em.n, stream, dev)[0]
    if workload == "alexnet_ds":
        return conv_entry(128, 15, 64, 64, 5, 1, 2, "fwd", stream, dev, "conv_igemm_kernel<64,64,fwd> 5x5 64->64 @15x15, batch 128")
    if workload == "mlp":
        return server_entries(em.n, stream, dev)[0]
    return conv_entry(128, 32, 16, 16, 3, 1, 1, "wgrad", stream, dev,
                      "conv_wgrad_kernel<1,1> + reduce, 3x3 16->16 @32x32, batch 128")


def measure_others(workload, em):
    dev, stream = em.dev, em.streams[0]
    out = []
    if workload == "resnet110":
        for (H, C) in ((32, 16), (16, 32), (8, 64)):
            for which in ("fwd", "dgrad", "wgrad"):
                out.append(conv_entry(128, H, C, C, 3, 1, 1, which, stream, dev, "conv %s 3x3 %d->%d @%dx%d, batch 128" % (which, C, C, H, H)))
        out += list(server_entries(em.n, stream, dev))
        out += list(server_entries(25_000_000, stream, dev))
    elif workload != "stress":
        out += list(server_entries(em.n, stream, dev))
    else:
        out.append(server_entries(em.n, stream, dev)[1])
    return out
