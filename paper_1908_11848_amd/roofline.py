"""Per-kernel measurements for the benchmark's roofline fields.

Every case launches one kernel family of the worker step (or of the server) at the shape and
launch configuration the ResNet-110 / batch 128 workload uses, through the exported `dsspk_*`
launchers.  `measure_*` time `reps` back-to-back launches on ONE stream with HIP events recorded
on that same stream.  Run as a program it launches every case a few times and exits, which is
what the hardware-counter passes are taken on:

    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d gpurun_out/pmc_fetch -o pmc \
        -- python3 -m paper_1908_11848_amd.roofline
    rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d gpurun_out/pmc_write -o pmc \
        -- python3 -m paper_1908_11848_amd.roofline

Algorithmic work per launch is stated with each case.  Peaks: fp32 matrix cores 157.3 TFLOP/s
(256 CUs x 4 SIMDs x 64 FLOP/cycle x 2.4 GHz), HBM 8 TB/s.  HBM traffic per launch (`traffic`)
comes from profiles/traffic_counters.json (counter values scaled by what the same counter reads
for the snapshot-copy kernel of known size) and is reported as null as soon as the kernel's
source file differs from the one the counters were taken on.
"""
import hashlib
import json
import os

import torch

from . import binding as B

PEAK_MFMA_F32 = 157.3e12
PEAK_HBM = 8.0e12
_HERE = os.path.dirname(os.path.abspath(__file__))
_COUNTERS = os.path.join(os.path.dirname(_HERE), "profiles", "traffic_counters.json")

STAGES = ((32, 16), (16, 32), (8, 64))      # (height = width, channels) of the three ResNet stages
BATCH = 128


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


def source_hash(fname):
    with open(os.path.join(_HERE, "csrc", fname), "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()[:16]


def _traffic(key, src):
    """HBM bytes per launch from the stored counters, or None if absent / the kernel changed."""
    try:
        with open(_COUNTERS) as f:
            db = json.load(f)
    except OSError:
        return None
    e = db.get("kernels", {}).get(key)
    if not e or db.get("source_hash", {}).get(src) != source_hash(src):
        return None
    return int(e["fetch_bytes"] + e["write_bytes"])


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
        fn = lambda st: L.dsspk_conv_fwd(st, x.data_ptr(), w.data_ptr(), None, y.data_ptr(), N, H, H, Cin, Cout, k, k, s, p, 0, None)
    elif which == "dgrad":
        fn = lambda st: L.dsspk_conv_bwd_data(st, dy.data_ptr(), w.data_ptr(), None, dx.data_ptr(), N, H, H, Cin, Cout, k, k, s, p)
    else:
        fn = lambda st: L.dsspk_conv_bwd_weight(st, x.data_ptr(), dy.data_ptr(), dw.data_ptr(), scr.data_ptr(), N, H, H, Cin, Cout, k, k, s, p)
    return fn, flops, (x, w, y, dy, dx, dw, scr)


def _bn_case(H, C, which, dev):
    """BN of the second convolution of a block: forward with identity shortcut + ReLU, backward with mask."""
    L = B.lib()
    M = BATCH * H * H
    x = torch.randn(M, C, device=dev)
    y = torch.empty_like(x)
    da = torch.randn_like(x)
    dx = torch.empty_like(x)
    sc = torch.randn_like(x)
    g, b = torch.ones(C, device=dev), torch.zeros(C, device=dev)
    stats, dg, db = torch.empty(2 * C, device=dev), torch.empty(C, device=dev), torch.empty(C, device=dev)
    scr = torch.empty(L.dsspk_bn_scratch_floats(M, C), device=dev)
    fwd = lambda st: L.dsspk_bn_fwd(st, x.data_ptr(), g.data_ptr(), b.data_ptr(), y.data_ptr(), stats.data_ptr(),
                                    scr.data_ptr(), M, C, 1e-5, 1, 1, sc.data_ptr(), BATCH, H, H, 0)
    bwd = lambda st: L.dsspk_bn_bwd(st, x.data_ptr(), g.data_ptr(), stats.data_ptr(), da.data_ptr(), y.data_ptr(),
                                    dx.data_ptr(), dg.data_ptr(), db.data_ptr(), scr.data_ptr(), M, C)
    red = lambda st: L.dsspk_bn_bwd_reduce(st, x.data_ptr(), stats.data_ptr(), da.data_ptr(), y.data_ptr(), scr.data_ptr(), M, C)
    keep = (x, y, da, dx, sc, g, b, stats, dg, db, scr)
    tensor = 4.0 * M * C
    if which == "fwd":      # stats: read x; apply: read x, shortcut, write y
        return fwd, 4 * tensor, keep, fwd
    if which == "bwd_reduce":  # bn_bwd_partial_kernel alone: read x, da, out, write dz
        return red, 4 * tensor, keep, fwd
    return bwd, 7 * tensor, keep, fwd      # reduce as above; dx: read x, dz, write dx


def cases(dev, n_params=1_733_812):
    """[(key, description, bound, work per launch (FLOP or bytes), launcher, source file, keep-alive)]"""
    out = []
    for H, C in STAGES:
        for which, src in (("fwd", "k_conv3x3.hip"), ("dgrad", "k_conv3x3.hip"), ("wgrad", "k_conv3x3.hip" if C < 64 else "k_conv.hip")):
            fn, flops, keep = _conv_case(BATCH, H, C, C, 3, 1, 1, which, dev)
            out.append(("conv_%s_%dx%dx%d" % (which, H, H, C), "conv %s 3x3 %d->%d @%dx%d, batch %d" % (which, C, C, H, H, BATCH),
                        "mfma", flops, fn, src, keep))
    for H, C in STAGES:
        for which, what in (("fwd", "batch norm forward, 2 kernels (+shortcut, ReLU)"), ("bwd", "batch norm backward, 2 kernels"),
                            ("bwd_reduce", "bn_bwd_partial_kernel (sums + ReLU mask)")):
            fn, nbytes, keep, prep = _bn_case(H, C, which, dev)
            out.append(("bn_%s_%dx%dx%d" % (which, H, H, C), "%s @%dx%dx%d, batch %d" % (what, H, H, C, BATCH),
                        "hbm", nbytes, fn, "k_elem.hip", (keep, prep)))
    L = B.lib()
    for n in sorted({n_params, 25_000_000}):
        w = torch.randn(n, device=dev)
        g = torch.randn(n, device=dev) * 1e-3
        dst = torch.empty(n, device=dev)
        st = torch.zeros(2, dtype=torch.int64, device=dev)
        out.append(("apply_%d" % n, "apply_kernel (%d params)" % n, "hbm", 12.0 * n,
                    lambda s, w=w, g=g, st=st, n=n: L.dsspk_apply(s, w.data_ptr(), g.data_ptr(), n, 1e-3, st.data_ptr(), 1),
                    "k_server.hip", (w, g, st)))
        out.append(("pull_%d" % n, "pull_kernel (%d params)" % n, "hbm", 8.0 * n,
                    lambda s, w=w, dst=dst, st=st, n=n: L.dsspk_pull(s, dst.data_ptr(), w.data_ptr(), n, st[1:].data_ptr(), st.data_ptr()),
                    "k_server.hip", (w, dst, st)))
    return out


def _entry(case, t):
    key, desc, bound, work, fn, src, keep = case
    if bound == "mfma":
        achieved, peak, unit, wl = work / t / 1e12, PEAK_MFMA_F32 / 1e12, "TFLOP/s", "%.1f MFLOP" % (work / 1e6)
    else:
        achieved, peak, unit, wl = work / t / 1e9, PEAK_HBM / 1e9, "GB/s", "%.2f MB" % (work / 1e6)
    return {"kernel": desc, "bound": bound, "achieved": round(achieved, 3), "peak": peak, "unit": unit,
            "frac": round(achieved / peak, 5), "traffic": _traffic(key, src), "work_per_launch": wl,
            "avg_us": round(t * 1e6, 2)}


def measure_all(dev, stream, n_params):
    out = {}
    for case in cases(dev, n_params):
        if case[0].startswith("bn_bwd"):
            case[6][1](stream.cuda_stream)          # forward once so that the statistics exist
        out[case[0]] = _entry(case, _time(case[4], stream))
    return out


def measure(workload, em):
    """(dominant kernel entry, list of the other entries).  The dominant kernel family by GPU time
    in the ResNet-110 profile is bn_bwd_partial_kernel, timed here at the first stage's shape; for the
    server stress it is the apply kernel."""
    allm = measure_all(em.dev, em.streams[0], em.n)
    if workload == "resnet110":
        top = "bn_bwd_reduce_32x32x16"
    elif workload == "alexnet_ds":
        top = "conv_fwd_8x8x64"
    else:
        top = "apply_%d" % em.n
    return allm[top], [v for k, v in allm.items() if k != top]


if __name__ == "__main__":
    dev = torch.device("cuda:0")
    st = torch.cuda.Stream()
    for case in cases(dev):
        if case[0].startswith("bn_bwd"):
            case[6][1](st.cuda_stream)
        with torch.cuda.stream(st):
            for _ in range(3):
                case[4](st.cuda_stream)
        st.synchronize()
        print(case[0], "launched", flush=True)
