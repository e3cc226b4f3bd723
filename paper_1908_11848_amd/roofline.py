"""Per-kernel measurements for the benchmark's roofline fields.

Every case launches one kernel family of the worker step (or of the server) at the shape and
launch configuration the ResNet-110 / batch 128 workload uses, through the exported `dsspk_*`
launchers.  `measure_*` time `reps` back-to-back launches on ONE stream with HIP events recorded
on that same stream.  Run as a program it launches every case a few times and exits, which is
what the hardware-counter passes are taken on:

    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d out/pmc_fetch -o pmc \
        -- python3 -m paper_1908_11848_amd.roofline
    rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d out/pmc_write -o pmc \
        -- python3 -m paper_1908_11848_amd.roofline

Algorithmic work per launch, with T = 4 * N * H * H * C bytes (one activation tensor of the stage) and
W = (4/9) * 2 * N * H * H * C * 9 * C FLOP, the matrix-core work of one 3x3 convolution by minimal filtering
(16 instead of 36 multiplications per 2x2 tile and channel pair; the direct form would be 9/4 W):
    conv_fwd       plain forward convolution + statistics records            W,  2 T  (read x, write y)
    conv_fwd_bn    records merge + forward convolution with BN + shortcut    W,  4 T  (read z, shortcut; write a, y)
                   + ReLU folded into its loader (2 kernels)
    conv_bwd_fused d-input AND d-filter convolution of a layer in one kernel 2W, 6 T  (read dz, xc, add, x, xc of the next BN;
                   (stages 1-2): BN backward in its loader, shortcut                  write out) + its own partial sums and
                   gradient, ReLU mask + sum records in its epilogue,                 the carried reduction's
                   carrying the previous layer's d-filter reduction
    conv_dgrad_bn  the same without the d-filter part (stage 3), dx stored   W,  7 T  + the carried reduction's partial sums
    conv_wgrad     d-filter convolution, stage 1 (stage 3), carrying the     W,  2 T + its partial sums
                   BN sums job
    bn_fwd / bn_bwd  stand-alone batch-norm kernels (irregular layers only)      4 T / 7 T
    apply / pull   server update and snapshot copy                               12 / 8 bytes per parameter
    apply_pull     update + the pusher's snapshot in one pass                    16 bytes per parameter
    apply_many4    four simultaneous pushes + one snapshot in one pass           28 bytes per parameter (56 one by one)
A case is bound by whichever of its two floors is higher: its FLOP at 157.3 TFLOP/s (fp32 matrix cores: 256 CUs
x 4 SIMDs x 64 FLOP/cycle x 2.4 GHz) or its bytes at 8 TB/s (HBM); with minimal filtering that is HBM for every
3x3 case.  HBM traffic per launch (`traffic`)
comes from profiles/traffic_counters.json (counter values scaled by what the same counter reads
for the snapshot-copy kernel of known size) and is reported as null as soon as the kernel's
source file differs from the one the counters were taken on.
"""
import ctypes
import hashlib
import json
import os

PEAK_MFMA_F32 = 157.3e12
PEAK_HBM = 8.0e12
_HERE = os.path.dirname(os.path.abspath(__file__))
_COUNTERS = os.path.join(os.path.dirname(_HERE), "profiles", "traffic_counters.json")

STAGES = ((32, 16), (16, 32), (8, 64))      # (height = width, channels) of the three ResNet stages
BATCH = 128
N_PARAMS = 1_733_812                         # ResNet-110, 10 classes
SOURCES = ("k_conv3x3.hip", "k_conv.hip", "k_elem.hip", "k_server.hip", "jobs.hpp", "bn_merge.hpp", "mma.hpp")


def case_list(n_params=N_PARAMS):
    """[(key, kernels per launch, kernels launched once beforehand)] in launch order; no GPU needed."""
    out = []
    for H, C in STAGES:
        out += [("conv_fwd_%dx%dx%d" % (H, H, C), 1, 0), ("conv_fwd_bn_%dx%dx%d" % (H, H, C), 2, 1)]
        if C < 64:
            out += [("conv_bwd_fused_%dx%dx%d" % (H, H, C), 1, 0)]
        else:
            out += [("conv_dgrad_bn_%dx%dx%d" % (H, H, C), 1, 1), ("conv_wgrad_%dx%dx%d" % (H, H, C), 1, 0)]
    out += [("bn_fwd_32x32x16", 2, 0), ("bn_bwd_32x32x16", 2, 2)]
    for n in sorted({n_params, 25_000_000}):
        out += [("apply_%d" % n, 1, 0), ("pull_%d" % n, 1, 0)]
    out += [("apply_pull_25000000", 1, 0), ("apply_many4_25000000", 1, 0)]
    return out


def _time(fn, stream, reps=50, warm=5):
    import torch
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


def _traffic(key, srcs):
    """HBM bytes per launch from the stored counters, or None if absent / a source of the kernel changed."""
    try:
        with open(_COUNTERS) as f:
            db = json.load(f)
    except OSError:
        return None
    e = db.get("kernels", {}).get(key)
    if not e or any(db.get("source_hash", {}).get(s) != source_hash(s) for s in srcs):
        return None
    return int(e["fetch_bytes"] + e["write_bytes"])


_CONV_SRCS = ("k_conv3x3.hip", "k_conv.hip", "jobs.hpp", "bn_merge.hpp", "mma.hpp")


def _conv_cases(H, C, dev):
    """The four fused convolution launches of a regular layer of the stage, on random data."""
    import torch
    from . import binding as B
    L = B.lib()
    N = BATCH
    M = N * H * H
    t = lambda: torch.randn(N, H, H, C, device=dev)
    x, z, sc, a, y = t(), t(), t(), t(), t()
    dz, xc, add, act, xcp, dx = t(), t(), t(), t(), t(), t()
    w = torch.randn(3, 3, C, C, device=dev) * 0.1
    gamma, beta = torch.ones(C, device=dev), torch.zeros(C, device=dev)
    stats = torch.cat([torch.zeros(C, device=dev), torch.ones(C, device=dev)])
    stats_o = torch.empty(2 * C, device=dev)
    tot = torch.zeros(2 * C, device=dev)
    dgam, dbet = torch.empty(C, device=dev), torch.empty(C, device=dev)
    parts = L.dsspk_conv_fwd_stat_parts(N, H, H, C, C, 3, 3, 1, 1)
    recA = torch.empty(L.dsspk_bn_scratch_floats(M, C), device=dev)
    recB = torch.empty_like(recA)
    rec = torch.empty(2 * parts * C, device=dev)
    scr = torch.empty(L.dsspk_conv_wgrad_scratch_floats(N, H, H, C, C, 3, 3, 1, 1), device=dev)
    dw = torch.empty(9 * C * C, device=dev)
    E = 9 * C * C
    ch = ctypes.c_int(0)
    T = 4.0 * M * C
    F = 2.0 * M * C * 9 * C * 4.0 / 9.0          # executed on the matrix cores (minimal filtering)
    fwd = lambda s: L.dsspk_conv_fwd(s, x.data_ptr(), w.data_ptr(), None, z.data_ptr(), N, H, H, C, C, 3, 3, 1, 1, 0, recA.data_ptr())
    fwd_bn = lambda s: L.dsspk_conv_fwd_prebn(s, z.data_ptr(), recA.data_ptr(), parts, gamma.data_ptr(), beta.data_ptr(), 1e-5,
                                              sc.data_ptr(), a.data_ptr(), stats_o.data_ptr(), w.data_ptr(), y.data_ptr(),
                                              recB.data_ptr(), N, H, C)
    wgrad = lambda s: L.dsspk_conv_bwd_weight_parts(s, x.data_ptr(), dx.data_ptr(), scr.data_ptr(), N, H, H, C, C, 3, 3, 1, 1,
                                                    rec.data_ptr(), parts, C, tot.data_ptr(), dgam.data_ptr(), dbet.data_ptr(),
                                                    ctypes.byref(ch))
    chunks = L.dsspk_conv_wgrad_scratch_floats(N, H, H, C, C, 3, 3, 1, 1) // E
    dgrad_bn = lambda s: L.dsspk_conv_bwd_data_bn(s, dz.data_ptr(), xc.data_ptr(), stats.data_ptr(), gamma.data_ptr(), tot.data_ptr(),
                                                  dx.data_ptr(), w.data_ptr(), add.data_ptr(), add.data_ptr(), act.data_ptr(),
                                                  xcp.data_ptr(), stats.data_ptr(), rec.data_ptr(), scr.data_ptr(), dw.data_ptr(),
                                                  E, chunks, N, H, C)
    scr2 = torch.zeros_like(scr)
    fused = lambda s: L.dsspk_conv_bwd_data_bn_wgrad(s, dz.data_ptr(), xc.data_ptr(), stats.data_ptr(), gamma.data_ptr(), tot.data_ptr(),
                                                     w.data_ptr(), add.data_ptr(), add.data_ptr(), xcp.data_ptr(), stats.data_ptr(),
                                                     rec.data_ptr(), act.data_ptr(), scr.data_ptr(), scr2.data_ptr(), dw.data_ptr(),
                                                     E, chunks, N, H, C)
    keep = (x, z, sc, a, y, dz, xc, add, act, xcp, dx, w, gamma, beta, stats, stats_o, tot, dgam, dbet, recA, recB, rec, scr, scr2, dw, ch)
    part_bytes = 4.0 * chunks * E
    desc = "%d->%d @%dx%d, batch %d" % (C, C, H, H, N)
    head = [
        ("conv_fwd_%dx%dx%d" % (H, H, C), "conv 3x3 forward + statistics records " + desc, F, 2 * T, fwd, None, keep),
        ("conv_fwd_bn_%dx%dx%d" % (H, H, C), "records merge + conv 3x3 forward with BN, shortcut, ReLU in its loader " + desc,
         F, 4 * T, fwd_bn, fwd, keep)]
    if C < 64:
        return head + [
            ("conv_bwd_fused_%dx%dx%d" % (H, H, C), "conv 3x3 d-input + d-filter in one kernel: BN backward in its loader, shortcut "
             "gradient, ReLU mask + sum records in its epilogue, carrying a d-filter reduction " + desc,
             2 * F, 6 * T + 2 * part_bytes + 4.0 * E, fused, None, keep)]
    return head + [
        ("conv_dgrad_bn_%dx%dx%d" % (H, H, C), "conv 3x3 d-input with BN backward in its loader, shortcut gradient, ReLU mask + "
         "sum records in its epilogue, carrying a d-filter reduction " + desc, F, 7 * T + part_bytes + 4.0 * E, dgrad_bn, wgrad, keep),
        ("conv_wgrad_%dx%dx%d" % (H, H, C), "conv 3x3 d-filter stage 1, carrying the BN sums " + desc, F, 2 * T + part_bytes, wgrad, None, keep),
    ]


def _bn_cases(H, C, dev):
    import torch
    from . import binding as B
    L = B.lib()
    M = BATCH * H * H
    x = torch.randn(M, C, device=dev)
    y, da, dx, sc = torch.empty_like(x), torch.randn_like(x), torch.empty_like(x), torch.randn_like(x)
    g, b = torch.ones(C, device=dev), torch.zeros(C, device=dev)
    stats, dg, db = torch.empty(2 * C, device=dev), torch.empty(C, device=dev), torch.empty(C, device=dev)
    scr = torch.empty(L.dsspk_bn_scratch_floats(M, C), device=dev)
    fwd = lambda st: L.dsspk_bn_fwd(st, x.data_ptr(), g.data_ptr(), b.data_ptr(), y.data_ptr(), stats.data_ptr(),
                                    scr.data_ptr(), M, C, 1e-5, 1, 1, sc.data_ptr(), BATCH, H, H, 0)
    bwd = lambda st: L.dsspk_bn_bwd(st, x.data_ptr(), g.data_ptr(), stats.data_ptr(), da.data_ptr(), y.data_ptr(),
                                    dx.data_ptr(), dg.data_ptr(), db.data_ptr(), scr.data_ptr(), M, C)
    keep = (x, y, da, dx, sc, g, b, stats, dg, db, scr)
    T = 4.0 * M * C
    tag = "%dx%dx%d" % (H, H, C)
    return [("bn_fwd_" + tag, "stand-alone batch norm forward, 2 kernels (+shortcut, ReLU) @%s, batch %d" % (tag, BATCH), 0.0, 4 * T, fwd, None, keep),
            ("bn_bwd_" + tag, "stand-alone batch norm backward, 2 kernels @%s, batch %d" % (tag, BATCH), 0.0, 7 * T, bwd, fwd, keep)]


def cases(dev, n_params=N_PARAMS):
    """[(key, description, FLOP per launch, bytes per launch, launcher, launcher to run once beforehand or None,
    source files, keep-alive)] in the order of case_list()."""
    import torch
    from . import binding as B
    out = []
    for H, C in STAGES:
        out += [c[:6] + (_CONV_SRCS, c[6]) for c in _conv_cases(H, C, dev)]
    out += [c[:6] + (("k_elem.hip", "bn_merge.hpp"), c[6]) for c in _bn_cases(32, 16, dev)]
    L = B.lib()
    for n in sorted({n_params, 25_000_000}):
        w = torch.randn(n, device=dev)
        g = torch.randn(n, device=dev) * 1e-3
        dst = torch.empty(n, device=dev)
        st = torch.zeros(2, dtype=torch.int64, device=dev)
        pw, pg, pd, ps = w.data_ptr(), g.data_ptr(), dst.data_ptr(), st.data_ptr()      # pointers taken once: these
        out.append(("apply_%d" % n, "apply_kernel (%d params)" % n, 0.0, 12.0 * n,      # kernels are as short as a launch
                    lambda s, pw=pw, pg=pg, ps=ps, n=n: L.dsspk_apply(s, pw, pg, n, 1e-3, ps, 1),
                    None, ("k_server.hip",), (w, g, st)))
        out.append(("pull_%d" % n, "pull_kernel (%d params)" % n, 0.0, 8.0 * n,
                    lambda s, pw=pw, pd=pd, ps=ps, n=n: L.dsspk_pull(s, pd, pw, n, ps + 8, ps),
                    None, ("k_server.hip",), (w, dst, st)))
    # the two fused server kernels at the stress size: apply + the pusher's pull in one pass (16 B/param), and four
    # simultaneous pushes with one snapshot in one pass (4 * 4 + 8 + 4 = 28 B/param instead of 4 * 12 + 8 = 56)
    n = 25_000_000
    w = torch.randn(n, device=dev)
    gs = [torch.randn(n, device=dev) * 1e-3 for _ in range(4)]
    dst = torch.empty(n, device=dev)
    st = torch.zeros(2, dtype=torch.int64, device=dev)
    pw, pd, ps = w.data_ptr(), dst.data_ptr(), st.data_ptr()
    pg = gs[0].data_ptr()
    out.append(("apply_pull_%d" % n, "apply_pull_kernel: update + the pusher's snapshot in one pass (%d params)" % n, 0.0, 16.0 * n,
                lambda s, pw=pw, pg=pg, pd=pd, ps=ps, n=n: L.dsspk_apply_pull(s, pw, pg, pd, n, 1e-3, ps, ps + 8, 1),
                None, ("k_server.hip",), (w, gs, dst, st)))
    g_arr = (ctypes.c_void_p * 4)(*[g.data_ptr() for g in gs])
    d_arr = (ctypes.c_void_p * 1)(pd)
    a_arr = (ctypes.c_int * 1)(4)
    s_arr = (ctypes.c_void_p * 1)(ps + 8)
    out.append(("apply_many4_%d" % n, "apply_many_kernel: 4 simultaneous pushes + 1 snapshot in one pass (%d params)" % n, 0.0, 28.0 * n,
                lambda s, pw=pw, ps=ps, n=n: L.dsspk_apply_many(s, pw, 4, g_arr, n, 1e-3, 1, d_arr, a_arr, s_arr, ps, 1),
                None, ("k_server.hip",), (w, gs, dst, st, g_arr, d_arr, a_arr, s_arr)))
    assert [c[0] for c in out] == [k for k, _, _ in case_list(n_params)]
    return out


def _entry(case, t):
    key, desc, flops, nbytes, fn, prep, srcs, keep = case
    t_mfma, t_hbm = flops / PEAK_MFMA_F32, nbytes / PEAK_HBM
    if t_mfma > t_hbm:
        bound, achieved, peak, unit = "mfma", flops / t / 1e12, PEAK_MFMA_F32 / 1e12, "TFLOP/s"
    else:
        bound, achieved, peak, unit = "hbm", nbytes / t / 1e9, PEAK_HBM / 1e9, "GB/s"
    return {"kernel": desc, "bound": bound, "achieved": round(achieved, 3), "peak": peak, "unit": unit,
            "frac": round(achieved / peak, 5), "traffic": _traffic(key, srcs),
            "work_per_launch": "%.1f MFLOP, %.2f MB" % (flops / 1e6, nbytes / 1e6), "avg_us": round(t * 1e6, 2)}


def measure_all(dev, stream, n_params):
    out = {}
    for case in cases(dev, n_params):
        if case[5]:
            case[5](stream.cuda_stream)          # once: what the case consumes (records, statistics, partial sums) exists
        out[case[0]] = _entry(case, _time(case[4], stream))
    return out


def _alexnet_conv2_case(dev):
    """Forward of the AlexNet-style network's second convolution (5x5, 64 -> 64 at 15x15, bias + ReLU), its largest layer."""
    import torch
    from . import binding as B
    L = B.lib()
    N, H, C = BATCH, 15, 64
    x = torch.randn(N, H, H, C, device=dev)
    w = torch.randn(5, 5, C, C, device=dev) * 0.05
    b = torch.zeros(C, device=dev)
    y = torch.empty(N, H, H, C, device=dev)
    fn = lambda s: L.dsspk_conv_fwd(s, x.data_ptr(), w.data_ptr(), b.data_ptr(), y.data_ptr(), N, H, H, C, C, 5, 5, 1, 2, 1, None)
    flops = 2.0 * N * H * H * C * 25 * C
    return ("alexnet_conv2_fwd", "conv 5x5 forward + bias + ReLU 64->64 @15x15, batch %d (implicit GEMM)" % N, flops,
            2 * 4.0 * N * H * H * C, fn, None, ("k_conv.hip", "mma.hpp"), (x, w, b, y))


def measure(workload, em):
    """(dominant kernel entry, list of the other entries).  The kernel with the largest share of GPU time in the
    ResNet-110 profile is the fused backward convolution kernel of the first stage; for the server stress it is the apply kernel."""
    allm = measure_all(em.dev, em.streams[0], em.n)
    if workload.startswith("resnet"):
        top = "conv_bwd_fused_32x32x16"
    elif workload.startswith("alexnet"):
        case = _alexnet_conv2_case(em.dev)
        top = case[0]
        allm[top] = _entry(case, _time(case[4], em.streams[0]))
    else:
        top = "apply_%d" % em.n
    return allm[top], [v for k, v in allm.items() if k != top]


if __name__ == "__main__":
    import torch
    dev = torch.device("cuda:0")
    st = torch.cuda.Stream()
    for case in cases(dev):
        with torch.cuda.stream(st):
            if case[5]:
                case[5](st.cuda_stream)
            for _ in range(3):
                case[4](st.cuda_stream)
        st.synchronize()
        print(case[0], "launched", flush=True)
