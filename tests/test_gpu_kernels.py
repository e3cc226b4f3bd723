"""Each HIP kernel family against the oracle's layer function on the same seeded inputs.

Sizes span several tiles and ragged tails; one case per convolution kind has the full
benchmark shape (batch 128).  Tolerances: the kernels accumulate in fp32 (matrix cores or
fixed-order trees), the oracle in fp64; for a sum of n products of O(1) terms the fp32 error is
about sqrt(n) * 6e-8 relative to the operand scale, so 2e-6 relative L2 covers every case here
with an order of magnitude to spare.  Integer outputs (arg-max positions) and copies are
bit-exact.
"""
import os

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_1908_11848_amd import binding as B          # noqa: E402
from gpu_util import dev, empty, host, max_abs, stream_ptr  # noqa: E402
import gpu_util                                                # noqa: E402

TOL = 2e-6
ELEM_TOL = 2e-5         # largest element-wise error, relative to the largest expected magnitude of the tensor


def rel_l2(a, b, elem_tol=ELEM_TOL):
    """Relative L2 error of a against b.  Every comparison in this file is also held element by element: no single
    element may be off by more than elem_tol of the tensor's largest expected magnitude (a norm can hide one wrong
    element of a large tensor; this cannot), and none may be NaN."""
    a, b = np.asarray(a), np.asarray(b)
    assert a.shape == b.shape or a.size == b.size
    assert np.isfinite(a).all()
    e = max_abs(a, b)
    if os.environ.get("DSSP_TEST_LOG_ELEM"):
        with open(os.environ["DSSP_TEST_LOG_ELEM"], "a") as f:
            f.write("%.3e %.3e %s\n" % (e, gpu_util.rel_l2(a, b), os.environ.get("PYTEST_CURRENT_TEST", "")))
    assert e < elem_tol, ("element-wise error", e)
    return gpu_util.rel_l2(a, b)


def rc(x):
    assert x == 0, "launcher returned %d" % x


def f32(rng, shape, scale=1.0):
    return (rng.standard_normal(shape) * scale).astype(np.float32)


# ------------------------------------------------------------------ server kernels
@pytest.mark.parametrize("n", [1, 3, 4, 1023, 1 << 20, (1 << 22) + 5])
def test_apply_and_pull(n):
    g = np.random.default_rng(n)
    w0, gr = f32(g, n), f32(g, n, 1e-3)
    w, grd = dev(w0), dev(gr)
    stamps = torch.zeros(2, dtype=torch.int64, device="cuda")
    scale = np.float32(0.05) / np.float32(8)
    rc(B.lib().dsspk_apply(stream_ptr(), w.data_ptr(), grd.data_ptr(), n, float(scale), stamps.data_ptr(), 7))
    want = w0.astype(np.float64) - np.float64(scale) * gr.astype(np.float64)       # Alg. 1 server step 2
    got = host(w)
    assert np.all(np.abs(got - want) <= np.spacing(np.abs(want).astype(np.float32)))   # one rounding
    dst = empty(n)
    rc(B.lib().dsspk_pull(stream_ptr(), dst.data_ptr(), w.data_ptr(), n, stamps[1:].data_ptr(), stamps.data_ptr()))
    assert np.array_equal(host(dst), got)                                           # bit-exact copy
    assert host(stamps).tolist() == [7, 7]


@pytest.mark.parametrize("n", [3, 1024, 100003])
def test_apply_and_pull_in_one_pass(n):
    """w -= scale * g with the new weights also written to a snapshot: the same bits as apply followed by pull."""
    g = np.random.default_rng(n)
    w0, gr = f32(g, n), f32(g, n, 1e-2)
    L = B.lib()
    s = stream_ptr()
    W1, W2, G = dev(w0), dev(w0), dev(gr)
    d1, d2 = empty(n), empty(n)
    st1 = torch.zeros(2, dtype=torch.int64, device="cuda"); st2 = torch.zeros(2, dtype=torch.int64, device="cuda")
    rc(L.dsspk_apply(s, W1.data_ptr(), G.data_ptr(), n, 0.37, st1.data_ptr(), 5))
    rc(L.dsspk_pull(s, d1.data_ptr(), W1.data_ptr(), n, st1[1:].data_ptr(), st1.data_ptr()))
    rc(L.dsspk_apply_pull(s, W2.data_ptr(), G.data_ptr(), d2.data_ptr(), n, 0.37, st2.data_ptr(), st2[1:].data_ptr(), 5))
    assert np.array_equal(host(W1), host(W2)) and np.array_equal(host(d1), host(d2)) and np.array_equal(host(d2), host(W2))
    assert host(st1).tolist() == host(st2).tolist() == [5, 5]
    assert rel_l2(host(W2), w0.astype(np.float64) - np.float32(0.37).astype(np.float64) * gr.astype(np.float64)) < 1e-6


@pytest.mark.parametrize("n,m,after", [(1, 1, [1]), (3, 2, [1, 2]), (1027, 3, [1, 1, 3]), (100003, 5, [2, 5, 5]), ((1 << 20) + 1, 16, list(range(1, 17))),
                                       (4096, 7, []), (262147, 4, [4])])
def test_aggregated_apply_equals_single_applies_and_pulls(n, m, after):
    """m simultaneous pushes in one pass over the weights (Alg. 1, server step 2, "aggregated"): the weights and every
    snapshot taken between two of the pushes carry the bits m single applies and pulls would have left."""
    g = np.random.default_rng(n + m)
    w0 = f32(g, n)
    grads = [f32(g, n, 1e-2) for _ in range(m)]
    L = B.lib()
    s = stream_ptr()
    scale = 0.05 / 8
    # one by one
    W1 = dev(w0)
    G = [dev(x) for x in grads]
    st1 = torch.zeros(1 + len(after), dtype=torch.int64, device="cuda")
    snaps1 = [empty(n) for _ in after]
    for j in range(m):
        rc(L.dsspk_apply(s, W1.data_ptr(), G[j].data_ptr(), n, scale, st1.data_ptr(), 100 + j))
        for d, a in enumerate(after):
            if a == j + 1:
                rc(L.dsspk_pull(s, snaps1[d].data_ptr(), W1.data_ptr(), n, st1[1 + d:].data_ptr(), st1.data_ptr()))
    # together
    import ctypes
    W2 = dev(w0)
    st2 = torch.zeros(1 + len(after), dtype=torch.int64, device="cuda")
    snaps2 = [empty(n) for _ in after]
    gp = (ctypes.c_void_p * m)(*[x.data_ptr() for x in G])
    nd = len(after)
    dp = (ctypes.c_void_p * max(nd, 1))(*[x.data_ptr() for x in snaps2])
    da = (ctypes.c_int * max(nd, 1))(*after)
    ds = (ctypes.c_void_p * max(nd, 1))(*[st2[1 + d:].data_ptr() for d in range(nd)])
    rc(L.dsspk_apply_many(s, W2.data_ptr(), m, gp, n, scale, nd, dp, da, ds, st2.data_ptr(), 100))
    assert np.array_equal(host(W1), host(W2))
    for a, b in zip(snaps1, snaps2):
        assert np.array_equal(host(a), host(b))
    assert host(st1).tolist() == host(st2).tolist()
    want = w0.astype(np.float64) - np.float64(np.float32(scale)) * np.sum([x.astype(np.float64) for x in grads], axis=0)
    assert rel_l2(host(W2), want) < 1e-6 and max_abs(host(W2), want) < 1e-6
    # rejected on the host: too many pushes, a snapshot index out of order, a snapshot that is the weight vector
    assert L.dsspk_apply_many(s, W2.data_ptr(), 17, gp, n, scale, 0, None, None, None, st2.data_ptr(), 1) == -1
    if nd >= 2 and after[0] != after[-1]:
        bad = (ctypes.c_int * nd)(*reversed(after))
        assert L.dsspk_apply_many(s, W2.data_ptr(), m, gp, n, scale, nd, dp, bad, ds, st2.data_ptr(), 1) == -1
    if nd:
        dp_bad = (ctypes.c_void_p * nd)(*([W2.data_ptr()] + [x.data_ptr() for x in snaps2[1:]]))
        assert L.dsspk_apply_many(s, W2.data_ptr(), m, gp, n, scale, nd, dp_bad, da, ds, st2.data_ptr(), 1) == -1


def test_device_clock_stamp_and_bounded_hold():
    """The clock kernels of the wall-clock mode: stamps on one stream increase, and a hold keeps the stream until the
    iteration has lasted the given multiple of its real duration (capped, so it always ends)."""
    L = B.lib()
    s = stream_ptr()
    khz = L.dsspk_clock_khz()
    assert khz >= 1000
    t = torch.zeros(8, dtype=torch.int64, device="cuda")
    x = torch.randn(1 << 24, device="cuda")
    y = (x * 2 + 1) * 1.0001                                                 # (first use loads these kernels)
    torch.cuda.synchronize()
    rc(L.dsspk_clock_stamp(s, t.data_ptr(), None))
    y = x * 2 + 1                                                            # some real work on the stream: about a millisecond
    for _ in range(20):
        y = y * 1.0001
    rc(L.dsspk_clock_stretch(s, t.data_ptr(), 3000, 100 * khz, t[1:].data_ptr(), t[2:].data_ptr()))
    rc(L.dsspk_clock_stamp(s, t[3:].data_ptr(), t[4:].data_ptr()))
    rc(L.dsspk_clock_stretch(s, t.data_ptr(), 100000, khz // 2, t[5:].data_ptr(), t[6:].data_ptr()))   # 100x, capped at 0.5 ms
    start, arrival, left, after_a, after_b, arr2, left2, _ = host(t).tolist()
    assert start < arrival <= left <= after_a == after_b <= arr2 <= left2
    spent = arrival - start
    assert spent > 0 and left - start >= 3 * spent - 2 and left - start < 3 * spent + khz // 2      # 3x, within 0.5 ms
    assert khz // 2 <= left2 - arr2 < khz // 2 + khz // 2                                           # the cap, not 100x
    assert L.dsspk_clock_stamp(s, None, None) == -1 and L.dsspk_clock_stretch(s, None, 2000, 1, t.data_ptr(), None) == -1


# ------------------------------------------------------------------ GEMM (fully connected layers)
@pytest.mark.parametrize("m,n_in,n_out", [(32, 3072, 256), (32, 256, 10), (128, 3136, 384), (128, 192, 10),
                                          (128, 64, 100), (37, 100, 75), (1, 16, 1)])
def test_fc_forward_backward(oracle_nn, m, n_in, n_out):
    g = np.random.default_rng(m * 131 + n_out)
    x, w, b, dy = f32(g, (m, n_in)), f32(g, (n_in, n_out), 0.1), f32(g, n_out), f32(g, (m, n_out))
    X, W, Bv, DY = dev(x), dev(w), dev(b), dev(dy)
    y = empty((m, n_out)); dx = empty((m, n_in)); dw = empty((n_in, n_out)); db = empty(n_out)
    s = stream_ptr()
    L = B.lib()
    rc(L.dsspk_gemm(s, X.data_ptr(), n_in, 1, W.data_ptr(), n_out, 1, y.data_ptr(), n_out, m, n_out, n_in, Bv.data_ptr(), 0))
    rc(L.dsspk_gemm(s, DY.data_ptr(), n_out, 1, W.data_ptr(), 1, n_out, dx.data_ptr(), n_in, m, n_in, n_out, None, 0))
    rc(L.dsspk_gemm(s, X.data_ptr(), 1, n_in, DY.data_ptr(), n_out, 1, dw.data_ptr(), n_out, n_in, n_out, m, None, 0))
    rc(L.dsspk_colsum(s, DY.data_ptr(), db.data_ptr(), None, m, n_out))
    x64, w64, dy64 = x.astype(np.float64), w.astype(np.float64), dy.astype(np.float64)
    yo = oracle_nn.fc_fwd(x64, w64, b.astype(np.float64))
    dxo, dwo, dbo = oracle_nn.fc_bwd(x64, w64, dy64)
    assert rel_l2(host(y), yo) < TOL
    assert rel_l2(host(dx), dxo) < TOL
    assert rel_l2(host(dw), dwo) < TOL
    assert rel_l2(host(db), dbo) < TOL
    yr = empty((m, n_out))
    rc(L.dsspk_gemm(s, X.data_ptr(), n_in, 1, W.data_ptr(), n_out, 1, yr.data_ptr(), n_out, m, n_out, n_in, Bv.data_ptr(), 1))
    assert rel_l2(host(yr), np.maximum(yo, 0)) < TOL
    # the same forward product with the reduction index split over layers of workgroups (few output tiles, long K)
    layers = L.dsspk_gemm_splitk_layers(m, n_out, n_in)
    assert layers >= 1 and (layers > 1) == (n_in >= 3072)
    for lay in sorted({layers, 1, 3}):
        if lay * 16 > n_in and lay > 1:
            continue
        scratch = empty(lay * m * n_out)
        ys = empty((m, n_out))
        rc(L.dsspk_gemm_splitk(s, X.data_ptr(), n_in, 1, W.data_ptr(), n_out, 1, ys.data_ptr(), n_out, m, n_out, n_in,
                               Bv.data_ptr(), 1, scratch.data_ptr(), lay))
        assert rel_l2(host(ys), np.maximum(yo, 0)) < TOL
    if layers > 1:
        assert L.dsspk_gemm_splitk(s, X.data_ptr(), n_in, 1, W.data_ptr(), n_out, 1, ys.data_ptr(), n_out, m, n_out, n_in,
                                   Bv.data_ptr(), 1, None, layers) == -1


@pytest.mark.parametrize("M,N", [(1, 1), (1024, 64), (1025, 64), (131072, 64), (28800, 64), (5000, 100)])
def test_column_sums_of_tall_matrices(M, N):
    """Bias gradients of the convolutions: one pass for short matrices, row slabs + their sum for tall ones."""
    g = np.random.default_rng(M + N)
    x = f32(g, (M, N))
    L = B.lib()
    s = stream_ptr()
    X = dev(x); out = empty(N)
    need = L.dsspk_colsum_scratch_floats(M, N)
    assert (need > 0) == (M > 1024)
    scr = empty(max(1, need))
    rc(L.dsspk_colsum(s, X.data_ptr(), out.data_ptr(), scr.data_ptr() if need else None, M, N))
    assert rel_l2(host(out), x.astype(np.float64).sum(0)) < TOL
    if need:
        assert L.dsspk_colsum(s, X.data_ptr(), out.data_ptr(), None, M, N) == -1


# ------------------------------------------------------------------ convolution
CONV_CASES = [  # N, H, Cin, Cout, k, stride, pad, bias+relu
    (3, 32, 3, 16, 3, 1, 1, False),
    (2, 32, 16, 16, 3, 1, 1, False),
    (2, 32, 16, 32, 3, 2, 1, False),
    (3, 16, 32, 32, 3, 1, 1, False),
    (2, 16, 32, 64, 3, 2, 1, False),
    (5, 8, 64, 64, 3, 1, 1, False),
    (2, 32, 3, 64, 5, 1, 2, True),
    (3, 15, 64, 64, 5, 1, 2, True),
    (1, 7, 16, 16, 3, 1, 1, False),          # fewer pixels than one tile
    (2, 8, 64, 128, 3, 1, 1, True),          # wider than one channel tile: the d-filter kernel works in channel slices
    (3, 9, 96, 80, 3, 2, 1, False),
    (2, 7, 128, 192, 5, 1, 2, True),
    (2, 12, 3, 96, 5, 1, 2, True),
    (3, 16, 3, 32, 3, 1, 1, False),          # few input channels, tiles of whole image rows: the gather reads staged rows
    (5, 8, 3, 16, 5, 1, 2, True),
    (2, 64, 3, 16, 3, 1, 1, False),
    (3, 32, 5, 32, 3, 1, 0, True),           # no padding: 30 columns, tiles are not whole rows (gather from global memory)
    (128, 32, 3, 64, 5, 1, 2, True),         # first layer of the AlexNet-style net, batch 128
    (2, 12, 16, 32, 5, 2, 2, False),         # stride 2 on an even grid: the d-input kernel works by parity class of the pixel
    (3, 8, 32, 64, 1, 2, 0, False),          # 1x1 stride 2: three of the four classes receive no gradient at all
    (2, 10, 16, 16, 4, 2, 1, False),         # even filter size
    (2, 8, 32, 48, 3, 1, 1, False),          # widths between the d-filter tile kernel's instantiations
    (2, 8, 16, 64, 3, 1, 1, True),
    (2, 8, 64, 32, 3, 1, 1, False),
    (128, 32, 16, 16, 3, 1, 1, False),       # benchmark shapes, batch 128
    (128, 16, 32, 32, 3, 1, 1, False),
    (128, 8, 64, 64, 3, 1, 1, False),
    (128, 32, 16, 32, 3, 2, 1, False),
]


def random_conv_cases(seed=20, count=48):
    """Seeded shapes across the generic kernels' paths: few / 16-multiple input channels, widths between the tile sizes,
    even and odd pixel grids, strides 1-3, filter sizes 1-5, with and without padding."""
    g = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        N, H = int(g.integers(1, 4)), int(g.choice([4, 6, 7, 8, 9, 12, 16]))
        Cin = int(g.choice([1, 3, 5, 16, 32, 48, 64, 80, 96]))
        Cout = int(g.choice([16, 32, 48, 64, 80, 96, 128]))
        k, s, p = int(g.integers(1, 6)), int(g.integers(1, 4)), int(g.integers(0, 3))
        if H + 2 * p < k or (Cin % 16 and k * k * Cin > 80):      # the element-wise d-filter kernel holds 80 (tap, ci) rows
            continue
        cases.append((N, H, Cin, Cout, k, s, p, bool(g.integers(0, 2))))
    return cases


@pytest.mark.parametrize("case", CONV_CASES + random_conv_cases(), ids=lambda c: "x".join(map(str, c)))
def test_conv_forward_dgrad_wgrad(oracle_nn, case):
    N, H, Cin, Cout, k, s, p, br = case
    g = np.random.default_rng(hash(case) % (1 << 31))
    x, w = f32(g, (N, H, H, Cin)), f32(g, (k, k, Cin, Cout), (2.0 / (k * k * Cin)) ** 0.5)
    b = f32(g, Cout) if br else None
    Ho = (H + 2 * p - k) // s + 1
    dy = f32(g, (N, Ho, Ho, Cout))
    X, W, DY = dev(x), dev(w), dev(dy)
    Bv = dev(b) if br else None
    st = stream_ptr()
    L = B.lib()
    y = empty((N, Ho, Ho, Cout))
    rc(L.dsspk_conv_fwd(st, X.data_ptr(), W.data_ptr(), Bv.data_ptr() if br else None, y.data_ptr(),
                        N, H, H, Cin, Cout, k, k, s, p, int(br), None))
    x64, w64, dy64 = x.astype(np.float64), w.astype(np.float64), dy.astype(np.float64)
    yo = oracle_nn.conv2d_fwd(x64, w64, b.astype(np.float64) if br else None, s, p)
    if br:
        yo = np.maximum(yo, 0)
    assert rel_l2(host(y), yo) < TOL
    assert np.max(np.abs(host(y) - yo)) < 2e-5
    dxo, dwo, _ = oracle_nn.conv2d_bwd(x64, w64, dy64, s, p, False, need_dx=Cin % 16 == 0)
    scratch = empty(L.dsspk_conv_wgrad_scratch_floats(N, H, H, Cin, Cout, k, k, s, p))
    dw = empty((k, k, Cin, Cout))
    rc(L.dsspk_conv_bwd_weight(st, X.data_ptr(), DY.data_ptr(), dw.data_ptr(), scratch.data_ptr(),
                               N, H, H, Cin, Cout, k, k, s, p))
    assert rel_l2(host(dw), dwo) < TOL
    if Cin % 16 == 0:
        dx = empty((N, H, H, Cin))
        rc(L.dsspk_conv_bwd_data(st, DY.data_ptr(), W.data_ptr(), None, dx.data_ptr(), N, H, H, Cin, Cout, k, k, s, p))
        assert rel_l2(host(dx), dxo) < TOL
        rc(L.dsspk_conv_bwd_data(st, DY.data_ptr(), W.data_ptr(), X.data_ptr(), dx.data_ptr(), N, H, H, Cin, Cout, k, k, s, p))
        assert rel_l2(host(dx), dxo + x64) < TOL              # with the shortcut's gradient added in the epilogue


@pytest.mark.parametrize("N,H,C", [(3, 32, 16), (5, 16, 32), (4, 8, 64)])
def test_minimal_filtering_on_inputs_with_a_large_common_offset(oracle_nn, N, H, C):
    """The 3x3 kernels form differences of neighbouring inputs before they multiply (Winograd's patch transform), so
    their rounding error scales with the magnitude of the inputs, not of the result.  Post-ReLU activations are all
    positive; here the inputs sit at 8 +- 1 and every output channel's filter sums to zero, so the offset cancels
    in the result, which is several times smaller than the inputs: the error, relative to the result, must stay at
    the fp32 level all the same."""
    g = np.random.default_rng(1000 * C + N)
    x = (8.0 + g.standard_normal((N, H, H, C))).astype(np.float32)
    w = g.standard_normal((3, 3, C, C)) * (2.0 / (9 * C)) ** 0.5
    wf = (w - w.mean(axis=(0, 1, 2), keepdims=True)).astype(np.float32)      # forward: zero sum per output channel
    wb = (w - w.mean(axis=(0, 1, 3), keepdims=True)).astype(np.float32)      # d-input: zero sum per input channel
    dy = (8.0 + g.standard_normal((N, H, H, C))).astype(np.float32)
    X, WF, WB, DY = dev(x), dev(wf), dev(wb), dev(dy)
    st, L = stream_ptr(), B.lib()
    y, dx = empty((N, H, H, C)), empty((N, H, H, C))
    rc(L.dsspk_conv_fwd(st, X.data_ptr(), WF.data_ptr(), None, y.data_ptr(), N, H, H, C, C, 3, 3, 1, 1, 0, None))
    rc(L.dsspk_conv_bwd_data(st, DY.data_ptr(), WB.data_ptr(), None, dx.data_ptr(), N, H, H, C, C, 3, 3, 1, 1))
    x64, dy64 = x.astype(np.float64), dy.astype(np.float64)
    yo = oracle_nn.conv2d_fwd(x64, wf.astype(np.float64), None, 1, 1)
    dxo, _, _ = oracle_nn.conv2d_bwd(x64, wb.astype(np.float64), dy64, 1, 1, False, need_dx=True)
    e_y, e_dx = rel_l2(host(y), yo), rel_l2(host(dx), dxo)
    print("offset inputs %dx%dx%d: forward %.2e, d-input %.2e; interior |y| rms %.2f" % (H, H, C, e_y, e_dx, np.sqrt(np.mean(yo[:, 1:-1, 1:-1] ** 2))))
    assert e_y < TOL and e_dx < TOL


@pytest.mark.parametrize("N,H,C", [(3, 32, 16), (5, 16, 32), (4, 8, 64), (128, 32, 16), (128, 8, 64)])
def test_conv_emits_batchnorm_statistics(oracle_nn, N, H, C):
    """conv -> BN with the statistics taken from the convolution kernel's per-tile records."""
    g = np.random.default_rng(N + H + C)
    x, w = f32(g, (N, H, H, C)), f32(g, (3, 3, C, C), (2.0 / (9 * C)) ** 0.5)
    gamma, beta = (1 + 0.2 * g.standard_normal(C)).astype(np.float32), f32(g, C, 0.3)
    L = B.lib()
    st = stream_ptr()
    parts = L.dsspk_conv_fwd_stat_parts(N, H, H, C, C, 3, 3, 1, 1)
    assert parts > 0
    M = N * H * H
    X, W, Ga, Be = dev(x), dev(w), dev(gamma), dev(beta)
    y = empty((N, H, H, C)); out = empty((N, H, H, C)); stats = empty(2 * C)
    scratch = empty(L.dsspk_bn_scratch_floats(M, C))
    rc(L.dsspk_conv_fwd(st, X.data_ptr(), W.data_ptr(), None, y.data_ptr(), N, H, H, C, C, 3, 3, 1, 1, 0, scratch.data_ptr()))
    rc(L.dsspk_bn_fwd(st, y.data_ptr(), Ga.data_ptr(), Be.data_ptr(), out.data_ptr(), stats.data_ptr(), scratch.data_ptr(),
                      M, C, 1e-5, 1, 0, None, 0, 0, 0, parts))
    yo = oracle_nn.conv2d_fwd(x.astype(np.float64), w.astype(np.float64), None, 1, 1)
    oo, mean, invstd = oracle_nn.bn_fwd(yo, gamma.astype(np.float64), beta.astype(np.float64))
    assert rel_l2(host(stats)[:C], mean) < 5e-6 and rel_l2(host(stats)[C:], invstd) < TOL
    assert rel_l2(host(out), np.maximum(oo, 0)) < 5e-6


@pytest.mark.parametrize("N,H,C,with_sc", [(3, 32, 16, False), (5, 16, 32, True), (4, 8, 64, True), (128, 32, 16, True), (128, 8, 64, False)])
def test_conv_with_batchnorm_folded_into_its_loader(oracle_nn, N, H, C, with_sc):
    """c -> [BN + (shortcut) + ReLU folded into the loader] -> conv, against the three oracle layers;
    the side outputs (activation, mean / invstd, statistics records of y) are checked too."""
    g = np.random.default_rng(N * 7 + H + C)
    x = f32(g, (N, H, H, C))
    w0, w1 = f32(g, (3, 3, C, C), (2.0 / (9 * C)) ** 0.5), f32(g, (3, 3, C, C), (2.0 / (9 * C)) ** 0.5)
    gamma, beta = (1 + 0.2 * g.standard_normal(C)).astype(np.float32), f32(g, C, 0.3)
    sc = f32(g, (N, H, H, C)) if with_sc else None
    L = B.lib()
    st = stream_ptr()
    M = N * H * H
    parts = L.dsspk_conv_fwd_stat_parts(N, H, H, C, C, 3, 3, 1, 1)
    X, W0, W1, Ga, Be = dev(x), dev(w0), dev(w1), dev(gamma), dev(beta)
    SC = dev(sc) if with_sc else None
    c = empty((N, H, H, C)); a = empty((N, H, H, C)); y = empty((N, H, H, C)); stats = empty(2 * C)
    recA, recB = empty(L.dsspk_bn_scratch_floats(M, C)), empty(L.dsspk_bn_scratch_floats(M, C))
    rc(L.dsspk_conv_fwd(st, X.data_ptr(), W0.data_ptr(), None, c.data_ptr(), N, H, H, C, C, 3, 3, 1, 1, 0, recA.data_ptr()))
    rc(L.dsspk_conv_fwd_prebn(st, c.data_ptr(), recA.data_ptr(), parts, Ga.data_ptr(), Be.data_ptr(), 1e-5,
                              SC.data_ptr() if with_sc else None, a.data_ptr(), stats.data_ptr(), W1.data_ptr(), y.data_ptr(),
                              recB.data_ptr(), N, H, C))
    co = oracle_nn.conv2d_fwd(x.astype(np.float64), w0.astype(np.float64), None, 1, 1)
    bo, mean, invstd = oracle_nn.bn_fwd(co, gamma.astype(np.float64), beta.astype(np.float64))
    ao = np.maximum(bo + (sc if with_sc else 0), 0)
    yo = oracle_nn.conv2d_fwd(ao, w1.astype(np.float64), None, 1, 1)
    assert rel_l2(host(stats)[:C], mean) < 5e-6 and rel_l2(host(stats)[C:], invstd) < TOL
    assert rel_l2(host(a), ao) < 5e-6
    assert rel_l2(host(y), yo) < 5e-6
    # the records of y merge to y's statistics
    out = empty((N, H, H, C)); st2 = empty(2 * C)
    rc(L.dsspk_bn_fwd(st, y.data_ptr(), Ga.data_ptr(), Be.data_ptr(), out.data_ptr(), st2.data_ptr(), recB.data_ptr(),
                      M, C, 1e-5, 0, 0, None, 0, 0, 0, parts))
    _, mean2, invstd2 = oracle_nn.bn_fwd(yo, gamma.astype(np.float64), beta.astype(np.float64))
    assert rel_l2(host(st2)[:C], mean2) < 2e-5 and rel_l2(host(st2)[C:], invstd2) < 5e-6


@pytest.mark.parametrize("N,H,C,with_add", [(3, 32, 16, True), (5, 16, 32, False), (4, 8, 64, True), (128, 16, 32, True)])
def test_dgrad_with_relu_mask_and_batchnorm_records(oracle_nn, N, H, C, with_add):
    """d-input convolution whose epilogue masks by the saved activation and emits the sum records of the batch
    norm behind it; followed by that batch norm's dx kernel.  Against: oracle d-input, mask, oracle BN backward."""
    g = np.random.default_rng(N * 11 + H + C)
    M = N * H * H
    dy, w = f32(g, (N, H, H, C)), f32(g, (3, 3, C, C), (2.0 / (9 * C)) ** 0.5)
    add = f32(g, (N, H, H, C)) if with_add else None
    xc = f32(g, (N, H, H, C), 2.0) + np.float32(0.5)                    # the batch norm's input
    gamma, beta = (1 + 0.2 * g.standard_normal(C)).astype(np.float32), f32(g, C, 0.3)
    L = B.lib()
    st = stream_ptr()
    parts = L.dsspk_conv_fwd_stat_parts(N, H, H, C, C, 3, 3, 1, 1)
    XC, Ga, Be, DY, W = dev(xc), dev(gamma), dev(beta), dev(dy), dev(w)
    ADD = dev(add) if with_add else None
    act = empty((N, H, H, C)); stats = empty(2 * C); rec = empty(L.dsspk_bn_scratch_floats(M, C))
    rc(L.dsspk_bn_fwd(st, XC.data_ptr(), Ga.data_ptr(), Be.data_ptr(), act.data_ptr(), stats.data_ptr(), rec.data_ptr(),
                      M, C, 1e-5, 1, 0, None, 0, 0, 0, 0))                # forward: act = ReLU(BN(xc)), saves mean / invstd
    dz = empty((N, H, H, C)); dx = empty((N, H, H, C)); dgam = empty(C); dbet = empty(C)
    rc(L.dsspk_conv_bwd_data_post(st, DY.data_ptr(), W.data_ptr(), ADD.data_ptr() if with_add else None, dz.data_ptr(),
                                  act.data_ptr(), XC.data_ptr(), stats.data_ptr(), rec.data_ptr(), N, H, C))
    rc(L.dsspk_bn_bwd_dx(st, XC.data_ptr(), Ga.data_ptr(), stats.data_ptr(), dz.data_ptr(), dx.data_ptr(), dgam.data_ptr(),
                         dbet.data_ptr(), rec.data_ptr(), M, C, parts))
    x64 = np.zeros((N, H, H, C))
    dxo, _, _ = oracle_nn.conv2d_bwd(x64, w.astype(np.float64), dy.astype(np.float64), 1, 1, False)
    r = dxo + (add if with_add else 0)
    mask = host(act) > 0                                               # decisions of the forward pass (same bits on both sides)
    dzo = np.where(mask, r, 0)
    assert rel_l2(host(dz), dzo) < TOL
    _, mean, invstd = oracle_nn.bn_fwd(xc.astype(np.float64), gamma.astype(np.float64), beta.astype(np.float64))
    dxb, dgo, dbo = oracle_nn.bn_bwd(xc.astype(np.float64), gamma.astype(np.float64), mean, invstd, dzo)
    assert rel_l2(host(dgam), dgo) < 5e-6 and rel_l2(host(dbet), dbo) < 5e-6
    assert rel_l2(host(dx), dxb) < 5e-6


@pytest.mark.parametrize("N,H,C,with_add,carry", [(3, 32, 16, True, True), (5, 16, 32, False, True), (4, 8, 64, True, False),
                                                  (128, 32, 16, True, True), (128, 8, 64, True, True)])
def test_dgrad_with_batchnorm_backward_in_its_loader(oracle_nn, N, H, C, with_add, carry):
    """dz -> [batch-norm backward folded into the loader] -> d-input convolution (+ add, in place) -> ReLU mask +
    records of the next batch norm; the kernel optionally carries a d-filter reduction.  Against the oracle's
    BN backward, d-input convolution and BN backward again."""
    g = np.random.default_rng(N * 13 + H + C)
    M = N * H * H
    w = f32(g, (3, 3, C, C), (2.0 / (9 * C)) ** 0.5)
    xa = f32(g, (N, H, H, C), 1.5) - np.float32(0.3)                    # input of batch norm A (behind the convolution)
    xb = f32(g, (N, H, H, C), 2.0) + np.float32(0.5)                    # input of batch norm B (ahead of it)
    ga, gb = (1 + 0.2 * g.standard_normal(C)).astype(np.float32), (1 + 0.2 * g.standard_normal(C)).astype(np.float32)
    be = f32(g, C, 0.3)
    dz = f32(g, (N, H, H, C)) * (g.random((N, H, H, C)) < 0.6)          # masked gradient at A's output
    dz = dz.astype(np.float32)
    add = f32(g, (N, H, H, C)) if with_add else None
    L = B.lib()
    st = stream_ptr()
    parts = L.dsspk_conv_fwd_stat_parts(N, H, H, C, C, 3, 3, 1, 1)
    XA, XB, GA, GB, BE, DZ, W = dev(xa), dev(xb), dev(ga), dev(gb), dev(be), dev(dz), dev(w)
    tmp = empty((N, H, H, C)); actb = empty((N, H, H, C)); sta = empty(2 * C); stb = empty(2 * C)
    scr = empty(L.dsspk_bn_scratch_floats(M, C))
    rc(L.dsspk_bn_fwd(st, XA.data_ptr(), GA.data_ptr(), BE.data_ptr(), tmp.data_ptr(), sta.data_ptr(), scr.data_ptr(),
                      M, C, 1e-5, 1, 0, None, 0, 0, 0, 0))
    rc(L.dsspk_bn_fwd(st, XB.data_ptr(), GB.data_ptr(), BE.data_ptr(), actb.data_ptr(), stb.data_ptr(), scr.data_ptr(),
                      M, C, 1e-5, 1, 0, None, 0, 0, 0, 0))
    _, mean_a, invstd_a = oracle_nn.bn_fwd(xa.astype(np.float64), ga.astype(np.float64), be.astype(np.float64))
    xhat = (xa.astype(np.float64) - mean_a) * invstd_a
    tot = np.concatenate([dz.astype(np.float64).sum((0, 1, 2)), (dz * xhat).sum((0, 1, 2))]).astype(np.float32)
    TOT = dev(tot)
    E, chunks = 9 * C * C, 37
    part = f32(g, (chunks, E))
    PART = dev(part); red = empty(E)
    dx = empty((N, H, H, C)); rec = empty(2 * parts * C)
    out = dev(add) if with_add else empty((N, H, H, C))                 # in place over the add operand
    rc(L.dsspk_conv_bwd_data_bn(st, DZ.data_ptr(), XA.data_ptr(), sta.data_ptr(), GA.data_ptr(), TOT.data_ptr(), dx.data_ptr(),
                                W.data_ptr(), out.data_ptr() if with_add else None, out.data_ptr(),
                                actb.data_ptr(), XB.data_ptr(), stb.data_ptr(), rec.data_ptr(),
                                PART.data_ptr() if carry else None, red.data_ptr(), E, chunks, N, H, C))
    dxo, _, _ = oracle_nn.bn_bwd(xa.astype(np.float64), ga.astype(np.float64), mean_a, invstd_a, dz.astype(np.float64))
    assert rel_l2(host(dx), dxo) < 5e-6
    r, _, _ = oracle_nn.conv2d_bwd(np.zeros((N, H, H, C)), w.astype(np.float64), dxo, 1, 1, False)
    r = r + (add if with_add else 0)
    dzo = np.where(host(actb) > 0, r, 0)
    assert rel_l2(host(out), dzo) < 5e-6
    if carry:
        assert rel_l2(host(red), part.astype(np.float64).sum(0)) < TOL
        ref = empty(E)
        rc(L.dsspk_wgrad_reduce(st, PART.data_ptr(), ref.data_ptr(), E, chunks))
        assert np.array_equal(host(red), host(ref))                     # same bits whoever carries the job
    totb = empty(2 * C); dgam = empty(C); dbet = empty(C)
    rc(L.dsspk_bn_bwd_totals(st, rec.data_ptr(), parts, C, totb.data_ptr(), dgam.data_ptr(), dbet.data_ptr()))
    _, mean_b, invstd_b = oracle_nn.bn_fwd(xb.astype(np.float64), gb.astype(np.float64), be.astype(np.float64))
    _, dgo, dbo = oracle_nn.bn_bwd(xb.astype(np.float64), gb.astype(np.float64), mean_b, invstd_b, dzo)
    assert rel_l2(host(dgam), dgo) < 5e-6 and rel_l2(host(dbet), dbo) < 5e-6
    assert np.array_equal(host(totb), np.concatenate([host(dbet), host(dgam)]))


@pytest.mark.parametrize("N,H,C,with_add", [(3, 32, 16, True), (5, 16, 32, False), (128, 32, 16, True), (128, 16, 32, True)])
def test_dinput_and_dfilter_in_one_kernel(oracle_nn, N, H, C, with_add):
    """The fused backward kernel of a regular layer: BN backward in the loader, d-input convolution with mask and
    records, and the d-filter partial sums from the same LDS tiles; a reduction job of an earlier layer rides along."""
    g = np.random.default_rng(N * 19 + H + C)
    M = N * H * H
    w = f32(g, (3, 3, C, C), (2.0 / (9 * C)) ** 0.5)
    xa = f32(g, (N, H, H, C), 1.5) - np.float32(0.3)                    # input of batch norm A (behind the convolution)
    xb = f32(g, (N, H, H, C), 2.0) + np.float32(0.5)                    # input of batch norm B (ahead of it)
    ga, gb = (1 + 0.2 * g.standard_normal(C)).astype(np.float32), (1 + 0.2 * g.standard_normal(C)).astype(np.float32)
    be = f32(g, C, 0.3)
    dz = (f32(g, (N, H, H, C)) * (g.random((N, H, H, C)) < 0.6)).astype(np.float32)
    add = f32(g, (N, H, H, C)) if with_add else None
    L = B.lib()
    st = stream_ptr()
    parts = L.dsspk_conv_fwd_stat_parts(N, H, H, C, C, 3, 3, 1, 1)
    chunks = L.dsspk_conv_bwd_fused_chunks(N, H, C)
    assert chunks > 0
    XA, XB, GA, GB, BE, DZ, W = dev(xa), dev(xb), dev(ga), dev(gb), dev(be), dev(dz), dev(w)
    tmp = empty((N, H, H, C)); actb = empty((N, H, H, C)); sta = empty(2 * C); stb = empty(2 * C)
    scr = empty(L.dsspk_bn_scratch_floats(M, C))
    rc(L.dsspk_bn_fwd(st, XA.data_ptr(), GA.data_ptr(), BE.data_ptr(), tmp.data_ptr(), sta.data_ptr(), scr.data_ptr(),
                      M, C, 1e-5, 1, 0, None, 0, 0, 0, 0))
    rc(L.dsspk_bn_fwd(st, XB.data_ptr(), GB.data_ptr(), BE.data_ptr(), actb.data_ptr(), stb.data_ptr(), scr.data_ptr(),
                      M, C, 1e-5, 1, 0, None, 0, 0, 0, 0))
    _, mean_a, invstd_a = oracle_nn.bn_fwd(xa.astype(np.float64), ga.astype(np.float64), be.astype(np.float64))
    xhat = (xa.astype(np.float64) - mean_a) * invstd_a
    tot = np.concatenate([dz.astype(np.float64).sum((0, 1, 2)), (dz * xhat).sum((0, 1, 2))]).astype(np.float32)
    TOT = dev(tot)
    E, old_chunks = 9 * C * C, 19
    part = f32(g, (old_chunks, E))
    PART = dev(part); red = empty(E)
    rec = empty(2 * parts * C); partial = empty(chunks * E); dw = empty((3, 3, C, C))
    out = dev(add) if with_add else empty((N, H, H, C))                 # in place over the add operand
    x_in = host(actb)                                                   # the convolution's input is B's post-ReLU output
    rc(L.dsspk_conv_bwd_data_bn_wgrad(st, DZ.data_ptr(), XA.data_ptr(), sta.data_ptr(), GA.data_ptr(), TOT.data_ptr(),
                                      W.data_ptr(), out.data_ptr() if with_add else None, out.data_ptr(),
                                      XB.data_ptr(), stb.data_ptr(), rec.data_ptr(),
                                      actb.data_ptr(), partial.data_ptr(), PART.data_ptr(), red.data_ptr(), E, old_chunks, N, H, C))
    rc(L.dsspk_wgrad_reduce(st, partial.data_ptr(), dw.data_ptr(), E, chunks))
    dxo, _, _ = oracle_nn.bn_bwd(xa.astype(np.float64), ga.astype(np.float64), mean_a, invstd_a, dz.astype(np.float64))
    r, dwo, _ = oracle_nn.conv2d_bwd(x_in.astype(np.float64), w.astype(np.float64), dxo, 1, 1, False)
    assert rel_l2(host(dw), dwo) < 5e-6
    r = r + (add if with_add else 0)
    dzo = np.where(host(actb) > 0, r, 0)
    assert rel_l2(host(out), dzo) < 5e-6
    assert rel_l2(host(red), part.astype(np.float64).sum(0)) < TOL
    totb = empty(2 * C); dgam = empty(C); dbet = empty(C)
    rc(L.dsspk_bn_bwd_totals(st, rec.data_ptr(), parts, C, totb.data_ptr(), dgam.data_ptr(), dbet.data_ptr()))
    _, mean_b, invstd_b = oracle_nn.bn_fwd(xb.astype(np.float64), gb.astype(np.float64), be.astype(np.float64))
    _, dgo, dbo = oracle_nn.bn_bwd(xb.astype(np.float64), gb.astype(np.float64), mean_b, invstd_b, dzo)
    assert rel_l2(host(dgam), dgo) < 5e-6 and rel_l2(host(dbet), dbo) < 5e-6


@pytest.mark.parametrize("N,H,C", [(3, 32, 16), (5, 16, 32), (4, 8, 64), (7, 8, 64), (128, 16, 32), (128, 8, 64)])
def test_wgrad_in_two_stages_carrying_batchnorm_sums(oracle_nn, N, H, C):
    """Stage 1 of the d-filter convolution with the batch-norm sums job as extra workgroups, stage 2 on its own."""
    g = np.random.default_rng(N * 17 + H + C)
    x, dy = f32(g, (N, H, H, C)), f32(g, (N, H, H, C))
    G = 4 * N if H == 32 else (2 * N if H == 16 else N)
    rec = f32(g, (G, C, 2))
    L = B.lib()
    st = stream_ptr()
    X, DY, REC = dev(x), dev(dy), dev(rec)
    scr = empty(L.dsspk_conv_wgrad_scratch_floats(N, H, H, C, C, 3, 3, 1, 1))
    tot = empty(2 * C); dgam = empty(C); dbet = empty(C); dw = empty((3, 3, C, C))
    import ctypes
    chunks = ctypes.c_int(0)
    rc(L.dsspk_conv_bwd_weight_parts(st, X.data_ptr(), DY.data_ptr(), scr.data_ptr(), N, H, H, C, C, 3, 3, 1, 1,
                                     REC.data_ptr(), G, C, tot.data_ptr(), dgam.data_ptr(), dbet.data_ptr(), ctypes.byref(chunks)))
    assert chunks.value >= 1
    rc(L.dsspk_wgrad_reduce(st, scr.data_ptr(), dw.data_ptr(), 9 * C * C, chunks.value))
    _, dwo, _ = oracle_nn.conv2d_bwd(x.astype(np.float64), np.zeros((3, 3, C, C)), dy.astype(np.float64), 1, 1, False)
    assert rel_l2(host(dw), dwo) < TOL
    sums = rec.astype(np.float64).sum(0)
    assert rel_l2(host(dbet), sums[:, 0]) < TOL and rel_l2(host(dgam), sums[:, 1]) < TOL
    ref = empty(2 * C); d1 = empty(C); d2 = empty(C)
    rc(L.dsspk_bn_bwd_totals(st, REC.data_ptr(), G, C, ref.data_ptr(), d1.data_ptr(), d2.data_ptr()))
    assert np.array_equal(host(tot), host(ref)) and np.array_equal(host(tot), np.concatenate([host(dbet), host(dgam)]))


# ------------------------------------------------------------------ elementwise / pooling
@pytest.mark.parametrize("n", [5, 64, 100003])
def test_relu_bwd_and_add(n):
    g = np.random.default_rng(n)
    n4 = (n + 3) // 4 * 4
    a, dy = f32(g, n4), f32(g, n4)
    a[::7] = 0.0
    A, DY = dev(a), dev(dy)
    rc(B.lib().dsspk_relu_bwd(stream_ptr(), DY.data_ptr(), A.data_ptr(), n))
    got = host(DY)
    assert np.array_equal(got[:n], np.where(a[:n] > 0, dy[:n], 0)) and np.array_equal(got[n:], dy[n:])
    rc(B.lib().dsspk_add(stream_ptr(), DY.data_ptr(), A.data_ptr(), n))
    assert np.array_equal(host(DY)[:n], got[:n] + a[:n])


@pytest.mark.parametrize("N,H,C", [(2, 32, 64), (3, 15, 64), (1, 5, 4), (128, 15, 64), (2, 9, 6), (1, 4, 3)])
def test_maxpool(oracle_nn, N, H, C):        # C = 6, 3: channel counts the 16-byte kernels do not take (scalar kernels)
    g = np.random.default_rng(H)
    x = f32(g, (N, H, H, C))
    Ho = (H - 3) // 2 + 1
    dy = f32(g, (N, Ho, Ho, C))
    X, DY = dev(x), dev(dy)
    y = empty((N, Ho, Ho, C)); arg = empty((N, Ho, Ho, C), torch.uint8); dx = empty((N, H, H, C))
    rc(B.lib().dsspk_maxpool_fwd(stream_ptr(), X.data_ptr(), y.data_ptr(), arg.data_ptr(), N, H, H, C))
    rc(B.lib().dsspk_maxpool_bwd(stream_ptr(), DY.data_ptr(), arg.data_ptr(), dx.data_ptr(), N, H, H, C))
    yo, argo, _ = oracle_nn.maxpool_fwd(x.astype(np.float64), 3, 2, None, 0.0)
    assert np.array_equal(host(arg), argo.astype(np.uint8))           # same inputs, exact comparisons
    assert np.array_equal(host(y).astype(np.float64), yo)
    dxo = oracle_nn.maxpool_bwd(dy.astype(np.float64), argo, x.shape, 3, 2)
    assert rel_l2(host(dx), dxo) < TOL
    # with the backward pass of the ReLU in front of the pooling folded in (mask from the pooling's input)
    dxm = empty((N, H, H, C))
    rc(B.lib().dsspk_maxpool_bwd_relu(stream_ptr(), DY.data_ptr(), arg.data_ptr(), X.data_ptr(), dxm.data_ptr(), N, H, H, C))
    assert np.array_equal(host(dxm), np.where(x > 0, host(dx), np.float32(0)))


# ------------------------------------------------------------------ batch normalisation (+ shortcut, ReLU)
@pytest.mark.parametrize("N,H,C,mode,relu", [(5, 32, 16, 0, 1), (3, 16, 32, 1, 1), (5, 8, 64, 2, 1), (2, 16, 32, 2, 1),
                                             (3, 7, 16, 0, 0), (128, 32, 16, 1, 1), (128, 8, 64, 0, 1)])
def test_batchnorm_forward_backward(oracle_nn, N, H, C, mode, relu):
    g = np.random.default_rng(N * 1000 + H * 10 + mode)
    M = N * H * H
    x = f32(g, (N, H, H, C), 2.0) + np.float32(1.5)
    gamma, beta = (1 + 0.2 * g.standard_normal(C)).astype(np.float32), f32(g, C, 0.3)
    da = f32(g, (N, H, H, C))
    sc = None
    if mode == 1:
        sc = f32(g, (N, H, H, C))
    elif mode == 2:
        sc = f32(g, (N, 2 * H, 2 * H, C // 2))
    L = B.lib()
    st = stream_ptr()
    X, Ga, Be, DA = dev(x), dev(gamma), dev(beta), dev(da)
    SC = dev(sc) if sc is not None else None
    y = empty((N, H, H, C)); stats = empty(2 * C); scratch = empty(L.dsspk_bn_scratch_floats(M, C))
    rc(L.dsspk_bn_fwd(st, X.data_ptr(), Ga.data_ptr(), Be.data_ptr(), y.data_ptr(), stats.data_ptr(), scratch.data_ptr(),
                      M, C, 1e-5, relu, mode, SC.data_ptr() if SC is not None else None, N, H, H, 0))
    x64 = x.astype(np.float64)
    yo, mean, invstd = oracle_nn.bn_fwd(x64, gamma.astype(np.float64), beta.astype(np.float64))
    if mode == 1:
        yo = yo + sc
    elif mode == 2:
        yo = yo + oracle_nn.shortcut_pad_fwd(sc.astype(np.float64), C)
    zo = yo
    if relu:
        yo = np.maximum(yo, 0)
    assert rel_l2(host(stats)[:C], mean) < TOL and rel_l2(host(stats)[C:], invstd) < TOL
    got = host(y)
    assert rel_l2(got, yo) < TOL
    # backward; the ReLU mask is taken from the saved forward output on both sides
    dx = empty((N, H, H, C)); dgam = empty(C); dbet = empty(C)
    rc(L.dsspk_bn_bwd(st, X.data_ptr(), Ga.data_ptr(), stats.data_ptr(), DA.data_ptr(), y.data_ptr() if relu else None,
                      dx.data_ptr(), dgam.data_ptr(), dbet.data_ptr(), scratch.data_ptr(), M, C))
    mask = (got > 0) if relu else np.ones_like(got, dtype=bool)
    near = np.abs(zo) < 1e-5                                  # decisions the two precisions may take differently
    assert np.array_equal(mask[~near], (zo > 0)[~near] if relu else mask[~near])
    dz = np.where(mask, da, 0).astype(np.float64)
    dxo, dgo, dbo = oracle_nn.bn_bwd(x64, gamma.astype(np.float64), mean, invstd, dz)
    assert np.array_equal(host(DA), dz.astype(np.float32))    # masked gradient written back in place
    assert rel_l2(host(dx), dxo) < 5e-6
    assert rel_l2(host(dgam), dgo) < TOL and rel_l2(host(dbet), dbo) < TOL


def test_shortcut_gap_softmax(oracle_nn):
    g = np.random.default_rng(5)
    L = B.lib()
    st = stream_ptr()
    N, Ho, C = 3, 8, 64
    dy, dx0 = f32(g, (N, Ho, Ho, C)), f32(g, (N, 2 * Ho, 2 * Ho, C // 2))
    DY, DX = dev(dy), dev(dx0)
    rc(L.dsspk_shortcut_bwd_acc(st, DY.data_ptr(), DX.data_ptr(), N, Ho, Ho, C))
    want = dx0.astype(np.float64)
    oracle_nn.shortcut_pad_bwd_acc(dy.astype(np.float64), want)
    assert rel_l2(host(DX), want) < 1e-7
    x = f32(g, (5, 8, 8, 64))
    X = dev(x); y = empty((5, 64)); dxx = empty((5, 8, 8, 64))
    rc(L.dsspk_gap_fwd(st, X.data_ptr(), y.data_ptr(), 5, 64, 64))
    assert rel_l2(host(y), oracle_nn.gap_fwd(x.astype(np.float64))) < TOL
    rc(L.dsspk_gap_bwd(st, y.data_ptr(), dxx.data_ptr(), 5, 64, 64))
    assert rel_l2(host(dxx), oracle_nn.gap_bwd(host(y).astype(np.float64), x.shape)) < TOL
    for m, C in [(128, 100), (32, 10), (7, 3)]:
        z = f32(g, (m, C), 4.0)
        lab = g.integers(0, C, m).astype(np.int32)
        Z, Y = dev(z), dev(lab)
        dz = empty((m, C)); loss = empty(1)
        rc(L.dsspk_softmax_xent(st, Z.data_ptr(), Y.data_ptr(), dz.data_ptr(), loss.data_ptr(), m, C))
        lo, dzo = oracle_nn.softmax_xent(z.astype(np.float64), lab)
        assert abs(host(loss)[0] - lo) < 2e-6 * max(1, abs(lo))
        assert rel_l2(host(dz), dzo) < TOL


# ------------------------------------------------------------------ streams and hardware queues
def test_streams_are_grouped_by_hardware_queue():
    pool = [torch.cuda.Stream() for _ in range(10)]
    streams = pool + [pool[3], pool[0]]
    queue, nq = B.dssp_stream_queues(streams)
    # a process has 4 hardware queues unless GPU_MAX_HW_QUEUES says otherwise, so ten streams must share some
    assert 1 <= nq <= int(os.environ.get("GPU_MAX_HW_QUEUES", 4)) and sorted(set(queue)) == list(range(nq))
    assert queue[0] == 0 and all(queue[i] <= max(queue[:i]) + 1 for i in range(1, len(queue)))   # numbered by first appearance
    assert queue[10] == queue[3] and queue[11] == queue[0]                                       # the same stream twice
    again, nq2 = B.dssp_stream_queues(streams)
    assert (again, nq2) == (queue, nq)
    # the grouping is real: a spin on one stream holds up a stream of the same queue and no stream of another
    if nq > 1:
        a = queue.index(0)
        other = next(i for i, q in enumerate(queue) if q != 0)
        pair, _ = B.dssp_stream_queues([streams[a], streams[other]])
        assert pair == [0, 1]
    same = [i for i, q in enumerate(queue[:10]) if q == queue[0]]
    if len(same) > 1:
        pair, n_pair = B.dssp_stream_queues([streams[same[0]], streams[same[1]]])
        assert pair == [0, 0] and n_pair == 1
    with pytest.raises(B.DsspError):
        B.dssp_stream_queues([pool[0]] * 65)
