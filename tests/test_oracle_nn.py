"""Pins of the oracle's numerics (oracle/nn_layers.c, nn.py, ps.py).

Nothing here compares the oracle with itself: the checks are central finite
differences of the loss (Alg. 1, worker step 4: the gradient is the derivative
of the mean mini-batch loss), torch's fp64 autograd on the same network (a
library special case), brute-force Python loops, closed forms and invariants.
"""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from paper_1908_11848_amd import inputs


def seg_table(net):
    out = []
    for name, shape in net.segments():
        kind = {"w": inputs.KIND_WEIGHT, "b": inputs.KIND_BETA if ".bn" in name else inputs.KIND_BIAS,
                "g": inputs.KIND_GAMMA}[name.rsplit(".", 1)[1]]
        out.append((kind, int(np.prod(shape)), int(np.prod(shape[:-1])) if kind == inputs.KIND_WEIGHT else 0))
    return out


def rel(a, b):
    return float(np.linalg.norm(np.asarray(a, dtype=np.float64) - b) / max(np.linalg.norm(b), 1e-300))


# ------------------------------------------------------------------ finite differences
def test_mlp_gradient_finite_differences(oracle_nn):
    net = oracle_nn.MLP(n_in=12, hidden=7, n_classes=5)
    g = np.random.default_rng(0)
    w = g.standard_normal(net.n_params()) * 0.5
    x = g.standard_normal((6, 12))
    y = g.integers(0, 5, 6).astype(np.int32)
    loss, grad, _ = net.loss_and_grad(w, x, y)
    h = 1e-6
    fd = np.empty_like(w)
    for i in range(w.size):
        wp, wm = w.copy(), w.copy()
        wp[i] += h
        wm[i] -= h
        fd[i] = (net.loss_and_grad(wp, x, y)[0] - net.loss_and_grad(wm, x, y)[0]) / (2 * h)
    assert rel(grad, fd) < 1e-7
    # the loss itself, from the definition
    P = net.unpack(w)
    z = np.maximum(x @ P["fc1.w"] + P["fc1.b"], 0) @ P["fc2.w"] + P["fc2.b"]
    ref = np.mean(np.log(np.exp(z).sum(1)) - z[np.arange(6), y])
    assert abs(loss - ref) < 1e-12


def test_resnet_directional_finite_difference(oracle_nn):
    net = oracle_nn.ResNetCifar(n=1, n_classes=7)
    g = np.random.default_rng(1)
    w = inputs.init_weights(seg_table(net), 4, jitter=0.1).astype(np.float64)
    x = g.standard_normal((4, 32, 32, 3))
    y = g.integers(0, 7, 4).astype(np.int32)
    _, grad, _ = net.loss_and_grad(w, x, y)
    for k in range(3):
        v = g.standard_normal(w.size)
        v /= np.linalg.norm(v)
        h = 1e-6
        fd = (net.loss_and_grad(w + h * v, x, y)[0] - net.loss_and_grad(w - h * v, x, y)[0]) / (2 * h)
        assert abs(fd - grad @ v) < 1e-6 * max(1.0, abs(fd))


# ------------------------------------------------------------------ torch fp64 autograd (library special case)
def t_param(P, name, conv=False, fc=False):
    a = torch.tensor(P[name], dtype=torch.float64)
    if conv:
        a = a.permute(3, 2, 0, 1)        # [KH][KW][Cin][Cout] -> [Cout][Cin][KH][KW]
    if fc:
        a = a.t()                        # [in][out] -> [out][in]
    return a.contiguous().requires_grad_(True)


def back_to_flat(net, tp):
    G = {}
    for name, shape in net.segments():
        g = tp[name].grad
        if len(shape) == 4:
            g = g.permute(2, 3, 1, 0)
        elif len(shape) == 2:
            g = g.t()
        G[name] = g.contiguous().numpy()
    return net.pack(G)


def test_alexnet_against_torch_autograd(oracle_nn):
    net = oracle_nn.AlexNetDS(n_classes=10)
    g = np.random.default_rng(2)
    w = inputs.init_weights(seg_table(net), 2, jitter=0.1).astype(np.float64)
    x = g.standard_normal((3, 32, 32, 3))
    y = g.integers(0, 10, 3).astype(np.int32)
    loss, grad, trace = net.loss_and_grad(w, x, y)
    P = net.unpack(w)
    tp = {n: t_param(P, n, conv=len(s) == 4, fc=len(s) == 2) for n, s in net.segments()}
    h = torch.tensor(x).permute(0, 3, 1, 2)
    h = F.max_pool2d(F.relu(F.conv2d(h, tp["conv1.w"], tp["conv1.b"], padding=2)), 3, 2)
    h = F.max_pool2d(F.relu(F.conv2d(h, tp["conv2.w"], tp["conv2.b"], padding=2)), 3, 2)
    h = h.permute(0, 2, 3, 1).reshape(3, -1)          # (h, w, c) flatten order
    h = F.relu(F.linear(h, tp["fc1.w"], tp["fc1.b"]))
    h = F.relu(F.linear(h, tp["fc2.w"], tp["fc2.b"]))
    z = F.linear(h, tp["fc3.w"], tp["fc3.b"])
    L = F.cross_entropy(z, torch.tensor(y, dtype=torch.long))
    L.backward()
    assert abs(loss - L.item()) < 1e-12
    assert rel(trace["logits"], z.detach().numpy()) < 1e-13
    assert rel(grad, back_to_flat(net, tp)) < 1e-12


def test_alexnet_3conv_against_torch_autograd(oracle_nn):
    net = oracle_nn.AlexNet3C(n_classes=10)
    g = np.random.default_rng(5)
    w = inputs.init_weights(seg_table(net), 2, jitter=0.1).astype(np.float64)
    x = g.standard_normal((3, 32, 32, 3))
    y = g.integers(0, 10, 3).astype(np.int32)
    loss, grad, trace = net.loss_and_grad(w, x, y)
    P = net.unpack(w)
    tp = {n: t_param(P, n, conv=len(s) == 4, fc=len(s) == 2) for n, s in net.segments()}
    h = torch.tensor(x).permute(0, 3, 1, 2)
    h = F.max_pool2d(F.relu(F.conv2d(h, tp["conv1.w"], tp["conv1.b"], padding=2)), 3, 2)
    h = F.max_pool2d(F.relu(F.conv2d(h, tp["conv2.w"], tp["conv2.b"], padding=2)), 3, 2)
    h = F.relu(F.conv2d(h, tp["conv3.w"], tp["conv3.b"], padding=1))
    h = h.permute(0, 2, 3, 1).reshape(3, -1)          # (h, w, c) flatten order
    h = F.relu(F.linear(h, tp["fc1.w"], tp["fc1.b"]))
    z = F.linear(h, tp["fc2.w"], tp["fc2.b"])
    L = F.cross_entropy(z, torch.tensor(y, dtype=torch.long))
    L.backward()
    assert abs(loss - L.item()) < 1e-12
    assert rel(trace["logits"], z.detach().numpy()) < 1e-13
    assert rel(grad, back_to_flat(net, tp)) < 1e-12
    assert net.n_params() == 4864 + 102464 + 36928 + 3136 * 384 + 384 + 3850


@pytest.mark.parametrize("n", [1, 2])
def test_resnet_against_torch_autograd(oracle_nn, n):
    net = oracle_nn.ResNetCifar(n=n, n_classes=11)
    g = np.random.default_rng(3)
    w = inputs.init_weights(seg_table(net), 4, jitter=0.1).astype(np.float64)
    m = 5
    x = g.standard_normal((m, 32, 32, 3))
    y = g.integers(0, 11, m).astype(np.int32)
    loss, grad, trace = net.loss_and_grad(w, x, y)
    P = net.unpack(w)
    tp = {nm: t_param(P, nm, conv=len(s) == 4, fc=len(s) == 2) for nm, s in net.segments()}

    def bn(h, pre):
        return F.batch_norm(h, None, None, tp[pre + ".g"], tp[pre + ".b"], training=True, eps=1e-5)

    h = torch.tensor(x).permute(0, 3, 1, 2)
    h = F.relu(bn(F.conv2d(h, tp["stem.conv.w"], padding=1), "stem.bn"))
    for name, cin, cout, stride in net.blocks:
        o = F.relu(bn(F.conv2d(h, tp[name + ".conv1.w"], stride=stride, padding=1), name + ".bn1"))
        o = bn(F.conv2d(o, tp[name + ".conv2.w"], padding=1), name + ".bn2")
        sc = h if stride == 1 and cin == cout else F.pad(h[:, :, ::2, ::2], (0, 0, 0, 0, 0, cout - cin))
        h = F.relu(o + sc)
    z = F.linear(h.mean((2, 3)), tp["fc.w"], tp["fc.b"])
    L = F.cross_entropy(z, torch.tensor(y, dtype=torch.long))
    L.backward()
    assert abs(loss - L.item()) < 1e-11
    assert rel(grad, back_to_flat(net, tp)) < 1e-10


# ------------------------------------------------------------------ brute force / closed forms / invariants
def test_conv_forward_brute_force(oracle_nn):
    g = np.random.default_rng(4)
    for (H, W, Cin, Cout, K, s, p) in [(5, 6, 2, 3, 3, 1, 1), (7, 7, 3, 2, 5, 1, 2), (6, 6, 2, 4, 3, 2, 1)]:
        x = g.standard_normal((2, H, W, Cin))
        w = g.standard_normal((K, K, Cin, Cout))
        b = g.standard_normal(Cout)
        y = oracle_nn.conv2d_fwd(x, w, b, s, p)
        Ho, Wo = (H + 2 * p - K) // s + 1, (W + 2 * p - K) // s + 1
        assert y.shape == (2, Ho, Wo, Cout)
        for n, ho, wo, co in itertools.product(range(2), range(Ho), range(Wo), range(Cout)):
            acc = b[co]
            for kh, kw, ci in itertools.product(range(K), range(K), range(Cin)):
                hi, wi = ho * s + kh - p, wo * s + kw - p
                if 0 <= hi < H and 0 <= wi < W:
                    acc += x[n, hi, wi, ci] * w[kh, kw, ci, co]
            assert abs(acc - y[n, ho, wo, co]) < 1e-12


def test_conv_backward_is_adjoint(oracle_nn):
    # <conv(x; w), dy> is bilinear: its derivative along dx is <conv(dx; w), dy>, along dw <conv(x; dw), dy>
    g = np.random.default_rng(5)
    for (H, Cin, Cout, K, s, p) in [(8, 3, 4, 3, 1, 1), (8, 3, 4, 3, 2, 1), (9, 2, 3, 5, 1, 2), (7, 2, 2, 3, 2, 1)]:
        x = g.standard_normal((2, H, H, Cin))
        w = g.standard_normal((K, K, Cin, Cout))
        y = oracle_nn.conv2d_fwd(x, w, None, s, p)
        dy = g.standard_normal(y.shape)
        dx, dw, db = oracle_nn.conv2d_bwd(x, w, dy, s, p, True)
        ex, ew = g.standard_normal(x.shape), g.standard_normal(w.shape)
        assert abs(np.vdot(dx, ex) - np.vdot(oracle_nn.conv2d_fwd(ex, w, None, s, p), dy)) < 1e-10
        assert abs(np.vdot(dw, ew) - np.vdot(oracle_nn.conv2d_fwd(x, ew, None, s, p), dy)) < 1e-10
        assert np.allclose(db, dy.sum((0, 1, 2)), atol=1e-12)


def test_bn_invariants(oracle_nn):
    g = np.random.default_rng(6)
    x = g.standard_normal((4, 5, 5, 3)) * 3 + 2
    y, mean, invstd = oracle_nn.bn_fwd(x, np.ones(3), np.zeros(3))
    assert np.allclose(y.mean((0, 1, 2)), 0, atol=1e-13)
    assert np.allclose(y.var((0, 1, 2)), 1, atol=1e-5)             # eps = 1e-5 inside the root
    assert np.allclose(mean, x.mean((0, 1, 2))) and np.allclose(invstd, 1 / np.sqrt(x.var((0, 1, 2)) + 1e-5))
    gamma = g.standard_normal(3)
    dy = g.standard_normal(x.shape)
    dx, dgamma, dbeta = oracle_nn.bn_bwd(x, gamma, mean, invstd, dy)
    assert np.allclose(dx.sum((0, 1, 2)), 0, atol=1e-12)           # shifting x by a constant changes nothing
    assert np.allclose((dx * (x - mean)).sum((0, 1, 2)), 0, atol=1e-4 * np.abs(dx).max())   # nor (to eps) scaling
    assert np.allclose(dbeta, dy.sum((0, 1, 2)))


def test_softmax_xent_closed_forms(oracle_nn):
    z = np.zeros((4, 10))
    loss, dz = oracle_nn.softmax_xent(z, np.array([0, 3, 5, 9], dtype=np.int32))
    assert abs(loss - np.log(10)) < 1e-14
    assert np.allclose(dz.sum(1), 0, atol=1e-16)
    assert np.isclose(dz[1, 3], (0.1 - 1) / 4) and np.isclose(dz[1, 2], 0.1 / 4)
    big = np.array([[1000.0, 0.0, -1000.0]])
    loss, dz = oracle_nn.softmax_xent(big, np.array([0], dtype=np.int32))
    assert np.isfinite(loss) and abs(loss) < 1e-12


def test_maxpool_and_tie_breaks(oracle_nn):
    x = np.zeros((1, 5, 5, 1))
    x[0, 1, 1, 0] = 2.0
    x[0, 2, 2, 0] = 2.0 + 1e-6          # near tie in the top-left window
    x[0, 4, 4, 0] = 1.0
    y, arg, gap = oracle_nn.maxpool_fwd(x, 3, 2, None, 1e-4)
    assert y.shape == (1, 2, 2, 1) and arg[0, 0, 0, 0] == 8 and abs(gap[0, 0, 0, 0] - 1e-6) < 1e-12
    assert arg[0, 1, 1, 0] == 0 and y[0, 1, 1, 0] == 2.0 + 1e-6     # (2,2) is position 0 of window (1,1)
    dx = oracle_nn.maxpool_bwd(np.ones((1, 2, 2, 1)), arg, x.shape, 3, 2)
    assert dx[0, 2, 2, 0] == 4.0 and dx.sum() == 4.0                # the centre wins all four windows
    forced = np.full((1, 2, 2, 1), -1, dtype=np.int32)
    forced[0, 0, 0, 0] = 4                                          # (1,1): within tolerance of the max
    y2, arg2, _ = oracle_nn.maxpool_fwd(x, 3, 2, forced, 1e-4)
    assert arg2[0, 0, 0, 0] == 4 and y2[0, 0, 0, 0] == 2.0
    forced[0, 0, 0, 0] = 0                                          # value 0: not a tie -> refused
    with pytest.raises(ValueError):
        oracle_nn.maxpool_fwd(x, 3, 2, forced, 1e-4)
    z = np.array([[1e-6, -0.5, 0.7]])
    f = np.array([[0, -1, -1]], dtype=np.int8)
    a, act = oracle_nn.relu_fwd(z, f, 1e-4)
    assert list(act[0]) == [0, 0, 1] and a[0, 0] == 0.0
    with pytest.raises(ValueError):
        oracle_nn.relu_fwd(z, np.array([[-1, 1, -1]], dtype=np.int8), 1e-4)


def test_shortcut_and_gap(oracle_nn):
    g = np.random.default_rng(7)
    x = g.standard_normal((2, 6, 6, 3))
    y = oracle_nn.shortcut_pad_fwd(x, 6)
    assert np.array_equal(y[..., :3], x[:, ::2, ::2, :]) and not y[..., 3:].any()
    dy = g.standard_normal(y.shape)
    dx = np.zeros_like(x)
    oracle_nn.shortcut_pad_bwd_acc(dy, dx)
    assert abs(np.vdot(dx, x) - np.vdot(dy, y)) < 1e-12              # adjoint of the forward map
    p = oracle_nn.gap_fwd(x)
    assert np.allclose(p, x.mean((1, 2)))
    assert np.allclose(oracle_nn.gap_bwd(p, x.shape).sum((1, 2)), p)


def test_param_counts(oracle_nn):
    assert oracle_nn.make_net("mlp", 10).n_params() == 789_258
    assert oracle_nn.make_net("alexnet_ds", 10).n_params() == 1_387_786
    assert oracle_nn.make_net("resnet110", 100).n_params() == 1_733_812      # "about 1.7M"


# ------------------------------------------------------------------ server numerics
def tiny_problem(oracle_nn, K, pool, m=4):
    net = oracle_nn.MLP(n_in=10, hidden=6, n_classes=4)
    g = np.random.default_rng(8)
    w0 = g.standard_normal(net.n_params()) * 0.3
    xs = [[g.standard_normal((m, 10)) for _ in range(pool)] for _ in range(K)]
    ys = [[g.integers(0, 4, m).astype(np.int32) for _ in range(pool)] for _ in range(K)]
    return net, w0, xs, ys


def test_bsp_is_synchronous_averaged_sgd(oracle_nn):
    # Sec. I-A: with s_L = r_max = 0 every worker starts each round from the same weights, so a
    # round equals one step of SGD on the gradient averaged over the K workers (brute force below).
    from oracle import ps
    K, rounds, lr = 3, 6, 0.1
    net, w0, xs, ys = tiny_problem(oracle_nn, K, rounds)
    d = np.random.default_rng(9).integers(500, 1500, (K, rounds + 1))
    out = ps.run(K, 0, 0, lr, w0, d, ps.model_grad_fn(net, xs, ys), quota=rounds)
    w = w0.copy()
    for n in range(rounds):
        gs = [net.loss_and_grad(w, xs[p][n], ys[p][n])[1] for p in range(K)]
        w = w - lr * np.mean(gs, axis=0)
    assert rel(out["w"], w) < 1e-14
    assert out["state"].version == K * rounds


def test_rmax0_weights_equal_ssp_and_apply_closed_form(oracle_nn):
    from oracle import ps
    K, n = 4, 64
    d = np.random.default_rng(10).integers(500, 3000, (K, 40))
    gfix = [np.full(n, 2.0 ** -(p + 3)) for p in range(K)]                 # powers of two: exact sums
    out = ps.run(K, 2, 5, 0.5, np.ones(n), d, lambda p, i, w: (0.0, gfix[p]), total=50)
    counts = np.bincount([r["worker"] for r in out["pushes"]], minlength=K)
    want = 1.0 - (0.5 / K) * sum(counts[p] * 2.0 ** -(p + 3) for p in range(K))
    assert np.array_equal(out["w"], np.full(n, want))                      # w0 - scale * sum of pushed g
    assert out["state"].version == 50 == sum(out["state"].t)
