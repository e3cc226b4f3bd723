"""Oracle, part 2b: the three networks and their mini-batch gradient, in fp64.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

gradient = (1/m) sum_i d loss((x_i, y_i), w) / dw   (Alg. 1, worker step 4),
loss = softmax cross-entropy.  Layers are the direct-loop C functions of
nn_layers.c (built by oracle/build.py); this file only chains them.

Flat parameter vector (an interface shared with the library as *data layout*,
not code): layers in forward order; a convolution stores its filter as
[KH][KW][Cin][Cout] followed by its bias [Cout] if it has one; batch norm
stores gamma[C] then beta[C]; a fully connected layer its weight [in][out]
then bias [out].  Images are [m][32][32][3]; a feature map is flattened in
(h, w, c) order before the first fully connected layer.

Discrete decisions.  ReLU's derivative and max-pooling's routing are decided
by comparisons of floating-point values.  Where such a comparison is closer
than `ambig_tol`, both outcomes are equally valid results of the method; the
caller may then name the outcome (`tie_break`), and any attempt to force an
outcome that is NOT within `ambig_tol` of a tie is rejected.  Every decision
and its margin is returned in the trace.
"""

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

_D = ctypes.POINTER(ctypes.c_double)
_I8 = ctypes.POINTER(ctypes.c_int8)
_I32 = ctypes.POINTER(ctypes.c_int32)


def lib():
    global _LIB
    if _LIB is None:
        path = os.path.join(_HERE, "liboracle_nn.so")
        if not os.path.exists(path):
            raise RuntimeError("oracle/liboracle_nn.so missing: run `python oracle/build.py`")
        _LIB = ctypes.CDLL(path)
        _LIB.softmax_xent.restype = ctypes.c_double
    return _LIB


def _d(a):
    return a.ctypes.data_as(_D) if a is not None else None


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


# ----------------------------------------------------------------- layers
def conv2d_fwd(x, w, b, stride, pad):
    N, H, W, Cin = x.shape
    KH, KW, _, Cout = w.shape
    Ho, Wo = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1
    y = np.empty((N, Ho, Wo, Cout))
    lib().conv2d_fwd(_d(x), _d(w), _d(b), _d(y), N, H, W, Cin, Cout, KH, KW, stride, pad)
    return y


def conv2d_bwd(x, w, dy, stride, pad, has_bias, need_dx=True):
    N, H, W, Cin = x.shape
    KH, KW, _, Cout = w.shape
    dw = np.empty_like(w)
    db = np.empty(Cout) if has_bias else None
    lib().conv2d_bwd_weight(_d(x), _d(dy), _d(dw), _d(db), N, H, W, Cin, Cout, KH, KW, stride, pad)
    dx = None
    if need_dx:
        dx = np.empty_like(x)
        lib().conv2d_bwd_data(_d(w), _d(dy), _d(dx), N, H, W, Cin, Cout, KH, KW, stride, pad)
    return dx, dw, db


def fc_fwd(x, w, b):
    m, n_in = x.shape
    y = np.empty((m, w.shape[1]))
    lib().fc_fwd(_d(x), _d(w), _d(b), _d(y), m, n_in, w.shape[1])
    return y


def fc_bwd(x, w, dy, need_dx=True):
    m, n_in = x.shape
    dx = np.empty_like(x) if need_dx else None
    dw = np.empty_like(w)
    db = np.empty(w.shape[1])
    lib().fc_bwd(_d(x), _d(w), _d(dy), _d(dx), _d(dw), _d(db), m, n_in, w.shape[1])
    return dx, dw, db


def relu_fwd(z, forced, ambig_tol):
    """Returns (a, active).  forced: None or int8 array with -1 = free."""
    active = np.full(z.shape, -1, dtype=np.int8)
    if forced is not None:
        forced = np.asarray(forced, dtype=np.int8).reshape(z.shape)
        sel = forced >= 0
        if np.any(np.abs(z[sel]) > ambig_tol):
            raise ValueError("tie-break forces a ReLU decision that is not ambiguous")
        active[sel] = forced[sel]
    a = np.empty_like(z)
    lib().relu_fwd(_d(z), _d(a), active.ctypes.data_as(_I8), ctypes.c_size_t(z.size))
    return a, active


def relu_bwd(da, active):
    dz = np.empty_like(da)
    lib().relu_bwd(_d(da), active.ctypes.data_as(_I8), _d(dz), ctypes.c_size_t(da.size))
    return dz


def maxpool_fwd(x, k, s, forced, ambig_tol):
    """Returns (y, arg, gap).  forced: None or int32 array with -1 = free."""
    N, H, W, C = x.shape
    Ho, Wo = (H - k) // s + 1, (W - k) // s + 1
    y = np.empty((N, Ho, Wo, C))
    gap = np.empty((N, Ho, Wo, C))
    arg = np.full((N, Ho, Wo, C), -1, dtype=np.int32)
    if forced is not None:
        forced = np.asarray(forced, dtype=np.int32).reshape(arg.shape)
        arg[...] = forced
    lib().maxpool_fwd(_d(x), _d(y), arg.ctypes.data_as(_I32), _d(gap), N, H, W, C, k, s)
    if forced is not None and np.any(forced >= 0):
        free = np.full(arg.shape, -1, dtype=np.int32)
        ymax = np.empty_like(y)
        lib().maxpool_fwd(_d(x), _d(ymax), free.ctypes.data_as(_I32), _d(gap), N, H, W, C, k, s)
        if np.any(ymax - y > ambig_tol):
            raise ValueError("tie-break forces a max-pool choice that is not ambiguous")
    return y, arg, gap


def maxpool_bwd(dy, arg, in_shape, k, s):
    N, H, W, C = in_shape
    dx = np.empty(in_shape)
    lib().maxpool_bwd(_d(dy), arg.ctypes.data_as(_I32), _d(dx), N, H, W, C, k, s)
    return dx


def bn_fwd(x, gamma, beta, eps=1e-5):
    C = x.shape[-1]
    M = x.size // C
    y = np.empty_like(x)
    mean, invstd = np.empty(C), np.empty(C)
    lib().bn_fwd(_d(x), _d(gamma), _d(beta), _d(y), _d(mean), _d(invstd),
                 ctypes.c_size_t(M), C, ctypes.c_double(eps))
    return y, mean, invstd


def bn_bwd(x, gamma, mean, invstd, dy):
    C = x.shape[-1]
    M = x.size // C
    dx = np.empty_like(x)
    dgamma, dbeta = np.empty(C), np.empty(C)
    lib().bn_bwd(_d(x), _d(gamma), _d(mean), _d(invstd), _d(dy), _d(dx), _d(dgamma), _d(dbeta),
                 ctypes.c_size_t(M), C)
    return dx, dgamma, dbeta


def gap_fwd(x):
    N, H, W, C = x.shape
    y = np.empty((N, C))
    lib().gap_fwd(_d(x), _d(y), N, H * W, C)
    return y


def gap_bwd(dy, in_shape):
    N, H, W, C = in_shape
    dx = np.empty(in_shape)
    lib().gap_bwd(_d(dy), _d(dx), N, H * W, C)
    return dx


def shortcut_pad_fwd(x, Cout):
    N, H, W, Cin = x.shape
    y = np.empty((N, (H + 1) // 2, (W + 1) // 2, Cout))
    lib().shortcut_pad_fwd(_d(x), _d(y), N, H, W, Cin, Cout)
    return y


def shortcut_pad_bwd_acc(dy, dx):
    N, H, W, Cin = dx.shape
    lib().shortcut_pad_bwd_acc(_d(dy), _d(dx), N, H, W, Cin, dy.shape[-1])


def softmax_xent(z, labels):
    m, C = z.shape
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    dz = np.empty_like(z)
    loss = lib().softmax_xent(_d(z), labels.ctypes.data_as(_I32), _d(dz), m, C)
    return float(loss), dz


# ----------------------------------------------------------------- networks
class _Net:
    """Common part: flat-vector slicing, decision bookkeeping."""

    ambig_tol = 1e-4

    def segments(self):
        """[(name, shape)] in flat-vector order."""
        raise NotImplementedError

    def n_params(self):
        return sum(int(np.prod(s)) for _, s in self.segments())

    def unpack(self, w):
        w = _f64(w)
        assert w.size == self.n_params(), (w.size, self.n_params())
        out, off = {}, 0
        for name, shape in self.segments():
            n = int(np.prod(shape))
            out[name] = np.ascontiguousarray(w[off:off + n].reshape(shape))
            off += n
        return out

    def pack(self, grads):
        return np.concatenate([_f64(grads[name]).reshape(-1) for name, _ in self.segments()])

    def loss_and_grad(self, w, x, y, tie_break=None):
        """-> (loss, flat gradient, trace).  trace[("relu", i)] = dict(z=, active=),
        trace[("pool", i)] = dict(x=, arg=, gap=), trace["logits"]."""
        raise NotImplementedError


class MLP(_Net):
    """3072 - hidden - classes, ReLU between (two fully connected layers)."""

    def __init__(self, n_in=3072, hidden=256, n_classes=10):
        self.n_in, self.hidden, self.n_classes = n_in, hidden, n_classes

    def segments(self):
        return [("fc1.w", (self.n_in, self.hidden)), ("fc1.b", (self.hidden,)),
                ("fc2.w", (self.hidden, self.n_classes)), ("fc2.b", (self.n_classes,))]

    def loss_and_grad(self, w, x, y, tie_break=None):
        tb = tie_break or {}
        P = self.unpack(w)
        x0 = _f64(x).reshape(len(y), -1)
        z1 = fc_fwd(x0, P["fc1.w"], P["fc1.b"])
        a1, act1 = relu_fwd(z1, tb.get(("relu", 0)), self.ambig_tol)
        z2 = fc_fwd(a1, P["fc2.w"], P["fc2.b"])
        loss, dz2 = softmax_xent(z2, y)
        G = {}
        da1, G["fc2.w"], G["fc2.b"] = fc_bwd(a1, P["fc2.w"], dz2)
        dz1 = relu_bwd(da1, act1)
        _, G["fc1.w"], G["fc1.b"] = fc_bwd(x0, P["fc1.w"], dz1, need_dx=False)
        trace = {("relu", 0): dict(z=z1, active=act1), "logits": z2}
        return loss, self.pack(G), trace


class AlexNetDS(_Net):
    """conv5x5x64 - maxpool3s2 - conv5x5x64 - maxpool3s2 - FC384 - FC192 - FC classes.
    Convolutions: stride 1, zero padding 2, bias, ReLU.  Pools: no padding, floor."""

    def __init__(self, n_classes=10):
        self.n_classes = n_classes

    def segments(self):
        return [("conv1.w", (5, 5, 3, 64)), ("conv1.b", (64,)),
                ("conv2.w", (5, 5, 64, 64)), ("conv2.b", (64,)),
                ("fc1.w", (7 * 7 * 64, 384)), ("fc1.b", (384,)),
                ("fc2.w", (384, 192)), ("fc2.b", (192,)),
                ("fc3.w", (192, self.n_classes)), ("fc3.b", (self.n_classes,))]

    def loss_and_grad(self, w, x, y, tie_break=None):
        tb = tie_break or {}
        tol = self.ambig_tol
        P = self.unpack(w)
        x0 = _f64(x)
        m = x0.shape[0]
        z1 = conv2d_fwd(x0, P["conv1.w"], P["conv1.b"], 1, 2)
        a1, act1 = relu_fwd(z1, tb.get(("relu", 0)), tol)
        p1, arg1, gap1 = maxpool_fwd(a1, 3, 2, tb.get(("pool", 0)), tol)
        z2 = conv2d_fwd(p1, P["conv2.w"], P["conv2.b"], 1, 2)
        a2, act2 = relu_fwd(z2, tb.get(("relu", 1)), tol)
        p2, arg2, gap2 = maxpool_fwd(a2, 3, 2, tb.get(("pool", 1)), tol)
        f0 = p2.reshape(m, -1)
        z3 = fc_fwd(f0, P["fc1.w"], P["fc1.b"])
        a3, act3 = relu_fwd(z3, tb.get(("relu", 2)), tol)
        z4 = fc_fwd(a3, P["fc2.w"], P["fc2.b"])
        a4, act4 = relu_fwd(z4, tb.get(("relu", 3)), tol)
        z5 = fc_fwd(a4, P["fc3.w"], P["fc3.b"])
        loss, dz5 = softmax_xent(z5, y)
        G = {}
        da4, G["fc3.w"], G["fc3.b"] = fc_bwd(a4, P["fc3.w"], dz5)
        da3, G["fc2.w"], G["fc2.b"] = fc_bwd(a3, P["fc2.w"], relu_bwd(da4, act4))
        df0, G["fc1.w"], G["fc1.b"] = fc_bwd(f0, P["fc1.w"], relu_bwd(da3, act3))
        da2 = maxpool_bwd(df0.reshape(p2.shape), arg2, a2.shape, 3, 2)
        dp1, G["conv2.w"], G["conv2.b"] = conv2d_bwd(p1, P["conv2.w"], relu_bwd(da2, act2), 1, 2, True)
        da1 = maxpool_bwd(dp1, arg1, a1.shape, 3, 2)
        _, G["conv1.w"], G["conv1.b"] = conv2d_bwd(x0, P["conv1.w"], relu_bwd(da1, act1), 1, 2, True,
                                                   need_dx=False)
        trace = {("relu", 0): dict(z=z1, active=act1), ("relu", 1): dict(z=z2, active=act2),
                 ("relu", 2): dict(z=z3, active=act3), ("relu", 3): dict(z=z4, active=act4),
                 ("pool", 0): dict(x=a1, arg=arg1, gap=gap1), ("pool", 1): dict(x=a2, arg=arg2, gap=gap2),
                 "logits": z5}
        return loss, self.pack(G), trace


class AlexNet3C(_Net):
    """The paper's reduced AlexNet (Sec. V-A3: three convolutional and two fully connected layers; the paper
    gives no widths, these are this repository's reading, on the pattern of the two-convolution network above):
    conv5x5x64 - maxpool3s2 - conv5x5x64 - maxpool3s2 - conv3x3x64 - FC384 - FC classes.
    Convolutions: stride 1, zero padding 2 (5x5) / 1 (3x3), bias, ReLU.  Pools: no padding, floor."""

    def __init__(self, n_classes=10):
        self.n_classes = n_classes

    def segments(self):
        return [("conv1.w", (5, 5, 3, 64)), ("conv1.b", (64,)),
                ("conv2.w", (5, 5, 64, 64)), ("conv2.b", (64,)),
                ("conv3.w", (3, 3, 64, 64)), ("conv3.b", (64,)),
                ("fc1.w", (7 * 7 * 64, 384)), ("fc1.b", (384,)),
                ("fc2.w", (384, self.n_classes)), ("fc2.b", (self.n_classes,))]

    def loss_and_grad(self, w, x, y, tie_break=None):
        tb = tie_break or {}
        tol = self.ambig_tol
        P = self.unpack(w)
        x0 = _f64(x)
        m = x0.shape[0]
        z1 = conv2d_fwd(x0, P["conv1.w"], P["conv1.b"], 1, 2)
        a1, act1 = relu_fwd(z1, tb.get(("relu", 0)), tol)
        p1, arg1, gap1 = maxpool_fwd(a1, 3, 2, tb.get(("pool", 0)), tol)
        z2 = conv2d_fwd(p1, P["conv2.w"], P["conv2.b"], 1, 2)
        a2, act2 = relu_fwd(z2, tb.get(("relu", 1)), tol)
        p2, arg2, gap2 = maxpool_fwd(a2, 3, 2, tb.get(("pool", 1)), tol)
        z3 = conv2d_fwd(p2, P["conv3.w"], P["conv3.b"], 1, 1)
        a3, act3 = relu_fwd(z3, tb.get(("relu", 2)), tol)
        f0 = a3.reshape(m, -1)
        z4 = fc_fwd(f0, P["fc1.w"], P["fc1.b"])
        a4, act4 = relu_fwd(z4, tb.get(("relu", 3)), tol)
        z5 = fc_fwd(a4, P["fc2.w"], P["fc2.b"])
        loss, dz5 = softmax_xent(z5, y)
        G = {}
        da4, G["fc2.w"], G["fc2.b"] = fc_bwd(a4, P["fc2.w"], dz5)
        df0, G["fc1.w"], G["fc1.b"] = fc_bwd(f0, P["fc1.w"], relu_bwd(da4, act4))
        dp2, G["conv3.w"], G["conv3.b"] = conv2d_bwd(p2, P["conv3.w"], relu_bwd(df0.reshape(a3.shape), act3), 1, 1, True)
        da2 = maxpool_bwd(dp2, arg2, a2.shape, 3, 2)
        dp1, G["conv2.w"], G["conv2.b"] = conv2d_bwd(p1, P["conv2.w"], relu_bwd(da2, act2), 1, 2, True)
        da1 = maxpool_bwd(dp1, arg1, a1.shape, 3, 2)
        _, G["conv1.w"], G["conv1.b"] = conv2d_bwd(x0, P["conv1.w"], relu_bwd(da1, act1), 1, 2, True,
                                                   need_dx=False)
        trace = {("relu", 0): dict(z=z1, active=act1), ("relu", 1): dict(z=z2, active=act2),
                 ("relu", 2): dict(z=z3, active=act3), ("relu", 3): dict(z=z4, active=act4),
                 ("pool", 0): dict(x=a1, arg=arg1, gap=gap1), ("pool", 1): dict(x=a2, arg=arg2, gap=gap2),
                 "logits": z5}
        return loss, self.pack(G), trace


class ResNetCifar(_Net):
    """6n+2-layer CIFAR ResNet (n = 18 gives ResNet-110): conv3x3(3->16)-BN-ReLU,
    three stages of n basic blocks with 16/32/64 channels (conv-BN-ReLU-conv-BN,
    + shortcut, ReLU); the first block of stages 2 and 3 has stride 2 and the
    parameter-free shortcut (subsample, zero channels appended); global average
    pool; FC.  Convolutions carry no bias.  BN uses batch statistics."""

    def __init__(self, n=18, n_classes=100):
        self.n, self.n_classes = n, n_classes
        self.blocks = []          # (name, cin, cout, stride)
        cin = 16
        for si, cout in enumerate((16, 32, 64)):
            for bi in range(n):
                stride = 2 if (si > 0 and bi == 0) else 1
                self.blocks.append(("s%d.b%d" % (si + 1, bi), cin, cout, stride))
                cin = cout

    def segments(self):
        seg = [("stem.conv.w", (3, 3, 3, 16)), ("stem.bn.g", (16,)), ("stem.bn.b", (16,))]
        for name, cin, cout, _ in self.blocks:
            seg += [(name + ".conv1.w", (3, 3, cin, cout)), (name + ".bn1.g", (cout,)), (name + ".bn1.b", (cout,)),
                    (name + ".conv2.w", (3, 3, cout, cout)), (name + ".bn2.g", (cout,)), (name + ".bn2.b", (cout,))]
        seg += [("fc.w", (64, self.n_classes)), ("fc.b", (self.n_classes,))]
        return seg

    def loss_and_grad(self, w, x, y, tie_break=None):
        tb = tie_break or {}
        tol = self.ambig_tol
        P = self.unpack(w)
        x0 = _f64(x)
        trace, G = {}, {}
        ri = 0
        # ---- forward
        c0 = conv2d_fwd(x0, P["stem.conv.w"], None, 1, 1)
        z0, mu0, is0 = bn_fwd(c0, P["stem.bn.g"], P["stem.bn.b"])
        a, act0 = relu_fwd(z0, tb.get(("relu", ri)), tol)
        trace[("relu", ri)] = dict(z=z0, active=act0)
        ri += 1
        saved = []
        for name, cin, cout, stride in self.blocks:
            xin = a
            c1 = conv2d_fwd(xin, P[name + ".conv1.w"], None, stride, 1)
            z1, mu1, is1 = bn_fwd(c1, P[name + ".bn1.g"], P[name + ".bn1.b"])
            a1, act1 = relu_fwd(z1, tb.get(("relu", ri)), tol)
            trace[("relu", ri)] = dict(z=z1, active=act1)
            c2 = conv2d_fwd(a1, P[name + ".conv2.w"], None, 1, 1)
            b2, mu2, is2 = bn_fwd(c2, P[name + ".bn2.g"], P[name + ".bn2.b"])
            sc = xin if (stride == 1 and cin == cout) else shortcut_pad_fwd(xin, cout)
            z2 = b2 + sc
            a, act2 = relu_fwd(z2, tb.get(("relu", ri + 1)), tol)
            trace[("relu", ri + 1)] = dict(z=z2, active=act2)
            ri += 2
            saved.append((xin, c1, mu1, is1, act1, a1, c2, mu2, is2, act2))
        feat = a
        pooled = gap_fwd(feat)
        logits = fc_fwd(pooled, P["fc.w"], P["fc.b"])
        loss, dlogits = softmax_xent(logits, y)
        trace["logits"] = logits
        # ---- backward
        dpooled, G["fc.w"], G["fc.b"] = fc_bwd(pooled, P["fc.w"], dlogits)
        da = gap_bwd(dpooled, feat.shape)
        for (name, cin, cout, stride), sv in zip(reversed(self.blocks), reversed(saved)):
            xin, c1, mu1, is1, act1, a1, c2, mu2, is2, act2 = sv
            dz2 = relu_bwd(da, act2)
            dc2, G[name + ".bn2.g"], G[name + ".bn2.b"] = bn_bwd(c2, P[name + ".bn2.g"], mu2, is2, dz2)
            da1, G[name + ".conv2.w"], _ = conv2d_bwd(a1, P[name + ".conv2.w"], dc2, 1, 1, False)
            dz1 = relu_bwd(da1, act1)
            dc1, G[name + ".bn1.g"], G[name + ".bn1.b"] = bn_bwd(c1, P[name + ".bn1.g"], mu1, is1, dz1)
            dxin, G[name + ".conv1.w"], _ = conv2d_bwd(xin, P[name + ".conv1.w"], dc1, stride, 1, False)
            if stride == 1 and cin == cout:
                dxin += dz2
            else:
                shortcut_pad_bwd_acc(dz2, dxin)
            da = dxin
        dz0 = relu_bwd(da, act0)
        dc0, G["stem.bn.g"], G["stem.bn.b"] = bn_bwd(c0, P["stem.bn.g"], mu0, is0, dz0)
        _, G["stem.conv.w"], _ = conv2d_bwd(x0, P["stem.conv.w"], dc0, 1, 1, False, need_dx=False)
        return loss, self.pack(G), trace


def make_net(model, n_classes):
    """model: 'mlp' | 'alexnet_ds' | 'alexnet_3c' | 'resnet110' | 'resnet<6n+2>'."""
    if model == "mlp":
        return MLP(n_classes=n_classes)
    if model == "alexnet_ds":
        return AlexNetDS(n_classes=n_classes)
    if model == "alexnet_3c":
        return AlexNet3C(n_classes=n_classes)
    if model.startswith("resnet"):
        depth = int(model[len("resnet"):])
        assert (depth - 2) % 6 == 0
        return ResNetCifar(n=(depth - 2) // 6, n_classes=n_classes)
    raise ValueError(model)
