"""CPU oracle for the mini-batch loss and its gradient (TEST INFRASTRUCTURE ONLY).

``grad f(y^a)`` in update (8a) of the paper is the gradient of the average
cross-entropy of a network over a mini-batch (Section 1.1).  This module writes
the four networks of the workloads as plain numpy, one definition per layer,
forward and hand-derived backward, float64 by default.  Nothing here is used by
the product path; it shares no code with the HIP kernels.

Conventions (they define the function the device must reproduce):

* activations are channels-last ``[B, H, W, C]``; a convolution weight is
  ``[Cout, kh, kw, Cin]``; a fully connected weight is ``[out, in]`` with the
  input flattened in (h, w, c) order;
* one replica's parameters are a flat vector, segments in execution order,
  weight before bias (see :func:`layout`);
* loss = mean over the batch of softmax cross-entropy; ReLU'(0) = 0; 2x2
  max-pooling with stride 2 routes the gradient to the first maximum in
  row-major window order;
* batch normalisation (training): per-channel statistics over (B, H, W) of
  the replica's own batch, biased variance inside the normalisation, eps 1e-5;
  running statistics updated with momentum 0.1 and the unbiased variance;
  evaluation uses the running statistics.

* dropout (Section 4: 0.25 for LeNet, 0.3 / 0.4 for the wide residual networks, 0.5 for All-CNN) is
  off unless a ``drop`` description is passed: a unit is kept when a counter-based hash of
  (seed, inner step, replica, dropout site, element index) is at least p * 2^24 in its top 24
  bits, kept units are scaled by 1 / (1 - p); evaluation applies no dropout.  The paper names the
  rates only; the sites are a reading: LeNet after each pooling and after fc's ReLU, All-CNN after
  its two stride-2 convolutions, wide residual blocks between their two convolutions.  The hash is
  two rounds of a 32-bit multiply-xorshift finaliser (the device implements the same definition;
  the two sides share no code).
* ``lenet`` with ``bn=1`` (Section 4.2 lists batch-norm for LeNet): batch-norm follows both
  convolutions and fc1, before the ReLU.

Architectures (sizes are parameters so tests can shrink them):
``mlp``      in-hidden-classes, ReLU.
``lenet``    conv k x k (valid) - ReLU - pool - conv k x k - ReLU - pool - fc - ReLU - fc.
``allcnn``   All-CNN-C: 3x3 convs ca/ca/ca(stride 2)/cb/cb/cb(stride 2)/cb, 1x1 convs cb/classes,
             pad 1 on every 3x3, ReLU after all but the last, global average pool.
``wrn``      WRN-(6 nb + 4)-k with pre-activation basic blocks: conv 3->16, three
             groups of nb blocks at widths 16k/32k/64k (strides 1/2/2), BN-ReLU,
             global average pool, fc.  A block is BN-ReLU-conv3x3-BN-ReLU-conv3x3
             plus identity, or plus a strided 1x1 conv of the pre-activated input
             when the shape changes.
"""
from __future__ import annotations

import numpy as np

BN_EPS = 1e-5
BN_MOMENTUM = 0.1


# ----------------------------------------------------------------------------
# architecture descriptions
# ----------------------------------------------------------------------------
def arch(model: str, **kw):
    """Full-size architectures of the workloads, with keyword overrides for small tests."""
    if model == "mlp":
        a = dict(model="mlp", H=28, W=28, C=1, hidden=128, classes=10)
    elif model == "lenet":
        a = dict(model="lenet", H=28, W=28, C=1, c1=20, c2=50, k=5, fc=500, classes=10, bn=0)
    elif model == "allcnn":
        a = dict(model="allcnn", H=32, W=32, C=3, ca=96, cb=192, classes=10)
    elif model == "wrn":
        a = dict(model="wrn", H=32, W=32, C=3, base=16, widen=4, nb=2, classes=10)
    else:
        raise ValueError(model)
    a.update(kw)
    return a


def _seg(name, shape, kind, fan_in):
    return dict(name=name, shape=tuple(int(s) for s in shape), kind=kind, fan_in=int(fan_in))


def _conv_segs(name, cout, k, cin, bias=True):
    segs = [_seg(name + ".w", (cout, k, k, cin), "weight", k * k * cin)]
    if bias:
        segs.append(_seg(name + ".b", (cout,), "bias", k * k * cin))
    return segs


def _bn_segs(name, c):
    return [_seg(name + ".g", (c,), "bn_gamma", c), _seg(name + ".b", (c,), "bn_beta", c)]


def wrn_blocks(a):
    """(name, cin, cout, stride) for every basic block, in order."""
    widths = [a["base"] * a["widen"], 2 * a["base"] * a["widen"], 4 * a["base"] * a["widen"]]
    blocks, cin = [], a["base"]
    for gi, wd in enumerate(widths):
        for bi in range(a["nb"]):
            stride = (1 if gi == 0 else 2) if bi == 0 else 1
            blocks.append((f"g{gi + 1}b{bi + 1}", cin, wd, stride))
            cin = wd
    return blocks


def layout(a):
    """Ordered parameter segments of one replica (name, shape, kind, fan_in)."""
    m = a["model"]
    segs = []
    if m == "mlp":
        d = a["H"] * a["W"] * a["C"]
        segs += [_seg("fc1.w", (a["hidden"], d), "weight", d), _seg("fc1.b", (a["hidden"],), "bias", d)]
        segs += [_seg("fc2.w", (a["classes"], a["hidden"]), "weight", a["hidden"]),
                 _seg("fc2.b", (a["classes"],), "bias", a["hidden"])]
    elif m == "lenet":
        k = a["k"]
        h1, w1 = (a["H"] - k + 1) // 2, (a["W"] - k + 1) // 2
        h2, w2 = (h1 - k + 1) // 2, (w1 - k + 1) // 2
        d = h2 * w2 * a["c2"]
        bn = a.get("bn", 0)
        segs += _conv_segs("conv1", a["c1"], k, a["C"])
        if bn:
            segs += _bn_segs("bn1", a["c1"])
        segs += _conv_segs("conv2", a["c2"], k, a["c1"])
        if bn:
            segs += _bn_segs("bn2", a["c2"])
        segs += [_seg("fc1.w", (a["fc"], d), "weight", d), _seg("fc1.b", (a["fc"],), "bias", d)]
        if bn:
            segs += _bn_segs("bn3", a["fc"])
        segs += [_seg("fc2.w", (a["classes"], a["fc"]), "weight", a["fc"]),
                 _seg("fc2.b", (a["classes"],), "bias", a["fc"])]
    elif m == "allcnn":
        ca, cb = a["ca"], a["cb"]
        chans = [(a["C"], ca, 3), (ca, ca, 3), (ca, ca, 3), (ca, cb, 3), (cb, cb, 3), (cb, cb, 3),
                 (cb, cb, 3), (cb, cb, 1), (cb, a["classes"], 1)]
        for i, (ci, co, k) in enumerate(chans):
            segs += _conv_segs(f"conv{i + 1}", co, k, ci)
    elif m == "wrn":
        segs += _conv_segs("conv1", a["base"], 3, a["C"], bias=False)
        for name, cin, cout, stride in wrn_blocks(a):
            segs += _bn_segs(name + ".bn1", cin)
            segs += _conv_segs(name + ".conv1", cout, 3, cin, bias=False)
            segs += _bn_segs(name + ".bn2", cout)
            segs += _conv_segs(name + ".conv2", cout, 3, cout, bias=False)
            if cin != cout or stride != 1:
                segs += _conv_segs(name + ".sc", cout, 1, cin, bias=False)
        cl = 4 * a["base"] * a["widen"]
        segs += _bn_segs("bn_out", cl)
        segs += [_seg("fc.w", (a["classes"], cl), "weight", cl), _seg("fc.b", (a["classes"],), "bias", cl)]
    else:
        raise ValueError(m)
    return segs


def n_params(a) -> int:
    return int(sum(np.prod(s["shape"]) for s in layout(a)))


def bn_layers(a):
    """(name, channels) of every batch-norm layer in execution order (running-stat buffers follow it)."""
    return [(s["name"][:-2], s["shape"][0]) for s in layout(a) if s["kind"] == "bn_gamma"]


def new_bn_state(a, dtype=np.float64):
    """Running statistics of one replica: mean 0, variance 1."""
    return {name: [np.zeros(c, dtype), np.ones(c, dtype)] for name, c in bn_layers(a)}


def unpack(a, flat):
    """Views of a flat parameter vector, keyed by segment name."""
    out, off = {}, 0
    for s in layout(a):
        size = int(np.prod(s["shape"]))
        out[s["name"]] = flat[off:off + size].reshape(s["shape"])
        off += size
    assert off == flat.shape[0], (off, flat.shape)
    return out


# ----------------------------------------------------------------------------
# a minimal reverse-mode tape: each primitive records how to push its output
# gradient back to its inputs
# ----------------------------------------------------------------------------
class Var:
    __slots__ = ("v", "g")

    def __init__(self, v):
        self.v = v
        self.g = None

    def acc(self, g):
        self.g = g if self.g is None else self.g + g


class Tape:
    def __init__(self):
        self.back = []
        self.relu_margin = np.inf  # smallest non-zero |input| any ReLU saw (diagnostic, see relu())
        self.pool_margin = np.inf  # smallest lead of a positive window maximum over the runner-up (see maxpool2())
        self.decisions = []        # (kind, margin, largest |input|) of every ReLU / max-pool, in forward order

    def backward(self):
        for fn in reversed(self.back):
            fn()


def conv2d(t, x, w, b, stride, pad):
    """out[b,ho,wo,co] = sum_{i,j,ci} xpad[b, ho*s+i, wo*s+j, ci] * w[co,i,j,ci] (+ b[co])."""
    B, H, W, Cin = x.v.shape
    Cout, kh, kw, _ = w.v.shape
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    xp = np.zeros((B, H + 2 * pad, W + 2 * pad, Cin), x.v.dtype)
    xp[:, pad:pad + H, pad:pad + W, :] = x.v
    out = np.zeros((B, Ho, Wo, Cout), x.v.dtype)

    def window(arr, i, j):
        return arr[:, i:i + stride * (Ho - 1) + 1:stride, j:j + stride * (Wo - 1) + 1:stride, :]

    for i in range(kh):
        for j in range(kw):
            out += np.tensordot(window(xp, i, j), w.v[:, i, j, :], axes=([3], [1]))
    if b is not None:
        out += b.v
    o = Var(out)

    def back():
        dout = o.g
        dw = np.zeros_like(w.v)
        dxp = np.zeros_like(xp)
        for i in range(kh):
            for j in range(kw):
                dw[:, i, j, :] = np.tensordot(dout, window(xp, i, j), axes=([0, 1, 2], [0, 1, 2]))
                window(dxp, i, j)[...] += np.tensordot(dout, w.v[:, i, j, :], axes=([3], [0]))
        w.acc(dw)
        if b is not None:
            b.acc(dout.sum(axis=(0, 1, 2)))
        x.acc(dxp[:, pad:pad + H, pad:pad + W, :])

    t.back.append(back)
    return o


def linear(t, x, w, b):
    """out = x_flat @ w^T + b, input flattened in (h, w, c) order."""
    xf = x.v.reshape(x.v.shape[0], -1)
    o = Var(xf @ w.v.T + b.v)

    def back():
        w.acc(o.g.T @ xf)
        b.acc(o.g.sum(axis=0))
        x.acc((o.g @ w.v).reshape(x.v.shape))

    t.back.append(back)
    return o


def relu(t, x):
    """max(x, 0).  The gradient jumps where an input crosses zero, so two correct implementations in
    different precisions may disagree there; the tape records how close the inputs came to that."""
    o = Var(np.maximum(x.v, 0))
    nz = np.abs(x.v[x.v != 0])
    if nz.size:
        t.relu_margin = min(t.relu_margin, float(nz.min()))
    t.decisions.append(("relu", float(nz.min()) if nz.size else np.inf, float(nz.max()) if nz.size else 0.0))
    t.back.append(lambda: x.acc(o.g * (x.v > 0)))
    return o


def maxpool2(t, x):
    """2x2 window, stride 2, floor; gradient to the first maximum in row-major window order."""
    B, H, W, C = x.v.shape
    Ho, Wo = H // 2, W // 2
    win = np.stack([x.v[:, i:2 * Ho:2, j:2 * Wo:2, :] for i in (0, 1) for j in (0, 1)], axis=0)
    idx = np.argmax(win, axis=0)          # first maximum on ties
    o = Var(np.take_along_axis(win, idx[None], axis=0)[0])
    # diagnostic, outside the arithmetic: how close any window came to routing its gradient elsewhere.  Windows
    # whose maximum is not positive do not count: behind a ReLU they are ties at zero that carry no gradient.
    top2 = np.sort(win, axis=0)[-2:]
    lead = (top2[1] - top2[0])[top2[1] > 0]
    if lead.size:
        t.pool_margin = min(t.pool_margin, float(lead.min()))
    t.decisions.append(("maxpool", float(lead.min()) if lead.size else np.inf, float(np.abs(win).max())))

    def back():
        dx = np.zeros_like(x.v)
        for q, (i, j) in enumerate([(0, 0), (0, 1), (1, 0), (1, 1)]):
            dx[:, i:2 * Ho:2, j:2 * Wo:2, :] += o.g * (idx == q)
        x.acc(dx)

    t.back.append(back)
    return o


def gap(t, x):
    """Global average pool over (H, W)."""
    B, H, W, C = x.v.shape
    o = Var(x.v.mean(axis=(1, 2)))
    t.back.append(lambda: x.acc(np.broadcast_to(o.g[:, None, None, :] / (H * W), x.v.shape).copy()))
    return o


def batchnorm(t, x, gam, bet, stats, train):
    """Per-channel normalisation over (B, H, W); ``stats`` = [running_mean, running_var]."""
    C = x.v.shape[-1]
    xf = x.v.reshape(-1, C)
    M = xf.shape[0]
    if train:
        mean = xf.mean(axis=0)
        var = ((xf - mean) ** 2).mean(axis=0)
        stats[0] = (1 - BN_MOMENTUM) * stats[0] + BN_MOMENTUM * mean
        stats[1] = (1 - BN_MOMENTUM) * stats[1] + BN_MOMENTUM * var * (M / max(M - 1, 1))
    else:
        mean, var = stats[0], stats[1]
    rstd = 1.0 / np.sqrt(var + BN_EPS)
    xhat = (xf - mean) * rstd
    o = Var((xhat * gam.v + bet.v).reshape(x.v.shape))

    def back():
        dy = o.g.reshape(-1, C)
        gam.acc((dy * xhat).sum(axis=0))
        bet.acc(dy.sum(axis=0))
        dxhat = dy * gam.v
        if train:
            dx = rstd * (dxhat - dxhat.mean(axis=0) - xhat * (dxhat * xhat).mean(axis=0))
        else:
            dx = rstd * dxhat
        x.acc(dx.reshape(x.v.shape))

    t.back.append(back)
    return o


def mix32(x):
    """32-bit multiply-xorshift finaliser on uint32 arrays (wraps modulo 2^32)."""
    x = np.asarray(x, dtype=np.uint32).copy()
    x ^= x >> np.uint32(16)
    x *= np.uint32(0x7FEB352D)
    x ^= x >> np.uint32(15)
    x *= np.uint32(0x846CA68B)
    x ^= x >> np.uint32(16)
    return x


def dropout_keep(seed, step, replica, site, count, p):
    """Boolean keep-mask of ``count`` elements for dropout probability ``p`` (taken in float32)."""
    m32 = (1 << 32) - 1
    key = mix32(np.uint32((int(seed) + 0x9E3779B9 * int(step)) & m32))
    key = mix32(key ^ np.uint32((int(replica) * 0x85EBCA6B + int(site) * 0xC2B2AE35 + 1) & m32))
    idx = np.arange(count, dtype=np.uint32)
    h = mix32(mix32(idx ^ key) + key)
    thresh = int(np.floor(float(np.float32(p)) * (1 << 24)))
    return (h >> np.uint32(8)) >= np.uint32(thresh)


def dropout(t, x, keep, p):
    """Inverted dropout with a given keep-mask (flat, in the element order of ``x``)."""
    scale = 1.0 / (1.0 - float(np.float32(p)))
    m = keep.reshape(x.v.shape).astype(x.v.dtype) * x.v.dtype.type(scale)
    o = Var(x.v * m)
    t.back.append(lambda: x.acc(o.g * m))
    return o


def add(t, p, q):
    o = Var(p.v + q.v)

    def back():
        p.acc(o.g)
        q.acc(o.g)

    t.back.append(back)
    return o


def round_bf16(a):
    """Nearest value with an 8-bit significand (the bfloat16 grid), ties to the even significand; the exponent
    range is taken as unbounded (nothing in these networks comes near bfloat16's limits)."""
    a = np.asarray(a, dtype=np.float64)
    m, e = np.frexp(a)                       # a = m * 2^e, 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0) / 256.0, e)


class StoredVar(Var):
    """A tensor kept in a reduced-precision format, and with it its gradient: every contribution that arrives
    is added to what is stored so far and the sum is rounded again (a backward pass that keeps gradients in the
    format adds to them in place, in the reverse of the order in which the tensor was read going forward)."""
    __slots__ = ("q",)

    def __init__(self, v, q):
        super().__init__(v)
        self.q = q

    def acc(self, g):
        tot = g if self.g is None else self.g + g
        self.g = self.q(tot).astype(self.v.dtype)


def store(t, x, q):
    """A tensor as it is kept between layers when the workload computes in reduced precision: the values
    rounded by ``q`` on the way forward, and the gradient that arrives for them rounded on the way back
    (gradients of activations are kept in the same format).  ``q = None``: exact storage, nothing happens."""
    if q is None:
        return x
    o = StoredVar(q(x.v).astype(x.v.dtype), q)
    t.back.append(lambda: x.acc(o.g))
    return o


def softmax_xent(t, logits, labels, q=None):
    """Mean over the batch of -log softmax(logits)[label]; also returns the predicted classes.
    ``q`` rounds the gradient handed to the logits (see :func:`store`)."""
    z = logits.v - logits.v.max(axis=1, keepdims=True)
    logp = z - np.log(np.exp(z).sum(axis=1, keepdims=True))
    B = z.shape[0]
    loss = -logp[np.arange(B), labels].mean()
    pred = np.argmax(logits.v, axis=1)

    def back():
        d = np.exp(logp)
        d[np.arange(B), labels] -= 1.0
        logits.acc(d / B if q is None else q(d / B).astype(d.dtype))

    t.back.append(back)
    return loss, pred


# ----------------------------------------------------------------------------
# networks
# ----------------------------------------------------------------------------
def forward(a, P, x, t, train=True, bn_state=None, drop=None, q=None):
    """Logits of architecture ``a`` with parameter Vars ``P`` on images ``x`` (a Var).

    ``drop`` = dict(p, seed, step, replica) switches dropout on (training only).
    ``q`` (see :func:`store`) switches reduced-precision storage on: the images, every layer output that a
    later layer reads, and the weights of the contractions are rounded by it; biases, batch-norm parameters,
    the logits and all sums stay exact.  A layer output is what the layer hands on: a convolution together
    with the bias, the residual and the ReLU behind it; a batch-norm together with its ReLU."""
    m = a["model"]
    site = [0]

    def keep(h):
        return store(t, h, q)

    def W(name):
        """A weight as the contraction reads it: rounded copy of the master value; the gradient of the copy is
        the gradient of the master value, unrounded (weight gradients are sums kept exact)."""
        if q is None:
            return P[name]
        w = P[name]
        o = Var(q(w.v).astype(w.v.dtype))
        t.back.append(lambda: w.acc(o.g))
        return o

    def dropped(h):
        if not train or drop is None or drop["p"] <= 0:
            return h
        mask = dropout_keep(drop["seed"], drop["step"], drop["replica"], site[0], h.v.size, drop["p"])
        site[0] += 1
        return keep(dropout(t, h, mask, drop["p"]))

    x = keep(x)
    if m == "mlp":
        h = keep(relu(t, linear(t, x, W("fc1.w"), P["fc1.b"])))
        return linear(t, h, W("fc2.w"), P["fc2.b"])
    if m == "lenet":
        bn = a.get("bn", 0)

        def act(h, name):
            if bn:
                h = batchnorm(t, keep(h), P[name + ".g"], P[name + ".b"], bn_state[name], train)
            return keep(relu(t, h))

        h = dropped(maxpool2(t, act(conv2d(t, x, W("conv1.w"), P["conv1.b"], 1, 0), "bn1")))
        h = dropped(maxpool2(t, act(conv2d(t, h, W("conv2.w"), P["conv2.b"], 1, 0), "bn2")))
        h = dropped(act(linear(t, h, W("fc1.w"), P["fc1.b"]), "bn3"))   # batch-norm over the batch, per feature
        return linear(t, h, W("fc2.w"), P["fc2.b"])
    if m == "allcnn":
        strides = [1, 1, 2, 1, 1, 2, 1, 1, 1]
        pads = [1, 1, 1, 1, 1, 1, 1, 0, 0]
        h = x
        for i in range(9):
            h = conv2d(t, h, W(f"conv{i + 1}.w"), P[f"conv{i + 1}.b"], strides[i], pads[i])
            if i < 8:
                h = relu(t, h)
            h = keep(h)
            if strides[i] == 2:
                h = dropped(h)
        return gap(t, h)
    if m == "wrn":
        h = keep(conv2d(t, x, W("conv1.w"), None, 1, 1))
        for name, cin, cout, stride in wrn_blocks(a):
            o = keep(relu(t, batchnorm(t, h, P[name + ".bn1.g"], P[name + ".bn1.b"], bn_state[name + ".bn1"], train)))
            u = keep(conv2d(t, o, W(name + ".conv1.w"), None, stride, 1))
            u = keep(relu(t, batchnorm(t, u, P[name + ".bn2.g"], P[name + ".bn2.b"], bn_state[name + ".bn2"], train)))
            u = conv2d(t, dropped(u), W(name + ".conv2.w"), None, 1, 1)
            if cin != cout or stride != 1:
                sc = keep(conv2d(t, o, W(name + ".sc.w"), None, stride, 0))
            else:
                sc = h
            h = keep(add(t, u, sc))
        h = keep(relu(t, batchnorm(t, h, P["bn_out.g"], P["bn_out.b"], bn_state["bn_out"], train)))
        return linear(t, keep(gap(t, h)), W("fc.w"), P["fc.b"])
    raise ValueError(m)


def loss_and_grad(a, flat, images, labels, bn_state=None, dtype=np.float64, drop=None, diag=None, storage=None):
    """Mini-batch loss at the flat parameter vector and its gradient (same packing).

    ``storage="bf16"``: activations, their gradients and the weights inside the contractions are kept on the
    bfloat16 grid (see :func:`forward`), everything else exact -- the workloads that compute in bf16 with fp32
    master weights.  Rounding decides ReLU masks, so a comparison that should be sharper than the rounding
    itself has to take those decisions in the same precision on both sides; the sums stay float64 here.

    In training mode batch-norm running statistics in ``bn_state`` are updated in place.  A dict passed
    as ``diag`` receives ``relu_margin``, the smallest non-zero |input| of any ReLU in the pass, and ``pool_margin``,
    the smallest lead of a positive max-pool winner over the runner-up of its window, and ``decisions``, one
    (kind, margin, largest |input|) per ReLU / max-pool in forward order.
    """
    flat = np.asarray(flat, dtype=dtype)
    t = Tape()
    P = {k: Var(v) for k, v in unpack(a, flat).items()}
    x = Var(np.asarray(images, dtype=dtype))
    q = _storage_rounding(storage)
    logits = forward(a, P, x, t, train=True, bn_state=bn_state, drop=drop, q=q)
    loss, _ = softmax_xent(t, logits, np.asarray(labels), q=q)
    t.backward()
    if diag is not None:
        diag["relu_margin"] = t.relu_margin
        diag["pool_margin"] = t.pool_margin
        diag["decisions"] = list(t.decisions)
    grad = np.concatenate([P[s["name"]].g.reshape(-1) for s in layout(a)])
    return float(loss), grad


def _storage_rounding(storage):
    if storage is None:
        return None
    if storage == "bf16":
        return round_bf16
    raise ValueError(storage)


def evaluate(a, flat, images, labels, bn_state=None, dtype=np.float64, storage=None):
    """Mean loss and number of misclassified samples (batch-norm in evaluation mode)."""
    flat = np.asarray(flat, dtype=dtype)
    t = Tape()
    P = {k: Var(v) for k, v in unpack(a, flat).items()}
    logits = forward(a, P, Var(np.asarray(images, dtype=dtype)), t, train=False, bn_state=bn_state,
                     q=_storage_rounding(storage))
    loss, pred = softmax_xent(t, logits, np.asarray(labels))
    return float(loss), int(np.sum(pred != np.asarray(labels)))


def logits_only(a, flat, images, bn_state=None, train=True, dtype=np.float64, storage=None):
    flat = np.asarray(flat, dtype=dtype)
    P = {k: Var(v) for k, v in unpack(a, flat).items()}
    return forward(a, P, Var(np.asarray(images, dtype=dtype)), Tape(), train=train, bn_state=bn_state,
                   q=_storage_rounding(storage)).v


def flops_forward_per_image(a) -> int:
    """2*M*N*K summed over the contractions of one forward pass, per image (for roofline figures)."""
    m = a["model"]
    total = 0

    def conv(h, w, cin, cout, k, stride, pad):
        ho, wo = (h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1
        return 2 * ho * wo * cout * k * k * cin, ho, wo

    if m == "mlp":
        d = a["H"] * a["W"] * a["C"]
        return 2 * d * a["hidden"] + 2 * a["hidden"] * a["classes"]
    if m == "lenet":
        f, h, w = conv(a["H"], a["W"], a["C"], a["c1"], a["k"], 1, 0)
        total += f
        h, w = h // 2, w // 2
        f, h, w = conv(h, w, a["c1"], a["c2"], a["k"], 1, 0)
        total += f
        h, w = h // 2, w // 2
        return total + 2 * h * w * a["c2"] * a["fc"] + 2 * a["fc"] * a["classes"]
    if m == "allcnn":
        ca, cb = a["ca"], a["cb"]
        spec = [(a["C"], ca, 3, 1, 1), (ca, ca, 3, 1, 1), (ca, ca, 3, 2, 1), (ca, cb, 3, 1, 1), (cb, cb, 3, 1, 1),
                (cb, cb, 3, 2, 1), (cb, cb, 3, 1, 1), (cb, cb, 1, 1, 0), (cb, a["classes"], 1, 1, 0)]
        h, w = a["H"], a["W"]
        for ci, co, k, s, p in spec:
            f, h, w = conv(h, w, ci, co, k, s, p)
            total += f
        return total
    if m == "wrn":
        h, w = a["H"], a["W"]
        f, h, w = conv(h, w, a["C"], a["base"], 3, 1, 1)
        total += f
        for name, cin, cout, stride in wrn_blocks(a):
            if cin != cout or stride != 1:
                total += conv(h, w, cin, cout, 1, stride, 0)[0]
            f, h, w = conv(h, w, cin, cout, 3, stride, 1)
            total += f
            f, h, w = conv(h, w, cout, cout, 3, 1, 1)
            total += f
        return total + 2 * 4 * a["base"] * a["widen"] * a["classes"]
    raise ValueError(m)
