"""Single-kernel parity of the memory-bound layer kernels (batch-norm, pooling, global average pool, dropout,
bias gradient, loss) against the oracle's layer functions, through the C ABI, in both activation formats.

For bf16 the inputs are drawn on the bf16 grid, so both sides see exactly the same numbers; the kernels compute
in fp32 and round once on the store, so outputs must agree with the oracle's float64 result to half a bf16 ulp
(2^-8 relative, plus 2e-5 of the largest entry for values that cancel), fp32 sums to 2e-5 of the largest entry,
and everything that is a selection or a mask (max-pool, dropout, ReLU masks) exactly.
"""
import numpy as np
import pytest

from oracle import nets as onets

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1707_00424_amd import binding as pb
    pb.lib()
    return torch, pb


def grid(a, dtype):
    return onets.round_bf16(a).astype(np.float32) if dtype else np.asarray(a, np.float32)


def up(torch, a, dtype):
    t = torch.as_tensor(np.ascontiguousarray(a, np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if dtype else t.contiguous()


def down(t):
    return t.float().cpu().numpy().astype(np.float64)


def near(name, got, ref, dtype, sums=False):
    scale = max(np.abs(ref).max(), 1e-30)
    rel = 0.0 if (sums or not dtype) else 2.0 ** -8
    bound = rel * np.abs(ref) + 2e-5 * scale
    bad = np.abs(got - ref) > bound
    assert not bad.any(), f"{name}: {bad.sum()} of {bad.size} outside tolerance, worst {np.max(np.abs(got - ref) - bound):.3e}"


def clear_of_the_kink(x, gamma, beta, dtype):
    """Moves the few entries of x whose batch-norm output lies within 1e-4 of zero (relative to the largest)
    away from it, so that no ReLU decision of the layer depends on rounding; checked with the oracle's own
    batch-norm.  x [B, H, W, C] float32 on the grid of the format, returned likewise."""
    x = x.copy()
    for _ in range(20):
        pre = onets.batchnorm(onets.Tape(), onets.Var(x.astype(np.float64)), onets.Var(gamma.astype(np.float64)),
                              onets.Var(beta.astype(np.float64)), [np.zeros(x.shape[-1]), np.ones(x.shape[-1])], True).v
        risky = np.abs(pre) < 1e-4 * np.abs(pre).max()
        if not risky.any():
            return x
        x[risky] = grid(x[risky] + 0.5, dtype)
    raise AssertionError("could not move the inputs away from the kink")


ACT = [
    # n, B, H, W, C
    (2, 3, 5, 7, 3),        # odd everything: scalar paths
    (3, 4, 8, 8, 16),       # 16-byte vector paths
    (2, 9, 6, 4, 40),       # vector path, channel count not a power of two
    (1, 2, 16, 16, 256),    # wide
    (2, 37, 1, 1, 500),     # a fully connected layer's activations (LeNet's fc1 with batch-norm)
]
FULL = [(3, 128, 32, 32, 64), (3, 128, 8, 8, 256)]   # WRN-16-4's first and last batch-norm at the size the bench runs


@pytest.mark.parametrize("shape", ACT + FULL)
@pytest.mark.parametrize("dtype", [0, 1])
def test_batchnorm_relu_forward_backward(gpu, shape, dtype):
    torch, pb = gpu
    n, B, H, W, C = shape
    rng = np.random.default_rng(hash(shape) % (2 ** 31))
    x = grid(rng.standard_normal((n, B, H, W, C)) * 1.5 + rng.standard_normal(C), dtype)
    dout = grid(rng.standard_normal((n, B, H, W, C)), dtype)
    extra = grid(rng.standard_normal((n, B, H, W, C)), dtype)
    gamma = (1 + 0.2 * rng.standard_normal((n, C))).astype(np.float32)
    beta = (0.3 * rng.standard_normal((n, C))).astype(np.float32)
    x = np.stack([clear_of_the_kink(x[r], gamma[r], beta[r], dtype) for r in range(n)])
    run0 = np.stack([rng.standard_normal((n, C)), 0.5 + rng.random((n, C))], axis=1).astype(np.float32)   # [n, 2, C]
    desc = pb.parle_act_desc(dtype, n, B, H, W, C)
    tdt = torch.bfloat16 if dtype else torch.float32
    scratch = torch.zeros(pb.parle_k_layer_scratch_bytes(desc) // 8, dtype=torch.float64, device="cuda")
    dx_, dd, da = up(torch, x, dtype), up(torch, dout, dtype), up(torch, extra, dtype)
    dg, db = up(torch, gamma, 0), up(torch, beta, 0)
    saved = torch.zeros((n, 2, C), dtype=torch.float32, device="cuda")
    running = up(torch, run0, 0)
    out = torch.zeros((n, B, H, W, C), dtype=tdt, device="cuda")
    pb.parle_k_bn_forward(desc, dx_, dg, db, scratch, saved, running, out)
    sums = torch.zeros((n, 2, C), dtype=torch.float32, device="cuda")
    dgam, dbet = torch.zeros((n, C), dtype=torch.float32, device="cuda"), torch.zeros((n, C), dtype=torch.float32, device="cuda")
    g1 = torch.zeros((n, B, H, W, C), dtype=tdt, device="cuda")
    g2 = torch.zeros_like(g1)
    pb.parle_k_bn_backward(desc, dx_, dd, dg, db, saved, None, scratch, sums, dgam, dbet, g1)
    pb.parle_k_bn_backward(desc, dx_, dd, dg, db, saved, da, scratch, sums, dgam, dbet, g2)
    torch.cuda.synchronize()
    for r in range(n):
        t = onets.Tape()
        xv, gv, bv = onets.Var(x[r].astype(np.float64)), onets.Var(gamma[r].astype(np.float64)), onets.Var(beta[r].astype(np.float64))
        stats = [run0[r, 0].astype(np.float64), run0[r, 1].astype(np.float64)]
        pre = onets.batchnorm(t, xv, gv, bv, stats, True)
        o = onets.relu(t, pre)
        o.g = dout[r].astype(np.float64)
        t.backward()
        assert np.abs(pre.v).min() >= 1e-4 * np.abs(pre.v).max()        # no ReLU decision hangs on rounding
        near(f"bn out[{r}]", down(out[r]), o.v, dtype)
        xf = x[r].reshape(-1, C).astype(np.float64)
        near("saved mean", down(saved[r, 0]), xf.mean(axis=0), 0)
        near("saved rstd", down(saved[r, 1]), 1 / np.sqrt(xf.var(axis=0) + 1e-5), 0)
        near("running mean", down(running[r, 0]), stats[0], 0)
        near("running var", down(running[r, 1]), stats[1], 0)
        near(f"bn dx[{r}]", down(g1[r]), xv.g, dtype)
        near(f"bn dx + add[{r}]", down(g2[r]), xv.g + extra[r], dtype)
        near("dgamma", down(dgam[r]), gv.g, 0, sums=True)
        near("dbeta", down(dbet[r]), bv.g, 0, sums=True)


@pytest.mark.parametrize("shape", ACT[:4] + [(2, 3, 9, 7, 8), (3, 128, 24, 24, 20)])
@pytest.mark.parametrize("dtype", [0, 1])
def test_maxpool_forward_backward_exact(gpu, shape, dtype):
    torch, pb = gpu
    n, B, H, W, C = shape
    if H < 2 or W < 2:
        pytest.skip("no window")
    rng = np.random.default_rng(hash(shape) % (2 ** 31))
    # a coarse grid of values makes equal maxima inside a window common: the first one must win
    x = grid(np.round(rng.standard_normal((n, B, H, W, C)) * 2) / 2, dtype)
    dy = grid(rng.standard_normal((n, B, H // 2, W // 2, C)), dtype)
    desc = pb.parle_act_desc(dtype, n, B, H, W, C)
    tdt = torch.bfloat16 if dtype else torch.float32
    dx_, ddy = up(torch, x, dtype), up(torch, dy, dtype)
    out = torch.zeros((n, B, H // 2, W // 2, C), dtype=tdt, device="cuda")
    g_plain = torch.full((n, B, H, W, C), 7.0, dtype=tdt, device="cuda")
    g_mask = torch.full((n, B, H, W, C), 7.0, dtype=tdt, device="cuda")
    pb.parle_k_maxpool_forward(desc, dx_, out)
    pb.parle_k_maxpool_backward(desc, dx_, ddy, 0, g_plain)
    pb.parle_k_maxpool_backward(desc, dx_, ddy, 1, g_mask)
    torch.cuda.synchronize()
    for r in range(n):
        t = onets.Tape()
        xv = onets.Var(x[r].astype(np.float64))
        o = onets.maxpool2(t, xv)
        o.g = dy[r].astype(np.float64)
        t.backward()
        assert np.array_equal(down(out[r]), o.v)
        assert np.array_equal(down(g_plain[r]), xv.g)
        assert np.array_equal(down(g_mask[r]), xv.g * (x[r] > 0))


@pytest.mark.parametrize("shape", ACT + [(3, 128, 8, 8, 10), (3, 128, 8, 8, 256)])
@pytest.mark.parametrize("dtype", [0, 1])
def test_global_average_pool(gpu, shape, dtype):
    torch, pb = gpu
    n, B, H, W, C = shape
    rng = np.random.default_rng(hash(shape) % (2 ** 31))
    x = grid(rng.standard_normal((n, B, H, W, C)) + 0.5, dtype)
    dy = grid(rng.standard_normal((n, B, C)), dtype)
    desc = pb.parle_act_desc(dtype, n, B, H, W, C)
    tdt = torch.bfloat16 if dtype else torch.float32
    dx_, ddy = up(torch, x, dtype), up(torch, dy, dtype)
    o32 = torch.zeros((n, B, C), dtype=torch.float32, device="cuda")
    oact = torch.zeros((n, B, C), dtype=tdt, device="cuda")
    gin = torch.zeros((n, B, H, W, C), dtype=tdt, device="cuda")
    pb.parle_k_gap_forward(desc, 1, dx_, o32)
    pb.parle_k_gap_forward(desc, 0, dx_, oact)
    pb.parle_k_gap_backward(desc, ddy, gin)
    torch.cuda.synchronize()
    for r in range(n):
        t = onets.Tape()
        xv = onets.Var(x[r].astype(np.float64))
        o = onets.gap(t, xv)
        o.g = dy[r].astype(np.float64)
        t.backward()
        near("gap fp32", down(o32[r]), o.v, 0)
        near("gap", down(oact[r]), o.v, dtype)
        near("gap backward", down(gin[r]), xv.g, dtype)


@pytest.mark.parametrize("shape", ACT[:4] + [(3, 128, 16, 16, 96)])
@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("p", [0.25, 0.5])
def test_dropout_masks_and_scale(gpu, shape, dtype, p):
    torch, pb = gpu
    n, B, H, W, C = shape
    rng = np.random.default_rng(hash(shape) % (2 ** 31))
    x = grid(rng.standard_normal((n, B, H, W, C)), dtype)
    src = grid(rng.standard_normal((n, B, H, W, C)), dtype)
    desc = pb.parle_act_desc(dtype, n, B, H, W, C)
    tdt = torch.bfloat16 if dtype else torch.float32
    seed, step, site = 12345, 7, 2
    dstep = torch.tensor([step], dtype=torch.int64, device="cuda")
    dx_, ds = up(torch, x, dtype), up(torch, src, dtype)
    out = torch.zeros((n, B, H, W, C), dtype=tdt, device="cuda")
    out_m = torch.zeros_like(out)
    pb.parle_k_dropout(desc, dx_, None, seed, dstep, site, p, out)
    pb.parle_k_dropout(desc, dx_, ds, seed, dstep, site, p, out_m)
    torch.cuda.synchronize()
    for r in range(n):
        keep = onets.dropout_keep(seed, step, r, site, x[r].size, p)
        t = onets.Tape()
        o = onets.dropout(t, onets.Var(x[r].astype(np.float64)), keep, p)
        got, got_m = down(out[r]), down(out_m[r])
        assert np.array_equal(got != 0, (o.v != 0))                      # the mask, bit for bit
        near("dropout", got, o.v, dtype)
        near("dropout behind a ReLU", got_m, o.v * (src[r] > 0), dtype)


@pytest.mark.parametrize("shape", ACT + [(3, 128, 32, 32, 96), (3, 128, 8, 8, 10)])
@pytest.mark.parametrize("dtype", [0, 1])
def test_bias_gradient(gpu, shape, dtype):
    torch, pb = gpu
    n, B, H, W, C = shape
    rng = np.random.default_rng(hash(shape) % (2 ** 31))
    dy = grid(rng.standard_normal((n, B, H, W, C)) + 0.1, dtype)
    desc = pb.parle_act_desc(dtype, n, B, H, W, C)
    scratch = torch.zeros(pb.parle_k_layer_scratch_bytes(desc) // 8, dtype=torch.float64, device="cuda")
    grad = torch.zeros((n, C), dtype=torch.float32, device="cuda")
    pb.parle_k_bias_grad(desc, up(torch, dy, dtype), scratch, grad)
    torch.cuda.synchronize()
    for r in range(n):
        # the oracle's bias gradient: backward of a 1x1 convolution with a bias
        t = onets.Tape()
        xv, wv, bv = onets.Var(np.zeros((B, H, W, 1))), onets.Var(np.zeros((C, 1, 1, 1))), onets.Var(np.zeros(C))
        o = onets.conv2d(t, xv, wv, bv, 1, 0)
        o.g = dy[r].astype(np.float64)
        t.backward()
        near("bias gradient", down(grad[r]), bv.g, 0, sums=True)


@pytest.mark.parametrize("n,B,C", [(1, 1, 2), (3, 128, 10), (2, 37, 7), (6, 128, 10)])
@pytest.mark.parametrize("dtype", [0, 1])
def test_softmax_cross_entropy(gpu, n, B, C, dtype):
    torch, pb = gpu
    rng = np.random.default_rng(1000 * n + 10 * B + C)
    logits = (rng.standard_normal((n, B, C)) * 3).astype(np.float32)
    labels = rng.integers(0, C, (n, B)).astype(np.int32)
    tdt = torch.bfloat16 if dtype else torch.float32
    loss = torch.zeros(n, dtype=torch.float32, device="cuda")
    dl = torch.zeros((n, B, C), dtype=tdt, device="cuda")
    pb.parle_k_softmax_xent(dtype, up(torch, logits, 0), torch.as_tensor(labels).cuda(), loss, dl)
    torch.cuda.synchronize()
    for r in range(n):
        t = onets.Tape()
        lv = onets.Var(logits[r].astype(np.float64))
        ref, _ = onets.softmax_xent(t, lv, labels[r])
        t.backward()
        assert abs(loss[r].item() - ref) <= 1e-5 * abs(ref) + 1e-6
        near("dlogits", down(dl[r]), lv.g, dtype)


@pytest.mark.parametrize("n,B,D,C,mask", [(1, 1, 3, 2, 0), (3, 128, 128, 10, 1), (6, 128, 500, 10, 1), (3, 128, 256, 10, 0),
                                          (2, 37, 70, 7, 1), (3, 128, 640, 10, 0), (2, 5, 64, 16, 1)])
@pytest.mark.parametrize("dtype", [0, 1])
def test_classifier_head(gpu, n, B, D, C, mask, dtype):
    """Last fully connected layer + loss + its input gradient in one kernel, against the oracle's three steps."""
    torch, pb = gpu
    rng = np.random.default_rng(7 * n + 13 * B + D + C + mask)
    q = (lambda a: up(torch, a, 1).float().cpu().numpy()) if dtype else (lambda a: np.asarray(a, np.float32))
    feat = q(rng.standard_normal((n, B, D)))
    if mask:
        feat = np.maximum(feat, 0)          # the output of a ReLU
    w = q(rng.standard_normal((n, C, D)) / np.sqrt(D) * 2)
    bias = rng.standard_normal((n, C)).astype(np.float32)
    labels = rng.integers(0, C, (n, B)).astype(np.int32)
    tdt = torch.bfloat16 if dtype else torch.float32
    loss_img = torch.zeros((n, B), dtype=torch.float32, device="cuda")
    loss = torch.zeros(n, dtype=torch.float32, device="cuda")
    dl = torch.zeros((n, B, C), dtype=tdt, device="cuda")
    df = torch.full((n, B, D), 7.0, dtype=tdt, device="cuda")
    pb.parle_k_fc_head(dtype, up(torch, feat, dtype), up(torch, w, dtype), torch.as_tensor(bias).cuda(),
                       torch.as_tensor(labels).cuda(), mask, loss_img, loss, dl, df)
    torch.cuda.synchronize()
    for r in range(n):
        t = onets.Tape()
        pre = onets.Var(feat[r].astype(np.float64))
        fv = onets.relu(t, pre) if mask else pre    # feat >= 0 already: relu is the identity forward, the mask backward
        wv, bv = onets.Var(w[r].astype(np.float64)), onets.Var(bias[r].astype(np.float64))
        lv = onets.linear(t, fv, wv, bv)
        ref, _ = onets.softmax_xent(t, lv, labels[r])
        t.backward()
        assert abs(loss[r].item() - ref) <= 1e-5 * abs(ref) + 1e-6
        assert abs(loss_img[r].double().mean().item() - ref) <= 1e-5 * abs(ref) + 1e-6
        near("dlogits", down(dl[r]), lv.g, dtype)
        # the input gradient from the dlogits as stored (the weight gradient reads the same values)
        t2 = onets.Tape()
        pre2 = onets.Var(feat[r].astype(np.float64))
        fv2 = onets.relu(t2, pre2) if mask else pre2
        lv2 = onets.linear(t2, fv2, wv, bv)
        lv2.g = down(dl[r])
        t2.backward()
        near("dfeat", down(df[r]), pre2.g, dtype)


@pytest.mark.parametrize("n,B,H,W,C", [(1, 1, 1, 1, 2), (3, 128, 8, 8, 10), (2, 9, 5, 3, 7), (2, 6, 12, 11, 16)])
@pytest.mark.parametrize("dtype", [0, 1])
def test_pooling_head(gpu, n, B, H, W, C, dtype):
    """Global average pool over class maps + loss + the pool's backward pass in one kernel, against the oracle's steps."""
    torch, pb = gpu
    rng = np.random.default_rng(3 * n + 5 * B + H * W + C)
    q = (lambda a: up(torch, a, 1).float().cpu().numpy()) if dtype else (lambda a: np.asarray(a, np.float32))
    feat = q(rng.standard_normal((n, B, H, W, C)) * 3)
    labels = rng.integers(0, C, (n, B)).astype(np.int32)
    tdt = torch.bfloat16 if dtype else torch.float32
    loss_img = torch.zeros((n, B), dtype=torch.float32, device="cuda")
    loss = torch.zeros(n, dtype=torch.float32, device="cuda")
    dl = torch.zeros((n, B, C), dtype=tdt, device="cuda")
    df = torch.full((n, B, H, W, C), 7.0, dtype=tdt, device="cuda")
    desc = pb.parle_act_desc(dtype, n, B, H, W, C)
    pb.parle_k_gap_head(desc, up(torch, feat, dtype), torch.as_tensor(labels).cuda(), loss_img, loss, dl, df)
    torch.cuda.synchronize()
    for r in range(n):
        t = onets.Tape()
        fv = onets.Var(feat[r].astype(np.float64))
        lv = onets.gap(t, fv)
        ref, _ = onets.softmax_xent(t, lv, labels[r])
        t.backward()
        assert abs(loss[r].item() - ref) <= 1e-5 * abs(ref) + 1e-6
        near("dlogits", down(dl[r]), lv.g, dtype)
        # the pool's backward pass applied to the dlogits as stored
        t2 = onets.Tape()
        fv2 = onets.Var(feat[r].astype(np.float64))
        lv2 = onets.gap(t2, fv2)
        lv2.g = down(dl[r])
        t2.backward()
        near("dfeat", down(df[r]), fv2.g, dtype)
