"""Single-kernel parity of the replica-grouped convolution kernels (forward, backward-data,
backward-weight) against the oracle's convolution, through the C ABI.

For bf16 the inputs are drawn on the bf16 grid, so both sides see exactly the same numbers and no
ReLU decision depends on input rounding; what remains is the accumulation order (fp32 on the MFMA
units vs float64) and the final rounding of bf16 outputs (half an ulp = 2^-9 relative).
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


def to_bf16_grid(a):
    """Round float32 values to the nearest bf16 (ties to even), returned as float32."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32).astype(np.uint64)
    u = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return u.astype(np.uint32).view(np.float32)


def upload(torch, a, dtype):
    t = torch.as_tensor(np.ascontiguousarray(a, np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if dtype else t.contiguous()


def download(t):
    return t.float().cpu().numpy().astype(np.float64)


def oracle_conv(x, w, bias, resid, relu, stride, pad, dy=None, mask_relu_input=False):
    """Forward output and (if dy given) input / weight gradients of one replica, float64."""
    t = onets.Tape()
    xv, wv = onets.Var(x.astype(np.float64)), onets.Var(w.astype(np.float64))
    bv = onets.Var(bias.astype(np.float64)) if bias is not None else None
    o = onets.conv2d(t, xv, wv, bv, stride, pad)
    if resid is not None:
        o = onets.add(t, o, onets.Var(resid.astype(np.float64)))
    if relu:
        o = onets.relu(t, o)
    if dy is None:
        return o.v, None, None
    o.g = dy.astype(np.float64)
    t.backward()
    return o.v, xv.g, wv.g


def oracle_bias_grad(x, w_shape, dy, stride, pad):
    """Gradient of the layer's bias under the output gradient dy, by the oracle's convolution backward."""
    t = onets.Tape()
    bv = onets.Var(np.zeros(w_shape[0]))
    o = onets.conv2d(t, onets.Var(x.astype(np.float64)), onets.Var(np.zeros(w_shape)), bv, stride, pad)
    o.g = dy.astype(np.float64)
    t.backward()
    return bv.g


def check_weight_and_bias_gradient(torch, pb, desc, dy_dev, x_dev, gw):
    """The form that takes the bias gradient along: same weight gradient; returns the bias part
    [n][cout] (None when the kernel that runs this layer leaves it to the caller, then untouched)."""
    n, Cout = desc.n, desc.cout
    wsize = Cout * desc.k * desc.k * desc.cin
    scratch = torch.zeros(max(pb.parle_k_conv_scratch_bytes(desc) // 4, 4), dtype=torch.float32, device="cuda")
    gwb = torch.full((n, wsize + Cout), float("nan"), dtype=torch.float32, device="cuda")
    took = pb.parle_k_conv_backward_weight_bias(desc, dy_dev, x_dev, scratch, gwb)
    torch.cuda.synchronize()
    # the same kernel; only the grouping of the split sums may differ with the row length (16-byte vectors or not)
    assert float((gwb[:, :wsize] - gw.reshape(n, wsize)).abs().max()) <= 2e-6 * float(gw.abs().max())
    if not took:
        assert bool(torch.isnan(gwb[:, wsize:]).all())
        return None
    return download(gwb[:, wsize:])


CASES = [
    # n, B, H, W, Cin, Cout, k, stride, pad
    (2, 3, 9, 7, 3, 10, 3, 1, 1),       # scalar gathers, narrow output
    (2, 5, 8, 8, 8, 16, 3, 1, 1),       # vector gathers
    (3, 4, 11, 9, 16, 48, 3, 2, 1),     # stride 2, odd extent
    (2, 2, 12, 12, 24, 96, 3, 1, 1),    # 96-wide tile
    (2, 2, 8, 8, 40, 100, 3, 2, 1),     # 128-wide tile with a ragged edge
    (2, 6, 6, 6, 32, 200, 1, 1, 0),     # 1x1, two 128-wide tiles
    (2, 3, 10, 10, 5, 7, 5, 1, 0),      # 5x5 valid, odd channels
    (2, 37, 1, 1, 136, 72, 1, 1, 0),    # fully connected
    (1, 2, 8, 8, 16, 32, 1, 2, 0),      # strided 1x1 (shortcut)
    (2, 3, 16, 16, 32, 40, 3, 1, 1),    # stride-1 "same" conv, one image per 256-pixel tile (LDS patch path)
    (2, 5, 8, 8, 64, 96, 3, 1, 1),      # four images per tile, last tile ragged
    (1, 2, 32, 32, 32, 20, 3, 1, 1),    # four tiles per image, narrow output
    (2, 2, 16, 16, 64, 64, 3, 1, 1),    # both directions on the patch path
    (2, 4, 16, 16, 32, 64, 3, 2, 1),    # stride 2, power-of-two image: backward-data rows grouped by parity class
    (1, 3, 8, 8, 32, 32, 3, 2, 1),      # same, tiles spanning several classes and images
    (2, 3, 16, 8, 16, 32, 1, 2, 0),     # strided 1x1: three of four parity classes reach no tap
    (1, 2, 32, 32, 32, 128, 3, 1, 1),   # backward-weight with nine taps per wavefront: two column blocks, 4 dy tiles
    (1, 3, 16, 16, 64, 160, 3, 1, 1),   # same, 5 dy tiles per workgroup
    (1, 2, 16, 16, 32, 224, 3, 1, 1),   # 7 tiles of 32 output channels: no whole grouping of dy tiles, the transpose-read kernel
    (2, 3, 8, 8, 32, 128, 3, 1, 1),     # same, two 8 x 8 images per block, odd batch
    (1, 2, 24, 16, 32, 192, 3, 1, 1),   # same, two groups of 3 dy tiles, three row blocks per image
    (2, 4, 12, 12, 3, 16, 3, 1, 1),     # whole contraction in one tile (K = 27): first-layer kernel, ragged last tile
    (2, 3, 14, 14, 1, 20, 5, 1, 0),     # same, K = 25, one input channel, 'valid' 5x5
    (1, 5, 16, 16, 3, 96, 3, 2, 1),     # same, stride 2, three 32-channel tiles
    (2, 4, 12, 12, 20, 50, 5, 1, 0),    # LeNet's second conv: backward-data over 50 channels (8-byte gathers in fp32)
    (1, 3, 8, 8, 6, 40, 3, 1, 1),       # forward over 6 channels: 8-byte gathers, 64-wide tile with a ragged edge
    (1, 2, 16, 16, 160, 320, 3, 1, 1),  # WRN-28-10 widths: 320 outputs = 2 x 128 + 64, 160 (backward-data) = 96 + 64
    (2, 2, 32, 32, 64, 96, 3, 2, 1),    # stride-2 backward-data, four parity classes per workgroup: 2 x 2 blocks per image
    (1, 3, 16, 32, 96, 64, 3, 2, 1),    # same, image not square, 96-wide column block
    (1, 2, 16, 16, 160, 32, 3, 2, 1),   # same, 160 channels = 96 + a ragged second block
    (2, 2, 16, 16, 16, 64, 3, 1, 1),    # patch path with half a channel chunk (the first block of the residual networks)
    (1, 2, 16, 16, 40, 48, 3, 1, 1),    # same, one full chunk and a ragged one, in both directions
    (2, 3, 6, 7, 8, 12, 5, 1, 2),       # padded 5x5 window on 6 x 7 pixels, 8 channels
    (1, 2, 8, 8, 32, 10, 2, 1, 0),      # 2x2 window, no padding
    (2, 5, 12, 12, 20, 50, 5, 1, 0),    # LeNet's second convolution: fp32 backward-data with the per-tap products in LDS
    (1, 3, 7, 9, 6, 13, 3, 1, 1),       # same path, padded 3x3 window, odd sizes (63 output pixels, 13 output channels)
    (2, 3, 16, 16, 128, 96, 3, 2, 1),   # stride-2 forward with the input patch in LDS (128 channels or more): two 8 x 8 outputs per tile, odd batch
    (1, 4, 32, 32, 136, 128, 3, 2, 1),  # same, 16 output columns (half an image per tile), a ragged channel chunk
    (1, 2, 32, 32, 128, 320, 3, 2, 1),  # same, 320 outputs = 128 + 128 + 64
    (3, 128, 1, 1, 784, 128, 1, 1, 0),  # the MLP's first layer: contraction split over the wavefronts of a workgroup
    (2, 20, 1, 1, 504, 10, 1, 1, 0),    # same, ten outputs, contraction not a multiple of the four quarters
]


def _takes_bias(case, dtype):
    """Layers whose weight-gradient kernel also writes the bias gradient: the small first-layer kernels when the
    window leaves one of their 32 contraction columns free, and in bf16 the stride-1 3x3 kernel and the
    transpose-read kernel (channel counts that are multiples of 8, at least 32 outputs)."""
    n, B, H, W, Cin, Cout, k, stride, pad = case
    K = k * k * Cin
    if dtype == 0:       # every fp32 kernel but the per-image LDS one of a few-channel layer under a wide window
        if K <= 32 and Cout <= 32:
            return K < 32
        P, Q = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
        window = (stride == 1 and k >= 2 and P * Q <= 64 and P * Q % 8 == 0 and 128 <= K <= 512 and Cout <= 64
                  and (H + 2 * pad) * (W + 2 * pad) * Cin <= 6144)
        return not window
    if K <= 32 and Cout % 8 == 0:
        return K < 32
    return Cin % 8 == 0 and Cout % 8 == 0 and Cout >= 32


def tolerances(dtype, ref):
    scale = np.abs(ref).max()
    if dtype == 0:
        return 0.0, 2e-5 * scale
    return 2.0 ** -8, 2e-5 * scale


def assert_near(name, got, ref, rel, absol):
    err = np.abs(got - ref)
    bound = rel * np.abs(ref) + absol
    bad = err > bound
    assert not bad.any(), f"{name}: {bad.sum()} of {bad.size} outside tolerance, worst {np.max(err - bound):.3e}"


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("dtype", [0, 1])
def test_conv_kernels_match_oracle(gpu, case, dtype):
    torch, pb = gpu
    n, B, H, W, Cin, Cout, k, stride, pad = case
    rng = np.random.default_rng(hash(case) % (2 ** 31))
    q = to_bf16_grid if dtype else (lambda a: np.asarray(a, np.float32))
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    x = q(rng.standard_normal((n, B, H, W, Cin)))
    w = q(rng.standard_normal((n, Cout, k, k, Cin)) / np.sqrt(k * k * Cin))
    bias = rng.standard_normal((n, Cout)).astype(np.float32)
    resid = q(rng.standard_normal((n, B, Ho, Wo, Cout)))
    dy = q(rng.standard_normal((n, B, Ho, Wo, Cout)))
    mask = q(rng.standard_normal((n, B, H, W, Cin)))
    prev = q(rng.standard_normal((n, B, H, W, Cin)))
    desc = pb.parle_conv_desc(dtype, n, B, H, W, Cin, Cout, k, stride, pad)
    tdt = torch.bfloat16 if dtype else torch.float32
    dx_, dw_, dres = upload(torch, x, dtype), upload(torch, w, dtype), upload(torch, resid, dtype)
    dbias, ddy, dmask = upload(torch, bias, 0), upload(torch, dy, dtype), upload(torch, mask, dtype)

    # forward: plain, and with bias + residual + ReLU
    y1 = torch.zeros((n, B, Ho, Wo, Cout), dtype=tdt, device="cuda")
    y2 = torch.zeros_like(y1)
    pb.parle_k_conv_forward(desc, dx_, dw_, None, None, 0, y1)
    pb.parle_k_conv_forward(desc, dx_, dw_, dbias, dres, 1, y2)
    # backward data: plain write, then masked accumulate onto an existing gradient
    wt = torch.zeros(n * Cout * k * k * Cin, dtype=tdt, device="cuda")
    g1 = torch.zeros((n, B, H, W, Cin), dtype=tdt, device="cuda")
    g2 = upload(torch, prev, dtype)
    pb.parle_k_conv_backward_data(desc, ddy, dw_, None, 0, wt, g1)
    pb.parle_k_conv_backward_data(desc, ddy, dw_, dmask, 1, wt, g2)
    # backward weight
    sb = pb.parle_k_conv_scratch_bytes(desc)
    scratch = torch.zeros(max(sb // 4, 4), dtype=torch.float32, device="cuda")
    gw = torch.zeros((n, Cout, k, k, Cin), dtype=torch.float32, device="cuda")
    pb.parle_k_conv_backward_weight(desc, ddy, dx_, scratch, gw)
    torch.cuda.synchronize()
    gb = check_weight_and_bias_gradient(torch, pb, desc, ddy, dx_, gw)
    assert (gb is not None) == _takes_bias(case, dtype), "which kernels take the bias gradient along changed"

    for r in range(n):
        if gb is not None:
            rdb = oracle_bias_grad(x[r], w[r].shape, dy[r], stride, pad)
            assert_near(f"bias gradient[{r}]", gb[r], rdb, 0.0, 2e-5 * np.abs(dy[r]).sum(axis=(0, 1, 2)).max())
        ref1, rdx, rdw = oracle_conv(x[r], w[r], None, None, False, stride, pad, dy[r])
        ref2, _, _ = oracle_conv(x[r], w[r], bias[r], resid[r], True, stride, pad)
        assert_near(f"fwd[{r}]", download(y1[r]), ref1, *tolerances(dtype, ref1))
        assert_near(f"fwd+epilogue[{r}]", download(y2[r]), ref2, *tolerances(dtype, ref2))
        assert_near(f"dgrad[{r}]", download(g1[r]), rdx, *tolerances(dtype, rdx))
        ref_acc = prev[r].astype(np.float64) + rdx * (mask[r] > 0)
        rel, ab = tolerances(dtype, ref_acc)
        assert_near(f"dgrad masked accumulate[{r}]", download(g2[r]), ref_acc, rel, ab)
        assert_near(f"wgrad[{r}]", download(gw[r]), rdw, 0.0, 2e-5 * np.abs(rdw).max())


@pytest.mark.parametrize("case,expect_sums", [
    # n, B, H, W, Cin, Cout, k, stride, pad; does the kernel that runs the layer take the sums?
    ((2, 8, 16, 16, 16, 64, 3, 1, 1), True),      # 64-wide blocks
    ((2, 3, 16, 16, 32, 128, 3, 1, 1), True),     # one 128-wide block
    ((1, 6, 8, 8, 64, 320, 3, 1, 1), True),       # 320 = 128 + 128 + 64: the narrower last block; 4 images per tile, 6 images
    ((3, 128, 32, 32, 64, 64, 3, 1, 1), True),    # WRN-16-4 group 1 at full size: 512 partial rows
    ((3, 128, 8, 8, 256, 256, 3, 1, 1), True),    # WRN-16-4 group 3 at full size
    ((2, 4, 16, 16, 32, 160, 3, 1, 1), False),    # 96-wide blocks: no sums, the caller reduces
    ((2, 4, 16, 16, 32, 64, 3, 2, 1), False),     # stride 2, 64 outputs: a tile shape that takes none
    ((2, 5, 16, 16, 128, 64, 3, 2, 1), True),     # stride 2 with the patch in LDS (128 input channels or more): 64-wide blocks, odd batch
    ((1, 6, 16, 16, 160, 320, 3, 2, 1), True),    # same, 320 outputs = 128 + 128 + a 64-wide last block
    ((2, 5, 16, 16, 64, 128, 3, 2, 1), True),     # stride 2 (first convolution of a group): 128-row tiles, 2 x 2 wavefronts
    ((1, 6, 16, 16, 32, 320, 3, 2, 1), True),     # same, 320 outputs = 256 + a ragged second block
    ((3, 128, 32, 32, 64, 128, 3, 2, 1), True),   # WRN-16-4 group 2's first convolution at full size
    ((2, 4, 16, 16, 32, 160, 3, 2, 1), False),    # stride 2, 160 outputs: 96-wide tiles
    ((2, 9, 16, 16, 3, 16, 3, 1, 1), True),       # the first layer (whole contraction in one tile), a ragged last tile
    ((3, 128, 32, 32, 3, 16, 3, 1, 1), True),     # WRN's first layer at full size
])
def test_conv_epilogue_column_sums(gpu, case, expect_sums):
    """The sums a convolution leaves for the batch-norm behind it are the column sums of exactly what it stored
    (bf16 values) and of their squares, to fp32 summation accuracy; with a residual as in the second convolution
    of a block."""
    torch, pb = gpu
    n, B, H, W, Cin, Cout, k, stride, pad = case
    rng = np.random.default_rng(hash(case) % (2 ** 31))
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    x = upload(torch, to_bf16_grid(rng.standard_normal((n, B, H, W, Cin))), 1)
    w = upload(torch, to_bf16_grid(rng.standard_normal((n, Cout, k, k, Cin)) / np.sqrt(k * k * Cin)), 1)
    # a per-channel offset makes mean^2 >> variance in some channels, where one-pass variances are delicate
    shift = np.linspace(-4.0, 4.0, Cout).astype(np.float32)
    resid = upload(torch, to_bf16_grid(rng.standard_normal((n, B, Ho, Wo, Cout)) + shift), 1)
    desc = pb.parle_conv_desc(1, n, B, H, W, Cin, Cout, k, stride, pad)
    cap = 1024
    for res in (None, resid):
        y = torch.zeros((n, B, Ho, Wo, Cout), dtype=torch.bfloat16, device="cuda")
        y_plain = torch.zeros_like(y)
        partial = torch.full((n * cap * 2 * Cout,), float("nan"), dtype=torch.float64, device="cuda")
        S = pb.parle_k_conv_forward_colsums(desc, x, w, res, y, partial, cap)
        pb.parle_k_conv_forward(desc, x, w, None, res, 0, y_plain)
        torch.cuda.synchronize()
        assert torch.equal(y, y_plain), "the sums must not change what is stored"
        if not expect_sums:
            assert S == 0 and bool(torch.isnan(partial).all())
            continue
        M = B * Ho * Wo
        span = 256 if S == (M + 255) // 256 else 128      # rows of y per partial row: the kernel's row tile
        assert S == (M + span - 1) // span
        used = n * S * 2 * Cout          # [n][S][2][Cout], replicas S rows apart
        got = partial[:used].cpu().numpy().reshape(n, S, 2, Cout)
        assert np.isfinite(got).all() and bool(torch.isnan(partial[used:]).all())
        yv = y.double().cpu().numpy().reshape(n, M, Cout)
        # per partial row: the rows of its tile
        pad_rows = S * span - M
        yt = np.concatenate([yv, np.zeros((n, pad_rows, Cout))], axis=1).reshape(n, S, span, Cout)
        ref1, ref2 = yt.sum(axis=2), (yt * yt).sum(axis=2)
        scale1 = np.abs(yt).sum(axis=2) + 1e-30
        assert np.max(np.abs(got[:, :, 0] - ref1) / scale1) < 1e-5   # one element of 256 left out would show as 4e-3
        assert np.max(np.abs(got[:, :, 1] - ref2) / (ref2 + 1e-30)) < 1e-5


@pytest.mark.parametrize("layer", [
    # full-size layers of the workloads at the launch shapes the bench times (batch 128): dtype, n, B, H, W, Cin, Cout, k, stride, pad
    (1, 3, 128, 32, 32, 96, 96, 3, 1, 1),      # All-CNN-C conv2
    (1, 3, 128, 16, 16, 192, 192, 3, 2, 1),    # All-CNN-C conv6 (stride 2)
    (1, 3, 128, 32, 32, 16, 64, 3, 1, 1),      # WRN-16-4 group 1
    (1, 3, 128, 16, 16, 128, 128, 3, 1, 1),    # WRN-16-4 group 2: 64-wide column blocks, two per pixel tile
    (1, 3, 128, 8, 8, 256, 256, 3, 1, 1),      # WRN-16-4 group 3
    (1, 3, 128, 32, 32, 3, 96, 3, 1, 1),       # All-CNN-C conv1: the first layer (whole contraction in one tile)
    (1, 3, 128, 32, 32, 3, 16, 3, 1, 1),       # WRN conv1
    (1, 3, 128, 8, 8, 192, 192, 1, 1, 0),      # All-CNN-C conv8: 1x1
    (1, 3, 128, 8, 8, 192, 10, 1, 1, 0),       # All-CNN-C conv9: 1x1, ten outputs
    (1, 3, 128, 32, 32, 64, 128, 1, 2, 0),     # WRN-16-4 g2b1 shortcut: 1x1, stride 2
    (1, 3, 128, 32, 32, 160, 320, 3, 2, 1),    # WRN-28-10 g2b1.conv1: 160 -> 320, stride 2
    (1, 3, 128, 16, 16, 320, 320, 3, 1, 1),    # WRN-28-10 group 2
    (0, 6, 128, 28, 28, 1, 20, 5, 1, 0),       # LeNet conv1, fp32, six replicas
    (0, 6, 128, 12, 12, 20, 50, 5, 1, 0),      # LeNet conv2, fp32 (backward-data in two passes)
])
def test_full_size_layers_sampled(gpu, layer):
    """Forward and backward-data are checked on sampled images (rows are independent); the weight gradient on
    sampled output and input channels, summed over all 128 images by the oracle's own convolution backward
    (the gradient entry (co, i, j, ci) depends only on channel co of dy and channel ci of x)."""
    torch, pb = gpu
    dtype, n, B, H, W, Cin, Cout, k, stride, pad = layer
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    gen = torch.Generator(device="cuda").manual_seed(7)
    tdt = torch.bfloat16 if dtype else torch.float32
    x = torch.randn((n, B, H, W, Cin), generator=gen, device="cuda").to(tdt)
    w = (torch.randn((n, Cout, k, k, Cin), generator=gen, device="cuda") / np.sqrt(k * k * Cin)).to(tdt)
    dy = torch.randn((n, B, Ho, Wo, Cout), generator=gen, device="cuda").to(tdt)
    desc = pb.parle_conv_desc(dtype, n, B, H, W, Cin, Cout, k, stride, pad)
    y = torch.zeros((n, B, Ho, Wo, Cout), dtype=tdt, device="cuda")
    dx = torch.zeros((n, B, H, W, Cin), dtype=tdt, device="cuda")
    wt = torch.zeros(n * Cout * k * k * Cin, dtype=tdt, device="cuda")
    gw = torch.zeros((n, Cout, k, k, Cin), dtype=torch.float32, device="cuda")
    scratch = torch.zeros(max(pb.parle_k_conv_scratch_bytes(desc) // 4, 4), dtype=torch.float32, device="cuda")
    pb.parle_k_conv_forward(desc, x, w, None, None, 0, y)
    pb.parle_k_conv_backward_data(desc, dy, w, None, 0, wt, dx)
    pb.parle_k_conv_backward_weight(desc, dy, x, scratch, gw)
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    for r in (0, n - 1):
        wr = download(w[r])
        for b in (0, int(rng.integers(1, B - 1)), B - 1):
            ry, rdx, _ = oracle_conv(download(x[r, b:b + 1]), wr, None, None, False, stride, pad, download(dy[r, b:b + 1]))
            assert_near("fwd", download(y[r, b:b + 1]), ry, *tolerances(dtype, ry))
            assert_near("dgrad", download(dx[r, b:b + 1]), rdx, *tolerances(dtype, rdx))
        got = download(gw[r])
        scale = np.abs(got).max()
        cos = np.sort(rng.choice(Cout, size=min(Cout, 6), replace=False))
        cis = np.sort(rng.choice(Cin, size=min(Cin, 6), replace=False))
        xs, dys = download(x[r][..., cis]), download(dy[r][..., cos])
        _, _, rdw = oracle_conv(xs, np.zeros((len(cos), k, k, len(cis))), None, None, False, stride, pad, dys)
        sub = got[cos][:, :, :, cis]
        assert np.abs(rdw).max() > 0.2 * scale                       # the sample is not a corner of small entries
        assert_near("wgrad", sub, rdw, 1e-5, 2e-5 * scale)
    gb = check_weight_and_bias_gradient(torch, pb, desc, dy, x, gw)
    assert (gb is not None) == _takes_bias(layer[1:], dtype)
    if gb is not None:
        for r in (0, n - 1):
            cos = np.sort(rng.choice(Cout, size=min(Cout, 6), replace=False))
            dys = download(dy[r][..., cos])
            rdb = oracle_bias_grad(download(x[r][..., :1]), (len(cos), k, k, 1), dys, stride, pad)
            assert_near("bias gradient", gb[r][cos], rdb, 0.0, 2e-5 * np.abs(dys).sum(axis=(0, 1, 2)).max())
