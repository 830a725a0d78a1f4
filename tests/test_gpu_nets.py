"""GPU parity of the replica-batched forward / loss / backward and of whole Parle cycles on networks.

The device path (C ABI) and the CPU oracle (float64) get the same seeded images, labels and initial
parameters.  Bars:
  * fp32 compute: every state tensor within 1e-5 (relative 2-norm and max-abs relative to the largest
    entry) after L inner steps and the outer step -- the bound the workload definition states;
    raw gradients of one step within 1e-4 (fp32 rounding of a gradient is a few 1e-5 of its size; on its
    way into the state it is multiplied by eta <= 0.1 and set against parameters that are larger than one
    step of them, which is what keeps the state inside 1e-5);
  * bf16 compute (fp32 master weights): losses and state tensors within 2e-2.
"""
import numpy as np
import pytest

from oracle import nets as onets
from oracle import parle as oparle
from oracle import trainer as otrainer
from paper_1707_00424_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1707_00424_amd import binding as pb
    pb.lib()
    return torch, pb


def rel2(got, ref):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    return np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)


def relmax(got, ref):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    return np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30)


def check(name, got, ref, tol, max_factor=1.0):
    """2-norm relative error <= tol and max-abs error <= max_factor * tol * max|ref|."""
    assert np.isfinite(np.asarray(got)).all(), name
    assert rel2(got, ref) <= tol, f"{name}: rel 2-norm {rel2(got, ref):.3e} > {tol}"
    assert relmax(got, ref) <= tol * max_factor, f"{name}: rel max {relmax(got, ref):.3e} > {tol * max_factor}"


def segment_errors(layout, got, ref):
    """Per parameter segment: (name, relative 2-norm error, cosine) of got against ref, both [N] or [n, N]."""
    out, off = [], 0
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    for s in layout:
        size = int(np.prod(s["shape"]))
        g, r = got[..., off:off + size].ravel(), ref[..., off:off + size].ravel()
        den = np.sqrt((g * g).sum() * (r * r).sum())
        out.append((s["name"], rel2(g, r), float((g * r).sum() / den) if den > 0 else 1.0))
        off += size
    return out


def model_pair(pb, a):
    """Library model id and arch[] for an oracle architecture dict."""
    m = a["model"]
    if m == "mlp":
        return pb.MODEL_MLP, (a["hidden"],)
    if m == "lenet":
        return pb.MODEL_LENET, (a["c1"], a["c2"], a["k"], a["fc"])
    if m == "allcnn":
        return pb.MODEL_ALLCNN_C, (a["ca"], a["cb"])
    return pb.MODEL_WRN, (a["base"], a["widen"], a["nb"])


def make(pb, a, n, B, bf16=0, seed=0, distinct_init=False, oracle_dtype=np.float64, storage=None, **kw):
    model, arch = model_pair(pb, a)
    base = dict(n_replicas=n, L=25, eta_inner=0.1, eta_outer=0.1, momentum=0.9, alpha=0.75, gamma0=0.03, rho0=1.0)
    base.update(kw)
    cfg = pb.make_config(model=model, batch=B, compute_bf16=bf16, in_h=a["H"], in_w=a["W"], in_c=a["C"],
                         n_classes=a["classes"], arch=arch, lenet_bn=a.get("bn", 0), **base)
    lay = pb.parle_query_layout(cfg)
    assert [(s["name"], s["shape"]) for s in lay] == [(s["name"], s["shape"]) for s in onets.layout(a)]
    wi = "uniform" if a["model"] in ("mlp", "lenet") else "he_normal"
    if distinct_init:
        x0 = np.stack([synth.init_params(lay, seed + 17 * i, wi) for i in range(n)])
    else:
        x0 = np.tile(synth.init_params(lay, seed, wi), (n, 1))
    P = pb.Parle(cfg, x0)
    ocfg = oparle.ParleConfig(**{k: v for k, v in base.items() if k not in ("fuse_outer", "graph_block")})
    O = otrainer.ParleNet(a, ocfg, x0, dtype=oracle_dtype, storage=storage)
    return P, O


def dev(torch, a, dtype=None):
    return torch.as_tensor(np.ascontiguousarray(a)).cuda()


SMALL = {
    # odd channel counts and sizes: scalar gather paths, ragged tiles
    "mlp_odd": onets.arch("mlp", H=5, W=3, C=1, hidden=37, classes=7),
    "lenet_odd": onets.arch("lenet", H=14, W=12, C=1, c1=3, c2=5, k=3, fc=21, classes=4),
    "allcnn_odd": onets.arch("allcnn", H=12, W=10, C=3, ca=5, cb=7, classes=3),
    "wrn_odd": onets.arch("wrn", H=8, W=12, C=3, base=3, widen=2, nb=1, classes=5),
    # channel counts that take the 16-byte vector paths and more than one tile
    "mlp_vec": onets.arch("mlp", H=8, W=8, C=1, hidden=72, classes=10),
    "lenet_vec": onets.arch("lenet", H=20, W=20, C=1, c1=8, c2=16, k=5, fc=40, classes=10),
    "allcnn_vec": onets.arch("allcnn", H=16, W=16, C=3, ca=16, cb=40, classes=10),
    "wrn_vec": onets.arch("wrn", H=16, W=16, C=3, base=8, widen=2, nb=2, classes=10),
}


@pytest.mark.parametrize("name", list(SMALL))
@pytest.mark.parametrize("bf16", [0, 1])
def test_one_step_loss_and_gradient(gpu, name, bf16):
    torch, pb = gpu
    a = SMALL[name]
    n, B = 2, 9
    P, O = make(pb, a, n, B, bf16=bf16, seed=3, distinct_init=True, storage="bf16" if bf16 else None)
    X, Y = synth.image_batches(5, 1, n, B, a["H"], a["W"], a["C"], a["classes"])
    loss = torch.zeros(n, dtype=torch.float32, device="cuda")
    P.parle_inner_step(dev(torch, X[0]), dev(torch, Y[0]), loss)
    ref_loss = O.inner_step(X[0], Y[0])
    got = P.state()
    if bf16:
        # The oracle keeps activations, their gradients and the weights inside the contractions on the bf16 grid,
        # as the device does, and sums exactly; the device sums in fp32.  The two passes are then equal value for
        # value unless some fp32 sum lands on the other side of a bf16 rounding boundary than the exact sum
        # (about 3e-5 of the stored values).  One such value, one ulp apart, moves the roundings of what follows
        # and with them a gradient computed in bf16 by up to ~10 % (the oracle shows this on itself:
        # tests/test_oracle_chaos.py).  So a replica either has no such event, and then every segment of its
        # gradient matches to 1e-4 (measured 1e-9 .. 7e-5) and its loss to 1e-6, or it has one, and then the
        # loss is held to 2e-3 and the gradient by direction and size only.
        lay = onets.layout(a)
        got_loss = loss.cpu().numpy()
        sharp = 0
        for r in range(n):
            g, ref = got["grad"][r].astype(np.float64), O.last_grad[r]
            worst = max(err for _, err, _ in segment_errors(lay, g, ref))
            if worst <= 1e-4:
                sharp += 1
                assert abs(got_loss[r] / ref_loss[r] - 1) <= 1e-6, (name, r)
            else:
                assert abs(got_loss[r] / ref_loss[r] - 1) <= 2e-3, (name, r)
                cos = (g * ref).sum() / np.sqrt((g * g).sum() * (ref * ref).sum())
                assert cos >= 0.95 and abs(np.linalg.norm(g) / np.linalg.norm(ref) - 1) <= 0.1, (name, r, cos)
        print(f"{name} bf16: {sharp} of {n} replicas free of rounding events, held to 1e-4 per segment")
        return
    np.testing.assert_allclose(loss.cpu().numpy(), ref_loss, rtol=1e-5)
    for r in range(n):
        check(f"{name} grad[{r}]", got["grad"][r], O.last_grad[r], 1e-4)
    # per-segment check so that a small layer cannot hide behind a large one
    off = 0
    for s in onets.layout(a):
        size = int(np.prod(s["shape"]))
        check(f"{name} grad {s['name']}", got["grad"][:, off:off + size], O.last_grad[:, off:off + size], 1e-4)
        off += size
    for t in ("y", "z", "vy"):
        check(f"{name} {t}", got[t], getattr(O.st, t), 1e-5)


MANY_CLASSES = {
    # more classes than the one-kernel heads take (16): the last layer, the loss and the pool keep their own kernels;
    # 300 features: more than the fully connected head takes (256)
    "mlp_17": onets.arch("mlp", H=6, W=6, C=1, hidden=40, classes=17),
    "mlp_300": onets.arch("mlp", H=6, W=6, C=1, hidden=300, classes=10),
    "allcnn_18": onets.arch("allcnn", H=8, W=8, C=3, ca=8, cb=16, classes=18),
    "wrn_20": onets.arch("wrn", H=8, W=8, C=3, base=4, widen=2, nb=1, classes=20),
}


@pytest.mark.parametrize("name", list(MANY_CLASSES))
def test_heads_beyond_the_one_kernel_limits(gpu, name):
    torch, pb = gpu
    a = MANY_CLASSES[name]
    n, B = 2, 7
    P, O = make(pb, a, n, B, seed=5, distinct_init=True)
    X, Y = synth.image_batches(6, 1, n, B, a["H"], a["W"], a["C"], a["classes"])
    loss = torch.zeros(n, dtype=torch.float32, device="cuda")
    P.parle_inner_step(dev(torch, X[0]), dev(torch, Y[0]), loss)
    ref_loss = O.inner_step(X[0], Y[0])
    np.testing.assert_allclose(loss.cpu().numpy(), ref_loss, rtol=1e-5)
    got = P.state()
    for seg, err, _ in segment_errors(onets.layout(a), got["grad"].astype(np.float64), O.last_grad):
        assert err <= 1e-4, (name, seg, err)


TINY_BF16 = {
    # few enough stored values that about half of the replicas see no rounding event at all
    "allcnn": onets.arch("allcnn", H=8, W=8, C=3, ca=8, cb=16, classes=5),
    "wrn": onets.arch("wrn", H=8, W=8, C=3, base=2, widen=2, nb=2, classes=5),      # identity and shortcut blocks
    "wrn_wide": onets.arch("wrn", H=8, W=8, C=3, base=8, widen=1, nb=1, classes=5),  # 16-byte vector kernels
    "lenet_bn": onets.arch("lenet", H=12, W=12, C=1, c1=4, c2=8, k=3, fc=16, classes=5, bn=1),
}


@pytest.mark.parametrize("name", list(TINY_BF16))
def test_bf16_event_free_replicas_match_to_1e_4(gpu, name):
    """Sixteen replicas (own weights, own batch of five images) of a tiny network in bf16 against the oracle in its
    bf16 storage mode.  A replica in which no fp32 sum fell on the other side of a bf16 rounding boundary than the
    exact sum must agree with the oracle to 1e-4 on every gradient segment and 1e-6 on the loss -- that is every
    kernel of the forward and backward pass, every residual add, shortcut and gradient accumulation, value for
    value.  The others (see test_one_step_loss_and_gradient) are held by direction and size.  At least a quarter of
    the replicas must be of the first kind: a wrong kernel would show as an "event" in every replica."""
    torch, pb = gpu
    a, n, B = TINY_BF16[name], 16, 5
    P, O = make(pb, a, n, B, bf16=1, seed=11, distinct_init=True, storage="bf16")
    X, Y = synth.image_batches(12, 1, n, B, a["H"], a["W"], a["C"], a["classes"])
    loss = torch.zeros(n, dtype=torch.float32, device="cuda")
    P.parle_inner_step(dev(torch, X[0]), dev(torch, Y[0]), loss)
    ref_loss = O.inner_step(X[0], Y[0])
    got, got_loss, lay = P.state(), loss.cpu().numpy(), onets.layout(a)
    sharp, worst_sharp = 0, 0.0
    for r in range(n):
        g, ref = got["grad"][r].astype(np.float64), O.last_grad[r]
        worst = max(err for _, err, _ in segment_errors(lay, g, ref))
        if worst <= 1e-4:
            sharp += 1
            worst_sharp = max(worst_sharp, worst)
            assert abs(got_loss[r] / ref_loss[r] - 1) <= 1e-6, (name, r)
        else:
            assert abs(got_loss[r] / ref_loss[r] - 1) <= 5e-3, (name, r)
            cos = (g * ref).sum() / np.sqrt((g * g).sum() * (ref * ref).sum())
            assert cos >= 0.9 and abs(np.linalg.norm(g) / np.linalg.norm(ref) - 1) <= 0.15, (name, r, cos)
    print(f"{name} bf16: {sharp} of {n} replicas free of rounding events (worst segment error {worst_sharp:.1e})")
    assert sharp >= 4


@pytest.mark.parametrize("name", ["mlp_odd", "lenet_odd", "allcnn_odd", "wrn_odd"])
def test_one_replica_one_image(gpu, name):
    """Degenerate sizes: n = 1 replica, a mini-batch of one image (the batch-norm statistics of the residual
    network are then over the pixels of that image alone); one inner step and an outer step, fp32."""
    torch, pb = gpu
    a = SMALL[name]
    P, O = make(pb, a, 1, 1, bf16=0, seed=11, L=1)
    X, Y = synth.image_batches(8, 1, 1, 1, a["H"], a["W"], a["C"], a["classes"])
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    P.parle_inner_step(dev(torch, X[0]), dev(torch, Y[0]), loss)
    ref_loss = O.inner_step(X[0], Y[0])
    assert O.relu_margin > 2e-6, O.relu_margin   # no pre-activation within float32 rounding of the kink
    np.testing.assert_allclose(loss.cpu().numpy(), ref_loss, rtol=1e-5)
    check(f"{name} grad", P.state()["grad"], O.last_grad, 1e-4)
    P.parle_outer_step()
    O.outer_step()
    got = P.state()
    for t in ("x", "y", "z", "vx", "x_ref"):
        check(f"{name} {t}", got[t], getattr(O.st, t), 1e-5)


def _cycle(pb, torch, a, n, B, L, bf16, seed, outer=1, **kw):
    P, O = make(pb, a, n, B, bf16=bf16, seed=seed, L=L, **kw)
    X, Y = synth.image_batches(seed, L * outer, n, B, a["H"], a["W"], a["C"], a["classes"])
    dX, dY = dev(torch, X), dev(torch, Y)
    loss = torch.zeros((L * outer, n), dtype=torch.float32, device="cuda")
    ref_loss = np.zeros((L * outer, n))
    for k in range(L * outer):
        P.parle_inner_step(dX[k], dY[k], loss[k])
        ref_loss[k] = O.inner_step(X[k], Y[k])
        if (k + 1) % L == 0:
            P.parle_outer_step()
            O.outer_step()
    return P, O, loss.cpu().numpy(), ref_loss


def test_config1_mlp_full_cycle(gpu):
    """n = 3 replicas of the 784-128-10 MLP, batch 128, L = 25 inner steps + 1 outer step, fp32."""
    torch, pb = gpu
    P, O, loss, ref_loss = _cycle(pb, torch, onets.arch("mlp"), 3, 128, 25, 0, seed=0)
    got = P.state()
    for t in ("x", "y", "z", "vy", "vx", "x_ref"):
        check(t, got[t], getattr(O.st, t), 1e-5)
    np.testing.assert_allclose(loss, ref_loss, rtol=1e-4, atol=2e-6)
    assert ref_loss[-1].mean() < ref_loss[0].mean()          # it trains


def _push_state(P, O, torch, names):
    """Overwrite the device state tensors with the oracle's (rounded to fp32)."""
    N = P.sizes.n_params
    for t in names:
        getattr(P, t)[:, :N].copy_(torch.as_tensor(getattr(O.st, t).astype(np.float32)))


# Which ReLU / max-pool decisions (numbered in forward order: ReLU, pool, ReLU, pool, ReLU) enter the gradient of a
# LeNet layer: those between the layer's output and the loss.  fc2 has none behind it.
LENET_FIRST_SITE = {"conv1": 0, "conv2": 2, "fc1": 4, "fc2": 5}
# A decision is "at risk" when its margin is within what fp32 accumulation of the pre-activation can be off by:
# 64 ulp of the largest input of that ReLU / pool (measured: the float32 oracle's pre-activations differ from the
# float64 ones by up to 15 ulp of the largest entry on conv1, contraction length 25; fc1 sums 800 terms).
RISK_ULPS = 64.0


def _at_risk(decisions, first_site):
    return any(m <= RISK_ULPS * 2.0 ** -24 * scale for _, m, scale in decisions[first_site:])


def test_config3_lenet_every_step_from_the_oracle_state(gpu):
    """n = 6 replicas of LeNet (20/50 channels, 5x5, fc 500), batch 128, L = 25 + outer step, fp32, step size 0.1.

    This network (no batch-norm) at step size 0.1 amplifies a single differing ReLU / max-pool
    decision into 1e-3 differences within 25 steps -- the oracle's own float32 mode departs from
    its float64 mode that much (tests/test_oracle_chaos.py).  So each of the 25 inner steps and
    the outer step is checked from the SAME state: the oracle's trajectory is pushed to the device
    before every step, and what the device makes of it must match to 1e-5 on the parameters.

    The sharp bars (gradient of a segment within 1e-4, its slice of y, z within 1e-5 of the largest entry,
    element by element) apply to every (step, replica, segment) whose gradient no at-risk decision enters: the
    oracle reports, per ReLU and max-pool, how close any input came to zero / any winner to its runner-up, and a
    decision can only change the gradients of the layers below it.  Only where a decision behind a segment was
    within rounding does the wide guard apply (1e-2 on that segment's gradient, 100x on single entries)."""
    torch, pb = gpu
    a, n, B, L = onets.arch("lenet"), 6, 128, 25
    P, O = make(pb, a, n, B, seed=0)
    X, Y = synth.image_batches(0, L, n, B, a["H"], a["W"], a["C"], a["classes"])
    dX, dY = dev(torch, X), dev(torch, Y)
    loss = torch.zeros(n, dtype=torch.float32, device="cuda")
    segs, off = [], 0
    for sg in onets.layout(a):
        size = int(np.prod(sg["shape"]))
        segs.append((sg["name"], off, off + size, LENET_FIRST_SITE[sg["name"].split(".")[0]]))
        off += size
    sharp = wide = 0
    worst_sharp = worst_wide = 0.0
    for k in range(L):
        _push_state(P, O, torch, ("y", "z", "vy"))
        P.parle_inner_step(dX[k], dY[k], loss)
        ref_loss = O.inner_step(X[k], Y[k])
        got = P.state()
        np.testing.assert_allclose(loss.cpu().numpy(), ref_loss, rtol=1e-5)
        for t in ("y", "z"):
            check(f"step {k} {t}", got[t], getattr(O.st, t), 1e-5, max_factor=100)
        for r in range(n):
            assert len(O.last_decisions[r]) == 5
            for name, lo, hi, site in segs:
                gerr = rel2(got["grad"][r, lo:hi], O.last_grad[r, lo:hi])
                if not _at_risk(O.last_decisions[r], site):
                    sharp += 1
                    worst_sharp = max(worst_sharp, gerr)
                    assert gerr <= 1e-4, (k, r, name, gerr)
                    for t in ("y", "z"):
                        ref = getattr(O.st, t)[r]
                        e = np.abs(got[t][r, lo:hi] - ref[lo:hi]).max()
                        assert e <= 1e-5 * np.abs(ref).max(), (k, r, name, t, e)
                else:
                    wide += 1
                    worst_wide = max(worst_wide, gerr)
                    assert gerr <= 1e-2, (k, r, name, gerr)
        assert rel2(got["vy"], O.st.vy) <= 2e-3, k
    _push_state(P, O, torch, ("y", "z", "vy"))
    P.parle_outer_step()
    O.outer_step()
    got = P.state()
    for t in ("x", "y", "z", "vy", "vx", "x_ref"):
        check("outer " + t, got[t], getattr(O.st, t), 1e-5)
    print(f"config 3 teacher-forced: {sharp} (step, replica, segment) triples held to 1e-4 (worst {worst_sharp:.2e}), "
          f"{wide} behind an at-risk decision held to 1e-2 (worst {worst_wide:.2e})")
    assert sharp >= 0.25 * (sharp + wide)         # a good share of the run is held to the sharp bar


def test_config3_lenet_free_running_at_step_size_0p1(gpu):
    """The same workload free-running at step size 0.1: 25 inner steps + the outer step with no state push.
    The workload definition names no step size for this network; 0.1 is the value of the MLP workload and of the
    paper's LeNet, which has batch-norm.  Without it the run is unstable on these inputs (the oracle's loss jumps
    from 2.0 to 3.8 at step 15) and any two float32 computations end up O(0.1 - 1) apart: the oracle's own
    float32 mode leaves its float64 mode by 7e-2 on y, the device by 0.57 (measured).  Nothing sharper than "of the same order" can be asserted of such a
    run;
    the figures are printed for the record, the sharp checks of this workload are the teacher-forced test above
    and the free-running run at step size 0.01 below."""
    torch, pb = gpu
    a, n, B, L = onets.arch("lenet"), 6, 128, 25
    P, O = make(pb, a, n, B, seed=0)
    O32 = otrainer.ParleNet(a, O.cfg, O.st.x.astype(np.float32), dtype=np.float32)
    X, Y = synth.image_batches(0, L, n, B, a["H"], a["W"], a["C"], a["classes"])
    dX, dY = dev(torch, X), dev(torch, Y)
    first_dev = first_32 = None
    for k in range(L):
        P.parle_inner_step(dX[k], dY[k], None)
        O.inner_step(X[k], Y[k])
        O32.inner_step(X[k], Y[k])
        d_dev, d_32 = rel2(P.state()["y"], O.st.y), rel2(O32.st.y, O.st.y)
        if first_dev is None and d_dev > 1e-5:
            first_dev = k
        if first_32 is None and d_32 > 1e-5:
            first_32 = k
    got = P.state()
    report = {}
    for t in ("y", "z"):
        report[t] = (rel2(got[t], getattr(O.st, t)), rel2(getattr(O32.st, t), getattr(O.st, t)))
    P.parle_outer_step()
    O.outer_step()
    O32.outer_step()
    got = P.state()
    for t in ("x", "x_ref"):
        report[t] = (rel2(got[t], getattr(O.st, t)), rel2(getattr(O32.st, t), getattr(O.st, t)))
    print("config 3 free-running at step size 0.1, distance to the float64 oracle (device / float32 oracle): "
          + ", ".join(f"{t} {d:.2e} / {o:.2e}" for t, (d, o) in report.items())
          + f"; first inner step beyond 1e-5: device {first_dev}, float32 oracle {first_32}")
    for t, (d, o) in report.items():
        assert np.isfinite(d) and d <= max(30 * o, 1e-5), (t, d, o)


def test_config3_lenet_free_running_small_step(gpu):
    """The same workload free-running (no state push) at step size 0.01, where the dynamics do not
    amplify rounding: all 25 inner steps and the outer step, 1e-5 on every parameter tensor."""
    torch, pb = gpu
    P, O, loss, ref_loss = _cycle(pb, torch, onets.arch("lenet"), 6, 128, 25, 0, seed=0, eta_inner=0.01,
                                  eta_outer=0.01)
    got = P.state()
    for t in ("x", "y", "z", "x_ref"):
        check(t, got[t], getattr(O.st, t), 1e-5, max_factor=100)
    np.testing.assert_allclose(loss, ref_loss, rtol=1e-3, atol=2e-6)
    assert ref_loss[-1].mean() < ref_loss[0].mean()


@pytest.mark.parametrize("name", ["allcnn_vec", "wrn_vec", "lenet_vec"])
def test_reduced_bf16_cycles(gpu, name):
    """bf16 compute with fp32 master weights on reduced widths, two outer steps, scoping on."""
    torch, pb = gpu
    P, O, loss, ref_loss = _cycle(pb, torch, SMALL[name], 3, 32, 5, 1, seed=1, outer=2, scoping_B=4, gamma0=0.05,
                                  eta_inner=0.05)
    got = P.state()
    for t in ("x", "y", "z", "x_ref"):
        check(t, got[t], getattr(O.st, t), 2e-2)
    np.testing.assert_allclose(loss, ref_loss, rtol=2e-2)
    k, od, g, r = P.parle_get_state()
    assert (k, od) == (10, 2) and abs(g - O.st.g) < 1e-6 and abs(r - O.st.r) < 1e-6


# Per-segment bars (relative 2-norm error, cosine) for bf16 gradients at full size against the oracle in its bf16
# storage mode.  At this size some fp32 sum always lands on the other side of a bf16 rounding boundary than the
# exact sum, and from there on the two computations round differently (tests/test_oracle_chaos.py): what is left is
# the agreement that two correct bf16 implementations have.  Measured worst segments: All-CNN-C 1.5e-2 / 0.9999
# (whole gradient 2e-3); WRN-16-4 0.23 / 0.974 (whole gradient 8-10 %: thirteen batch-norms whose backward pass
# subtracts means); WRN-28-10 at batch 4 0.36 / 0.935.  A zero, a mis-scaled or a mis-routed gradient of any segment
# fails every one of these.
BF16_SEG = {"allcnn": (4e-2, 0.999), "wrn": (0.4, 0.93), "wrn28": (0.6, 0.85)}


@pytest.mark.parametrize("model", ["allcnn", "wrn"])
def test_config4_config5_full_size_step(gpu, model):
    """n = 3 replicas of All-CNN-C / WRN-16-4 at full size (batch 128, 3x32x32), bf16 compute with
    fp32 master weights: one inner step and the outer step (scoping on for WRN).  The oracle runs
    in its float32 mode here (its float64 mode needs minutes at this size; the bar is 2e-2), with
    activations kept on the bf16 grid as on the device.

    One step moves the parameters by far less than 2e-2 of their size, so the parameters themselves cannot
    fail that bar; what is held to the oracle is the MOVE: the gradient of every parameter segment of every
    replica (relative 2-norm and cosine), and the displacements y - x_0, z - x_0 and x - x_0 per segment."""
    torch, pb = gpu
    a, n, B = onets.arch(model), 3, 128
    kw = dict(scoping_B=390) if model == "wrn" else {}
    P, O = make(pb, a, n, B, bf16=1, seed=0, oracle_dtype=np.float32, storage="bf16", **kw)
    x0 = O.st.x.astype(np.float64).copy()
    lay = onets.layout(a)
    BF16_SEG_REL, BF16_SEG_COS = BF16_SEG[model]
    X, Y = synth.image_batches(0, 1, n, B, a["H"], a["W"], a["C"], a["classes"])
    loss = torch.zeros(n, dtype=torch.float32, device="cuda")
    P.parle_inner_step(dev(torch, X[0]), dev(torch, Y[0]), loss)
    ref_loss = O.inner_step(X[0], Y[0])
    got = P.state()
    np.testing.assert_allclose(loss.cpu().numpy(), ref_loss, rtol=2e-2)
    worst = ("", 0.0, 1.0)
    for r in range(n):
        for name, err, cos in segment_errors(lay, got["grad"][r], O.last_grad[r]):
            if err > worst[1]:
                worst = (f"{name}[{r}]", err, cos)
            assert err <= BF16_SEG_REL and cos >= BF16_SEG_COS, (model, r, name, err, cos)
    print(f"{model}: worst gradient segment {worst[0]}: rel {worst[1]:.3e}, cos {worst[2]:.5f}")
    for t in ("y", "z"):
        for name, err, cos in segment_errors(lay, got[t] - x0, getattr(O.st, t) - x0):
            assert err <= BF16_SEG_REL and cos >= BF16_SEG_COS, (model, t, name, err, cos)
    P.parle_outer_step()
    O.outer_step()
    got = P.state()
    for t in ("x", "y", "z", "x_ref"):
        check(t, got[t], getattr(O.st, t), 2e-2)
    for name, err, cos in segment_errors(lay, got["x"] - x0, O.st.x - x0):
        assert err <= BF16_SEG_REL and cos >= BF16_SEG_COS, (model, "x", name, err, cos)
    k, od, g, r = P.parle_get_state()
    assert (k, od) == (1, 1) and abs(g - O.st.g) <= 1e-6 * O.st.g and abs(r - O.st.r) <= 1e-6 * O.st.r
    if model == "wrn":
        stats = P.bn_stats.cpu().numpy().reshape(n, -1)
        for rr in range(n):
            ref = np.concatenate([np.concatenate(O.bn[rr][nm]) for nm, _ in onets.bn_layers(a)])
            check("bn running stats", stats[rr], ref, 2e-2)


@pytest.mark.parametrize("name,bf16", [("lenet_odd", 0), ("wrn_vec", 0), ("wrn_odd", 1), ("allcnn_vec", 1)])
def test_eval_matches_oracle(gpu, name, bf16):
    torch, pb = gpu
    a = SMALL[name]
    n, B, L = 2, 8, 3
    P, O, _, _ = _cycle(pb, torch, a, n, B, L, bf16, seed=2, distinct_init=True)
    X, Y = synth.image_batches(9, 1, 1, 13, a["H"], a["W"], a["C"], a["classes"])
    tol = 1e-4 if not bf16 else 3e-2
    for which in (-1, 0, 1):
        loss, nerr, sp = P.parle_eval(which, dev(torch, X[0, 0]), dev(torch, Y[0, 0]))
        rl, rn, rsp = O.eval(which, X[0, 0], Y[0, 0])
        assert abs(loss - rl) <= tol * abs(rl), (which, loss, rl)
        assert abs(sp - rsp) <= 1e-4 * rsp + 1e-12
        if not bf16:
            assert nerr == rn
        else:
            assert abs(nerr - rn) <= 2
    if a["model"] == "wrn":
        # running statistics of every BN layer (per replica)
        got = P.bn_stats.cpu().numpy().reshape(n, -1)
        for r in range(n):
            ref = np.concatenate([np.concatenate(O.bn[r][name_]) for name_, _ in onets.bn_layers(a)])
            check("bn running stats", got[r], ref, 1e-4 if not bf16 else 2e-2)


def test_eval_reports_a_non_finite_loss_and_the_context_stays_usable(gpu):
    torch, pb = gpu
    a = SMALL["mlp_vec"]
    P, O = make(pb, a, 2, 8, seed=4)
    X, Y = synth.image_batches(9, 1, 1, 8, a["H"], a["W"], a["C"], a["classes"])
    xd, yd = dev(torch, X[0, 0]), dev(torch, Y[0, 0])
    good = P.parle_eval(1, xd, yd)
    at = pb.parle_query_layout(P.cfg)[-1]["offset"]      # a bias of the last layer: it reaches the logits directly
    kept = float(P.x[1, at])
    P.x[1, at] = float("nan")
    torch.cuda.synchronize()
    with pytest.raises(pb.ParleError) as e:
        P.parle_eval(1, xd, yd)
    assert e.value.status == pb.PARLE_ENONFINITE and "finite" in str(e.value)
    # the other replica is untouched, and the poisoned one evaluates as before once the value is back
    loss0, _, _ = P.parle_eval(0, xd, yd, want_spread=False)
    assert np.isfinite(loss0)
    P.x[1, at] = kept
    torch.cuda.synchronize()
    assert P.parle_eval(1, xd, yd) == good


# ---------------------------------------------------------------------------------------------
# Elastic-SGD (Section 2.2) on networks, and blocks of inner steps replayed from a HIP graph
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name,bf16,tol", [("mlp_vec", 0, 1e-5), ("wrn_vec", 1, 2e-2)])
def test_elastic_sgd_on_networks(gpu, name, bf16, tol):
    torch, pb = gpu
    # bf16 gradients agree with exact arithmetic only in direction (see test_one_step_loss_and_gradient), and with
    # no proximal term pulling the iterate back the difference adds up step by step: fewer, smaller steps there
    a, n, B = SMALL[name], 3, 16
    steps, every, eta = (4, 2, 0.02) if bf16 else (8, 4, 0.05)
    model, arch = model_pair(pb, a)
    base = dict(n_replicas=n, L=every, eta_inner=eta, eta_outer=0.05, momentum=0.9, rho0=1.0, scoping_B=3)
    cfg = pb.make_config(model=model, batch=B, compute_bf16=bf16, in_h=a["H"], in_w=a["W"], in_c=a["C"],
                         n_classes=a["classes"], arch=arch, algorithm=pb.ALG_ELASTIC, **base)
    lay = pb.parle_query_layout(cfg)
    wi = "uniform" if a["model"] in ("mlp", "lenet") else "he_normal"
    x0 = np.stack([synth.init_params(lay, 5 + 17 * i, wi) for i in range(n)])
    P = pb.Parle(cfg, x0)
    O = otrainer.ElasticNet(a, oparle.ParleConfig(**base), x0)
    X, Y = synth.image_batches(4, steps, n, B, a["H"], a["W"], a["C"], a["classes"])
    dX, dY = dev(torch, X), dev(torch, Y)
    loss = torch.zeros((steps, n), dtype=torch.float32, device="cuda")
    ref_loss = np.zeros((steps, n))
    for k in range(steps):
        P.parle_inner_step(dX[k], dY[k], loss[k])
        ref_loss[k] = O.step(X[k], Y[k])
        if (k + 1) % every == 0:
            P.parle_outer_step()
            O.scope()
    got = P.state()
    check("xa", got["y"], O.st.xa, tol)
    check("x", got["x_ref"], O.st.x, tol)
    if not bf16:
        check("v", got["vy"], O.st.v, 1e-4)
    np.testing.assert_allclose(loss.cpu().numpy(), ref_loss, rtol=max(tol, 1e-4), atol=2e-6)
    Xe, Ye = synth.image_batches(9, 1, 1, 11, a["H"], a["W"], a["C"], a["classes"])
    for which in (-1, 1):
        l, nerr, sp = P.parle_eval(which, dev(torch, Xe[0, 0]), dev(torch, Ye[0, 0]))
        rl, rn, rsp = O.eval(which, Xe[0, 0], Ye[0, 0])
        assert abs(l - rl) <= max(tol, 1e-4) * 2 * abs(rl) and abs(sp - rsp) <= max(tol, 1e-4) * 2 * rsp


@pytest.mark.parametrize("name,bf16,alg", [("lenet_vec", 0, 0), ("wrn_vec", 1, 0), ("mlp_vec", 0, 1)])
def test_inner_block_graph_replays_equal_step_by_step(gpu, name, bf16, alg):
    """A block of inner steps through parle_inner_block with graph_block = 1: first call step by step,
    second call records and replays, later calls replay.  Every block is compared bit for bit with a
    second context that runs parle_inner_step; outer steps (eager kernels, scoping that changes the
    multipliers the captured launches read) and synchronisations sit between the replays."""
    torch, pb = gpu
    a, n, B, L, blocks = SMALL[name], 2, 8, 4, 5
    model, arch = model_pair(pb, a)
    base = dict(n_replicas=n, L=L, eta_inner=0.05, eta_outer=0.1, momentum=0.9, gamma0=0.03, rho0=1.0, scoping_B=2,
                algorithm=alg)
    mk = lambda graph: pb.make_config(model=model, batch=B, compute_bf16=bf16, in_h=a["H"], in_w=a["W"], in_c=a["C"],
                                      n_classes=a["classes"], arch=arch, graph_block=graph, **base)
    lay = pb.parle_query_layout(mk(0))
    wi = "uniform" if a["model"] in ("mlp", "lenet") else "he_normal"
    x0 = np.tile(synth.init_params(lay, 2, wi), (n, 1))
    Pg, Ps = pb.Parle(mk(1), x0), pb.Parle(mk(0), x0)
    X, Y = synth.image_batches(6, L, n, B, a["H"], a["W"], a["C"], a["classes"])
    dX, dY = dev(torch, X), dev(torch, Y)
    loss_g = torch.zeros((L, n), dtype=torch.float32, device="cuda")
    loss_s = torch.zeros((L, n), dtype=torch.float32, device="cuda")
    for b in range(blocks):
        Pg.parle_inner_block(dX, dY, loss_g)
        for k in range(L):
            Ps.parle_inner_step(dX[k], dY[k], loss_s[k])
        sg, ss = Pg.state(), Ps.state()
        for t in ("y", "z", "vy", "grad", "x_ref"):
            assert np.array_equal(sg[t], ss[t]), (b, t)
        assert np.array_equal(loss_g.cpu().numpy(), loss_s.cpu().numpy()), b
        loss_g.zero_()
        Pg.parle_outer_step()
        Ps.parle_outer_step()
        assert Pg.parle_get_state() == Ps.parle_get_state()
        sg, ss = Pg.state(), Ps.state()
        for t in ("x", "y", "z", "vx", "x_ref"):
            assert np.array_equal(sg[t], ss[t]), (b, "outer", t)
    # other arguments: step by step again, and remembered in place of the old ones
    Pg.parle_inner_block(dX[:2].contiguous(), dY[:2].contiguous(), None)
    for k in range(2):
        Ps.parle_inner_step(dX[k], dY[k], None)
    assert np.array_equal(Pg.state()["y"], Ps.state()["y"])
    assert Pg.parle_get_state()[0] == blocks * L + 2


def test_wrn_28_10_one_step_reduced_batch(gpu):
    """WRN-28-10 (Section 4.3, 36.5 million weights) as arch = (16, 10, 4): one inner step and the outer step for one
    replica on a batch of 4 (the oracle needs seconds), bf16 compute with fp32 master weights."""
    torch, pb = gpu
    a, n, B = onets.arch("wrn", widen=10, nb=4), 1, 4
    P, O = make(pb, a, n, B, bf16=1, seed=0, oracle_dtype=np.float32, storage="bf16")
    BF16_SEG_REL, BF16_SEG_COS = BF16_SEG["wrn28"]
    assert abs(P.sizes.n_params / 1e6 - 36.5) < 0.1
    X, Y = synth.image_batches(0, 1, n, B, a["H"], a["W"], a["C"], a["classes"])
    loss = torch.zeros(n, dtype=torch.float32, device="cuda")
    P.parle_inner_step(dev(torch, X[0]), dev(torch, Y[0]), loss)
    ref_loss = O.inner_step(X[0], Y[0])
    np.testing.assert_allclose(loss.cpu().numpy(), ref_loss, rtol=2e-2)
    got = P.state()
    g, ref = got["grad"][0].astype(np.float64), O.last_grad[0].astype(np.float64)
    cos = (g * ref).sum() / np.sqrt((g * g).sum() * (ref * ref).sum())
    assert cos >= 0.9 and abs(np.linalg.norm(g) / np.linalg.norm(ref) - 1) <= 0.1, cos
    for name, err, cos in segment_errors(onets.layout(a), g, ref):
        assert err <= BF16_SEG_REL and cos >= BF16_SEG_COS, (name, err, cos)
    P.parle_outer_step()
    O.outer_step()
    got = P.state()
    for t in ("x", "y", "z", "x_ref"):
        check(t, got[t], getattr(O.st, t), 2e-2)
    # evaluation at the reference: 17 952 running statistics per replica are averaged into the workspace
    Xe, Ye = synth.image_batches(3, 1, 1, 4, a["H"], a["W"], a["C"], a["classes"])
    for which in (-1, 0):
        el, en, _ = P.parle_eval(which, dev(torch, Xe[0, 0]), dev(torch, Ye[0, 0]))
        rl, rn, _ = O.eval(which, Xe[0, 0], Ye[0, 0])
        assert abs(el - rl) <= 3e-2 * abs(rl) and abs(en - rn) <= 1, (which, el, rl, en, rn)


# ---------------------------------------------------------------------------------------------
# dropout (Section 4 rates) and LeNet with batch-norm (Section 4.2)
# ---------------------------------------------------------------------------------------------
DROP = {
    "lenet_bn": (onets.arch("lenet", H=20, W=20, C=1, c1=8, c2=16, k=5, fc=40, classes=10, bn=1), 0.25),
    "lenet": (SMALL["lenet_vec"], 0.25),
    "allcnn": (SMALL["allcnn_vec"], 0.5),
    "wrn": (SMALL["wrn_vec"], 0.3),
}


@pytest.mark.parametrize("name", list(DROP))
def test_dropout_one_step_fp32(gpu, name):
    """Same keep-masks on both sides (they are a function of seed, step, replica, site and element index):
    loss, gradient and the updated state of one step agree as without dropout; the step counter keys the
    mask, so the case starts from a restored state with k = 7."""
    torch, pb = gpu
    a, p = DROP[name]
    n, B = 2, 9
    P, O = make(pb, a, n, B, bf16=0, seed=3, distinct_init=True, dropout=p, dropout_seed=1234)
    P.parle_set_state(7, 0, 0.03, 1.0)
    O.st.k = 7
    X, Y = synth.image_batches(5, 2, n, B, a["H"], a["W"], a["C"], a["classes"])
    loss = torch.zeros(n, dtype=torch.float32, device="cuda")
    for k in range(2):
        P.parle_inner_step(dev(torch, X[k]), dev(torch, Y[k]), loss)
        ref_loss = O.inner_step(X[k], Y[k])
        np.testing.assert_allclose(loss.cpu().numpy(), ref_loss, rtol=1e-5)
        got = P.state()
        for r in range(n):
            check(f"{name} grad[{r}] step {k}", got["grad"][r], O.last_grad[r], 1e-4)
        for t in ("y", "z", "vy"):
            check(f"{name} {t}", got[t], getattr(O.st, t), 1e-5)
    # dropout really is on: the same loss without it is another number
    l_on = onets.loss_and_grad(a, O.st.y[0], X[0][0], Y[0][0], bn_state=onets.new_bn_state(a),
                               drop=dict(p=p, seed=1234, step=0, replica=0))[0]
    l_off = onets.loss_and_grad(a, O.st.y[0], X[0][0], Y[0][0], bn_state=onets.new_bn_state(a))[0]
    assert abs(l_on - l_off) > 1e-6
    # evaluation applies no dropout
    Xe, Ye = synth.image_batches(9, 1, 1, 11, a["H"], a["W"], a["C"], a["classes"])
    for which in (-1, 0):
        l, nerr, _ = P.parle_eval(which, dev(torch, Xe[0, 0]), dev(torch, Ye[0, 0]))
        rl, rn, _ = O.eval(which, Xe[0, 0], Ye[0, 0])
        assert abs(l - rl) <= 1e-4 * abs(rl) and nerr == rn


@pytest.mark.parametrize("name", ["lenet_bn", "allcnn", "wrn"])
def test_dropout_bf16_cycle_and_graph_replay(gpu, name):
    """bf16 compute with dropout through a block of inner steps replayed from a HIP graph (the masks read the
    step counter from device memory, so every replay draws new masks) against the oracle."""
    torch, pb = gpu
    a, p = DROP[name]
    n, B, L, blocks = 2, 16, 3, 3
    P, O = make(pb, a, n, B, bf16=1, seed=1, L=L, dropout=p, dropout_seed=77, eta_inner=0.02, graph_block=1)
    X, Y = synth.image_batches(1, L, n, B, a["H"], a["W"], a["C"], a["classes"])
    dX, dY = dev(torch, X), dev(torch, Y)
    loss = torch.zeros((L, n), dtype=torch.float32, device="cuda")
    for b in range(blocks):                        # step by step, then record + replay, then replay
        P.parle_inner_block(dX, dY, loss)
        ref = np.stack([O.inner_step(X[k], Y[k]) for k in range(L)])
        np.testing.assert_allclose(loss.cpu().numpy(), ref, rtol=3e-2)
        P.parle_outer_step()
        O.outer_step()
    got = P.state()
    for t in ("x", "y", "z", "x_ref"):
        check(t, got[t], getattr(O.st, t), 2e-2)
    assert P.parle_get_state()[0] == blocks * L


@pytest.mark.parametrize("n,fraction,alg", [(3, 0.5, "parle"), (6, 0.25, "parle"), (3, 0.5, "elastic")])
def test_split_data_between_replicas(gpu, n, fraction, alg):
    """Section 5: every replica draws its mini-batches from its own subset of one data set (50 % each for three
    replicas, 25 % each for six), All-CNN with dropout 0.5 and weight decay 1e-3, Parle and Elastic-SGD.  The
    library sees nothing but per-replica batch tensors, so the bar is the usual one against the oracle.

    With 8 images per batch one ReLU input that rounds to the other side of zero in fp32 moves a filter's
    gradient by a part in a few hundred (the mask is a step function), so the seeded inputs are chosen,
    and checked through the oracle, to keep every ReLU input further from zero than fp32 rounding reaches."""
    torch, pb = gpu
    a, B, L, outer = SMALL["allcnn_odd"], 8, 3, 2
    X, Y, idx, shards = synth.split_image_batches(30, L * outer, n, B, a["H"], a["W"], a["C"], 96, fraction,
                                                  a["classes"])
    for r in range(n):
        assert np.isin(idx[:, r], shards[r]).all()
    dX, dY = dev(torch, X), dev(torch, Y)
    loss = torch.zeros((L * outer, n), dtype=torch.float32, device="cuda")
    ref_loss = np.zeros((L * outer, n))
    kw = dict(L=L, dropout=0.5, dropout_seed=5, weight_decay=1e-3, eta_inner=0.05, eta_outer=0.05, scoping_B=4)
    if alg == "parle":
        P, O = make(pb, a, n, B, bf16=0, seed=3, distinct_init=True, **kw)
        step, sync = O.inner_step, O.outer_step
    else:
        model, arch = model_pair(pb, a)
        base = dict(n_replicas=n, momentum=0.9, rho0=1.0, **kw)
        cfg = pb.make_config(model=model, batch=B, compute_bf16=0, in_h=a["H"], in_w=a["W"], in_c=a["C"],
                             n_classes=a["classes"], arch=arch, algorithm=pb.ALG_ELASTIC, **base)
        x0 = np.stack([synth.init_params(pb.parle_query_layout(cfg), 3 + 17 * i, "he_normal") for i in range(n)])
        P, O = pb.Parle(cfg, x0), otrainer.ElasticNet(a, oparle.ParleConfig(**base), x0)
        step, sync = O.step, O.scope
    for k in range(L * outer):
        P.parle_inner_step(dX[k], dY[k], loss[k])
        ref_loss[k] = step(X[k], Y[k])
        if (k + 1) % L == 0:
            P.parle_outer_step()
            sync()
    got = P.state()
    assert O.relu_margin > 2e-6, O.relu_margin
    np.testing.assert_allclose(loss.cpu().numpy(), ref_loss, rtol=1e-4, atol=2e-6)
    if alg == "parle":
        for t in ("x", "y", "z", "vy", "x_ref"):
            check(t, got[t], getattr(O.st, t), 1e-5)
    else:
        check("xa", got["y"], O.st.xa, 1e-5)
        check("x", got["x_ref"], O.st.x, 1e-5)


@pytest.mark.parametrize("name,bf16", [("allcnn_vec", 1), ("wrn_vec", 0)])
def test_second_stream_changes_nothing(gpu, name, bf16, monkeypatch):
    """Weight and bias gradients run on a second stream beside the input-gradient chain; switching that off
    (one stream) must give the same bits: same kernels, same fixed-order reductions, only their timing differs."""
    torch, pb = gpu
    a, n, B, L = SMALL[name], 3, 16, 3
    X, Y = synth.image_batches(2, L, n, B, a["H"], a["W"], a["C"], a["classes"])
    dX, dY = dev(torch, X), dev(torch, Y)
    states = []
    for overlap in ("1", "0"):
        monkeypatch.setenv("PARLE_OVERLAP_WGRAD", overlap)      # read when the context is created
        P, _ = make(pb, a, n, B, bf16=bf16, seed=4, distinct_init=True, L=L)
        loss = torch.zeros((L, n), dtype=torch.float32, device="cuda")
        for k in range(L):
            P.parle_inner_step(dX[k], dY[k], loss[k])
        P.parle_outer_step()
        got = P.state()
        states.append((loss.cpu().numpy(), got["grad"], got["y"], got["x"]))
        P.close()
    for u, v in zip(*states):
        np.testing.assert_array_equal(u, v)


@pytest.mark.parametrize("model", ["allcnn", "wrn"])
def test_full_size_streams_change_nothing(gpu, model, monkeypatch):
    """Full-size layers switch on what the reduced networks do not reach (bias gradients on a third stream in
    All-CNN-C, the kernels chosen for 128 x 32 x 32 batches): two inner steps and an outer step with the extra
    streams must give the bits of the same steps on one stream."""
    torch, pb = gpu
    a, n, B, L = onets.arch(model), 3, 128, 2
    mdl, arch = model_pair(pb, a)
    cfg = pb.make_config(model=mdl, n_replicas=n, batch=B, L=L, compute_bf16=1, in_h=a["H"], in_w=a["W"], in_c=a["C"],
                         n_classes=a["classes"], arch=arch, eta_inner=0.01, eta_outer=0.01, gamma0=0.03, rho0=1.0,
                         fuse_outer=1, graph_block=0)
    x0 = np.tile(synth.init_params(pb.parle_query_layout(cfg), 0, "he_normal"), (n, 1))
    X, Y = synth.image_batches(1, L, n, B, a["H"], a["W"], a["C"], a["classes"])
    dX, dY = dev(torch, X), dev(torch, Y)
    states = []
    for overlap in ("1", "0"):
        monkeypatch.setenv("PARLE_OVERLAP_WGRAD", overlap)      # read when the context is created
        P = pb.Parle(cfg, x0)
        loss = torch.zeros((L, n), dtype=torch.float32, device="cuda")
        for k in range(L):
            P.parle_inner_step(dX[k], dY[k], loss[k])
        P.parle_outer_step()
        torch.cuda.synchronize()
        states.append([loss.clone()] + [getattr(P, t).clone() for t in ("grad", "y", "x", "x_ref")])
        P.close()
    for u, v in zip(*states):
        assert torch.equal(u, v)
    assert np.isfinite(states[0][0].cpu().numpy()).all()


@pytest.mark.parametrize("model", ["allcnn", "wrn"])
def test_full_size_first_layer_reading_fp32_images_changes_nothing(gpu, model, monkeypatch):
    """In bf16 mode the first layer's kernels gather the caller's fp32 images and round each value as they gather it;
    with that switched off a copy kernel rounds the images first.  Same values either way: two inner steps and an
    outer step must give the same bits."""
    torch, pb = gpu
    a, n, B, L = onets.arch(model), 3, 128, 2
    mdl, arch = model_pair(pb, a)
    cfg = pb.make_config(model=mdl, n_replicas=n, batch=B, L=L, compute_bf16=1, in_h=a["H"], in_w=a["W"], in_c=a["C"],
                         n_classes=a["classes"], arch=arch, eta_inner=0.01, eta_outer=0.01, gamma0=0.03, rho0=1.0,
                         fuse_outer=1, graph_block=0)
    x0 = np.tile(synth.init_params(pb.parle_query_layout(cfg), 0, "he_normal"), (n, 1))
    X, Y = synth.image_batches(1, L, n, B, a["H"], a["W"], a["C"], a["classes"])
    dX, dY = dev(torch, X), dev(torch, Y)
    states = []
    for direct in ("1", "0"):
        monkeypatch.setenv("PARLE_IMAGES_DIRECT", direct)      # read when the context is created
        P = pb.Parle(cfg, x0)
        loss = torch.zeros((L, n), dtype=torch.float32, device="cuda")
        for k in range(L):
            P.parle_inner_step(dX[k], dY[k], loss[k])
        P.parle_outer_step()
        ev = P.parle_eval(-1, dX[0, 0], dY[0, 0])
        torch.cuda.synchronize()
        states.append([loss.clone()] + [getattr(P, t).clone() for t in ("grad", "y", "x", "x_ref")] +
                      [torch.tensor([float(v) for v in ev[:2]])])
        P.close()
    for u, v in zip(*states):
        assert torch.equal(u, v)
    assert np.isfinite(states[0][0].cpu().numpy()).all()


@pytest.mark.parametrize("model,bf16", [("allcnn", 1), ("lenet", 0), ("mlp", 0)])
def test_full_size_bias_gradient_inside_the_weight_gradient_kernels(gpu, model, bf16, monkeypatch):
    """The weight-gradient kernels take a layer's bias gradient (the column sums of dy) along; switched off, the
    column-sum kernels compute it.  Same inputs, two orders of fp32 additions: after one inner step every segment of
    the gradient agrees to 2e-6 of its norm (a dropped row, tile or split would show as 1e-3 or more)."""
    torch, pb = gpu
    a = onets.arch(model)
    n, B = (6 if model == "lenet" else 3), 128
    mdl, arch = model_pair(pb, a)
    cfg = pb.make_config(model=mdl, n_replicas=n, batch=B, L=1, compute_bf16=bf16, in_h=a["H"], in_w=a["W"],
                         in_c=a["C"], n_classes=a["classes"], arch=arch, eta_inner=0.01, eta_outer=0.01, gamma0=0.03,
                         rho0=1.0, fuse_outer=1, graph_block=0)
    layout = pb.parle_query_layout(cfg)
    x0 = np.tile(synth.init_params(layout, 0, "he_normal" if bf16 else "uniform"), (n, 1))
    X, Y = synth.image_batches(3, 1, n, B, a["H"], a["W"], a["C"], a["classes"])
    dX, dY = dev(torch, X), dev(torch, Y)
    grads = []
    for inside in ("1", "0"):
        monkeypatch.setenv("PARLE_BIAS_IN_WGRAD", inside)      # read when the context is created
        P = pb.Parle(cfg, x0)
        loss = torch.zeros((1, n), dtype=torch.float32, device="cuda")
        P.parle_inner_step(dX[0], dY[0], loss[0])
        torch.cuda.synchronize()
        grads.append(P.grad.cpu().numpy()[:, :P.sizes.n_params])
        P.close()
    assert any(s["kind"] == "bias" for s in layout)
    worst = max(e for _, e, _ in segment_errors(layout, grads[0], grads[1]))
    assert 0 < np.abs(grads[1]).max() < np.inf
    assert worst <= 2e-6, segment_errors(layout, grads[0], grads[1])


@pytest.mark.parametrize("model", ["allcnn", "wrn"])
def test_full_size_blocks_from_the_graph_equal_step_by_step(gpu, model):
    """The launch configuration that bench.py times (n = 3, batch 128, 3x32x32, bf16 compute, blocks of L = 25
    inner steps replayed from a HIP graph, fused outer step, scoping on for WRN) against a second context that
    enqueues every step: bit for bit, over a step-by-step block, the recording block and a replayed one.
    (The step-by-step path is the one test_config4_config5_full_size_step holds against the oracle.)"""
    torch, pb = gpu
    a, n, B, L, blocks = onets.arch(model), 3, 128, 25, 3
    mdl, arch = model_pair(pb, a)
    mk = lambda graph: pb.make_config(model=mdl, n_replicas=n, batch=B, L=L, compute_bf16=1, in_h=a["H"], in_w=a["W"],
                                      in_c=a["C"], n_classes=a["classes"], arch=arch, eta_inner=0.01, eta_outer=0.01,
                                      gamma0=0.03, rho0=1.0, fuse_outer=1, scoping_B=390 if model == "wrn" else 0,
                                      graph_block=graph)
    x0 = np.tile(synth.init_params(pb.parle_query_layout(mk(0)), 0, "he_normal"), (n, 1))
    Pg, Ps = pb.Parle(mk(1), x0), pb.Parle(mk(0), x0)
    X, Y = synth.image_batches(0, L, n, B, a["H"], a["W"], a["C"], a["classes"])
    dX, dY = dev(torch, X), dev(torch, Y)
    loss_g = torch.zeros((L, n), dtype=torch.float32, device="cuda")
    loss_s = torch.zeros((L, n), dtype=torch.float32, device="cuda")
    for b in range(blocks):
        Pg.parle_inner_block(dX, dY, loss_g)
        for k in range(L):
            Ps.parle_inner_step(dX[k], dY[k], loss_s[k])
        assert torch.equal(loss_g, loss_s), b
        assert np.isfinite(loss_g.cpu().numpy()).all()
        Pg.parle_outer_step()
        Ps.parle_outer_step()
        for t in ("x", "y", "z", "vy", "vx", "x_ref", "grad"):
            assert torch.equal(getattr(Pg, t), getattr(Ps, t)), (b, t)
        if model == "wrn":
            assert torch.equal(Pg.bn_stats, Ps.bn_stats), b
        loss_g.zero_()
    assert Pg.parle_get_state() == Ps.parle_get_state()
    assert Pg.parle_get_state()[0] == blocks * L
