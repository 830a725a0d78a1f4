"""GPU parity of the memory-bound Parle kernels against the CPU oracle (updates (8a)-(8d), rule (9)).

Tolerance: 1e-5 relative in the 2-norm per state tensor and 1e-5 * max|oracle| element-wise, the
bound the workload definition states for fp32 parameters.  The oracle runs in float64 on the same
float32 inputs.  The bf16 copy of y is an encoding: it must equal round-to-nearest-even of the
device's own fp32 y bit for bit.
"""
import numpy as np
import pytest

from oracle import parle as oparle
from paper_1707_00424_amd import synth

pytestmark = pytest.mark.gpu

TOL = 1e-5


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1707_00424_amd import binding as pb
    pb.lib()
    return torch, pb


def assert_close(name, got, ref, tol=TOL):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.isfinite(got).all(), name
    den = np.linalg.norm(ref)
    err = np.linalg.norm(got - ref)
    assert err <= tol * max(den, 1e-30) + 1e-30, f"{name}: rel 2-norm error {err / max(den, 1e-30):.3e}"
    mx = np.abs(got - ref).max() if got.size else 0.0
    assert mx <= tol * max(np.abs(ref).max(), 1e-30) + 1e-30, f"{name}: max abs error {mx:.3e}"


def bf16_rne_bits(a32):
    u = np.ascontiguousarray(a32, np.float32).view(np.uint32).astype(np.uint64)
    return (((u + 0x7FFF + ((u >> 16) & 1)) >> 16) & 0xFFFF).astype(np.uint16)


def _dev(torch, a, n_pad=None):
    t = torch.as_tensor(np.asarray(a, np.float32)).cuda()
    if n_pad is not None and t.shape[-1] != n_pad:
        out = torch.zeros(t.shape[:-1] + (n_pad,), dtype=torch.float32, device="cuda")
        out[..., :t.shape[-1]] = t
        return out
    return t.contiguous()


@pytest.mark.parametrize("n,N", [(1, 4), (3, 1000), (8, 70_001), (5, 262_144 + 4)])
@pytest.mark.parametrize("bf", [0, 1])
def test_inner_update_kernel(gpu, n, N, bf):
    torch, pb = gpu
    rng = np.random.default_rng(100 + n)
    n_pad = (N + 3) // 4 * 4
    G, x, y, vy, z = (rng.standard_normal((n, N)).astype(np.float32) * s for s in (1e-2, 0.05, 0.05, 0.02, 0.05))
    cfg = oparle.ParleConfig(n_replicas=n, eta_inner=0.1, momentum=0.9, alpha=0.75, weight_decay=5e-4, gamma0=0.03)
    st = oparle.ParleState(x=x.astype(np.float64), y=y.astype(np.float64), z=z.astype(np.float64),
                           vy=vy.astype(np.float64), vx=np.zeros((n, N)), x_ref=np.zeros(N), g=float(np.float32(0.03)))
    oparle.inner_update(st, G, cfg)
    dG, dx, dy, dvy, dz = (_dev(torch, a, n_pad) for a in (G, x, y, vy, z))
    d16 = torch.zeros((n, n_pad), dtype=torch.bfloat16, device="cuda") if bf else None
    pb.parle_k_inner_update(dG, dx, dy, dvy, dz, d16, 0.1, 0.9, 0.75, 5e-4, 0.03)
    torch.cuda.synchronize()
    assert_close("y", dy[:, :N].cpu().numpy(), st.y)
    assert_close("vy", dvy[:, :N].cpu().numpy(), st.vy)
    assert_close("z", dz[:, :N].cpu().numpy(), st.z)
    assert np.array_equal(dx[:, :N].cpu().numpy(), x) and np.array_equal(dG[:, :N].cpu().numpy(), G)
    if n_pad > N:
        assert not dy[:, N:].any() and not dz[:, N:].any() and not dvy[:, N:].any()
    if bf:
        got = d16.view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got, bf16_rne_bits(dy.cpu().numpy()))


@pytest.mark.parametrize("n,N", [(1, 8), (2, 1028), (3, 50_000), (8, 300_004), (11, 4096)])
def test_replica_mean_kernel(gpu, n, N):
    torch, pb = gpu
    x = synth.flat_params(7, n, N)
    dx = _dev(torch, x)
    dr = torch.full((N,), 7.0, dtype=torch.float32, device="cuda")
    pb.parle_k_replica_mean(dx, dr)
    torch.cuda.synchronize()
    assert_close("x_ref", dr.cpu().numpy(), oparle.replica_mean(x.astype(np.float64)), tol=1e-6)
    # identical replicas, n <= 2: the sum and the division are exact in fp32 too
    if n in (1, 2):
        same = _dev(torch, np.tile(x[0], (n, 1)))
        pb.parle_k_replica_mean(same, dr)
        torch.cuda.synchronize()
        assert np.array_equal(dr.cpu().numpy(), x[0])


@pytest.mark.parametrize("n,N", [(1, 16), (3, 10_000), (8, 131_076), (9, 2052)])
@pytest.mark.parametrize("mode", ["unfused", "fused", "lagged"])
@pytest.mark.parametrize("reset_flags,bf", [(3, 0), (0, 1), (1, 0)])
def test_outer_update_kernel(gpu, n, N, mode, reset_flags, bf):
    torch, pb = gpu
    rng = np.random.default_rng(200 + n)
    x, z, vx, y, vy = (rng.standard_normal((n, N)).astype(np.float32) * s for s in (0.05, 0.05, 0.01, 0.05, 0.02))
    stale = rng.standard_normal(N).astype(np.float32) * 0.05
    cfg = oparle.ParleConfig(n_replicas=n, eta_outer=0.1, momentum=0.9, gamma0=0.03, rho0=1.0, xa_mode=0,
                             xref_mode=1 if mode == "lagged" else 0, reset_flags=reset_flags)
    st = oparle.ParleState(x=x.astype(np.float64), y=y.astype(np.float64), z=z.astype(np.float64),
                           vy=vy.astype(np.float64), vx=vx.astype(np.float64), x_ref=stale.astype(np.float64),
                           g=float(np.float32(0.03)), r=1.0, inner_since_outer=1)
    oparle.outer_step(st, cfg)
    dx, dz, dvx, dy, dvy = (_dev(torch, a) for a in (x, z, vx, y, vy))
    dr = _dev(torch, stale)
    d16 = torch.zeros((n, N), dtype=torch.bfloat16, device="cuda") if bf else None
    if mode == "unfused":
        pb.parle_k_replica_mean(dx, dr)
    pb.parle_k_outer_update(dx, dz, dvx, dy, dvy, dr, d16, 0.1, 0.9, 0.03, 1.0, reset_flags,
                            fuse_mean=0 if mode == "unfused" else 1, lagged=1 if mode == "lagged" else 0)
    torch.cuda.synchronize()
    for name, t, ref in (("x", dx, st.x), ("z", dz, st.z), ("vx", dvx, st.vx), ("y", dy, st.y), ("vy", dvy, st.vy)):
        assert_close(name, t.cpu().numpy(), ref)
    assert_close("x_ref", dr.cpu().numpy(), st.x_ref)
    assert np.array_equal(dy.cpu().numpy(), dx.cpu().numpy())
    if bf:
        assert np.array_equal(d16.view(torch.int16).cpu().numpy().view(np.uint16), bf16_rne_bits(dx.cpu().numpy()))


def test_spread_kernel(gpu):
    torch, pb = gpu
    for n, N in [(1, 4), (3, 1000), (8, 1_000_004)]:
        x = synth.flat_params(9, n, N)
        ref = synth.flat_params(10, 1, N)[0]
        partial = torch.zeros(4096, dtype=torch.float64, device="cuda")
        out = torch.zeros(1, dtype=torch.float32, device="cuda")
        pb.parle_k_spread(_dev(torch, x), _dev(torch, ref), partial, out)
        torch.cuda.synchronize()
        want = float(((x.astype(np.float64) - ref.astype(np.float64)) ** 2).sum())
        assert abs(out.item() - want) <= 2e-6 * want


def _run_flat(pb, torch, n, N, inner, outer_every, seed, **cfgkw):
    """Same seeded inputs through the library (C ABI) and the oracle."""
    x0 = synth.flat_params(seed, n, N)
    base = dict(n_replicas=n, L=outer_every, eta_inner=0.1, eta_outer=0.1, momentum=0.9, alpha=0.75, gamma0=0.03,
                rho0=1.0)
    base.update(cfgkw)
    ocfg = oparle.ParleConfig(**{k: v for k, v in base.items() if k != "fuse_outer"})
    st = oparle.init_state(x0, ocfg)
    P = pb.Parle(pb.make_config(model=pb.MODEL_FLAT, n_params=N, **base), x0)
    for k in range(inner):
        G = synth.flat_grads(seed, k, n, N)
        P.grad[:, :N].copy_(torch.as_tensor(G))
        P.parle_inner_step()
        oparle.inner_update(st, G, ocfg)
        if (k + 1) % outer_every == 0:
            P.parle_outer_step()
            oparle.outer_step(st, ocfg)
    return P, st


@pytest.mark.parametrize("fuse", [0, 1])
def test_flat_workload_reduced_size_all_104_steps(gpu, fuse):
    """The update-only workload (n = 8, 100 inner + 4 outer updates) at a reduced odd length."""
    torch, pb = gpu
    P, st = _run_flat(pb, torch, 8, 250_003, 100, 25, seed=0, fuse_outer=fuse)
    got = P.state()
    for name in ("x", "y", "z", "vy", "vx"):
        assert_close(name, got[name], getattr(st, name))
    assert_close("x_ref", got["x_ref"], st.x_ref)
    assert P.parle_get_state()[:2] == (100, 4)
    _, _, sp = P.parle_eval()
    assert abs(sp - oparle.spread(st)) <= 1e-5 * oparle.spread(st)
    N, n_pad = P.sizes.n_params, P.sizes.n_pad
    assert n_pad > N and not P.y[:, N:].any() and not P.x[:, N:].any() and not P.x_ref[N:].any()


def test_flat_scoping_and_modes(gpu):
    torch, pb = gpu
    for kw in (dict(scoping_B=2, gamma0=0.01, rho0=1.0), dict(xa_mode=1), dict(xref_mode=1, fuse_outer=1),
               dict(reset_flags=0), dict(weight_decay=1e-3, momentum=0.0)):
        P, st = _run_flat(pb, torch, 3, 5_001, 12, 3, seed=3, **kw)
        got = P.state()
        for name in ("x", "y", "z", "vy", "vx"):
            assert_close(str(kw) + name, got[name], getattr(st, name))
        k, od, g, r = P.parle_get_state()
        assert (k, od) == (12, 4) and abs(g - st.g) <= 1e-6 * st.g and abs(r - st.r) <= 1e-6 * st.r


def test_flat_full_size_sampled_columns(gpu):
    """n = 8, N = 36.5M (the timed configuration): one inner and one outer update; the oracle
    recomputes a random sample of columns (the path is column-wise independent)."""
    torch, pb = gpu
    n, N = 8, 36_500_000
    cols = np.sort(np.random.default_rng(5).choice(N, 200_000, replace=False))
    cols = np.concatenate([[0, 1, 2, 3, N - 1, N - 2], cols])
    cfg = pb.make_config(model=pb.MODEL_FLAT, n_replicas=n, n_params=N, gamma0=0.03, rho0=1.0)
    gen = torch.Generator(device="cpu").manual_seed(11)
    x0 = (torch.randn((n, N), generator=gen) * 0.05)
    G = (torch.randn((n, N), generator=gen) * 1e-2)
    P = pb.Parle(cfg, x0.numpy())
    P.grad[:, :N].copy_(G)
    P.parle_inner_step()
    P.parle_outer_step()
    ocfg = oparle.ParleConfig(n_replicas=n, gamma0=0.03, rho0=1.0)
    # the reference needs whole columns only: the sample is a smaller instance of the same problem
    st = oparle.init_state(x0.numpy()[:, cols], ocfg)
    oparle.inner_update(st, G.numpy()[:, cols], ocfg)
    oparle.outer_step(st, ocfg)
    torch.cuda.synchronize()
    idx = torch.as_tensor(cols).cuda()
    for name in ("x", "y", "z", "vy", "vx"):
        assert_close(name, getattr(P, name)[:, idx].cpu().numpy(), getattr(st, name))
    assert_close("x_ref", P.x_ref[idx].cpu().numpy(), st.x_ref)


def test_determinism_and_fixed_point(gpu):
    torch, pb = gpu
    outs = []
    for _ in range(2):
        P, _ = _run_flat(pb, torch, 4, 10_000, 6, 3, seed=4)
        outs.append(P.state())
    for k in outs[0]:
        assert np.array_equal(outs[0][k], outs[1][k]), k
    # zero gradients and two identical replicas (their fp32 mean is exact): nothing may ever change
    row = synth.flat_params(6, 1, 3000)
    P = pb.Parle(pb.make_config(model=pb.MODEL_FLAT, n_replicas=2, n_params=3000, gamma0=0.03), np.tile(row, (2, 1)))
    for _ in range(2):
        for _ in range(3):
            P.parle_inner_step()
        P.parle_outer_step()
    s = P.state()
    for k in ("x", "y", "z"):
        assert np.array_equal(s[k], np.tile(row, (2, 1))), k
    assert np.array_equal(s["x_ref"], row[0]) and not s["vx"].any() and not s["vy"].any()


def test_call_order_and_argument_errors(gpu):
    torch, pb = gpu
    P = pb.Parle(pb.make_config(model=pb.MODEL_FLAT, n_replicas=2, n_params=100), np.zeros((2, 100), np.float32))
    with pytest.raises(pb.ParleError) as e:
        P.parle_outer_step()
    assert e.value.status == pb.PARLE_ESTATE and "inner step" in str(e.value)
    with pytest.raises(pb.ParleError) as e:
        P.parle_inner_step(images=P.x)
    assert e.value.status == pb.PARLE_EINVAL
    P.parle_inner_step()
    P.parle_outer_step()
    P.parle_set_state(50, 2, 0.5, 2.0)
    assert P.parle_get_state() == (50, 2, 0.5, 2.0)


# ---------------------------------------------------------------------------------------------
# Elastic-SGD (Section 2.2) with scoping on rho
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,N", [(1, 4), (3, 1000), (8, 70_004), (9, 2052)])
@pytest.mark.parametrize("bf", [0, 1])
def test_elastic_step_kernel(gpu, n, N, bf):
    from oracle import elastic as oel
    torch, pb = gpu
    rng = np.random.default_rng(300 + n)
    G, xa, v = (rng.standard_normal((n, N)).astype(np.float32) * s for s in (1e-2, 0.05, 0.02))
    ref = rng.standard_normal(N).astype(np.float32) * 0.05
    cfg = oparle.ParleConfig(n_replicas=n, eta_inner=0.1, eta_outer=0.05, momentum=0.9, weight_decay=5e-4, rho0=1.5)
    st = oel.ElasticState(xa=xa.astype(np.float64), v=v.astype(np.float64), x=ref.astype(np.float64), r=1.5)
    oel.step(st, G, cfg)
    dG, dxa, dv, dr = (_dev(torch, a) for a in (G, xa, v, ref))
    d16 = torch.zeros((n, N), dtype=torch.bfloat16, device="cuda") if bf else None
    pb.parle_k_elastic_step(dG, dxa, dv, dr, d16, 0.1, 0.05, 0.9, 5e-4, 1.5)
    torch.cuda.synchronize()
    assert_close("xa", dxa.cpu().numpy(), st.xa)
    assert_close("v", dv.cpu().numpy(), st.v)
    assert_close("x", dr.cpu().numpy(), st.x)
    assert np.array_equal(dG.cpu().numpy(), G)
    if bf:
        assert np.array_equal(d16.view(torch.int16).cpu().numpy().view(np.uint16), bf16_rne_bits(dxa.cpu().numpy()))


def test_elastic_flat_workload_with_scoping(gpu):
    """Elastic-SGD through the C ABI on the update-only inputs: 40 steps, rule (9) on rho every 5."""
    from oracle import elastic as oel
    torch, pb = gpu
    n, N, steps, every = 4, 30_001, 40, 5
    x0 = synth.flat_params(21, n, N)
    base = dict(n_replicas=n, L=every, eta_inner=0.1, eta_outer=0.1, momentum=0.9, rho0=1.0, scoping_B=3,
                weight_decay=1e-4)
    ocfg = oparle.ParleConfig(**base)
    st = oel.init_state(x0, ocfg)
    P = pb.Parle(pb.make_config(model=pb.MODEL_FLAT, n_params=N, algorithm=pb.ALG_ELASTIC, **base), x0)
    for k in range(steps):
        G = synth.flat_grads(21, k, n, N)
        P.grad[:, :N].copy_(torch.as_tensor(G))
        P.parle_inner_step()
        oel.step(st, G, ocfg)
        if (k + 1) % every == 0:
            P.parle_outer_step()
            oel.scope(st, ocfg)
    got = P.state()
    assert_close("xa", got["y"], st.xa)
    assert_close("v", got["vy"], st.v)
    assert_close("x", got["x_ref"], st.x)
    k, od, g, r = P.parle_get_state()
    assert (k, od) == (steps, steps // every) and abs(r - st.r) <= 1e-6 * st.r and st.r > 1.0
    _, _, sp = P.parle_eval()
    want = float(((st.xa - st.x) ** 2).sum())
    assert abs(sp - want) <= 1e-5 * want


def test_entropy_sgd_is_parle_with_one_replica(gpu):
    """n = 1, no elastic term: the device's (8a)-(8c) against Entropy-SGD written directly from (6a)-(6c)
    (Section 2.1) on f(x) = |x - c|^2 / 2 with exact gradients, printed-equation scaling (xa_mode = 1)."""
    torch, pb = gpu
    rng = np.random.default_rng(31)
    N, L, eta_p, eta, g, alpha = 1003, 5, 0.05, 0.7, 0.3, 0.75
    c, x0 = rng.standard_normal(N), rng.standard_normal(N)
    P = pb.Parle(pb.make_config(model=pb.MODEL_FLAT, n_replicas=1, n_params=N, L=L, eta_inner=eta_p, eta_outer=eta,
                                gamma0=g, rho0=0.0, momentum=0.0, alpha=alpha, xa_mode=1, fuse_outer=1),
                 x0[None].astype(np.float32))
    cd = torch.as_tensor(c.astype(np.float32)).cuda()
    x = x0.astype(np.float32).astype(np.float64)
    c64 = c.astype(np.float32).astype(np.float64)
    for _ in range(3):
        y, z = x.copy(), x.copy()
        for _ in range(L):
            P.grad[0, :N].copy_(P.y[0, :N] - cd)          # exact gradient of f at the device's y
            P.parle_inner_step()
            y = y - eta_p * ((y - c64) + g * (y - x))        # (6a) without the noise term, as the paper runs it
            z = alpha * z + (1 - alpha) * y                  # (6b)
        P.parle_outer_step()
        x_before = x
        x = x - eta * (x - z)                                # (6c)
        assert_close("x", P.state()["x"][0], x)
        assert_close("x_ref", P.state()["x_ref"], x_before)  # the mean is taken before the replica moves


@pytest.mark.parametrize("count", [4, 4 * 1023, 4 * (256 * 4 * 7 + 5)])
def test_stream_reference_kernel_moves_what_it_says(gpu, count):
    """The measurement aid: every array it claims to read reaches the result and every array it claims to
    write is written in full and nothing beyond (ragged tails, one to many blocks)."""
    torch, pb = gpu
    rng = np.random.default_rng(count)
    src = rng.standard_normal(5 * count).astype(np.float32)
    pattern = np.tile(np.array([1, 2, 3, 4], np.float32), count // 4)
    for r, w in [(1, 1), (5, 3), (0, 1), (1, 0)]:
        d_src = torch.as_tensor(src).cuda()
        d_dst = torch.full((3 * count + 8,), -7.0, dtype=torch.float32, device="cuda")
        pb.parle_k_stream_reference(r, w, count, d_src, d_dst)
        got = d_dst.cpu().numpy()
        want = pattern.copy()
        for i in range(r):                      # summed in array order, like the kernel
            want = want + src[i * count:(i + 1) * count]
        for j in range(w):
            np.testing.assert_array_equal(got[j * count:(j + 1) * count], want)
        assert (got[w * count:] == -7.0).all()
    with pytest.raises(pb.ParleError):
        pb.parle_k_stream_reference(2, 2, count, d_src, d_dst)
    with pytest.raises(pb.ParleError):
        pb.parle_k_stream_reference(1, 1, count + 2, d_src, d_dst)
