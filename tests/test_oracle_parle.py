"""Pins for oracle/parle.py against what the paper and the mathematics fix.

Each test names the passage it leans on.  None of them retypes the oracle's own
formula: they use closed forms, independently written short loops for the
algorithms the paper says Parle reduces to, invariants and brute force.
"""
import numpy as np
import pytest

from oracle import parle


def _cfg(n, **kw):
    base = dict(n_replicas=n, L=25, eta_inner=0.1, eta_outer=0.1, momentum=0.9, alpha=0.75,
                gamma0=0.03, rho0=1.0)
    base.update(kw)
    return parle.ParleConfig(**base)


def _quad_grad(y, c):
    """Gradient of f(y) = 0.5 ||y - c||^2."""
    return y - c


# ---- (8d) with eta'' = rho/n, Section 3.1: the reference is the replica average -------------------
def test_mean_closed_form_bruteforce():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 37))
    ref = np.array([sum(x[a, i] for a in range(5)) / 5 for i in range(37)])
    assert np.allclose(parle.replica_mean(x), ref, rtol=0, atol=1e-15)
    assert np.allclose(parle.replica_mean(x), np.mean(x, axis=0), rtol=0, atol=1e-15)


@pytest.mark.parametrize("n", [1, 2, 4, 8])
def test_mean_of_identical_replicas_is_exact(n):
    # float32-valued inputs widened to float64: sums of up to 8 of them and the division by a
    # power of two are exact, so the mean must return the row bit for bit
    row = np.random.default_rng(1).standard_normal(101).astype(np.float32).astype(np.float64)
    x = np.tile(row, (n, 1))
    assert np.array_equal(parle.replica_mean(x), row)


def test_mean_residuals_sum_to_zero():
    x = np.random.default_rng(2).standard_normal((6, 50))
    assert np.abs((x - parle.replica_mean(x)).sum(axis=0)).max() < 1e-14


# ---- (8a) with the proximal term off is Nesterov SGD on f; with mu = 0 plain SGD --------------------
def test_inner_reduces_to_plain_sgd():
    rng = np.random.default_rng(3)
    c, x0 = rng.standard_normal(20), rng.standard_normal((1, 20))
    cfg = _cfg(1, gamma0=0.0, rho0=0.0, momentum=0.0)
    st = parle.init_state(x0, cfg)
    y = x0[0].copy()
    for _ in range(7):
        parle.inner_update(st, _quad_grad(st.y, c), cfg)
        y = y - 0.1 * (y - c)                      # plain SGD, written here
        assert np.allclose(st.y[0], y, rtol=0, atol=1e-15)
    # closed form for the quadratic: y_k - c = 0.9^k (y_0 - c)
    assert np.allclose(st.y[0] - c, 0.9 ** 7 * (x0[0] - c), atol=1e-14)


def test_inner_nesterov_matches_lookahead_form():
    """Nesterov's method in its textbook two-sequence form (gradient taken at the look-ahead point):
    v_{k+1} = mu v_k - lr grad(th_k + mu v_k), th_{k+1} = th_k + v_{k+1}.  The parameters the
    framework-style form carries are the look-ahead points p_k = th_k + mu v_k."""
    rng = np.random.default_rng(4)
    c, x0 = rng.standard_normal(9), rng.standard_normal((1, 9))
    cfg = _cfg(1, gamma0=0.0, rho0=0.0)
    st = parle.init_state(x0, cfg)
    mu, lr = 0.9, 0.1
    th, v = x0[0].copy(), np.zeros(9)
    for _ in range(12):
        parle.inner_update(st, _quad_grad(st.y, c), cfg)
        v = mu * v - lr * _quad_grad(th + mu * v, c)
        th = th + v
        assert np.allclose(st.y[0], th + mu * v, atol=1e-14)


# ---- full cycle is one SGD step when L = 1, alpha = 0, mu = 0, eta = 1 and (8c) as printed --------
def test_full_cycle_reduces_to_sgd_on_x():
    rng = np.random.default_rng(5)
    c, x0 = rng.standard_normal(15), rng.standard_normal((1, 15))
    cfg = _cfg(1, L=1, gamma0=0.0, rho0=0.0, momentum=0.0, alpha=0.0, eta_outer=1.0, xa_mode=1)
    st = parle.init_state(x0, cfg)
    x = x0[0].copy()
    for _ in range(5):
        parle.inner_update(st, _quad_grad(st.y, c), cfg)
        parle.outer_step(st, cfg)
        x = x - 0.1 * (x - c)
        assert np.allclose(st.x[0], x, atol=1e-15)
        assert np.array_equal(st.y[0], st.x[0])


def test_unscaled_mode_with_zero_couplings_never_moves_x():
    rng = np.random.default_rng(6)
    x0 = rng.standard_normal((3, 11)).astype(np.float32)
    cfg = _cfg(3, gamma0=0.0, rho0=0.0, xa_mode=0)
    st = parle.init_state(x0, cfg, dtype=np.float32)
    for _ in range(3):
        parle.inner_update(st, rng.standard_normal((3, 11)), cfg)
    parle.outer_step(st, cfg)
    assert np.array_equal(st.x, x0)


# ---- n = 1, no elastic term: (8a)-(8c) are Entropy-SGD (6a)-(6c) ---------------------------------------
def test_parle_n1_is_entropy_sgd():
    rng = np.random.default_rng(7)
    c, x0 = rng.standard_normal(13), rng.standard_normal(13)
    L, eta_p, eta, gam_inv, alpha = 4, 0.05, 0.7, 0.3, 0.75
    cfg = _cfg(1, L=L, eta_inner=eta_p, eta_outer=eta, gamma0=gam_inv, rho0=0.0, momentum=0.0, alpha=alpha,
               xa_mode=1)
    st = parle.init_state(x0[None], cfg)
    # Entropy-SGD written directly from (6a)-(6c): y starts at x, L steps, then the x update.
    x = x0.copy()
    for _ in range(3):
        y, z = x.copy(), x.copy()
        for _ in range(L):
            y = y - eta_p * ((y - c) + gam_inv * (y - x))
            z = alpha * z + (1 - alpha) * y
            parle.inner_update(st, _quad_grad(st.y, c), cfg)
        x = x - eta * (x - z)
        parle.outer_step(st, cfg)
        assert np.allclose(st.x[0], x, atol=1e-14)


# ---- (8b): exponential average ---------------------------------------------------------------------------
def test_z_average_closed_forms():
    x0 = np.full((1, 4), 2.0)
    cfg = _cfg(1, gamma0=0.0, rho0=0.0, momentum=0.0, eta_inner=1.0, alpha=0.75)
    st = parle.init_state(x0, cfg)
    # constant gradient -1 with lr 1 makes y_k = 2 + k; z_0 = 2
    for _ in range(6):
        parle.inner_update(st, -np.ones((1, 4)), cfg)
    k = 6
    # z_k = a^k z_0 + (1-a) sum_{j=1..k} a^(k-j) (2 + j)
    a = 0.75
    zk = a ** k * 2.0 + (1 - a) * sum(a ** (k - j) * (2.0 + j) for j in range(1, k + 1))
    assert np.allclose(st.z, zk, atol=1e-14)
    # alpha = 0 makes z = y; zero gradient keeps z where it is
    cfg0 = _cfg(1, gamma0=0.0, rho0=0.0, alpha=0.0)
    st0 = parle.init_state(x0, cfg0)
    parle.inner_update(st0, np.ones((1, 4)), cfg0)
    assert np.array_equal(st0.z, st0.y)


def test_fixed_point_is_bit_exact():
    row = np.random.default_rng(8).standard_normal(33).astype(np.float32).astype(np.float64)
    cfg = _cfg(4)
    st = parle.init_state(np.tile(row, (4, 1)), cfg)
    for _ in range(3):
        for _ in range(5):
            parle.inner_update(st, np.zeros((4, 33)), cfg)
        parle.outer_step(st, cfg)
    for t in (st.x, st.y, st.z):
        assert np.array_equal(t, np.tile(row, (4, 1)))
    assert np.array_equal(st.x_ref, row) and not st.vx.any() and not st.vy.any()


# ---- (8c): elastic contraction toward the reference -------------------------------------------------------
def test_elastic_contraction_factor_and_mean_preserved():
    rng = np.random.default_rng(9)
    x0 = rng.standard_normal((5, 21))
    eta, r = 0.1, 1.7
    cfg = _cfg(5, gamma0=0.0, rho0=r, momentum=0.0, eta_outer=eta)
    st = parle.init_state(x0, cfg)
    m0 = x0.mean(axis=0)
    for t in range(1, 5):
        parle.inner_update(st, np.zeros_like(x0), cfg)     # zero gradient: y, z stay at x
        parle.outer_step(st, cfg)
        assert np.allclose(st.x - m0, (1 - eta * r) ** t * (x0 - m0), atol=1e-14)
        assert np.allclose(st.x.mean(axis=0), m0, atol=1e-14)


def test_elastic_contraction_with_momentum_recurrence():
    """With Nesterov momentum the deviation e_t = x^a - mean obeys a scalar linear recurrence:
    v_t = mu v_{t-1} + r e_{t-1};  e_t = e_{t-1} - eta (r e_{t-1} + mu v_t)."""
    x0 = np.array([[1.0], [-1.0]])
    eta, r, mu = 0.1, 0.8, 0.9
    cfg = _cfg(2, gamma0=0.0, rho0=r, momentum=mu, eta_outer=eta)
    st = parle.init_state(x0, cfg)
    e, v = 1.0, 0.0
    for _ in range(8):
        parle.inner_update(st, np.zeros_like(x0), cfg)
        parle.outer_step(st, cfg)
        v = mu * v + r * e
        e = e - eta * (r * e + mu * v)
        assert np.allclose(st.x[:, 0], [e, -e], atol=1e-14)


def test_lagged_reference_mode_uses_previous_mean():
    x0 = np.array([[0.0], [2.0]])
    cfg = _cfg(2, gamma0=0.0, rho0=1.0, momentum=0.0, eta_outer=0.5, xref_mode=1)
    st = parle.init_state(x0, cfg)
    st.x_ref = np.array([10.0])                       # a stale reference
    parle.inner_update(st, np.zeros_like(x0), cfg)
    parle.outer_step(st, cfg)
    assert np.allclose(st.x[:, 0], [0 - 0.5 * (0 - 10), 2 - 0.5 * (2 - 10)])
    assert np.allclose(st.x_ref, [1.0])               # refreshed from the replicas before they moved


def test_quadratic_collapse(  # Section 2.4: for convex f replicas and reference collapse to one point
):
    rng = np.random.default_rng(10)
    c, x0 = rng.standard_normal(8), rng.standard_normal((3, 8)) * 3
    cfg = _cfg(3, L=5, momentum=0.0, gamma0=0.5, rho0=1.0, xa_mode=1, eta_outer=0.5)
    st = parle.init_state(x0, cfg)
    prev = np.inf
    for _ in range(400):
        for _ in range(cfg.L):
            parle.inner_update(st, _quad_grad(st.y, c), cfg)
        parle.outer_step(st, cfg)
        sp = parle.spread(st)
        assert sp <= prev + 1e-18
        prev = sp
    assert np.abs(st.x - c).max() < 1e-6 and np.abs(st.x_ref - c).max() < 1e-6


# ---- rule (9): scoping --------------------------------------------------------------------------------------
def test_scoping_closed_form_and_clips():
    B = 2
    cfg = _cfg(1, gamma0=0.01, rho0=1.0, gamma_max=1.0, rho_max=10.0, scoping_B=B)
    for t in range(40):
        g, r = parle.scoping_multipliers(cfg, t)
        gamma_paper = max(100.0 * (1 - 1 / (2 * B)) ** t, 1.0)
        rho_paper = max(1.0 * (1 - 1 / (2 * B)) ** t, 0.1)
        assert np.isclose(g, 1 / gamma_paper, rtol=1e-14) and np.isclose(r, 1 / rho_paper, rtol=1e-14)
    assert parle.scoping_multipliers(cfg, 40) == (1.0, 10.0)
    # iterated product form: one factor per completed outer step
    g = 0.01
    for t in range(10):
        assert np.isclose(parle.scoping_multipliers(cfg, t)[0], min(g, 1.0), rtol=1e-13)
        g = g / (1 - 1 / (2 * B))
    off = _cfg(1, gamma0=0.03, rho0=1.0, scoping_B=0)
    assert parle.scoping_multipliers(off, 1000) == (0.03, 1.0)


def test_scoping_applied_after_the_outer_step_that_used_old_value():
    cfg = _cfg(2, gamma0=0.5, rho0=1.0, rho_max=10.0, scoping_B=1, momentum=0.0, eta_outer=0.1)
    x0 = np.array([[1.0], [-1.0]])
    st = parle.init_state(x0, cfg)
    parle.inner_update(st, np.zeros_like(x0), cfg)
    parle.outer_step(st, cfg)
    assert np.allclose(st.x[:, 0], [0.9, -0.9])        # used r = 1
    assert np.isclose(st.r, 2.0) and np.isclose(st.g, 1.0)   # 1/(1 - 1/2) = 2; g clipped at 1


def test_outer_step_requires_an_inner_step():
    cfg = _cfg(2)
    st = parle.init_state(np.zeros((2, 3)), cfg)
    with pytest.raises(RuntimeError):
        parle.outer_step(st, cfg)


def test_weight_decay_is_gradient_of_l2_term():
    """f includes the regulariser (Section 1.1): wd * y is the gradient of 0.5 wd ||y||^2."""
    x0 = np.array([[2.0, -4.0]])
    cfg = _cfg(1, gamma0=0.0, rho0=0.0, momentum=0.0, weight_decay=0.5, eta_inner=0.1)
    st = parle.init_state(x0, cfg)
    parle.inner_update(st, np.zeros_like(x0), cfg)
    assert np.allclose(st.y, x0 * (1 - 0.05))
