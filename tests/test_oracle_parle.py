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


# ---- (8c) in its default form: the unscaled gradient of local entropy, g (x^a - z^a) ------------------------
def test_outer_step_default_mode_hand_computed_numbers():
    """Two scalar replicas, momentum 0, z != x, g = 0.5, r = 1, eta = 0.1; numbers worked by hand:
    mean = 2;  replica 0: d = 0.5 (1 - 0.5) + 1 (1 - 2) = -0.75  ->  x = 1.075;
               replica 1: d = 0.5 (3 - 3.5) + 1 (3 - 2) =  0.75  ->  x = 2.925."""
    cfg = _cfg(2, gamma0=0.5, rho0=1.0, momentum=0.0, eta_outer=0.1, xa_mode=0)
    st = parle.init_state(np.array([[1.0], [3.0]]), cfg)
    st.z = np.array([[0.5], [3.5]])
    st.inner_since_outer = 1
    parle.outer_step(st, cfg)
    assert np.allclose(st.x[:, 0], [1.075, 2.925], rtol=0, atol=1e-15)
    assert np.allclose(st.x_ref, [2.0]) and np.array_equal(st.y, st.x) and np.array_equal(st.z, st.x)
    # the printed form of (8c) (coefficient 1 on x - z) from the same state: d = 0.5 - 1, -0.5 + 1
    cfg1 = _cfg(2, gamma0=0.5, rho0=1.0, momentum=0.0, eta_outer=0.1, xa_mode=1)
    st = parle.init_state(np.array([[1.0], [3.0]]), cfg1)
    st.z = np.array([[0.5], [3.5]])
    st.inner_since_outer = 1
    parle.outer_step(st, cfg1)
    assert np.allclose(st.x[:, 0], [1.05, 2.95], rtol=0, atol=1e-15)


def test_outer_step_default_mode_with_momentum_two_steps_hand_computed():
    """One replica (so the elastic term vanishes), g = 0.5, eta = 0.1, momentum 0.9, z held at 0 by hand:
    step 1: d = 0.5 * 2 = 1, v = 1, x = 2 - 0.1 (1 + 0.9) = 1.81;
    step 2: d = 0.905, v = 0.9 + 0.905 = 1.805, x = 1.81 - 0.1 (0.905 + 1.6245) = 1.55705."""
    cfg = _cfg(1, gamma0=0.5, rho0=1.0, momentum=0.9, eta_outer=0.1, xa_mode=0)
    st = parle.init_state(np.array([[2.0]]), cfg)
    for want in (1.81, 1.55705):
        st.z = np.zeros((1, 1))
        st.inner_since_outer = 1
        parle.outer_step(st, cfg)
        assert np.allclose(st.x, want, rtol=0, atol=1e-14)


def test_default_outer_step_is_gradient_descent_on_local_entropy_of_a_quadratic():
    """Remark "Scoping and learning rate annealing": grad f_gamma(x) = (x - <y>) / gamma.  For
    f(y) = c y^2 / 2 the Gibbs measure of (3) is Gaussian with mean x / (1 + gamma c), so
    grad f_gamma(x) = c x / (1 + gamma c) in closed form.  With exact gradients the y-chain of (8a)
    settles at that mean and z follows it, so one default-mode outer step (no elastic term, no momentum)
    must be x <- x - eta c x / (1 + gamma c)."""
    c, gamma, eta = 3.0, 0.25, 0.2
    cfg = _cfg(1, L=400, gamma0=1.0 / gamma, rho0=0.0, momentum=0.0, eta_inner=0.05, eta_outer=eta, alpha=0.75,
               xa_mode=0)
    st = parle.init_state(np.array([[1.5, -0.7]]), cfg)
    x = np.array([1.5, -0.7])
    for _ in range(3):
        for _ in range(cfg.L):
            parle.inner_update(st, c * st.y, cfg)
        assert np.allclose(st.z[0], x / (1 + gamma * c), atol=1e-12)
        parle.outer_step(st, cfg)
        x = x - eta * c * x / (1 + gamma * c)
        assert np.allclose(st.x[0], x, atol=1e-12)


def test_first_outer_step_uses_the_initial_couplings():
    """Rule (9) with exponent floor(k/L) counted in completed outer steps: the outer step that closes the
    first block still sees gamma_0 and rho_0.  g0 = 0.5 doubles to 1 (B = 1) only afterwards:
    d = 0.5 (1 - 0) + 1 (1 - 0) with the mean of +-1 at 0 -> x = 1 - 0.1 * 1.5 = 0.85."""
    cfg = _cfg(2, gamma0=0.5, rho0=1.0, gamma_max=4.0, rho_max=10.0, scoping_B=1, momentum=0.0, eta_outer=0.1)
    st = parle.init_state(np.array([[1.0], [-1.0]]), cfg)
    st.z = np.zeros((2, 1))
    st.inner_since_outer = 1
    parle.outer_step(st, cfg)
    assert np.allclose(st.x[:, 0], [0.85, -0.85], rtol=0, atol=1e-15)
    assert st.g == 1.0 and st.r == 2.0
    # the next inner step is pulled with the doubled g = 1: from y = x + 1, d = 1, y - x = 1 - 0.1 = 0.9
    st.y = st.x + 1.0
    parle.inner_update(st, np.zeros((2, 1)), cfg)
    assert np.allclose(st.y - st.x, 0.9, rtol=0, atol=1e-15)


# ---- the reset after the outer step (y^a <- x^a is stated; z^a and the y-momentum are readings) ---------------
def test_reset_clears_the_y_momentum_and_the_flag_that_keeps_it():
    """Constant gradient 1, no couplings (x never moves), eta' = 0.1, mu = 0.9.  By hand:
    block 1: v = 1, y = -0.19; v = 1.9, y = -0.19 - 0.1 (1 + 1.71) = -0.461.
    fresh chain after the reset: v = 1, y = -0.19.
    momentum carried over instead: v = 0.9 * 1.9 + 1 = 2.71, y = 0 - 0.1 (1 + 2.439) = -0.3439."""
    for flags, first in ((3, -0.19), (1, -0.3439)):
        cfg = _cfg(1, gamma0=0.0, rho0=0.0, momentum=0.9, eta_inner=0.1, reset_flags=flags)
        st = parle.init_state(np.zeros((1, 1)), cfg)
        parle.inner_update(st, np.ones((1, 1)), cfg)
        assert np.allclose(st.y, -0.19, atol=1e-15)
        parle.inner_update(st, np.ones((1, 1)), cfg)
        assert np.allclose(st.y, -0.461, atol=1e-15)
        parle.outer_step(st, cfg)
        assert st.x[0, 0] == 0.0 and st.y[0, 0] == 0.0
        parle.inner_update(st, np.ones((1, 1)), cfg)
        assert np.allclose(st.y, first, atol=1e-15), flags


def test_reset_of_z_and_the_flag_that_keeps_it():
    """alpha = 0.5, constant gradient -1, eta' = 1, no momentum: y = 1, z = 0.5 after one step.  The outer step
    (no couplings) leaves x = 0; bit 0 of reset_flags restarts z at x, without it z stays 0.5."""
    for flags, want in ((3, 0.0), (2, 0.5)):
        cfg = _cfg(1, gamma0=0.0, rho0=0.0, momentum=0.0, eta_inner=1.0, alpha=0.5, reset_flags=flags)
        st = parle.init_state(np.zeros((1, 1)), cfg)
        parle.inner_update(st, -np.ones((1, 1)), cfg)
        assert st.y[0, 0] == 1.0 and st.z[0, 0] == 0.5
        parle.outer_step(st, cfg)
        assert st.z[0, 0] == want and st.y[0, 0] == 0.0


def test_weight_decay_acts_on_y_not_on_x():
    """f contains the regulariser (Section 1.1), so its gradient in (8a) is taken where the data gradient
    is: at y.  With zero data gradient and no coupling y_k = (1 - eta' wd)^k y_0; by hand 2 -> 1.9 -> 1.805
    (the decay of the anchor x instead would give 1.8).  With the proximal term on, by hand:
    step 1: d = 0.5 * 2 = 1, y = 1.9;  step 2: d = 0.5 * 1.9 + 0.3 (1.9 - 2) = 0.92, y = 1.808."""
    cfg = _cfg(1, gamma0=0.0, rho0=0.0, momentum=0.0, weight_decay=0.5, eta_inner=0.1)
    st = parle.init_state(np.array([[2.0]]), cfg)
    for k in range(1, 6):
        parle.inner_update(st, np.zeros((1, 1)), cfg)
        assert np.allclose(st.y, 2.0 * 0.95 ** k, atol=1e-15)
    cfg = _cfg(1, gamma0=0.3, rho0=0.0, momentum=0.0, weight_decay=0.5, eta_inner=0.1)
    st = parle.init_state(np.array([[2.0]]), cfg)
    parle.inner_update(st, np.zeros((1, 1)), cfg)
    parle.inner_update(st, np.zeros((1, 1)), cfg)
    assert np.allclose(st.y, 1.808, atol=1e-15)


def test_spread_closed_form():
    """Two replicas at +-e around a reference at their mean: sum_a ||x^a - x||^2 = 2 ||e||^2."""
    e = np.array([3.0, -4.0, 12.0])                       # ||e||^2 = 169
    cfg = _cfg(2)
    st = parle.init_state(np.stack([5.0 + e, 5.0 - e]), cfg)
    assert np.allclose(st.x_ref, 5.0) and parle.spread(st) == 338.0
    st = parle.init_state(np.tile(e, (4, 1)), _cfg(4))    # collapsed ensemble
    assert parle.spread(st) == 0.0
