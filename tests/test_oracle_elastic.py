"""Pins for oracle/elastic.py (Elastic-SGD of Section 2.2 with scoping on rho).

Closed forms of the linear dynamics, reductions to independently written SGD
loops, invariants.  None of them retypes the oracle's formula.
"""
import numpy as np
import pytest

from oracle import elastic, parle


def _cfg(n, **kw):
    base = dict(n_replicas=n, L=25, eta_inner=0.1, eta_outer=0.1, momentum=0.0, gamma0=0.0, rho0=1.0)
    base.update(kw)
    return parle.ParleConfig(**base)


def test_single_replica_uncoupled_is_nesterov_sgd():
    # n = 1 and r = 0: the replica runs SGD with Nesterov's momentum on f, written here independently
    rng = np.random.default_rng(0)
    c, x0 = rng.standard_normal(17), rng.standard_normal((1, 17))
    cfg = _cfg(1, rho0=0.0, momentum=0.9)
    st = elastic.init_state(x0, cfg)
    p, buf = x0[0].copy(), np.zeros(17)
    for _ in range(9):
        elastic.step(st, st.xa - c, cfg)
        g = p - c
        buf = 0.9 * buf + g
        p = p - 0.1 * (g + 0.9 * buf)
        assert np.allclose(st.xa[0], p, rtol=0, atol=1e-15)


def test_zero_gradient_linear_dynamics_closed_form():
    # G = 0, mu = 0: with m the replica mean, e = m - x and delta^a = x^a - m,
    #   delta^a_{k+1} = (1 - eta r) delta^a_k        (each replica contracts onto the mean)
    #   e_{k+1}       = (1 - eta r - eta_ref) e_k    (mean and reference approach each other)
    #   x_{k+1} + ... the weighted centre (eta_ref m + eta r x) / (eta_ref + eta r) never moves.
    rng = np.random.default_rng(1)
    n, N, eta, eta_ref, r = 4, 23, 0.1, 0.25, 3.0
    cfg = _cfg(n, eta_inner=eta, eta_outer=eta_ref, rho0=r)
    x0 = rng.standard_normal((n, N))
    st = elastic.init_state(x0, cfg)
    st.x = rng.standard_normal(N)                      # a reference away from the mean
    m0, xr0 = x0.mean(axis=0), st.x.copy()
    centre0 = (eta_ref * m0 + eta * r * xr0) / (eta_ref + eta * r)
    for k in range(1, 13):
        elastic.step(st, np.zeros((n, N)), cfg)
        m = st.xa.mean(axis=0)
        assert np.allclose(st.xa - m, (1 - eta * r) ** k * (x0 - m0), atol=1e-14)
        assert np.allclose(m - st.x, (1 - eta * r - eta_ref) ** k * (m0 - xr0), atol=1e-14)
        assert np.allclose((eta_ref * m + eta * r * st.x) / (eta_ref + eta * r), centre0, atol=1e-14)


def test_reference_uses_replicas_before_the_move():
    # one step from a reference equal to the replica mean: whatever the gradients are, the
    # reference must not move (the average in its update is over the old replicas)
    rng = np.random.default_rng(2)
    cfg = _cfg(3, momentum=0.9)
    x0 = rng.standard_normal((3, 11))
    st = elastic.init_state(x0, cfg)
    ref0 = st.x.copy()
    elastic.step(st, rng.standard_normal((3, 11)), cfg)
    assert np.array_equal(st.x, ref0)
    assert not np.allclose(st.xa.mean(axis=0), ref0)


def test_identical_replicas_and_zero_gradient_is_a_fixed_point():
    cfg = _cfg(4, momentum=0.9, rho0=2.0)
    row = np.random.default_rng(3).standard_normal(19).astype(np.float32).astype(np.float64)
    st = elastic.init_state(np.tile(row, (4, 1)), cfg)
    for _ in range(5):
        elastic.step(st, np.zeros((4, 19)), cfg)
    assert np.array_equal(st.xa, np.tile(row, (4, 1))) and np.array_equal(st.x, row)


def test_quadratic_collapse_to_the_minimiser():
    # convex f: replicas and reference all end at the minimiser (Section 2.4)
    rng = np.random.default_rng(4)
    c = rng.standard_normal(9)
    cfg = _cfg(3, momentum=0.9, rho0=1.0)
    st = elastic.init_state(rng.standard_normal((3, 9)), cfg)
    for _ in range(600):
        elastic.step(st, st.xa - c, cfg)
    assert np.abs(st.xa - c).max() < 1e-9 and np.abs(st.x - c).max() < 1e-9


def test_weight_decay_is_part_of_f():
    # f(x) = wd/2 ||x||^2 alone, r = 0, mu = 0: x_k = (1 - eta wd)^k x_0
    cfg = _cfg(2, rho0=0.0, weight_decay=0.5)
    x0 = np.random.default_rng(5).standard_normal((2, 7))
    st = elastic.init_state(x0, cfg)
    for _ in range(6):
        elastic.step(st, np.zeros((2, 7)), cfg)
    assert np.allclose(st.xa, (1 - 0.1 * 0.5) ** 6 * x0, atol=1e-15)


def test_scoping_on_rho_only_closed_form():
    # rule (9): rho_k = rho_0 (1 - 1/(2B))^k clipped at 1/rho_max; the proximal multiplier is untouched
    cfg = _cfg(2, rho0=1.0, rho_max=10.0, scoping_B=2, gamma0=0.0)
    st = elastic.init_state(np.zeros((2, 3)), cfg)
    for k in range(1, 15):
        elastic.scope(st, cfg)
        assert st.r == pytest.approx(min(1.0 / (1.0 * 0.75 ** k), 10.0), rel=1e-14)
    assert st.r == 10.0
