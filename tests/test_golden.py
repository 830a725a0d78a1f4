"""The values Section 3.1 prints (tests/golden/hyperparameters_section_3_1.txt) against the oracle.

The fixture is in the paper's notation (gamma, rho); the oracle computes with the multipliers g = 1/gamma and
r = 1/rho, so the test converts on its own side and evaluates rule (9) in the paper's form.
"""
import math
import pathlib

import numpy as np

from oracle import parle

GOLDEN = pathlib.Path(__file__).parent / "golden" / "hyperparameters_section_3_1.txt"


def _read():
    vals = {}
    for line in GOLDEN.read_text().splitlines():
        line = line.strip()
        if line and not line.startswith("#"):
            name, value = line.split()
            vals[name] = float(value)
    return vals


def test_oracle_defaults_are_the_papers_values():
    p = _read()
    cfg = parle.ParleConfig(n_replicas=3)
    assert cfg.L == p["L"] and cfg.alpha == p["alpha"] and cfg.momentum == p["momentum"]
    assert math.isclose(1.0 / cfg.gamma0, p["gamma_0"], rel_tol=1e-15)
    assert math.isclose(1.0 / cfg.rho0, p["rho_0"], rel_tol=1e-15)
    assert math.isclose(1.0 / cfg.gamma_max, p["gamma_floor"], rel_tol=1e-15)
    assert math.isclose(1.0 / cfg.rho_max, p["rho_floor"], rel_tol=1e-15)


def test_rule_9_with_the_papers_values_on_a_dataset_of_cifar_size():
    # B = mini-batches in the dataset: 50 000 images in batches of 128 -> 390 whole ones
    p, B = _read(), 390
    cfg = parle.ParleConfig(n_replicas=1, scoping_B=B)
    q = 1.0 - 1.0 / (2.0 * B)
    # first outer step at which each floor binds, from the closed form of (9)
    t_gamma = math.ceil(math.log(p["gamma_floor"] / p["gamma_0"]) / math.log(q))
    t_rho = math.ceil(math.log(p["rho_floor"] / p["rho_0"]) / math.log(q))
    assert 3000 < t_gamma < 4000 and 1500 < t_rho < 2000   # ln 100 * 780 = 3592, ln 10 * 780 = 1796
    for t in (0, 1, 2, 25, t_rho - 1, t_rho, t_rho + 1, t_gamma - 1, t_gamma, t_gamma + 1, 10000):
        g, r = parle.scoping_multipliers(cfg, t)
        gamma = max(p["gamma_0"] * q ** t, p["gamma_floor"])
        rho = max(p["rho_0"] * q ** t, p["rho_floor"])
        assert np.isclose(1.0 / g, gamma, rtol=1e-12) and np.isclose(1.0 / r, rho, rtol=1e-12)
    assert parle.scoping_multipliers(cfg, t_gamma)[0] == 1.0 / p["gamma_floor"]
    assert parle.scoping_multipliers(cfg, t_gamma - 1)[0] < 1.0 / p["gamma_floor"]
    assert parle.scoping_multipliers(cfg, t_rho)[1] == 1.0 / p["rho_floor"]
    assert parle.scoping_multipliers(cfg, t_rho - 1)[1] < 1.0 / p["rho_floor"]


def test_state_follows_rule_9_one_factor_per_outer_step():
    p, B = _read(), 4
    cfg = parle.ParleConfig(n_replicas=2, scoping_B=B, L=2)
    st = parle.init_state(np.array([[1.0, 2.0], [3.0, -1.0]]), cfg)
    q = 1.0 - 1.0 / (2.0 * B)
    for t in range(60):
        assert np.isclose(1.0 / st.g, max(p["gamma_0"] * q ** t, p["gamma_floor"]), rtol=1e-12)
        assert np.isclose(1.0 / st.r, max(p["rho_0"] * q ** t, p["rho_floor"]), rtol=1e-12)
        for _ in range(cfg.L):
            parle.inner_update(st, np.zeros_like(st.x), cfg)
        parle.outer_step(st, cfg)
    assert st.g == 1.0 and st.r == 10.0
