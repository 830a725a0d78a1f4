"""CPU oracle for the Parle replica-coupled update (TEST INFRASTRUCTURE ONLY).

This file is the slow, plain reference the HIP path is checked against.  It is
imported only by tests, the smoke check and the CPU-baseline leg of the bench;
the product path never calls it and shares no code with it.

Everything follows Section 3 of the paper (updates (8a)-(8d), the
hyper-parameter choices of Section 3.1 with the scoping rule (9), and the
remark on Nesterov's momentum), written in the *multiplier* convention

    g = 1 / gamma_paper,      r = 1 / rho_paper,

so the proximal force of (8a) is ``g * (y - x^a)`` and the elastic force of
(8c) is ``r * (x^a - x_ref)``.  Decaying gamma, rho in (9) is growing g, r.

Readings taken where the paper is silent (each is a flag so tests can flip it):

* Nesterov form: ``v <- mu v + d ; p <- p - lr (d + mu v)`` with v = 0 at start.
* coefficient on (x^a - z^a) in (8c): ``xa_mode = 1`` is the printed equation
  (coefficient 1, Remark "Scoping and learning rate annealing"); ``xa_mode = 0``
  keeps the unscaled local-entropy gradient ``g (x^a - z^a)`` stated in the
  same remark.
* reference used by (8c): ``xref_mode = 0`` forms the mean (8d, eta'' = rho/n)
  of the current replicas first and uses it; ``xref_mode = 1`` is the literal
  order of the printed equations (use the stored reference, then refresh it
  from the replicas as they were before the move).
* y^a is reset to x^a after the outer step (stated); ``reset_flags`` bit 0 also
  restarts z^a at x^a and bit 1 clears the y-momentum.
* the outer step runs after every completed block of inner steps, not at k = 0.

Arithmetic is float64 by default; ``dtype=np.float32`` exists only so the
CPU-baseline timing uses the same width as the device.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass
class ParleConfig:
    n_replicas: int
    L: int = 25                      # Section 3.1
    eta_inner: float = 0.1           # eta'  in (8a)
    eta_outer: float = 0.1           # eta   in (8c)
    momentum: float = 0.9            # Nesterov remark
    alpha: float = 0.75              # Section 3.1
    weight_decay: float = 0.0        # regulariser inside f, Section 1.1
    gamma0: float = 0.01             # multiplier 1/gamma_0, gamma_0 = 10^2
    rho0: float = 1.0                # multiplier 1/rho_0,   rho_0   = 1
    gamma_max: float = 1.0           # gamma clipped at 1   -> g <= 1
    rho_max: float = 10.0            # rho clipped at 0.1   -> r <= 10
    scoping_B: int = 0               # mini-batches in the dataset; 0 = no scoping
    xa_mode: int = 0
    xref_mode: int = 0
    reset_flags: int = 3
    dropout: float = 0.0             # Section 4 (networks only); 0 = off
    dropout_seed: int = 0


@dataclass
class ParleState:
    x: np.ndarray                    # [n, N] replicas x^a
    y: np.ndarray                    # [n, N] inner iterates y^a
    z: np.ndarray                    # [n, N] running averages z^a
    vy: np.ndarray                   # [n, N] momentum of y^a
    vx: np.ndarray                   # [n, N] momentum of x^a
    x_ref: np.ndarray                # [N]    reference x
    k: int = 0                       # inner steps taken
    outer_done: int = 0              # floor(k / L) in (9)
    inner_since_outer: int = 0
    g: float = 0.0
    r: float = 0.0
    hist: list = field(default_factory=list)


def replica_mean(x: np.ndarray) -> np.ndarray:
    """(8d) with eta'' = rho / n: the reference is the plain average of the replicas."""
    n = x.shape[0]
    acc = np.zeros(x.shape[1], dtype=x.dtype)
    for a in range(n):
        acc = acc + x[a]
    return acc / x.dtype.type(n)


def scoping_multipliers(cfg: ParleConfig, outer_done: int):
    """Rule (9): gamma_k = gamma_0 (1 - 1/(2B))^floor(k/L), same for rho, both clipped from below.

    Returned as multipliers g = 1/gamma_k, r = 1/rho_k (clipped from above).
    """
    if cfg.scoping_B <= 0:
        return float(cfg.gamma0), float(cfg.rho0)
    decay = (1.0 - 1.0 / (2.0 * cfg.scoping_B)) ** outer_done
    gamma_paper = (1.0 / cfg.gamma0) * decay if cfg.gamma0 > 0 else np.inf
    rho_paper = (1.0 / cfg.rho0) * decay if cfg.rho0 > 0 else np.inf
    gamma_paper = max(gamma_paper, 1.0 / cfg.gamma_max)
    rho_paper = max(rho_paper, 1.0 / cfg.rho_max)
    g = 0.0 if np.isinf(gamma_paper) else 1.0 / gamma_paper
    r = 0.0 if np.isinf(rho_paper) else 1.0 / rho_paper
    return float(g), float(r)


def init_state(x0: np.ndarray, cfg: ParleConfig, dtype=np.float64) -> ParleState:
    """Start of training: y^a = z^a = x^a, momenta zero, reference = replica mean."""
    x = np.array(x0, dtype=dtype, copy=True)
    assert x.ndim == 2 and x.shape[0] == cfg.n_replicas
    g, r = scoping_multipliers(cfg, 0)
    return ParleState(x=x, y=x.copy(), z=x.copy(), vy=np.zeros_like(x), vx=np.zeros_like(x),
                      x_ref=replica_mean(x), g=g, r=r)


def inner_update(st: ParleState, grad: np.ndarray, cfg: ParleConfig) -> None:
    """One inner step for every replica: (8a) with Nesterov momentum, then (8b).

    ``grad[a]`` is the mini-batch gradient of the data loss at y^a; the weight
    decay part of f and the proximal force are added here.
    """
    dt = st.y.dtype.type
    G = np.asarray(grad, dtype=st.y.dtype)
    mu, eta, alpha = dt(cfg.momentum), dt(cfg.eta_inner), dt(cfg.alpha)
    for a in range(cfg.n_replicas):
        d = G[a] + dt(cfg.weight_decay) * st.y[a] + dt(st.g) * (st.y[a] - st.x[a])
        st.vy[a] = mu * st.vy[a] + d
        st.y[a] = st.y[a] - eta * (d + mu * st.vy[a])
        st.z[a] = alpha * st.z[a] + (dt(1) - alpha) * st.y[a]
    st.k += 1
    st.inner_since_outer += 1


def outer_step(st: ParleState, cfg: ParleConfig) -> None:
    """(8c) with Nesterov momentum, (8d) as the replica mean, the reset of y^a, then rule (9)."""
    if st.inner_since_outer < 1:
        raise RuntimeError("outer step needs at least one inner step since the last one")
    dt = st.x.dtype.type
    mu, eta = dt(cfg.momentum), dt(cfg.eta_outer)
    c_z = dt(st.g) if cfg.xa_mode == 0 else dt(1)
    if cfg.xref_mode == 0:
        st.x_ref = replica_mean(st.x)
        ref_used = st.x_ref
    else:
        ref_used = st.x_ref
        st.x_ref = replica_mean(st.x)
    for a in range(cfg.n_replicas):
        d = c_z * (st.x[a] - st.z[a]) + dt(st.r) * (st.x[a] - ref_used)
        st.vx[a] = mu * st.vx[a] + d
        st.x[a] = st.x[a] - eta * (d + mu * st.vx[a])
        st.y[a] = st.x[a].copy()
        if cfg.reset_flags & 1:
            st.z[a] = st.x[a].copy()
        if cfg.reset_flags & 2:
            st.vy[a] = np.zeros_like(st.vy[a])
    st.outer_done += 1
    st.inner_since_outer = 0
    st.g, st.r = scoping_multipliers(cfg, st.outer_done)


def spread(st: ParleState) -> float:
    """Sum over replicas of ||x^a - x_ref||^2 (how far the ensemble is from collapse, Section 2.4)."""
    return float(sum(np.sum((st.x[a] - st.x_ref) ** 2) for a in range(st.x.shape[0])))
