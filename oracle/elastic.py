"""CPU oracle for Elastic-SGD with scoping on rho (TEST INFRASTRUCTURE ONLY).

Imported only by tests, the smoke check and the CPU-baseline leg of the bench;
the product path never calls it and shares no code with it.

Follows the Elastic-SGD updates of Section 2.2 of the paper (the two coupled
equations for the replicas x^a and the reference x), in the multiplier
convention r = 1 / rho_paper, with the scoping rule (9) of Section 3.1 applied
to rho alone (Sections 2.4 and 4.3 use Elastic-SGD that way):

    x^a <- x^a - eta [ grad f(x^a) + r (x^a - x) ]        for every replica a
    x   <- x   - eta ( x - (1/n) sum_a x^a )

Readings taken where the paper is silent:

* both equations are evaluated at the old iterates and applied together: the
  replica average in the second one is over the x^a before this step's move;
* the replicas move with Nesterov's momentum (the experiments use it for every
  algorithm), in the form ``v <- mu v + d ; p <- p - lr (d + mu v)``; the
  reference has no momentum (same reason as the remark on (8d));
* the replicas use ``eta_inner`` and the reference ``eta_outer`` of the shared
  config (the printed equations use one eta);
* rule (9) advances once per call of :func:`scope`, which the caller invokes
  every L steps, exactly as the outer step does for Parle;
* the reference starts at the average of the initial replicas.

Arithmetic is float64 by default.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from .parle import ParleConfig, replica_mean, scoping_multipliers


@dataclass
class ElasticState:
    xa: np.ndarray                   # [n, N] replicas x^a
    v: np.ndarray                    # [n, N] their momentum
    x: np.ndarray                    # [N]    reference
    k: int = 0
    scoped: int = 0                  # exponent of rule (9)
    r: float = 0.0


def init_state(x0: np.ndarray, cfg: ParleConfig, dtype=np.float64) -> ElasticState:
    xa = np.array(x0, dtype=dtype, copy=True)
    assert xa.ndim == 2 and xa.shape[0] == cfg.n_replicas
    _, r = scoping_multipliers(cfg, 0)
    return ElasticState(xa=xa, v=np.zeros_like(xa), x=replica_mean(xa), r=r)


def step(st: ElasticState, grad: np.ndarray, cfg: ParleConfig) -> None:
    """One Elastic-SGD step for all replicas and the reference (Section 2.2)."""
    dt = st.xa.dtype.type
    G = np.asarray(grad, dtype=st.xa.dtype)
    mu, eta, eta_ref = dt(cfg.momentum), dt(cfg.eta_inner), dt(cfg.eta_outer)
    old_mean = replica_mean(st.xa)
    old_ref = st.x
    for a in range(cfg.n_replicas):
        d = G[a] + dt(cfg.weight_decay) * st.xa[a] + dt(st.r) * (st.xa[a] - old_ref)
        st.v[a] = mu * st.v[a] + d
        st.xa[a] = st.xa[a] - eta * (d + mu * st.v[a])
    st.x = old_ref - eta_ref * (old_ref - old_mean)
    st.k += 1


def scope(st: ElasticState, cfg: ParleConfig) -> None:
    """Rule (9) on rho: one more factor (1 - 1/(2B)), clipped."""
    st.scoped += 1
    _, st.r = scoping_multipliers(cfg, st.scoped)
