"""CPU oracle: Parle on a network = oracle/nets.py gradients fed to oracle/parle.py updates.

TEST INFRASTRUCTURE ONLY (tests, smoke check, CPU-baseline timing).  One call
of :func:`inner_step` is what Section 3 of the paper does per mini-batch for
all replicas: gradient of the mini-batch loss at y^a, then (8a)-(8b);
:func:`outer_step` is (8c)-(8d), the reset, and rule (9).
"""
from __future__ import annotations

import numpy as np

from . import nets, parle


class ParleNet:
    """``storage="bf16"`` keeps activations, their gradients and the weights inside the contractions on the
    bfloat16 grid (nets.loss_and_grad); the state of (8a)-(8d) and all sums stay in ``dtype``."""

    def __init__(self, a, cfg: parle.ParleConfig, x0, dtype=np.float64, storage=None):
        self.a, self.cfg, self.dtype, self.storage = a, cfg, dtype, storage
        self.st = parle.init_state(x0, cfg, dtype=dtype)
        self.bn = [nets.new_bn_state(a, dtype) for _ in range(cfg.n_replicas)]
        self.relu_margin = np.inf  # smallest non-zero |ReLU input| over all steps so far (diagnostic)
        # per replica, of the last step: smallest distance of any ReLU input from zero / of any positive max-pool
        # winner from its runner-up -- how close the step came to a decision that rounding could take differently
        self.last_margins = np.full(cfg.n_replicas, np.inf)
        self.last_decisions = [[] for _ in range(cfg.n_replicas)]   # per replica: nets.loss_and_grad's `decisions`

    def inner_step(self, images, labels):
        """images ``[n, B, H, W, C]``, labels ``[n, B]``; returns the per-replica losses at y^a."""
        n = self.cfg.n_replicas
        losses = np.zeros(n)
        G = np.zeros_like(self.st.y)
        for a_i in range(n):
            drop = (dict(p=self.cfg.dropout, seed=self.cfg.dropout_seed, step=self.st.k, replica=a_i)
                    if self.cfg.dropout > 0 else None)
            diag = {}
            losses[a_i], G[a_i] = nets.loss_and_grad(self.a, self.st.y[a_i], images[a_i], labels[a_i],
                                                     bn_state=self.bn[a_i], dtype=self.dtype, drop=drop, diag=diag,
                                                     storage=self.storage)
            self.relu_margin = min(self.relu_margin, diag["relu_margin"])
            self.last_margins[a_i] = min(diag["relu_margin"], diag["pool_margin"])
            self.last_decisions[a_i] = diag["decisions"]
        parle.inner_update(self.st, G, self.cfg)
        self.last_grad = G
        return losses

    def outer_step(self):
        parle.outer_step(self.st, self.cfg)

    def eval(self, which, images, labels):
        """Loss / error count of the reference (which = -1, batch-norm statistics averaged over the
        replicas) or of replica ``which`` (its x^a), plus the ensemble spread."""
        if which < 0:
            flat = self.st.x_ref
            bn = {k: [np.mean([b[k][0] for b in self.bn], axis=0), np.mean([b[k][1] for b in self.bn], axis=0)]
                  for k in self.bn[0]}
        else:
            flat, bn = self.st.x[which], self.bn[which]
        loss, nerr = nets.evaluate(self.a, flat, images, labels, bn_state=bn, dtype=self.dtype, storage=self.storage)
        sp = float(sum(np.sum((self.st.x[i] - self.st.x_ref) ** 2) for i in range(self.cfg.n_replicas)))
        return loss, nerr, sp


class ElasticNet:
    """Elastic-SGD (Section 2.2) on a network: gradient of the mini-batch loss at every replica x^a,
    then one coupled step of the replicas and the reference; :func:`scope` is rule (9) on rho."""

    def __init__(self, a, cfg: parle.ParleConfig, x0, dtype=np.float64):
        from . import elastic
        self._el = elastic
        self.a, self.cfg, self.dtype = a, cfg, dtype
        self.st = elastic.init_state(x0, cfg, dtype=dtype)
        self.bn = [nets.new_bn_state(a, dtype) for _ in range(cfg.n_replicas)]
        self.relu_margin = np.inf  # smallest non-zero |ReLU input| over all steps so far (diagnostic)

    def step(self, images, labels):
        n = self.cfg.n_replicas
        losses = np.zeros(n)
        G = np.zeros_like(self.st.xa)
        for a_i in range(n):
            drop = (dict(p=self.cfg.dropout, seed=self.cfg.dropout_seed, step=self.st.k, replica=a_i)
                    if self.cfg.dropout > 0 else None)
            diag = {}
            losses[a_i], G[a_i] = nets.loss_and_grad(self.a, self.st.xa[a_i], images[a_i], labels[a_i],
                                                     bn_state=self.bn[a_i], dtype=self.dtype, drop=drop, diag=diag)
            self.relu_margin = min(self.relu_margin, diag["relu_margin"])
        self._el.step(self.st, G, self.cfg)
        self.last_grad = G
        return losses

    def scope(self):
        self._el.scope(self.st, self.cfg)

    def eval(self, which, images, labels):
        if which < 0:
            flat = self.st.x
            bn = {k: [np.mean([b[k][0] for b in self.bn], axis=0), np.mean([b[k][1] for b in self.bn], axis=0)]
                  for k in self.bn[0]}
        else:
            flat, bn = self.st.xa[which], self.bn[which]
        loss, nerr = nets.evaluate(self.a, flat, images, labels, bn_state=bn, dtype=self.dtype)
        sp = float(sum(np.sum((self.st.xa[i] - self.st.x) ** 2) for i in range(self.cfg.n_replicas)))
        return loss, nerr, sp
