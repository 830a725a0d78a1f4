"""Why the LeNet workload is checked step by step from a shared state (tests/test_gpu_nets.py).

The oracle in float32 and the same oracle in float64 are the same algorithm; they differ only in
rounding.  On the LeNet workload at step size 0.1 one differing ReLU / max-pool decision is enough
to separate the two trajectories by far more than 1e-5 within L = 25 inner steps, so no float32
implementation can be held to 1e-5 against the float64 trajectory there; at step size 0.01 the two
stay together.  This pins the tolerance policy, not a kernel."""
import numpy as np

from oracle import nets, parle, trainer
from paper_1707_00424_amd import synth


def _gap(eta, steps):
    a = nets.arch("lenet")
    n = 2
    x0 = np.tile(synth.init_params(nets.layout(a), 0, "uniform"), (n, 1))
    X, Y = synth.image_batches(0, steps, n, 128, 28, 28, 1)
    cfg = parle.ParleConfig(n_replicas=n, gamma0=0.03, rho0=1.0, eta_inner=eta, eta_outer=eta)
    o64, o32 = trainer.ParleNet(a, cfg, x0), trainer.ParleNet(a, cfg, x0, dtype=np.float32)
    for k in range(steps):
        o64.inner_step(X[k], Y[k])
        o32.inner_step(X[k], Y[k])
    return np.linalg.norm(o32.st.y - o64.st.y) / np.linalg.norm(o64.st.y)


def test_float32_oracle_leaves_float64_oracle_at_step_size_0p1():
    assert _gap(0.1, 25) > 1e-4


def test_float32_oracle_stays_with_float64_oracle_at_step_size_0p01():
    assert _gap(0.01, 25) < 1e-6
