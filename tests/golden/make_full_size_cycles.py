"""Writes tests/golden/full_size_cycle_{allcnn,wrn}.npz: what the CPU oracle makes of the two bf16 workloads at
their full size (three replicas, batch 128, 3x32x32 inputs, L = 25 inner steps per block, updates (8a)-(8d) of
Section 3, rule (9) for the residual network), one block + outer step for All-CNN-C and two for WRN-16-4.

Calls only oracle/ and the seeded input generators; takes 10-30 minutes of CPU per network, which is why the
result is stored instead of being recomputed by the GPU test (tests/test_gpu_full_cycles.py).  The oracle runs
in its float32 mode (the comparison bar is the bf16 one, 2e-2).

Stored per block b: the sampled entries (fixed seeded positions, up to SAMPLES per parameter segment, the same
for every replica and tensor) of y, z, vy after the 25th inner step and of x, vx, x_ref after the outer step;
the 2-norm of every segment of y - x_start and x - x_start over ALL its entries; the couplings g, r after the
outer step; batch-norm running statistics; and the per-step losses of all replicas.

    python tests/golden/make_full_size_cycles.py [allcnn] [wrn]
"""
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import nets, parle, trainer  # noqa: E402
from paper_1707_00424_amd import synth  # noqa: E402

SAMPLES = 384
RECIPES = {
    # step sizes: 0.1 makes All-CNN-C (no batch-norm) overflow within three steps on these inputs and drives
    # the residual network's loss to 1e-3 within one block, where a relative bar on the loss says nothing;
    # 0.01 is also what Section 4.4 starts WRN-16-4 with
    "allcnn": dict(model="allcnn", n=3, batch=128, L=25, blocks=1, seed=0, eta_inner=0.01, eta_outer=0.01,
                   momentum=0.9, alpha=0.75, gamma0=0.03, rho0=1.0, scoping_B=0, weight_init="he_normal"),
    "wrn": dict(model="wrn", n=3, batch=128, L=25, blocks=2, seed=0, eta_inner=0.01, eta_outer=0.01,
                momentum=0.9, alpha=0.75, gamma0=0.03, rho0=1.0, scoping_B=390, weight_init="he_normal"),
}


def sample_positions(layout, seed):
    """Sorted flat positions inside a replica row, up to SAMPLES per segment; plus the segment boundaries."""
    rng = np.random.default_rng([seed, 9009])
    pos, bounds, off = [], [0], 0
    for s in layout:
        size = int(np.prod(s["shape"]))
        take = np.sort(rng.choice(size, size=min(size, SAMPLES), replace=False)) + off
        pos.append(take)
        off += size
        bounds.append(bounds[-1] + len(take))
    return np.concatenate(pos).astype(np.int64), np.asarray(bounds, np.int64)


def segment_norms(layout, delta):
    out, off = np.zeros((delta.shape[0], len(layout))), 0
    for i, s in enumerate(layout):
        size = int(np.prod(s["shape"]))
        out[:, i] = np.linalg.norm(delta[:, off:off + size].astype(np.float64), axis=1)
        off += size
    return out


def make(name):
    rc = RECIPES[name]
    a = nets.arch(rc["model"])
    lay = nets.layout(a)
    n, B, L = rc["n"], rc["batch"], rc["L"]
    x0 = np.tile(synth.init_params(lay, rc["seed"], rc["weight_init"]), (n, 1))
    cfg = parle.ParleConfig(n_replicas=n, L=L, eta_inner=rc["eta_inner"], eta_outer=rc["eta_outer"],
                            momentum=rc["momentum"], alpha=rc["alpha"], gamma0=rc["gamma0"], rho0=rc["rho0"],
                            scoping_B=rc["scoping_B"])
    O = trainer.ParleNet(a, cfg, x0, dtype=np.float32)
    steps = L * rc["blocks"]
    X, Y = synth.image_batches(rc["seed"], steps, n, B, a["H"], a["W"], a["C"], a["classes"])
    pos, bounds = sample_positions(lay, rc["seed"])
    out = dict(recipe=json.dumps(rc), positions=pos, segment_bounds=bounds,
               segment_names=np.array([s["name"] for s in lay]))
    losses = np.zeros((steps, n))
    t0 = time.time()
    for b in range(rc["blocks"]):
        start = O.st.x.copy()
        for k in range(b * L, (b + 1) * L):
            losses[k] = O.inner_step(X[k], Y[k])
            print(f"{name}: step {k + 1}/{steps} loss {losses[k].round(4)} {time.time() - t0:.0f} s", flush=True)
        for t in ("y", "z", "vy"):
            out[f"b{b}_{t}"] = getattr(O.st, t)[:, pos].astype(np.float32)
        out[f"b{b}_grad"] = O.last_grad[:, pos].astype(np.float32)
        out[f"b{b}_ynorm"] = segment_norms(lay, O.st.y - start)
        O.outer_step()
        for t in ("x", "vx"):
            out[f"b{b}_{t}"] = getattr(O.st, t)[:, pos].astype(np.float32)
        out[f"b{b}_x_ref"] = O.st.x_ref[pos].astype(np.float32)
        out[f"b{b}_xnorm"] = segment_norms(lay, O.st.x - start)
        out[f"b{b}_gr"] = np.array([O.st.g, O.st.r])
        if nets.bn_layers(a):
            out[f"b{b}_bn"] = np.stack([np.concatenate([np.concatenate(O.bn[r][nm]) for nm, _ in nets.bn_layers(a)])
                                        for r in range(n)]).astype(np.float32)
    out["losses"] = losses
    out["relu_margin"] = np.array(O.relu_margin)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"full_size_cycle_{name}.npz")
    np.savez_compressed(path, **out)
    print(f"wrote {path} ({os.path.getsize(path) / 1e6:.2f} MB) in {time.time() - t0:.0f} s", flush=True)


if __name__ == "__main__":
    for which in (sys.argv[1:] or list(RECIPES)):
        make(which)
