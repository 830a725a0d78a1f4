"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

Nothing in here is part of the method: no update rule, no network arithmetic.
The functions only draw random numbers (numpy ``default_rng``) in the shapes
and distributions of the workloads:

* class-conditional Gaussian images: every class has a mean image whose pixels
  are N(0,1); a sample is its class mean plus N(0,1) noise; labels are uniform
  over the classes.  They stand in for the 1x28x28 and 3x32x32 ten-class image
  sets the paper trains on (Section 4), which are not available here.
* flat parameter / gradient vectors for the update-only workload.
* initial network parameters, drawn segment by segment from a *layout* the
  caller supplies (name, shape, kind, fan_in); the layout itself comes from
  whichever implementation is under test, never from this module.

Images are channels-last: ``[steps, n, B, H, W, C]`` float32; labels int32.
"""
from __future__ import annotations

import numpy as np


def class_means(seed: int, n_classes: int, h: int, w: int, c: int) -> np.ndarray:
    """Mean image of every class, pixels ~ N(0,1); float32 ``[n_classes, h, w, c]``."""
    rng = np.random.default_rng([seed, 1001])
    return rng.standard_normal((n_classes, h, w, c)).astype(np.float32)


def image_batches(seed: int, steps: int, n: int, batch: int, h: int, w: int, c: int,
                  n_classes: int = 10):
    """``steps`` distinct mini-batches for each of ``n`` replicas.

    Returns (images ``[steps, n, batch, h, w, c]`` float32, labels ``[steps, n, batch]`` int32).
    """
    means = class_means(seed, n_classes, h, w, c)
    rng = np.random.default_rng([seed, 2002])
    labels = rng.integers(0, n_classes, size=(steps, n, batch)).astype(np.int32)
    noise = rng.standard_normal((steps, n, batch, h, w, c)).astype(np.float32)
    images = means[labels] + noise
    return np.ascontiguousarray(images, dtype=np.float32), labels


def flat_params(seed: int, n: int, n_params: int, std: float = 0.05) -> np.ndarray:
    """Replica parameters for the update-only workload: i.i.d. N(0, std^2), float32 ``[n, n_params]``."""
    rng = np.random.default_rng([seed, 3003])
    out = np.empty((n, n_params), dtype=np.float32)
    for a in range(n):
        out[a] = rng.standard_normal(n_params, dtype=np.float32) * np.float32(std)
    return out


def flat_grads(seed: int, step: int, n: int, n_params: int, std: float = 1e-2) -> np.ndarray:
    """Synthetic gradients for inner update number ``step``: i.i.d. N(0, std^2), float32 ``[n, n_params]``."""
    rng = np.random.default_rng([seed, 4004, step])
    out = np.empty((n, n_params), dtype=np.float32)
    for a in range(n):
        out[a] = rng.standard_normal(n_params, dtype=np.float32) * np.float32(std)
    return out


def init_params(layout, seed: int, weight_init: str = "he_normal") -> np.ndarray:
    """Draw one replica's initial parameters, float32 ``[sum of segment sizes]``.

    ``layout`` is a sequence of dicts with keys ``name``, ``shape``, ``kind`` and
    ``fan_in``.  kind ``weight``: N(0, 2/fan_in) for ``weight_init="he_normal"``
    (keeps the activation scale through ReLU layers; used for the deep
    convolutional networks) or U(-1/sqrt(fan_in), 1/sqrt(fan_in)) for
    ``"uniform"`` (the default initialisation of the framework the paper's
    implementation used; used for the MLP and LeNet, which train stably with it
    at step size 0.1); ``bias``: U(-1/sqrt(fan_in), 1/sqrt(fan_in)); ``bn_gamma``:
    1 + 0.1 N(0,1); ``bn_beta``: 0.1 N(0,1).  Segments are drawn in order from
    one generator, so the vector depends only on (layout, seed, weight_init).
    """
    rng = np.random.default_rng([seed, 5005])
    parts = []
    for seg in layout:
        size = int(np.prod(seg["shape"]))
        kind = seg["kind"]
        fan_in = float(seg["fan_in"])
        if kind == "weight" and weight_init == "uniform":
            b = 1.0 / np.sqrt(fan_in)
            v = rng.uniform(-b, b, size)
        elif kind == "weight" and weight_init == "he_normal":
            v = rng.standard_normal(size) * np.sqrt(2.0 / fan_in)
        elif kind == "weight":
            raise ValueError(f"unknown weight_init {weight_init!r}")
        elif kind == "bias":
            b = 1.0 / np.sqrt(fan_in)
            v = rng.uniform(-b, b, size)
        elif kind == "bn_gamma":
            v = 1.0 + 0.1 * rng.standard_normal(size)
        elif kind == "bn_beta":
            v = 0.1 * rng.standard_normal(size)
        else:
            raise ValueError(f"unknown segment kind {kind!r}")
        parts.append(v.astype(np.float32))
    return np.concatenate(parts) if parts else np.zeros(0, np.float32)


def split_shards(seed: int, n_samples: int, n: int, fraction: float) -> np.ndarray:
    """Index sets of a data set divided between ``n`` replicas (Section 5: every replica sees only a
    subset, all subsets have the same size and every sample lies in at least one of them).

    The samples are permuted once; replica ``a`` takes the cyclic window of ``ceil(fraction * n_samples)``
    permuted samples that starts at ``a * n_samples // n``.  Needs ``n * fraction >= 1`` so that the windows
    cover the set.  Returns int64 ``[n, m]``.
    """
    m = int(np.ceil(fraction * n_samples))
    if n * m < n_samples or m > n_samples:
        raise ValueError("subsets of this size cannot cover the data set")
    perm = np.random.default_rng([seed, 5005]).permutation(n_samples)
    starts = (np.arange(n) * n_samples) // n
    return perm[(starts[:, None] + np.arange(m)[None, :]) % n_samples].astype(np.int64)


def split_image_batches(seed: int, steps: int, n: int, batch: int, h: int, w: int, c: int,
                        n_samples: int, fraction: float, n_classes: int = 10):
    """Mini-batches for ``n`` replicas that each draw from their own subset of one fixed synthetic
    data set of ``n_samples`` class-conditional Gaussian images (Section 5; 50 % for three replicas and
    25 % for six in Table 2).  A replica walks its subset in reshuffled epochs.

    Returns (images ``[steps, n, batch, h, w, c]`` float32, labels ``[steps, n, batch]`` int32,
    sample index ``[steps, n, batch]`` int64, shards ``[n, m]`` int64).
    """
    means = class_means(seed, n_classes, h, w, c)
    rng = np.random.default_rng([seed, 6006])
    all_labels = rng.integers(0, n_classes, size=n_samples).astype(np.int32)
    all_images = means[all_labels] + rng.standard_normal((n_samples, h, w, c)).astype(np.float32)
    shards = split_shards(seed, n_samples, n, fraction)
    m = shards.shape[1]
    index = np.empty((steps, n, batch), dtype=np.int64)
    for a in range(n):
        order_rng = np.random.default_rng([seed, 7007, a])
        need = steps * batch
        walk = np.concatenate([shards[a][order_rng.permutation(m)] for _ in range(-(-need // m))])[:need]
        index[:, a, :] = walk.reshape(steps, batch)
    images = np.ascontiguousarray(all_images[index], dtype=np.float32)
    return images, all_labels[index], index, shards
