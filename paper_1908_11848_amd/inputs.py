"""Seeded synthetic inputs: iteration-time tables, mini-batches, initial weights.

This module holds no arithmetic of the method.  Everything it produces is
handed, as plain arrays, both to the library and to whatever it is checked
against, so neither side draws random numbers of its own.

The data stand in for CIFAR-10 / CIFAR-100 (Sec. V-A2): same shape (32x32x3
images, 10 or 100 classes), same mini-batch size as Sec. V-B (128), pixel
values ~ N(0,1), labels uniform.  Iteration-time tables stand in for the
paper's clusters: homogeneous (Sec. V-A1) and mixed-GPU (Sec. V-C).
"""

import numpy as np

BASE_SEED = 190811848
TICKS_PER_UNIT = 1_000_000          # 1 tick = 1e-6 of the nominal iteration time

# purposes
WEIGHTS, DATA, LABELS, MULTIPLIERS, JITTER, GRADS = 0, 1, 2, 3, 4, 5

# kinds of a parameter segment
KIND_WEIGHT, KIND_BIAS, KIND_GAMMA, KIND_BETA = 0, 1, 2, 3


def rng(config, purpose):
    return np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * config + purpose))


def to_ticks(d):
    return np.maximum(np.rint(np.asarray(d, dtype=np.float64) * TICKS_PER_UNIT), 1).astype(np.int64)


def durations(config, K, n, jittered=False):
    """int64 [K][n] ticks for the numbered workload configuration (1..5)."""
    if config == 1:      # 1.0 * (1 + 0.1 z), z ~ N(0,1)
        z = rng(1, JITTER).standard_normal((K, n))
        return to_ticks(np.maximum(1.0 * (1.0 + 0.1 * z), 0.05))
    if config == 2:      # homogeneous, +-5 % uniform jitter
        return to_ticks(rng(2, JITTER).uniform(0.95, 1.05, (K, n)))
    if config == 3:      # heterogeneous 1, 1, 2, 3.5 with lognormal(0, 0.1) jitter
        m = np.array([1.0, 1.0, 2.0, 3.5])[:K]
        if K > 4:
            m = np.concatenate([m, rng(3, MULTIPLIERS).uniform(1.0, 3.5, K - 4)])
        z = rng(3, JITTER).standard_normal((K, n))
        return to_ticks(m[:, None] * np.exp(0.1 * z))
    if config == 4:      # multipliers drawn once, uniform in [1, 2.5]
        m = rng(4, MULTIPLIERS).uniform(1.0, 2.5, K)
        d = np.repeat(m[:, None], n, axis=1)
        if jittered:
            d = d * np.exp(0.1 * rng(4, JITTER).standard_normal((K, n)))
        return to_ticks(d)
    if config == 5:      # multipliers uniform in [1, 4], lognormal jitter
        m = rng(5, MULTIPLIERS).uniform(1.0, 4.0, K)
        z = rng(5, JITTER).standard_normal((K, n))
        return to_ticks(m[:, None] * np.exp(0.1 * z))
    raise ValueError(config)


def batches(config, K, pool, m, n_classes, flat=False):
    """xs[p][j] float32 [m,32,32,3] (or [m,3072]), ys[p][j] int32 [m]."""
    gx, gy = rng(config, DATA), rng(config, LABELS)
    xs = [[gx.standard_normal((m, 32, 32, 3), dtype=np.float32) for _ in range(pool)] for _ in range(K)]
    ys = [[gy.integers(0, n_classes, m).astype(np.int32) for _ in range(pool)] for _ in range(K)]
    if flat:
        xs = [[x.reshape(m, -1) for x in row] for row in xs]
    return xs, ys


def init_weights(segments, config, jitter=0.0):
    """segments: [(kind, size, fan_in)] in flat order -> float32 vector.
    Weights ~ N(0, 2/fan_in); gamma = 1, beta = bias = 0, each plus
    jitter * N(0,1) (tests use jitter > 0 so that no term is hidden by a zero)."""
    g = rng(config, WEIGHTS)
    parts = []
    for kind, size, fan_in in segments:
        z = g.standard_normal(size)
        if kind == KIND_WEIGHT:
            v = z * np.sqrt(2.0 / fan_in)
        elif kind == KIND_GAMMA:
            v = 1.0 + jitter * z
        else:
            v = jitter * z
        parts.append(v.astype(np.float32))
    return np.concatenate(parts)


def stress_grads(K, n, sigma=1e-3):
    """One fixed gradient buffer per worker, ~ N(0, sigma^2), float32 [K][n]."""
    g = rng(5, GRADS)
    return [g.standard_normal(n, dtype=np.float32) * np.float32(sigma) for _ in range(K)]


def stress_weights(n):
    return rng(5, WEIGHTS).standard_normal(n, dtype=np.float32)
