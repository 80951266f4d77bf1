"""Seeded synthetic inputs (features, labels, initial models, flat gradients).

This module holds no arithmetic of the method: it only draws the random inputs
that stand in for the acoustic training data, with the shapes of the paper's
workload (21-frame segments of 260-dimensional features, context-dependent
state labels; Section IV) and of the five benchmark configurations.  Both the
tests (which hand the arrays to the CPU oracle and to the HIP library) and the
benchmark use it.
"""
from collections import namedtuple
import numpy as np

Workload = namedtuple(
    "Workload",
    "name L pattern input_dim hidden layers bidirectional bottleneck classes batch frames "
    "flat_params precision init_scale label_dist lr steps straggler_p")

# pattern: 0 fixed ring, 1 random ring, 2 delay-by-one; precision: 0 fp32, 1 bf16 GEMM operands
WORKLOADS = {
    "cfg1": Workload("cfg1", 4, 0, 40, 64, 1, 0, 0, 100, 4, 20, 0, 0, 0.1, "uniform", 0.1, 5, 0.0),
    "cfg2": Workload("cfg2", 8, 1, 120, 256, 2, 1, 0, 1000, 32, 21, 0, 0, 0.05, "uniform", 0.1, 20, 0.0),
    "cfg3": Workload("cfg3", 16, 2, 260, 512, 4, 1, 0, 9000, 64, 21, 0, 1, 0.05, "zipf", 0.1, 20, 0.0),
    "cfg4": Workload("cfg4", 16, 2, 260, 1024, 6, 1, 256, 32000, 128, 21, 0, 1, 0.05, "zipf", 0.1, 10, 0.0),
    "cfg5": Workload("cfg5", 64, 1, 0, 0, 0, 0, 0, 0, 0, 0, 135_000_000, 0, 0.05, "", 0.1, 50, 0.1),
}

_TAG_FEATS, _TAG_LABELS, _TAG_INIT, _TAG_FLATG, _TAG_FLATX = 11, 12, 13, 14, 15


def _rng(seed, *key):
    return np.random.default_rng([int(seed)] + [int(k) for k in key])


def features(seed, step, learner, frames, batch, input_dim):
    """[T][B][I] float32, N(0,1)."""
    return _rng(seed, _TAG_FEATS, step, learner).standard_normal(
        (frames, batch, input_dim), dtype=np.float32)


def zipf_cdf(classes, s=1.1):
    p = (np.arange(classes, dtype=np.float64) + 1.0) ** (-s)
    c = np.cumsum(p)
    return c / c[-1]


def labels(seed, step, learner, frames, batch, classes, dist="uniform", cdf=None):
    """[T][B] int32; uniform over classes, or Zipf(s=1.1) by inverse CDF."""
    r = _rng(seed, _TAG_LABELS, step, learner)
    if dist == "uniform":
        return r.integers(0, classes, size=(frames, batch), dtype=np.int32)
    if cdf is None:
        cdf = zipf_cdf(classes)
    u = r.random((frames, batch))
    return np.minimum(np.searchsorted(cdf, u, side="right"), classes - 1).astype(np.int32)


def initial_model(seed, n, scale):
    """[n] float32, U(-scale, scale): the common initial model w_0."""
    return _rng(seed, _TAG_INIT).uniform(-scale, scale, size=n).astype(np.float32)


def flat_gradient(seed, learner, n, std=1e-3, chunk=None):
    """[n] float32 ~ N(0, std^2) for the model-free stress workload."""
    g = _rng(seed, _TAG_FLATG, learner).standard_normal(n, dtype=np.float32)
    g *= np.float32(std)
    return g


def flat_initial(seed, learner, n, scale=0.05):
    """[n] float32 U(-scale, scale), drawn independently per learner."""
    r = _rng(seed, _TAG_FLATX, learner)
    x = r.random(n, dtype=np.float32)
    x *= np.float32(2 * scale)
    x -= np.float32(scale)
    return x


def batch(wl, seed, step, learner, cdf=None):
    f = features(seed, step, learner, wl.frames, wl.batch, wl.input_dim)
    y = labels(seed, step, learner, wl.frames, wl.batch, wl.classes, wl.label_dist, cdf)
    return f, y
