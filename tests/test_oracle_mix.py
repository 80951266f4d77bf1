"""Pins for the oracle's mixing + update step and the recurrence (CPU only)."""
import numpy as np
import pytest

from oracle import schedule as S
from oracle import adpsgd as A


def _rand(L, P, seed=0):
    r = np.random.default_rng(seed)
    return (r.uniform(-1, 1, (L, P)).astype(np.float32),
            (r.standard_normal((L, P)) * 1e-2).astype(np.float32))


@pytest.mark.parametrize("mix,pattern", [(S.MIX_PAIR, S.FIXED_RING), (S.MIX_PAIR, S.RANDOM_RING),
                                         (S.MIX_TRI, S.FIXED_RING), (S.MIX_TRI, S.RANDOM_RING),
                                         (S.MIX_ALL, S.D1D)])
@pytest.mark.parametrize("L", [1, 2, 3, 5, 8])
def test_mixing_equals_dense_matrix_product(mix, pattern, L):
    # Eq. 2: the mixed models are the rows of T_k applied to the learners' models.
    x, g = _rand(L, 37, L)
    for k in range(4):
        p = 0.3 if mix == S.MIX_PAIR else 0.0
        order, partner, active = S.schedule(pattern, 1, k, L, p)
        T = S.mixing_matrix(mix, order, partner, active)
        got = A.mix_update(x, g, mix, order, partner, active, 0.25)
        ref = T @ x.astype(np.float64) - 0.25 * g.astype(np.float64) * np.array(active)[:, None]
        assert np.abs(got - ref).max() < 4e-7
        x = got


@pytest.mark.parametrize("mix,pattern", [(S.MIX_PAIR, S.RANDOM_RING), (S.MIX_ALL, S.D1D)])
def test_mixing_preserves_the_learner_average(mix, pattern):
    # Columns of T_k sum to one, so mixing alone (lr = 0) keeps the average.
    L = 8
    x, g = _rand(L, 1000)
    order, partner, active = S.schedule(pattern, 2, 0, L, 0.2 if mix == S.MIX_PAIR else 0.0)
    y = A.mix_update(x, g, mix, order, partner, active, 0.0)
    assert np.abs(y.astype(np.float64).mean(0) - x.astype(np.float64).mean(0)).max() < 2e-7


def test_pair_mix_only_is_exact_pair_mean_and_stragglers_are_untouched():
    L = 8
    x, g = _rand(L, 500)
    order, partner, active = S.schedule(S.RANDOM_RING, 11, 3, L, 0.4)
    assert 0 < sum(active) < L
    y = A.mix_update(x, g, S.MIX_PAIR, order, partner, active, 0.5)
    for i in range(L):
        if not active[i]:
            assert (y[i].view(np.uint32) == x[i].view(np.uint32)).all()
    y0 = A.mix_update(x, g, S.MIX_PAIR, order, partner, active, 0.0)
    for i in range(L):
        j = partner[i]
        if j != i:
            # (a+b)/2 in float32 is the correctly rounded mean (no overflow here)
            ref = ((x[i].astype(np.float64) + x[j].astype(np.float64)) / 2).astype(np.float32)
            assert (y0[i] == ref).all() and (y0[i].view(np.uint32) == y0[j].view(np.uint32)).all()


def test_allreduce_mixing_reaches_consensus_in_one_step():
    # Section III-A: T = 11'/L gives identical local models after one averaging.
    L = 16
    x, g = _rand(L, 300)
    order, partner, active = S.schedule(S.D1D, 0, 0, L)
    y = A.mix_update(x, g, S.MIX_ALL, order, partner, active, 0.0)
    for i in range(1, L):
        assert (y[i].view(np.uint32) == y[0].view(np.uint32)).all()
    assert np.abs(y[0] - x.astype(np.float64).mean(0)).max() < 2e-7


def test_single_learner_is_plain_sgd():
    x, g = _rand(1, 200)
    for pattern, mix in [(S.FIXED_RING, S.MIX_PAIR), (S.RANDOM_RING, S.MIX_PAIR), (S.D1D, S.MIX_ALL)]:
        order, partner, active = S.schedule(pattern, 0, 0, 1)
        y = A.mix_update(x, g, mix, order, partner, active, 0.1)
        ref = x[0] - np.float32(0.1) * g[0]
        assert (y[0] == ref).all()


def test_model_averaging_equals_gradient_averaging_for_plain_sgd():
    # Section III-A: with identical models and T = 11'/L one step of model
    # averaging is SGD with the averaged gradient.
    L, P = 8, 400
    r = np.random.default_rng(0)
    w = r.uniform(-1, 1, P).astype(np.float32)
    g = r.standard_normal((L, P)).astype(np.float32)
    o = A.Oracle(L, S.D1D, 0, flat_params=P, w0=w)
    o.step(None, 0.1, grads=g)
    ref = w.astype(np.float64) - 0.1 * g.astype(np.float64).mean(0)
    assert np.abs(o.average() - ref).max() < 1e-6
    # and the next mixing makes every learner equal that model
    o.step(None, 0.0, grads=np.zeros_like(g))
    assert np.abs(o.x - ref).max() < 1e-6


def test_consensus_speed_ordering():
    # Sections III-B/C/D: allreduce reaches consensus in one step, the random
    # ring mixes faster than the fixed ring.
    L, P, n = 16, 64, 12
    x0 = np.random.default_rng(5).uniform(-1, 1, (L, P)).astype(np.float32)
    zeros = np.zeros((L, P), np.float32)
    dist = {}
    for name, pattern, mix in [("fm", S.FIXED_RING, S.MIX_PAIR), ("rm", S.RANDOM_RING, S.MIX_PAIR),
                               ("d1d", S.D1D, S.MIX_ALL)]:
        o = A.Oracle(L, pattern, 3, flat_params=P, x0=x0, mix=mix, tau=0)
        for _ in range(n):
            o.step(None, 0.0, grads=zeros)
        xd = o.x.astype(np.float64)
        dist[name] = ((xd - xd.mean(0)) ** 2).sum()
    assert dist["d1d"] < 1e-10 < dist["rm"] < dist["fm"]


def test_init_model_generator_range_and_mean():
    w = A.init_model(0, 4000, 0.1)
    assert w.dtype == np.float32 and np.abs(w).max() <= 0.1
    assert abs(w.mean()) < 0.01 and abs(w.std() - 0.1 / np.sqrt(3)) < 0.005
