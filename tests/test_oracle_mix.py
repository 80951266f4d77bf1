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
    if mix == S.MIX_TRI and L < 3:      # Eq. 9's circulant has three distinct positions per row
        order, partner, active = S.schedule(pattern, 1, 0, L, 0.0)
        with pytest.raises(ValueError):
            S.mixing_matrix(mix, order, partner, active)
        with pytest.raises(ValueError):
            A.mix_update(x, g, mix, order, partner, active, 0.25)
        return
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


# ---- consensus distance -------------------------------------------------------------------------

def test_consensus_distance_is_the_plain_definition():
    # brute force on a tiny case, element by element in Python floats
    x = np.array([[1.0, 2.0, -1.0], [3.0, 2.0, 0.5], [5.0, -4.0, 0.0]], dtype=np.float32)
    tot = 0.0
    for e in range(3):
        mean = sum(float(x[i, e]) for i in range(3)) / 3.0
        tot += sum((float(x[i, e]) - mean) ** 2 for i in range(3))
    assert abs(A.consensus_distance(x) - tot) < 1e-12
    assert A.consensus_distance(np.ones((4, 7), np.float32) * 3.25) == 0.0          # consensus reached
    # shifting every learner by the same vector changes nothing; scaling by c scales by c^2
    r = np.random.default_rng(0)
    y = r.standard_normal((5, 11))
    assert abs(A.consensus_distance(y + r.standard_normal(11)) - A.consensus_distance(y)) < 1e-12
    assert abs(A.consensus_distance(3.0 * y) - 9.0 * A.consensus_distance(y)) < 1e-10


@pytest.mark.parametrize("L", [4, 5, 9, 16])
def test_ring_mixing_contracts_the_consensus_distance_by_the_spectral_bound(L):
    # Section II (Eq. 5-7) with the fixed-ring operator of Eq. 9: without gradients every application of
    # T^f shrinks sum_i ||x_i - xbar||^2 by at least lambda_hat^2, lambda_hat the second largest eigenvalue
    # magnitude of T^f, whose spectrum Eq. 10 gives in closed form: (1 + 2 cos(2 pi j / L)) / 3.
    lam = sorted(abs((1.0 + 2.0 * np.cos(2.0 * np.pi * j / L)) / 3.0) for j in range(L))
    lam_hat = lam[-2]
    ora = A.Oracle(L, S.FIXED_RING, 3, flat_params=400, mix=S.MIX_TRI,
                   x0=np.random.default_rng(L).uniform(-1, 1, (L, 400)).astype(np.float32))
    zero = np.zeros((L, 400), np.float32)
    prev = ora.consensus()
    xbar0 = ora.average()
    for k in range(6):
        ora.step(None, 0.0, grads=zero)
        cur = ora.consensus()
        assert cur <= lam_hat ** 2 * prev * (1 + 1e-5) + 1e-9, (k, cur, prev)
        prev = cur
    assert np.abs(ora.average() - xbar0).max() < 1e-6             # doubly stochastic: the mean stays


def test_allreduce_mixing_has_zero_consensus_distance_after_one_step():
    L = 6
    ora = A.Oracle(L, S.D1D, 1, flat_params=100, tau=0, x0=np.random.default_rng(1).uniform(-1, 1, (L, 100)).astype(np.float32))
    assert ora.consensus() > 1.0
    ora.step(None, 0.0, grads=np.zeros((L, 100), np.float32))
    assert ora.consensus() == 0.0
