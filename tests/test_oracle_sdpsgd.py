"""Pins of the oracle's synchronous baseline (SDPSGD: Section III-A, Algorithm 2): every learner
updates its own model, then all models are averaged, W_{k+1} = (W_k - a g(W_k)) 11'/L."""
import numpy as np
import pytest

from oracle import schedule as S
from oracle import adpsgd as A
from oracle import lstm
from oracle.lstm import Shape
from paper_2110_11199_amd import synth


def _rand(L, P, seed=0):
    r = np.random.default_rng(seed)
    return r.uniform(-1, 1, (L, P)).astype(np.float32), r.standard_normal((L, P)).astype(np.float32)


@pytest.mark.parametrize("L", [1, 2, 5, 16])
def test_equals_dense_product_with_the_averaging_matrix(L):
    # brute force in float64: (W - a G) T with T = 11'/L, rows = learners
    x, g = _rand(L, 257, L)
    order, partner, active = S.schedule(S.SDPSGD, 0, 0, L)
    y = A.mix_update(x, g, S.MIX_ALL, order, partner, active, 0.25, update_first=True)
    T = S.mixing_matrix(S.MIX_ALL, order, partner, active)
    ref = T @ (x.astype(np.float64) - 0.25 * g.astype(np.float64))
    assert np.abs(y - ref).max() < 1e-6
    # the other order of the same operations (mix, then update) is a different model per learner
    z = A.mix_update(x, g, S.MIX_ALL, order, partner, active, 0.25)
    if L > 1:
        assert np.abs(z - y).max() > 1e-2
    # ... whose learner average is the synchronous model (T is doubly stochastic)
    assert np.abs(z.astype(np.float64).mean(0) - y[0]).max() < 1e-6


def test_all_learners_hold_the_same_model_after_every_iteration():
    L, P = 8, 300
    x0, g = _rand(L, P, 3)
    o = A.Oracle(L, S.SDPSGD, 0, flat_params=P, x0=x0)
    assert o.mix == S.MIX_ALL and o.tau == 0 and o.update_first
    for k in range(3):
        o.step(None, 0.1, grads=g * np.float32(k + 1))
        for i in range(1, L):
            assert (o.x[i].view(np.uint32) == o.x[0].view(np.uint32)).all()
        assert o.consensus() == 0.0


def test_model_averaging_is_gradient_averaging_exactly_on_dyadic_data():
    # Section III-A: for plain SGD, averaging the updated models is SGD with the averaged gradient.
    # With a common model, lr = 1/2, L = 8 and gradients that are small multiples of 2^-8 every
    # operation is exact in float32, so the two sides agree bit for bit.
    L, P = 8, 512
    r = np.random.default_rng(1)
    w = (r.integers(-2048, 2048, P) / 256.0).astype(np.float32)
    g = (r.integers(-512, 512, (L, P)) / 256.0).astype(np.float32)
    o = A.Oracle(L, S.SDPSGD, 0, flat_params=P, w0=w)
    o.step(None, 0.5, grads=g)
    gbar = g.astype(np.float64).mean(0)
    ref = (w.astype(np.float64) - 0.5 * gbar).astype(np.float32)
    assert (ref.astype(np.float64) == w.astype(np.float64) - 0.5 * gbar).all()     # representable
    assert (o.x[0] == ref).all()


def test_single_learner_is_plain_sgd():
    x, g = _rand(1, 100, 9)
    order, partner, active = S.schedule(S.SDPSGD, 0, 0, 1)
    y = A.mix_update(x, g, S.MIX_ALL, order, partner, active, 0.1, update_first=True)
    assert (y[0] == x[0] - np.float32(0.1) * g[0]).all()


def test_rejects_what_the_baseline_does_not_define():
    with pytest.raises(ValueError):
        A.Oracle(4, S.SDPSGD, 0, flat_params=8, w0=np.zeros(8, np.float32), straggler_p=0.1)
    with pytest.raises(ValueError):
        A.Oracle(4, S.SDPSGD, 0, flat_params=8, w0=np.zeros(8, np.float32), tau=1)
    with pytest.raises(ValueError):
        A.Oracle(4, S.SDPSGD, 0, flat_params=8, w0=np.zeros(8, np.float32), mix=S.MIX_PAIR)
    x, g = _rand(4, 8)
    with pytest.raises(ValueError):
        A.mix_update(x, g, S.MIX_ALL, [0, 1, 2, 3], [0, 1, 2, 3], [1, 0, 1, 1], 0.1, update_first=True)


def test_L_learners_of_batch_B_are_one_learner_of_batch_LB():
    # With identical models the mean of the learners' minibatch gradients is the gradient of the mean
    # loss over all L*B segments, so the synchronous baseline on L learners follows plain SGD of a
    # single learner on the concatenated batch (Section III-A; Algorithm 1's 1/M mean).
    L, steps, lr = 4, 3, 0.3
    small = Shape(6, 5, 1, 1, 0, 7, 3, 4)
    big = Shape(6, 5, 1, 1, 0, 7, 3 * L, 4)
    P = lstm.param_count(small)
    assert P == lstm.param_count(big)
    w0 = synth.initial_model(4, P, 0.3)
    many = A.Oracle(L, S.SDPSGD, 0, shape=small, w0=w0)
    one = A.Oracle(1, S.FIXED_RING, 0, shape=big, w0=w0)
    for k in range(steps):
        b = [(synth.features(0, k, i, 4, 3, 6), synth.labels(0, k, i, 4, 3, 7)) for i in range(L)]
        many.step(b, lr)
        cat = (np.concatenate([f for f, _ in b], axis=1), np.concatenate([y for _, y in b], axis=1))
        one.step([cat], lr)
        assert np.abs(many.x[0] - one.x[0]).max() < 2e-6, k
        assert abs(float(np.mean(many.last_losses)) - float(one.last_losses[0])) < 1e-5
