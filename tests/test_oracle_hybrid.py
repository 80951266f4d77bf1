"""Pins for the oracle's hybrid (super-learner) mixing and learning-rate schedules (CPU only).

Hybrid strategy (Section V): synchronous mean inside super-learners of S learners, the asynchronous ring
across the G = L/S super-learners.  Its matrix is the Kronecker product of the ring operator over G
positions with 11'/S, so its spectrum is the ring's spectrum (Eq. 10 for the fixed ring with weights 1/3)
padded with zeros: that, double stochasticity, the dense product and the two ends S = 1 (the plain ring)
and S = L (the all-learner mean) pin it."""
import math
import os

import numpy as np
import pytest

from oracle import schedule as S
from oracle import adpsgd as A
from oracle import lr as LR

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rand(L, P, seed=0):
    r = np.random.default_rng(seed)
    return (r.uniform(-1, 1, (L, P)).astype(np.float32), (r.standard_normal((L, P)) * 1e-2).astype(np.float32))


CASES = [(S.MIX_HYBRID_PAIR, S.FIXED_RING, 8, 2), (S.MIX_HYBRID_PAIR, S.RANDOM_RING, 12, 4), (S.MIX_HYBRID_PAIR, S.RANDOM_RING, 10, 2),
         (S.MIX_HYBRID_PAIR, S.FIXED_RING, 6, 3), (S.MIX_HYBRID_TRI, S.FIXED_RING, 12, 4), (S.MIX_HYBRID_TRI, S.RANDOM_RING, 15, 3),
         (S.MIX_HYBRID_TRI, S.RANDOM_RING, 16, 2), (S.MIX_HYBRID_TRI, S.FIXED_RING, 5, 5), (S.MIX_HYBRID_PAIR, S.FIXED_RING, 7, 1)]


@pytest.mark.parametrize("mix,pattern,L,Sz", CASES)
def test_hybrid_matrix_is_doubly_stochastic_symmetric_and_matches_the_update(mix, pattern, L, Sz):
    G = L // Sz
    x, g = _rand(L, 41, L)
    for k in range(4):
        order, partner, active = S.schedule(pattern, 5, k, G)
        T = S.mixing_matrix(mix, order, partner, active, Sz)
        assert T.shape == (L, L)
        assert np.allclose(T.sum(axis=0), 1, atol=1e-15) and np.allclose(T.sum(axis=1), 1, atol=1e-15)
        assert np.allclose(T, T.T) and (T >= 0).all()
        # Kronecker structure: ring operator over super-learners, spread evenly over the S x S blocks
        Tg = np.ones((1, 1)) if G == 1 else S.mixing_matrix(S.ring_mix_of(mix), order, partner, active)
        assert np.allclose(T, np.kron(Tg, np.full((Sz, Sz), 1.0 / Sz)), atol=1e-15)
        got = A.mix_update(x, g, mix, order, partner, active, 0.25, group_size=Sz)
        ref = T @ x.astype(np.float64) - 0.25 * g.astype(np.float64)
        assert np.abs(got - ref).max() < 5e-7
        x = got


@pytest.mark.parametrize("L,Sz", [(16, 1), (16, 2), (16, 4), (24, 4), (12, 12)])
def test_hybrid_fixed_ring_spectrum_is_eq10_over_the_super_learners_padded_with_zeros(L, Sz):
    G = L // Sz
    order, partner, active = S.schedule(S.FIXED_RING, 0, 0, G)
    T = S.mixing_matrix(S.MIX_HYBRID_TRI, order, partner, active, Sz)
    ev = np.sort(np.linalg.eigvalsh(T))
    ring = [1 / 3 + 2 / 3 * math.cos(2 * math.pi * m / G) for m in range(G)] if G > 1 else [1.0]
    ref = np.sort(ring + [0.0] * (L - G))
    assert np.allclose(ev, ref, atol=1e-12)
    if Sz == 1:      # no hierarchy: the paper's T^f itself
        assert np.allclose(T, S.mixing_matrix(S.MIX_TRI, order, partner, active), atol=1e-15)
    if G == 1:       # one super-learner: allreduce over everybody
        assert np.allclose(T, np.full((L, L), 1.0 / L), atol=1e-15)


def test_second_eigenvalue_shrinks_as_super_learners_grow():
    # fewer, larger super-learners: a shorter ring, a larger spectral gap (Eq. 10 with L replaced by G)
    L = 48
    lam = []
    for Sz in (1, 2, 4, 8, 16):
        G = L // Sz
        order, partner, active = S.schedule(S.FIXED_RING, 0, 0, G)
        ev = np.sort(np.abs(np.linalg.eigvalsh(S.mixing_matrix(S.MIX_HYBRID_TRI, order, partner, active, Sz))))
        lam.append(ev[-2])
        assert abs(ev[-2] - abs(1 / 3 + 2 / 3 * math.cos(2 * math.pi / G))) < 1e-12
    assert all(a > b for a, b in zip(lam, lam[1:]))


@pytest.mark.parametrize("mix,ring", [(S.MIX_HYBRID_PAIR, S.MIX_PAIR), (S.MIX_HYBRID_TRI, S.MIX_TRI)])
def test_hybrid_ends_are_the_plain_ring_and_the_global_mean_bit_for_bit(mix, ring):
    L = 9
    x, g = _rand(L, 300, 3)
    order, partner, active = S.schedule(S.RANDOM_RING, 8, 2, L)
    a = A.mix_update(x, g, mix, order, partner, active, 0.3, group_size=1)
    b = A.mix_update(x, g, ring, order, partner, active, 0.3)
    assert (a.view(np.uint32) == b.view(np.uint32)).all()
    order1, partner1, active1 = S.schedule(S.RANDOM_RING, 8, 2, 1)
    c = A.mix_update(x, g, mix, order1, partner1, active1, 0.3, group_size=L)
    d = A.mix_update(x, g, S.MIX_ALL, order, partner, active, 0.3)
    assert (c.view(np.uint32) == d.view(np.uint32)).all()


def test_hybrid_mixing_alone_makes_a_super_learner_identical_and_keeps_the_average():
    L, Sz = 12, 3
    x, g = _rand(L, 500, 1)
    order, partner, active = S.schedule(S.RANDOM_RING, 3, 0, L // Sz)
    y = A.mix_update(x, g, S.MIX_HYBRID_TRI, order, partner, active, 0.0, group_size=Sz)
    for a in range(L // Sz):
        for i in range(a * Sz + 1, (a + 1) * Sz):
            assert (y[i].view(np.uint32) == y[a * Sz].view(np.uint32)).all()
    assert np.abs(y.astype(np.float64).mean(0) - x.astype(np.float64).mean(0)).max() < 3e-7
    # exact in dyadic arithmetic: integers scaled by 2^-6, super-learners of 4, pairwise ring
    r = np.random.default_rng(0)
    xi = (r.integers(-64, 64, (8, 50)) * 2.0 ** -6).astype(np.float32)
    order, partner, active = S.schedule(S.FIXED_RING, 0, 1, 2)
    yi = A.mix_update(xi, np.zeros_like(xi), S.MIX_HYBRID_PAIR, order, partner, active, 0.0, group_size=4)
    assert (yi == xi.astype(np.float64).mean(0).astype(np.float32)).all()      # two matched super-learners: global mean


def test_hybrid_rejects_what_it_is_not_defined_for():
    x, g = _rand(8, 5)
    order, partner, active = S.schedule(S.FIXED_RING, 0, 0, 2)
    with pytest.raises(ValueError):       # a ring of two super-learners has no distinct left and right neighbour
        A.mix_update(x, g, S.MIX_HYBRID_TRI, order, partner, active, 0.1, group_size=4)
    with pytest.raises(ValueError):       # 8 learners are not 2 x 3
        A.mix_update(x, g, S.MIX_HYBRID_PAIR, order, partner, active, 0.1, group_size=3)
    with pytest.raises(ValueError):
        A.Oracle(8, S.D1D, 0, flat_params=5, x0=x, mix=S.MIX_HYBRID_PAIR, group_size=2)
    with pytest.raises(ValueError):
        A.Oracle(8, S.FIXED_RING, 0, flat_params=5, x0=x, mix=S.MIX_HYBRID_PAIR, group_size=2, straggler_p=0.1)


def test_hybrid_recurrence_runs_on_the_super_learner_schedule():
    L, Sz, P = 8, 2, 64
    x, g = _rand(L, P, 9)
    ora = A.Oracle(L, S.RANDOM_RING, 4, flat_params=P, x0=x, mix=S.MIX_HYBRID_PAIR, group_size=Sz)
    cur = x
    for k in range(3):
        ora.step(None, 0.1, grads=g)
        order, partner, active = S.schedule(S.RANDOM_RING, 4, k, L // Sz)
        assert ora.last_schedule == (order, partner, active)
        cur = A.mix_update(cur, g, S.MIX_HYBRID_PAIR, order, partner, active, 0.1, group_size=Sz)
        assert (cur.view(np.uint32) == ora.x.view(np.uint32)).all()


def test_learning_rate_schedules_give_the_papers_numbers():
    with open(os.path.join(GOLDEN, "lr_schedule_paper.txt")) as fh:
        rows = [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 10
    for name, epoch, rate in rows:
        if name == "baseline":
            got = LR.lr_at_epoch(int(epoch), 0.1)
        else:
            got = LR.lr_at_epoch(int(epoch), 3.2, start=0.32, warmup_epochs=10, hold_until=10)
        assert abs(got - float(rate)) < 1e-12 * max(1.0, float(rate)), (name, epoch, got)
    # the anneal factor between consecutive epochs after the hold is 1/sqrt(2); the warm-up is linear
    for e in range(11, 16):
        assert abs(LR.lr_at_epoch(e + 1, 0.1) / LR.lr_at_epoch(e, 0.1) - 1 / math.sqrt(2)) < 1e-15
    w = [LR.lr_at_epoch(e, 3.2, start=0.32, warmup_epochs=10) for e in range(1, 11)]
    assert np.allclose(np.diff(w), 0.32, atol=1e-12)
    assert LR.lr_at_epoch(11, 3.2, start=0.32, warmup_epochs=10) == pytest.approx(3.2 / math.sqrt(2), rel=1e-15)
    with pytest.raises(ValueError):
        LR.lr_at_epoch(0, 0.1)
