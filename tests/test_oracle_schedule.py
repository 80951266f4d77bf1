"""Pins for the oracle's schedule generator (CPU only).

Each test checks oracle/schedule.py against something the paper or the
mathematics fixes, not against itself."""
import itertools
import math
import os
import numpy as np
import pytest

from oracle import schedule as S

GOLDEN_DIR = os.path.join(os.path.dirname(__file__), "golden")


def test_splitmix64_published_vectors():
    # First three outputs of the SplitMix64 generator started at state 0
    # (published reference values of that algorithm).
    st, outs = 0, []
    for _ in range(3):
        st = (st + S.GOLDEN) & S.MASK64
        outs.append(S.mix64(st))
    assert outs == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


@pytest.mark.parametrize("pattern", [S.FIXED_RING, S.RANDOM_RING, S.D1D])
@pytest.mark.parametrize("L", [1, 2, 3, 4, 5, 8, 9, 16, 64])
@pytest.mark.parametrize("p", [0.0, 0.3])
def test_pair_matrix_is_symmetric_doubly_stochastic(pattern, L, p):
    # Algorithm 1 requires a doubly stochastic T_k; the matching is an involution.
    for k in range(6):
        order, partner, active = S.schedule(pattern, 7, k, L, p)
        assert sorted(order) == list(range(L))
        for i in range(L):
            assert partner[partner[i]] == i
            if not active[i]:
                assert partner[i] == i
        T = S.mixing_matrix(S.MIX_PAIR, order, partner, active)
        assert (T >= 0).all()
        assert (T.sum(axis=0) == 1.0).all() and (T.sum(axis=1) == 1.0).all()
        assert (T == T.T).all()
        assert set(np.unique(T)) <= {0.0, 0.5, 1.0}


@pytest.mark.parametrize("L", [2, 3, 4, 7, 8, 16])
def test_fixed_ring_matching_follows_the_ring_and_connects_it(L):
    # Partners are ring neighbours; two consecutive iterations connect the whole
    # ring (a single unit eigenvalue of the product), so consensus is reachable.
    Ts = []
    for k in range(2):
        order, partner, active = S.schedule(S.FIXED_RING, 0, k, L)
        assert order == list(range(L))
        for i in range(L):
            assert partner[i] == i or (partner[i] - i) % L in (1, L - 1)
        n_self = sum(partner[i] == i for i in range(L))
        assert n_self == (L % 2)
        Ts.append(S.mixing_matrix(S.MIX_PAIR, order, partner, active))
    ev = np.sort(np.abs(np.linalg.eigvals(Ts[0] @ Ts[1])))
    assert abs(ev[-1] - 1.0) < 1e-12
    if L > 2:
        assert ev[-2] < 1.0 - 1e-6


def test_fisher_yates_is_uniform_over_all_permutations():
    # Section III-C: sigma is a uniformly random permutation. Chi-square over the
    # 24 permutations of L=4 from 24000 iterations (dof 23; 99.99% quantile ~ 57).
    L, n = 4, 24000
    counts = {p: 0 for p in itertools.permutations(range(L))}
    for k in range(n):
        counts[tuple(S.ring_order(S.RANDOM_RING, 12345, k, L))] += 1
    exp = n / 24.0
    chi2 = sum((c - exp) ** 2 / exp for c in counts.values())
    assert chi2 < 57.0
    assert min(counts.values()) > 0


def test_mask_rate_and_independence_of_permutation_stream():
    L, n, p = 64, 400, 0.1
    tot = sum(sum(S.active_mask(3, k, L, p)) for k in range(n))
    rate = 1.0 - tot / (L * n)
    assert abs(rate - p) < 4 * math.sqrt(p * (1 - p) / (L * n))
    # the ring order does not depend on the mask probability
    assert S.schedule(S.RANDOM_RING, 3, 5, L, 0.0)[0] == S.schedule(S.RANDOM_RING, 3, 5, L, 0.5)[0]


@pytest.mark.parametrize("L", [6, 8, 16, 64])
def test_tri_fixed_matrix_eigenvalues_closed_form(L):
    # Appendix A: eigenvalues of the circulant T^f are 1/3 + 2/3 cos(2 pi k / L);
    # Eq. for lambda-hat in Section III-B.
    order, partner, active = S.schedule(S.FIXED_RING, 0, 0, L)
    T = S.mixing_matrix(S.MIX_TRI, order, partner, active)
    assert np.allclose(T.sum(axis=0), 1) and np.allclose(T.sum(axis=1), 1)
    assert np.allclose(T[0, [0, 1, L - 1]], 1.0 / 3.0) and np.count_nonzero(T[0]) == 3
    ev = np.sort(np.linalg.eigvalsh(T))
    ref = np.sort([1 / 3 + 2 / 3 * math.cos(2 * math.pi * k / L) for k in range(L)])
    assert np.allclose(ev, ref, atol=1e-12)
    lam_hat = 1 / 3 + 2 / 3 * math.cos(2 * math.pi / L)
    assert abs(np.sort(np.abs(ev))[-2] - lam_hat) < 1e-12
    # bound on the distance to consensus after t steps (Section III-A/B)
    U = np.full((L, L), 1.0 / L)
    Tt = np.eye(L)
    for t in range(1, 12):
        Tt = Tt @ T
        assert np.linalg.norm(Tt - U, 2) <= lam_hat ** t + 1e-12


def test_tri_gram_matrix_first_row():
    # Appendix B prints T^f' T^f: first row (3,2,1,0,...,0,1,2)/9 for L > 5.
    L = 9
    order, partner, active = S.schedule(S.FIXED_RING, 0, 0, L)
    T = S.mixing_matrix(S.MIX_TRI, order, partner, active)
    G = T.T @ T
    ref = np.zeros(L)
    ref[[0, 1, 2, L - 2, L - 1]] = np.array([3, 2, 1, 1, 2]) / 9.0
    assert np.allclose(G[0], ref, atol=1e-15)
    assert np.allclose(G[1], np.roll(ref, 1), atol=1e-15)


def test_tri_random_ring_expected_gram_and_consensus_bound():
    # Appendix B: E[T^r' T^r] has 1/3 on the diagonal and 2/(3(L-1)) elsewhere;
    # Section III-C bound E||prod T^r - 11'/L||_2 <= sqrt(L-1)/sqrt(3)^k.
    L, n = 8, 6000
    acc = np.zeros((L, L))
    for k in range(n):
        order, partner, active = S.schedule(S.RANDOM_RING, 99, k, L)
        T = S.mixing_matrix(S.MIX_TRI, order, partner, active)
        assert np.allclose(T, T.T)
        acc += T.T @ T
    E = acc / n
    assert np.allclose(np.diag(E), 1.0 / 3.0, atol=1e-12)   # holds for every permutation
    off = E[~np.eye(L, dtype=bool)]
    assert abs(off.mean() - 2.0 / (3 * (L - 1))) < 1e-12
    assert np.abs(off - 2.0 / (3 * (L - 1))).max() < 0.01     # Monte-Carlo, pins uniformity
    U = np.full((L, L), 1.0 / L)
    steps, runs = 8, 300
    norms = np.zeros(steps)
    for r in range(runs):
        Pm = np.eye(L)
        for k in range(steps):
            order, partner, active = S.schedule(S.RANDOM_RING, 1000 + r, k, L)
            Pm = Pm @ S.mixing_matrix(S.MIX_TRI, order, partner, active)
            norms[k] += np.linalg.norm(Pm - U, 2)
    norms /= runs
    for k in range(steps):
        assert norms[k] <= math.sqrt(L - 1) / math.sqrt(3) ** (k + 1) * 1.02


@pytest.mark.parametrize("L", [16, 32, 64])
def test_decay_to_consensus_at_the_learner_counts_of_the_figure(L):
    # Section IV (the figure on convergence speed to consensus, L = 16, 32, 64): the fixed ring's distance
    # to consensus is exactly lambda-hat^k (T^f is symmetric, so the bound of Section III-B is attained),
    # the random ring's mean distance stays below sqrt(L-1)/sqrt(3)^k (Section III-C) and falls below
    # the fixed ring's within a few iterations; allreduce is at consensus after one.
    U = np.full((L, L), 1.0 / L)
    lam_hat = 1 / 3 + 2 / 3 * math.cos(2 * math.pi / L)
    order, partner, active = S.schedule(S.FIXED_RING, 0, 0, L)
    Tf = S.mixing_matrix(S.MIX_TRI, order, partner, active)
    steps, runs = 10, 30
    fixed = np.zeros(steps)
    Pf = np.eye(L)
    for k in range(steps):
        Pf = Pf @ Tf
        fixed[k] = np.linalg.norm(Pf - U, 2)
        assert abs(fixed[k] - lam_hat ** (k + 1)) < 1e-12
    rand = np.zeros(steps)
    for r in range(runs):
        Pm = np.eye(L)
        for k in range(steps):
            order, partner, active = S.schedule(S.RANDOM_RING, 500 + r, k, L)
            Pm = Pm @ S.mixing_matrix(S.MIX_TRI, order, partner, active)
            rand[k] += np.linalg.norm(Pm - U, 2) / runs
    for k in range(steps):
        assert rand[k] <= math.sqrt(L - 1) / math.sqrt(3) ** (k + 1) * 1.05
    assert rand[-1] < 0.1 * fixed[-1]              # random mixing is far ahead after ten iterations
    order, partner, active = S.schedule(S.D1D, 0, 0, L)
    assert np.linalg.norm(S.mixing_matrix(S.MIX_ALL, order, partner, active) - U, 2) < 1e-15


def test_given_straggler_mask_follows_the_same_unmatching_rule():
    # a learner observed to be late (Section IV-D) instead of a drawn one: same ring order and matching, the
    # straggler and its partner are unmatched, the matrix stays symmetric and doubly stochastic
    L = 8
    for pattern in (S.FIXED_RING, S.RANDOM_RING):
        for k in range(4):
            o0, p0, a0 = S.schedule(pattern, 7, k, L)
            mask = [1] * L
            mask[3] = 0
            o1, p1, a1 = S.schedule(pattern, 7, k, L, active=mask)
            assert o1 == o0 and a1 == mask
            j = p0[3]
            assert p1[3] == 3 and p1[j] == j
            assert all(p1[i] == p0[i] for i in range(L) if i not in (3, j))
            T = S.mixing_matrix(S.MIX_PAIR, o1, p1, a1)
            assert np.allclose(T, T.T) and np.allclose(T.sum(axis=0), 1) and T[3, 3] == 1.0
    # a drawn mask handed back in gives the drawn schedule
    o, p, a = S.schedule(S.RANDOM_RING, 5, 2, L, 0.4)
    assert S.schedule(S.RANDOM_RING, 5, 2, L, 0.0, active=a) == (o, p, a)
    with pytest.raises(ValueError):
        S.schedule(S.FIXED_RING, 0, 0, L, active=[1] * (L - 1))


def test_all_matrix_is_uniform():
    order, partner, active = S.schedule(S.D1D, 0, 3, 16)
    T = S.mixing_matrix(S.MIX_ALL, order, partner, active)
    assert (T == 1.0 / 16).all()


def test_stored_schedule_vectors():
    # The paper defines no partner sequence; these vectors were written by
    # tests/golden/make_schedule_vectors.py (oracle only) and pin the generator
    # against accidental change.  The HIP library is compared with them too.
    path = os.path.join(GOLDEN_DIR, "schedule_vectors.txt")
    with open(path) as fh:
        rows = [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]
    assert rows
    for row in rows:
        pattern, seed, k, L, p = int(row[0]), int(row[1]), int(row[2]), int(row[3]), float(row[4])
        vals = list(map(int, row[5:]))
        order, partner, active = S.schedule(pattern, seed, k, L, p)
        assert vals == order + partner + active
