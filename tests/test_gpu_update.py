"""GPU: the fused mixing + SGD update in model-free mode, bit-exact against the oracle."""
import numpy as np
import pytest

from oracle import schedule as S
from oracle import adpsgd as A

pytestmark = pytest.mark.gpu


def _run(L, P, pattern, steps, p=0.0, mix=None, tau=None, seed=3, lr=0.1, group_size=0, tune=()):
    import torch
    from paper_2110_11199_amd import binding as Bd
    r = np.random.default_rng(seed)
    x0 = r.uniform(-0.05, 0.05, (L, P)).astype(np.float32)
    x0[0, : min(P, 3)] = [1e-39, -0.0, 1e38][: min(P, 3)]        # a denormal, a signed zero, a huge value (three of
    #                                                               them still sum below the float32 maximum)
    g = (r.standard_normal((L, P)) * 1e-3).astype(np.float32)
    cfg = Bd.make_config(L, pattern, seed=seed, flat_params=P, straggler_p=p,
                         mix=Bd.MIX_DEFAULT if mix is None else mix, tau=-1 if tau is None else tau, group_size=group_size)
    eng = Bd.Adpsgd(cfg)
    for key, value in tune:
        eng.tune(key, value)
    for i in range(L):
        eng.set_params(i, torch.from_numpy(x0[i]).cuda())
    gd = [torch.from_numpy(g[i]).cuda() for i in range(L)]
    ora = A.Oracle(L, pattern, seed, flat_params=P, x0=x0, straggler_p=p, mix=mix, tau=tau, group_size=max(group_size, 1))
    G = L // group_size if group_size else L
    for k in range(steps):
        eng.step(gd, lr)
        ora.step(None, lr, grads=g)
        got_s = eng.schedule(k)
        assert tuple(v[:G] for v in got_s) == tuple(ora.last_schedule)
        assert all(v[G:] == [-1] * (L - G) for v in got_s)
        got = np.stack([eng.params(i).cpu().numpy() for i in range(L)])
        assert (got.view(np.uint32) == ora.x.view(np.uint32)).all(), (k, np.abs(got - ora.x).max())
    eng.close()


@pytest.mark.parametrize("P", [1, 3, 4, 1023, 4096, 100003, 1 << 20])
def test_pairwise_random_ring_with_stragglers(P):
    print("update pair P", P, flush=True)
    _run(8, P, S.RANDOM_RING, 6, p=0.3)


@pytest.mark.parametrize("split", [0, 64, 128])
@pytest.mark.parametrize("L,P,p", [(8, 1, 0.3), (8, 3, 0.0), (8, 4, 0.3), (7, 1023, 0.3), (2, 70001, 0.0), (64, 20003, 0.2), (128, 1000, 0.1)])
def test_pairwise_update_with_one_or_both_members_of_a_pair_per_thread(L, P, p, split):
    # both forms of the pairwise kernel (a thread owns both members of a pair, or one and gets the partner's model through
    # LDS), forced: unmatched learners, stragglers, P % 4 tails, fewer than four elements, in place and ping-pong (tau = 1)
    from paper_2110_11199_amd import binding as Bd
    print("update pair split", L, P, p, split, flush=True)
    _run(L, P, S.RANDOM_RING, 4, p=p, tune=[(Bd.TUNE_PAIR_SPLIT, split)])
    _run(L, P, S.FIXED_RING, 3, tune=[(Bd.TUNE_PAIR_SPLIT, split)])
    _run(L, P, S.D1D, 3, mix=S.MIX_PAIR, tune=[(Bd.TUNE_PAIR_SPLIT, split)])


def test_pairwise_update_at_a_size_that_takes_the_split_form_by_default():
    print("update pair, 6 x (1M + 1) elements", flush=True)
    _run(6, (1 << 20) + 1, S.RANDOM_RING, 3, p=0.2)


@pytest.mark.parametrize("L", [1, 2, 3, 5, 64])
def test_pairwise_fixed_ring(L):
    print("update fixed L", L, flush=True)
    _run(L, 70001, S.FIXED_RING, 4)


@pytest.mark.parametrize("L,P", [(1, 5), (4, 70001), (16, 4096), (128, 1000)])
def test_delay_by_one_global_mean(L, P):
    print("update d1d", L, P, flush=True)
    _run(L, P, S.D1D, 4)


@pytest.mark.parametrize("L,P,chunk", [(4, 70001, 1024), (16, 70003, 4096), (5, 1 << 20, 65536), (16, 4099, 16 << 20), (128, 3000, 1024)])
def test_global_mean_in_two_kernels_per_chunk(L, P, chunk):
    # the mean of a chunk of the index first, then one pass per learner: bit-identical to the single kernel and the oracle;
    # ragged last chunks, P % 4 tails, chunks larger than the model, in place (tau = 0) and ping-pong (tau = 1)
    from paper_2110_11199_amd import binding as Bd
    print("update d1d two kernels", L, P, chunk, flush=True)
    _run(L, P, S.D1D, 3, tune=[(Bd.TUNE_MEAN_CHUNK, chunk)])
    _run(L, P, S.FIXED_RING, 3, mix=S.MIX_ALL, tau=0, tune=[(Bd.TUNE_MEAN_CHUNK, chunk)])


@pytest.mark.parametrize("L", [3, 4, 5, 16, 128])
@pytest.mark.parametrize("pattern", [S.FIXED_RING, S.RANDOM_RING])
def test_ring_neighbour_thirds(L, pattern):
    # the circulant operator T^f of Eq. 9 (and T^r = P' T^f P on the random ring), in place and bit-exact
    print("update tri L", L, pattern, flush=True)
    _run(L, 70001 if L < 100 else 1003, pattern, 5, mix=S.MIX_TRI)


@pytest.mark.parametrize("P", [1, 3, 4, 1023, 100003])
def test_ring_neighbour_thirds_sizes_and_delay(P):
    _run(7, P, S.RANDOM_RING, 4, mix=S.MIX_TRI)
    _run(7, P, S.D1D, 3, mix=S.MIX_TRI)              # tau = 1: ping-pong buffers


@pytest.mark.parametrize("seg", [1, 2, 4, 8])
@pytest.mark.parametrize("L,P", [(3, 70001), (5, 4099), (16, 70003), (64, 20001), (128, 1003), (13, 2)])
def test_ring_neighbour_thirds_with_the_ring_in_segments(L, P, seg):
    # a thread owns `seg` ring positions, a workgroup the whole ring of its element positions: segments that do not
    # divide the ring, rings shorter than a segment (falls back to the single walk), P % 4 tails, fewer than four
    # elements, in place (tau = 0) and ping-pong (tau = 1); bit-exact against the oracle like the single walk
    from paper_2110_11199_amd import binding as Bd
    print("update tri segments", L, P, seg, flush=True)
    _run(L, P, S.RANDOM_RING, 3, mix=S.MIX_TRI, tune=[(Bd.TUNE_TRI_SEGMENT, seg)])
    _run(L, P, S.D1D, 2, mix=S.MIX_TRI, tune=[(Bd.TUNE_TRI_SEGMENT, seg)])


def test_ring_neighbour_thirds_at_a_size_that_takes_the_segmented_walk_by_default():
    print("update tri, 4 x (4M + 3) elements", flush=True)
    _run(4, (4 << 20) + 3, S.RANDOM_RING, 2, mix=S.MIX_TRI)


@pytest.mark.parametrize("seg", [2, 4, 8])
@pytest.mark.parametrize("L,P", [(3, 70001), (5, 4099), (16, 70003), (64, 20001), (128, 1003), (13, 2)])
def test_synchronous_baseline_update_with_the_learners_in_segments(L, P, seg):
    # the sum of the updated models runs through the segments of a workgroup in learner order: the same additions in the
    # same order as one thread per position, bit-exact against the oracle; segments that do not divide L, L <= seg
    # (falls back), P % 4 tails, fewer than four elements
    from paper_2110_11199_amd import binding as Bd
    print("update sync segments", L, P, seg, flush=True)
    _run(L, P, S.SDPSGD, 3, tune=[(Bd.TUNE_SYNC_SEGMENT, seg)])


def test_synchronous_baseline_update_at_a_size_that_takes_the_segments_by_default():
    print("update sync, 4 x (4M + 1) elements", flush=True)
    _run(4, (4 << 20) + 1, S.SDPSGD, 2)


def test_ring_neighbour_thirds_rejects_stragglers_and_rings_of_fewer_than_three():
    from paper_2110_11199_amd import binding as Bd
    for cfg in (Bd.make_config(4, S.RANDOM_RING, flat_params=16, straggler_p=0.1, mix=Bd.MIX_TRI),
                Bd.make_config(1, S.FIXED_RING, flat_params=16, mix=Bd.MIX_TRI),
                Bd.make_config(2, S.RANDOM_RING, flat_params=16, mix=Bd.MIX_TRI)):
        with pytest.raises(Bd.AdpsgdError) as ei:
            Bd.adpsgd_workspace_bytes(cfg)
        assert ei.value.code == Bd.EINVAL


@pytest.mark.parametrize("L,P", [(1, 5), (3, 1001), (16, 70001), (64, 300000)])
def test_consensus_distance_and_its_contraction(L, P):
    import torch
    from paper_2110_11199_amd import binding as Bd
    r = np.random.default_rng(L)
    x0 = r.uniform(-1, 1, (L, P)).astype(np.float32)
    mix = S.MIX_TRI if L >= 3 else S.MIX_PAIR          # the ring-neighbour operator needs three learners
    eng = Bd.Adpsgd(Bd.make_config(L, S.FIXED_RING, flat_params=P, mix=mix))
    for i in range(L):
        eng.set_params(i, torch.from_numpy(x0[i]).cuda())
    ora = A.Oracle(L, S.FIXED_RING, 0, flat_params=P, x0=x0, mix=mix)
    zero = np.zeros((L, P), np.float32)
    gz = [torch.zeros(P, device="cuda") for _ in range(L)]
    for k in range(3):
        ref = ora.consensus()
        got = eng.consensus()
        assert abs(got - ref) <= 1e-11 * max(ref, 1e-30), (k, got, ref)      # both fp64, different summation order
        eng.step(gz, 0.0)
        ora.step(None, 0.0, grads=zero)
    eng.close()


@pytest.mark.parametrize("mix", [S.MIX_HYBRID_PAIR, S.MIX_HYBRID_TRI])
@pytest.mark.parametrize("L,Sz", [(8, 2), (12, 4), (15, 3), (16, 1), (16, 16), (6, 1), (128, 2), (128, 8), (10, 2)])
def test_hybrid_super_learner_mixing(mix, L, Sz):
    # Section V: synchronous mean inside super-learners of Sz learners, the ring operator across them; bit-exact, in place
    if mix == S.MIX_HYBRID_TRI and L // Sz == 2:
        pytest.skip("a ring of two super-learners has no distinct left and right neighbour")
    print("update hybrid", mix, L, Sz, flush=True)
    for pattern in (S.FIXED_RING, S.RANDOM_RING):
        _run(L, 70001 if L < 100 else 1003, pattern, 4, mix=mix, group_size=Sz)


@pytest.mark.parametrize("P", [1, 3, 4, 1023, 100003, 1 << 20])
def test_hybrid_super_learner_mixing_sizes_and_delay(P):
    _run(12, P, S.RANDOM_RING, 4, mix=S.MIX_HYBRID_PAIR, group_size=3)
    _run(12, P, S.FIXED_RING, 4, mix=S.MIX_HYBRID_TRI, group_size=3)
    _run(12, P, S.RANDOM_RING, 3, mix=S.MIX_HYBRID_TRI, group_size=2, tau=1)      # ping-pong buffers
    _run(12, P, S.FIXED_RING, 3, mix=S.MIX_HYBRID_PAIR, group_size=6, tau=1)


def test_hybrid_mixing_alone_makes_every_super_learner_identical():
    import torch
    from paper_2110_11199_amd import binding as Bd
    L, Sz, P = 12, 4, 10007
    r = np.random.default_rng(5)
    eng = Bd.Adpsgd(Bd.make_config(L, S.RANDOM_RING, flat_params=P, mix=Bd.MIX_HYBRID_TRI, group_size=Sz))
    for i in range(L):
        eng.set_params(i, torch.from_numpy(r.uniform(-1, 1, P).astype(np.float32)).cuda())
    before = eng.average().cpu().numpy().astype(np.float64)
    eng.step([torch.zeros(P, device="cuda") for _ in range(L)], 0.0)
    for a in range(L // Sz):
        first = eng.params(a * Sz).cpu().numpy().view(np.uint32)
        for i in range(a * Sz + 1, (a + 1) * Sz):
            assert (eng.params(i).cpu().numpy().view(np.uint32) == first).all()
    assert np.abs(eng.average().cpu().numpy() - before).max() < 1e-6      # doubly stochastic: the learner average stays
    eng.close()


def test_given_straggler_masks_bit_exact_and_rejected_where_undefined():
    import torch
    from paper_2110_11199_amd import binding as Bd
    L, P = 7, 5003
    r = np.random.default_rng(2)
    x0 = r.uniform(-1, 1, (L, P)).astype(np.float32)
    g = (r.standard_normal((L, P)) * 1e-2).astype(np.float32)
    eng = Bd.Adpsgd(Bd.make_config(L, S.RANDOM_RING, seed=9, flat_params=P))
    for i in range(L):
        eng.set_params(i, torch.from_numpy(x0[i]).cuda())
    gd = [torch.from_numpy(g[i]).cuda() for i in range(L)]
    ora = A.Oracle(L, S.RANDOM_RING, 9, flat_params=P, x0=x0)
    for k in range(6):
        mask = [int(v) for v in r.integers(0, 2, L)] if k != 3 else [1] * L
        eng.step([gd[i] if mask[i] else None for i in range(L)], 0.2, active=mask)
        ora.step(None, 0.2, grads=g, active=mask)
        got = np.stack([eng.params(i).cpu().numpy() for i in range(L)])
        assert (got.view(np.uint32) == ora.x.view(np.uint32)).all(), k
    eng.close()
    for cfg in (Bd.make_config(4, S.D1D, flat_params=8), Bd.make_config(4, S.FIXED_RING, flat_params=8, mix=Bd.MIX_TRI),
                Bd.make_config(4, S.FIXED_RING, flat_params=8, tau=1)):
        e = Bd.Adpsgd(cfg)
        gz = [torch.zeros(8, device="cuda") for _ in range(4)]
        e.step(gz, 0.1, active=[1, 1, 1, 1])          # nobody sits out: fine everywhere
        with pytest.raises(Bd.AdpsgdError) as ei:
            e.step(gz, 0.1, active=[1, 0, 1, 1])
        assert ei.value.code == Bd.EINVAL
        e.close()


def test_slow_learner_wall_clock_model():
    # Section IV-D: with one learner 8 times slower the ring variants go on without it, delay-by-one waits for it.
    # The masks that were realised depend on timing; whatever they were, replaying them through the oracle must give
    # the library's models bit for bit.
    import torch
    from paper_2110_11199_amd import binding as Bd, straggler_model as SM
    L, P, iters, grad_us = 6, 20011, 12, 3000
    base = SM.run(Bd.FIXED_RING, L, P, 1, iters, grad_us, seed=1)
    base["engine"].close()
    assert all(sum(m) == L for m in base["masks"])
    per_iter = base["seconds"] / iters
    assert per_iter > grad_us * 1e-6
    for pattern in (Bd.FIXED_RING, Bd.RANDOM_RING):
        r = np.random.default_rng(4)
        x0 = r.uniform(-1, 1, (L, P)).astype(np.float32)
        run = SM.run(pattern, L, P, 8, iters, grad_us, seed=1, x0=[torch.from_numpy(x0[i]).cuda() for i in range(L)])
        skipped = sum(1 - m[0] for m in run["masks"])
        assert skipped >= iters // 2                                      # the slow learner missed most iterations ...
        assert run["seconds"] / iters < 2.0 * per_iter                    # ... and nobody waited for it
        ora = A.Oracle(L, pattern, 1, flat_params=P, x0=x0)
        g = np.stack([t.cpu().numpy() for t in run["grads"]])
        for m in run["masks"]:
            ora.step(None, 0.1, grads=g, active=m)
        got = np.stack([run["engine"].params(i).cpu().numpy() for i in range(L)])
        assert (got.view(np.uint32) == ora.x.view(np.uint32)).all()
        run["engine"].close()
    d1d = SM.run(Bd.D1D, L, P, 8, 6, grad_us, seed=1)
    d1d["engine"].close()
    assert all(sum(m) == L for m in d1d["masks"])
    assert d1d["seconds"] / 6 > 6.0 * per_iter                            # every iteration took the slow learner's time


def test_delay_by_one_with_pairwise_mixing_and_ring_with_global_mean():
    _run(6, 5001, S.D1D, 4, mix=S.MIX_PAIR)
    _run(6, 5001, S.FIXED_RING, 3, mix=S.MIX_ALL, tau=0)


def test_all_stragglers_is_identity_and_average_is_learner_mean():
    import torch
    from paper_2110_11199_amd import binding as Bd
    L, P = 4, 1001
    r = np.random.default_rng(0)
    x0 = r.uniform(-1, 1, (L, P)).astype(np.float32)
    cfg = Bd.make_config(L, S.RANDOM_RING, flat_params=P, straggler_p=0.999)
    eng = Bd.Adpsgd(cfg)
    for i in range(L):
        eng.set_params(i, torch.from_numpy(x0[i]).cuda())
    gd = [torch.ones(P, device="cuda") for _ in range(L)]
    ks = [k for k in range(50) if sum(S.schedule(S.RANDOM_RING, 0, k, L, 0.999)[2]) == 0]
    assert len(ks) > 40
    eng.step(gd, 0.1)
    if 0 in ks:
        got = np.stack([eng.params(i).cpu().numpy() for i in range(L)])
        assert (got.view(np.uint32) == x0.view(np.uint32)).all()
    cur = np.stack([eng.params(i).cpu().numpy() for i in range(L)])
    s = cur[0].copy()
    for j in range(1, L):
        s = s + cur[j]
    assert (eng.average().cpu().numpy() == s * (np.float32(1) / np.float32(L))).all()
    eng.close()


@pytest.mark.parametrize("L,P", [(1, 5), (3, 2), (4, 70001), (16, 4096), (128, 1003), (8, 1 << 20)])
def test_synchronous_baseline_update_then_mean(L, P):
    print("update sdpsgd", L, P, flush=True)
    _run(L, P, S.SDPSGD, 4)


def test_synchronous_baseline_keeps_the_learners_identical():
    import torch
    from paper_2110_11199_amd import binding as Bd
    L, P = 6, 10007
    r = np.random.default_rng(8)
    x0 = r.uniform(-1, 1, (L, P)).astype(np.float32)
    eng = Bd.Adpsgd(Bd.make_config(L, S.SDPSGD, flat_params=P))
    for i in range(L):
        eng.set_params(i, torch.from_numpy(x0[i]).cuda())
    g = [torch.from_numpy((r.standard_normal(P) * 1e-2).astype(np.float32)).cuda() for _ in range(L)]
    eng.step(g, 0.1)
    first = eng.params(0).cpu().numpy().view(np.uint32)
    for i in range(1, L):
        assert (eng.params(i).cpu().numpy().view(np.uint32) == first).all()
    assert eng.consensus() == 0.0
    eng.close()
