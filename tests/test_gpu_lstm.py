"""GPU: LSTM gradient and full ADPSGD iterations against the CPU oracle.

Tolerances (per tensor, max|diff| / max|ref|): 1e-4 with fp32 GEMM operands,
2e-2 with bf16 GEMM operands; the schedule is compared exactly."""
import numpy as np
import pytest

from oracle import lstm, schedule as S, adpsgd as A
from oracle.lstm import Shape
from paper_2110_11199_amd import synth
from tests.gpu_util import rel_err

pytestmark = pytest.mark.gpu

TOL = {0: 1e-4, 1: 2e-2}
# bf16 mode against the oracle run with its GEMM operands rounded to bf16 as well: what is
# left is summation order and values that land on
# the other side of a bf16 rounding boundary (one bf16 ulp = 2^-8 relative).
TOL_EMULATED = 1e-2


def _engine(shape, L, pattern, prec, seed=0, **kw):
    from paper_2110_11199_amd import binding as Bd
    cfg = Bd.make_config(L, pattern, seed=seed, input_dim=shape.input_dim, hidden=shape.hidden,
                         layers=shape.layers, bidirectional=shape.bidirectional, bottleneck=shape.bottleneck,
                         classes=shape.classes, batch=shape.batch, frames=shape.frames, precision=prec, **kw)
    return Bd.Adpsgd(cfg)


def _batches(shape, L, k, seed=0):
    return [(synth.features(seed, k, i, shape.frames, shape.batch, shape.input_dim),
             synth.labels(seed, k, i, shape.frames, shape.batch, shape.classes)) for i in range(L)]


def _to_dev(batches):
    import torch
    return [(torch.from_numpy(f).cuda(), torch.from_numpy(y).cuda()) for f, y in batches]


def _per_tensor_err(shape, got, ref):
    worst = 0.0
    for name, off, r, c in lstm.layout(shape)[0]:
        worst = max(worst, rel_err(got[off:off + r * c], ref[off:off + r * c]))
    return worst


SHAPES = [
    Shape(40, 64, 1, 0, 0, 100, 4, 20),       # the tiny benchmark shape
    Shape(12, 32, 2, 1, 0, 52, 5, 7),         # bidirectional, ragged batch
    Shape(24, 36, 2, 1, 16, 40, 33, 3),       # bottleneck, hidden not a multiple of 8/32, batch 33
    Shape(20, 64, 1, 1, 0, 300, 70, 4),       # batch 70 (64-row tiles + tail), several class tiles
    Shape(16, 32, 3, 0, 8, 36, 130, 2),       # batch 130 (128-row tiles + tail), unidirectional
    Shape(8, 8, 1, 1, 4, 8, 9, 1),            # one frame: no recurrence (9 rows: with 2 the bf16 rounding of a single
                                              # operand shows up as 2.2e-2 in a bias gradient, in the oracle's own bf16 run too)
    Shape(24, 192, 2, 1, 16, 64, 130, 3),     # hidden 192: ragged unit tiles of the direct-to-LDS kernels, batch 130
    Shape(16, 128, 1, 1, 0, 40, 48, 4),       # batch 48: the 64-row recurrent tile configuration
    Shape(8, 32, 1, 0, 0, 1500, 3, 2),        # 1500 classes: softmax rows of 4 float4 per thread
    Shape(8, 32, 1, 0, 0, 5000, 3, 2),        # 5000 classes: softmax rows on 512 threads
    Shape(16, 72, 2, 1, 0, 32, 20, 5),        # small-batch recurrent kernels: three unit tiles, the last one ragged
    Shape(12, 20, 1, 1, 0, 24, 32, 3),        # batch 32, hidden 20: half-empty last k-chunk (fp32); staged kernels (bf16)
    Shape(12, 264, 1, 1, 0, 20, 7, 4),        # hidden 264: more k-chunks than one pass of a workgroup's waves takes
]


@pytest.mark.parametrize("prec", [0, 1])
@pytest.mark.parametrize("shape", SHAPES)
def test_gradient_matches_oracle(shape, prec):
    import torch
    print("lstm grad", shape, prec, flush=True)
    L = 2
    P = lstm.param_count(shape)
    w0 = synth.initial_model(1, P, 0.2)
    eng = _engine(shape, L, S.FIXED_RING, prec)
    assert eng.P == P
    from paper_2110_11199_amd import binding as Bd
    assert [(o, r, c) for _, o, r, c in lstm.layout(shape)[0]] == Bd.adpsgd_layout(eng.h)
    eng.set_params(-1, torch.from_numpy(w0).cuda())
    b = _batches(shape, L, 0)
    eng.step(_to_dev(b), 0.0)
    losses = eng.losses()
    for i in range(L):
        loss, g = lstm.loss_and_grad(shape, w0, b[i][0], b[i][1], np.float32)
        got = eng.grads(i).cpu().numpy()
        assert np.isfinite(got).all()
        assert _per_tensor_err(shape, got, g) < TOL[prec], (i, _per_tensor_err(shape, got, g))
        assert abs(losses[i] - loss) < TOL[prec] * abs(loss)
        if prec:
            _, ge = lstm.loss_and_grad(shape, w0, b[i][0], b[i][1], np.float32, bf16_gemm=True)
            assert _per_tensor_err(shape, got, ge) < TOL_EMULATED, (i, _per_tensor_err(shape, got, ge))
    eng.close()


def _run_recurrence(shape, L, pattern, prec, steps, lr, seed=0, scale=0.1, tune=(), drop_straggler_batches=False, **kw):
    import torch
    P = lstm.param_count(shape)
    w0 = synth.initial_model(seed, P, scale)
    eng = _engine(shape, L, pattern, prec, seed=seed, **kw)
    for key, value in tune:
        eng.tune(key, value)
    eng.set_params(-1, torch.from_numpy(w0).cuda())
    ora = A.Oracle(L, pattern, seed, shape=shape, w0=w0, straggler_p=kw.get("straggler_p", 0.0), mix=kw.get("mix"),
                   group_size=max(kw.get("group_size", 1), 1))
    emu = A.Oracle(L, pattern, seed, shape=shape, w0=w0, bf16_gemm=True, mix=kw.get("mix"),
                   straggler_p=kw.get("straggler_p", 0.0), group_size=max(kw.get("group_size", 1), 1)) if prec else None
    for k in range(steps):
        b = _batches(shape, L, k, seed)
        db = _to_dev(b)
        if drop_straggler_batches:      # a straggler's minibatch is not read: hand over no pointers for it
            act_k = S.schedule(pattern, seed, k, L, kw.get("straggler_p", 0.0))[2]
            db = [db[i] if act_k[i] else (None, None) for i in range(L)]
        eng.step(db, lr)
        ora.step(b, lr)
        G = L // kw["group_size"] if kw.get("group_size") else L
        assert tuple(v[:G] for v in eng.schedule(k)) == tuple(ora.last_schedule)
        active = ora.last_schedule[2] if G == L else [1] * L
        np.testing.assert_allclose(eng.losses(), ora.last_losses, rtol=TOL[prec])      # a straggler reports 0 on both sides
        for i in range(L):
            got_x = eng.params(i).cpu().numpy()
            if active[i]:
                got_g = eng.grads(i).cpu().numpy()
                assert _per_tensor_err(shape, got_g, ora.last_grads[i]) < TOL[prec], (k, i)
            assert _per_tensor_err(shape, got_x, ora.x[i]) < TOL[prec], (k, i)
        if emu is not None:
            emu.step(b, lr)
            for i in range(L):
                if active[i]:
                    assert _per_tensor_err(shape, eng.grads(i).cpu().numpy(), emu.last_grads[i]) < TOL_EMULATED, (k, i)
    eng.close()
    return ora


def test_tiny_config_five_steps_fixed_ring():
    print("cfg1 recurrence", flush=True)
    wl = synth.WORKLOADS["cfg1"]
    shape = Shape(wl.input_dim, wl.hidden, wl.layers, wl.bidirectional, wl.bottleneck, wl.classes, wl.batch, wl.frames)
    _run_recurrence(shape, wl.L, wl.pattern, 0, wl.steps, wl.lr, scale=wl.init_scale)


def test_random_ring_with_stragglers_small_model():
    print("random ring + stragglers", flush=True)
    _run_recurrence(Shape(12, 16, 1, 1, 0, 20, 3, 4), 6, S.RANDOM_RING, 0, 5, 0.2, seed=4, straggler_p=0.3)
    _run_recurrence(Shape(12, 16, 1, 1, 0, 20, 3, 4), 6, S.RANDOM_RING, 0, 5, 0.2, seed=4, straggler_p=0.3,
                    drop_straggler_batches=True)


@pytest.mark.parametrize("prec", [0, 1])
def test_random_ring_with_stragglers_at_a_real_size(prec):
    # stragglers on a model whose GEMMs run on the large-tile and direct-to-LDS kernels (hidden 256, batch 96,
    # 8 learners): the gradient phase runs on the compacted list of active learners
    print("random ring + stragglers, hidden 256", prec, flush=True)
    seed = 9
    assert any(0 < sum(S.schedule(S.RANDOM_RING, seed, k, 8, 0.3)[2]) < 8 for k in range(3))
    _run_recurrence(Shape(64, 256, 2, 1, 64, 512, 96, 5), 8, S.RANDOM_RING, prec, 3, 0.2, seed=seed, scale=0.05,
                    straggler_p=0.3, drop_straggler_batches=True)


def test_every_learner_a_straggler_leaves_everything_unchanged():
    import torch
    shape = Shape(12, 16, 1, 1, 0, 20, 3, 4)
    L, seed, p = 3, 0, 0.97
    ks = [k for k in range(40) if sum(S.schedule(S.FIXED_RING, seed, k, L, p)[2]) == 0]
    assert ks and ks[0] == 0, ks[:3]     # iteration 0 has no active learner with this seed
    eng = _engine(shape, L, S.FIXED_RING, 0, seed=seed, straggler_p=p)
    w0 = synth.initial_model(seed, eng.P, 0.1)
    eng.set_params(-1, torch.from_numpy(w0).cuda())
    eng.step([(None, None)] * L, 0.5)
    assert (eng.losses() == 0).all()
    for i in range(L):
        assert (eng.params(i).cpu().numpy().view(np.uint32) == w0.view(np.uint32)).all()
    eng.close()


def test_label_out_of_range_is_reported_not_repaired_silently():
    import torch
    from paper_2110_11199_amd import binding as Bd
    shape = Shape(12, 16, 1, 1, 0, 20, 3, 4)
    for bad in (-1, shape.classes, 1 << 30):
        eng = _engine(shape, 2, S.FIXED_RING, 0)
        eng.set_params(-1, torch.from_numpy(synth.initial_model(0, eng.P, 0.1)).cuda())
        b = _batches(shape, 2, 0)
        eng.step(_to_dev(b), 0.1)
        eng.status()                                   # clean so far
        b[1][1][2, 1] = bad
        eng.step(_to_dev(b), 0.1)
        with pytest.raises(Bd.AdpsgdError) as ei:
            eng.losses()
        assert ei.value.code == Bd.EINVAL and "label" in str(ei.value)
        with pytest.raises(Bd.AdpsgdError) as ei:      # sticky: the step after the flag has reached the host is refused
            eng.step(_to_dev(_batches(shape, 2, 1)), 0.1)
        assert ei.value.code == Bd.EINVAL
        with pytest.raises(Bd.AdpsgdError):
            eng.status()
        eng.close()


@pytest.mark.parametrize("prec", [0, 1])
def test_delay_by_one_small_model(prec):
    print("d1d small", prec, flush=True)
    # weights U(-0.1, 0.1): with 12 frames per minibatch and weights of 0.3 the bf16 operand rounding
    # alone reaches 2.2e-2 on the smallest tensors
    ora = _run_recurrence(Shape(12, 16, 2, 1, 8, 20, 3, 4), 4, S.D1D, prec, 4, 0.3, seed=2, scale=0.1)
    assert ora.tau == 1


@pytest.mark.parametrize("prec", [0, 1])
def test_ring_neighbour_mixing_small_model(prec):
    print("ring neighbours (weights 1/3), model-bearing", prec, flush=True)
    ora = _run_recurrence(Shape(12, 16, 2, 1, 8, 20, 5, 4), 5, S.RANDOM_RING, prec, 4, 0.3, seed=5, scale=0.1, mix=S.MIX_TRI)
    assert ora.mix == S.MIX_TRI


@pytest.mark.parametrize("prec", [0, 1])
@pytest.mark.parametrize("mix", [S.MIX_HYBRID_PAIR, S.MIX_HYBRID_TRI])
def test_hybrid_super_learners_small_model(prec, mix):
    print("hybrid super-learners, model-bearing", prec, mix, flush=True)
    ora = _run_recurrence(Shape(12, 16, 2, 1, 8, 20, 5, 4), 6, S.RANDOM_RING, prec, 4, 0.3, seed=5, scale=0.1, mix=mix, group_size=2)
    assert ora.hybrid and ora.ring_size == 3


@pytest.mark.parametrize("prec", [0, 1])
def test_synchronous_baseline_small_model(prec):
    print("sdpsgd small, model-bearing", prec, flush=True)
    ora = _run_recurrence(Shape(12, 16, 2, 1, 8, 20, 5, 4), 4, S.SDPSGD, prec, 4, 0.3, seed=6, scale=0.1)
    assert ora.update_first and ora.consensus() == 0.0


@pytest.mark.parametrize("case", ["pair", "tri", "tri_d1d", "sync"])
def test_segmented_update_kernels_write_the_bf16_copy_of_a_small_model(case):
    # the update kernels that large models take by default (one member of a pair per thread; the ring or the learners in
    # segments), forced on a small bf16 model: the bf16 copy of the next gradient point they write feeds the next iteration
    from paper_2110_11199_amd import binding as Bd
    print("segmented update kernels, bf16 model", case, flush=True)
    shape = Shape(12, 32, 2, 1, 0, 52, 5, 7)
    if case == "pair":
        _run_recurrence(shape, 5, S.RANDOM_RING, 1, 3, 0.1, tune=((Bd.TUNE_PAIR_SPLIT, 64),), straggler_p=0.2)
    elif case == "tri":
        _run_recurrence(shape, 5, S.RANDOM_RING, 1, 3, 0.1, tune=((Bd.TUNE_TRI_SEGMENT, 2),), mix=S.MIX_TRI)
    elif case == "tri_d1d":
        _run_recurrence(shape, 5, S.D1D, 1, 3, 0.1, tune=((Bd.TUNE_TRI_SEGMENT, 2),), mix=S.MIX_TRI)
    else:
        _run_recurrence(shape, 5, S.SDPSGD, 1, 3, 0.1, tune=((Bd.TUNE_SYNC_SEGMENT, 2),))


@pytest.mark.parametrize("groups", [2, 3, 5])
def test_forward_recurrence_in_learner_groups(groups):
    # large models run the forward recurrence group of learners by group of learners (all frames of a group
    # first); forced here on a small one, 5 learners in 2 + 3, 1 + 1 + 3 and 1 + 1 + 1 + 1 + 1
    from paper_2110_11199_amd import binding as Bd
    print("forward recurrence in learner groups", groups, flush=True)
    for prec in (0, 1):
        _run_recurrence(Shape(12, 64, 2, 1, 0, 20, 40, 3), 5, S.RANDOM_RING, prec, 2, 0.2, seed=7, scale=0.1,
                        tune=[(Bd.TUNE_REC_FWD_GROUPS, groups)])


@pytest.mark.parametrize("prec", [0, 1])
@pytest.mark.parametrize("shape", [SHAPES[0], SHAPES[1], SHAPES[10]])
def test_small_batches_on_the_staged_kernels_too(shape, prec):
    # batches of at most 32 rows normally take the small-batch kernels; switched off, the register-staged
    # kernels with their 32-row tiles run the same recurrence
    from paper_2110_11199_amd import binding as Bd
    print("staged kernels, small batch", shape, prec, flush=True)
    _run_recurrence(shape, 2, S.FIXED_RING, prec, 2, 0.1, tune=((Bd.TUNE_REC_DIRECT, 0),))


def test_tuning_is_per_handle():
    # two handles in one process: forcing the register-staged kernels on one must not change the other
    import torch
    from paper_2110_11199_amd import binding as Bd
    shape = Shape(64, 64, 1, 1, 0, 64, 40, 3)
    w0 = synth.initial_model(3, lstm.param_count(shape), 0.1)
    b = _batches(shape, 2, 0)
    out = []
    for forced in (False, True, False):
        a = _engine(shape, 2, S.FIXED_RING, 1)
        other = _engine(shape, 2, S.FIXED_RING, 1)
        if forced:
            other.tune(Bd.TUNE_REC_DIRECT, 0)
            other.tune(Bd.TUNE_GEMM_TILE, 0)
        for e in (a, other):
            e.set_params(-1, torch.from_numpy(w0).cuda())
            e.step(_to_dev(b), 0.1)
        out.append(a.grads(0).cpu().numpy().copy())
        a.close(); other.close()
    assert (out[0].view(np.uint32) == out[1].view(np.uint32)).all() and (out[0].view(np.uint32) == out[2].view(np.uint32)).all()
    with pytest.raises(Bd.AdpsgdError):
        e = _engine(shape, 2, S.FIXED_RING, 1)
        try:
            e.tune(Bd.TUNE_GEMM_TILE, 7)
        finally:
            e.close()


def test_library_initial_model_matches_generator_spec():
    import torch
    shape = Shape(8, 8, 1, 0, 0, 8, 2, 2)
    eng = _engine(shape, 3, S.FIXED_RING, 0, seed=77, init_scale=0.1)
    ref = A.init_model(77, eng.P, 0.1)
    for i in range(3):
        assert (eng.params(i).cpu().numpy() == ref).all()      # same w_0 on every learner
    eng.close()


PERSIST_SHAPES = [
    Shape(64, 128, 2, 1, 0, 64, 40, 5),       # hidden 128, batch 40: two row tiles, ragged
    Shape(64, 128, 1, 0, 0, 64, 128, 3),      # one direction, batch 128: four row tiles
    Shape(64, 256, 2, 1, 32, 96, 100, 4),     # hidden 256, batch 100: four row tiles, ragged; bottleneck
    Shape(32, 256, 1, 1, 0, 64, 64, 6),       # batch 64: two full row tiles
    Shape(32, 128, 1, 1, 0, 64, 9, 1),        # a single frame: no recurrent product at all
]


@pytest.mark.parametrize("shape", PERSIST_SHAPES)
def test_persistent_recurrent_kernels_match_oracle(shape):
    # all frames of a layer in one launch, W_h resident in registers, workgroups of a (learner, direction) pair
    # synchronised once per frame: forced on small shapes; 3 learners, stragglers in some iterations
    from paper_2110_11199_amd import binding as Bd
    print("persistent recurrent kernels", shape, flush=True)
    _run_recurrence(shape, 3, S.RANDOM_RING, 1, 3, 0.2, seed=11, scale=0.08, straggler_p=0.25,
                    tune=[(Bd.TUNE_REC_PERSISTENT, 1)])


def test_persistent_recurrent_kernels_in_several_launches():
    # hidden 256: 8 workgroups per (learner, direction) pair, 32 pairs per launch on 256 compute units;
    # 20 learners x 2 directions = 40 pairs run as 32 + 8
    from paper_2110_11199_amd import binding as Bd
    print("persistent recurrent kernels, 40 pairs", flush=True)
    _run_recurrence(Shape(32, 256, 1, 1, 0, 32, 33, 3), 20, S.D1D, 1, 2, 0.2, seed=12, scale=0.08,
                    tune=[(Bd.TUNE_REC_PERSISTENT, 1)])


def test_persistent_and_per_frame_kernels_agree_closely():
    # same arithmetic up to the summation order of the recurrent products: far inside the tolerance against the oracle
    import torch
    from paper_2110_11199_amd import binding as Bd
    shape = Shape(64, 256, 2, 1, 0, 64, 72, 5)
    w0 = synth.initial_model(3, lstm.param_count(shape), 0.08)
    b = _batches(shape, 2, 0)
    out = []
    for persistent in (0, 1):
        e = _engine(shape, 2, S.FIXED_RING, 1)
        e.tune(Bd.TUNE_REC_PERSISTENT, persistent)
        e.set_params(-1, torch.from_numpy(w0).cuda())
        e.step(_to_dev(b), 0.1)
        e.status()
        out.append(e.grads(0).cpu().numpy().copy())
        e.close()
    assert _per_tensor_err(shape, out[1], out[0]) < 4e-3


def test_persistent_kernel_wait_runs_out_and_is_reported():
    # a wait bound of 0 microseconds: the first workgroup that has to wait for its pair gives up, the others
    # follow, every workgroup returns; the handle reports the failure and refuses further steps
    import torch
    from paper_2110_11199_amd import binding as Bd
    shape = Shape(32, 128, 1, 1, 0, 32, 16, 4)
    e = _engine(shape, 2, S.FIXED_RING, 1)
    e.tune(Bd.TUNE_REC_PERSISTENT, 1)
    e.tune(Bd.TUNE_REC_WAIT_US, 0)
    e.set_params(-1, torch.from_numpy(synth.initial_model(0, e.P, 0.1)).cuda())
    e.step(_to_dev(_batches(shape, 2, 0)), 0.1)
    with pytest.raises(Bd.AdpsgdError) as ei:
        e.status()
    assert ei.value.code == Bd.EHIP and "wait" in str(ei.value)
    with pytest.raises(Bd.AdpsgdError) as ei:
        e.step(_to_dev(_batches(shape, 2, 1)), 0.1)
    assert ei.value.code == Bd.EHIP
    e.close()
