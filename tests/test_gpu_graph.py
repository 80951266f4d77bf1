"""GPU: iterations recorded into a HIP graph and replayed (adpsgd_capture_begin / _end, adpsgd_graph_replay).

A replay must give what the same adpsgd_step calls give when made directly, bit for bit, on EVERY replay, also with the
program's own eager work and synchronisations between the replays; the directly stepped engine is itself held to the
oracle here (and in test_gpu_lstm.py / test_gpu_update.py)."""
import numpy as np
import pytest

from oracle import lstm, schedule as S, adpsgd as A
from oracle.lstm import Shape
from paper_2110_11199_amd import synth
from tests.gpu_util import rel_err

pytestmark = pytest.mark.gpu

SHAPE = Shape(40, 64, 1, 0, 0, 100, 4, 20)        # the tiny benchmark shape


def _engine(shape, L, pattern, prec, stream, seed=0, **kw):
    import torch
    from paper_2110_11199_amd import binding as Bd
    cfg = Bd.make_config(L, pattern, seed=seed, input_dim=shape.input_dim, hidden=shape.hidden, layers=shape.layers,
                         bidirectional=shape.bidirectional, bottleneck=shape.bottleneck, classes=shape.classes,
                         batch=shape.batch, frames=shape.frames, precision=prec, **kw)
    with torch.cuda.stream(stream):               # the handle works on the stream that is current at its creation
        return Bd.Adpsgd(cfg)


def _batch(shape, L, k, seed=0):
    return [(synth.features(seed, k, i, shape.frames, shape.batch, shape.input_dim),
             synth.labels(seed, k, i, shape.frames, shape.batch, shape.classes)) for i in range(L)]


def _bits(t):
    return t.cpu().numpy().view(np.uint32)


@pytest.mark.parametrize("pattern,prec", [(S.FIXED_RING, 0), (S.D1D, 1), (S.D1D, 0), (S.SDPSGD, 0)])
def test_replayed_iterations_equal_direct_ones_on_every_replay(pattern, prec):
    import torch
    from paper_2110_11199_amd import binding as Bd
    print("graph replay", pattern, prec, flush=True)
    L, lr, shape = 4, 0.1, SHAPE
    w0 = synth.initial_model(5, lstm.param_count(shape), 0.1)
    s = torch.cuda.Stream()
    eng = _engine(shape, L, pattern, prec, s)
    ref = _engine(shape, L, pattern, prec, s)
    ora = A.Oracle(L, pattern, 0, shape=shape, w0=w0)
    with torch.cuda.stream(s):
        for e in (eng, ref):
            e.set_params(-1, torch.from_numpy(w0).cuda())
        b0 = _batch(shape, L, 0)
        dev0 = [(torch.from_numpy(f).cuda(), torch.from_numpy(y).cuda()) for f, y in b0]
        eng.step(dev0, lr); ref.step(dev0, lr); ora.step(b0, lr)          # one iteration before the recording
        # the buffers the recorded iterations read: refilled before every replay
        bufs = [[(torch.empty_like(dev0[i][0]), torch.empty_like(dev0[i][1])) for i in range(L)] for _ in range(2)]
        s.synchronize()
        eng.capture_begin()
        with pytest.raises(Bd.AdpsgdError):       # nothing but steps while recording
            eng.losses()
        eng.step(bufs[0], lr)
        eng.step(bufs[1], lr)
        g = eng.capture_end()
        assert Bd.adpsgd_graph_steps(g) == 2 and Bd.adpsgd_iteration(eng.h) == 1      # nothing has run yet
        k = 1
        for replay in range(3):
            for j in range(2):
                b = _batch(shape, L, k + j)
                for i in range(L):
                    bufs[j][i][0].copy_(torch.from_numpy(b[i][0]))
                    bufs[j][i][1].copy_(torch.from_numpy(b[i][1]))
                ref.step([(torch.from_numpy(f).cuda(), torch.from_numpy(y).cuda()) for f, y in b], lr)
                ora.step(b, lr)
            Bd.adpsgd_graph_replay(g)
            k += 2
            assert Bd.adpsgd_iteration(eng.h) == k == Bd.adpsgd_iteration(ref.h)
            # the program's own eager work and a synchronisation between the replays
            scratch = torch.randn(1 << 16, device="cuda").sum().item()
            assert np.isfinite(scratch)
            np.testing.assert_array_equal(eng.losses(), ref.losses())
            for i in range(L):
                assert (_bits(eng.params(i)) == _bits(ref.params(i))).all(), (replay, i)
                assert (_bits(eng.grads(i)) == _bits(ref.grads(i))).all(), (replay, i)
        # the handle goes on from where the replays left it
        b = _batch(shape, L, k)
        dev = [(torch.from_numpy(f).cuda(), torch.from_numpy(y).cuda()) for f, y in b]
        eng.step(dev, lr); ref.step(dev, lr); ora.step(b, lr)
        tol = 2e-2 if prec else 1e-4
        for i in range(L):
            assert (_bits(eng.params(i)) == _bits(ref.params(i))).all()
            got = eng.params(i).cpu().numpy()
            for name, off, r, c in lstm.layout(shape)[0]:
                assert rel_err(got[off:off + r * c], ora.x[i][off:off + r * c]) < tol, (name, i)
        Bd.adpsgd_graph_destroy(g)
    eng.close(); ref.close()


def test_replay_of_the_model_free_update_is_bit_exact_against_the_oracle():
    import torch
    from paper_2110_11199_amd import binding as Bd
    print("graph replay, model-free", flush=True)
    L, P, lr = 8, 100003, 0.1
    s = torch.cuda.Stream()
    rng = np.random.default_rng(3)
    x0 = rng.uniform(-0.05, 0.05, (L, P)).astype(np.float32)
    cfg = Bd.make_config(L, S.FIXED_RING, seed=0, flat_params=P)
    with torch.cuda.stream(s):
        eng = Bd.Adpsgd(cfg)
        for i in range(L):
            eng.set_params(i, torch.from_numpy(x0[i]).cuda())
        gbuf = [[torch.empty(P, device="cuda") for _ in range(L)] for _ in range(2)]
        s.synchronize()
        eng.capture_begin()
        eng.step(gbuf[0], lr)
        eng.step(gbuf[1], lr)
        g = eng.capture_end()
        ora = A.Oracle(L, S.FIXED_RING, 0, flat_params=P, x0=x0.copy())
        for replay in range(3):
            for j in range(2):
                gr = rng.normal(0, 1e-3, (L, P)).astype(np.float32)
                for i in range(L):
                    gbuf[j][i].copy_(torch.from_numpy(gr[i]))
                ora.step(None, lr, grads=gr)
            Bd.adpsgd_graph_replay(g)
            torch.cuda.synchronize()
            for i in range(L):
                assert (_bits(eng.params(i)) == ora.x[i].view(np.uint32)).all(), (replay, i)
        Bd.adpsgd_graph_destroy(g)
    eng.close()


def test_what_cannot_be_recorded_is_refused():
    import torch
    from paper_2110_11199_amd import binding as Bd
    print("graph refusals", flush=True)
    L, P = 4, 4096
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        grads = [torch.zeros(P, device="cuda") for _ in range(L)]
        # the random ring and drawn stragglers change the schedule every iteration
        for kw in (dict(pattern=S.RANDOM_RING), dict(pattern=S.FIXED_RING, straggler_p=0.1)):
            eng = Bd.Adpsgd(Bd.make_config(L, kw.pop("pattern"), seed=0, flat_params=P, **kw))
            with pytest.raises(Bd.AdpsgdError) as ei:
                eng.capture_begin()
            assert ei.value.code == Bd.EINVAL
            eng.step(grads, 0.1)                 # the handle still works
            eng.close()
        eng = Bd.Adpsgd(Bd.make_config(L, S.FIXED_RING, seed=0, flat_params=P))
        # an odd number of iterations on an alternating pattern
        eng.capture_begin()
        eng.step(grads, 0.1)
        with pytest.raises(Bd.AdpsgdError) as ei:
            eng.capture_end()
        assert ei.value.code == Bd.EINVAL and Bd.adpsgd_iteration(eng.h) == 0
        # an empty recording
        eng.capture_begin()
        with pytest.raises(Bd.AdpsgdError):
            eng.capture_end()
        # a replay at the other parity
        eng.capture_begin()
        eng.step(grads, 0.1); eng.step(grads, 0.1)
        g = eng.capture_end()
        eng.step(grads, 0.1)
        with pytest.raises(Bd.AdpsgdError) as ei:
            Bd.adpsgd_graph_replay(g)
        assert ei.value.code == Bd.EINVAL
        eng.step(grads, 0.1)
        Bd.adpsgd_graph_replay(g)                # parity restored
        torch.cuda.synchronize()
        assert Bd.adpsgd_iteration(eng.h) == 4
        eng.close()
        # the recording outlives its handle: it can be destroyed, not replayed
        with pytest.raises(Bd.AdpsgdError):
            Bd.adpsgd_graph_replay(g)
        Bd.adpsgd_graph_destroy(g)
    # a handle on the null stream
    eng = Bd.Adpsgd(Bd.make_config(L, S.FIXED_RING, seed=0, flat_params=P))
    if eng.stream.cuda_stream == 0:
        with pytest.raises(Bd.AdpsgdError):
            eng.capture_begin()
    eng.close()
