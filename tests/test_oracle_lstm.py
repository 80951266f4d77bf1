"""Pins for the oracle's LSTM loss/gradient and the full recurrence (CPU only)."""
import math
import numpy as np
import pytest
import torch

from oracle import lstm, schedule as S, adpsgd as A
from oracle.lstm import Shape


def _data(shape, seed=0, scale=0.3):
    r = np.random.default_rng(seed)
    P = lstm.param_count(shape)
    w = r.uniform(-scale, scale, P)
    f = r.standard_normal((shape.frames, shape.batch, shape.input_dim))
    y = r.integers(0, shape.classes, (shape.frames, shape.batch))
    return w, f, y


def test_parameter_counts_of_the_benchmark_shapes():
    assert lstm.param_count(Shape(40, 64, 1, 0, 0, 100, 4, 20)) == 33380
    assert lstm.param_count(Shape(120, 256, 2, 1, 0, 1000, 32, 21)) == 2860008
    assert lstm.param_count(Shape(260, 512, 4, 1, 0, 9000, 64, 21)) == 31277864
    assert lstm.param_count(Shape(260, 1024, 6, 1, 256, 32000, 128, 21)) == 145145344


@pytest.mark.parametrize("shape", [
    Shape(3, 4, 1, 0, 0, 5, 2, 3),
    Shape(3, 4, 2, 1, 0, 5, 2, 4),
    Shape(4, 3, 2, 1, 2, 6, 3, 3),
    Shape(2, 2, 3, 0, 3, 4, 1, 5),
])
def test_gradient_matches_central_finite_differences(shape):
    w, f, y = _data(shape, 1)
    loss, grad = lstm.loss_and_grad(shape, w, f, y, np.float64)
    P = w.size
    idx = np.random.default_rng(2).choice(P, size=min(P, 120), replace=False)
    eps = 1e-6
    for e in idx:
        wp, wm = w.copy(), w.copy()
        wp[e] += eps
        wm[e] -= eps
        lp = lstm.loss_and_grad(shape, wp, f, y, np.float64, want_grad=False)[0]
        lm = lstm.loss_and_grad(shape, wm, f, y, np.float64, want_grad=False)[0]
        fd = (lp - lm) / (2 * eps)
        assert abs(fd - grad[e]) < 1e-8 + 1e-6 * abs(fd), (e, fd, grad[e])


def test_float32_oracle_agrees_with_float64():
    shape = Shape(8, 12, 2, 1, 4, 20, 4, 6)
    w, f, y = _data(shape, 3, 0.2)
    l64, g64 = lstm.loss_and_grad(shape, w, f, y, np.float64)
    l32, g32 = lstm.loss_and_grad(shape, w.astype(np.float32), f.astype(np.float32), y, np.float32)
    assert g32.dtype == np.float32
    assert abs(l32 - l64) < 1e-6 * abs(l64) + 1e-6
    assert np.abs(g32 - g64).max() < 1e-5 * np.abs(g64).max()


def test_zero_model_gives_log_C_and_single_class_gives_zero():
    shape = Shape(5, 4, 2, 1, 0, 7, 3, 4)
    _, f, y = _data(shape)
    loss, grad = lstm.loss_and_grad(shape, np.zeros(lstm.param_count(shape)), f, y, np.float64)
    assert abs(loss - math.log(7)) < 1e-14
    lay = {n: (o, r, c) for n, o, r, c in lstm.layout(shape)[0]}
    o, r, c = lay["bo"]
    counts = np.bincount(y.reshape(-1), minlength=7) / y.size
    assert np.allclose(grad[o:o + c], 1.0 / 7 - counts, atol=1e-15)   # softmax - onehot, averaged
    shape1 = shape._replace(classes=1)
    w, f, y = _data(shape1)
    loss, grad = lstm.loss_and_grad(shape1, w, f, np.zeros_like(y), np.float64)
    assert loss == 0.0 and np.abs(grad).max() == 0.0


def test_single_frame_reduces_to_a_gated_feedforward_layer():
    # T = 1: no recurrence.  h = sigma(o) * tanh(sigma(i) * tanh(g)), written with
    # scalar loops straight from the LSTM cell definition.
    shape = Shape(3, 2, 1, 0, 0, 4, 2, 1)
    w, f, y = _data(shape, 4, 0.8)
    lay = {n: (o, r, c) for n, o, r, c in lstm.layout(shape)[0]}
    H, I, C = 2, 3, 4
    Wx = w[lay["Wx0"][0]:][:4 * H * I].reshape(4 * H, I)
    b = w[lay["b0"][0]:][:4 * H]
    Wo = w[lay["Wo"][0]:][:C * H].reshape(C, H)
    bo = w[lay["bo"][0]:][:C]
    tot = 0.0
    for n in range(2):
        a = [sum(Wx[r, k] * f[0, n, k] for k in range(I)) + b[r] for r in range(4 * H)]
        sg = lambda v: 1 / (1 + math.exp(-v))
        h = [sg(a[3 * H + u]) * math.tanh(sg(a[u]) * math.tanh(a[2 * H + u])) for u in range(H)]
        z = [sum(Wo[c, u] * h[u] for u in range(H)) + bo[c] for c in range(C)]
        tot -= z[y[0, n]] - math.log(sum(math.exp(v) for v in z))
    loss, _ = lstm.loss_and_grad(shape, w, f, y, np.float64)
    assert abs(loss - tot / 2) < 1e-13


def test_zero_recurrent_weights_make_frames_independent():
    shape = Shape(4, 5, 1, 1, 0, 6, 2, 5)
    w, f, y = _data(shape, 6)
    for n, o, r, c in lstm.layout(shape)[0]:
        if n.startswith("Wh"):
            w[o:o + r * c] = 0
    # with W_h = 0 the cell state still carries over (c_t depends on c_{t-1}), so
    # also close the forget path by a very negative forget bias
    lay = {n: (o, r, c) for n, o, r, c in lstm.layout(shape)[0]}
    o, r, c = lay["b0"]
    H = shape.hidden
    for d in range(2):
        w[o + d * 4 * H + H: o + d * 4 * H + 2 * H] = -700.0
    perm = np.array([3, 0, 4, 1, 2])
    l1 = lstm.loss_and_grad(shape, w, f, y, np.float64, want_grad=False)[0]
    l2 = lstm.loss_and_grad(shape, w, f[perm], y[perm], np.float64, want_grad=False)[0]
    assert abs(l1 - l2) < 1e-14


class _TorchModel(torch.nn.Module):
    def __init__(self, shape):
        super().__init__()
        D = 2 if shape.bidirectional else 1
        self.rnn = torch.nn.LSTM(shape.input_dim, shape.hidden, shape.layers,
                                 bidirectional=bool(shape.bidirectional)).double()
        F = D * shape.hidden
        self.proj = torch.nn.Linear(F, shape.bottleneck).double() if shape.bottleneck else None
        self.out = torch.nn.Linear(shape.bottleneck or F, shape.classes).double()

    def forward(self, x):
        y, _ = self.rnn(x)
        if self.proj is not None:
            y = self.proj(y)
        return self.out(y)


@pytest.mark.parametrize("shape", [Shape(5, 6, 1, 0, 0, 7, 3, 4), Shape(5, 6, 3, 1, 4, 9, 2, 6)])
def test_against_stock_cpu_lstm(shape):
    # An installed framework's LSTM (gate order i,f,g,o; its second bias set to
    # zero) + linear layers + mean cross-entropy, differentiated by autograd.
    w, f, y = _data(shape, 8)
    m = _TorchModel(shape)
    lay = {n: (o, r, c) for n, o, r, c in lstm.layout(shape)[0]}
    H, D = shape.hidden, (2 if shape.bidirectional else 1)

    def slab(name, d=None, rows=None):
        o, r, c = lay[name]
        a = w[o:o + r * c].reshape(r, c)
        return a if d is None else a[d * rows:(d + 1) * rows]

    pairs = []   # (torch parameter, (name, d))
    with torch.no_grad():
        for l in range(shape.layers):
            for d in range(D):
                sfx = "_l%d%s" % (l, "_reverse" if d else "")
                getattr(m.rnn, "weight_ih" + sfx).copy_(torch.from_numpy(slab("Wx%d" % l, d, 4 * H)))
                getattr(m.rnn, "weight_hh" + sfx).copy_(torch.from_numpy(slab("Wh%d" % l, d, 4 * H)))
                getattr(m.rnn, "bias_ih" + sfx).copy_(
                    torch.from_numpy(slab("b%d" % l).reshape(-1)[d * 4 * H:(d + 1) * 4 * H]))
                getattr(m.rnn, "bias_hh" + sfx).zero_()
                pairs += [(getattr(m.rnn, "weight_ih" + sfx), ("Wx%d" % l, d)),
                          (getattr(m.rnn, "weight_hh" + sfx), ("Wh%d" % l, d)),
                          (getattr(m.rnn, "bias_ih" + sfx), ("b%d" % l, d))]
        if shape.bottleneck:
            m.proj.weight.copy_(torch.from_numpy(slab("Wp")))
            m.proj.bias.copy_(torch.from_numpy(slab("bp").reshape(-1)))
        m.out.weight.copy_(torch.from_numpy(slab("Wo")))
        m.out.bias.copy_(torch.from_numpy(slab("bo").reshape(-1)))
    logits = m(torch.from_numpy(f))
    loss_t = torch.nn.functional.cross_entropy(logits.reshape(-1, shape.classes),
                                               torch.from_numpy(y.reshape(-1)))
    loss_t.backward()
    loss, grad = lstm.loss_and_grad(shape, w, f, y, np.float64)
    assert abs(loss - loss_t.item()) < 1e-12
    G = {n: grad[o:o + r * c].reshape(r, c) for n, (o, r, c) in lay.items()}
    for p, (name, d) in pairs:
        ref = p.grad.numpy()
        got = G[name].reshape(-1)[d * 4 * H:(d + 1) * 4 * H] if name.startswith("b") else G[name][d * 4 * H:(d + 1) * 4 * H]
        assert np.abs(got - ref).max() < 1e-12, name
    assert np.abs(G["Wo"] - m.out.weight.grad.numpy()).max() < 1e-12
    assert np.abs(G["bo"].reshape(-1) - m.out.bias.grad.numpy()).max() < 1e-12
    if shape.bottleneck:
        assert np.abs(G["Wp"] - m.proj.weight.grad.numpy()).max() < 1e-12
        assert np.abs(G["bp"].reshape(-1) - m.proj.bias.grad.numpy()).max() < 1e-12


def test_bf16_rounding_rule():
    a = np.array([1.0, 1.00390625, 1.01171875, -3.14159, 0.0, 1e-40], np.float32)
    r = lstm.round_bf16(a)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 ties to 1 + 2^-6
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == np.float32(1.015625)
    assert (r.view(np.uint32) & 0xFFFF == 0).all()
    assert abs(r[3] - a[3]) <= abs(a[3]) * 2.0 ** -8


def _batches(shape, L, k, seed=0):
    out = []
    for i in range(L):
        r = np.random.default_rng([seed, k, i])
        out.append((r.standard_normal((shape.frames, shape.batch, shape.input_dim)).astype(np.float32),
                    r.integers(0, shape.classes, (shape.frames, shape.batch)).astype(np.int32)))
    return out


def test_recurrence_single_learner_is_plain_sgd():
    shape = Shape(4, 4, 1, 1, 0, 5, 2, 3)
    w0 = np.random.default_rng(0).uniform(-0.3, 0.3, lstm.param_count(shape)).astype(np.float32)
    o = A.Oracle(1, S.FIXED_RING, 0, shape=shape, w0=w0)
    x = w0.copy()
    for k in range(3):
        b = _batches(shape, 1, k)
        o.step(b, 0.2)
        _, g = lstm.loss_and_grad(shape, x, b[0][0], b[0][1], np.float32)
        x = x - np.float32(0.2) * g
        assert (o.x[0] == x).all()


def test_recurrence_same_initial_model_and_delay_by_one():
    # Algorithm 1 starts every learner from w_0; with delay-by-one the gradient
    # of iteration k is evaluated at the models of iteration k-1 (Section III-D).
    shape = Shape(4, 4, 1, 0, 0, 5, 2, 3)
    L = 4
    w0 = np.random.default_rng(1).uniform(-0.3, 0.3, lstm.param_count(shape)).astype(np.float32)
    o = A.Oracle(L, S.D1D, 0, shape=shape, w0=w0)
    assert o.tau == 1 and o.mix == S.MIX_ALL
    assert all((o.x[i] == w0).all() for i in range(L))
    b0, b1, b2 = (_batches(shape, L, k) for k in range(3))
    o.step(b0, 0.5)
    x1 = o.x.copy()
    o.step(b1, 0.5)
    x2 = o.x.copy()
    for i in range(L):
        g_at_x0 = lstm.loss_and_grad(shape, w0, b1[i][0], b1[i][1], np.float32)[1]
        g_at_x1 = lstm.loss_and_grad(shape, x1[i], b1[i][0], b1[i][1], np.float32)[1]
        assert (o.last_grads[i] == g_at_x0).all()
        assert np.abs(g_at_x1 - g_at_x0).max() > 1e-6
    o.step(b2, 0.5)
    for i in range(L):
        g_at_x1 = lstm.loss_and_grad(shape, x1[i], b2[i][0], b2[i][1], np.float32)[1]
        assert (o.last_grads[i] == g_at_x1).all()
    # models stay heterogeneous under delay-by-one although mixing is a full average
    assert np.abs(x2[0] - x2[1]).max() > 0
