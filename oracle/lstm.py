"""Oracle: loss and gradient of the stacked (bi)directional LSTM acoustic model
(test infrastructure; plain numpy, one library matmul per GEMM step).

Model (Section IV of the paper): N stacked LSTM layers, optionally
bidirectional with the two directions' outputs concatenated, an optional
*linear* bottleneck projection, an affine output layer, softmax, and the
cross-entropy loss averaged over all frames of the minibatch (the 1/M mean of
Algorithm 1 taken over B segments x T frames).  The LSTM is unrolled over the T
frames of a segment with zero initial state (segments do not overlap).

Readings where the paper is silent: vanilla LSTM (no peepholes, clipping or
recurrent projection), gate blocks ordered (i, f, g, o), one bias per gate.

Flat parameter layout (all row-major, rows = output units):
  for each layer l:  W_x[l] [D][4H][I_l],  W_h[l] [D][4H][H],  b[l] [D][4H]
  then (if bottleneck) W_p [Bn][D*H], b_p [Bn]
  then W_o [C][F], b_o [C]          with F = Bn or D*H
where I_0 = input_dim and I_l = D*H above.
"""
from collections import namedtuple
import numpy as np

Shape = namedtuple("Shape", "input_dim hidden layers bidirectional bottleneck classes batch frames")


def layout(shape):
    """[(name, offset, rows, cols)] of every tensor in the flat vector, and P."""
    D = 2 if shape.bidirectional else 1
    H = shape.hidden
    out, off = [], 0
    for l in range(shape.layers):
        Il = shape.input_dim if l == 0 else D * H
        out.append(("Wx%d" % l, off, D * 4 * H, Il)); off += D * 4 * H * Il
        out.append(("Wh%d" % l, off, D * 4 * H, H)); off += D * 4 * H * H
        out.append(("b%d" % l, off, 1, D * 4 * H)); off += D * 4 * H
    F = D * H
    if shape.bottleneck > 0:
        out.append(("Wp", off, shape.bottleneck, F)); off += shape.bottleneck * F
        out.append(("bp", off, 1, shape.bottleneck)); off += shape.bottleneck
        F = shape.bottleneck
    out.append(("Wo", off, shape.classes, F)); off += shape.classes * F
    out.append(("bo", off, 1, shape.classes)); off += shape.classes
    return out, off


def param_count(shape):
    return layout(shape)[1]


def round_bf16(a):
    """Round float32 values to the nearest bfloat16 (ties to even), returned as
    float32.  Used only by the optional bf16-operand emulation."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    out = (r & 0xFFFFFFFF).astype(np.uint32).view(np.float32).reshape(a.shape)
    return np.where(np.isfinite(a), out, a)


def _sigmoid(a):
    one = a.dtype.type(1)
    return one / (one + np.exp(-a))


class _Views:
    def __init__(self, shape, vec):
        self.t = {}
        for name, off, r, c in layout(shape)[0]:
            self.t[name] = vec[off:off + r * c].reshape(r, c)


def loss_and_grad(shape, w, feats, labels, dtype=np.float32, bf16_gemm=False,
                  want_grad=True):
    """Mean cross-entropy over the B*T frames and its gradient w.r.t. the flat
    parameter vector.  feats [T][B][I], labels [T][B] (ints).

    dtype selects the arithmetic (float32 = the parity oracle, float64 = the
    version used for finite-difference pins).  bf16_gemm rounds both operands
    of every matmul to bfloat16 first (diagnostic only)."""
    T, B = shape.frames, shape.batch
    H, D = shape.hidden, (2 if shape.bidirectional else 1)
    C = shape.classes
    w = np.asarray(w, dtype=dtype)
    P = param_count(shape)
    assert w.shape == (P,)
    V = _Views(shape, w).t

    def mm(a, b):
        if bf16_gemm:
            a = round_bf16(a.astype(np.float32)).astype(dtype)
            b = round_bf16(b.astype(np.float32)).astype(dtype)
        return a @ b

    x = np.asarray(feats, dtype=dtype).reshape(T, B, shape.input_dim)
    saved = []
    inp = x
    for l in range(shape.layers):
        Il = inp.shape[2]
        Wx, Wh, b = V["Wx%d" % l], V["Wh%d" % l], V["b%d" % l].reshape(-1)
        out = np.zeros((T, B, D * H), dtype=dtype)
        per_dir = []
        for d in range(D):
            Wxd, Whd, bd = Wx[d * 4 * H:(d + 1) * 4 * H], Wh[d * 4 * H:(d + 1) * 4 * H], b[d * 4 * H:(d + 1) * 4 * H]
            gx = (mm(inp.reshape(T * B, Il), Wxd.T) + bd).reshape(T, B, 4 * H)
            gates = np.zeros((T, B, 4 * H), dtype=dtype)   # post-activation i,f,g,o
            cs = np.zeros((T, B, H), dtype=dtype)
            hs = np.zeros((T, B, H), dtype=dtype)
            h_prev = np.zeros((B, H), dtype=dtype)
            c_prev = np.zeros((B, H), dtype=dtype)
            ts = range(T) if d == 0 else range(T - 1, -1, -1)
            for t in ts:
                a = gx[t] + mm(h_prev, Whd.T)
                i = _sigmoid(a[:, 0:H])
                f = _sigmoid(a[:, H:2 * H])
                g = np.tanh(a[:, 2 * H:3 * H])
                o = _sigmoid(a[:, 3 * H:4 * H])
                c = f * c_prev + i * g
                h = o * np.tanh(c)
                gates[t, :, 0:H], gates[t, :, H:2 * H] = i, f
                gates[t, :, 2 * H:3 * H], gates[t, :, 3 * H:4 * H] = g, o
                cs[t], hs[t] = c, h
                h_prev, c_prev = h, c
            out[:, :, d * H:(d + 1) * H] = hs
            per_dir.append((gates, cs, hs))
        saved.append((inp, per_dir))
        inp = out

    top = inp.reshape(T * B, D * H)
    if shape.bottleneck > 0:
        z = mm(top, V["Wp"].T) + V["bp"].reshape(-1)
    else:
        z = top
    logits = mm(z, V["Wo"].T) + V["bo"].reshape(-1)
    y = np.asarray(labels).reshape(T * B).astype(np.int64)
    mx = logits.max(axis=1, keepdims=True)
    e = np.exp(logits - mx)
    s = e.sum(axis=1, keepdims=True)
    rows = np.arange(T * B)
    logp_y = (logits[rows, y] - mx[:, 0]) - np.log(s[:, 0])
    n = dtype(T * B)
    loss = -(logp_y.sum() / n)
    if not want_grad:
        return loss, None

    grad = np.zeros(P, dtype=dtype)
    G = _Views(shape, grad).t
    dlogits = e / s
    dlogits[rows, y] -= dtype(1)
    dlogits = dlogits / n
    G["Wo"][:] = mm(dlogits.T, z)
    G["bo"][:] = dlogits.sum(axis=0)
    dz = mm(dlogits, V["Wo"])
    if shape.bottleneck > 0:
        G["Wp"][:] = mm(dz.T, top)
        G["bp"][:] = dz.sum(axis=0)
        dtop = mm(dz, V["Wp"])
    else:
        dtop = dz
    dout = dtop.reshape(T, B, D * H)

    for l in range(shape.layers - 1, -1, -1):
        inp_l, per_dir = saved[l]
        Il = inp_l.shape[2]
        Wx, Wh = V["Wx%d" % l], V["Wh%d" % l]
        dinp = np.zeros((T, B, Il), dtype=dtype)
        for d in range(D):
            gates, cs, hs = per_dir[d]
            Wxd, Whd = Wx[d * 4 * H:(d + 1) * 4 * H], Wh[d * 4 * H:(d + 1) * 4 * H]
            da = np.zeros((T, B, 4 * H), dtype=dtype)
            hprev_all = np.zeros((T, B, H), dtype=dtype)
            dh_rec = np.zeros((B, H), dtype=dtype)
            dc_rec = np.zeros((B, H), dtype=dtype)
            # reverse of the processing order of this direction
            ts = range(T - 1, -1, -1) if d == 0 else range(T)
            step = -1 if d == 0 else 1   # index of the previous processed frame = t + step
            for t in ts:
                tp = t + step
                inside = 0 <= tp < T
                c_prev = cs[tp] if inside else np.zeros((B, H), dtype=dtype)
                if inside:
                    hprev_all[t] = hs[tp]
                i, f = gates[t, :, 0:H], gates[t, :, H:2 * H]
                g, o = gates[t, :, 2 * H:3 * H], gates[t, :, 3 * H:4 * H]
                tc = np.tanh(cs[t])
                dh = dout[t, :, d * H:(d + 1) * H] + dh_rec
                do = dh * tc
                dc = dc_rec + dh * o * (dtype(1) - tc * tc)
                di, dg, df = dc * g, dc * i, dc * c_prev
                dc_rec = dc * f
                da[t, :, 0:H] = di * i * (dtype(1) - i)
                da[t, :, H:2 * H] = df * f * (dtype(1) - f)
                da[t, :, 2 * H:3 * H] = dg * (dtype(1) - g * g)
                da[t, :, 3 * H:4 * H] = do * o * (dtype(1) - o)
                dh_rec = mm(da[t], Whd)
            da2 = da.reshape(T * B, 4 * H)
            G["Wx%d" % l][d * 4 * H:(d + 1) * 4 * H] = mm(da2.T, inp_l.reshape(T * B, Il))
            G["Wh%d" % l][d * 4 * H:(d + 1) * 4 * H] = mm(da2.T, hprev_all.reshape(T * B, H))
            G["b%d" % l].reshape(-1)[d * 4 * H:(d + 1) * 4 * H] = da2.sum(axis=0)
            if l > 0:
                dinp += mm(da2, Wxd).reshape(T, B, Il)
        dout = dinp
    return loss, grad
