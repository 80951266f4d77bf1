"""Oracle: the ADPSGD recurrence (test infrastructure; plain numpy, float32).

State x_i^k (one flat float32 vector per learner), i = 0..L-1.  One iteration
(Algorithm 1 and Eq. 2 of the paper, W_{k+1} = W_k T_k - a_k g(Phi_k, xi_k)):

  1. (order, partner, active) = schedule(seed, k)
  2. every active learner evaluates its minibatch gradient at x_i^{k-tau}
     (tau = 0: Algorithm 3, the local model before mixing; tau = 1: delay by
     one, Eq. for Phi_k in Section III-D, with x^{-1} := x^0)
  3. x_i^{k+1} = sum_j T_k[i, j] x_j^k - lr * g_i^k ; a straggler keeps x_i^k.

Rounding order of step 3 in float32 (the paper states none; this is the
formula evaluated left to right, every operation rounded once, no fused
multiply-add):
  PAIR  m = (x_i + x_j) * 0.5            (self-matched: m = x_i)
  TRI   m = ((x_left + x_i) + x_right) * (1/3)
  ALL   m = (((x_0 + x_1) + x_2) + ...) * (1/L)
  x_i^{k+1} = m - (lr * g_i)

The synchronous baseline (SDPSGD: Section III-A, Algorithm 2) applies the same
operations in the other order, W_{k+1} = (W_k - a_k g(W_k, xi_k)) T with
T = 11'/L: every learner updates its own model, then all models are averaged,
  u_j = x_j - (lr * g_j)
  x_i^{k+1} = (((u_0 + u_1) + u_2) + ...) * (1/L)      for every i,
so all learners hold the same model after every iteration.

The hybrid strategy of Section V (super-learners of S consecutive learners that
average synchronously, joined by the asynchronous ring): the mean of every
super-learner a first, then the ring operator on those means,
  m_a = (((x_{aS} + x_{aS+1}) + ...) + x_{aS+S-1}) * (1/S)
  PAIR  m = (m_a + m_b) * 0.5   (b the matched super-learner; unmatched: m = m_a)
  TRI   m = ((m_left + m_a) + m_right) * (1/3)      (a single super-learner: m = m_a)
  x_i^{k+1} = m - (lr * g_i)     for every learner i of super-learner a.
"""
import numpy as np
from . import schedule as S
from . import lstm


def init_model(seed, P, scale):
    """w_0[e] = (2 u01(seed, INIT, 0, e) - 1) * scale, rounded to float32."""
    out = np.empty(P, dtype=np.float32)
    for e in range(P):
        out[e] = np.float32((2.0 * S.u01(seed, S.STREAM_INIT, 0, e) - 1.0) * float(np.float32(scale)))
    return out


def mix_update(x, g, mix, order, partner, active, lr, update_first=False, group_size=1):
    """One application of step 3 to x [L][P] float32 with g [L][P] float32.
    Returns the new [L][P] array; x is not modified.
    update_first: the synchronous baseline's order (local update, then the
    average of all learners); defined for the all-learner mean with nobody
    inactive.
    group_size: hybrid mixes only; order / partner / active then describe the
    ring of the L / group_size super-learners."""
    x = np.asarray(x, dtype=np.float32)
    L = x.shape[0]
    lr = np.float32(lr)
    out = np.empty_like(x)
    ring = S.ring_mix_of(mix)
    if ring is not None:
        Sz = int(group_size)
        G = len(order)
        if Sz < 1 or G * Sz != L or update_first or not all(active):
            raise ValueError("hybrid mixing: L = G * group_size learners, nobody inactive")
        if ring == S.MIX_TRI and G == 2:
            raise ValueError("ring-neighbour mixing across super-learners needs at least 3 of them (or a single one)")
        means = []
        for a in range(G):
            s = x[a * Sz].copy()
            for j in range(1, Sz):
                s = s + x[a * Sz + j]
            means.append(s * (np.float32(1.0) / np.float32(Sz)))
        pos = {order[p]: p for p in range(G)}
        for a in range(G):
            if G == 1:
                m = means[a]
            elif ring == S.MIX_PAIR:
                b = partner[a]
                m = means[a] if b == a else (means[a] + means[b]) * np.float32(0.5)
            else:
                p = pos[a]
                left, right = order[(p - 1) % G], order[(p + 1) % G]
                m = ((means[left] + means[a]) + means[right]) * (np.float32(1.0) / np.float32(3.0))
            for i in range(a * Sz, (a + 1) * Sz):
                out[i] = m - (lr * np.asarray(g[i], dtype=np.float32))
        return out
    if update_first:
        if mix != S.MIX_ALL or not all(active):
            raise ValueError("update-then-average is the all-learner mean over every learner")
        s = x[0] - (lr * np.asarray(g[0], dtype=np.float32))
        for j in range(1, L):
            s = s + (x[j] - (lr * np.asarray(g[j], dtype=np.float32)))
        out[:] = s * (np.float32(1.0) / np.float32(L))
        return out
    if mix == S.MIX_TRI and L < 3:
        raise ValueError("ring-neighbour mixing (weights 1/3, Eq. 9) needs at least 3 learners")
    if mix == S.MIX_ALL:
        s = x[0].copy()
        for j in range(1, L):
            s = s + x[j]
        m_all = s * (np.float32(1.0) / np.float32(L))
    pos = {order[p]: p for p in range(L)}
    for i in range(L):
        if not active[i]:
            out[i] = x[i]
            continue
        if mix == S.MIX_ALL:
            m = m_all
        elif mix == S.MIX_PAIR:
            j = partner[i]
            m = x[i] if j == i else (x[i] + x[j]) * np.float32(0.5)
        elif mix == S.MIX_TRI:
            p = pos[i]
            left, right = order[(p - 1) % L], order[(p + 1) % L]
            m = ((x[left] + x[i]) + x[right]) * (np.float32(1.0) / np.float32(3.0))
        else:
            raise ValueError("mix")
        out[i] = m - (lr * np.asarray(g[i], dtype=np.float32))
    return out


def consensus_distance(x):
    """sum_i ||x_i - xbar||^2 over the rows x_i of x, xbar their mean; everything in float64."""
    x = np.asarray(x, dtype=np.float64)
    xbar = x.mean(axis=0)
    d = x - xbar
    return float((d * d).sum())


class Oracle:
    """L learners, model-bearing (shape given) or model-free (flat_params)."""

    def __init__(self, L, pattern, seed, shape=None, flat_params=0, mix=None, tau=None,
                 straggler_p=0.0, w0=None, x0=None, bf16_gemm=False, group_size=1):
        self.L, self.pattern, self.seed = L, pattern, seed
        self.group_size = int(group_size)
        self.hybrid = S.ring_mix_of(mix) is not None
        if self.hybrid and (self.group_size < 1 or L % self.group_size or straggler_p > 0.0 or pattern in (S.D1D, S.SDPSGD)):
            raise ValueError("hybrid mixing: a ring pattern, L a multiple of group_size, no stragglers")
        self.ring_size = L // self.group_size if self.hybrid else L
        self.shape = shape
        self.P = lstm.param_count(shape) if shape is not None else int(flat_params)
        self.mix = mix if mix is not None else (S.MIX_ALL if pattern in (S.D1D, S.SDPSGD) else S.MIX_PAIR)
        self.tau = tau if tau is not None else (1 if pattern == S.D1D else 0)
        self.update_first = pattern == S.SDPSGD
        if self.update_first and (self.mix != S.MIX_ALL or self.tau != 0 or straggler_p > 0.0):
            raise ValueError("the synchronous baseline averages all learners, without staleness or stragglers")
        self.straggler_p = straggler_p
        self.bf16_gemm = bf16_gemm
        if x0 is not None:
            self.x = np.array(x0, dtype=np.float32).reshape(L, self.P)
        else:
            self.x = np.tile(np.asarray(w0, dtype=np.float32).reshape(1, self.P), (L, 1))
        self.x_prev = self.x.copy()      # x^{-1} := x^0
        self.k = 0
        self.last_grads = None
        self.last_losses = None
        self.last_schedule = None

    def gradient_point(self):
        return self.x_prev if self.tau == 1 else self.x

    def step(self, batches, lr, grads=None, workers=1, active=None):
        """batches: list of (feats, labels) per learner; or grads [L][P] given
        directly in model-free mode.  workers > 1 spreads the outer loop over the
        learners, whose gradients are independent of each other (Algorithm 1: the
        learners run concurrently), over that many threads; every learner's
        arithmetic is unchanged, so the result is the same as with one.
        active: the learners that take part, given by the caller (the others are
        the iteration's stragglers) instead of the seeded draw."""
        if active is not None and (self.hybrid or self.tau != 0 or self.mix != S.MIX_PAIR) and not all(active):
            raise ValueError("a learner can sit out only on a ring with pairwise mixing and tau = 0")
        order, partner, active = S.schedule(self.pattern, self.seed, self.k, self.ring_size, self.straggler_p, active)
        self.last_schedule = (order, partner, active)
        if self.hybrid:      # the schedule is over super-learners; every learner computes a gradient
            active = [1] * self.L
        if grads is None:
            at = self.gradient_point()
            grads = np.zeros((self.L, self.P), dtype=np.float32)
            losses = np.zeros(self.L, dtype=np.float32)

            def one(i):
                feats, labels = batches[i]
                losses[i], grads[i] = lstm.loss_and_grad(self.shape, at[i], feats, labels,
                                                         np.float32, self.bf16_gemm)
            todo = [i for i in range(self.L) if active[i]]
            if workers > 1:
                from concurrent.futures import ThreadPoolExecutor
                with ThreadPoolExecutor(max_workers=workers) as ex:
                    list(ex.map(one, todo))
            else:
                for i in todo:
                    one(i)
            self.last_losses = losses
        self.last_grads = grads
        if self.hybrid:
            new = mix_update(self.x, grads, self.mix, order, partner, [1] * self.ring_size, lr, False, self.group_size)
        else:
            new = mix_update(self.x, grads, self.mix, order, partner, active, lr, self.update_first)
        self.x_prev = self.x
        self.x = new
        self.k += 1

    def average(self):
        """Output model of Algorithm 1: the learner average (float64 mean)."""
        return self.x.astype(np.float64).mean(axis=0)

    def consensus(self):
        """Consensus distance sum_i ||x_i - xbar||^2 of the learners' models (float64): the quantity that
        the mixing operator contracts by its second largest eigenvalue magnitude (Section II, Eq. 5-7)."""
        return consensus_distance(self.x)
