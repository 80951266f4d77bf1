"""Oracle: the per-iteration communication schedule (test infrastructure).

What the paper fixes
  * every iteration selects a doubly stochastic mixing matrix T_k (Algorithm 1);
  * fixed mixing uses the learners' ring order as is (Section III-B);
  * random mixing draws a fresh permutation of the ring each iteration with a
    Fisher-Yates shuffle (Section III-C);
  * delay-by-one mixes with T = 11'/L (Section III-D);
  * the synchronous baseline (SDPSGD, Section III-A, Algorithm 2) uses the same
    T = 11'/L, applied after every learner's local update; it has no ring order
    to choose and waits for every learner.

What it leaves open, and the reading taken here
  * the random source: a stateless counter-based 64-bit generator,
    u64(seed, stream, k, idx) = mix(mix(mix(seed + GOLDEN*(stream+1)) + k) + idx)
    with the SplitMix64 output function as `mix`;
  * pairwise mixing (x_i + x_j)/2 on a ring: a perfect matching along the ring
    order, whose phase alternates with k on the fixed ring so that the ring is
    connected over two iterations; on the random ring the phase is 0;
  * a straggler (inactive learner) takes no part in the iteration; the learner
    it would have been matched with keeps its own model for the mixing term.

Hierarchy (Section V, the hybrid strategy and its figure): consecutive blocks of
S learners form super-learners that average synchronously among themselves, and
the G = L/S super-learners form the asynchronous ring.  The schedule of such a
run is the schedule above over the G super-learners; the mixing matrix is the
ring operator over super-learners with every entry spread evenly over the S x S
block of its two groups.
"""
import numpy as np

MASK64 = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15

STREAM_PERM = 1   # Fisher-Yates draws
STREAM_MASK = 2   # straggler mask draws
STREAM_INIT = 3   # initial model draws

FIXED_RING, RANDOM_RING, D1D, SDPSGD = 0, 1, 2, 3
MIX_PAIR, MIX_TRI, MIX_ALL = 0, 1, 2
MIX_HYBRID_PAIR, MIX_HYBRID_TRI = 3, 4    # synchronous mean inside super-learners, PAIR / TRI ring across them


def mix64(z):
    """SplitMix64 output function on a 64-bit integer."""
    z &= MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
    return z ^ (z >> 31)


def u64(seed, stream, k, idx):
    a = mix64(seed + GOLDEN * (stream + 1))
    b = mix64(a + k)
    return mix64(b + idx)


def u01(seed, stream, k, idx):
    """Uniform double in [0,1): the top 53 bits of u64."""
    return (u64(seed, stream, k, idx) >> 11) * (1.0 / 9007199254740992.0)


def ring_order(pattern, seed, k, L):
    """Ring order r_k: identity, or a Fisher-Yates (Durstenfeld) shuffle of it
    for the random ring (Section III-C)."""
    r = list(range(L))
    if pattern == RANDOM_RING:
        for p in range(L - 1, 0, -1):
            q = u64(seed, STREAM_PERM, k, p) % (p + 1)
            r[p], r[q] = r[q], r[p]
    return r


def active_mask(seed, k, L, straggler_p):
    """active[i] = 0 when learner i is a straggler in iteration k."""
    if straggler_p <= 0.0:
        return [1] * L
    p = float(np.float32(straggler_p))
    return [1 if u01(seed, STREAM_MASK, k, i) >= p else 0 for i in range(L)]


def schedule(pattern, seed, k, L, straggler_p=0.0, active=None):
    """(order, partner, active) for iteration k.

    partner is the pairwise matching (an involution; partner[i] == i means that
    learner i mixes with nobody this iteration).  active: the stragglers of the
    iteration given by the caller (a learner that is observed to be late,
    Section IV-D) instead of drawn with probability straggler_p."""
    order = ring_order(pattern, seed, k, L)
    active = active_mask(seed, k, L, straggler_p) if active is None else [1 if a else 0 for a in active]
    if len(active) != L:
        raise ValueError("one flag per learner")
    phase = (k % 2) if pattern != RANDOM_RING else 0
    partner = list(range(L))
    for m in range(L // 2):
        a = order[(2 * m + phase) % L]
        b = order[(2 * m + 1 + phase) % L]
        if a != b:
            partner[a], partner[b] = b, a
    for i in range(L):
        if not active[i]:
            j = partner[i]
            partner[j] = j
            partner[i] = i
    return order, partner, active


def ring_mix_of(mix):
    """The ring operator a hybrid mix applies across super-learners (None for a plain mix)."""
    return {MIX_HYBRID_PAIR: MIX_PAIR, MIX_HYBRID_TRI: MIX_TRI}.get(mix)


def mixing_matrix(mix, order, partner, active, group_size=1):
    """Dense T_k (float64) such that the mixed model of learner i is
    sum_j T[i, j] x_j  (Algorithm 1, model averaging step).

    Hybrid mixes: order / partner / active describe the ring of the G = len(order)
    super-learners; learner i belongs to super-learner i // group_size and the
    result is the (G * group_size)-square matrix
    T[i, j] = T_ring[i // S, j // S] / S  (the synchronous mean inside a
    super-learner composed with the ring operator across super-learners)."""
    if ring_mix_of(mix) is not None:
        G, Sz = len(order), int(group_size)
        if Sz < 1:
            raise ValueError("group_size")
        if G == 1:
            Tg = np.ones((1, 1))
        else:
            Tg = mixing_matrix(ring_mix_of(mix), order, partner, active)
        T = np.zeros((G * Sz, G * Sz))
        for i in range(G * Sz):
            for j in range(G * Sz):
                T[i, j] = Tg[i // Sz, j // Sz] / Sz
        return T
    L = len(order)
    T = np.zeros((L, L))
    if mix == MIX_ALL:
        T[:] = 1.0 / L
    elif mix == MIX_PAIR:
        for i in range(L):
            j = partner[i]
            if j == i:
                T[i, i] = 1.0
            else:
                T[i, i] = 0.5
                T[i, j] = 0.5
    elif mix == MIX_TRI:
        # Eq. (T^f) on the ring order: T^r = P' T^f P (Section III-C).  The circulant of Eq. 9 has three
        # distinct positions per row (left neighbour, self, right neighbour): it is defined for L >= 3.
        if L < 3:
            raise ValueError("ring-neighbour mixing (weights 1/3) needs at least 3 learners")
        for p in range(L):
            i = order[p]
            for q in (p - 1, p, p + 1):
                T[i, order[q % L]] += 1.0 / 3.0
    else:
        raise ValueError("mix")
    for i in range(L):
        if not active[i] and mix == MIX_PAIR:
            assert T[i, i] == 1.0
    return T
