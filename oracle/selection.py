"""SpaCO chunk selection, compensation factor and per-call chunk weights (oracle).

TEST INFRASTRUCTURE ONLY (see the package docstring).

Alg. 2 draws t different chunks out of the k (selection step) but names no generator.
This build fixes one so that the host library and this oracle can be compared
bit for bit:

  * integer stream: SplitMix64 (Steele, Lea, Flood 2014; Vigna's public-domain
    reference): state += 0x9E3779B97F4A7C15, output = finaliser(state);
  * stream key for (seed, step): state0 = finaliser(seed ^ finaliser(step + GOLDEN));
  * bounded draw in [0, m): rejection sampling, accept u < floor(2^64 / m) * m,
    return u mod m (so every residue is exactly equally likely);
  * t of k without replacement: the first t steps of a Fisher-Yates shuffle of
    0 .. k-1 (position i swaps with i + draw(k - i));
  * output sorted in descending order, which is the order in which the chunks
    must be back-propagated (reverse order, as in Alg. 1's second loop).
"""
from __future__ import annotations

import numpy as np

_MASK = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15


def _finalise(z):
    z &= _MASK
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK
    return z ^ (z >> 31)


class SplitMix64:
    """The SplitMix64 stream started from a given 64-bit state."""

    def __init__(self, state):
        self.state = state & _MASK

    def next(self):
        self.state = (self.state + _GOLDEN) & _MASK
        return _finalise(self.state)

    def below(self, m):
        """Uniform integer in [0, m) by rejection."""
        limit = ((1 << 64) // m) * m
        while True:
            u = self.next()
            if u < limit:
                return u % m


def stream_for(seed, step):
    return SplitMix64(_finalise((seed & _MASK) ^ _finalise((step + _GOLDEN) & _MASK)))


def select_chunks(seed, step, k, t):
    """Alg. 2, selection step: t distinct chunk indices of 0..k-1, descending."""
    if not (1 <= t <= k):
        raise ValueError("need 1 <= t <= k")
    rng = stream_for(seed, step)
    perm = list(range(k))
    for i in range(t):
        r = i + rng.below(k - i)
        perm[i], perm[r] = perm[r], perm[i]
    return np.array(sorted(perm[:t], reverse=True), dtype=np.int32)


def select_bernoulli(seed, step, k, q):
    """Independent inclusion of every chunk with probability q (the law under which the survival argument of
    Sec. 5, "Compensation Factor", is exact): chunk i is selected iff the i-th draw of the (seed, step) stream is
    below floor(q * 2^64).  Returns the selected indices, descending (possibly empty)."""
    if not (0.0 < q <= 1.0):
        raise ValueError("need 0 < q <= 1")
    rng = stream_for(seed, step)
    threshold = int(q * 2.0 ** 64) if q < 1.0 else 1 << 64     # exact: scaling a double by a power of two
    picked = [i for i in range(k) if rng.next() < threshold]
    return np.array(picked[::-1], dtype=np.int32)


def compensation_factor(k, t, cap=None):
    """k/t (Sec. 5, "Compensation Factor"), optionally limited to `cap` (Sec. 6.4)."""
    lam = k / t
    return lam if cap is None else min(lam, cap)


def chunk_weights(selected, j, factor):
    """Weight vector w[0..j] of the backward call for chunk j.

    w[i] = factor for an earlier selected chunk, w[j] = 1 for the chunk's own
    rows, 0 for every chunk that is not selected (Alg. 2; appendix listing).
    fp32, because that is the type the library's weight argument has.
    """
    w = np.zeros(j + 1, dtype=np.float32)
    for i in selected:
        if i < j:
            w[int(i)] = factor
    w[j] = 1.0
    return w


def gather_row_weights(selected, i, k, factor):
    """Row weights of the backward call for selected chunk i when the calls run in the transposed order (each call
    forms the finished gradient rows of its own chunk from its own and every later chunk's queries): one weight per
    chunk i .. k-1, 1 for chunk i itself, `factor` for a later selected chunk, 0 otherwise.  This is Alg. 2's
    weighting read column by column: call m deposits `factor` on an earlier selected chunk i (chunk_weights(sel, m)[i])
    exactly when m itself is back-propagated.  fp32."""
    w = np.zeros(k - i, dtype=np.float32)
    for m in selected:
        if i < m < k:
            w[int(m) - i] = factor
    w[0] = 1.0
    return w


def path_count(n, p):
    """Number of gradient chains of length p (p edges, p + 1 nodes) in the complete DAG on n chunks
    (Sec. 5, "Challenges in Unbiased Estimation", the binomial formula for d_p)."""
    from math import comb
    return comb(n, p + 1)


def path_ratio(k, t, p):
    """Dense-to-sparse ratio of the chain counts, k(k-1)...(k-p) / (t(t-1)...(t-p)) (same passage);
    its reciprocal is the probability that one given chain survives a uniform draw of t of the k chunks."""
    num = den = 1
    for i in range(p + 1):
        num *= k - i
        den *= t - i
    return num / den


def percall_weights(seed, step, j, t):
    """Policy "every chunk back-propagated, each call with its own draw": call j draws m = min(t, j) of its j
    earlier chunks uniformly (stream keyed by (seed, step * 2^20 + j)) and weights them j / m, its own rows 1.
    Every earlier chunk is included with probability m / j, so the expected weight of each is 1: the layer's dK/dV
    are unbiased, and dQ is exact because every chunk is back-propagated (one reading of "a few uniformly sampled
    earlier chunks plus the current chunk").  Returns w[0..j] (fp32)."""
    w = np.zeros(j + 1, dtype=np.float32)
    w[j] = 1.0
    m = min(t, j)
    if m > 0:
        for i in select_chunks(seed, step * (1 << 20) + j, j, m):
            w[int(i)] = np.float32(j / m)
    return w
