"""Pins for the oracle's column-weighted dQ (an unbiased sparse estimate of dQ; not in the paper, which keeps dQ
exact in Alg. 2): a finite-difference definition that shares no formula with it, the special case w = 1, and the
expectation over every selection under the sampling laws the library's host routines offer."""
import itertools

import numpy as np

from oracle import attention as A


def _inputs(seed, B, Hq, Hkv, N, D):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((B, Hq, N, D)), rng.standard_normal((B, Hkv, N, D)),
            rng.standard_normal((B, Hkv, N, D)), rng.standard_normal((B, Hq, N, D)))


def _loss_with_mixed_queries(q_var, q_fix, k, v, d_o, q_start, scale, cols):
    """L = sum(O * dO) of one head when the scores of the columns in `cols` are formed with q_var and all other
    scores with q_fix: a plain softmax forward.  Its gradient with respect to q_var at q_var = q_fix is the part
    of dQ that flows through the scores of those columns."""
    C, L = q_var.shape[0], q_start + q_var.shape[0]
    total = 0.0
    for r in range(C):
        p = q_start + r
        s = np.array([scale * ((q_var if c in cols else q_fix)[r] @ k[c]) for c in range(p + 1)])
        e = np.exp(s - s.max())
        o = (e / e.sum()) @ v[:p + 1]
        total += o @ d_o[r]
    return total


def test_weighted_dq_is_the_gradient_through_the_weighted_columns():
    B, Hq, Hkv, N, D, C = 1, 2, 1, 8, 3, 4
    Q, K, V, dO = _inputs(1, B, Hq, Hkv, N, D)
    s, q_start = 0.7, 4
    q = Q[:, :, q_start:]
    o, lse = A.chunk_attn_fwd(q, K, V, q_start, s)
    w = np.array([0.0, 2.5, 2.5, 0.0, 0.0, 1.0, 1.0, 0.25])      # per column, includes zero and fractional weights
    for tier in ("loops", "matmul"):
        got = A.chunk_attn_dq_weighted(q, K, V, o, lse, dO[:, :, q_start:], q_start, s, w, tier)
        want = np.zeros_like(got)
        eps = 1e-6
        for h in range(Hq):
            for wv in sorted(set(w) - {0.0}):
                cols = {c for c in range(N) if w[c] == wv}
                for r in range(C):
                    for d in range(D):
                        qp, qm = q[0, h].copy(), q[0, h].copy()
                        qp[r, d] += eps
                        qm[r, d] -= eps
                        fp = _loss_with_mixed_queries(qp, q[0, h], K[0, 0], V[0, 0], dO[0, h, q_start:], q_start, s, cols)
                        fm = _loss_with_mixed_queries(qm, q[0, h], K[0, 0], V[0, 0], dO[0, h, q_start:], q_start, s, cols)
                        want[0, h, r, d] += wv * (fp - fm) / (2 * eps)
        assert np.abs(got - want).max() <= 1e-7 * max(1.0, np.abs(want).max()), tier


def test_unit_weights_give_the_exact_dq_and_chunks_add_up():
    B, Hq, Hkv, N, D, C = 2, 4, 2, 24, 8, 6
    Q, K, V, dO = _inputs(2, B, Hq, Hkv, N, D)
    s, j = 0.35, 3
    q_start = j * C
    q, do = Q[:, :, q_start:q_start + C], dO[:, :, q_start:q_start + C]
    o, lse = A.chunk_attn_fwd(q, K, V, q_start, s)
    dq, _, _ = A.chunk_attn_bwd(q, K, V, o, lse, do, q_start, s)
    L = q_start + C
    assert np.abs(A.chunk_attn_dq_weighted(q, K, V, o, lse, do, q_start, s, np.ones(L)) - dq).max() <= 1e-13
    parts = []
    for i in range(j + 1):                                 # one chunk of columns at a time
        w = np.zeros(L)
        w[i * C:(i + 1) * C] = 1.0
        parts.append(A.chunk_attn_dq_weighted(q, K, V, o, lse, do, q_start, s, w))
    assert np.abs(sum(parts) - dq).max() <= 1e-13
    assert all(np.abs(x).max() > 1e-3 for x in parts)      # every chunk of columns matters in this example
    small = A.chunk_attn_dq_weighted(q[:1, :2, :2, :], K[:1, :1, :, :], V[:1, :1, :, :], o[:1, :2, :2], lse[:1, :2, :2],
                                     do[:1, :2, :2], q_start, s, np.linspace(0.5, 2.0, q_start + 2), "loops")
    same = A.chunk_attn_dq_weighted(q[:1, :2, :2, :], K[:1, :1, :, :], V[:1, :1, :, :], o[:1, :2, :2], lse[:1, :2, :2],
                                    do[:1, :2, :2], q_start, s, np.linspace(0.5, 2.0, q_start + 2), "matmul")
    assert np.abs(small - same).max() <= 1e-13


def test_expectation_over_all_selections():
    """Call j of a selected chunk visits its own columns (weight 1) and the columns of the other selected earlier
    chunks.  Fixed-size draw of t of k chunks: given j is selected, an earlier chunk is selected with probability
    (t-1)/(k-1), so weight (k-1)/(t-1) is exactly unbiased and the factor k/t of the paper's dK/dV rule leaves the
    cross terms scaled by k(t-1)/(t(k-1)).  Independent inclusion with probability p and weight 1/p is exactly
    unbiased as well."""
    B, Hq, Hkv, N, D, C = 1, 2, 1, 20, 4, 4
    k, t, j = 5, 3, 3
    Q, K, V, dO = _inputs(3, B, Hq, Hkv, N, D)
    s = 0.5
    q_start = j * C
    q, do = Q[:, :, q_start:q_start + C], dO[:, :, q_start:q_start + C]
    o, lse = A.chunk_attn_fwd(q, K, V, q_start, s)
    exact, _, _ = A.chunk_attn_bwd(q, K, V, o, lse, do, q_start, s)
    own = np.concatenate([np.zeros(q_start), np.ones(C)])
    own_part = A.chunk_attn_dq_weighted(q, K, V, o, lse, do, q_start, s, own)

    def estimate(earlier, weight):
        w = own.copy()
        for i in earlier:
            w[i * C:(i + 1) * C] = weight
        return A.chunk_attn_dq_weighted(q, K, V, o, lse, do, q_start, s, w)

    draws = [I for I in itertools.combinations(range(k), t) if j in I]
    for weight, cross in (((k - 1) / (t - 1), 1.0), (k / t, k * (t - 1) / (t * (k - 1)))):
        mean = sum(estimate([i for i in I if i < j], weight) for I in draws) / len(draws)
        want = own_part + cross * (exact - own_part)
        assert np.abs(mean - want).max() <= 1e-12 * np.abs(exact).max()
    p = 0.4
    mean = np.zeros_like(exact)
    for n in range(j + 1):
        for E in itertools.combinations(range(j), n):
            mean += p ** n * (1 - p) ** (j - n) * estimate(E, 1 / p)
    assert np.abs(mean - exact).max() <= 1e-12 * np.abs(exact).max()
    # the layer routine carries the same weights per chunk
    wq = np.array([2.0, 0.0, 2.0, 1.0])
    dQ, _, _ = A.weighted_layer(Q, K, V, dO, C, s, [(j, np.ones(j + 1), wq)])
    assert np.abs(dQ[:, :, q_start:q_start + C] - estimate([0, 2], 2.0)).max() <= 1e-13
