"""Pins for the SpaCO schedule in the oracle (Alg. 2 and the "Compensation Factor"
analysis of Sec. 5): degenerate case t = k, brute-force expectation over every
selection against the closed forms, weight-vector formulation, and the factor
values the paper states."""
import itertools
import os
from math import comb

import numpy as np
import pytest

from oracle import attention as A
from oracle import selection as S
from workloads import small_layer

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rel(x, ref):
    return np.abs(x - ref).max() / max(np.abs(ref).max(), 1e-300)


def layer(seed, B=1, Hq=4, Hkv=2, N=16, D=4):
    return {k: v.astype(np.float64) for k, v in small_layer(seed, B, Hq, Hkv, N, D).items()}


def pieces(x, C, s):
    """Per-call SeCO pieces: dQ_j and the contribution of call j to every chunk's rows."""
    N = x["q"].shape[2]
    k = N // C
    dq, dk, dv = {}, {}, {}
    for j in range(k):
        q = x["q"][:, :, j * C:(j + 1) * C]
        o, lse = A.chunk_attn_fwd(q, x["k"], x["v"], j * C, s)
        dq[j], dkj, dvj = A.chunk_attn_bwd(q, x["k"], x["v"], o, lse, x["do"][:, :, j * C:(j + 1) * C], j * C, s)
        for i in range(j + 1):
            dk[i, j] = dkj[:, :, i * C:(i + 1) * C]
            dv[i, j] = dvj[:, :, i * C:(i + 1) * C]
    return dq, dk, dv


def test_factor_values_stated_in_the_paper():
    with open(os.path.join(GOLDEN, "compensation_factor.txt")) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 9
    for k, t, cap, want in rows:
        got = S.compensation_factor(int(k), int(t), None if cap == "-" else float(cap))
        assert got == float(want)


def test_all_chunks_selected_is_seco():
    """t = k: factor 1 and every chunk back-propagated, i.e. Alg. 2 is Alg. 1."""
    x = layer(1)
    seco = A.seco_layer(x["q"], x["k"], x["v"], x["do"], 4, 0.5)
    spaco = A.spaco_layer(x["q"], x["k"], x["v"], x["do"], 4, 0.5, [0, 1, 2, 3],
                          S.compensation_factor(4, 4))
    for a, b in zip(seco, spaco):
        assert np.array_equal(a, b)


def test_unselected_chunks_receive_nothing():
    x = layer(2)
    _, _, dQ, gK, gV = A.spaco_layer(x["q"], x["k"], x["v"], x["do"], 4, 0.5, [3, 1], 2.0)
    for arr in (dQ, gK, gV):
        assert not arr[:, :, 0:4].any() and not arr[:, :, 8:12].any()
        assert arr[:, :, 4:8].any() and arr[:, :, 12:16].any()


@pytest.mark.parametrize("t", [1, 2, 3, 4])
def test_expectation_fixed_size_draw(t):
    """Alg. 2's draw (t distinct of k, every subset equally likely), enumerated.

    A chunk is selected with probability t/k and a pair with t(t-1)/(k(k-1)), so
      (k/t) E[dQ_j]  = dQ_j
      (k/t) E[gK_i]  = dK_i<-i + factor*(t-1)/(k-1) * sum_{j>i} dK_i<-j .
    With factor = k/t (paper) the cross terms carry k(t-1)/(t(k-1)); with
    factor = (k-1)/(t-1) the single-layer estimator is exactly unbiased up to
    the global t/k."""
    k, C, s = 4, 4, 0.5
    x = layer(3)
    dq, dk, dv = pieces(x, C, s)
    full = A.seco_layer(x["q"], x["k"], x["v"], x["do"], C, s)
    factors = [S.compensation_factor(k, t), 1.7]
    if t > 1:
        factors.append((k - 1) / (t - 1))
    for lam in factors:
        subsets = list(itertools.combinations(range(k), t))
        assert len(subsets) == comb(k, t)
        acc = [np.zeros_like(full[2]), np.zeros_like(full[3]), np.zeros_like(full[4])]
        for sub in subsets:
            out = A.spaco_layer(x["q"], x["k"], x["v"], x["do"], C, s, sub, lam)
            for a, o in zip(acc, out[2:]):
                a += o / len(subsets)
        cross = lam * (t - 1) / (k - 1)
        for i in range(k):
            rows = slice(i * C, (i + 1) * C)
            assert rel(k / t * acc[0][:, :, rows], dq[i]) < 1e-12
            want_k = dk[i, i] + cross * sum((dk[i, j] for j in range(i + 1, k)), np.zeros_like(dk[i, i]))
            want_v = dv[i, i] + cross * sum((dv[i, j] for j in range(i + 1, k)), np.zeros_like(dv[i, i]))
            assert rel(k / t * acc[1][:, :, rows], want_k) < 1e-12
            assert rel(k / t * acc[2][:, :, rows], want_v) < 1e-12
        if t > 1 and lam == (k - 1) / (t - 1):
            for a, f in zip(acc, full[2:]):
                assert rel(k / t * a, f) < 1e-12


@pytest.mark.parametrize("qprob", [0.25, 0.5, 0.8])
def test_expectation_independent_inclusion(qprob):
    """The survival argument of Sec. 5 (each link survives with probability t/k,
    independently) is exact when chunks are kept independently with probability
    q = t/k: with factor 1/q per hop and a global 1/q the estimator is unbiased."""
    k, C, s = 4, 4, 0.5
    x = layer(4)
    full = A.seco_layer(x["q"], x["k"], x["v"], x["do"], C, s)
    acc = [np.zeros_like(full[2]), np.zeros_like(full[3]), np.zeros_like(full[4])]
    total = 0.0
    for size in range(k + 1):
        for sub in itertools.combinations(range(k), size):
            pr = qprob ** size * (1 - qprob) ** (k - size)
            total += pr
            out = A.spaco_layer(x["q"], x["k"], x["v"], x["do"], C, s, sub, 1 / qprob)
            for a, o in zip(acc, out[2:]):
                a += pr * o
    assert abs(total - 1) < 1e-14
    for a, f in zip(acc, full[2:]):
        assert rel(a / qprob, f) < 1e-12


def test_weight_vector_formulation():
    """sum_j w_j[chunk(c)] * (call j's contribution) reproduces the schedule."""
    k, C, s = 4, 4, 0.5
    x = layer(5)
    sel = [3, 2, 0]
    lam = np.float32(4 / 3)
    _, _, _, gK, gV = A.spaco_layer(x["q"], x["k"], x["v"], x["do"], C, s, sel, float(lam))
    dq, dk, dv = pieces(x, C, s)
    gK2, gV2 = np.zeros_like(gK), np.zeros_like(gV)
    for j in sel:
        w = S.chunk_weights(sel, j, lam)
        assert w.dtype == np.float32 and w.shape == (j + 1,)
        for i in range(j + 1):
            gK2[:, :, i * C:(i + 1) * C] += float(w[i]) * dk[i, j]
            gV2[:, :, i * C:(i + 1) * C] += float(w[i]) * dv[i, j]
    assert rel(gK2, gK) < 1e-14 and rel(gV2, gV) < 1e-14
    assert list(S.chunk_weights(sel, 3, lam)) == [lam, 0.0, lam, 1.0]
    assert list(S.chunk_weights(sel, 0, lam)) == [1.0]


def test_ragged_last_chunk():
    x = layer(6, N=14)
    full = A.seco_layer(x["q"], x["k"], x["v"], x["do"], 14, 0.5)
    chunked = A.seco_layer(x["q"], x["k"], x["v"], x["do"], 4, 0.5)
    for a, b in zip(full, chunked):
        assert rel(b, a) < 1e-12
    sp = A.spaco_layer(x["q"], x["k"], x["v"], x["do"], 4, 0.5, [0, 1, 2, 3], 1.0)
    for a, b in zip(sp, chunked):
        assert np.array_equal(a, b)


def test_per_call_draw_policy_is_exactly_unbiased_by_enumeration():
    """Every chunk back-propagated; call j keeps m = min(t, j) of its j earlier chunks with weight j / m.
    Averaged over all draws of every call the layer's gK/gV equal SeCO's, and dQ is SeCO's for every draw."""
    import itertools
    from oracle import attention as A
    rng = np.random.default_rng(5)
    B, Hq, Hkv, N, D, C, t = 1, 2, 1, 16, 4, 4, 2
    Q, dO = rng.standard_normal((2, B, Hq, N, D))
    K, V = rng.standard_normal((2, B, Hkv, N, D))
    s = 0.5
    _, _, dq_ref, gk_ref, gv_ref = A.seco_layer(Q, K, V, dO, C, s)
    k = N // C
    per_call = []
    for j in range(k):
        m = min(t, j)
        subsets = list(itertools.combinations(range(j), m)) if m else [()]
        per_call.append([(j, np.array([(j / m if i in sub else 0.0) for i in range(j)] + [1.0])) for sub in subsets])
    gk_mean, gv_mean, n = 0.0, 0.0, 0
    for combo in itertools.product(*per_call):
        dq, gk, gv = A.weighted_layer(Q, K, V, dO, C, s, sorted(combo, key=lambda cw: -cw[0]))
        np.testing.assert_allclose(dq, dq_ref, rtol=0, atol=1e-13)
        gk_mean, gv_mean, n = gk_mean + gk, gv_mean + gv, n + 1
    assert n == 1 * 1 * 1 * 3            # draws: j=0: 1, j=1: 1 (m=1 of 1), j=2: C(2,2)=1, j=3: C(3,2)=3
    np.testing.assert_allclose(gk_mean / n, gk_ref, rtol=0, atol=1e-12 * np.abs(gk_ref).max())
    np.testing.assert_allclose(gv_mean / n, gv_ref, rtol=0, atol=1e-12 * np.abs(gv_ref).max())


def test_percall_weights_follow_the_policy():
    from oracle.selection import percall_weights
    for j, t in [(0, 4), (1, 4), (3, 4), (9, 4), (31, 8)]:
        w = percall_weights(7, 3, j, t)
        m = min(t, j)
        assert w.shape == (j + 1,) and w[j] == 1.0
        assert int((w[:j] != 0).sum()) == m
        if m:
            assert np.all(w[:j][w[:j] != 0] == np.float32(j / m))
    # inclusion frequency of an earlier chunk over many steps ~ m / j
    j, t, n = 8, 2, 4000
    hits = sum(percall_weights(1, step, j, t)[3] != 0 for step in range(n))
    assert abs(hits - n * t / j) < 6 * np.sqrt(n * (t / j) * (1 - t / j))
