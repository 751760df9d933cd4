"""Chunked causal attention and the SeCO / SpaCO schedules, CPU fp64 oracle.

TEST INFRASTRUCTURE ONLY (see the package docstring).  Everything here is fp64
NumPy; nothing is blocked, fused or reordered beyond what the definitions
below state.

What is computed (0-based chunks; the paper numbers them from 1)
----------------------------------------------------------------
The paper's forward recurrence (Eq. 1) lets chunk j see its own tokens and the
KV caches of every earlier chunk.  At one attention layer this means: query row
r of chunk j, at global position p = q_start + r, attends over cache columns
c = 0 .. p (the diagonal is included, as in any decoder-only LM).  The paper
never writes the attention arithmetic out; it is the textbook one:

    S[r,c]  = scale * sum_d Q[r,d] K[c,d]                      c <= p
    LSE[r]  = ln sum_{c<=p} exp(S[r,c])          (natural log, scaled scores)
    P[r,c]  = exp(S[r,c] - LSE[r])
    O[r,:]  = sum_c P[r,c] V[c,:]

and, for an upstream gradient dO of O,

    delta[r] = sum_d dO[r,d] O[r,d]
    dP[r,c]  = sum_d dO[r,d] V[c,d]
    dS       = P * (dP - delta)                      (softmax Jacobian)
    dQ[r,:]  = scale * sum_c dS[r,c] K[c,:]
    dK[c,:]  = scale * sum_{heads of the group} sum_r dS[r,c] Q[r,:]
    dV[c,:]  =         sum_{heads of the group} sum_r P[r,c]  dO[r,:]

Grouped-query attention: query head h reads KV head h // G, G = Hq // Hkv.

SeCO (Alg. 1, second loop): chunks are back-propagated in reverse order and
each call adds its dK/dV contribution, for every visible column, into a
persistent gradient buffer over the whole cache (the paper's m'_i.grad).
Column-weighted dQ (an extension the paper does not have; Alg. 2 keeps dQ exact):
dQ is a sum over cache columns of terms that need only that column's K and V rows
and the row's LSE and delta, so a call may visit a subset of the column chunks and
weight each visited chunk by the reciprocal of its inclusion probability:

    dQ_w[r,:] = scale * sum_c w[c] dS[r,c] K[c,:]

which is exact for w = 1 and an unbiased estimate of dQ whenever E[w[c]] = 1.

SpaCO (Alg. 2): only the selected chunks are back-propagated; what a call
deposits on an *earlier* selected chunk is multiplied by the compensation
factor, what it deposits on its own rows is not, and unselected chunks receive
nothing (the appendix listing's `grad + base * scaler`).

Layouts: Q, O, dO, dQ are [B, Hq, rows, D]; K, V, gK, gV are [B, Hkv, N, D].
"""
from __future__ import annotations

import math

import numpy as np

__all__ = [
    "chunk_attn_fwd",
    "chunk_attn_bwd",
    "chunk_attn_dq_weighted",
    "seco_layer",
    "spaco_layer",
    "weighted_layer",
]


def _as64(x):
    return np.asarray(x, dtype=np.float64)


def _check(q, k_cache, v_cache, q_start):
    B, Hq, C, D = q.shape
    Bk, Hkv, N, Dk = k_cache.shape
    if v_cache.shape != k_cache.shape:
        raise ValueError("K and V cache shapes differ")
    if Bk != B or Dk != D:
        raise ValueError("batch / head_dim mismatch between Q and the cache")
    if Hq % Hkv != 0:
        raise ValueError("n_q_heads must be a multiple of n_kv_heads")
    if q_start < 0 or q_start + C > N:
        raise ValueError("chunk does not fit in the cache")
    return B, Hq, Hkv, C, D, Hq // Hkv


# --------------------------------------------------------------------------
# Tier "loops": the definitions above, one scalar at a time (tiny inputs only)
# --------------------------------------------------------------------------

def _fwd_loops(q, k_cache, v_cache, q_start, scale):
    B, Hq, Hkv, C, D, G = _check(q, k_cache, v_cache, q_start)
    o = np.zeros((B, Hq, C, D))
    lse = np.zeros((B, Hq, C))
    for b in range(B):
        for h in range(Hq):
            g = h // G
            for r in range(C):
                p = q_start + r
                s = [scale * sum(q[b, h, r, d] * k_cache[b, g, c, d] for d in range(D))
                     for c in range(p + 1)]
                top = max(s)
                z = sum(math.exp(x - top) for x in s)
                lse[b, h, r] = top + math.log(z)
                for c in range(p + 1):
                    w = math.exp(s[c] - lse[b, h, r])
                    for d in range(D):
                        o[b, h, r, d] += w * v_cache[b, g, c, d]
    return o, lse


def _bwd_loops(q, k_cache, v_cache, o, lse, d_o, q_start, scale):
    B, Hq, Hkv, C, D, G = _check(q, k_cache, v_cache, q_start)
    L = q_start + C
    dq = np.zeros((B, Hq, C, D))
    dk = np.zeros((B, Hkv, L, D))
    dv = np.zeros((B, Hkv, L, D))
    for b in range(B):
        for h in range(Hq):
            g = h // G
            for r in range(C):
                p = q_start + r
                delta = sum(d_o[b, h, r, d] * o[b, h, r, d] for d in range(D))
                for c in range(p + 1):
                    s = scale * sum(q[b, h, r, d] * k_cache[b, g, c, d] for d in range(D))
                    prob = math.exp(s - lse[b, h, r])
                    dp = sum(d_o[b, h, r, d] * v_cache[b, g, c, d] for d in range(D))
                    ds = prob * (dp - delta)
                    for d in range(D):
                        dq[b, h, r, d] += scale * ds * k_cache[b, g, c, d]
                        dk[b, g, c, d] += scale * ds * q[b, h, r, d]
                        dv[b, g, c, d] += prob * d_o[b, h, r, d]
    return dq, dk, dv


# --------------------------------------------------------------------------
# Tier "matmul": the same formulas with one NumPy matmul per step and head
# --------------------------------------------------------------------------

def _visible(q_start, C, L):
    """mask[r, c] is True where column c is visible to row r (c <= q_start + r)."""
    return np.arange(L)[None, :] <= (q_start + np.arange(C))[:, None]


def _fwd_matmul(q, k_cache, v_cache, q_start, scale):
    B, Hq, Hkv, C, D, G = _check(q, k_cache, v_cache, q_start)
    L = q_start + C
    vis = _visible(q_start, C, L)
    o = np.empty((B, Hq, C, D))
    lse = np.empty((B, Hq, C))
    for b in range(B):
        for h in range(Hq):
            kk = k_cache[b, h // G, :L]
            vv = v_cache[b, h // G, :L]
            s = scale * (q[b, h] @ kk.T)
            s[~vis] = -np.inf
            top = s.max(axis=1, keepdims=True)
            e = np.exp(s - top)
            z = e.sum(axis=1, keepdims=True)
            lse[b, h] = (top + np.log(z))[:, 0]
            o[b, h] = (e / z) @ vv
    return o, lse


def _bwd_matmul(q, k_cache, v_cache, o, lse, d_o, q_start, scale):
    B, Hq, Hkv, C, D, G = _check(q, k_cache, v_cache, q_start)
    L = q_start + C
    vis = _visible(q_start, C, L)
    dq = np.empty((B, Hq, C, D))
    dk = np.zeros((B, Hkv, L, D))
    dv = np.zeros((B, Hkv, L, D))
    for b in range(B):
        for h in range(Hq):
            g = h // G
            kk = k_cache[b, g, :L]
            vv = v_cache[b, g, :L]
            s = scale * (q[b, h] @ kk.T)
            prob = np.where(vis, np.exp(s - lse[b, h][:, None]), 0.0)
            delta = (d_o[b, h] * o[b, h]).sum(axis=1, keepdims=True)
            dp = d_o[b, h] @ vv.T
            ds = prob * (dp - delta)
            dq[b, h] = scale * (ds @ kk)
            dk[b, g] += scale * (ds.T @ q[b, h])
            dv[b, g] += prob.T @ d_o[b, h]
    return dq, dk, dv


_FWD = {"loops": _fwd_loops, "matmul": _fwd_matmul}
_BWD = {"loops": _bwd_loops, "matmul": _bwd_matmul}


def chunk_attn_fwd(q, k_cache, v_cache, q_start, scale, tier="matmul"):
    """Forward of one chunk against the cache (Eq. 1 at the attention layer).

    q        [B, Hq, C, D]   queries of the chunk, global rows q_start .. q_start+C-1
    k_cache  [B, Hkv, N, D]  rows 0 .. q_start+C-1 are read (prefix + own chunk)
    returns  O [B, Hq, C, D], LSE [B, Hq, C]
    """
    return _FWD[tier](_as64(q), _as64(k_cache), _as64(v_cache), int(q_start), float(scale))


def chunk_attn_bwd(q, k_cache, v_cache, o, lse, d_o, q_start, scale, tier="matmul"):
    """Backward of one chunk (Alg. 1, `backprop(J_i)` at the attention layer).

    returns dQ [B, Hq, C, D] and this call's *unweighted* contributions
    dK, dV [B, Hkv, q_start+C, D] to every visible cache row.
    """
    return _BWD[tier](_as64(q), _as64(k_cache), _as64(v_cache), _as64(o), _as64(lse),
                      _as64(d_o), int(q_start), float(scale))


def chunk_attn_dq_weighted(q, k_cache, v_cache, o, lse, d_o, q_start, scale, col_weight, tier="matmul"):
    """dQ of one chunk with a weight per cache column: scale * sum_c col_weight[c] * dS[r,c] * K[c,:]
    (dS as in chunk_attn_bwd: the exact P, from the exact LSE, and the exact delta).

    col_weight  [q_start + C] non-negative weights, one per visible cache column
    returns     dQ_w [B, Hq, C, D]
    """
    q, k_cache, v_cache, o, lse, d_o = (_as64(x) for x in (q, k_cache, v_cache, o, lse, d_o))
    q_start, scale = int(q_start), float(scale)
    B, Hq, Hkv, C, D, G = _check(q, k_cache, v_cache, q_start)
    L = q_start + C
    w = _as64(col_weight)
    if w.shape != (L,):
        raise ValueError("one weight per visible cache column is needed")
    dq = np.zeros((B, Hq, C, D))
    if tier == "loops":
        for b in range(B):
            for h in range(Hq):
                g = h // G
                for r in range(C):
                    delta = sum(d_o[b, h, r, d] * o[b, h, r, d] for d in range(D))
                    for c in range(q_start + r + 1):
                        s = scale * sum(q[b, h, r, d] * k_cache[b, g, c, d] for d in range(D))
                        dp = sum(d_o[b, h, r, d] * v_cache[b, g, c, d] for d in range(D))
                        ds = math.exp(s - lse[b, h, r]) * (dp - delta)
                        for d in range(D):
                            dq[b, h, r, d] += scale * w[c] * ds * k_cache[b, g, c, d]
        return dq
    vis = _visible(q_start, C, L)
    for b in range(B):
        for h in range(Hq):
            kk = k_cache[b, h // G, :L]
            vv = v_cache[b, h // G, :L]
            prob = np.where(vis, np.exp(scale * (q[b, h] @ kk.T) - lse[b, h][:, None]), 0.0)
            delta = (d_o[b, h] * o[b, h]).sum(axis=1, keepdims=True)
            ds = prob * (d_o[b, h] @ vv.T - delta)
            dq[b, h] = scale * ((ds * w[None, :]) @ kk)
    return dq


def _chunks(N, chunk_len):
    """(q_start, length) of every chunk; the last one may be short."""
    return [(s, min(chunk_len, N - s)) for s in range(0, N, chunk_len)]


def seco_layer(Q, K, V, dO, chunk_len, scale, tier="matmul"):
    """SeCO at one attention layer (Alg. 1).

    Stage 1 runs the chunks in order; stage 2 rebuilds each chunk in reverse
    order and back-propagates it, adding its dK/dV into the persistent buffers
    gK, gV that play the role of the checkpoints' .grad fields.

    returns O [B,Hq,N,D], LSE [B,Hq,N], dQ [B,Hq,N,D], gK, gV [B,Hkv,N,D]
    """
    Q, K, V, dO = _as64(Q), _as64(K), _as64(V), _as64(dO)
    B, Hq, N, D = Q.shape
    O = np.zeros_like(Q)
    LSE = np.zeros((B, Hq, N))
    for s0, c in _chunks(N, chunk_len):                       # Alg. 1, first loop
        O[:, :, s0:s0 + c], LSE[:, :, s0:s0 + c] = chunk_attn_fwd(
            Q[:, :, s0:s0 + c], K, V, s0, scale, tier)
    dQ = np.zeros_like(Q)
    gK = np.zeros_like(K)
    gV = np.zeros_like(V)
    for s0, c in reversed(_chunks(N, chunk_len)):             # Alg. 1, second loop
        o_j, lse_j = chunk_attn_fwd(Q[:, :, s0:s0 + c], K, V, s0, scale, tier)
        dq, dk, dv = chunk_attn_bwd(Q[:, :, s0:s0 + c], K, V, o_j, lse_j,
                                    dO[:, :, s0:s0 + c], s0, scale, tier)
        dQ[:, :, s0:s0 + c] = dq
        gK[:, :, :s0 + c] += dk
        gV[:, :, :s0 + c] += dv
    return O, LSE, dQ, gK, gV


def spaco_layer(Q, K, V, dO, chunk_len, scale, selected, factor, tier="matmul"):
    """SpaCO at one attention layer (Alg. 2).

    selected  chunk indices that are back-propagated (any order; processed in
              descending order so that what later chunks left on an earlier
              chunk's rows is complete before that chunk is reached)
    factor    compensation factor applied to what a call deposits on earlier
              selected chunks (Sec. 5 "Compensation Factor": k/t, possibly capped)

    dQ is exact over all visible columns for a selected chunk and zero for an
    unselected one; rows of gK/gV that belong to unselected chunks stay zero.
    """
    Q, K, V, dO = _as64(Q), _as64(K), _as64(V), _as64(dO)
    B, Hq, N, D = Q.shape
    chunks = _chunks(N, chunk_len)
    sel = sorted({int(i) for i in selected}, reverse=True)
    if sel and (sel[0] >= len(chunks) or sel[-1] < 0):
        raise ValueError("selected chunk index out of range")
    O = np.zeros_like(Q)
    LSE = np.zeros((B, Hq, N))
    for s0, c in chunks:
        O[:, :, s0:s0 + c], LSE[:, :, s0:s0 + c] = chunk_attn_fwd(
            Q[:, :, s0:s0 + c], K, V, s0, scale, tier)
    dQ = np.zeros_like(Q)
    gK = np.zeros_like(K)
    gV = np.zeros_like(V)
    for j in sel:
        s0, c = chunks[j]
        o_j, lse_j = chunk_attn_fwd(Q[:, :, s0:s0 + c], K, V, s0, scale, tier)
        dq, dk, dv = chunk_attn_bwd(Q[:, :, s0:s0 + c], K, V, o_j, lse_j,
                                    dO[:, :, s0:s0 + c], s0, scale, tier)
        dQ[:, :, s0:s0 + c] = dq
        gK[:, :, s0:s0 + c] += dk[:, :, s0:s0 + c]            # own rows: weight 1
        gV[:, :, s0:s0 + c] += dv[:, :, s0:s0 + c]
        for i in sel:
            if i < j:                                         # earlier selected chunk
                t0, ci = chunks[i]
                gK[:, :, t0:t0 + ci] += factor * dk[:, :, t0:t0 + ci]
                gV[:, :, t0:t0 + ci] += factor * dv[:, :, t0:t0 + ci]
    return O, LSE, dQ, gK, gV


def weighted_layer(Q, K, V, dO, chunk_len, scale, calls, tier="matmul"):
    """A layer's backward under an arbitrary host policy: `calls` is a list of (j, w) with j the chunk that is
    back-propagated and w the weight vector w[0..j] its call uses (w[i] multiplies what the call deposits on the
    rows of chunk i; see the library's spaco_chunk_attn_bwd).  Calls are processed in the given order.

    Alg. 2 with its single draw is one such policy; so are the two other readings of "a few sampled earlier
    chunks plus the current chunk": one call for the last chunk only, or every chunk back-propagated with its own
    draw of earlier chunks.  A call may carry a third element wq[0..j]: its dQ is then the column-weighted one
    (chunk_attn_dq_weighted with weight wq[i] on the columns of chunk i).  returns dQ, gK, gV.
    """
    Q, K, V, dO = _as64(Q), _as64(K), _as64(V), _as64(dO)
    chunks = _chunks(Q.shape[2], chunk_len)
    dQ, gK, gV = np.zeros_like(Q), np.zeros_like(K), np.zeros_like(V)
    for call in calls:
        j, w = call[0], call[1]
        s0, c = chunks[j]
        o_j, lse_j = chunk_attn_fwd(Q[:, :, s0:s0 + c], K, V, s0, scale, tier)
        dq, dk, dv = chunk_attn_bwd(Q[:, :, s0:s0 + c], K, V, o_j, lse_j, dO[:, :, s0:s0 + c], s0, scale, tier)
        if len(call) > 2 and call[2] is not None:      # per-chunk weights of the dQ columns
            col_w = np.concatenate([np.full(chunks[i][1], float(call[2][i])) for i in range(j + 1)])
            dq = chunk_attn_dq_weighted(Q[:, :, s0:s0 + c], K, V, o_j, lse_j, dO[:, :, s0:s0 + c], s0, scale,
                                        col_w, tier)
        dQ[:, :, s0:s0 + c] = dq
        for i in range(j + 1):
            if w[i] != 0:
                t0, ci = chunks[i]
                gK[:, :, t0:t0 + ci] += float(w[i]) * dk[:, :, t0:t0 + ci]
                gV[:, :, t0:t0 + ci] += float(w[i]) * dv[:, :, t0:t0 + ci]
    return dQ, gK, gV
