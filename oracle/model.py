"""SeCO / SpaCO over a small multi-layer transformer, CPU fp64 oracle (Alg. 1 and Alg. 2 end to end).

TEST INFRASTRUCTURE ONLY (see the package docstring).  fp64 PyTorch on the CPU; autograd
supplies the per-layer derivatives, this file supplies the schedules of the paper:

  * `monolithic_grads`  - ordinary training step on the whole sequence: the reference the
    paper compares SeCO with (Sec. 4: the exactness claim, gradients equal to whole-sequence training);
  * `seco_grads`        - Alg. 1: stage 1 runs the chunks in inference mode and keeps the KV
    caches m'_1..m'_k of every layer as checkpoints; stage 2 rebuilds each chunk's graph in
    reverse order against those checkpoints, hands the gradient collected on m'_i over to
    the recomputed m_i, and back-propagates J_i, which deposits gradient on the earlier
    checkpoints;
  * `spaco_grads`       - Alg. 2: only the selected chunks are rebuilt, and the gradient handed
    over from m'_i to m_i is multiplied by the compensation factor, so that a chain through p
    caches carries factor^p (Sec. 5, "Compensation Factor" and "Implementation").
  * `dq_weights` of the last two (not in the paper, which keeps dQ exact): in the attention of
    layer l of the call for chunk i, the part of dQ that flows through the scores of the columns
    of chunk c is multiplied by dq_weights(i, l)[c]; dK and dV are untouched.  With weights whose
    expectation is 1, drawn independently per call and layer, the parameter gradients stay
    unbiased; one draw shared by the layers of a call does not (a path inside chunk i meets the
    columns of chunk c once per layer and would carry the square of the weight).

The model is a plain pre-norm decoder: RMSNorm, grouped-query causal attention (no positional
encoding, or optionally the rotary embedding of LLaMA: `rope_base`; keys are cached rotated), RMSNorm, two-matrix MLP with SiLU, tied to nothing, cross-entropy loss summed over
tokens; J_j is the loss of chunk j's tokens.  The chunk-level error components of Eq. 1 add
up to the sequence loss.
"""
from __future__ import annotations

from dataclasses import dataclass

import torch
import torch.nn.functional as F


@dataclass(frozen=True)
class ModelConfig:
    n_layers: int = 3
    d_model: int = 32
    n_q_heads: int = 4
    n_kv_heads: int = 2
    head_dim: int = 8
    d_ff: int = 48
    vocab: int = 17
    rope_base: float = 0.0     # > 1: rotary position embedding of queries and keys with this base; 0: none

    @property
    def scale(self):
        return float(self.head_dim) ** -0.5


def init_params(cfg: ModelConfig, seed: int, dtype=torch.float64):
    """Seeded random parameters (dict name -> tensor, requires_grad)."""
    g = torch.Generator().manual_seed(seed)
    def rnd(*shape, std):
        return (torch.randn(*shape, generator=g, dtype=torch.float64) * std).to(dtype).requires_grad_()
    p = {"emb": rnd(cfg.vocab, cfg.d_model, std=1.0), "head": rnd(cfg.d_model, cfg.vocab, std=cfg.d_model ** -0.5),
         "norm_f": (1 + 0.1 * torch.randn(cfg.d_model, generator=g, dtype=torch.float64)).to(dtype).requires_grad_()}
    for l in range(cfg.n_layers):
        s = cfg.d_model ** -0.5
        p[f"l{l}.norm1"] = (1 + 0.1 * torch.randn(cfg.d_model, generator=g, dtype=torch.float64)).to(dtype).requires_grad_()
        p[f"l{l}.norm2"] = (1 + 0.1 * torch.randn(cfg.d_model, generator=g, dtype=torch.float64)).to(dtype).requires_grad_()
        p[f"l{l}.wq"] = rnd(cfg.d_model, cfg.n_q_heads * cfg.head_dim, std=2 * s)
        p[f"l{l}.wk"] = rnd(cfg.d_model, cfg.n_kv_heads * cfg.head_dim, std=2 * s)
        p[f"l{l}.wv"] = rnd(cfg.d_model, cfg.n_kv_heads * cfg.head_dim, std=s)
        p[f"l{l}.wo"] = rnd(cfg.n_q_heads * cfg.head_dim, cfg.d_model, std=(cfg.n_q_heads * cfg.head_dim) ** -0.5)
        p[f"l{l}.w1"] = rnd(cfg.d_model, cfg.d_ff, std=s)
        p[f"l{l}.w2"] = rnd(cfg.d_ff, cfg.d_model, std=cfg.d_ff ** -0.5)
    return p


def _rmsnorm(x, g):
    return x * torch.rsqrt((x * x).mean(dim=-1, keepdim=True) + 1e-6) * g


def _rope(x, pos0, base):
    """Rotary embedding of x [B,H,C,D], row r at position pos0 + r: pair (i, i + D/2) turns by pos * base^(-2i/D)."""
    C, D = x.shape[2], x.shape[3]
    inv = torch.pow(torch.tensor(float(base), dtype=torch.float64), -2.0 * torch.arange(D // 2, dtype=torch.float64) / D)
    th = (pos0 + torch.arange(C, dtype=torch.float64))[:, None] * inv[None, :]
    cos, sin = torch.cos(th).to(x.dtype), torch.sin(th).to(x.dtype)
    a, b = x[..., :D // 2], x[..., D // 2:]
    return torch.cat([a * cos - b * sin, b * cos + a * sin], dim=-1)


def _attend(q, k_all, v_all, q_start, scale, col_w=None):
    """q [B,Hq,C,D] against cache rows 0 .. q_start+C-1 ([B,Hkv,L,D]), causal with the diagonal included.

    col_w [L] (optional): weight of each cache column on the gradient that reaches q through that column's score.
    The value of the scores is unchanged: they are written as s*(q' k^T) + s*w*((q - q') k'^T) with q', k' cut
    off from the graph, so k receives its ordinary gradient and q receives w[c] * s * k[c] per column."""
    G = q.shape[1] // k_all.shape[1]
    C, L = q.shape[2], k_all.shape[2]
    k_rep = k_all.repeat_interleave(G, 1)
    if col_w is None:
        s = scale * torch.einsum("bhrd,bhcd->bhrc", q, k_rep)
    else:
        s = scale * (torch.einsum("bhrd,bhcd->bhrc", q.detach(), k_rep) +
                     torch.einsum("bhrd,bhcd->bhrc", q - q.detach(), k_rep.detach()) * col_w)
    vis = torch.arange(L)[None, :] <= (q_start + torch.arange(C))[:, None]
    p = torch.softmax(s.masked_fill(~vis, float("-inf")), dim=-1)
    return torch.einsum("bhrc,bhcd->bhrd", p, v_all.repeat_interleave(G, 1))


def _chunk_forward(cfg, params, tokens, targets, q_start, caches, col_w=None):
    """One chunk through all layers (Eq. 1): returns (J_j, [(k_l, v_l)] of this chunk).

    caches[l] = (K_prefix, V_prefix) of the earlier chunks at layer l, [B,Hkv,q_start,D] (may be empty);
    col_w[l] = per-column weights of layer l's dQ (see _attend), or None."""
    B, C = tokens.shape
    x = params["emb"][tokens]
    new_kv = []
    for l in range(cfg.n_layers):
        h = _rmsnorm(x, params[f"l{l}.norm1"])
        q = (h @ params[f"l{l}.wq"]).view(B, C, cfg.n_q_heads, cfg.head_dim).transpose(1, 2)
        k = (h @ params[f"l{l}.wk"]).view(B, C, cfg.n_kv_heads, cfg.head_dim).transpose(1, 2)
        v = (h @ params[f"l{l}.wv"]).view(B, C, cfg.n_kv_heads, cfg.head_dim).transpose(1, 2)
        if cfg.rope_base > 1.0:
            q, k = _rope(q, q_start, cfg.rope_base), _rope(k, q_start, cfg.rope_base)
        new_kv.append((k, v))
        k_all = torch.cat([caches[l][0], k], dim=2)
        v_all = torch.cat([caches[l][1], v], dim=2)
        o = _attend(q, k_all, v_all, q_start, cfg.scale, None if col_w is None else col_w[l])
        x = x + o.transpose(1, 2).reshape(B, C, -1) @ params[f"l{l}.wo"]
        h = _rmsnorm(x, params[f"l{l}.norm2"])
        x = x + F.silu(h @ params[f"l{l}.w1"]) @ params[f"l{l}.w2"]
    logits = _rmsnorm(x, params["norm_f"]) @ params["head"]
    loss = F.cross_entropy(logits.reshape(B * C, -1), targets.reshape(B * C), reduction="sum")
    return loss, new_kv


def _empty_caches(cfg, B, dtype):
    z = torch.zeros(B, cfg.n_kv_heads, 0, cfg.head_dim, dtype=dtype)
    return [(z, z) for _ in range(cfg.n_layers)]


def _zero_grads(params):
    for t in params.values():
        t.grad = None


def _collect(params):
    return {n: (t.grad.clone() if t.grad is not None else torch.zeros_like(t)) for n, t in params.items()}


def monolithic_grads(cfg, params, tokens, targets):
    """Loss and parameter gradients of the whole sequence processed at once."""
    _zero_grads(params)
    loss, _ = _chunk_forward(cfg, params, tokens, targets, 0, _empty_caches(cfg, tokens.shape[0], params["emb"].dtype))
    loss.backward()
    return loss.detach(), _collect(params)


def _stage1(cfg, params, tokens, targets, chunk_len):
    """Alg. 1 / Alg. 2, first loop: all chunks in inference mode; returns the checkpoints
    ckpt[j][l] = (K, V) of chunk j at layer l as detached leaves that can collect gradient."""
    B, N = tokens.shape
    ckpt, total = [], 0.0
    with torch.no_grad():
        for s0 in range(0, N, chunk_len):
            caches = [(torch.cat([c[l][0] for c in ckpt], 2), torch.cat([c[l][1] for c in ckpt], 2)) if ckpt
                      else _empty_caches(cfg, B, params["emb"].dtype)[l] for l in range(cfg.n_layers)]
            loss, new_kv = _chunk_forward(cfg, params, tokens[:, s0:s0 + chunk_len], targets[:, s0:s0 + chunk_len], s0, caches)
            total += float(loss)
            ckpt.append([(k.detach().clone(), v.detach().clone()) for k, v in new_kv])
    for c in ckpt:
        for k, v in c:
            k.requires_grad_()
            v.requires_grad_()
    return ckpt, total


def _stage2(cfg, params, tokens, targets, chunk_len, ckpt, order, factor, dq_weights=None):
    """Second loop: for every chunk in `order` (descending) rebuild its graph against the checkpoints,
    hand factor * m'_i.grad to the recomputed m_i and back-propagate J_i.
    dq_weights(i, l) -> one weight per chunk 0..i for the dQ of layer l in the call of chunk i (or None)."""
    B, N = tokens.shape
    starts = list(range(0, N, chunk_len))
    for i in order:
        s0 = starts[i]
        caches = [(torch.cat([c[l][0] for c in ckpt[:i]], 2), torch.cat([c[l][1] for c in ckpt[:i]], 2)) if i
                  else _empty_caches(cfg, B, params["emb"].dtype)[l] for l in range(cfg.n_layers)]
        col_w = None
        if dq_weights is not None:
            lens = [min(chunk_len, N - a) for a in starts[:i + 1]]
            col_w = []
            for l in range(cfg.n_layers):
                w = dq_weights(i, l)
                col_w.append(None if w is None else torch.cat(
                    [torch.full((n,), float(x), dtype=params["emb"].dtype) for n, x in zip(lens, w)]))
        loss, new_kv = _chunk_forward(cfg, params, tokens[:, s0:s0 + chunk_len], targets[:, s0:s0 + chunk_len], s0, caches,
                                      col_w)
        roots, grads = [loss], [torch.ones_like(loss)]
        for l, (k, v) in enumerate(new_kv):
            gk, gv = ckpt[i][l][0].grad, ckpt[i][l][1].grad
            if gk is not None:            # gradient that later chunks left on the checkpoint m'_i
                roots += [k, v]
                grads += [factor * gk, factor * gv]
        torch.autograd.backward(roots, grads)


def seco_grads(cfg, params, tokens, targets, chunk_len, dq_weights=None):
    """Alg. 1: exact gradients with one chunk's graph alive at a time (dq_weights: see the module docstring)."""
    _zero_grads(params)
    ckpt, total = _stage1(cfg, params, tokens, targets, chunk_len)
    _stage2(cfg, params, tokens, targets, chunk_len, ckpt, range(len(ckpt) - 1, -1, -1), 1.0, dq_weights)
    return total, _collect(params)


def spaco_grads(cfg, params, tokens, targets, chunk_len, selected, factor, dq_weights=None):
    """Alg. 2: back-propagate only the selected chunks, relayed KV gradient scaled by `factor`."""
    _zero_grads(params)
    ckpt, total = _stage1(cfg, params, tokens, targets, chunk_len)
    _stage2(cfg, params, tokens, targets, chunk_len, ckpt, sorted({int(i) for i in selected}, reverse=True), float(factor),
            dq_weights)
    return total, _collect(params)
