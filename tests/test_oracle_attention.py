"""Pins for oracle/attention.py: library attention + autograd, finite differences,
closed-form special cases, tier cross-check, and the paper's exactness claims
(Eq. 1: chunk outputs are those of the full model; Sec. 4: SeCO gradients equal
full-sequence gradients up to rounding)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import attention as A
from workloads import small_layer


def rel(x, ref):
    return np.abs(x - ref).max() / max(np.abs(ref).max(), 1e-300)


def layer(seed, B=1, Hq=4, Hkv=2, N=24, D=8):
    t = small_layer(seed, B, Hq, Hkv, N, D)
    return {k: v.astype(np.float64) for k, v in t.items()}


def sdpa_full(q, k, v, scale, q_start=0):
    """Library attention (torch SDPA, fp64, CPU) with the chunk's visibility mask."""
    G = q.shape[1] // k.shape[1]
    C, L = q.shape[2], q_start + q.shape[2]
    tq = torch.from_numpy(q).requires_grad_()
    tk = torch.from_numpy(k[:, :, :L].copy()).requires_grad_()
    tv = torch.from_numpy(v[:, :, :L].copy()).requires_grad_()
    mask = torch.arange(L)[None, :] <= (q_start + torch.arange(C))[:, None]
    o = F.scaled_dot_product_attention(tq, tk.repeat_interleave(G, 1), tv.repeat_interleave(G, 1),
                                       attn_mask=mask, scale=scale)
    return o, (tq, tk, tv)


@pytest.mark.parametrize("tier", ["loops", "matmul"])
@pytest.mark.parametrize("q_start,C", [(0, 24), (0, 7), (8, 8), (13, 11)])
def test_forward_matches_library_attention(tier, q_start, C):
    x = layer(1)
    s = 0.37
    q = x["q"][:, :, q_start:q_start + C]
    o, lse = A.chunk_attn_fwd(q, x["k"], x["v"], q_start, s, tier)
    o_ref, _ = sdpa_full(q, x["k"], x["v"], s, q_start)
    assert rel(o, o_ref.detach().numpy()) < 1e-13
    # LSE against the library log-sum-exp of the visible scaled scores
    G = 2
    L = q_start + C
    scores = s * torch.einsum("bhrd,bhcd->bhrc", torch.from_numpy(q),
                              torch.from_numpy(x["k"][:, :, :L]).repeat_interleave(G, 1))
    mask = torch.arange(L)[None, :] <= (q_start + torch.arange(C))[:, None]
    lse_ref = torch.logsumexp(scores.masked_fill(~mask, float("-inf")), dim=-1).numpy()
    assert rel(lse, lse_ref) < 1e-13


@pytest.mark.parametrize("tier", ["loops", "matmul"])
@pytest.mark.parametrize("q_start,C", [(0, 24), (8, 8), (13, 11)])
def test_backward_matches_library_autograd(tier, q_start, C):
    x = layer(2)
    s = 0.41
    q = x["q"][:, :, q_start:q_start + C]
    d_o = x["do"][:, :, q_start:q_start + C]
    o, lse = A.chunk_attn_fwd(q, x["k"], x["v"], q_start, s, tier)
    dq, dk, dv = A.chunk_attn_bwd(q, x["k"], x["v"], o, lse, d_o, q_start, s, tier)
    o_ref, (tq, tk, tv) = sdpa_full(q, x["k"], x["v"], s, q_start)
    (o_ref * torch.from_numpy(d_o)).sum().backward()
    assert rel(dq, tq.grad.numpy()) < 1e-12
    assert rel(dk, tk.grad.numpy()) < 1e-12
    assert rel(dv, tv.grad.numpy()) < 1e-12


def test_tiers_agree():
    x = layer(3, B=2, Hq=4, Hkv=2, N=20, D=4)
    out_l = A.seco_layer(x["q"], x["k"], x["v"], x["do"], 6, 0.5, tier="loops")
    out_m = A.seco_layer(x["q"], x["k"], x["v"], x["do"], 6, 0.5, tier="matmul")
    for a, b in zip(out_l, out_m):
        assert rel(a, b) < 1e-13


@pytest.mark.parametrize("chunk_len", [1, 5, 8, 24, 100])
def test_chunk_outputs_equal_full_sequence_attention(chunk_len):
    """Eq. 1: the concatenated chunk outputs are the outputs of full causal attention."""
    x = layer(4)
    s = 1 / np.sqrt(8)
    O, LSE, _, _, _ = A.seco_layer(x["q"], x["k"], x["v"], x["do"], chunk_len, s)
    o_ref, _ = sdpa_full(x["q"], x["k"], x["v"], s, 0)
    assert rel(O, o_ref.detach().numpy()) < 1e-13
    O1, LSE1 = A.chunk_attn_fwd(x["q"], x["k"], x["v"], 0, s)
    assert rel(LSE, LSE1) < 1e-13


@pytest.mark.parametrize("chunk_len", [1, 5, 8, 24])
def test_seco_gradients_equal_full_sequence_backward(chunk_len):
    """Sec. 4 / App. "Additional Results": SeCO gradients match whole-sequence
    backpropagation beyond 12 decimal places in fp64."""
    x = layer(5, B=2, Hq=6, Hkv=2, N=24, D=8)
    s = 1 / np.sqrt(8)
    _, _, dQ, gK, gV = A.seco_layer(x["q"], x["k"], x["v"], x["do"], chunk_len, s)
    o_ref, (tq, tk, tv) = sdpa_full(x["q"], x["k"], x["v"], s, 0)
    (o_ref * torch.from_numpy(x["do"])).sum().backward()
    assert rel(dQ, tq.grad.numpy()) < 1e-12
    assert rel(gK, tk.grad.numpy()) < 1e-12
    assert rel(gV, tv.grad.numpy()) < 1e-12


@pytest.mark.parametrize("tier", ["loops", "matmul"])
def test_finite_differences(tier):
    x = layer(6, B=1, Hq=2, Hkv=1, N=7, D=3)
    s, q_start, C = 0.6, 3, 4
    q = x["q"][:, :, q_start:q_start + C].copy()
    d_o = x["do"][:, :, q_start:q_start + C]
    k, v = x["k"].copy(), x["v"].copy()

    def loss(q_, k_, v_):
        o_, _ = A.chunk_attn_fwd(q_, k_, v_, q_start, s, tier)
        return float((o_ * d_o).sum())

    o, lse = A.chunk_attn_fwd(q, k, v, q_start, s, tier)
    dq, dk, dv = A.chunk_attn_bwd(q, k, v, o, lse, d_o, q_start, s, tier)
    eps = 1e-6
    for arr, grad, which in ((q, dq, 0), (k, dk, 1), (v, dv, 2)):
        num = np.zeros_like(grad)
        it = np.nditer(grad, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = arr[idx]
            arr[idx] = old + eps
            up = loss(q, k, v)
            arr[idx] = old - eps
            dn = loss(q, k, v)
            arr[idx] = old
            num[idx] = (up - dn) / (2 * eps)
        assert rel(grad, num) < 1e-7, which


def test_closed_forms():
    x = layer(7, B=1, Hq=2, Hkv=1, N=16, D=4)
    s, q_start, C = 0.5, 8, 8
    q = x["q"][:, :, q_start:q_start + C]
    # zero queries: uniform attention over the p+1 visible columns
    o, lse = A.chunk_attn_fwd(np.zeros_like(q), x["k"], x["v"], q_start, s)
    for r in range(C):
        p = q_start + r
        assert np.allclose(o[0, :, r], x["v"][0, 0, :p + 1].mean(axis=0), rtol=1e-13, atol=0)
        assert np.allclose(lse[0, :, r], np.log(p + 1), rtol=1e-13)
    # first token of the sequence sees only itself
    o0, lse0 = A.chunk_attn_fwd(x["q"][:, :, :1], x["k"], x["v"], 0, s)
    assert np.allclose(o0[0, :, 0], x["v"][0, 0, 0], rtol=1e-14)
    assert np.allclose(lse0[0, :, 0], s * x["q"][0, :, 0] @ x["k"][0, 0, 0], rtol=1e-13)
    # constant value rows: O is that row, and no gradient reaches Q or K
    vc = np.broadcast_to(np.array([1.0, -2.0, 0.5, 3.0]), x["v"].shape).copy()
    o, lse = A.chunk_attn_fwd(q, x["k"], vc, q_start, s)
    assert np.allclose(o, vc[:, :1, :C].repeat(2, 1), rtol=1e-13)
    dq, dk, dv = A.chunk_attn_bwd(q, x["k"], vc, o, lse, x["do"][:, :, q_start:q_start + C], q_start, s)
    assert np.abs(dq).max() < 1e-13 and np.abs(dk).max() < 1e-13
    # rows of P sum to one  =>  column sums of dV equal the summed upstream gradient
    o, lse = A.chunk_attn_fwd(q, x["k"], x["v"], q_start, s)
    d_o = x["do"][:, :, q_start:q_start + C]
    dq, dk, dv = A.chunk_attn_bwd(q, x["k"], x["v"], o, lse, d_o, q_start, s)
    assert np.allclose(dv.sum(axis=2), d_o.sum(axis=(1, 2))[:, None], rtol=1e-12)
    # O is a convex combination of visible value rows
    assert (o <= x["v"].max(axis=2, keepdims=True).repeat(2, 1) + 1e-12).all()
    assert (o >= x["v"].min(axis=2, keepdims=True).repeat(2, 1) - 1e-12).all()
    # softmax is shift invariant along a row: adding a constant vector u to every key,
    # with q.u the same for all columns, changes LSE by s*q.u and leaves O unchanged
    u = np.array([0.3, -0.1, 0.2, 0.05])
    o2, lse2 = A.chunk_attn_fwd(q, x["k"] + u, x["v"], q_start, s)
    assert np.allclose(o2, o, rtol=1e-12, atol=1e-14)
    assert np.allclose(lse2 - lse, s * (q @ u), rtol=1e-11, atol=1e-13)


def test_gqa_equals_repeated_heads():
    x = layer(8, B=1, Hq=6, Hkv=2, N=18, D=4)
    s = 0.5
    out_g = A.seco_layer(x["q"], x["k"], x["v"], x["do"], 6, s)
    kr, vr = x["k"].repeat(3, axis=1), x["v"].repeat(3, axis=1)
    out_m = A.seco_layer(x["q"], kr, vr, x["do"], 6, s)
    for i in range(3):
        assert rel(out_g[i], out_m[i]) < 1e-13
    for i in (3, 4):
        summed = out_m[i].reshape(1, 2, 3, 18, 4).sum(axis=2)
        assert rel(out_g[i], summed) < 1e-13


def test_argument_checks():
    x = layer(9)
    with pytest.raises(ValueError):
        A.chunk_attn_fwd(x["q"][:, :, :8], x["k"], x["v"], 20, 1.0)
    with pytest.raises(ValueError):
        A.chunk_attn_fwd(x["q"][:, :3, :8], x["k"], x["v"], 0, 1.0)
