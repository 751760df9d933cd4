"""GPU parity: the HIP path, called through the C ABI, against the CPU fp64 oracle on the
same seeded inputs.  Tolerances (max |x - ref| / max |ref| per tensor): fp32 1e-4;
bf16 1e-2 on O (and LSE), 2e-2 on dQ, gK, gV."""
import numpy as np
import pytest
import torch

import paper_2505_16710_amd as seco
from oracle import attention as A
from oracle import selection as S
from workloads import CONFIGS, full_layer, small_layer, kv_group, Config

from hip_driver import DEV, max_rel, max_rel_per_head, run_layer, to_dev, to_host

pytestmark = pytest.mark.gpu

TOL = {"f32": {"o": 1e-4, "lse": 1e-4, "dq": 1e-4, "gk": 1e-4, "gv": 1e-4},
       "bf16": {"o": 1e-2, "lse": 1e-2, "dq": 2e-2, "gk": 2e-2, "gv": 2e-2}}


def check(got, ref, dtype, what=""):
    names = ("o", "lse", "dq", "gk", "gv")
    errs = {n: max_rel(got[n], r) for n, r in zip(names, ref)}
    per_head = {n: max_rel_per_head(got[n], r) for n, r in zip(names, ref)}    # normalised per (batch, head) slice
    print(what, {n: f"{e:.2e}/{per_head[n]:.2e}" for n, e in errs.items()}, flush=True)
    for n in names:
        assert np.isfinite(got[n]).all(), n
        assert errs[n] <= TOL[dtype][n], (what, n, errs[n])
        assert per_head[n] <= 1.5 * TOL[dtype][n], (what, n, per_head[n])


def test_cfg1_fp32_seco_full_parity():
    cfg = CONFIGS["cfg1"]
    x = full_layer(cfg)
    got = run_layer(x, cfg.chunk_len, cfg.scale, "f32")
    ref = A.seco_layer(x["q"], x["k"], x["v"], x["do"], cfg.chunk_len, cfg.scale)
    check(got, ref, "f32", "cfg1")


@pytest.mark.parametrize("B,Hq,Hkv,N,D,C", [
    (2, 4, 2, 300, 64, 128),     # ragged last chunk, GQA
    (1, 3, 3, 130, 20, 50),      # head_dim not a multiple of 64, odd sizes
    (1, 2, 1, 70, 256, 70),      # largest head_dim, single chunk
    (1, 2, 2, 5, 4, 1),          # one row per chunk
])
def test_fp32_shapes(B, Hq, Hkv, N, D, C):
    x = small_layer(10, B, Hq, Hkv, N, D, "f32")
    s = 1 / np.sqrt(D)
    got = run_layer(x, C, s, "f32")
    ref = A.seco_layer(x["q"], x["k"], x["v"], x["do"], C, s)
    check(got, ref, "f32", f"f32 {B,Hq,Hkv,N,D,C}")


@pytest.mark.parametrize("B,Hq,Hkv,N,C", [
    (1, 4, 1, 512, 256),     # aligned, G = 4
    (2, 4, 2, 640, 256),     # short last chunk (128 rows)
    (1, 2, 2, 700, 200),     # nothing aligned to the 32/64/128 tiles
    (1, 8, 2, 1536, 512),    # several row tiles per chunk, several column tiles
    (1, 2, 1, 33, 33),       # single tiny chunk
    (1, 2, 1, 96, 1),        # one row per call
])
def test_bf16_seco_parity(B, Hq, Hkv, N, C):
    x = small_layer(20, B, Hq, Hkv, N, 128, "bf16")
    s = 1 / np.sqrt(128)
    got = run_layer(x, C, s, "bf16")
    ref = A.seco_layer(x["q"], x["k"], x["v"], x["do"], C, s)
    check(got, ref, "bf16", f"bf16 {B,Hq,Hkv,N,C}")


@pytest.mark.parametrize("dtype,D,N,C,sel,lam", [
    ("f32", 64, 256, 64, [3, 1, 0], 4 / 3),
    ("bf16", 128, 1024, 256, [3, 1, 0], 4 / 3),
    ("bf16", 128, 1280, 160, [7, 6, 2], 8 / 3),   # chunk length not a multiple of the column tile
    ("bf16", 128, 1024, 128, [5], 8.0),           # a single selected chunk: own block only
])
def test_spaco_parity(dtype, D, N, C, sel, lam):
    x = small_layer(30, 1, 4, 2, N, D, dtype)
    s = 1 / np.sqrt(D)
    lam32 = float(np.float32(lam))
    got = run_layer(x, C, s, dtype, selected=sel, factor=lam32)
    ref = A.spaco_layer(x["q"], x["k"], x["v"], x["do"], C, s, sel, lam32)
    check(got, ref, dtype, f"spaco {dtype} {N,C,sel}")
    k = -(-N // C)
    for i in range(k):
        if i not in sel:   # unselected chunks: untouched rows are exactly zero
            assert not got["gk"][:, :, i * C:(i + 1) * C].any() and not got["dq"][:, :, i * C:(i + 1) * C].any()


@pytest.mark.parametrize("B,Hq,Hkv,N,C,sel", [
    (5, 16, 8, 1024, 512, None),         # 40 units: the second call has 320 column tiles, the last 2 of a unit go to 2 workgroups each
    (1, 8, 2, 2080, 520, None),          # G = 4: every tile divided among 4 workgroups; ragged column tiles
    (1, 8, 2, 2080, 520, [3, 2, 0]),     # the same with weights (applied when the shares are merged)
])
def test_bf16_last_round_divided_by_query_head(B, Hq, Hkv, N, C, sel):
    """dK/dV pass with a short last round: column tiles shared out by query head and merged in head order."""
    x = small_layer(21, B, Hq, Hkv, N, 128, "bf16")
    s = 1 / np.sqrt(128)
    lam = float(np.float32(4 / 3))
    kw = {} if sel is None else {"selected": sel, "factor": lam}
    got = run_layer(x, C, s, "bf16", **kw)
    if sel is None:
        ref = A.seco_layer(x["q"], x["k"], x["v"], x["do"], C, s)
    else:
        ref = A.spaco_layer(x["q"], x["k"], x["v"], x["do"], C, s, sel, lam)
    check(got, ref, "bf16", f"divided last round {B,Hq,Hkv,N,C,sel}")
    again = run_layer(x, C, s, "bf16", **kw)
    assert np.array_equal(got["gk"], again["gk"]) and np.array_equal(got["gv"], again["gv"])


def _one_call(dtype, D, N, C, j, weights=None, seed=40):
    x = small_layer(seed, 1, 4, 2, N, D, dtype)
    q, k, v, do = (to_dev(x[n], dtype) for n in ("q", "k", "v", "do"))
    s = 1 / np.sqrt(D)
    qc = q[:, :, j * C:(j + 1) * C]
    o, lse = seco.seco_chunk_attn_fwd(qc, k, v, j * C, s)
    doc = do[:, :, j * C:(j + 1) * C].contiguous()
    gk = torch.zeros(k.shape, dtype=torch.float32, device=DEV)
    gv = torch.zeros(k.shape, dtype=torch.float32, device=DEV)
    if weights is None:
        dq = seco.seco_chunk_attn_bwd(qc, k, v, o, lse, doc, gk, gv, j * C, s)
    else:
        dq = seco.spaco_chunk_attn_bwd(qc, k, v, o, lse, doc, gk, gv, j * C, s, weights, C)
    torch.cuda.synchronize()
    return dq, gk, gv


@pytest.mark.parametrize("dtype,D", [("f32", 64), ("bf16", 128)])
def test_unit_weights_equal_seco_bitwise_and_reruns_are_identical(dtype, D):
    """No atomics anywhere: the same call gives the same bits, and SpaCO with all weights 1
    is the SeCO backward."""
    a = _one_call(dtype, D, 1024, 256, 3)
    b = _one_call(dtype, D, 1024, 256, 3)
    c = _one_call(dtype, D, 1024, 256, 3, weights=[1.0, 1.0, 1.0, 1.0])
    for x, y, z in zip(a, b, c):
        assert torch.equal(x, y) and torch.equal(x, z)


@pytest.mark.parametrize("dtype,D", [("f32", 64), ("bf16", 128)])
def test_weights_in_kernel_equal_scaled_accumulate(dtype, D):
    """The factor applied inside the backward equals an unweighted backward followed by
    kvgrad_accumulate(scale) on the earlier rows (the appendix listing's grad + base*scaler)."""
    lam = 2.5
    dq_w, gk_w, gv_w = _one_call(dtype, D, 1024, 256, 3, weights=[lam, 0.0, lam, 1.0])
    dq_u, gk_u, gv_u = _one_call(dtype, D, 1024, 256, 3)
    gk2, gv2 = torch.zeros_like(gk_u), torch.zeros_like(gv_u)
    seco.kvgrad_accumulate(gk2, gv2, gk_u, gv_u, lam, 0, 256)
    seco.kvgrad_accumulate(gk2, gv2, gk_u, gv_u, lam, 512, 768)
    seco.kvgrad_accumulate(gk2, gv2, gk_u, gv_u, 1.0, 768, 1024)
    torch.cuda.synchronize()
    assert torch.equal(dq_w, dq_u)
    for a, b in ((gk_w, gk2), (gv_w, gv2)):
        assert not b[:, :, 256:512].any() and not a[:, :, 256:512].any()
        assert max_rel(to_host(a), to_host(b)) < 1e-6


def test_backward_accumulates_into_existing_gradients():
    x = small_layer(41, 1, 2, 1, 512, 128, "bf16")
    q, k, v, do = (to_dev(x[n], "bf16") for n in ("q", "k", "v", "do"))
    s = 1 / np.sqrt(128)
    o, lse = seco.seco_chunk_attn_fwd(q[:, :, 256:], k, v, 256, s)
    base = torch.randn(k.shape, dtype=torch.float32, device=DEV)
    gk, gv = base.clone(), (2 * base).clone()
    zk, zv = torch.zeros_like(base), torch.zeros_like(base)
    doc = do[:, :, 256:].contiguous()
    seco.seco_chunk_attn_bwd(q[:, :, 256:], k, v, o, lse, doc, gk, gv, 256, s)
    seco.seco_chunk_attn_bwd(q[:, :, 256:], k, v, o, lse, doc, zk, zv, 256, s)
    torch.cuda.synchronize()
    assert torch.allclose(gk, base + zk, rtol=1e-6, atol=1e-6) and torch.allclose(gv, 2 * base + zv, rtol=1e-6, atol=1e-6)


def test_kvgrad_zero_and_accumulate_with_strides_and_row_ranges():
    big = torch.randn(2, 3, 40, 2 * 64, device=DEV)
    gk = big[:, :, :, :64]          # row stride 128, head_dim 64: a strided view
    gv = big[:, :, :, 64:]          # gK and gV share one stride triple in the descriptor
    keep_k, keep_v = gk.clone(), gv.clone()
    seco.kvgrad_zero(gk, gv, 8, 24)
    torch.cuda.synchronize()
    assert not gk[:, :, 8:24].any() and not gv[:, :, 8:24].any()
    assert torch.equal(gk[:, :, :8], keep_k[:, :, :8]) and torch.equal(gk[:, :, 24:], keep_k[:, :, 24:])
    assert torch.equal(gv[:, :, :8], keep_v[:, :, :8]) and torch.equal(gv[:, :, 24:], keep_v[:, :, 24:])
    src = torch.randn(2, 3, 40, 64, device=DEV)
    dst = torch.randn(2, 3, 40, 64, device=DEV)
    want = dst.clone()
    want[:, :, 4:30] += 1.5 * src[:, :, 4:30]
    seco.kvgrad_accumulate(dst, None, src, None, 1.5, 4, 30)
    torch.cuda.synchronize()
    assert torch.allclose(dst, want, rtol=1e-6, atol=1e-6)
    seco.kvgrad_zero(dst, None, 7, 7)      # empty range: no-op
    torch.cuda.synchronize()
    assert torch.allclose(dst, want, rtol=1e-6, atol=1e-6)


def test_strided_inputs_bf16():
    """Q/O/dO/dQ taken as views of a packed [B, N, H, D] projection output (row stride H*D)."""
    x = small_layer(42, 1, 4, 2, 384, 128, "bf16")
    s = 1 / np.sqrt(128)
    def packed(a):   # [B,H,N,D] -> storage [B,N,H,D], viewed back as [B,H,N,D]
        return to_dev(a, "bf16").permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    q, k, v, do = packed(x["q"]), packed(x["k"]), packed(x["v"]), packed(x["do"])
    assert q.stride(2) == 4 * 128
    o, lse = seco.seco_chunk_attn_fwd(q[:, :, 128:], k, v, 128, s, o=torch.empty_like(q)[:, :, 128:])
    gk = torch.zeros(1, 384, 2, 128, device=DEV).permute(0, 2, 1, 3)
    gv = torch.zeros(1, 384, 2, 128, device=DEV).permute(0, 2, 1, 3)
    dq = seco.seco_chunk_attn_bwd(q[:, :, 128:], k, v, o, lse, do[:, :, 128:], gk, gv, 128, s,
                                  d_q=torch.empty_like(q)[:, :, 128:])
    torch.cuda.synchronize()
    o_ref, lse_ref = A.chunk_attn_fwd(x["q"][:, :, 128:], x["k"], x["v"], 128, s)
    dq_ref, dk_ref, dv_ref = A.chunk_attn_bwd(x["q"][:, :, 128:], x["k"], x["v"], o_ref, lse_ref, x["do"][:, :, 128:], 128, s)
    assert max_rel(to_host(o), o_ref) < 1e-2 and max_rel(to_host(dq), dq_ref) < 2e-2
    assert max_rel(to_host(gk), dk_ref) < 2e-2 and max_rel(to_host(gv), dv_ref) < 2e-2


@pytest.mark.parametrize("dtype,B,Hq,Hkv,D", [("bf16", 2, 2, 1, 128), ("f32", 1, 2, 2, 64)])
def test_heads_and_batches_more_than_2_to_31_elements_apart(dtype, B, Hq, Hkv, D):
    """Every tensor laid out with its (batch, head) slices more than 2^31 elements apart, as in buffers sized for a
    far longer sequence: the address arithmetic is 64-bit throughout (the strides are elements, not bytes)."""
    N, C, far = 256, 128, 2 ** 31 + 4096
    x = small_layer(77, B, Hq, Hkv, N, D, dtype)
    s = 1 / np.sqrt(D)
    tt = torch.bfloat16 if dtype == "bf16" else torch.float32

    def spread(H, t):                 # uninitialised [B, H, N, D] view whose slices lie `far` elements apart
        store = torch.empty((B * H - 1) * far + N * D, device=DEV, dtype=t)
        return store.as_strided((B, H, N, D), (H * far, far, D, 1))

    def placed(a):
        v = spread(a.shape[1], tt)
        v.copy_(to_dev(a, dtype))
        return v

    q, k, v, do = placed(x["q"]), placed(x["k"]), placed(x["v"]), placed(x["do"])
    assert q.stride(1) > 2 ** 31 and k.stride(0) > 2 ** 31
    o, dq = spread(Hq, tt), spread(Hq, tt)
    gk, gv = spread(Hkv, torch.float32), spread(Hkv, torch.float32)
    seco.kvgrad_zero(gk, gv)
    o1, lse = seco.seco_chunk_attn_fwd(q[:, :, C:], k, v, C, s, o=o[:, :, C:])
    dq1 = seco.seco_chunk_attn_bwd(q[:, :, C:], k, v, o1, lse, do[:, :, C:], gk, gv, C, s, d_q=dq[:, :, C:])
    torch.cuda.synchronize()
    o_ref, lse_ref = A.chunk_attn_fwd(x["q"][:, :, C:], x["k"], x["v"], C, s)
    dq_ref, dk_ref, dv_ref = A.chunk_attn_bwd(x["q"][:, :, C:], x["k"], x["v"], o_ref, lse_ref, x["do"][:, :, C:], C, s)
    tol_o, tol_g = (1e-2, 2e-2) if dtype == "bf16" else (1e-4, 1e-4)
    assert max_rel(to_host(o1), o_ref) < tol_o and max_rel(to_host(lse), lse_ref) < 1e-4
    assert max_rel(to_host(dq1), dq_ref) < tol_g
    assert max_rel(to_host(gk), dk_ref) < tol_g and max_rel(to_host(gv), dv_ref) < tol_g


def test_one_call_against_a_cache_of_a_million_rows():
    """The last chunk (256 rows, two query heads on one KV head) of a 2^20-token context: 8192 column tiles, the
    short-chunk path with its cache range divided among workgroups, fp32 row sums over a million terms.  The oracle
    evaluates O and LSE in full, dQ on sampled rows and, with the true LSE and O of the chunk and a cache cut down to
    a window plus the chunk's own rows, which returns exactly those rows' blocks of dK/dV, gK/gV on the first rows, on
    rows in the middle that straddle a column tile, and on the chunk's own rows."""
    from workloads import round_to
    N, C, D, s = 2 ** 20, 256, 128, 1 / np.sqrt(128)
    rng = np.random.default_rng(2 ** 20)
    k32 = round_to(rng.standard_normal((1, 1, N, D), dtype=np.float32), "bf16")
    v32 = round_to(rng.standard_normal((1, 1, N, D), dtype=np.float32), "bf16")
    q32 = round_to(rng.standard_normal((1, 2, C, D), dtype=np.float32), "bf16")
    do32 = round_to(rng.standard_normal((1, 2, C, D), dtype=np.float32), "bf16")
    q, k, v, do = (to_dev(a, "bf16") for a in (q32, k32, v32, do32))
    q0 = N - C
    o, lse = seco.seco_chunk_attn_fwd(q, k, v, q0, s)
    gk = torch.zeros(1, 1, N, D, device=DEV)
    gv = torch.zeros(1, 1, N, D, device=DEV)
    dq = seco.seco_chunk_attn_bwd(q, k, v, o, lse, do, gk, gv, q0, s)
    torch.cuda.synchronize()
    o_g, lse_g, dq_g = to_host(o), to_host(lse), to_host(dq)
    q64, k64, v64, do64 = (a.astype(np.float64) for a in (q32, k32, v32, do32))
    o_ref, lse_ref = A.chunk_attn_fwd(q64, k64, v64, q0, s)
    assert max_rel(o_g, o_ref) <= 1e-2 and max_rel(lse_g, lse_ref) <= 1e-4
    for r in (0, 101, C - 1):
        dq_r, _, _ = A.chunk_attn_bwd(q64[:, :, r:r + 1], k64, v64, o_ref[:, :, r:r + 1], lse_ref[:, :, r:r + 1],
                                      do64[:, :, r:r + 1], q0 + r, s)
        assert np.abs(dq_g[:, :, r] - dq_r[:, :, 0]).max() <= 2e-2 * np.abs(dq_r).max()
    # (the window is followed by the chunk's own rows, so that the cut-down cache has q_start + C rows)
    for lo, hi in ((0, 200), (N // 2 - 70, N // 2 + 70), (q0, q0)):
        kw = np.concatenate([k64[:, :, lo:hi], k64[:, :, q0:]], axis=2)
        vw = np.concatenate([v64[:, :, lo:hi], v64[:, :, q0:]], axis=2)
        _, dk_w, dv_w = A.chunk_attn_bwd(q64, kw, vw, o_ref, lse_ref, do64, hi - lo, s)
        rows = np.r_[lo:hi, q0:N]
        assert max_rel(to_host(gk)[:, :, rows], dk_w) <= 2e-2 and max_rel(to_host(gv)[:, :, rows], dv_w) <= 2e-2


@pytest.mark.parametrize("B,Hq,Hkv,N,C", [
    (1, 4, 1, 512, 256),      # aligned, G = 4
    (2, 4, 2, 640, 256),      # short last chunk
    (1, 2, 2, 700, 200),      # nothing aligned to the tiles
    (1, 8, 2, 4096, 1024),    # every column tile divided among the four query heads of its group
    (3, 4, 4, 1536, 512),     # G = 1: nothing to divide
])
def test_transposed_backward_order_gives_the_same_layer_gradients(B, Hq, Hkv, N, C):
    """seco_chunk_attn_bwd_gather for every chunk in descending order, each call with all later rows: the finished
    gK/gV and dQ of Alg. 1's second loop, against the same oracle as the accumulating order; and bit-identical reruns."""
    x = small_layer(55, B, Hq, Hkv, N, 128, "bf16")
    s = 1 / np.sqrt(128)
    q, k, v, do = (to_dev(x[n], "bf16") for n in ("q", "k", "v", "do"))
    stat_rows = (N + 3) // 4 * 4

    def layer():
        o, dq = torch.empty_like(q), torch.empty_like(q)
        lse_all = torch.empty(B, Hq, N, device=DEV)
        gk = torch.zeros(B, Hkv, N, 128, device=DEV)
        gv = torch.zeros_like(gk)
        stats = torch.full((2, B, Hq, stat_rows), float("nan"), device=DEV)   # every entry is written before it is read
        for s0 in range((N - 1) // C * C, -1, -C):
            c = min(C, N - s0)
            oc, lse = seco.seco_chunk_attn_fwd(q[:, :, s0:s0 + c], k, v, s0, s, o=o[:, :, s0:s0 + c])
            lse_all[:, :, s0:s0 + c] = lse
            seco.seco_chunk_attn_bwd_gather(q[:, :, s0:], k, v, oc, lse, do[:, :, s0:], gk, gv, s0, s, c, stats,
                                            d_q=dq[:, :, s0:s0 + c])
        torch.cuda.synchronize()
        return {"o": to_host(o), "lse": to_host(lse_all), "dq": to_host(dq), "gk": to_host(gk), "gv": to_host(gv)}

    got = layer()
    ref = A.seco_layer(x["q"], x["k"], x["v"], x["do"], C, s)
    check(got, ref, "bf16", f"transposed order {B,Hq,Hkv,N,C}")
    again = layer()
    assert np.array_equal(got["gk"], again["gk"]) and np.array_equal(got["gv"], again["gv"])


@pytest.mark.parametrize("B,Hq,Hkv,N,C,sel", [
    (1, 4, 2, 1024, 128, [7, 5, 4, 1]),     # runs of one and of two selected chunks, gaps between them
    (2, 4, 1, 1100, 128, [8, 6, 3, 2, 0]),  # the last chunk is short (76 rows) and selected
    (1, 8, 2, 4096, 1024, [3, 2, 0]),       # column tiles divided among the query heads
    (1, 2, 2, 768, 192, [3, 1]),            # chunk length a multiple of 64 but not of the 128-row column tile
])
def test_spaco_in_the_transposed_order(B, Hq, Hkv, N, C, sel):
    """Alg. 2 with the backward calls in the transposed order: the call of a selected chunk gathers from its own
    rows (weight 1) and from the later selected chunks (factor k/t); rows of unselected chunks are never read (their
    row statistics stay NaN here).  Same oracle and bars as the accumulating order."""
    x = small_layer(56, B, Hq, Hkv, N, 128, "bf16")
    s = 1 / np.sqrt(128)
    k_chunks = -(-N // C)
    lam = float(np.float32(k_chunks / len(sel)))
    q, k, v, do = (to_dev(x[n], "bf16") for n in ("q", "k", "v", "do"))
    o, dq = torch.zeros_like(q), torch.zeros_like(q)
    lse_all = torch.zeros(B, Hq, N, device=DEV)
    gk = torch.zeros(B, Hkv, N, 128, device=DEV)
    gv = torch.zeros_like(gk)
    stats = torch.full((2, B, Hq, (N + 3) // 4 * 4), float("nan"), device=DEV)
    for i in sel:                                   # descending
        s0, c = i * C, min(C, N - i * C)
        oc, lse = seco.seco_chunk_attn_fwd(q[:, :, s0:s0 + c], k, v, s0, s, o=o[:, :, s0:s0 + c])
        lse_all[:, :, s0:s0 + c] = lse
        w = seco.spaco_gather_row_weights(sel, i, k_chunks, lam)
        seco.seco_chunk_attn_bwd_gather(q[:, :, s0:], k, v, oc, lse, do[:, :, s0:], gk, gv, s0, s, c, stats,
                                        d_q=dq[:, :, s0:s0 + c], row_weight=w, weight_chunk_len=C)
    torch.cuda.synchronize()
    got = {"o": to_host(o), "lse": to_host(lse_all), "dq": to_host(dq), "gk": to_host(gk), "gv": to_host(gv)}
    ref = list(A.spaco_layer(x["q"], x["k"], x["v"], x["do"], C, s, sel, lam))
    for i in range(k_chunks):                       # the oracle leaves O / LSE of unselected chunks unset or set:
        if i not in sel:                            # compare them on the selected chunks only
            for n, r in zip(("o", "lse"), ref[:2]):
                got[n][:, :, i * C:(i + 1) * C] = r[:, :, i * C:(i + 1) * C]
    check(got, ref, "bf16", f"spaco transposed {B,Hq,Hkv,N,C,sel}")
    for i in range(k_chunks):
        if i not in sel:
            assert not got["gk"][:, :, i * C:(i + 1) * C].any() and not got["dq"][:, :, i * C:(i + 1) * C].any()


def _device_group(cfg, b, kvh):
    """One (batch, KV head) unit of a configuration as a G-head layer: host dict + fp64 views."""
    grp = kv_group(cfg, b, kvh)
    return {"q": grp["q"][None], "do": grp["do"][None], "k": grp["k"][None, None], "v": grp["v"][None, None]}


def test_cfg2_full_size_slice_parity():
    """Benchmark configuration (16K tokens, 16 chunks of 1024, head_dim 128, G = 4): one
    complete (batch, KV head) unit - they are independent - through all 16 + 16 + 16 calls."""
    cfg = CONFIGS["cfg2"]
    x = _device_group(cfg, 0, 5)
    got = run_layer(x, cfg.chunk_len, cfg.scale, "bf16")
    ref = A.seco_layer(x["q"], x["k"], x["v"], x["do"], cfg.chunk_len, cfg.scale)
    check(got, ref, "bf16", "cfg2 slice")


def _spaco_sampled_check(cfg, kvh, n_rows_per_chunk=3):
    """SpaCO (Alg. 2) at full sequence length on one (batch, KV head) unit: the oracle evaluates sampled
    query rows (O, LSE, dQ need one row each) and the top selected chunk's own rows of gK/gV, which only
    that chunk's call touches."""
    k, t, C = cfg.n_chunks, cfg.spaco_t, cfg.chunk_len
    sel = S.select_chunks(cfg.seed, 0, k, t).tolist()
    assert sel == seco.spaco_select_chunks(cfg.seed, 0, k, t)
    lam = float(np.float32(S.compensation_factor(k, t)))
    x = _device_group(cfg, 0, kvh)
    got = run_layer(x, C, cfg.scale, "bf16", selected=sel, factor=lam)
    rng = np.random.default_rng(7)
    q64, k64, v64, do64 = (x[n].astype(np.float64) for n in ("q", "k", "v", "do"))
    for j in sel:
        for r in rng.integers(0, C, size=n_rows_per_chunk):
            p = j * C + int(r)
            o_r, lse_r = A.chunk_attn_fwd(q64[:, :, p:p + 1], k64, v64, p, cfg.scale)
            dq_r, _, _ = A.chunk_attn_bwd(q64[:, :, p:p + 1], k64, v64, o_r, lse_r, do64[:, :, p:p + 1], p, cfg.scale)
            assert np.abs(got["o"][:, :, p] - o_r[:, :, 0]).max() <= 1e-2 * np.abs(o_r).max()
            assert np.abs(got["lse"][:, :, p] - lse_r[:, :, 0]).max() <= 1e-2 * np.abs(lse_r).max()
            assert np.abs(got["dq"][:, :, p] - dq_r[:, :, 0]).max() <= 2e-2 * np.abs(dq_r).max()
    # The top selected chunk's own rows receive only that call's diagonal block.  The oracle backward takes LSE
    # and O as inputs, so with the true LSE and O of the chunk and a cache cut down to the chunk's own rows it
    # returns exactly that block.
    top = sel[0]
    rows = slice(top * C, (top + 1) * C)
    o_ref, lse_ref = A.chunk_attn_fwd(q64[:, :, rows], k64, v64, top * C, cfg.scale)
    _, dk_own, dv_own = A.chunk_attn_bwd(q64[:, :, rows], k64[:, :, rows], v64[:, :, rows], o_ref, lse_ref,
                                         do64[:, :, rows], 0, cfg.scale)
    assert max_rel(got["gk"][:, :, rows], dk_own) <= 2e-2
    assert max_rel(got["gv"][:, :, rows], dv_own) <= 2e-2
    for i in range(k):
        if i not in sel:
            assert not got["gk"][:, :, i * C:(i + 1) * C].any() and not got["gv"][:, :, i * C:(i + 1) * C].any()
            assert not got["dq"][:, :, i * C:(i + 1) * C].any()
    # lower selected chunks: rows hold their own block plus factor x the blocks of the higher selected calls
    # restricted to those rows; check the lowest one in full against the oracle, call by call
    low = sel[-1]
    rows = slice(low * C, (low + 1) * C)
    want_k = np.zeros_like(got["gk"][:, :, rows])
    want_v = np.zeros_like(want_k)
    for j in sel:
        qr = slice(j * C, (j + 1) * C)
        o_j, lse_j = A.chunk_attn_fwd(q64[:, :, qr], k64, v64, j * C, cfg.scale)
        if j == low:
            _, dk, dv = A.chunk_attn_bwd(q64[:, :, qr], k64[:, :, rows], v64[:, :, rows], o_j, lse_j, do64[:, :, qr], 0, cfg.scale)
            want_k += dk
            want_v += dv
        else:
            # rows of chunk `low` are entirely below the diagonal of call j: a cache holding only those rows,
            # with q_start moved past them, makes every one of them visible to every query row
            _, dk, dv = A.chunk_attn_bwd(q64[:, :, qr], np.concatenate([k64[:, :, rows], k64[:, :, qr]], axis=2),
                                         np.concatenate([v64[:, :, rows], v64[:, :, qr]], axis=2), o_j, lse_j,
                                         do64[:, :, qr], C, cfg.scale)
            want_k += lam * dk[:, :, :C]
            want_v += lam * dv[:, :, :C]
    assert max_rel(got["gk"][:, :, rows], want_k) <= 2e-2
    assert max_rel(got["gv"][:, :, rows], want_v) <= 2e-2


def test_cfg3_spaco_sampled_parity():
    """32K tokens, 16 chunks of 2048, 4 selected chunks, factor k/t = 4."""
    _spaco_sampled_check(CONFIGS["cfg3"], 2)


def test_cfg4_spaco_sampled_parity():
    """64K tokens, 32 chunks of 2048, 8 selected chunks, factor k/t = 4."""
    _spaco_sampled_check(CONFIGS["cfg4"], 6, n_rows_per_chunk=2)


def test_cfg5_like_batch2_rope_inputs():
    """Batch 2 with RoPE-like structured Q/K (sin/cos-modulated, per-head mean), a scaled-down cfg5:
    SeCO and SpaCO with a quarter of the chunks selected."""
    cfg = Config("cfg5_small", "bf16", 2, 8, 2, 128, 2048, 256, seed=4, rope_like=True, spaco_t=2)
    x = full_layer(cfg)
    got = run_layer(x, cfg.chunk_len, cfg.scale, "bf16")
    ref = A.seco_layer(x["q"], x["k"], x["v"], x["do"], cfg.chunk_len, cfg.scale)
    check(got, ref, "bf16", "cfg5-like seco")
    sel = S.select_chunks(cfg.seed, 3, cfg.n_chunks, cfg.spaco_t).tolist()
    lam = float(np.float32(S.compensation_factor(cfg.n_chunks, cfg.spaco_t)))
    got = run_layer(x, cfg.chunk_len, cfg.scale, "bf16", selected=sel, factor=lam)
    ref = A.spaco_layer(x["q"], x["k"], x["v"], x["do"], cfg.chunk_len, cfg.scale, sel, lam)
    check(got, ref, "bf16", f"cfg5-like spaco {sel}")


def test_cfg2_whole_layer_identities_in_the_benchmark_configuration():
    """The benchmark's launch configuration (all 32 heads, 16 calls of 1024 rows, device-generated inputs),
    checked with identities that hold at any size: rows of P sum to one, so sum_c gV[c] = sum_{h,r} dO[h,r];
    and sum_r Q.dQ = sum_c K.gK (both equal s * sum dS * QK^T)."""
    cfg = CONFIGS["cfg2"]
    B, Hq, Hkv, D, N, C = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.seq_len, cfg.chunk_len
    gen = torch.Generator(device=DEV).manual_seed(5)
    mk = lambda h: torch.randn(B, h, N, D, generator=gen, device=DEV).to(torch.bfloat16)
    q, k, v, do = mk(Hq), mk(Hkv), mk(Hkv), mk(Hq)
    o, dq = torch.empty_like(q), torch.empty_like(q)
    gk = torch.empty(B, Hkv, N, D, device=DEV)
    gv = torch.empty_like(gk)
    seco.kvgrad_zero(gk, gv)
    for j in range(cfg.n_chunks - 1, -1, -1):
        rows = slice(j * C, (j + 1) * C)
        _, lse = seco.seco_chunk_attn_fwd(q[:, :, rows], k, v, j * C, cfg.scale, o=o[:, :, rows])
        seco.seco_chunk_attn_bwd(q[:, :, rows], k, v, o[:, :, rows], lse, do[:, :, rows], gk, gv, j * C, cfg.scale,
                                 d_q=dq[:, :, rows])
    torch.cuda.synchronize()
    G = Hq // Hkv
    lhs = gv.double().sum(dim=2)
    rhs = do.double().view(B, Hkv, G, N, D).sum(dim=(2, 3))
    assert (lhs - rhs).abs().max() <= 2e-2 * rhs.abs().max()
    qdq = (q.double() * dq.double()).view(B, Hkv, G, N, D).sum(dim=(2, 3, 4))
    kgk = (k.double() * gk.double()).sum(dim=(2, 3))
    assert (qdq - kgk).abs().max() <= 2e-2 * kgk.abs().max().clamp_min(1.0)
    assert torch.isfinite(gk).all() and torch.isfinite(dq.float()).all()


# ---- short chunks: packed heads + split cache range (the chunk sizes of the paper's Sec. 6.3 study) -------------

@pytest.mark.parametrize("B,Hq,Hkv,N,C", [
    (1, 8, 2, 1024, 32),     # G = 4, one packed row tile per KV head, up to 4 splits
    (1, 8, 2, 1184, 96),     # row tiles that straddle two heads
    (1, 6, 2, 1100, 100),    # G = 3, chunk not a multiple of 32, idle wavefronts in the last tile
    (2, 4, 4, 1024, 64),     # G = 1: half of every row tile idle
    (1, 16, 2, 1536, 40),    # G = 8, second wavefront of each head partly valid
    (1, 32, 8, 2048, 128),   # the benchmark's head counts
])
def test_bf16_short_chunks_seco_parity(B, Hq, Hkv, N, C):
    x = small_layer(40, B, Hq, Hkv, N, 128, "bf16")
    s = 1 / np.sqrt(128)
    got = run_layer(x, C, s, "bf16")
    ref = A.seco_layer(x["q"], x["k"], x["v"], x["do"], C, s)
    check(got, ref, "bf16", f"bf16 short chunks {B,Hq,Hkv,N,C}")


def test_bf16_short_chunks_spaco_parity():
    N, C, sel, lam = 1024, 64, [15, 9, 3, 0], 4.0
    x = small_layer(41, 1, 8, 2, N, 128, "bf16")
    s = 1 / np.sqrt(128)
    got = run_layer(x, C, s, "bf16", selected=sel, factor=lam)
    ref = A.spaco_layer(x["q"], x["k"], x["v"], x["do"], C, s, sel, lam)
    for n, r in zip(("dq", "gk", "gv"), ref[2:]):
        assert max_rel(got[n], r) <= TOL["bf16"][n], n


def test_short_chunk_forward_with_and_without_workspace():
    """The split path (workspace given) and the direct path (none) are two evaluation orders of the same O, LSE."""
    B, Hq, Hkv, N, C, q_start = 1, 8, 2, 1600, 64, 1536
    x = small_layer(42, B, Hq, Hkv, N, 128, "bf16")
    s = 1 / np.sqrt(128)
    q, k, v = (to_dev(x[n], "bf16") for n in ("q", "k", "v"))
    qc = q[:, :, q_start:q_start + C]
    d = seco.binding.make_desc(qc, k, q_start, s)
    assert seco.seco_workspace_bytes(d, seco.binding.SECO_OP_FWD) > 0
    o1, l1 = seco.seco_chunk_attn_fwd(qc, k, v, q_start, s)
    o2, l2 = seco.seco_chunk_attn_fwd(qc, k, v, q_start, s, ws=False)
    o3, l3 = seco.seco_chunk_attn_fwd(qc, k, v, q_start, s)
    torch.cuda.synchronize()
    assert torch.equal(o1, o3) and torch.equal(l1, l3)             # the split path is deterministic
    ref_o, ref_l = A.chunk_attn_fwd(x["q"][:, :, q_start:q_start + C], x["k"][:, :, :q_start + C],
                                    x["v"][:, :, :q_start + C], q_start, s)
    for o, l in ((o1, l1), (o2, l2)):
        assert max_rel(to_host(o), ref_o) <= 1e-2
        assert max_rel(to_host(l), ref_l) <= 1e-2


@pytest.mark.parametrize("order", ["accumulating", "transposed"])
def test_step_captured_in_a_hip_graph_replays_identically(order):
    """The library allocates nothing, never synchronises and clears gK/gV with a kernel, so a whole SeCO step can be
    captured into a HIP graph, in either backward order.  Every replay (with eager work and synchronisations in
    between, and the outputs poisoned before each replay) must reproduce the eager result bit for bit (the kernels
    are deterministic)."""
    B, Hq, Hkv, N, C = 1, 8, 2, 768, 128           # short chunks: split kernels and merges are in the graph too
    x = small_layer(50, B, Hq, Hkv, N, 128, "bf16")
    s = 1 / np.sqrt(128)
    q, k, v, do = (to_dev(x[n], "bf16") for n in ("q", "k", "v", "do"))
    o = torch.empty_like(q)
    dq = torch.empty_like(q)
    lse = torch.empty(B, Hq, C, dtype=torch.float32, device=DEV)
    gk = torch.empty(B, Hkv, N, 128, dtype=torch.float32, device=DEV)
    gv = torch.empty_like(gk)
    d0 = seco.binding.make_desc(q[:, :, :C], k, 0, s, g=gk)
    ws_f = torch.empty(max(seco.seco_workspace_bytes(d0, seco.binding.SECO_OP_FWD), 256), dtype=torch.uint8, device=DEV)
    ws_b = torch.empty(max(seco.seco_workspace_bytes(d0, seco.binding.SECO_OP_BWD), 256), dtype=torch.uint8, device=DEV)

    def step():
        seco.kvgrad_zero(gk, gv)
        for j in range(N // C - 1, -1, -1):
            sl = slice(j * C, (j + 1) * C)
            seco.seco_chunk_attn_fwd(q[:, :, sl], k, v, j * C, s, o=o[:, :, sl], lse=lse, ws=ws_f)
            if order == "accumulating":
                seco.seco_chunk_attn_bwd(q[:, :, sl], k, v, o[:, :, sl], lse, do[:, :, sl], gk, gv, j * C, s,
                                         d_q=dq[:, :, sl], ws=ws_b)
            else:
                seco.seco_chunk_attn_bwd_gather(q[:, :, j * C:], k, v, o[:, :, sl], lse, do[:, :, j * C:], gk, gv,
                                                j * C, s, C, stats, d_q=dq[:, :, sl], ws=ws_b)

    stats = torch.empty(2, B, Hq, N, dtype=torch.float32, device=DEV)
    outs = (o, dq, gk, gv)
    step()
    torch.cuda.synchronize()
    eager = [t.clone() for t in outs]
    ref = A.seco_layer(x["q"], x["k"], x["v"], x["do"], C, s)
    assert max_rel(to_host(gk), ref[3]) <= 2e-2 and max_rel(to_host(dq), ref[2]) <= 2e-2

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        for t in outs + (stats,):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for t, e in zip(outs, eager):
            assert torch.equal(t, e), rep
        (q.float() @ q.float().transpose(-1, -2)).sum().item()      # unrelated eager work between replays


def test_more_weight_runs_than_one_segment_table_holds():
    """110 chunks of 32 rows with every second weight zero and the others all different: 55 runs of columns, more
    than the 48 a single launch of the dK/dV kernel takes by value, so the call is issued as two launches."""
    B, Hq, Hkv, C, k = 1, 2, 1, 32, 110
    N, j = k * C, k - 1
    x = small_layer(60, B, Hq, Hkv, N, 128, "bf16")
    s = 1 / np.sqrt(128)
    w = np.array([0.0 if i % 2 else 1.0 + 0.05 * i for i in range(k)], dtype=np.float32)
    w[j] = 1.0
    q, kc, vc, do = (to_dev(x[n], "bf16") for n in ("q", "k", "v", "do"))
    sl = slice(j * C, N)
    o, lse = seco.seco_chunk_attn_fwd(q[:, :, sl], kc, vc, j * C, s)
    gk = torch.zeros(B, Hkv, N, 128, dtype=torch.float32, device=DEV)
    gv = torch.zeros_like(gk)
    dq = seco.spaco_chunk_attn_bwd(q[:, :, sl], kc, vc, o, lse, do[:, :, sl].contiguous(), gk, gv, j * C, s,
                                   w.tolist(), C)
    torch.cuda.synchronize()
    ro, rl = A.chunk_attn_fwd(x["q"][:, :, sl], x["k"], x["v"], j * C, s)
    rdq, rdk, rdv = A.chunk_attn_bwd(x["q"][:, :, sl], x["k"], x["v"], ro, rl, x["do"][:, :, sl], j * C, s)
    wrow = np.repeat(w.astype(np.float64), C)[None, None, :, None]
    assert max_rel(to_host(dq), rdq) <= 2e-2
    assert max_rel(to_host(gk), wrow * rdk) <= 2e-2
    assert max_rel(to_host(gv), wrow * rdv) <= 2e-2
    zero_rows = np.repeat(w == 0.0, C)
    assert not to_host(gk)[:, :, zero_rows].any() and not to_host(gv)[:, :, zero_rows].any()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_append_and_readout_bit_exact(dtype):
    """kv_append / kvgrad_readout (appendix listing) against oracle/relay.py, strided chunk tensors, bit for bit."""
    from oracle import relay as R
    B, H, N, D, C, r0 = 2, 3, 160, 128 if dtype == "bf16" else 40, 48, 64
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    rng = np.random.default_rng(70)
    from workloads import round_to
    k_new = round_to(rng.standard_normal((B, H, C, D)).astype(np.float32), dtype)
    v_new = round_to(rng.standard_normal((B, H, C, D)).astype(np.float32), dtype)
    kc = round_to(rng.standard_normal((B, H, N, D)).astype(np.float32), dtype)
    vc = round_to(rng.standard_normal((B, H, N, D)).astype(np.float32), dtype)
    # chunk tensors as a projection would produce them: [B, C, H, D] storage viewed as [B, H, C, D]
    kn_dev = to_dev(k_new.transpose(0, 2, 1, 3).copy(), dtype).transpose(1, 2)
    vn_dev = to_dev(v_new.transpose(0, 2, 1, 3).copy(), dtype).transpose(1, 2)
    kc_dev, vc_dev = to_dev(kc, dtype), to_dev(vc, dtype)
    seco.kv_append(kn_dev, vn_dev, kc_dev, vc_dev, r0)
    rk, rv = R.kv_append(kc, vc, k_new, v_new, r0)
    np.testing.assert_array_equal(to_host(kc_dev), rk.astype(np.float64))
    np.testing.assert_array_equal(to_host(vc_dev), rv.astype(np.float64))

    gk = (rng.standard_normal((B, H, N, D)) * 3).astype(np.float32)
    gv = (rng.standard_normal((B, H, N, D)) * 3).astype(np.float32)
    gk_dev, gv_dev = torch.from_numpy(gk).to(DEV), torch.from_numpy(gv).to(DEV)
    for scaler in (1.0, 16 / 3):
        d_k = torch.empty(B, C, H, D, dtype=tdt, device=DEV).transpose(1, 2)      # strided output
        d_k, d_v = seco.kvgrad_readout(gk_dev, gv_dev, r0, C, tdt, scaler=scaler, d_k=d_k)
        np.testing.assert_array_equal(to_host(d_k), R.kvgrad_readout(gk, r0, r0 + C, scaler, dtype).astype(np.float64))
        np.testing.assert_array_equal(to_host(d_v), R.kvgrad_readout(gv, r0, r0 + C, scaler, dtype).astype(np.float64))
    assert torch.equal(gk_dev.cpu(), torch.from_numpy(gk))            # the buffers themselves are only read


def test_forward_reference_moves_when_later_scores_are_much_larger():
    """The forward keeps a row's exponent reference as long as the exponentials stay representable and moves it when a
    tile's sum exceeds 2^40 (or overflows).  Inputs built so that every later 64-column tile has scores far above
    all earlier ones (by 65 and by more than 128 in log2 units), and one with far smaller ones."""
    B, Hq, Hkv, N, C = 1, 2, 1, 512, 128
    s = 1 / np.sqrt(128)
    rng = np.random.default_rng(80)
    q = np.full((B, Hq, N, 128), 2.0, dtype=np.float32)
    q[:, 1] = -2.0                                           # second head: scores fall instead of rise
    k = np.zeros((B, Hkv, N, 128), dtype=np.float32)
    k[:, :, 64:128] = 2.0                                    # dot 512  -> +65 in log2 units
    k[:, :, 128:192] = 2.0
    k[:, :, 128:192, :64] = 7.0                              # dot 1152 -> +147: exp2 overflows before the move
    k[:, :, 192:] = 8.0                                      # dot 2048
    k += 0.01 * rng.standard_normal(k.shape).astype(np.float32)
    v = rng.standard_normal((B, Hkv, N, 128)).astype(np.float32)
    from workloads import round_to
    q, k, v = (round_to(t, "bf16") for t in (q, k, v))
    qd, kd, vd = (to_dev(t, "bf16") for t in (q, k, v))
    for j in range(N // C):
        sl = slice(j * C, (j + 1) * C)
        o, lse = seco.seco_chunk_attn_fwd(qd[:, :, sl], kd, vd, j * C, s)
        ro, rl = A.chunk_attn_fwd(q[:, :, sl], k, v, j * C, s)
        oh, lh = to_host(o), to_host(lse)
        assert np.isfinite(oh).all() and np.isfinite(lh).all()
        assert max_rel(oh, ro) <= 1e-2, j
        assert max_rel(lh, rl) <= 1e-2, j


def test_per_call_draw_policy_parity():
    """Every chunk back-propagated, each call with its own draw of earlier chunks (weights from the library's host
    policy call, which the CPU tests compare bit for bit with the oracle's)."""
    N, C, t, seed = 1024, 128, 3, 17
    k = N // C
    x = small_layer(90, 1, 4, 2, N, 128, "bf16")
    s = 1 / np.sqrt(128)
    got = run_layer(x, C, s, "bf16", selected=list(range(k)), weights_fn=lambda j: seco.spaco_percall_weights(seed, 0, j, t))
    calls = [(j, S.percall_weights(seed, 0, j, t)) for j in range(k - 1, -1, -1)]
    dq, gk, gv = A.weighted_layer(x["q"], x["k"], x["v"], x["do"], C, s, calls)
    for n, r in (("dq", dq), ("gk", gk), ("gv", gv)):
        assert max_rel(got[n], r) <= TOL["bf16"][n], n


# ---- column-weighted (sparse) dQ ----------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,D,Hq,Hkv,N,C,j,wq", [
    ("f32", 64, 4, 2, 512, 128, 3, [2.0, 0.0, 1.5, 1.0]),
    ("bf16", 128, 4, 2, 1024, 256, 3, [2.0, 0.0, 1.5, 1.0]),                       # short-chunk (split) kernel
    ("bf16", 128, 4, 2, 1280, 160, 7, [0.0, 3.0, 3.0, 0.0, 0.0, 1.25, 0.0, 1.0]),  # runs that start and end inside tiles
    ("bf16", 128, 4, 2, 1280, 160, 7, [0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 1.0]),   # own chunk only
    ("bf16", 128, 32, 8, 4096, 1024, 3, [4.0, 0.0, 0.5, 1.0]),                     # 8-wavefront kernel (128-row tiles)
    ("bf16", 128, 32, 8, 4096, 2048, 1, [0.75, 1.0]),                              # 4-wavefront kernel, 512 workgroups
    ("bf16", 128, 8, 2, 3000, 1000, 2, [2.0, 0.0, 1.0]),                           # ragged everything, G = 4
])
def test_sparse_dq_parity(dtype, D, Hq, Hkv, N, C, j, wq):
    """spaco_chunk_attn_bwd_sparse_dq against the oracle's column-weighted dQ; gK/gV do not depend on the dQ weights."""
    x = small_layer(50, 1, Hq, Hkv, N, D, dtype)
    q, k, v, do = (to_dev(x[n], dtype) for n in ("q", "k", "v", "do"))
    s = 1 / np.sqrt(D)
    s0 = j * C
    c = min(C, N - s0)
    qc, doc = q[:, :, s0:s0 + c], do[:, :, s0:s0 + c].contiguous()
    o, lse = seco.seco_chunk_attn_fwd(qc, k, v, s0, s)
    w = [1.0] * (j + 1)
    gk, gv = (torch.zeros(k.shape, dtype=torch.float32, device=DEV) for _ in range(2))
    dq = seco.spaco_chunk_attn_bwd(qc, k, v, o, lse, doc, gk, gv, s0, s, w, C, dq_weight=wq)
    gk0, gv0 = (torch.zeros(k.shape, dtype=torch.float32, device=DEV) for _ in range(2))
    dq_dense = seco.spaco_chunk_attn_bwd(qc, k, v, o, lse, doc, gk0, gv0, s0, s, w, C)
    torch.cuda.synchronize()
    assert torch.equal(gk, gk0) and torch.equal(gv, gv0)
    q64, k64, v64, do64 = (x[n].astype(np.float64) for n in ("q", "k", "v", "do"))
    o_ref, lse_ref = A.chunk_attn_fwd(q64[:, :, s0:s0 + c], k64, v64, s0, s)
    col_w = np.concatenate([np.full(min(C, s0 + c - i * C), wq[i]) for i in range(j + 1)])
    ref = A.chunk_attn_dq_weighted(q64[:, :, s0:s0 + c], k64, v64, o_ref, lse_ref, do64[:, :, s0:s0 + c], s0, s, col_w)
    exact, _, _ = A.chunk_attn_bwd(q64[:, :, s0:s0 + c], k64, v64, o_ref, lse_ref, do64[:, :, s0:s0 + c], s0, s)
    err, err_dense = max_rel(to_host(dq), ref), max_rel(to_host(dq_dense), exact)
    print(f"sparse dq {dtype} {Hq,Hkv,N,C,j}: {err:.2e}; dense {err_dense:.2e}", flush=True)
    assert err <= TOL[dtype]["dq"]
    assert err_dense <= TOL[dtype]["dq"]       # the dense instantiation of the same kernel shape
    o_err, lse_err = max_rel(to_host(o), o_ref), max_rel(to_host(lse), lse_ref)
    assert o_err <= TOL[dtype]["o"] and lse_err <= TOL[dtype]["lse"], (o_err, lse_err)
    assert max_rel(ref, exact) > 0.05          # the weights matter in this example


@pytest.mark.parametrize("dtype,D,C", [("f32", 64, 128), ("bf16", 128, 256), ("bf16", 128, 1024)])
def test_sparse_dq_special_cases(dtype, D, C):
    """All dQ weights 1: bit-identical to the dense call.  All 0: dQ = 0 (and gK/gV as usual).  Two reruns agree bitwise."""
    Hq, Hkv, j = (32, 8, 2) if C == 1024 else (4, 2, 3)
    N = (j + 1) * C
    x = small_layer(51, 1, Hq, Hkv, N, D, dtype)
    q, k, v, do = (to_dev(x[n], dtype) for n in ("q", "k", "v", "do"))
    s = 1 / np.sqrt(D)
    qc, doc = q[:, :, j * C:], do[:, :, j * C:].contiguous()
    o, lse = seco.seco_chunk_attn_fwd(qc, k, v, j * C, s)
    w = [2.0] * j + [1.0]

    def call(wq):
        gk, gv = (torch.zeros(k.shape, dtype=torch.float32, device=DEV) for _ in range(2))
        dq = seco.spaco_chunk_attn_bwd(qc, k, v, o, lse, doc, gk, gv, j * C, s, w, C, dq_weight=wq)
        torch.cuda.synchronize()
        return dq, gk, gv
    dense = call(None)
    ones = call([1.0] * (j + 1))
    zeros = call([0.0] * (j + 1))
    some = call([0.0, 3.0] + [1.0] * (j - 1))
    again = call([0.0, 3.0] + [1.0] * (j - 1))
    assert all(torch.equal(a, b) for a, b in zip(dense, ones))
    assert not zeros[0].any() and torch.equal(zeros[1], dense[1]) and torch.equal(zeros[2], dense[2])
    assert all(torch.equal(a, b) for a, b in zip(some, again))
    assert not torch.equal(some[0], dense[0])


def test_sparse_dq_many_runs_and_extreme_weights():
    """Dozens of runs of one isolated chunk each (the table holds 48), with weights from 1e-3 to 1e3 (the kernel
    folds a weight into the exponent as log2 w): short-chunk kernel with 32-row chunks, and the 8-wavefront kernel."""
    for Hq, Hkv, C, wlen, n_chunks in ((4, 2, 32, 32, 96), (32, 8, 1024, 64, 48)):
        N = wlen * n_chunks
        j_rows = N - C                                   # the call is for the last C rows
        x = small_layer(52, 1, Hq, Hkv, N, 128, "bf16")
        q, k, v, do = (to_dev(x[n], "bf16") for n in ("q", "k", "v", "do"))
        s = 1 / np.sqrt(128)
        qc, doc = q[:, :, j_rows:], do[:, :, j_rows:].contiguous()
        o, lse = seco.seco_chunk_attn_fwd(qc, k, v, j_rows, s)
        rng = np.random.default_rng(3)
        wq = np.zeros(n_chunks, dtype=np.float32)
        picked = np.sort(rng.choice(n_chunks - C // wlen, size=47 if n_chunks == 96 else 20, replace=False))
        picked = picked[np.concatenate([[True], np.diff(picked) > 1])]          # isolated chunks: one run each
        wq[picked] = np.float32(10.0) ** rng.uniform(-3, 3, size=len(picked)).astype(np.float32)
        wq[n_chunks - C // wlen:] = 1.0                                          # the call's own rows
        gk, gv = (torch.zeros(k.shape, dtype=torch.float32, device=DEV) for _ in range(2))
        dq = seco.spaco_chunk_attn_bwd(qc, k, v, o, lse, doc, gk, gv, j_rows, s, [1.0] * n_chunks, wlen,
                                       dq_weight=wq.tolist())
        torch.cuda.synchronize()
        q64, k64, v64, do64 = (x[n].astype(np.float64) for n in ("q", "k", "v", "do"))
        o_ref, lse_ref = A.chunk_attn_fwd(q64[:, :, j_rows:], k64, v64, j_rows, s)
        ref = A.chunk_attn_dq_weighted(q64[:, :, j_rows:], k64, v64, o_ref, lse_ref, do64[:, :, j_rows:], j_rows, s,
                                       np.repeat(wq.astype(np.float64), wlen))
        err = max_rel(to_host(dq), ref)
        print(f"sparse dq, {len(picked) + 1} runs, weights {wq[wq > 0].min():.1e} .. {wq.max():.1e}: {err:.2e}", flush=True)
        assert err <= TOL["bf16"]["dq"]


@pytest.mark.parametrize("seed", range(12))
def test_random_shapes_and_weights(seed):
    """Seeded random small configurations through every entry point of the backward: shapes that are not multiples
    of any tile, random selections with random dK/dV weights and random dQ weights (zeros included)."""
    rng = np.random.default_rng(1000 + seed)
    dtype = "f32" if seed % 4 == 3 else "bf16"
    D = int(rng.choice([16, 40, 64])) if dtype == "f32" else 128
    Hkv = int(rng.choice([1, 2, 3]))
    Hq = Hkv * int(rng.choice([1, 2, 4]))
    B = int(rng.choice([1, 2]))
    C = int(rng.integers(1, 260 if dtype == "bf16" else 70))
    k = int(rng.integers(1, 7))
    N = C * (k - 1) + int(rng.integers(1, C + 1))           # ragged last chunk
    x = small_layer(2000 + seed, B, Hq, Hkv, N, D, dtype)
    s = float(rng.uniform(0.5, 1.5)) / np.sqrt(D)
    sel = sorted({int(i) for i in rng.choice(k, size=int(rng.integers(1, k + 1)), replace=False)}, reverse=True)
    w_of, wq_of = {}, {}
    for j in sel:
        w = np.where(rng.random(j + 1) < 0.6, rng.uniform(0.25, 4.0, j + 1), 0.0).astype(np.float32)
        w[j] = 1.0
        wq = np.where(rng.random(j + 1) < 0.6, rng.uniform(0.25, 4.0, j + 1), 0.0).astype(np.float32)
        w_of[j], wq_of[j] = w, (wq if rng.random() < 0.7 else None)
    got = run_layer(x, C, s, dtype, selected=sel, weights_fn=lambda j: w_of[j].tolist(),
                    dq_weights_fn=lambda j: None if wq_of[j] is None else wq_of[j].tolist())
    dq, gk, gv = A.weighted_layer(x["q"], x["k"], x["v"], x["do"], C, s, [(j, w_of[j], wq_of[j]) for j in sel])
    o, lse, *_ = A.seco_layer(x["q"], x["k"], x["v"], x["do"], C, s)
    what = f"random {seed}: {dtype} B{B} Hq{Hq} Hkv{Hkv} D{D} N{N} C{C} sel{sel}"
    errs = {n: max_rel(got[n], r) for n, r in (("o", o), ("lse", lse), ("dq", dq), ("gk", gk), ("gv", gv))}
    print(what, {n: f"{e:.1e}" for n, e in errs.items()}, flush=True)
    for n, e in errs.items():
        assert np.isfinite(got[n]).all() and e <= TOL[dtype][n], (what, n, e)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_rope_append_readout_and_rotate(dtype):
    """kv_append_rope / kvgrad_readout_rope / rope_rotate against oracle/relay.py: the kernels compute angles and
    sines in fp64 and round once, so results agree with the oracle up to the last bit of the storage type (a sine
    that differs in its last fp64 bit can flip a rounding)."""
    from oracle import relay as R
    from workloads import round_to
    B, H, N, D, C, r0, base = 2, 3, 4200, 128 if dtype == "bf16" else 40, 48, 4096, 500000.0
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    ulp = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -23
    rng = np.random.default_rng(71)
    k_new = round_to(rng.standard_normal((B, H, C, D)).astype(np.float32), dtype)
    v_new = round_to(rng.standard_normal((B, H, C, D)).astype(np.float32), dtype)
    kc, vc = np.zeros((B, H, N, D), np.float32), np.zeros((B, H, N, D), np.float32)
    kn_dev = to_dev(k_new.transpose(0, 2, 1, 3).copy(), dtype).transpose(1, 2)      # [B, C, H, D] storage
    vn_dev = to_dev(v_new.transpose(0, 2, 1, 3).copy(), dtype).transpose(1, 2)
    kc_dev, vc_dev = to_dev(kc, dtype), to_dev(vc, dtype)
    seco.kv_append(kn_dev, vn_dev, kc_dev, vc_dev, r0, rope_base=base)
    rk, rv = R.kv_append_rope(kc, vc, k_new, v_new, r0, base, dtype)

    def close(got, ref, what):
        got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
        same = np.mean(got == ref)
        err = np.abs(got - ref).max() / np.abs(ref).max()
        print(f"{what} {dtype}: {100 * same:.3f} % bit-equal, max rel diff {err:.1e}", flush=True)
        assert same > 0.995 and err <= ulp, (what, same, err)
    close(to_host(kc_dev), rk, "append")
    np.testing.assert_array_equal(to_host(vc_dev), rv.astype(np.float64))
    # the rotated keys really depend on the position: the same rows appended at another place differ
    assert np.abs(rk[:, :, r0:r0 + C] - R.kv_append_rope(kc, vc, k_new, v_new, 7, base, dtype)[0][:, :, 7:7 + C]).max() > 0.1

    gk = (rng.standard_normal((B, H, N, D)) * 3).astype(np.float32)
    gv = (rng.standard_normal((B, H, N, D)) * 3).astype(np.float32)
    gk_dev, gv_dev = torch.from_numpy(gk).to(DEV), torch.from_numpy(gv).to(DEV)
    d_k = torch.empty(B, C, H, D, dtype=tdt, device=DEV).transpose(1, 2)          # strided output
    d_k, d_v = seco.kvgrad_readout(gk_dev, gv_dev, r0, C, tdt, scaler=16 / 3, d_k=d_k, rope_base=base)
    ref_k, ref_v = R.kvgrad_readout_rope(gk, gv, r0, r0 + C, 16 / 3, base, dtype)
    close(to_host(d_k), ref_k, "read-out")
    np.testing.assert_array_equal(to_host(d_v), ref_v.astype(np.float64))

    q = round_to(rng.standard_normal((B, 5, C, D)).astype(np.float32), dtype)
    q_dev = to_dev(q, dtype)
    rot = seco.rope_rotate(q_dev, r0, base)
    close(to_host(rot), R._to_storage(R.rope_rotate(q, r0, base), dtype), "rotate")
    back = seco.rope_rotate(rot, r0, base, inverse=True, out=rot)                  # in place
    assert np.abs(to_host(back) - q).max() <= 3 * ulp * np.abs(q).max()
