"""GPU parity at the benchmark's own launch shapes.

A chunk call picks its kernels from the number of work items: with all 32 query heads of the benchmark
configurations a call runs the direct forward / dQ kernels (the 8-wavefront shape at cfg2, the 4-wavefront shape at
cfg3, cfg4 and the long chunks of cfg5) and dK/dV column tiles with whole-tile read-modify-write, whereas a single
(batch, KV head) unit on its own would be sent down the short-chunk path.  The tests here therefore run the FULL
multi-unit shape on the GPU and let the fp64 oracle check whole (batch, KV head) units of it element by element
(units are independent, so a unit checked in full is a complete check of that unit), after asserting through
seco_launch_plan that the call really took the direct path.  Tolerances as everywhere: max |x - ref| / max |ref|
<= 1e-2 on O and LSE, 2e-2 on dQ, gK, gV; the same bound is also asserted per (batch, head) slice, times 1.5.
"""
import functools
import time

import numpy as np
import pytest
import torch

import paper_2505_16710_amd as seco
from oracle import attention as A
from oracle import selection as S
from workloads import CONFIGS, f32_to_bf16_bits, head_slice

from hip_driver import DEV, max_rel, max_rel_per_head, to_host

pytestmark = pytest.mark.gpu

TOL = {"o": 1e-2, "lse": 1e-2, "dq": 2e-2, "gk": 2e-2, "gv": 2e-2}


class DeviceLayer:
    """All heads of a configuration on the GPU (uploaded head by head), fp32 host copies of chosen units only."""

    def __init__(self, cfg, units):
        self.cfg, self.units = cfg, list(units)
        B, Hq, Hkv, N, D = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.seq_len, cfg.head_dim
        self.G = Hq // Hkv
        self.host = {u: {} for u in self.units}
        t0 = time.time()
        self.dev = {}
        for name, H in (("q", Hq), ("do", Hq), ("k", Hkv), ("v", Hkv)):
            t = torch.empty(B, H, N, D, dtype=torch.bfloat16, device=DEV)
            for b in range(B):
                for h in range(H):
                    x = head_slice(cfg, name, b, h)
                    t[b, h] = torch.from_numpy(f32_to_bf16_bits(x).view(np.int16)).to(DEV).view(torch.bfloat16)
                    kvh = h // self.G if H == Hq else h
                    if (b, kvh) in self.host:
                        self.host[(b, kvh)].setdefault(name, []).append(x.astype(np.float64))
            self.dev[name] = t
        print(f"{cfg.name}: inputs generated and uploaded in {time.time() - t0:.1f} s", flush=True)

    def unit(self, u):
        """fp64 oracle inputs of unit u = (batch, KV head): q, do [1, G, N, D]; k, v [1, 1, N, D]"""
        h = self.host[u]
        return {"q": np.stack(h["q"])[None], "do": np.stack(h["do"])[None], "k": h["k"][0][None, None],
                "v": h["v"][0][None, None]}


@functools.lru_cache(maxsize=1)
def _layer(name, units):
    return DeviceLayer(CONFIGS[name], units)


def _assert_direct(L, C, q_start, expect_row_tiles_at_least=None):
    q = L.dev["q"]
    d = seco.binding.make_desc(q[:, :, q_start:q_start + C], L.dev["k"], q_start, L.cfg.scale)
    n_col_tiles = -(-(q_start + C) // 128)
    plan = seco.seco_launch_plan(d, n_col_tiles)
    assert plan[0] == 1, plan                      # no division of the cache range: the direct kernels
    if expect_row_tiles_at_least is not None:
        assert plan[1] >= expect_row_tiles_at_least, plan
    return plan


def _one_call(L, C, j):
    """Forward + SeCO backward of chunk j alone on the full shape, gK/gV zeroed first.  Device tensors."""
    cfg = L.cfg
    q, k, v, do = (L.dev[n] for n in ("q", "k", "v", "do"))
    sl = slice(j * C, (j + 1) * C)
    gk = torch.zeros(k.shape, dtype=torch.float32, device=DEV)
    gv = torch.zeros_like(gk)
    o, lse = seco.seco_chunk_attn_fwd(q[:, :, sl], k, v, j * C, cfg.scale)                 # o: contiguous
    dq = seco.seco_chunk_attn_bwd(q[:, :, sl], k, v, o, lse, do[:, :, sl].contiguous(), gk, gv, j * C, cfg.scale)
    torch.cuda.synchronize()
    return o, lse, dq, gk, gv


def _check_unit_call(L, u, C, j, got, what):
    """One unit of one call against the oracle, element by element."""
    cfg, G = L.cfg, L.G
    b, kvh = u
    x = L.unit(u)
    sl = slice(j * C, (j + 1) * C)
    L_j = (j + 1) * C
    t0 = time.time()
    o_ref, lse_ref = A.chunk_attn_fwd(x["q"][:, :, sl], x["k"][:, :, :L_j], x["v"][:, :, :L_j], j * C, cfg.scale)
    dq_ref, dk_ref, dv_ref = A.chunk_attn_bwd(x["q"][:, :, sl], x["k"][:, :, :L_j], x["v"][:, :, :L_j], o_ref, lse_ref,
                                              x["do"][:, :, sl], j * C, cfg.scale)
    o, lse, dq, gk, gv = got
    hs = slice(kvh * G, (kvh + 1) * G)
    mine = {"o": to_host(o[b:b + 1, hs]), "lse": to_host(lse[b:b + 1, hs]), "dq": to_host(dq[b:b + 1, hs]),
            "gk": to_host(gk[b:b + 1, kvh:kvh + 1, :L_j]), "gv": to_host(gv[b:b + 1, kvh:kvh + 1, :L_j])}
    refs = {"o": o_ref, "lse": lse_ref, "dq": dq_ref, "gk": dk_ref, "gv": dv_ref}
    errs = {n: (max_rel(mine[n], refs[n]), max_rel_per_head(mine[n], refs[n])) for n in refs}
    print(f"{what} unit {u} call {j}: " + ", ".join(f"{n} {e[0]:.2e}/{e[1]:.2e}" for n, e in errs.items()) +
          f"  (oracle {time.time() - t0:.1f} s)", flush=True)
    for n, (e, eh) in errs.items():
        assert np.isfinite(mine[n]).all(), (what, n)
        assert e <= TOL[n] and eh <= 1.5 * TOL[n], (what, u, j, n, e, eh)
    # rows past the call's last visible row are never touched
    assert not gk[b, kvh, L_j:].any() and not gv[b, kvh, L_j:].any()


# ---- cfg3 shape: 4-wavefront direct forward, dense 4-wavefront dQ, whole-tile dK/dV ---------------------------------

CFG3_UNITS = ((0, 1), (0, 6))


@pytest.mark.parametrize("j", [0, 1, 7])
def test_cfg3_full_shape_calls_element_wise(j):
    """B 1, 32 / 8 heads, chunks of 2048: 512 row tiles, so the 4-wavefront direct kernels; call j covers 128 (j + 1)
    column tiles.  O, LSE, dense dQ, gK, gV of two whole units, every element."""
    L = _layer("cfg3", CFG3_UNITS)
    C = L.cfg.chunk_len
    plan = _assert_direct(L, C, j * C, expect_row_tiles_at_least=512)
    got = _one_call(L, C, j)
    for u in CFG3_UNITS:
        _check_unit_call(L, u, C, j, got, f"cfg3 {plan}")


def test_cfg3_full_shape_spaco_sampled():
    """cfg3 as specified: Alg. 2 with 4 of 16 chunks (seeded), factor k/t = 4, on the full 32-head launch; two units."""
    _spaco_full_launch_check(_layer("cfg3", CFG3_UNITS), CONFIGS["cfg3"], CFG3_UNITS)


def test_cfg3_full_shape_last_call_with_its_own_draw():
    """The other reading of cfg3's wording: the single call of the last chunk with 4 sampled earlier chunks plus
    itself (weights j / 4 on the drawn chunks, 1 on its own rows, from the library's host policy call, which the CPU
    tests compare with the oracle's bit for bit), on the full launch; dQ exact, gK / gV = weight x the call's dK / dV,
    unselected chunks untouched.  Two units, every element."""
    L = _layer("cfg3", CFG3_UNITS)
    cfg, G = L.cfg, L.G
    C, j = cfg.chunk_len, cfg.n_chunks - 1
    w = seco.spaco_percall_weights(cfg.seed, 0, j, cfg.spaco_t)
    assert np.array_equal(np.array(w, dtype=np.float32), S.percall_weights(cfg.seed, 0, j, cfg.spaco_t))
    assert sum(1 for x in w[:j] if x != 0) == cfg.spaco_t and w[j] == 1.0
    q, k, v, do = (L.dev[n] for n in ("q", "k", "v", "do"))
    sl = slice(j * C, (j + 1) * C)
    gk = torch.zeros(k.shape, dtype=torch.float32, device=DEV)
    gv = torch.zeros_like(gk)
    o, lse = seco.seco_chunk_attn_fwd(q[:, :, sl], k, v, j * C, cfg.scale)
    dq = seco.spaco_chunk_attn_bwd(q[:, :, sl], k, v, o, lse, do[:, :, sl].contiguous(), gk, gv, j * C, cfg.scale, w, C)
    torch.cuda.synchronize()
    wrow = np.repeat(np.array(w, dtype=np.float64), C)[None, None, :, None]
    for (b, kvh) in CFG3_UNITS:
        x = L.unit((b, kvh))
        o_ref, lse_ref = A.chunk_attn_fwd(x["q"][:, :, sl], x["k"], x["v"], j * C, cfg.scale)
        dq_ref, dk_ref, dv_ref = A.chunk_attn_bwd(x["q"][:, :, sl], x["k"], x["v"], o_ref, lse_ref, x["do"][:, :, sl],
                                                  j * C, cfg.scale)
        hs = slice(kvh * G, (kvh + 1) * G)
        gk_u, gv_u = to_host(gk[b:b + 1, kvh:kvh + 1]), to_host(gv[b:b + 1, kvh:kvh + 1])
        errs = {"dq": max_rel(to_host(dq[b:b + 1, hs]), dq_ref), "gk": max_rel(gk_u, wrow * dk_ref),
                "gv": max_rel(gv_u, wrow * dv_ref)}
        print(f"cfg3 last call, weights {[round(x, 2) for x in w]}, unit {(b, kvh)}: {errs}", flush=True)
        assert all(e <= TOL[n] for n, e in errs.items()), errs
        zero_rows = np.repeat(np.array(w) == 0.0, C)
        assert not gk_u[:, :, zero_rows].any() and not gv_u[:, :, zero_rows].any()


# ---- cfg2 shape: 8-wavefront forward and dQ with long tile loops, all 16 calls --------------------------------------

CFG2_UNITS = ((0, 2), (0, 5))


@functools.lru_cache(maxsize=1)
def _cfg2_whole_layer():
    L = _layer("cfg2", CFG2_UNITS)
    cfg = L.cfg
    C, k_chunks = cfg.chunk_len, cfg.n_chunks
    q, k, v, do = (L.dev[n] for n in ("q", "k", "v", "do"))
    o, dq = torch.empty_like(q), torch.empty_like(q)
    lse = torch.empty(q.shape[:3], dtype=torch.float32, device=DEV)
    gk = torch.full(k.shape, float("nan"), dtype=torch.float32, device=DEV)
    gv = torch.full_like(gk, float("nan"))
    seco.kvgrad_zero(gk, gv)
    for j in range(k_chunks - 1, -1, -1):
        plan = _assert_direct(L, C, j * C)
        assert plan[1] == 256                      # 256 row tiles of 128 rows: the 8-wavefront shape
        sl = slice(j * C, (j + 1) * C)
        _, l = seco.seco_chunk_attn_fwd(q[:, :, sl], k, v, j * C, cfg.scale, o=o[:, :, sl])
        lse[:, :, sl] = l
        seco.seco_chunk_attn_bwd(q[:, :, sl], k, v, o[:, :, sl], l, do[:, :, sl], gk, gv, j * C, cfg.scale,
                                 d_q=dq[:, :, sl])
    torch.cuda.synchronize()
    return L, (o, lse, dq, gk, gv)


@pytest.mark.parametrize("u", CFG2_UNITS)
def test_cfg2_full_shape_whole_layer_units(u):
    """cfg2 as the benchmark runs it (16 forward + backward call pairs on all 32 heads); one whole unit per test
    through the oracle's Alg. 1 loop."""
    L, (o, lse, dq, gk, gv) = _cfg2_whole_layer()
    cfg, G = L.cfg, L.G
    b, kvh = u
    x = L.unit(u)
    t0 = time.time()
    ref = A.seco_layer(x["q"], x["k"], x["v"], x["do"], cfg.chunk_len, cfg.scale)
    hs = slice(kvh * G, (kvh + 1) * G)
    mine = (to_host(o[b:b + 1, hs]), to_host(lse[b:b + 1, hs]), to_host(dq[b:b + 1, hs]),
            to_host(gk[b:b + 1, kvh:kvh + 1]), to_host(gv[b:b + 1, kvh:kvh + 1]))
    errs = {n: (max_rel(m, r), max_rel_per_head(m, r)) for n, m, r in zip(TOL, mine, ref)}
    print(f"cfg2 whole layer unit {u}: " + ", ".join(f"{n} {e[0]:.2e}/{e[1]:.2e}" for n, e in errs.items()) +
          f"  (oracle {time.time() - t0:.1f} s)", flush=True)
    for (n, (e, eh)), m in zip(errs.items(), mine):
        assert np.isfinite(m).all(), n
        assert e <= TOL[n] and eh <= 1.5 * TOL[n], (u, n, e, eh)


# ---- cfg5 at full size: batch 2, RoPE-like Q / K, chunks of 512 and of 4096 -----------------------------------------

CFG5_UNITS = ((0, 3), (1, 4))


@pytest.mark.parametrize("C,calls", [(512, (0, 1, 20)), (4096, (0, 2))])
def test_cfg5_full_size_seco_calls(C, calls):
    """SeCO call pairs of cfg5 (B 2, 32K tokens, sin/cos-modulated Q and K with a per-head mean) on the full launch;
    two whole units per call against the oracle.  Chunks of 512 run the 8-wavefront shape (256 row tiles), chunks of
    4096 the 4-wavefront shape (2048 row tiles)."""
    L = _layer("cfg5_c512", CFG5_UNITS)            # the cfg5 workloads share one seed: the tensors do not depend on C
    for j in calls:
        plan = _assert_direct(L, C, j * C)
        got = _one_call(L, C, j)
        for u in CFG5_UNITS:
            _check_unit_call(L, u, C, j, got, f"cfg5 C{C} {plan}")


@pytest.mark.parametrize("name", ["cfg5_c512", "cfg5_c4096"])
def test_cfg5_full_size_spaco_sampled(name):
    """Alg. 2 on the full cfg5 launch with the seeded selection (a quarter of the chunks, factor k/t = 4)."""
    _spaco_full_launch_check(_layer("cfg5_c512", CFG5_UNITS), CONFIGS[name], CFG5_UNITS)


CFG4_UNITS = ((0, 0), (0, 5))


def test_cfg4_full_shape_last_call_element_wise():
    """cfg4 (64K tokens, 32 chunks of 2048): the SeCO call pair of the LAST chunk on the full launch (65536 visible
    cache rows, 4096 column tiles, 16 rounds of the dK/dV pass), two whole units element by element."""
    L = _layer("cfg4", CFG4_UNITS)
    C, j = L.cfg.chunk_len, L.cfg.n_chunks - 1
    plan = _assert_direct(L, C, j * C, expect_row_tiles_at_least=512)
    got = _one_call(L, C, j)
    for u in CFG4_UNITS:
        _check_unit_call(L, u, C, j, got, f"cfg4 {plan}")


def test_cfg4_full_shape_spaco_sampled():
    """cfg4 as specified: Alg. 2 with 8 of 32 chunks (seeded), factor 4, on the full launch; two units."""
    _spaco_full_launch_check(_layer("cfg4", CFG4_UNITS), CONFIGS["cfg4"], CFG4_UNITS)


def _spaco_full_launch_check(L, cfg, units):
    """Alg. 2 on a full launch with the configuration's seeded selection: the oracle checks, on the given units,
    sampled query rows of every selected chunk (O, LSE, dQ), the own rows of the top selected chunk (gK/gV there come
    from that call alone), the rows of the lowest selected chunk in full (own block plus factor x the blocks of
    every higher selected call), and that unselected chunks stay exactly zero."""
    name = cfg.name
    k_chunks, t, C, scale = cfg.n_chunks, cfg.spaco_t, cfg.chunk_len, cfg.scale
    sel = S.select_chunks(cfg.seed, 0, k_chunks, t).tolist()
    assert sel == seco.spaco_select_chunks(cfg.seed, 0, k_chunks, t)
    lam = float(np.float32(S.compensation_factor(k_chunks, t)))
    q, k, v, do = (L.dev[n] for n in ("q", "k", "v", "do"))
    o, dq = torch.zeros_like(q), torch.zeros_like(q)
    lse = torch.zeros(q.shape[:3], dtype=torch.float32, device=DEV)
    gk = torch.full(k.shape, float("nan"), dtype=torch.float32, device=DEV)
    gv = torch.full_like(gk, float("nan"))
    seco.kvgrad_zero(gk, gv)
    for j in sel:                                   # descending
        _assert_direct(L, C, j * C)
        sl = slice(j * C, (j + 1) * C)
        _, l = seco.seco_chunk_attn_fwd(q[:, :, sl], k, v, j * C, scale, o=o[:, :, sl])
        lse[:, :, sl] = l
        seco.spaco_chunk_attn_bwd(q[:, :, sl], k, v, o[:, :, sl], l, do[:, :, sl], gk, gv, j * C, scale,
                                  seco.spaco_chunk_weights(sel, j, lam), C, d_q=dq[:, :, sl])
    torch.cuda.synchronize()
    rng = np.random.default_rng(11)
    G = L.G
    for (b, kvh) in units:
        x = L.unit((b, kvh))
        q64, k64, v64, do64 = x["q"], x["k"], x["v"], x["do"]
        hs = slice(kvh * G, (kvh + 1) * G)
        g = {"o": to_host(o[b:b + 1, hs]), "lse": to_host(lse[b:b + 1, hs]), "dq": to_host(dq[b:b + 1, hs]),
             "gk": to_host(gk[b:b + 1, kvh:kvh + 1]), "gv": to_host(gv[b:b + 1, kvh:kvh + 1])}
        for j in sel:
            for r in rng.integers(0, C, size=2):
                p = j * C + int(r)
                o_r, lse_r = A.chunk_attn_fwd(q64[:, :, p:p + 1], k64[:, :, :p + 1], v64[:, :, :p + 1], p, scale)
                dq_r, _, _ = A.chunk_attn_bwd(q64[:, :, p:p + 1], k64[:, :, :p + 1], v64[:, :, :p + 1], o_r, lse_r,
                                              do64[:, :, p:p + 1], p, scale)
                assert np.abs(g["o"][:, :, p] - o_r[:, :, 0]).max() <= 1e-2 * np.abs(o_r).max()
                assert np.abs(g["lse"][:, :, p] - lse_r[:, :, 0]).max() <= 1e-2 * np.abs(lse_r).max()
                assert np.abs(g["dq"][:, :, p] - dq_r[:, :, 0]).max() <= 2e-2 * np.abs(dq_r).max()
        # The oracle backward takes LSE and O as inputs, so with the true LSE and O of a chunk and a cache cut down
        # to some rows followed by the chunk's own rows it returns exactly those rows' blocks of dK/dV.
        fwd_of = {}
        for j in sel:
            qr = slice(j * C, (j + 1) * C)
            fwd_of[j] = A.chunk_attn_fwd(q64[:, :, qr], k64[:, :, :(j + 1) * C], v64[:, :, :(j + 1) * C], j * C, scale)
        top, low = sel[0], sel[-1]
        rows = slice(top * C, (top + 1) * C)
        _, dk_own, dv_own = A.chunk_attn_bwd(q64[:, :, rows], k64[:, :, rows], v64[:, :, rows], *fwd_of[top],
                                             do64[:, :, rows], 0, scale)
        assert max_rel(g["gk"][:, :, rows], dk_own) <= 2e-2 and max_rel(g["gv"][:, :, rows], dv_own) <= 2e-2
        rows = slice(low * C, (low + 1) * C)
        want_k = np.zeros_like(g["gk"][:, :, rows])
        want_v = np.zeros_like(want_k)
        for j in sel:
            qr = slice(j * C, (j + 1) * C)
            if j == low:
                _, dk, dv = A.chunk_attn_bwd(q64[:, :, qr], k64[:, :, rows], v64[:, :, rows], *fwd_of[j],
                                             do64[:, :, qr], 0, scale)
                want_k += dk
                want_v += dv
            else:
                _, dk, dv = A.chunk_attn_bwd(q64[:, :, qr], np.concatenate([k64[:, :, rows], k64[:, :, qr]], axis=2),
                                             np.concatenate([v64[:, :, rows], v64[:, :, qr]], axis=2), *fwd_of[j],
                                             do64[:, :, qr], C, scale)
                want_k += lam * dk[:, :, :C]
                want_v += lam * dv[:, :, :C]
        ek, ev = max_rel(g["gk"][:, :, rows], want_k), max_rel(g["gv"][:, :, rows], want_v)
        print(f"{name} unit {(b, kvh)} sel {sel}: lowest selected chunk gK {ek:.2e} gV {ev:.2e}", flush=True)
        assert ek <= 2e-2 and ev <= 2e-2
        for i in range(k_chunks):
            if i not in sel:
                cs = slice(i * C, (i + 1) * C)
                assert not g["gk"][:, :, cs].any() and not g["gv"][:, :, cs].any() and not g["dq"][:, :, cs].any()


# ---- large logits: structured Q / K whose scores are far from zero --------------------------------------------------

def test_backward_with_large_structured_logits():
    """One head_dim component of every key and query carries a large, nearly constant value (as the outlier
    components of trained models do), so every scaled score is about 24 in log2 units while the softmax itself stays
    spread out.  P = exp(S - LSE) then hangs on the low-order bits of S: any rounding of K (or Q) beyond the storage
    type before the score product shows up as a per-column error of several per cent in gV and gK."""
    from workloads import round_to
    B, Hq, Hkv, N, C, D = 1, 8, 2, 1024, 512, 128
    s = 1 / np.sqrt(D)
    rng = np.random.default_rng(321)
    q = rng.standard_normal((B, Hq, N, D)).astype(np.float32)
    k = rng.standard_normal((B, Hkv, N, D)).astype(np.float32)
    # (the larger share of the product sits on the query side: dQ = s dS K sums K's outlier against rows of dS that
    # cancel exactly, so the bf16 rounding of dS, which every bf16 attention backward has, would otherwise dominate)
    q[..., 5] = 32.0 + 0.1 * rng.standard_normal((B, Hq, N)).astype(np.float32)
    k[..., 5] = 6.0 + 0.3 * rng.standard_normal((B, Hkv, N)).astype(np.float32)
    v = rng.standard_normal((B, Hkv, N, D)).astype(np.float32)
    do = rng.standard_normal((B, Hq, N, D)).astype(np.float32)
    x = {n: round_to(a, "bf16") for n, a in (("q", q), ("k", k), ("v", v), ("do", do))}
    from hip_driver import run_layer
    got = run_layer(x, C, s, "bf16")
    ref = A.seco_layer(x["q"], x["k"], x["v"], x["do"], C, s)
    s_log2 = (x["q"][0, 0, -1].astype(np.float64) @ x["k"][0, 0].astype(np.float64).T) * s * np.log2(np.e)
    assert 15 < np.median(s_log2) < 40
    errs = {n: (max_rel(got[n], r), max_rel_per_head(got[n], r)) for n, r in zip(TOL, ref)}
    print("large logits: " + ", ".join(f"{n} {e[0]:.2e}/{e[1]:.2e}" for n, e in errs.items()), flush=True)
    for n, (e, eh) in errs.items():
        assert e <= TOL[n] and eh <= 1.5 * TOL[n], (n, e, eh)
