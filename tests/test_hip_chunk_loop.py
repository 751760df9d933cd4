"""GPU parity of the end-to-end SeCO / SpaCO step (Alg. 1, Alg. 2 over a multi-layer decoder) against the
fp64 model oracle: same seeded parameters and tokens on both sides, parameter gradients compared tensor by
tensor as max|x - ref| / max|ref|.

Tolerances: fp32 run 5e-4 (the kernels' own bar is 1e-4 per call; here three layers of fp32 GEMMs, norms and
the relay stack on top of each other), bf16 run 6e-2 (every activation and every relayed gradient is rounded to
bf16, 2^-9 relative each, through about 20 roundings per chain)."""
import pytest
import torch

from oracle import model as om

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _setup(cfg, seed, B, N, dtype):
    from paper_2505_16710_amd.chunk_loop import ChunkedDecoder
    p64 = om.init_params(cfg, seed)
    if dtype is torch.bfloat16:        # both sides start from the same bf16-representable parameters
        p64 = {n: t.detach().to(torch.bfloat16).to(torch.float64).requires_grad_() for n, t in p64.items()}
    pg = {n: t.detach().to(dtype).to(DEV).requires_grad_() for n, t in p64.items()}
    g = torch.Generator().manual_seed(seed + 100)
    tok = torch.randint(0, cfg.vocab, (B, N), generator=g)
    tgt = torch.randint(0, cfg.vocab, (B, N), generator=g)
    dec = ChunkedDecoder(pg, cfg.n_layers, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                         rope_base=cfg.rope_base if cfg.rope_base > 1.0 else None)
    return p64, dec, tok, tgt


def _compare(g_ref, g_gpu, tol):
    worst = 0.0
    for n, ref in g_ref.items():
        x = g_gpu[n].detach().to(torch.float64).cpu()
        err = float((x - ref).abs().max() / ref.abs().max().clamp_min(1e-30))
        worst = max(worst, err)
        assert err < tol, (n, err)
    return worst


F32_CFG = om.ModelConfig(n_layers=3, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=32, d_ff=96, vocab=29)
BF16_CFG = om.ModelConfig(n_layers=2, d_model=64, n_q_heads=2, n_kv_heads=1, head_dim=128, d_ff=96, vocab=29)


@pytest.mark.parametrize("N,C", [(96, 24), (100, 32)])
def test_seco_step_fp32_matches_whole_sequence_gradient(N, C):
    p64, dec, tok, tgt = _setup(F32_CFG, 5, 2, N, torch.float32)
    loss_ref, g_ref = om.monolithic_grads(F32_CFG, p64, tok, tgt)
    loss, g = dec.step(tok.to(DEV), tgt.to(DEV), C)
    assert abs(loss - float(loss_ref)) < 1e-4 * abs(float(loss_ref))
    _compare(g_ref, g, 5e-4)


def test_spaco_step_fp32_matches_oracle():
    N, C, sel, f = 160, 32, [4, 2, 1], 5.0 / 3.0
    p64, dec, tok, tgt = _setup(F32_CFG, 7, 2, N, torch.float32)
    _, g_ref = om.spaco_grads(F32_CFG, p64, tok, tgt, C, sel, f)
    _, g = dec.step(tok.to(DEV), tgt.to(DEV), C, selected=sel, factor=f)
    _compare(g_ref, g, 5e-4)
    # the compound factor really is exercised: with factor 1 the reference differs visibly
    _, g_one = om.spaco_grads(F32_CFG, p64, tok, tgt, C, sel, 1.0)
    assert max(float((g_one[n] - g_ref[n]).abs().max() / g_ref[n].abs().max()) for n in g_ref) > 1e-2


def test_seco_step_bf16_matmul_kernels():
    N, C = 256, 64
    p64, dec, tok, tgt = _setup(BF16_CFG, 9, 1, N, torch.bfloat16)
    _, g_ref = om.monolithic_grads(BF16_CFG, p64, tok, tgt)
    _, g = dec.step(tok.to(DEV), tgt.to(DEV), C)
    _compare(g_ref, g, 6e-2)


def test_spaco_step_bf16_matmul_kernels():
    N, C, sel, f = 320, 64, [4, 3, 0], 5.0 / 3.0
    p64, dec, tok, tgt = _setup(BF16_CFG, 11, 1, N, torch.bfloat16)
    _, g_ref = om.spaco_grads(BF16_CFG, p64, tok, tgt, C, sel, f)
    _, g = dec.step(tok.to(DEV), tgt.to(DEV), C, selected=sel, factor=f)
    _compare(g_ref, g, 6e-2)


@pytest.mark.parametrize("dtype,cfg", [(torch.float32, F32_CFG), (torch.bfloat16, BF16_CFG)])
def test_keeping_attention_outputs_gives_identical_gradients(dtype, cfg):
    """Stage 2 may take O and LSE from stage 1 instead of running the attention forward again: same values
    (deterministic kernels, same inputs), hence bit-identical gradients, for SeCO and SpaCO."""
    p64, dec, tok, tgt = _setup(cfg, 13, 1, 256, dtype)
    tok, tgt = tok.to(DEV), tgt.to(DEV)
    for kw in ({}, {"selected": [3, 1, 0], "factor": 4 / 3}):
        _, g_a = dec.step(tok, tgt, 64, **kw)
        g_a = {n: t.clone() for n, t in g_a.items()}
        _, g_b = dec.step(tok, tgt, 64, keep_attention_outputs=True, **kw)
        for n in g_a:
            assert torch.equal(g_a[n], g_b[n]), n


def test_whole_sequence_stage1_with_kept_outputs_matches_oracle():
    """Stage 1 as one plain forward over the whole sequence, stage 2 from its kept O / LSE: same gradients as the
    oracle's Alg. 1 / Alg. 2 (to the usual tolerance; the launches differ in shape from the chunked stage 1)."""
    N, C = 192, 32
    p64, dec, tok, tgt = _setup(F32_CFG, 15, 2, N, torch.float32)
    _, g_ref = om.monolithic_grads(F32_CFG, p64, tok, tgt)
    _, g = dec.step(tok.to(DEV), tgt.to(DEV), C, keep_attention_outputs=True, stage1_chunk_len=N)
    _compare(g_ref, g, 5e-4)
    sel, f = [5, 3, 0], 2.0
    _, g_ref = om.spaco_grads(F32_CFG, p64, tok, tgt, C, sel, f)
    _, g = dec.step(tok.to(DEV), tgt.to(DEV), C, selected=sel, factor=f, keep_attention_outputs=True, stage1_chunk_len=N)
    _compare(g_ref, g, 5e-4)
    # bf16 matrix-core kernels
    p64, dec, tok, tgt = _setup(BF16_CFG, 16, 1, 256, torch.bfloat16)
    _, g_ref = om.monolithic_grads(BF16_CFG, p64, tok, tgt)
    _, g = dec.step(tok.to(DEV), tgt.to(DEV), 64, keep_attention_outputs=True, stage1_chunk_len=256)
    _compare(g_ref, g, 6e-2)


@pytest.mark.parametrize("dtype,cfg,tol", [(torch.float32, F32_CFG, 5e-4), (torch.bfloat16, BF16_CFG, 6e-2)])
def test_column_weighted_dq_step_matches_oracle(dtype, cfg, tol):
    """Alg. 2 with, beyond the paper, a dQ that visits only some chunks, a different weight vector in every layer
    of every call (fixed here; a training loop would draw them)."""
    N, C, sel, f = 320, 64, [4, 3, 1, 0], 1.25
    p64, dec, tok, tgt = _setup(cfg, 13, 1, N, dtype)

    def wq(j, l):
        g = torch.Generator().manual_seed(1000 * j + l)
        w = [float(x) * 2.0 for x in (torch.rand(j, generator=g) < 0.5)] + [1.0]
        return w
    _, g_ref = om.spaco_grads(cfg, p64, tok, tgt, C, sel, f, dq_weights=wq)
    _, g = dec.step(tok.to(DEV), tgt.to(DEV), C, selected=sel, factor=f, dq_weights=wq)
    _compare(g_ref, g, tol)
    _, g_dense = om.spaco_grads(cfg, p64, tok, tgt, C, sel, f)
    assert max(float((g_dense[n] - g_ref[n]).abs().max() / g_ref[n].abs().max()) for n in g_ref) > 1e-2


@pytest.mark.parametrize("dtype,base_cfg,tol", [(torch.float32, F32_CFG, 5e-4), (torch.bfloat16, BF16_CFG, 6e-2)])
def test_step_with_rotary_embedding_matches_oracle(dtype, base_cfg, tol):
    """Queries rotated by rope_rotate, keys rotated on their way into the cache (kv_append_rope), the key gradient
    turned back at the read-out (kvgrad_readout_rope): SeCO against whole-sequence training, SpaCO against Alg. 2."""
    import dataclasses
    cfg = dataclasses.replace(base_cfg, rope_base=10000.0)
    N, C = 320, 64
    p64, dec, tok, tgt = _setup(cfg, 15, 1, N, dtype)
    _, g_ref = om.monolithic_grads(cfg, p64, tok, tgt)
    _, g = dec.step(tok.to(DEV), tgt.to(DEV), C, keep_attention_outputs=True)
    _compare(g_ref, g, tol)
    _, g_plain = om.monolithic_grads(base_cfg, p64, tok, tgt)          # the embedding is really there
    assert max(float((g_plain[n] - g_ref[n]).abs().max() / g_ref[n].abs().max()) for n in g_ref) > 1e-2
    sel, f = [4, 2, 1], 5.0 / 3.0
    _, g_ref = om.spaco_grads(cfg, p64, tok, tgt, C, sel, f)
    _, g = dec.step(tok.to(DEV), tgt.to(DEV), C, selected=sel, factor=f)
    _compare(g_ref, g, tol)


def test_seco_step_with_the_transposed_backward_order_matches_whole_sequence_training():
    """Alg. 1 with every layer's attention backward in the transposed order (seco_chunk_attn_bwd_gather): parameter
    gradients against ordinary whole-sequence training, ragged last chunk included, and against the accumulating
    order to rounding."""
    cfg, tol = BF16_CFG, 6e-2
    N, C = 448, 128
    p64, dec, tok, tgt = _setup(cfg, 19, 2, N, torch.bfloat16)
    _, g_ref = om.monolithic_grads(cfg, p64, tok, tgt)
    loss_t, g_t = dec.step(tok.to(DEV), tgt.to(DEV), C, transposed_backward=True)
    _compare(g_ref, g_t, tol)
    loss_a, g_a = dec.step(tok.to(DEV), tgt.to(DEV), C)
    assert loss_t == loss_a
    for n in g_a:
        d = (g_t[n].float() - g_a[n].float()).abs().max() / g_a[n].float().abs().max()
        assert float(d) < 2e-2, (n, float(d))


def test_spaco_step_with_the_transposed_backward_order_matches_oracle():
    """Alg. 2 with every layer's attention backward in the transposed order (row weights 1 / factor / 0)."""
    cfg, tol = BF16_CFG, 6e-2
    N, C = 320, 64
    p64, dec, tok, tgt = _setup(cfg, 23, 1, N, torch.bfloat16)
    sel, f = [4, 2, 1], 5.0 / 3.0
    _, g_ref = om.spaco_grads(cfg, p64, tok, tgt, C, sel, f)
    _, g = dec.step(tok.to(DEV), tgt.to(DEV), C, selected=sel, factor=f, transposed_backward=True)
    _compare(g_ref, g, tol)
