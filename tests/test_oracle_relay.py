"""Pins for oracle/relay.py (appendix listing: update_kv_cache, grad_hook, copy_grad)."""
import numpy as np
import torch

from oracle import relay as R


def test_append_equals_concatenation_of_the_chunks():
    rng = np.random.default_rng(0)
    B, H, D, C = 2, 3, 8, 5
    chunks_k = [rng.standard_normal((B, H, C, D)) for _ in range(4)]
    chunks_v = [rng.standard_normal((B, H, C, D)) for _ in range(4)]
    k = np.full((B, H, 4 * C, D), np.nan)
    v = np.full((B, H, 4 * C, D), np.nan)
    for j in range(4):
        k, v = R.kv_append(k, v, chunks_k[j], chunks_v[j], j * C)
        # what chunk j attends over is the concatenation of everything appended so far (the listing's return value)
        np.testing.assert_array_equal(k[:, :, :(j + 1) * C], np.concatenate(chunks_k[:j + 1], axis=2))
        np.testing.assert_array_equal(v[:, :, :(j + 1) * C], np.concatenate(chunks_v[:j + 1], axis=2))
        assert np.isnan(k[:, :, (j + 1) * C:]).all()          # later rows untouched


def test_bf16_rounding_against_torch_and_ties():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(100000) * 10.0 ** rng.integers(-20, 20, 100000)).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(R.round_fp32_to_bf16(x), ref)
    # exact ties: 1 + 2^-8 lies half-way between 1 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 -> 1 + 2^-6
    assert R.round_fp32_to_bf16(np.float32(1 + 2 ** -8)) == np.float32(1.0)
    assert R.round_fp32_to_bf16(np.float32(1 + 3 * 2 ** -8)) == np.float32(1 + 2 ** -6)
    assert R.round_fp32_to_bf16(np.float32(-0.0)).tobytes() == np.float32(-0.0).tobytes()


def test_readout_and_hook():
    rng = np.random.default_rng(2)
    g = rng.standard_normal((1, 2, 12, 8)).astype(np.float32)
    np.testing.assert_array_equal(R.kvgrad_readout(g, 4, 8, 1.0, "f32"), g[:, :, 4:8])
    np.testing.assert_array_equal(R.kvgrad_readout(g, 4, 8, 4.0, "f32"), 4 * g[:, :, 4:8])      # power of two: exact
    out = R.kvgrad_readout(g, 0, 12, 16 / 3, "bf16")
    exact = g.astype(np.float64) * (16 / 3)
    assert np.abs(out - exact).max() <= 2.0 ** -8 * np.abs(exact).max()                        # half an ulp of bf16 + fp32 product
    # the hook: a tensor that feeds a loss directly and through a detached copy whose gradient is handed over
    x = torch.randn(5, dtype=torch.float64, requires_grad=True)
    ck = x.detach().clone().requires_grad_()
    (3 * ck.sin()).sum().backward()                      # gradient collected on the checkpoint
    own = torch.autograd.grad((x ** 2).sum(), x)[0]
    hooked = R.hooked_gradient(own.numpy(), ck.grad.numpy(), 2.5)
    np.testing.assert_allclose(hooked, (2 * x + 2.5 * 3 * x.cos()).detach().numpy(), rtol=1e-14)
