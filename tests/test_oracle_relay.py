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


# ---- rotary position embedding of the keys (append) and of their gradient (read-out) ------------------------------

def test_rope_is_a_plane_rotation_by_position_times_frequency():
    rng = np.random.default_rng(0)
    # head_dim 2: one pair, frequency 1: the textbook rotation matrix
    x = rng.standard_normal((1, 1, 5, 2))
    got = R.rope_rotate(x, 3, 10000.0)
    for r in range(5):
        p = 3 + r
        want = np.array([[np.cos(p), -np.sin(p)], [np.sin(p), np.cos(p)]]) @ x[0, 0, r]
        assert np.abs(got[0, 0, r] - want).max() < 1e-14
    # general head_dim: pair (i, i + D/2) as a complex number times exp(i * p * base^(-2i/D))
    B, H, C, D, pos0, base = 2, 3, 7, 16, 11, 500000.0
    x = rng.standard_normal((B, H, C, D))
    z = x[..., :D // 2] + 1j * x[..., D // 2:]
    freq = np.array([base ** (-(2 * i) / D) for i in range(D // 2)])
    w = z * np.exp(1j * (pos0 + np.arange(C))[:, None] * freq[None, :])
    got = R.rope_rotate(x, pos0, base)
    assert np.abs(got[..., :D // 2] - w.real).max() < 1e-12 and np.abs(got[..., D // 2:] - w.imag).max() < 1e-12
    assert np.abs(R.rope_rotate(x, 0, base)[:, :, 0] - x[:, :, 0]).max() == 0.0            # position 0: identity
    assert np.abs(R.rope_angles([1], D, base)[0, 0] - 1.0) < 1e-15                          # first pair turns 1 rad per position


def test_rope_inverse_adjoint_and_relative_position():
    rng = np.random.default_rng(1)
    B, H, C, D, base = 1, 2, 6, 8, 10000.0
    x, y = rng.standard_normal((B, H, C, D)), rng.standard_normal((B, H, C, D))
    rx = R.rope_rotate(x, 40, base)
    assert np.abs(R.rope_rotate(rx, 40, base, inverse=True) - x).max() < 1e-13
    assert np.abs((rx ** 2).sum(-1) - (x ** 2).sum(-1)).max() < 1e-12                       # lengths are kept
    # the read-out applies the transpose: <R x, y> = <x, R^T y>
    assert abs((rx * y).sum() - (x * R.rope_rotate(y, 40, base, inverse=True)).sum()) < 1e-12
    # scores depend on the distance only: <R_m q, R_n k> = <R_(m-n) q, k>
    q, k = rng.standard_normal((1, 1, 1, D)), rng.standard_normal((1, 1, 1, D))
    for m, n in ((5, 2), (100, 97), (7, 7)):
        lhs = (R.rope_rotate(q, m, base) * R.rope_rotate(k, n, base)).sum()
        rhs = (R.rope_rotate(q, m - n, base) * k).sum()
        assert abs(lhs - rhs) < 1e-12


def test_append_and_readout_with_rope_round_to_the_storage_type():
    rng = np.random.default_rng(2)
    B, H, N, D, C, r0, base = 1, 2, 12, 8, 4, 8, 10000.0
    kc, vc = np.zeros((B, H, N, D), np.float32), np.zeros((B, H, N, D), np.float32)
    kn, vn = rng.standard_normal((B, H, C, D)).astype(np.float32), rng.standard_normal((B, H, C, D)).astype(np.float32)
    for dtype in ("f32", "bf16"):
        k2, v2 = R.kv_append_rope(kc, vc, kn, vn, r0, base, dtype)
        exact = R.rope_rotate(kn, r0, base)
        tol = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -23
        assert np.abs(k2[:, :, r0:r0 + C] - exact).max() <= tol * np.abs(exact).max()
        assert np.array_equal(v2[:, :, r0:r0 + C], vn) and not k2[:, :, :r0].any()
        g = rng.standard_normal((B, H, N, D)).astype(np.float32)
        dk, dv = R.kvgrad_readout_rope(g, g, r0, r0 + C, 1.5, base, dtype)
        want = R.rope_rotate(g[:, :, r0:r0 + C].astype(np.float64) * 1.5, r0, base, inverse=True)
        assert np.abs(dk - want).max() <= 2 * tol * np.abs(want).max()
        assert np.array_equal(dv, R.kvgrad_readout(g, r0, r0 + C, 1.5, dtype))
