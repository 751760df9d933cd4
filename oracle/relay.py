"""KV-cache append and KV-gradient hand-over (the three helper functions of the paper's appendix listing), oracle.

TEST INFRASTRUCTURE ONLY (see the package docstring).

The listing keeps the cache as a growing list and concatenates on every call; the quantities themselves are:

  * cache update: after chunk j has been appended, the keys / values a chunk attends over are the concatenation
    of the earlier chunks' and its own (`update_kv_cache` returns exactly that concatenation);
  * gradient hook: what reaches a recomputed key / value tensor is its own gradient plus `scaler` times the
    gradient collected on the checkpoint it replaces (`grad_hook`: grad + base * scaler; `copy_grad` installs the
    hook for every layer).  Alg. 2 uses scaler = k/t, Alg. 1 scaler = 1.

Here the cache is one array over the whole sequence, so the first is a row-range copy and the second a row-range
read-out; both are written with plain NumPy and no shared code with the HIP path.
"""
from __future__ import annotations

import numpy as np


def kv_append(k_cache, v_cache, k_new, v_new, row_begin):
    """Cache after appending the chunk whose first global row is row_begin: arrays [B, Hkv, N, D] (copied)."""
    k_out, v_out = np.array(k_cache, copy=True), np.array(v_cache, copy=True)
    c = k_new.shape[2]
    k_out[:, :, row_begin:row_begin + c] = k_new
    v_out[:, :, row_begin:row_begin + c] = v_new
    return k_out, v_out


def round_fp32_to_bf16(x):
    """fp32 -> bfloat16 by round-to-nearest, ties to even; returned as fp32 values that bf16 represents exactly."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    return r.astype(np.uint32).view(np.float32)


def kvgrad_readout(g, row_begin, row_end, scaler, dtype):
    """scaler * g[rows] in fp32 arithmetic, rounded to the storage type ("f32" | "bf16"): the `base * scaler`
    term of the gradient hook, for the rows of one chunk.  g: fp32 [B, Hkv, N, D]."""
    prod = (np.asarray(g, dtype=np.float32)[:, :, row_begin:row_end] * np.float32(scaler)).astype(np.float32)
    return round_fp32_to_bf16(prod) if dtype == "bf16" else prod


def hooked_gradient(own_grad, checkpoint_grad, scaler):
    """grad + base * scaler (the hook itself), fp64."""
    return np.asarray(own_grad, dtype=np.float64) + np.asarray(checkpoint_grad, dtype=np.float64) * float(scaler)


# ---- rotary position embedding on the way into the cache and out of the gradient buffer --------------------------
# Not part of the paper (its model code is not shown); LLaMA-3, the model of its experiments, rotates queries and
# keys before attention (RoFormer, Su et al. 2021, in the "rotate-half" pairing of the LLaMA code): the pair
# (x[i], x[i + D/2]), i < D/2, of the row at sequence position p turns by the angle p * base^(-2 i / D).  Keys are
# stored rotated, so the append applies the rotation and the gradient read-out its transpose (the inverse turn).

def rope_angles(positions, D, base):
    """theta[p, i] = positions[p] * base^(-2 i / D), i = 0 .. D/2 - 1 (fp64)."""
    i = np.arange(D // 2, dtype=np.float64)
    return np.asarray(positions, dtype=np.float64)[:, None] * np.power(float(base), -2.0 * i / D)[None, :]


def rope_rotate(x, pos0, base, inverse=False):
    """x [B, H, C, D] (fp64), row r at position pos0 + r; inverse=True turns the other way (the transpose)."""
    x = np.asarray(x, dtype=np.float64)
    C, D = x.shape[2], x.shape[3]
    th = rope_angles(pos0 + np.arange(C), D, base)
    cos, sin = np.cos(th), np.sin(th) * (-1.0 if inverse else 1.0)
    a, b = x[..., :D // 2], x[..., D // 2:]
    return np.concatenate([a * cos - b * sin, b * cos + a * sin], axis=-1)


def _to_storage(x64, dtype):
    x32 = np.asarray(x64, dtype=np.float64).astype(np.float32)          # fp64 -> fp32 -> storage type, as the kernels do
    return round_fp32_to_bf16(x32) if dtype == "bf16" else x32


def kv_append_rope(k_cache, v_cache, k_new, v_new, row_begin, base, dtype):
    """kv_append with the keys rotated for their positions row_begin + r and rounded to the storage type."""
    k_rot = _to_storage(rope_rotate(k_new, row_begin, base), dtype)
    return kv_append(k_cache, v_cache, k_rot, v_new, row_begin)


def kvgrad_readout_rope(gk, gv, row_begin, row_end, scaler, base, dtype):
    """Gradient handed to a chunk's un-rotated keys and its values: the key part of kvgrad_readout turned back."""
    prod = (np.asarray(gk, dtype=np.float32)[:, :, row_begin:row_end] * np.float32(scaler)).astype(np.float32)
    d_k = _to_storage(rope_rotate(prod, row_begin, base, inverse=True), dtype)
    return d_k, kvgrad_readout(gv, row_begin, row_end, scaler, dtype)
