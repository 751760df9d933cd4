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
