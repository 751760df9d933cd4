"""Helpers for the GPU tests: move seeded host arrays to the device, drive the C ABI through
the binding in the method's call order, and bring results back as fp64 NumPy arrays."""
import numpy as np
import torch

import paper_2505_16710_amd as seco
from workloads import f32_to_bf16_bits

DEV = "cuda:0"


def to_dev(x32, dtype):
    """fp32 host array (already storage-rounded) -> device tensor of the storage type."""
    if dtype == "bf16":
        bits = f32_to_bf16_bits(x32)
        return torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x32, dtype=np.float32)).to(DEV)


def to_host(t):
    return t.detach().to(torch.float64).cpu().numpy()


def chunk_list(N, C):
    return [(s, min(C, N - s)) for s in range(0, N, C)]


def run_layer(x, chunk_len, scale, dtype, selected=None, factor=1.0, weights_fn=None, dq_weights_fn=None):
    """SeCO (selected is None) or SpaCO schedule at one attention layer on the GPU.

    x: dict q, k, v, do of fp32 host arrays [B,H,N,D].  Returns dict of fp64 arrays
    o, lse (from the stage-1 forward of every chunk), dq, gk, gv.
    """
    q, k, v, do = (to_dev(x[n], dtype) for n in ("q", "k", "v", "do"))
    B, Hq, N, D = q.shape
    o = torch.empty_like(q)
    lse = torch.empty((B, Hq, N), dtype=torch.float32, device=DEV)
    dq = torch.zeros_like(q)
    gk = torch.full(k.shape, float("nan"), dtype=torch.float32, device=DEV)
    gv = torch.full(k.shape, float("nan"), dtype=torch.float32, device=DEV)
    chunks = chunk_list(N, chunk_len)
    for s0, c in chunks:                                   # stage 1
        oc, lc = seco.seco_chunk_attn_fwd(q[:, :, s0:s0 + c], k, v, s0, scale)
        o[:, :, s0:s0 + c] = oc
        lse[:, :, s0:s0 + c] = lc
    seco.kvgrad_zero(gk, gv)
    order = range(len(chunks) - 1, -1, -1) if selected is None else sorted(selected, reverse=True)
    for j in order:                                        # stage 2
        s0, c = chunks[j]
        qc = q[:, :, s0:s0 + c]
        oc, lc = seco.seco_chunk_attn_fwd(qc, k, v, s0, scale)
        doc = do[:, :, s0:s0 + c].contiguous()
        oc = oc.contiguous()
        if selected is None:
            dqc = seco.seco_chunk_attn_bwd(qc, k, v, oc, lc, doc, gk, gv, s0, scale)
        else:
            w = weights_fn(j) if weights_fn else seco.spaco_chunk_weights(selected, j, factor)
            wq = dq_weights_fn(j) if dq_weights_fn else None
            dqc = seco.spaco_chunk_attn_bwd(qc, k, v, oc, lc, doc, gk, gv, s0, scale, w, chunk_len, dq_weight=wq)
        dq[:, :, s0:s0 + c] = dqc
    torch.cuda.synchronize()
    return {"o": to_host(o), "lse": to_host(lse), "dq": to_host(dq), "gk": to_host(gk), "gv": to_host(gv)}


def max_rel(x, ref):
    """max |x - ref| / max |ref| per tensor."""
    return float(np.abs(x - ref).max() / max(np.abs(ref).max(), 1e-30))


def max_rel_per_head(x, ref):
    """The same error normalised per (batch, head) slice, worst slice: a head (or a KV head's gradient rows) of small
    magnitude cannot hide behind a large one.  Slices whose reference is identically zero must be zero."""
    x, ref = np.asarray(x, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    if x.ndim < 3:
        return max_rel(x, ref)
    ax = tuple(range(2, x.ndim))
    err = np.abs(x - ref).max(axis=ax)
    top = np.abs(ref).max(axis=ax)
    if (top == 0).any():
        assert not err[top == 0].any()
        top = np.where(top == 0, 1.0, top)
    return float((err / top).max())


def max_rel_floor(x, ref, floor=1e-3):
    """Element-wise relative error with an absolute floor: max |x - ref| / max(|ref|, floor * max |ref|)."""
    x, ref = np.asarray(x, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    den = np.maximum(np.abs(ref), floor * max(np.abs(ref).max(), 1e-30))
    return float((np.abs(x - ref) / den).max())
