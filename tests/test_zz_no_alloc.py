"""GPU test of seco_chunk_attn_bwd_noalloc, the backward entry point for callers that cannot allocate: its
workspace is a device array inside the library.  It runs the kernels of seco_chunk_attn_bwd with the same launch
plan, so its outputs must equal that entry point's bit for bit (and therefore meet the same oracle tolerances);
checked on two calls in a row, the second on a smaller input, whose scratch use overlaps what the first left."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2505_16710_amd as seco
from oracle import attention as A
from workloads import small_layer

from hip_driver import DEV, max_rel, to_dev, to_host

pytestmark = pytest.mark.gpu


def _both(x, j, Cn, dtype):
    D = x["q"].shape[-1]
    s = 1 / np.sqrt(D)
    q, k, v, do = (to_dev(x[n], dtype) for n in ("q", "k", "v", "do"))
    sl = slice(j * Cn, (j + 1) * Cn)
    qc, doc = q[:, :, sl], do[:, :, sl]
    o, lse = seco.seco_chunk_attn_fwd(qc, k, v, j * Cn, s, o=torch.empty_like(q)[:, :, sl])
    base = torch.randn(k.shape, dtype=torch.float32, device=DEV)       # the buffers are accumulated into
    gk_a, gv_a, gk_b, gv_b = base.clone(), (2 * base).clone(), base.clone(), (2 * base).clone()
    dq_a = seco.seco_chunk_attn_bwd(qc, k, v, o, lse, doc, gk_a, gv_a, j * Cn, s, d_q=torch.empty_like(q)[:, :, sl])
    dq_b = torch.full_like(q, float("nan"))[:, :, sl]
    seco.seco_chunk_attn_bwd_noalloc(qc, k, v, o, lse, doc, dq_b, gk_b, gv_b, j * Cn, s)
    torch.cuda.synchronize()
    assert torch.equal(dq_a, dq_b) and torch.equal(gk_a, gk_b) and torch.equal(gv_a, gv_b)
    o_ref, lse_ref = A.chunk_attn_fwd(x["q"][:, :, sl], x["k"], x["v"], j * Cn, s)
    dq_ref, dk_ref, dv_ref = A.chunk_attn_bwd(x["q"][:, :, sl], x["k"], x["v"], o_ref, lse_ref, x["do"][:, :, sl],
                                              j * Cn, s)
    tol = 2e-2 if dtype == "bf16" else 1e-4
    b64 = to_host(base)[:, :, :(j + 1) * Cn]
    assert max_rel(to_host(dq_b), dq_ref) <= tol
    assert max_rel(to_host(gk_b)[:, :, :(j + 1) * Cn] - b64, dk_ref) <= tol
    assert max_rel(to_host(gv_b)[:, :, :(j + 1) * Cn] - 2 * b64, dv_ref) <= tol


def test_noalloc_backward_equals_the_workspace_entry_point_twice_in_a_row():
    # first call: 8 (batch, KV head) units x 12 column tiles, the last ones shared out by query head (partials in
    # the scratch array), 4-wavefront direct dQ; second call: a smaller, short-chunk shape whose split dQ partials
    # and row statistics land where the first call's data were
    _both(small_layer(91, 2, 16, 4, 1536, 128, "bf16"), 2, 512, "bf16")
    _both(small_layer(92, 1, 4, 2, 640, 128, "bf16"), 4, 128, "bf16")
    _both(small_layer(93, 1, 4, 4, 256, 64, "f32"), 1, 128, "f32")


def test_noalloc_backward_rejects_what_does_not_fit():
    d = seco.binding.SecoDesc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim = 1, 64, 8, 128
    d.chunk_len, d.q_start, d.dtype, d.softmax_scale = 1 << 15, 0, seco.binding.SECO_BF16, 0.088
    for name in ("q_stride", "o_stride", "kv_stride", "g_stride"):
        setattr(d, name, (C.c_int64 * 3)(64 << 22, 1 << 22, 128))
    assert seco.seco_workspace_bytes(d, seco.binding.SECO_OP_BWD) > seco.binding.STATIC_SCRATCH_BYTES
    fake = C.c_void_p(0x1000)
    rc = seco.load_library().seco_chunk_attn_bwd_noalloc(C.byref(d), fake, fake, fake, fake, fake, fake, fake, fake,
                                                         fake, None)
    assert rc == -10
