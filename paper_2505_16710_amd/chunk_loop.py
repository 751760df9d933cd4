"""SeCO / SpaCO training step of a small decoder, driven through the C ABI (Alg. 1 and Alg. 2 end to end).

The attention of every layer, its backward and the whole KV-gradient relay run in the HIP library:
each layer owns a KV cache and a pair of fp32 KV-gradient buffers that live for the whole step, the
forward of a chunk is `seco_chunk_attn_fwd` against the cache, its backward is `seco_chunk_attn_bwd` /
`spaco_chunk_attn_bwd`, which deposits the chunk's dK/dV on every visible cache row, and the gradient
handed to the chunk's own recomputed K/V is simply the chunk's rows of those buffers (they hold what
the later chunks deposited plus the chunk's own diagonal block: the relay of Alg. 1, `m_i.grad <-
m'_i.grad`), read out by `kvgrad_readout`; new keys / values enter the cache through `kv_append`.  Under SpaCO the deposits on earlier selected chunks carry the compensation
factor, so a chain through p caches is scaled by factor^p (Sec. 5).

The projections, norms, MLP and loss around the attention are ordinary PyTorch GPU ops with autograd
(library GEMMs); only one chunk's graph is alive at a time, as in the paper.  There is no CPU path.

Model (fixed here so that a checker can build the same function): pre-norm decoder, RMSNorm with
eps 1e-6, grouped-query causal attention (optionally with rotary position embedding), MLP x + silu(h W1) W2, final
RMSNorm, linear head, cross-entropy summed over tokens.  Parameter names: emb, head, norm_f and
l{i}.norm1, l{i}.norm2, l{i}.wq, l{i}.wk, l{i}.wv, l{i}.wo, l{i}.w1, l{i}.w2, all stored [in, out].
"""
from __future__ import annotations

import torch
import torch.nn.functional as F

from . import binding as _b


class LayerState:
    """KV cache (storage dtype) and fp32 KV-gradient buffers of one layer, [B, Hkv, N, D]."""

    def __init__(self, B, Hkv, N, D, dtype, device):
        self.k = torch.zeros(B, Hkv, N, D, dtype=dtype, device=device)
        self.v = torch.zeros_like(self.k)
        self.gk = torch.empty(B, Hkv, N, D, dtype=torch.float32, device=device)
        self.gv = torch.empty_like(self.gk)
        self.kept = {}      # q_start -> (O, LSE) of stage 1, when attention outputs are kept for stage 2
        self.gather = None  # transposed backward order: (Q, dO, O, dQ of the layer, row statistics)
        self.gather_rows = None   # ... under Alg. 2: (selected chunks, factor, chunk length, number of chunks)

    def enable_gather(self, B, Hq, N, D, dtype, device):
        """Buffers of the transposed backward order: the layer's Q, dO, O and dQ over the whole sequence,
        [B, Hq, N, D] each (a call takes row ranges of them, so all share one set of strides), and the per-row
        statistics the dK/dV kernel reads, fp32 [2, B, Hq, N rounded up to 4]."""
        self.gather = tuple(torch.empty(B, Hq, N, D, dtype=dtype, device=device) for _ in range(4)) + (
            torch.empty(2, B, Hq, (N + 3) // 4 * 4, dtype=torch.float32, device=device),)


class ChunkAttention(torch.autograd.Function):
    """Attention of one chunk against a layer's cache; backward deposits into the layer's KV-gradient buffers."""

    @staticmethod
    def forward(ctx, q, k_new, v_new, state, q_start, scale, weights, weight_chunk_len, keep, dq_weights=None,
                rope_base=None):
        # keep: None = always compute; "store" = stage 1, remember (O, LSE); "reuse" = stage 2, take them back
        # (the rebuilt chunk has the same inputs and the kernels are deterministic, so the values are identical and
        # the cache rows already hold this chunk's K/V)
        if keep == "reuse":
            # the span of stage 1 that holds this chunk's rows (the chunk itself, or a longer span to cut from)
            s0, (o_all, lse_all) = max((kv for kv in state.kept.items() if kv[0] <= q_start), key=lambda kv: kv[0])
            a, b = q_start - s0, q_start - s0 + q.shape[2]
            if a == 0 and b == o_all.shape[2]:
                o, lse = o_all, lse_all
            else:
                o, lse = o_all[:, :, a:b].contiguous(), lse_all[:, :, a:b].contiguous()
        else:
            _b.kv_append(k_new, v_new, state.k, state.v, q_start, rope_base=rope_base)   # keys are cached rotated
            o, lse = _b.seco_chunk_attn_fwd(q, state.k, state.v, q_start, scale,
                                            o=torch.empty(q.shape, dtype=q.dtype, device=q.device))
            if keep == "store":
                state.kept[q_start] = (o, lse)
        ctx.save_for_backward(q, o, lse)
        ctx.state, ctx.q_start, ctx.scale, ctx.weights, ctx.wlen = state, q_start, scale, weights, weight_chunk_len
        ctx.dq_weights, ctx.rope_base = dq_weights, rope_base
        return o

    @staticmethod
    def backward(ctx, d_o):
        q, o, lse = ctx.saved_tensors
        st, s0, C = ctx.state, ctx.q_start, q.shape[2]
        d_o = d_o.contiguous()
        if st.gather is not None:
            # transposed order (Alg. 1 only): this chunk's finished gK/gV rows from its own and every later chunk's
            # query rows, whose Q and dO the layer has kept; nothing is added to earlier rows
            q_all, do_all, o_all, dq_all, stats = st.gather
            q_all[:, :, s0:s0 + C] = q
            do_all[:, :, s0:s0 + C] = d_o
            o_all[:, :, s0:s0 + C] = o
            row_w, wlen = None, None
            if st.gather_rows is not None:      # Alg. 2: 1 on the chunk's own rows, the factor on later selected chunks
                sel, factor, wlen, k = st.gather_rows
                j = s0 // wlen
                row_w = _b.spaco_gather_row_weights(sel, j, k, factor)
            d_q = _b.seco_chunk_attn_bwd_gather(q_all[:, :, s0:], st.k, st.v, o_all[:, :, s0:s0 + C], lse,
                                                do_all[:, :, s0:], st.gk, st.gv, s0, ctx.scale, C, stats,
                                                d_q=dq_all[:, :, s0:s0 + C], row_weight=row_w,
                                                weight_chunk_len=wlen).contiguous()
        elif ctx.weights is None and ctx.dq_weights is None:
            d_q = _b.seco_chunk_attn_bwd(q, st.k, st.v, o, lse, d_o, st.gk, st.gv, s0, ctx.scale)
        else:
            n_chunks = len(ctx.dq_weights) if ctx.weights is None else len(ctx.weights)
            w = [1.0] * n_chunks if ctx.weights is None else ctx.weights
            d_q = _b.spaco_chunk_attn_bwd(q, st.k, st.v, o, lse, d_o, st.gk, st.gv, s0, ctx.scale,
                                          w, ctx.wlen, dq_weight=ctx.dq_weights)
        d_k, d_v = _b.kvgrad_readout(st.gk, st.gv, s0, C, q.dtype, rope_base=ctx.rope_base)
        return d_q, d_k, d_v, None, None, None, None, None, None, None, None


class Rope(torch.autograd.Function):
    """Rotary position embedding of the chunk's queries (rope_rotate); the gradient is turned back."""

    @staticmethod
    def forward(ctx, x, pos_start, base):
        ctx.pos_start, ctx.base = pos_start, base
        return _b.rope_rotate(x.contiguous(), pos_start, base)

    @staticmethod
    def backward(ctx, d_out):
        return _b.rope_rotate(d_out.contiguous(), ctx.pos_start, ctx.base, inverse=True), None, None


def _rmsnorm(x, g):
    xf = x.float()
    return (xf * torch.rsqrt((xf * xf).mean(dim=-1, keepdim=True) + 1e-6)).to(x.dtype) * g


class ChunkedDecoder:
    """Holds the parameters (dict name -> leaf tensor on the GPU) and runs SeCO / SpaCO steps."""

    def __init__(self, params, n_layers, n_q_heads, n_kv_heads, head_dim, rope_base=None):
        self.p = params
        self.rope_base = rope_base      # rotary embedding of queries and keys (keys are cached rotated), or None
        self.n_layers, self.Hq, self.Hkv, self.D = n_layers, n_q_heads, n_kv_heads, head_dim
        self.scale = float(head_dim) ** -0.5
        _b.load_library()          # fail here, loudly, if the HIP library has not been built

    def _chunk(self, tokens, targets, q_start, states, weights, wlen, keep=None, dq_weights=None):
        p, B, C = self.p, tokens.shape[0], tokens.shape[1]
        x = p["emb"][tokens]
        for l in range(self.n_layers):
            h = _rmsnorm(x, p[f"l{l}.norm1"])
            q = (h @ p[f"l{l}.wq"]).view(B, C, self.Hq, self.D).transpose(1, 2)
            k = (h @ p[f"l{l}.wk"]).view(B, C, self.Hkv, self.D).transpose(1, 2)
            v = (h @ p[f"l{l}.wv"]).view(B, C, self.Hkv, self.D).transpose(1, 2)
            if self.rope_base is not None:
                q = Rope.apply(q, q_start, self.rope_base)
            o = ChunkAttention.apply(q, k, v, states[l], q_start, self.scale, weights, wlen, keep,
                                     None if dq_weights is None else dq_weights[l], self.rope_base)
            x = x + o.transpose(1, 2).reshape(B, C, self.Hq * self.D) @ p[f"l{l}.wo"]
            h = _rmsnorm(x, p[f"l{l}.norm2"])
            x = x + F.silu(h @ p[f"l{l}.w1"]) @ p[f"l{l}.w2"]
        logits = _rmsnorm(x, p["norm_f"]) @ p["head"]
        return F.cross_entropy(logits.reshape(B * C, -1).float(), targets.reshape(B * C), reduction="sum")

    def step(self, tokens, targets, chunk_len, selected=None, factor=1.0, keep_attention_outputs=False,
             stage1_chunk_len=None, dq_weights=None, transposed_backward=False):
        """One SeCO step (selected is None: Alg. 1) or SpaCO step (Alg. 2, `selected` chunk indices,
        relay factor `factor`).  Returns (sum of the chunk losses from stage 1, {name: gradient}).

        keep_attention_outputs: stage 1 keeps every layer's O and LSE (2 + 4/D bytes per query element: with 288 GB
        of HBM that is cheap), and the rebuilt chunks of stage 2 take them back instead of running the attention
        forward again; the gradients are bit-identical to the recomputing schedule.
        stage1_chunk_len: chunk length of the inference pass only (default chunk_len).  Stage 1 holds no graph, so on a
        GPU with room for one layer's activations of the whole sequence it can run as a single chunk (a plain
        prefill); together with keep_attention_outputs, stage 2 then launches backward kernels only.  The caches
        and kept outputs are then produced by differently shaped launches, so gradients agree with the chunked
        stage 1 to rounding, not bit for bit.
        dq_weights: optional callable (chunk j, layer l) -> one non-negative weight per chunk 0..j (or None): the dQ
        of that attention call visits only the chunks with a non-zero weight and scales their terms
        (spaco_chunk_attn_bwd_sparse_dq; not part of the paper).  For unbiased gradients the weights must have
        expectation 1 and be drawn independently for every layer of a call.
        transposed_backward: the attention backward in the transposed order (seco_chunk_attn_bwd_gather, under Alg. 2
        spaco_chunk_attn_bwd_gather; bf16 parameters): same gradients up to the order of summation."""
        p = self.p
        B, N = tokens.shape
        dtype, dev = p["emb"].dtype, p["emb"].device
        starts = list(range(0, N, chunk_len))
        states = [LayerState(B, self.Hkv, N, self.D, dtype, dev) for _ in range(self.n_layers)]
        if transposed_backward:
            if dq_weights is not None or dtype != torch.bfloat16:
                raise ValueError("the transposed backward order takes bf16 parameters and the exact dQ")
            if selected is not None and chunk_len % 64 != 0:
                raise ValueError("Alg. 2 in the transposed order needs a chunk length that is a multiple of 64")
            for st in states:
                st.enable_gather(B, self.Hq, N, self.D, dtype, dev)
                if selected is not None:
                    st.gather_rows = ({int(i) for i in selected}, float(factor), chunk_len, len(starts))
        for t in p.values():
            t.grad = None
        total = torch.zeros((), dtype=torch.float32, device=dev)
        c1 = stage1_chunk_len or chunk_len
        with torch.no_grad():                                           # stage 1: inference over all chunks
            for s0 in range(0, N, c1):
                total += self._chunk(tokens[:, s0:s0 + c1], targets[:, s0:s0 + c1], s0, states, None, 0,
                                     "store" if keep_attention_outputs else None)
        for st in states:
            _b.kvgrad_zero(st.gk, st.gv)
        if selected is None:
            order = list(range(len(starts) - 1, -1, -1))
        else:
            order = sorted({int(i) for i in selected}, reverse=True)
        for j in order:                                                 # stage 2: rebuild + back-propagate
            w = None if selected is None else _b.spaco_chunk_weights(order, j, factor)
            s0 = starts[j]
            wq = None if dq_weights is None else [dq_weights(j, l) for l in range(self.n_layers)]
            loss = self._chunk(tokens[:, s0:s0 + chunk_len], targets[:, s0:s0 + chunk_len], s0, states, w, chunk_len,
                               "reuse" if keep_attention_outputs else None, wq)
            loss.backward()
        grads = {n: (t.grad if t.grad is not None else torch.zeros_like(t)) for n, t in p.items()}
        return float(total), grads
