"""ctypes binding of include/seco.h: argument marshalling only.

Tensor arguments are torch tensors on the GPU, laid out [batch, head, row, head_dim] with a
contiguous last dimension (any outer strides).  The functions build the `seco_desc`, pass
raw device pointers and the current HIP stream, and raise SecoError on a non-zero status.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# SECO_LIBRARY overrides the path (e.g. to try a library built with other tile parameters)
_LIB_PATH = os.environ.get("SECO_LIBRARY") or os.path.join(_HERE, "libseco_hip.so")
_lib = None

SECO_F32, SECO_BF16 = 0, 1
SECO_OP_FWD, SECO_OP_BWD = 0, 1


class SecoDesc(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("chunk_len", C.c_int32), ("q_start", C.c_int32), ("dtype", C.c_int32), ("softmax_scale", C.c_float),
        ("q_stride", C.c_int64 * 3), ("o_stride", C.c_int64 * 3),
        ("kv_stride", C.c_int64 * 3), ("g_stride", C.c_int64 * 3),
    ]


class SecoError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {seco_strerror(status)} (status {status})")


def library_path():
    return _LIB_PATH


def load_library():
    """Load libseco_hip.so (built by paper_2505_16710_amd.build); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} not found: run `python -m paper_2505_16710_amd.build` "
                          "(there is no fallback path)")
    lib = C.CDLL(_LIB_PATH)
    vp, fp, i32, i64, sz = C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    dp = C.POINTER(SecoDesc)
    lib.seco_chunk_attn_fwd.argtypes = [dp, vp, vp, vp, vp, fp, vp, sz, vp]
    lib.seco_chunk_attn_bwd.argtypes = [dp, vp, vp, vp, vp, fp, vp, vp, fp, fp, vp, sz, vp]
    lib.spaco_chunk_attn_bwd.argtypes = [dp, vp, vp, vp, vp, fp, vp, vp, fp, fp,
                                         C.POINTER(C.c_float), i32, i32, vp, sz, vp]
    lib.spaco_chunk_attn_bwd_sparse_dq.argtypes = [dp, vp, vp, vp, vp, fp, vp, vp, fp, fp, C.POINTER(C.c_float),
                                                   C.POINTER(C.c_float), i32, i32, vp, sz, vp]
    lib.spaco_chunk_attn_bwd_sparse_dq.restype = C.c_int
    lib.seco_chunk_attn_bwd_noalloc.argtypes = [dp, vp, vp, vp, vp, fp, vp, vp, fp, fp, vp]
    lib.seco_chunk_attn_bwd_noalloc.restype = C.c_int
    lib.seco_chunk_attn_bwd_gather.argtypes = [dp, vp, vp, vp, vp, fp, vp, vp, fp, fp, fp, i64, i32, vp, sz, vp]
    lib.seco_chunk_attn_bwd_gather.restype = C.c_int
    lib.spaco_chunk_attn_bwd_gather.argtypes = [dp, vp, vp, vp, vp, fp, vp, vp, fp, fp, fp, i64, i32,
                                                C.POINTER(C.c_float), i32, i32, vp, sz, vp]
    lib.spaco_chunk_attn_bwd_gather.restype = C.c_int
    lib.kvgrad_zero.argtypes = [dp, fp, fp, i64, i64, vp]
    lib.kvgrad_accumulate.argtypes = [dp, fp, fp, fp, fp, C.c_float, i64, i64, vp]
    lib.kv_append.argtypes = [dp, vp, vp, vp, vp, vp]
    lib.kvgrad_readout.argtypes = [dp, fp, fp, vp, vp, C.c_float, vp]
    lib.kv_append.restype = lib.kvgrad_readout.restype = C.c_int
    lib.kv_append_rope.argtypes = [dp, vp, vp, vp, vp, C.c_float, vp]
    lib.kvgrad_readout_rope.argtypes = [dp, fp, fp, vp, vp, C.c_float, C.c_float, vp]
    lib.rope_rotate.argtypes = [dp, i32, vp, vp, i64, C.c_float, i32, vp]
    lib.kv_append_rope.restype = lib.kvgrad_readout_rope.restype = lib.rope_rotate.restype = C.c_int
    lib.spaco_select_chunks.argtypes = [C.c_uint64, C.c_uint64, i32, i32, C.POINTER(i32)]
    lib.spaco_chunk_weights.argtypes = [C.POINTER(i32), i32, i32, C.c_float, C.POINTER(C.c_float)]
    lib.spaco_gather_row_weights.argtypes = [C.POINTER(i32), i32, i32, i32, C.c_float, C.POINTER(C.c_float)]
    lib.spaco_gather_row_weights.restype = C.c_int
    lib.spaco_percall_weights.argtypes = [C.c_uint64, C.c_uint64, i32, i32, C.POINTER(C.c_float)]
    lib.spaco_percall_weights.restype = C.c_int
    lib.spaco_select_bernoulli.argtypes = [C.c_uint64, C.c_uint64, i32, C.c_double, C.POINTER(i32), C.POINTER(i32)]
    lib.spaco_select_bernoulli.restype = C.c_int
    lib.spaco_compensation_factor.argtypes = [i32, i32, C.c_float]
    lib.spaco_compensation_factor.restype = C.c_float
    lib.seco_workspace_bytes.argtypes = [dp, C.c_int]
    lib.seco_launch_plan.argtypes = [dp, i32, C.POINTER(i32)]
    lib.seco_launch_plan.restype = C.c_int
    lib.seco_device_info.argtypes = [C.POINTER(i32), C.POINTER(i32)]
    lib.seco_device_info.restype = C.c_int
    lib.seco_workspace_bytes.restype = sz
    lib.seco_strerror.argtypes = [C.c_int]
    lib.seco_strerror.restype = C.c_char_p
    lib.seco_profile_enable.argtypes = [C.c_int]
    lib.seco_profile_read.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.seco_profile_enable_kinds.argtypes = [C.c_uint32]
    lib.seco_profile_set_kinds.argtypes = [C.c_uint32]
    lib.seco_profile_set_kinds.restype = C.c_int
    lib.seco_profile_enable.restype = lib.seco_profile_read.restype = lib.seco_profile_enable_kinds.restype = C.c_int
    for name in ("seco_chunk_attn_fwd", "seco_chunk_attn_bwd", "spaco_chunk_attn_bwd", "kvgrad_zero",
                 "kvgrad_accumulate", "spaco_select_chunks", "spaco_chunk_weights"):
        getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def seco_strerror(status):
    return load_library().seco_strerror(int(status)).decode()


def _check(status, where):
    if status != 0:
        raise SecoError(status, where)


def _dtype_code(t):
    import torch
    if t.dtype == torch.bfloat16:
        return SECO_BF16
    if t.dtype == torch.float32:
        return SECO_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _strides3(t):
    if t.dim() != 4 or t.stride(3) != 1:
        raise ValueError("expected a [batch, head, row, head_dim] tensor with contiguous head_dim")
    return (C.c_int64 * 3)(t.stride(0), t.stride(1), t.stride(2))


def _stream(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def make_desc(q, k_cache, q_start, scale, o=None, g=None):
    """seco_desc for a chunk call; o defaults to q's strides, g to a contiguous fp32 cache."""
    B, Hq, Cn, D = q.shape
    d = SecoDesc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim = B, Hq, k_cache.shape[1], D
    d.chunk_len, d.q_start, d.dtype, d.softmax_scale = Cn, int(q_start), _dtype_code(q), float(scale)
    d.q_stride = _strides3(q)
    d.o_stride = _strides3(o if o is not None else q)
    d.kv_stride = _strides3(k_cache)
    d.g_stride = _strides3(g) if g is not None else _strides3(k_cache)
    return d


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else None


def _check_shared(k_cache, v_cache, gk=None, gv=None, lse=None):
    """The descriptor carries ONE stride triple for K and V and one for gK and gV, and the kernels index LSE as a
    contiguous fp32 [B, Hq, C] array: refuse tensors that do not fit that instead of computing on wrong addresses."""
    import torch
    if v_cache.stride() != k_cache.stride() or v_cache.shape != k_cache.shape:
        raise ValueError("k_cache and v_cache must share shape and strides")
    if gk is not None and gv is not None and (gv.stride() != gk.stride() or gv.shape != gk.shape):
        raise ValueError("gk and gv must share shape and strides")
    for g in (gk, gv):
        if g is not None and g.dtype != torch.float32:
            raise TypeError("gk / gv must be float32")
    if lse is not None and (lse.dtype != torch.float32 or not lse.is_contiguous()):
        raise ValueError("lse must be a contiguous float32 [B, Hq, C] tensor")


def seco_workspace_bytes(desc, op):
    n = load_library().seco_workspace_bytes(C.byref(desc), int(op))
    if n == C.c_size_t(-1).value:
        raise SecoError(-2, "seco_workspace_bytes")
    return n


def _workspace(desc, op, like):
    import torch
    n = seco_workspace_bytes(desc, op)
    return (torch.empty(max(n, 256), dtype=torch.uint8, device=like.device), n)


def seco_chunk_attn_fwd(q, k_cache, v_cache, q_start, scale, o=None, lse=None, stream=None, ws=None):
    """O, LSE of one chunk against cache rows [0, q_start + C).  Returns (o, lse).

    ws: optional uint8 workspace tensor (see seco_workspace_bytes); allocated here when the shape wants one,
    False to pass none."""
    import torch
    lib = load_library()
    if o is None:
        o = torch.empty_like(q)
    if lse is None:
        lse = torch.empty(q.shape[:3], dtype=torch.float32, device=q.device)
    if tuple(lse.shape) != tuple(q.shape[:3]):
        raise ValueError("lse must have shape [B, Hq, C]")
    _check_shared(k_cache, v_cache, lse=lse)
    d = make_desc(q, k_cache, q_start, scale, o=o)
    if ws is False:            # explicitly none: the library then takes the direct path
        ws = None
    elif ws is None and seco_workspace_bytes(d, SECO_OP_FWD) > 0:
        ws, _ = _workspace(d, SECO_OP_FWD, q)
    _check(lib.seco_chunk_attn_fwd(C.byref(d), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(o), _ptr(lse),
                                   _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)),
           "seco_chunk_attn_fwd")
    return o, lse


def seco_chunk_attn_bwd(q, k_cache, v_cache, o, lse, d_o, gk, gv, q_start, scale, d_q=None, ws=None, stream=None):
    """dQ of the chunk; adds the chunk's dK/dV into gk, gv (fp32, whole cache).  Returns d_q."""
    import torch
    lib = load_library()
    if d_q is None:
        d_q = torch.empty_strided(q.size(), q.stride(), dtype=q.dtype, device=q.device)
    if o.stride() != d_o.stride() or q.stride() != d_q.stride():
        raise ValueError("o/d_o and q/d_q must share strides")
    _check_shared(k_cache, v_cache, gk, gv, lse)
    d = make_desc(q, k_cache, q_start, scale, o=o, g=gk)
    if ws is None:
        ws, _ = _workspace(d, SECO_OP_BWD, q)
    _check(lib.seco_chunk_attn_bwd(C.byref(d), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(o), _ptr(lse), _ptr(d_o),
                                   _ptr(d_q), _ptr(gk), _ptr(gv), _ptr(ws), ws.numel() * ws.element_size(),
                                   _stream(stream)), "seco_chunk_attn_bwd")
    return d_q


STATIC_SCRATCH_BYTES = 40 << 20


def seco_chunk_attn_bwd_noalloc(q, k_cache, v_cache, o, lse, d_o, d_q, gk, gv, q_start, scale, stream=None):
    """seco_chunk_attn_bwd on the library's own static device scratch: no workspace argument, nothing allocated here
    or in the library (d_q must be supplied).  Returns d_q."""
    lib = load_library()
    if o.stride() != d_o.stride() or q.stride() != d_q.stride():
        raise ValueError("o/d_o and q/d_q must share strides")
    _check_shared(k_cache, v_cache, gk, gv, lse)
    d = make_desc(q, k_cache, q_start, scale, o=o, g=gk)
    _check(lib.seco_chunk_attn_bwd_noalloc(C.byref(d), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(o), _ptr(lse),
                                           _ptr(d_o), _ptr(d_q), _ptr(gk), _ptr(gv), _stream(stream)),
           "seco_chunk_attn_bwd_noalloc")
    return d_q


def spaco_chunk_attn_bwd(q, k_cache, v_cache, o, lse, d_o, gk, gv, q_start, scale, chunk_weight, weight_chunk_len,
                         d_q=None, ws=None, stream=None, dq_weight=None):
    """As seco_chunk_attn_bwd with per-chunk weights (host sequence of floats) on the dK/dV contributions.
    With dq_weight (one non-negative float per chunk) the call is spaco_chunk_attn_bwd_sparse_dq: dQ visits only
    the chunks with a non-zero dq weight and scales their terms by it."""
    import torch
    lib = load_library()
    if d_q is None:
        d_q = torch.empty_strided(q.size(), q.stride(), dtype=q.dtype, device=q.device)
    if o.stride() != d_o.stride() or q.stride() != d_q.stride():
        raise ValueError("o/d_o and q/d_q must share strides")
    _check_shared(k_cache, v_cache, gk, gv, lse)
    d = make_desc(q, k_cache, q_start, scale, o=o, g=gk)
    if ws is None:
        ws, _ = _workspace(d, SECO_OP_BWD, q)
    n = len(chunk_weight)
    w = (C.c_float * n)(*[float(x) for x in chunk_weight])
    if dq_weight is not None:
        if len(dq_weight) != n:
            raise ValueError("dq_weight and chunk_weight must have one entry per chunk")
        wq = (C.c_float * n)(*[float(x) for x in dq_weight])
        _check(lib.spaco_chunk_attn_bwd_sparse_dq(C.byref(d), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(o), _ptr(lse),
                                                  _ptr(d_o), _ptr(d_q), _ptr(gk), _ptr(gv), w, wq, n,
                                                  int(weight_chunk_len), _ptr(ws), ws.numel() * ws.element_size(),
                                                  _stream(stream)), "spaco_chunk_attn_bwd_sparse_dq")
        return d_q
    _check(lib.spaco_chunk_attn_bwd(C.byref(d), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(o), _ptr(lse), _ptr(d_o),
                                    _ptr(d_q), _ptr(gk), _ptr(gv), w, n, int(weight_chunk_len), _ptr(ws),
                                    ws.numel() * ws.element_size(), _stream(stream)), "spaco_chunk_attn_bwd")
    return d_q


def seco_chunk_attn_bwd_gather(q_rows, k_cache, v_cache, o, lse, d_o_rows, gk, gv, q_start, scale, chunk_len,
                               row_stats, d_q=None, ws=None, stream=None, row_weight=None, weight_chunk_len=None):
    """Backward of one chunk in the transposed order: dQ of the chunk's first `chunk_len` rows of q_rows, and the
    chunk's own gK/gV rows from all of q_rows / d_o_rows (the chunk's rows followed by every later row).
    row_stats: fp32 [2, B, Hq, stat_rows] kept by the caller over the whole backward pass.
    row_weight (host floats, one per chunk of weight_chunk_len rows counted from the call's first row; default
    chunk_len): the call is spaco_chunk_attn_bwd_gather."""
    import torch
    lib = load_library()
    qc, doc = q_rows[:, :, :chunk_len], d_o_rows[:, :, :chunk_len]
    if d_q is None:
        d_q = torch.empty_strided(qc.size(), qc.stride(), dtype=qc.dtype, device=qc.device)
    if o.stride() != doc.stride() or qc.stride() != d_q.stride():
        raise ValueError("o/d_o and q/d_q must share strides")
    _check_shared(k_cache, v_cache, gk, gv, lse)
    if row_stats.dtype != torch.float32 or not row_stats.is_contiguous() or row_stats.dim() != 4:
        raise ValueError("row_stats must be a contiguous fp32 [2, B, Hq, stat_rows] tensor")
    d = make_desc(qc, k_cache, q_start, scale, o=o, g=gk)
    if ws is None:
        ws, _ = _workspace(d, SECO_OP_BWD, qc)
    if row_weight is not None:
        n = len(row_weight)
        w = (C.c_float * n)(*[float(x) for x in row_weight])
        _check(lib.spaco_chunk_attn_bwd_gather(C.byref(d), _ptr(q_rows), _ptr(k_cache), _ptr(v_cache), _ptr(o),
                                               _ptr(lse), _ptr(d_o_rows), _ptr(d_q), _ptr(gk), _ptr(gv), _ptr(row_stats),
                                               int(row_stats.shape[3]), int(q_rows.shape[2] - chunk_len), w, n,
                                               int(weight_chunk_len or chunk_len), _ptr(ws),
                                               ws.numel() * ws.element_size(), _stream(stream)),
               "spaco_chunk_attn_bwd_gather")
        return d_q
    _check(lib.seco_chunk_attn_bwd_gather(C.byref(d), _ptr(q_rows), _ptr(k_cache), _ptr(v_cache), _ptr(o), _ptr(lse),
                                          _ptr(d_o_rows), _ptr(d_q), _ptr(gk), _ptr(gv), _ptr(row_stats),
                                          int(row_stats.shape[3]), int(q_rows.shape[2] - chunk_len), _ptr(ws),
                                          ws.numel() * ws.element_size(), _stream(stream)),
           "seco_chunk_attn_bwd_gather")
    return d_q


def _g_desc(g):
    d = SecoDesc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim = g.shape[0], g.shape[1], g.shape[1], g.shape[3]
    d.chunk_len, d.q_start, d.dtype, d.softmax_scale = 1, 0, SECO_F32, 1.0
    d.q_stride = d.o_stride = d.kv_stride = d.g_stride = _strides3(g)
    return d


def kvgrad_zero(gk, gv, row_begin=0, row_end=None, stream=None):
    """Zero rows [row_begin, row_end) of the fp32 KV-gradient buffers (either may be None)."""
    ref = gk if gk is not None else gv
    d = _g_desc(ref)
    if row_end is None:
        row_end = ref.shape[2]
    _check(load_library().kvgrad_zero(C.byref(d), _ptr(gk), _ptr(gv), int(row_begin), int(row_end), _stream(stream)),
           "kvgrad_zero")


def kvgrad_accumulate(dst_k, dst_v, src_k, src_v, scale, row_begin=0, row_end=None, stream=None):
    """dst[rows] += scale * src[rows] on fp32 KV-gradient buffers with identical strides."""
    ref = dst_k if dst_k is not None else dst_v
    d = _g_desc(ref)
    if row_end is None:
        row_end = ref.shape[2]
    for a, b in ((dst_k, src_k), (dst_v, src_v)):
        if a is not None and b is not None and a.stride() != b.stride():
            raise ValueError("dst and src must share strides")
    _check(load_library().kvgrad_accumulate(C.byref(d), _ptr(dst_k), _ptr(dst_v), _ptr(src_k), _ptr(src_v),
                                            float(scale), int(row_begin), int(row_end), _stream(stream)),
           "kvgrad_accumulate")


def _rows_desc(new, cache_or_g, row_begin, is_g):
    d = SecoDesc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim = new.shape[0], new.shape[1], new.shape[1], new.shape[3]
    d.chunk_len, d.q_start, d.dtype, d.softmax_scale = new.shape[2], int(row_begin), _dtype_code(new), 1.0
    d.q_stride = d.o_stride = _strides3(new)
    d.kv_stride = _strides3(new) if is_g else _strides3(cache_or_g)
    d.g_stride = _strides3(cache_or_g) if is_g else _strides3(new)
    return d


def kv_append(k_new, v_new, k_cache, v_cache, row_begin, stream=None, rope_base=None):
    """Write the chunk's keys / values ([B, Hkv, C, D]) into cache rows [row_begin, row_begin + C); with rope_base the
    keys are rotated for their positions on the way (kv_append_rope)."""
    d = _rows_desc(k_new, k_cache, row_begin, False)
    if v_new.stride() != k_new.stride() or v_cache.stride() != k_cache.stride():
        raise ValueError("k/v must share strides")
    if rope_base is not None:
        _check(load_library().kv_append_rope(C.byref(d), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                             float(rope_base), _stream(stream)), "kv_append_rope")
        return
    _check(load_library().kv_append(C.byref(d), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache), _stream(stream)),
           "kv_append")


def kvgrad_readout(gk, gv, row_begin, n_rows, dtype, scaler=1.0, d_k=None, d_v=None, stream=None, rope_base=None):
    """(d_k, d_v) = scaler * (gk, gv)[rows row_begin .. row_begin + n_rows) in the storage dtype; with rope_base the
    key part is turned back by the rows' rotary angles (kvgrad_readout_rope)."""
    import torch
    B, H, _, D = gk.shape
    if d_k is None:
        d_k = torch.empty(B, H, n_rows, D, dtype=dtype, device=gk.device)
    if d_v is None:
        d_v = torch.empty_strided(d_k.size(), d_k.stride(), dtype=dtype, device=gk.device)
    if gv.stride() != gk.stride() or d_v.stride() != d_k.stride():
        raise ValueError("gk/gv and d_k/d_v must share strides")
    d = _rows_desc(d_k, gk, row_begin, True)
    if rope_base is not None:
        _check(load_library().kvgrad_readout_rope(C.byref(d), _ptr(gk), _ptr(gv), _ptr(d_k), _ptr(d_v), float(scaler),
                                                  float(rope_base), _stream(stream)), "kvgrad_readout_rope")
        return d_k, d_v
    _check(load_library().kvgrad_readout(C.byref(d), _ptr(gk), _ptr(gv), _ptr(d_k), _ptr(d_v), float(scaler),
                                         _stream(stream)), "kvgrad_readout")
    return d_k, d_v


def rope_rotate(x, pos_start, rope_base, inverse=False, out=None, stream=None):
    """Rotary position embedding of x [B, H, C, D] (row r at position pos_start + r), or its inverse / transpose."""
    import torch
    if out is None:
        out = torch.empty_strided(x.size(), x.stride(), dtype=x.dtype, device=x.device)
    d = SecoDesc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim = x.shape[0], x.shape[1], x.shape[1], x.shape[3]
    d.chunk_len, d.q_start, d.softmax_scale = x.shape[2], 0, 1.0
    d.dtype = SECO_BF16 if x.dtype == torch.bfloat16 else SECO_F32
    d.q_stride = d.kv_stride = d.g_stride = _strides3(x)
    d.o_stride = _strides3(out)
    _check(load_library().rope_rotate(C.byref(d), x.shape[1], _ptr(x), _ptr(out), int(pos_start), float(rope_base),
                                      1 if inverse else 0, _stream(stream)), "rope_rotate")
    return out


def spaco_select_chunks(seed, step, k, t):
    """t distinct chunk indices of 0..k-1, descending (list of int)."""
    out = (C.c_int32 * max(int(t), 1))()
    _check(load_library().spaco_select_chunks(int(seed), int(step), int(k), int(t), out), "spaco_select_chunks")
    return list(out[:t])


def spaco_percall_weights(seed, step, j, t):
    """Weight vector w[0..j] of call j when every call draws min(t, j) of its earlier chunks itself (list of float)."""
    w = (C.c_float * (int(j) + 1))()
    _check(load_library().spaco_percall_weights(int(seed), int(step), int(j), int(t), w), "spaco_percall_weights")
    return list(w)


def spaco_select_bernoulli(seed, step, k, q):
    """Every chunk of 0..k-1 selected independently with probability q; indices descending (list of int)."""
    out = (C.c_int32 * max(int(k), 1))()
    n = C.c_int32(0)
    _check(load_library().spaco_select_bernoulli(int(seed), int(step), int(k), float(q), out, C.byref(n)),
           "spaco_select_bernoulli")
    return list(out[:n.value])


def spaco_compensation_factor(k, t, cap=0.0):
    """k/t, limited to cap when cap > 0."""
    lam = load_library().spaco_compensation_factor(int(k), int(t), float(cap))
    if lam < 0:
        raise SecoError(-8, "spaco_compensation_factor")
    return lam


def spaco_chunk_weights(selected, j, factor):
    """Weight vector w[0..j] of the backward call for chunk j (list of float)."""
    sel = (C.c_int32 * max(len(selected), 1))(*[int(i) for i in selected])
    w = (C.c_float * (int(j) + 1))()
    _check(load_library().spaco_chunk_weights(sel, len(selected), int(j), float(factor), w), "spaco_chunk_weights")
    return list(w)


def spaco_gather_row_weights(selected, i, k, factor):
    """Row weights w[0 .. k-i) of the transposed-order backward call for selected chunk i of k (list of float)."""
    sel = (C.c_int32 * max(len(selected), 1))(*[int(x) for x in selected])
    w = (C.c_float * (int(k) - int(i)))() if k > i else (C.c_float * 1)()
    _check(load_library().spaco_gather_row_weights(sel, len(selected), int(i), int(k), float(factor), w),
           "spaco_gather_row_weights")
    return list(w)


PROFILE_KINDS = ("fwd", "delta", "dq", "dkdv", "kvgrad", "merge")


def seco_launch_plan(desc, n_col_tiles):
    """(splits per row tile, row tiles, shared-out cache tiles per (batch, KV head), workgroups per such tile)."""
    out = (C.c_int32 * 4)()
    _check(load_library().seco_launch_plan(C.byref(desc), int(n_col_tiles), out), "seco_launch_plan")
    return tuple(out)


def seco_device_info():
    """(compute units, maximum engine clock in kHz) of the current HIP device."""
    cus, khz = C.c_int32(0), C.c_int32(0)
    _check(load_library().seco_device_info(C.byref(cus), C.byref(khz)), "seco_device_info")
    return cus.value, khz.value


def seco_profile_enable(on=True, kinds=None):
    """Time every kernel launch (on=True), none (False), or only the named kinds (subset of PROFILE_KINDS)."""
    if kinds is not None:
        mask = 0
        for k in kinds:
            mask |= 1 << PROFILE_KINDS.index(k)
        _check(load_library().seco_profile_enable_kinds(mask), "seco_profile_enable_kinds")
    else:
        _check(load_library().seco_profile_enable(1 if on else 0), "seco_profile_enable")


def seco_profile_set(kinds=None):
    """Change which kinds are timed (None: all, []: none) without dropping what has been recorded."""
    mask = 0
    for k in (PROFILE_KINDS if kinds is None else kinds):
        mask |= 1 << PROFILE_KINDS.index(k)
    _check(load_library().seco_profile_set_kinds(mask), "seco_profile_set_kinds")


def seco_profile_read():
    """{kind: (total_ms, launches)} of the kernels launched since profiling was enabled / last read."""
    ms = (C.c_double * len(PROFILE_KINDS))()
    n = (C.c_int64 * len(PROFILE_KINDS))()
    _check(load_library().seco_profile_read(ms, n), "seco_profile_read")
    return {k: (ms[i], n[i]) for i, k in enumerate(PROFILE_KINDS)}
