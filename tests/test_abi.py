"""CPU-side checks of the C ABI: the library loads, exports every declared symbol, rejects
bad arguments with the documented status codes (no launch happens on a validation error),
and its host-side chunk selection equals the oracle's bit for bit."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2505_16710_amd as seco
from paper_2505_16710_amd import binding as B
from oracle import selection as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = seco.load_library()
    header = open(os.path.join(ROOT, "include", "seco.h")).read()
    names = set(re.findall(r"^\s*(?:int|size_t|const char\*)\s+(\w+)\s*\(", header, flags=re.M))
    assert {"seco_chunk_attn_fwd", "seco_chunk_attn_bwd", "spaco_chunk_attn_bwd", "kvgrad_zero",
            "kvgrad_accumulate", "spaco_select_chunks", "spaco_chunk_weights", "seco_workspace_bytes",
            "seco_strerror"} <= names
    for n in names:
        assert hasattr(lib, n), n


def desc(**kw):
    d = B.SecoDesc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim = 1, 4, 2, 128
    d.chunk_len, d.q_start, d.dtype, d.softmax_scale = 256, 256, B.SECO_BF16, 0.088
    for name in ("q_stride", "o_stride", "kv_stride", "g_stride"):
        setattr(d, name, (C.c_int64 * 3)(4 * 512 * 128, 512 * 128, 128))
    for k, v in kw.items():
        setattr(d, k, v)
    return d


FAKE = C.c_void_p(0x1000)   # non-null, 16-byte aligned, never dereferenced: validation fails first


def fwd(d, q=FAKE, k=FAKE, v=FAKE, o=FAKE, lse=FAKE):
    return seco.load_library().seco_chunk_attn_fwd(C.byref(d), q, k, v, o, lse, None, 0, None)


def bwd(d, ws=C.c_void_p(0x1000), ws_bytes=1 << 30, gk=FAKE):
    return seco.load_library().seco_chunk_attn_bwd(C.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, gk, FAKE,
                                                   ws, ws_bytes, None)


def test_validation_status_codes():
    assert fwd(desc(dtype=7)) == -4
    assert fwd(desc(batch=0)) == -2
    assert fwd(desc(n_q_heads=3)) == -2
    assert fwd(desc(q_start=-1)) == -2
    assert fwd(desc(head_dim=96)) == -3
    assert fwd(desc(dtype=B.SECO_F32, head_dim=6)) == -3
    assert fwd(desc(dtype=B.SECO_F32, head_dim=260)) == -3
    assert fwd(desc(q_stride=(C.c_int64 * 3)(4 * 512 * 128, 512 * 128, 132))) == -5
    assert fwd(desc(kv_stride=(C.c_int64 * 3)(4 * 512 * 128, 512 * 128, 64))) == -5
    assert fwd(desc(), q=None) == -1
    assert fwd(desc(), k=C.c_void_p(0x1004)) == -5
    assert fwd(desc(q_start=1 << 30)) == -10
    assert fwd(desc(kv_stride=(C.c_int64 * 3)(1 << 40, 1 << 32, (1 << 22) + 8))) == -10   # row stride beyond the 32-bit tile offsets
    assert seco.load_library().seco_chunk_attn_fwd(None, FAKE, FAKE, FAKE, FAKE, FAKE, None, 0, None) == -1
    assert bwd(desc(), ws=None) == -6
    assert bwd(desc(), ws_bytes=16) == -6
    assert bwd(desc(), ws=C.c_void_p(0x1010)) == -6
    assert bwd(desc(), gk=None) == -1
    assert bwd(desc(g_stride=(C.c_int64 * 3)(0, 0, 126))) == -5


def test_spaco_weight_validation():
    lib = seco.load_library()
    d = desc()                       # kv_len = 512

    def call(w, n, wlen):
        arr = (C.c_float * max(len(w), 1))(*w)
        return lib.spaco_chunk_attn_bwd(C.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                                        arr, n, wlen, C.c_void_p(0x1000), 1 << 30, None)
    assert call([1.0], 1, 256) == -7             # does not cover 512 rows
    assert call([1.0, 1.0, 1.0], 3, 256) == -7   # one chunk too many
    assert call([1.0, float("nan")], 2, 256) == -7
    assert call([1.0, float("inf")], 2, 256) == -7
    assert call([1.0, 1.0], 2, 0) == -7
    assert lib.spaco_chunk_attn_bwd(C.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                                    None, 2, 256, C.c_void_p(0x1000), 1 << 30, None) == -1

    # weights of the dQ columns: finite and non-negative, at most 48 runs of equal non-zero weights
    def sparse(w, wq, n, wlen, dd=d):
        arr = (C.c_float * n)(*w)
        arq = (C.c_float * n)(*wq) if wq is not None else None
        return lib.spaco_chunk_attn_bwd_sparse_dq(C.byref(dd), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                                                  arr, arq, n, wlen, None, 0, None)
    assert sparse([1.0, 1.0], None, 2, 256) == -1
    assert sparse([1.0, 1.0], [-1.0, 1.0], 2, 256) == -7
    assert sparse([1.0, 1.0], [float("nan"), 1.0], 2, 256) == -7
    assert sparse([1.0, 1.0], [1.0, 1.0], 3, 256) == -7              # coverage is checked as for the dK/dV weights
    assert sparse([1.0, 1.0], [2.0, 1.0], 2, 256) == -6              # valid weights: the next check is the workspace
    assert sparse([1.0] * 128, [1.0 + (i % 2) for i in range(128)], 128, 4) == -10   # 128 runs
    assert sparse([1.0] * 128, [float(i % 2) for i in range(128)], 128, 4) == -10    # 64 runs
    assert sparse([1.0] * 128, [float(i % 4 == 0) for i in range(128)], 128, 4) == -6   # 32 runs fit


def test_kvgrad_validation_and_workspace_size():
    lib = seco.load_library()
    d = desc()
    assert lib.kvgrad_zero(C.byref(d), FAKE, FAKE, 5, 4, None) == -8
    assert lib.kvgrad_zero(C.byref(d), FAKE, FAKE, -1, 4, None) == -8
    assert lib.kvgrad_zero(C.byref(d), C.c_void_p(0x1008), FAKE, 0, 4, None) == -5
    assert lib.kvgrad_accumulate(C.byref(d), FAKE, None, None, None, 1.0, 0, 4, None) == -1
    assert lib.kvgrad_accumulate(C.byref(d), FAKE, None, FAKE, None, 1.0, 0, 4, None) == -8   # dst aliases src
    assert lib.kvgrad_zero(C.byref(d), None, None, 0, 4, None) == 0                           # nothing to do
    # long chunks (enough row tiles to fill the GPU): no forward workspace; the backward takes two values per query
    # row (delta and the log-sum-exp in the form the dK/dV kernel starts from; fp32: delta only) plus the sums
    # of the column tiles that the dK/dV pass divides by query head (at most 256 shares of 2 x 128 x 128 floats)
    big = desc(n_q_heads=32, n_kv_heads=8, chunk_len=1024)
    assert seco.seco_workspace_bytes(big, B.SECO_OP_FWD) == 0
    assert seco.seco_workspace_bytes(big, B.SECO_OP_BWD) == 2 * 32 * 1024 * 4 + 256 * 2 * 128 * 128 * 4
    # without grouped heads nothing is divided: delta only
    mha = desc(n_q_heads=8, n_kv_heads=8, chunk_len=4096)
    assert seco.seco_workspace_bytes(mha, B.SECO_OP_BWD) == 2 * 8 * 4096 * 4
    # fp32 never uses the split path
    assert seco.seco_workspace_bytes(desc(dtype=B.SECO_F32), B.SECO_OP_FWD) == 0
    # short chunk: 2 KV heads x 4 packed row tiles = 8 work items -> up to 64 splits of fp32 partials
    rows = 1 * 4 * 256
    assert seco.seco_workspace_bytes(d, B.SECO_OP_FWD) == 64 * rows * 128 * 4 + 64 * rows * 2 * 4
    assert seco.seco_workspace_bytes(d, B.SECO_OP_BWD) == 2 * rows * 4 + 64 * rows * 128 * 4
    assert bwd(d, ws_bytes=rows * 4) == -6            # delta alone is no longer enough for this shape
    assert seco.seco_workspace_bytes(desc(dtype=B.SECO_F32, chunk_len=3), B.SECO_OP_BWD) == 256   # rounded up to 256
    assert "head_dim" in seco.seco_strerror(-3) and seco.seco_strerror(0) == "ok"
    assert seco.seco_strerror(-99) == "unknown status"


def test_selection_matches_oracle_bit_exactly():
    grid = [(1, 1), (2, 1), (4, 2), (6, 4), (16, 4), (16, 16), (32, 8), (64, 16), (128, 8), (128, 32), (512, 8), (7, 3)]
    for k, t in grid:
        for seed in (0, 1, 2, 12345, 2 ** 63 + 5, 2 ** 64 - 1):
            for step in (0, 1, 17, 2 ** 40):
                assert seco.spaco_select_chunks(seed, step, k, t) == S.select_chunks(seed, step, k, t).tolist()
    lib = seco.load_library()
    out = (C.c_int32 * 4)()
    assert lib.spaco_select_chunks(0, 0, 4, 5, out) == -8
    assert lib.spaco_select_chunks(0, 0, 0, 0, out) == -8
    assert lib.spaco_select_chunks(0, 0, 4, 2, None) == -1


def test_chunk_weights_match_oracle():
    for sel, j, lam in (([3, 2, 0], 3, 4 / 3), ([3, 2, 0], 2, 2.0), ([5], 5, 8.0), ([7, 1], 4, 3.0), ([], 2, 2.0)):
        want = S.chunk_weights(sel, j, np.float32(lam))
        got = np.array(seco.spaco_chunk_weights(sel, j, lam), dtype=np.float32)
        assert np.array_equal(got, want)
    lib = seco.load_library()
    w = (C.c_float * 4)()
    assert lib.spaco_chunk_weights(None, 0, -1, 1.0, w) == -8
    assert lib.spaco_chunk_weights(None, 2, 1, 1.0, w) == -1


def test_gather_row_weights_match_oracle_and_are_the_transpose_of_the_chunk_weights():
    """Row weights of the transposed-order call for chunk i: library == oracle, and entry m - i equals what
    chunk_weights of call m puts on chunk i whenever call m takes place (m selected), 0 when it does not."""
    for sel, k, lam in (([3, 2, 0], 4, 4 / 3), ([5], 6, 8.0), ([7, 4, 1], 8, 3.0), ([9, 8, 7, 2], 10, 2.5), ([0], 3, 3.0)):
        for i in sel:
            want = S.gather_row_weights(sel, i, k, np.float32(lam))
            got = np.array(seco.spaco_gather_row_weights(sel, i, k, lam), dtype=np.float32)
            assert np.array_equal(got, want)
            for m in range(i, k):
                col = S.chunk_weights(sel, m, np.float32(lam))[i] if m in sel else np.float32(0)
                assert want[m - i] == col, (sel, i, m)
    lib = seco.load_library()
    w = (C.c_float * 4)()
    assert lib.spaco_gather_row_weights(None, 0, 2, 2, 1.0, w) == -8       # k must exceed i
    assert lib.spaco_gather_row_weights(None, 2, 0, 3, 1.0, w) == -1
    assert lib.spaco_gather_row_weights(None, 0, 1, 3, 1.0, None) == -1


def test_bernoulli_selection_matches_oracle_bit_exactly_and_has_the_right_rate():
    for k in (1, 5, 16, 128, 512):
        for q in (1.0, 0.5, 0.25, 1 / 3, 0.9, 1e-3, 8 / 128):
            for seed in (0, 7, 2 ** 64 - 1):
                for step in (0, 3, 2 ** 33):
                    got = seco.spaco_select_bernoulli(seed, step, k, q)
                    assert got == S.select_bernoulli(seed, step, k, q).tolist()
                    assert got == sorted(set(got), reverse=True) and all(0 <= i < k for i in got)
    assert seco.spaco_select_bernoulli(1, 2, 9, 1.0) == list(range(8, -1, -1))
    # inclusion frequency of every chunk over many steps ~ q (binomial, 6 sigma)
    k, q, n = 16, 0.25, 4000
    counts = np.zeros(k)
    for step in range(n):
        counts[seco.spaco_select_bernoulli(123, step, k, q)] += 1
    assert np.all(np.abs(counts - n * q) < 6 * np.sqrt(n * q * (1 - q)))
    # pairs are independent: joint frequency of chunks 2 and 11 ~ q^2
    joint = sum(1 for step in range(n) if {2, 11} <= set(seco.spaco_select_bernoulli(123, step, k, q)))
    assert abs(joint - n * q * q) < 6 * np.sqrt(n * q * q * (1 - q * q))
    lib = seco.load_library()
    out, cnt = (C.c_int32 * 4)(), C.c_int32(0)
    assert lib.spaco_select_bernoulli(0, 0, 4, 0.0, out, C.byref(cnt)) == -8
    assert lib.spaco_select_bernoulli(0, 0, 4, 1.5, out, C.byref(cnt)) == -8
    assert lib.spaco_select_bernoulli(0, 0, 4, float("nan"), out, C.byref(cnt)) == -8
    assert lib.spaco_select_bernoulli(0, 0, 4, 0.5, None, C.byref(cnt)) == -1


def test_compensation_factor_with_cap():
    """The library's factor against the values the paper states (tests/golden/compensation_factor.txt: k t cap factor)."""
    golden = os.path.join(ROOT, "tests", "golden", "compensation_factor.txt")
    rows = 0
    for line in open(golden):
        f = line.split("#")[0].split()
        if len(f) == 4:
            k, t, cap, lam = int(f[0]), int(f[1]), (0.0 if f[2] == "-" else float(f[2])), float(f[3])
            assert seco.spaco_compensation_factor(k, t, cap=cap) == np.float32(lam)
            assert S.compensation_factor(k, t, cap=None if cap == 0.0 else cap) == lam
            rows += 1
    assert rows >= 8
    assert abs(seco.spaco_compensation_factor(7, 3) - 7 / 3) < 1e-6
    with pytest.raises(seco.SecoError):
        seco.spaco_compensation_factor(4, 5)


def test_append_and_readout_validation():
    lib = seco.load_library()
    d = desc()
    assert lib.kv_append(C.byref(d), FAKE, FAKE, None, FAKE, None) == -1
    assert lib.kv_append(C.byref(d), C.c_void_p(0x1008), FAKE, FAKE, FAKE, None) == -5
    assert lib.kv_append(C.byref(desc(head_dim=96)), FAKE, FAKE, FAKE, FAKE, None) == -3
    assert lib.kvgrad_readout(C.byref(d), FAKE, None, None, None, 1.0, None) == -1
    assert lib.kvgrad_readout(C.byref(d), FAKE, FAKE, FAKE, FAKE, float("inf"), None) == -8
    assert lib.kvgrad_readout(C.byref(desc(dtype=B.SECO_F32, head_dim=12)), FAKE, FAKE, FAKE, FAKE, 1.0, None) == -3
    assert lib.kvgrad_readout(C.byref(d), None, None, None, None, 1.0, None) == 0           # nothing to do


def test_percall_weights_match_oracle_bit_exactly():
    for seed in (0, 5, 2 ** 64 - 1):
        for step in (0, 1, 4095):
            for j, t in [(0, 4), (1, 4), (2, 1), (7, 4), (15, 4), (31, 8), (127, 8)]:
                got = np.array(seco.spaco_percall_weights(seed, step, j, t), dtype=np.float32)
                np.testing.assert_array_equal(got, S.percall_weights(seed, step, j, t))
    lib = seco.load_library()
    assert lib.spaco_percall_weights(0, 0, -1, 4, (C.c_float * 1)()) == -8
    assert lib.spaco_percall_weights(0, 0, 3, 4, None) == -1


def test_launch_plan_host_logic():
    """The host arithmetic that shapes the launches: division of the cache rows among workgroups for short chunks,
    and the sharing-out of the dK/dV pass's last round by query head."""
    big = desc(n_q_heads=32, n_kv_heads=8, chunk_len=1024, q_start=0)
    units, G = 8, 4
    for n_col_tiles in range(0, 200):
        splits, row_tiles, n_tiles, hs = seco.seco_launch_plan(big, n_col_tiles)
        assert (splits, row_tiles) == (1, 256)                       # 256 row tiles: no division of the cache rows
        tail = units * n_col_tiles % 256
        if tail == 0 or tail > 128:
            assert (n_tiles, hs) == (0, 1)
        else:
            assert hs in (2, 4) and G % hs == 0 and n_tiles == -(-tail // units) <= n_col_tiles
            assert units * n_tiles * hs <= 256 and 1024 * (G // hs) >= 512
            assert hs == 4 or units * n_tiles * 4 > 256               # four ways whenever that fits in one round
    # the benchmark's calls: 8 (j + 1) cache tiles per (batch, KV head)
    assert [seco.seco_launch_plan(big, 8 * (j + 1))[2:] for j in range(4)] == [(8, 4), (16, 2), (0, 1), (0, 1)]
    # short chunks: nothing is shared out (a share must keep 512 query rows), the cache rows are divided instead
    short = desc(n_q_heads=32, n_kv_heads=8, chunk_len=128, q_start=128 * 100)
    splits, row_tiles, n_tiles, hs = seco.seco_launch_plan(short, 101)
    assert row_tiles == 8 * 4 and 2 <= splits <= 64 and (n_tiles, hs) == (0, 1)
    assert splits * row_tiles <= 640 and (128 * 101 + 63) // 64 // splits >= 4     # about 512 workgroups, >= 4 tiles each
    assert seco.seco_launch_plan(desc(n_q_heads=32, n_kv_heads=8, chunk_len=128, q_start=0), 1)[0] == 1   # too few rows to divide
    # no grouped heads: nothing to share out
    assert seco.seco_launch_plan(desc(n_q_heads=8, n_kv_heads=8, chunk_len=4096, q_start=0), 40)[2:] == (0, 1)
    lib = seco.load_library()
    out = (C.c_int32 * 4)()
    assert lib.seco_launch_plan(C.byref(desc(dtype=B.SECO_F32)), 4, out) == -4
    assert lib.seco_launch_plan(C.byref(big), -1, out) == -8
    assert lib.seco_launch_plan(C.byref(big), 4, None) == -1


def test_rope_entry_points_validate_their_arguments():
    lib = seco.load_library()
    d = desc()
    f32 = C.c_float
    assert lib.kv_append_rope(C.byref(d), FAKE, FAKE, FAKE, FAKE, f32(1.0), None) == -8           # base must be > 1
    assert lib.kv_append_rope(C.byref(d), FAKE, FAKE, FAKE, FAKE, f32(float("inf")), None) == -8
    assert lib.kv_append_rope(C.byref(d), FAKE, FAKE, None, FAKE, f32(1e4), None) == -1
    assert lib.kv_append_rope(C.byref(desc(dtype=B.SECO_F32, head_dim=20)), FAKE, FAKE, FAKE, FAKE, f32(1e4), None) == -3
    assert lib.kvgrad_readout_rope(C.byref(d), FAKE, FAKE, FAKE, FAKE, f32(float("nan")), f32(1e4), None) == -8
    assert lib.kvgrad_readout_rope(C.byref(d), FAKE, FAKE, FAKE, FAKE, f32(1.0), f32(0.5), None) == -8
    assert lib.kvgrad_readout_rope(C.byref(d), FAKE, None, FAKE, FAKE, f32(1.0), f32(1e4), None) == -1
    assert lib.rope_rotate(C.byref(d), 4, None, FAKE, 0, f32(1e4), 0, None) == -1
    assert lib.rope_rotate(C.byref(d), 0, FAKE, FAKE, 0, f32(1e4), 0, None) == -8
    assert lib.rope_rotate(C.byref(d), 4, FAKE, FAKE, -1, f32(1e4), 0, None) == -8
    assert lib.rope_rotate(C.byref(d), 4, C.c_void_p(0x1004), FAKE, 0, f32(1e4), 0, None) == -5


def test_device_info_rejects_null_and_reports_or_fails_cleanly():
    lib = B.load_library()
    one = C.c_int32(0)
    assert lib.seco_device_info(None, C.byref(one)) == -1 and lib.seco_device_info(C.byref(one), None) == -1
    cus, khz = C.c_int32(-7), C.c_int32(-7)
    rc = lib.seco_device_info(C.byref(cus), C.byref(khz))
    if rc == 0:                       # a GPU is present
        assert cus.value > 0 and khz.value > 0
    else:                             # no device: a status, and the outputs are left alone
        assert rc == -9 and (cus.value, khz.value) == (-7, -7)


def test_gather_backward_validates_its_arguments():
    """seco_chunk_attn_bwd_gather: bf16 only, row counts and the row-statistics length are checked before anything
    is enqueued (no GPU needed: every call here fails validation)."""
    lib = B.load_library()
    d = desc(dtype=B.SECO_BF16, head_dim=128, n_q_heads=4, n_kv_heads=2, chunk_len=256, q_start=512)
    p = C.c_void_p(4096)
    ws = C.c_void_p(1 << 20)
    n_ws = lib.seco_workspace_bytes(C.byref(d), B.SECO_OP_BWD)

    def call(dd=d, stat_rows=1024, later=256, stats=p, ws_bytes=n_ws):
        return lib.seco_chunk_attn_bwd_gather(C.byref(dd), p, p, p, p, p, p, p, p, p, stats, stat_rows, later, ws,
                                              ws_bytes, None)

    assert call(dd=desc(dtype=B.SECO_F32, head_dim=64, chunk_len=256, q_start=512)) == -4      # fp32: not provided
    assert call(stats=None) == -1
    assert call(later=-1) == -8
    assert call(stat_rows=1020) == -8          # shorter than q_start + chunk_len + later rows
    assert call(stat_rows=1026) == -8          # not a multiple of 4
    assert call(ws_bytes=n_ws - 1) == -6


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """include/seco.h compiles as C99 with warnings as errors, and a C program that takes the address of every
    declared function links against libseco_hip.so (no C++ or torch types at the boundary) and runs its host-only
    calls."""
    import subprocess
    header = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    names = sorted(set(re.findall(r"\b((?:seco|spaco|kvgrad|kv|rope)_\w+)\s*\(", open(os.path.join(header, "seco.h")).read())))
    assert len(names) >= 25
    src = tmp_path / "abi.c"
    src.write_text('#include <stdio.h>\n#include "seco.h"\nint main(void) {\n  void* f[] = {'
                   + ", ".join(f"(void*){n}" for n in names)
                   + '};\n  int32_t sel[3]; float w[6];\n'
                     '  if (spaco_select_chunks(1, 2, 8, 3, sel) != SECO_OK) return 1;\n'
                     '  if (!(sel[0] > sel[1] && sel[1] > sel[2] && sel[2] >= 0 && sel[0] < 8)) return 2;\n'
                     '  if (spaco_chunk_weights(sel, 3, 5, 2.0f, w) != SECO_OK) return 3;\n'
                     '  if (spaco_compensation_factor(32, 8, 2.0f) != 2.0f) return 4;\n'
                     '  printf("%d %s\\n", (int)(sizeof f / sizeof f[0]), seco_strerror(SECO_ERR_WORKSPACE));\n  return 0;\n}\n')
    exe = tmp_path / "abi"
    lib_dir = os.path.dirname(B.library_path())
    r = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-Wno-pedantic", "-I", header,
                        str(src), "-o", str(exe), "-L", lib_dir, "-l:libseco_hip.so", f"-Wl,-rpath,{lib_dir}"],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, (r.returncode, r.stderr)
    assert r.stdout.split()[0] == str(len(names))


def test_weighted_gather_backward_validates_its_weights():
    lib = B.load_library()
    d = desc(dtype=B.SECO_BF16, head_dim=128, n_q_heads=4, n_kv_heads=2, chunk_len=256, q_start=512)
    p = C.c_void_p(4096)
    ws = C.c_void_p(1 << 20)
    n_ws = lib.seco_workspace_bytes(C.byref(d), B.SECO_OP_BWD)

    def call(w, n=None, wlen=256, later=512):
        arr = (C.c_float * len(w))(*w) if w is not None else None
        return lib.spaco_chunk_attn_bwd_gather(C.byref(d), p, p, p, p, p, p, p, p, p, p, 4096, later, arr,
                                               len(w) if n is None and w is not None else (n or 0), wlen, ws, n_ws, None)

    assert call(None) == -1
    assert call([1.0, 2.0, 0.0], wlen=200) == -7          # chunk length of the weights not a multiple of 64
    assert call([1.0, 2.0]) == -7                          # does not cover the 768 rows handed in
    assert call([1.0, 2.0, 0.0, 1.0]) == -7                # covers more chunks than there are rows
    assert call([1.0, -2.0, 0.0]) == -7 and call([1.0, float("nan"), 0.0]) == -7
    assert call([1.0 + i % 2 for i in range(50)], wlen=64, later=50 * 64 - 256) == -10   # more than 24 runs


def test_binding_refuses_layouts_the_descriptor_cannot_express():
    """One stride triple serves K and V, one gK and gV, and LSE is indexed as a contiguous fp32 [B, Hq, C] array:
    the binding raises before anything reaches the library (CPU tensors suffice: no call is made)."""
    import torch
    q = torch.zeros(1, 4, 8, 128, dtype=torch.bfloat16)
    k = torch.zeros(1, 2, 16, 128, dtype=torch.bfloat16)
    v_other = torch.zeros(1, 16, 2, 128, dtype=torch.bfloat16).transpose(1, 2)      # same shape, other strides
    with pytest.raises(ValueError):
        seco.seco_chunk_attn_fwd(q, k, v_other, 8, 0.088)
    lse_view = torch.zeros(1, 4, 16)[:, :, ::2]
    with pytest.raises(ValueError):
        seco.seco_chunk_attn_fwd(q, k, k, 8, 0.088, lse=lse_view)
    with pytest.raises(ValueError):
        seco.seco_chunk_attn_fwd(q, k, k, 8, 0.088, lse=torch.zeros(1, 4, 8, dtype=torch.float64))
    o, lse = torch.zeros_like(q), torch.zeros(1, 4, 8)
    gk = torch.zeros(1, 2, 16, 128)
    gv_other = torch.zeros(1, 16, 2, 128).transpose(1, 2)
    with pytest.raises(ValueError):
        seco.seco_chunk_attn_bwd(q, k, k, o, lse, o, gk, gv_other, 8, 0.088, d_q=torch.zeros_like(q))
    with pytest.raises(ValueError):
        seco.seco_chunk_attn_bwd(q, k, v_other, o, lse, o, gk, gk, 8, 0.088, d_q=torch.zeros_like(q))
    with pytest.raises(ValueError):
        seco.seco_chunk_attn_bwd(q, k, k, o, lse_view, o, gk, gk, 8, 0.088, d_q=torch.zeros_like(q))
