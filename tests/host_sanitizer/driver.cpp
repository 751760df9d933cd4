// Host side of the C ABI under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only; built and run by
// tests/test_host_sanitizer.py).  The kernel launchers are recording stubs, so the device pointers below are fake
// and never dereferenced; what runs for real is everything the entry points do before a launch: validation, the
// column-segment tables of the dK/dV pass, the run tables of the column-weighted dQ and of the transposed order,
// the workspace layout, chunk selection and the weight vectors.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "seco.h"
#include "stub_launch.h"

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::fprintf(stderr, "%s:%d: CHECK failed: %s\n", __FILE__, __LINE__, #cond); \
      std::exit(1);                                                        \
    }                                                                      \
  } while (0)

static seco_desc desc(int dtype = SECO_BF16, int C = 256, int q_start = 256, int Hq = 4, int Hkv = 2, int D = 128) {
  seco_desc d;
  std::memset(&d, 0, sizeof(d));
  d.batch = 1; d.n_q_heads = Hq; d.n_kv_heads = Hkv; d.head_dim = D;
  d.chunk_len = C; d.q_start = q_start; d.dtype = dtype; d.softmax_scale = 0.088f;
  int64_t* ss[4] = {d.q_stride, d.o_stride, d.kv_stride, d.g_stride};
  for (auto s : ss) { s[0] = (int64_t)Hq << 22; s[1] = (int64_t)1 << 22; s[2] = D; }
  return d;
}

static void* const FAKE = reinterpret_cast<void*>(0x10000);
static float* const FAKEF = reinterpret_cast<float*>(0x10000);

int main() {
  // ---- validation codes (nothing may be launched) ----
  {
    seco_desc d = desc();
    g_stub.clear();
    seco_desc bad = d; bad.dtype = 7;
    CHECK(seco_chunk_attn_fwd(&bad, FAKE, FAKE, FAKE, FAKE, FAKEF, nullptr, 0, nullptr) == SECO_ERR_DTYPE);
    bad = d; bad.n_q_heads = 3;
    CHECK(seco_chunk_attn_fwd(&bad, FAKE, FAKE, FAKE, FAKE, FAKEF, nullptr, 0, nullptr) == SECO_ERR_SHAPE);
    bad = d; bad.head_dim = 96;
    CHECK(seco_chunk_attn_fwd(&bad, FAKE, FAKE, FAKE, FAKE, FAKEF, nullptr, 0, nullptr) == SECO_ERR_HEAD_DIM);
    bad = d; bad.q_stride[2] = 132;
    CHECK(seco_chunk_attn_fwd(&bad, FAKE, FAKE, FAKE, FAKE, FAKEF, nullptr, 0, nullptr) == SECO_ERR_ALIGN);
    bad = d; bad.q_start = 1 << 30;
    CHECK(seco_chunk_attn_fwd(&bad, FAKE, FAKE, FAKE, FAKE, FAKEF, nullptr, 0, nullptr) == SECO_ERR_TOO_LARGE);
    bad = d; bad.softmax_scale = NAN;
    CHECK(seco_chunk_attn_fwd(&bad, FAKE, FAKE, FAKE, FAKE, FAKEF, nullptr, 0, nullptr) == SECO_ERR_SHAPE);
    CHECK(seco_chunk_attn_fwd(&d, nullptr, FAKE, FAKE, FAKE, FAKEF, nullptr, 0, nullptr) == SECO_ERR_NULL);
    CHECK(seco_chunk_attn_fwd(nullptr, FAKE, FAKE, FAKE, FAKE, FAKEF, nullptr, 0, nullptr) == SECO_ERR_NULL);
    CHECK(seco_chunk_attn_bwd(&d, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, nullptr, 0, nullptr) ==
          SECO_ERR_WORKSPACE);
    CHECK(seco_chunk_attn_bwd(&d, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, FAKE, 16, nullptr) ==
          SECO_ERR_WORKSPACE);
    CHECK(seco_workspace_bytes(&bad, SECO_OP_BWD) == (size_t)-1);
    CHECK(seco_workspace_bytes(&d, 99) == (size_t)-1);
    CHECK(kvgrad_zero(&d, FAKEF, FAKEF, 5, 4, nullptr) == SECO_ERR_RANGE);
    CHECK(kvgrad_accumulate(&d, FAKEF, nullptr, FAKEF, nullptr, 1.f, 0, 4, nullptr) == SECO_ERR_RANGE);   // aliasing
    CHECK(g_stub.fwd + g_stub.dq + g_stub.dkdv + g_stub.zero + g_stub.axpy == 0);
  }
  // ---- dense backward: one segment over all visible rows; forward with and without the split workspace ----
  {
    seco_desc d = desc(SECO_BF16, 256, 768);               // kv_len 1024 = 8 column tiles of 128
    const size_t ws = seco_workspace_bytes(&d, SECO_OP_BWD);
    CHECK(ws != (size_t)-1 && ws > 0);
    g_stub.clear();
    CHECK(seco_chunk_attn_bwd(&d, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, FAKE, ws, nullptr) == SECO_OK);
    CHECK(g_stub.dq == 1 && g_stub.dkdv == 1 && g_stub.delta == 0 && g_stub.dq_tables.empty());
    const seco::SegTable& t = g_stub.dkdv_tables[0];
    CHECK(t.n == 1 && t.col_begin[0] == 0 && t.col_end[0] == 1024 && t.weight[0] == 1.f && t.tile_begin[1] == 8);
    CHECK(g_stub.last.n_splits > 1);                        // a short chunk: the cache range is divided
    g_stub.clear();
    CHECK(seco_chunk_attn_fwd(&d, FAKE, FAKE, FAKE, FAKE, FAKEF, nullptr, 0, nullptr) == SECO_OK);
    CHECK(g_stub.fwd == 1 && g_stub.last.n_splits == 1);    // no workspace: direct path
    const size_t wf = seco_workspace_bytes(&d, SECO_OP_FWD);
    CHECK(seco_chunk_attn_fwd(&d, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, wf, nullptr) == SECO_OK);
    CHECK(g_stub.last.n_splits > 1);
    // the same call on the library's own scratch array
    g_stub.clear();
    CHECK(seco_chunk_attn_bwd_noalloc(&d, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, nullptr) == SECO_OK);
    CHECK(g_stub.dq == 1 && g_stub.dkdv == 1 && g_stub.last.delta != nullptr);
    CHECK((reinterpret_cast<uintptr_t>(g_stub.last.delta) & 255u) == 0);
    seco_desc big = desc(SECO_BF16, 1 << 15, 0, 64, 8);
    CHECK(seco_workspace_bytes(&big, SECO_OP_BWD) > SECO_STATIC_SCRATCH_BYTES);
    CHECK(seco_chunk_attn_bwd_noalloc(&big, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, nullptr) ==
          SECO_ERR_TOO_LARGE);
    // fp32: the delta launch comes first
    seco_desc f = desc(SECO_F32, 100, 200, 4, 4, 64);
    g_stub.clear();
    CHECK(seco_chunk_attn_bwd(&f, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, FAKE,
                              seco_workspace_bytes(&f, SECO_OP_BWD), nullptr) == SECO_OK);
    CHECK(g_stub.delta == 1 && g_stub.dq == 1 && g_stub.dkdv == 1);
    CHECK(g_stub.dkdv_tables[0].tile_begin[1] == (300 + seco::kColTileF32 - 1) / seco::kColTileF32);
  }
  // ---- weights: merged runs, zero chunks skipped, ragged last chunk, more runs than one table holds ----
  {
    seco_desc d = desc(SECO_BF16, 160, 7 * 160);           // 8 chunks of 160 rows, kv_len 1280
    const size_t ws = seco_workspace_bytes(&d, SECO_OP_BWD);
    const float w[8] = {2.f, 2.f, 0.f, 0.5f, 0.f, 0.f, 2.f, 1.f};
    g_stub.clear();
    CHECK(spaco_chunk_attn_bwd(&d, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, w, 8, 160, FAKE, ws, nullptr) ==
          SECO_OK);
    CHECK(g_stub.dkdv == 1);
    const seco::SegTable& t = g_stub.dkdv_tables[0];
    CHECK(t.n == 4);
    CHECK(t.col_begin[0] == 0 && t.col_end[0] == 320 && t.weight[0] == 2.f && t.tile_begin[1] == 3);
    CHECK(t.col_begin[1] == 480 && t.col_end[1] == 640 && t.weight[1] == 0.5f && t.tile_begin[2] == 5);
    CHECK(t.col_begin[2] == 960 && t.col_end[2] == 1120 && t.weight[2] == 2.f && t.tile_begin[3] == 7);
    CHECK(t.col_begin[3] == 1120 && t.col_end[3] == 1280 && t.weight[3] == 1.f && t.tile_begin[4] == 9);
    const float bad[8] = {2.f, INFINITY, 0.f, 0.5f, 0.f, 0.f, 2.f, 1.f};
    CHECK(spaco_chunk_attn_bwd(&d, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, bad, 8, 160, FAKE, ws, nullptr) ==
          SECO_ERR_WEIGHTS);
    CHECK(spaco_chunk_attn_bwd(&d, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, w, 7, 160, FAKE, ws, nullptr) ==
          SECO_ERR_WEIGHTS);
    CHECK(spaco_chunk_attn_bwd(&d, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, w, 9, 160, FAKE, ws, nullptr) ==
          SECO_ERR_WEIGHTS);
    // all weights zero: the dQ pass runs, no dK/dV launch
    const float z[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    g_stub.clear();
    CHECK(spaco_chunk_attn_bwd(&d, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, z, 8, 160, FAKE, ws, nullptr) ==
          SECO_OK);
    CHECK(g_stub.dq == 1 && g_stub.dkdv == 0);
    // 110 chunks of 32 rows, every second weight zero, the others all different: 55 runs = 48 + 7
    seco_desc m = desc(SECO_BF16, 32, 109 * 32, 2, 1);
    std::vector<float> wm(110);
    for (int i = 0; i < 110; ++i) wm[i] = i % 2 ? 0.f : 1.f + 0.05f * i;
    wm[109] = 1.f;
    g_stub.clear();
    CHECK(spaco_chunk_attn_bwd(&m, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, wm.data(), 110, 32, FAKE,
                               seco_workspace_bytes(&m, SECO_OP_BWD), nullptr) == SECO_OK);
    CHECK(g_stub.dkdv == 2 && g_stub.dkdv_tables[0].n == 48 && g_stub.dkdv_tables[1].n == 8);
    int rows = 0;
    for (const auto& tb : g_stub.dkdv_tables) {
      CHECK(tb.tile_begin[tb.n] == tb.n);                   // one 32-row chunk = one (partly filled) column tile per run
      for (int i = 0; i < tb.n; ++i) rows += tb.col_end[i] - tb.col_begin[i];
    }
    CHECK(rows == 56 * 32);
    // column-weighted dQ: runs table, 48 runs at most
    const float wq[8] = {0.f, 3.f, 3.f, 0.f, 0.f, 1.25f, 0.f, 1.f};
    g_stub.clear();
    CHECK(spaco_chunk_attn_bwd_sparse_dq(&d, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, w, wq, 8, 160, FAKE, ws,
                                         nullptr) == SECO_OK);
    CHECK(g_stub.dq_tables.size() == 1 && g_stub.dq_tables[0].n == 3);
    CHECK(g_stub.dq_tables[0].col_begin[0] == 160 && g_stub.dq_tables[0].col_end[0] == 480);
    CHECK(g_stub.dq_tables[0].col_begin[2] == 1120 && g_stub.dq_tables[0].col_end[2] == 1280);
    const float ones[8] = {1, 1, 1, 1, 1, 1, 1, 1};
    g_stub.clear();
    CHECK(spaco_chunk_attn_bwd_sparse_dq(&d, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, w, ones, 8, 160, FAKE,
                                         ws, nullptr) == SECO_OK);
    CHECK(g_stub.dq_tables.empty());                        // all ones: the dense kernel
    std::vector<float> many(128), wone(128, 1.f);
    for (int i = 0; i < 128; ++i) many[i] = (float)(i % 2);
    seco_desc s4 = desc(SECO_BF16, 4, 127 * 4);
    CHECK(spaco_chunk_attn_bwd_sparse_dq(&s4, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, wone.data(),
                                         many.data(), 128, 4, FAKE, seco_workspace_bytes(&s4, SECO_OP_BWD), nullptr) ==
          SECO_ERR_TOO_LARGE);
  }
  // ---- transposed order: row runs ----
  {
    seco_desc d = desc(SECO_BF16, 128, 256);
    const size_t ws = seco_workspace_bytes(&d, SECO_OP_BWD);
    const float rw[6] = {1.f, 0.f, 4.f, 4.f, 0.f, 4.f};     // own chunk + 5 later chunks of 128 rows
    g_stub.clear();
    CHECK(spaco_chunk_attn_bwd_gather(&d, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, FAKEF, 1024, 640, rw, 6,
                                      128, FAKE, ws, nullptr) == SECO_OK);
    CHECK(g_stub.row_runs.size() == 1 && g_stub.row_runs[0].n == 3);
    CHECK(g_stub.row_runs[0].begin[1] == 256 && g_stub.row_runs[0].end[1] == 512 && g_stub.row_runs[0].log2w[1] == 2.f);
    CHECK(g_stub.dkdv_tables[0].col_begin[0] == 256 && g_stub.dkdv_tables[0].col_end[0] == 384);
    CHECK(spaco_chunk_attn_bwd_gather(&d, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, FAKEF, 1000, 640, rw, 6,
                                      128, FAKE, ws, nullptr) == SECO_ERR_RANGE);          // too few statistic rows
    CHECK(spaco_chunk_attn_bwd_gather(&d, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, FAKEF, 1024, 640, rw, 6,
                                      100, FAKE, ws, nullptr) == SECO_ERR_WEIGHTS);        // not a multiple of 64
    std::vector<float> alt(50);
    for (int i = 0; i < 50; ++i) alt[i] = (float)(1 - i % 2);
    seco_desc d64 = desc(SECO_BF16, 64, 0);
    CHECK(spaco_chunk_attn_bwd_gather(&d64, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, FAKEF, 3200, 49 * 64,
                                      alt.data(), 50, 64, FAKE, seco_workspace_bytes(&d64, SECO_OP_BWD), nullptr) ==
          SECO_ERR_TOO_LARGE);                                                              // 25 runs > 24
    g_stub.clear();
    CHECK(seco_chunk_attn_bwd_gather(&d, FAKE, FAKE, FAKE, FAKE, FAKEF, FAKE, FAKE, FAKEF, FAKEF, FAKEF, 1024, 640, FAKE, ws,
                                     nullptr) == SECO_OK);
    CHECK(g_stub.row_runs.empty() && g_stub.last.C == 768 && g_stub.last.stat_stride == 1024);
  }
  // ---- host policies: selection, weight vectors, launch plan ----
  {
    int32_t sel[16];
    for (uint64_t seed = 0; seed < 50; ++seed) {
      CHECK(spaco_select_chunks(seed, seed * 7, 16, 16, sel) == SECO_OK);
      for (int i = 0; i < 16; ++i) CHECK(sel[i] == 15 - i);
      CHECK(spaco_select_chunks(seed, 1, 13, 5, sel) == SECO_OK);
      for (int i = 0; i < 5; ++i) CHECK(sel[i] >= 0 && sel[i] < 13 && (i == 0 || sel[i] < sel[i - 1]));
    }
    CHECK(spaco_select_chunks(0, 0, 4, 5, sel) == SECO_ERR_RANGE);
    float w[16];
    int32_t s3[3] = {9, 4, 1};
    CHECK(spaco_chunk_weights(s3, 3, 9, 2.5f, w) == SECO_OK);
    CHECK(w[9] == 1.f && w[4] == 2.5f && w[1] == 2.5f && w[0] == 0.f && w[8] == 0.f);
    CHECK(spaco_gather_row_weights(s3, 3, 1, 12, 2.5f, w) == SECO_OK);
    CHECK(w[0] == 1.f && w[3] == 2.5f && w[8] == 2.5f && w[1] == 0.f && w[10] == 0.f);
    CHECK(spaco_percall_weights(3, 0, 15, 4, w) == SECO_OK);
    int nz = 0;
    for (int i = 0; i < 15; ++i) nz += w[i] != 0.f;
    CHECK(nz == 4 && w[15] == 1.f);
    int32_t out[64], n = -1;
    CHECK(spaco_select_bernoulli(5, 0, 64, 0.25, out, &n) == SECO_OK && n >= 0 && n <= 64);
    CHECK(spaco_select_bernoulli(5, 0, 64, 1.0, out, &n) == SECO_OK && n == 64);
    CHECK(spaco_compensation_factor(16, 4, 0.f) == 4.f && spaco_compensation_factor(16, 4, 2.f) == 2.f);
    CHECK(spaco_compensation_factor(4, 5, 0.f) < 0.f);
    int32_t plan[4];
    seco_desc c3 = desc(SECO_BF16, 2048, 14 * 2048, 32, 8);
    CHECK(seco_launch_plan(&c3, 15 * 16, plan) == SECO_OK && plan[0] == 1 && plan[1] == 512);
    seco_desc one = desc(SECO_BF16, 2048, 14 * 2048, 4, 1);
    CHECK(seco_launch_plan(&one, 15 * 16, plan) == SECO_OK && plan[0] > 1);
    CHECK(std::strcmp(seco_strerror(0), "ok") == 0 && std::strcmp(seco_strerror(-99), "unknown status") == 0);
    // appended rows, read-out, rotation: argument checks and dispatch
    seco_desc d = desc();
    g_stub.clear();
    CHECK(kv_append(&d, FAKE, FAKE, FAKE, FAKE, nullptr) == SECO_OK && g_stub.copy == 1);
    CHECK(kv_append_rope(&d, FAKE, FAKE, FAKE, FAKE, 500000.f, nullptr) == SECO_OK && g_stub.rope == 1 && g_stub.copy == 1);
    CHECK(kvgrad_readout_rope(&d, FAKEF, FAKEF, FAKE, FAKE, 2.f, 500000.f, nullptr) == SECO_OK && g_stub.rope == 2);
    CHECK(kv_append_rope(&d, FAKE, FAKE, FAKE, FAKE, 0.5f, nullptr) == SECO_ERR_RANGE);
    CHECK(kv_append(&d, FAKE, nullptr, nullptr, nullptr, nullptr) == SECO_ERR_NULL);
    CHECK(rope_rotate(&d, 0, FAKE, FAKE, 0, 10000.f, 0, nullptr) == SECO_ERR_RANGE);
    CHECK(kvgrad_readout(&d, FAKEF, FAKEF, FAKE, FAKE, INFINITY, nullptr) == SECO_ERR_RANGE);
  }
  std::puts("host sanitizer run: all checks passed");
  return 0;
}
