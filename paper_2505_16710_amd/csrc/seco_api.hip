// Host side of the C ABI: argument validation, segment tables and kernel dispatch.
// Nothing here allocates device memory or synchronises the stream.
#include <cmath>
#include <cstring>
#include <algorithm>
#include <mutex>
#include <vector>

#include "seco_internal.h"

namespace seco {

int device_cus() {
  static const int cus = [] {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      return n;
    (void)hipGetLastError();
    return kDefaultCUs;
  }();
  return cus;
}

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_desc(const seco_desc* d) {
  if (!d) return SECO_ERR_NULL;
  if (d->dtype != SECO_F32 && d->dtype != SECO_BF16) return SECO_ERR_DTYPE;
  if (d->batch < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->head_dim < 1 || d->chunk_len < 1 || d->q_start < 0)
    return SECO_ERR_SHAPE;
  if (d->n_q_heads % d->n_kv_heads != 0) return SECO_ERR_SHAPE;
  if ((int64_t)d->q_start + d->chunk_len > (int64_t)1 << 30) return SECO_ERR_TOO_LARGE;
  if (d->batch > 65535 || d->n_q_heads > 65535) return SECO_ERR_TOO_LARGE;
  if ((int64_t)d->batch * d->n_q_heads * ((d->chunk_len + 3) / 4) > (int64_t)1 << 31) return SECO_ERR_TOO_LARGE;
  if (d->dtype == SECO_BF16) {
    if (d->head_dim != 128) return SECO_ERR_HEAD_DIM;
  } else if (d->head_dim % 4 != 0 || d->head_dim > 256) {
    return SECO_ERR_HEAD_DIM;
  }
  if (!std::isfinite(d->softmax_scale) || !(d->softmax_scale > 0.f)) return SECO_ERR_SHAPE;
  return SECO_OK;
}

// strides in elements; rows must start on 16-byte boundaries
int check_strides(const int64_t s[3], int elem_bytes, int D) {
  const int64_t per16 = 16 / elem_bytes;
  for (int i = 0; i < 3; ++i)
    if (s[i] < 0 || s[i] % per16 != 0) return SECO_ERR_ALIGN;
  if (s[2] < D) return SECO_ERR_ALIGN;
  // the kernels address the rows of a tile with 32-bit byte offsets from the tile's first row
  if (s[2] > ((int64_t)1 << 22)) return SECO_ERR_TOO_LARGE;
  return SECO_OK;
}

AttnParams make_params(const seco_desc* d) {
  AttnParams p;
  std::memset(&p, 0, sizeof(p));
  p.B = d->batch;
  p.Hq = d->n_q_heads;
  p.Hkv = d->n_kv_heads;
  p.D = d->head_dim;
  p.C = d->chunk_len;
  p.q_start = d->q_start;
  p.G = d->n_q_heads / d->n_kv_heads;
  p.scale = d->softmax_scale;
  p.stat_stride = d->chunk_len;
  p.stat_off = 0;
  for (int i = 0; i < 3; ++i) {
    p.qs[i] = d->q_stride[i];
    p.os[i] = d->o_stride[i];
    p.kvs[i] = d->kv_stride[i];
    p.gs[i] = d->g_stride[i];
  }
  return p;
}

// one fp32 value per query row: delta; the bf16 path keeps a second array (LSE in the form its dK/dV kernel uses)
size_t row_stat_bytes(const seco_desc* d) {
  const size_t n = (size_t)d->batch * d->n_q_heads * d->chunk_len * sizeof(float);
  return (n + 255) & ~(size_t)255;
}
size_t delta_bytes(const seco_desc* d) { return (d->dtype == SECO_BF16 ? 2 : 1) * row_stat_bytes(d); }

size_t round256(size_t n) { return (n + 255) & ~(size_t)255; }

// workspace of the short-chunk (split) path; 0 when the shape never uses it
size_t split_part_bytes(const seco_desc* d) {   // partial O or partial dQ, fp32
  if (d->dtype != SECO_BF16) return 0;
  const SplitPlan pl = split_plan(d->batch, d->n_kv_heads, d->n_q_heads / d->n_kv_heads, d->chunk_len);
  if (pl.max_splits < 2) return 0;
  return round256((size_t)pl.max_splits * d->batch * d->n_q_heads * d->chunk_len * d->head_dim * sizeof(float));
}
size_t split_ml_bytes(const seco_desc* d) {     // (max, sum) of the forward partials
  if (split_part_bytes(d) == 0) return 0;
  const SplitPlan pl = split_plan(d->batch, d->n_kv_heads, d->n_q_heads / d->n_kv_heads, d->chunk_len);
  return round256((size_t)pl.max_splits * d->batch * d->n_q_heads * d->chunk_len * 2 * sizeof(float));
}
// number of splits of this call (1: direct path)
int splits_for(const seco_desc* d) {
  if (split_part_bytes(d) == 0) return 1;
  const SplitPlan pl = split_plan(d->batch, d->n_kv_heads, d->n_q_heads / d->n_kv_heads, d->chunk_len);
  return split_count(pl, d->q_start + d->chunk_len);
}

// workspace of the dK/dV pass for the column tiles it divides by query head (bf16, grouped heads only)
size_t tail_part_bytes(const seco_desc* d) {
  if (d->dtype != SECO_BF16 || d->n_q_heads / d->n_kv_heads < 2) return 0;
  return (size_t)device_cus() * 2 * kColTileBf16 * 128 * sizeof(float);   // at most one share per CU (tail_plan)
}
// the partial dQ of the split path and the divided dK/dV tiles are never live together: they share one region
size_t bwd_part_bytes(const seco_desc* d) { return std::max(split_part_bytes(d), tail_part_bytes(d)); }

int check_fwd_like(const seco_desc* d) {
  int rc = check_desc(d);
  if (rc) return rc;
  const int eb = d->dtype == SECO_BF16 ? 2 : 4;
  if ((rc = check_strides(d->q_stride, eb, d->head_dim))) return rc;
  if ((rc = check_strides(d->o_stride, eb, d->head_dim))) return rc;
  if ((rc = check_strides(d->kv_stride, eb, d->head_dim))) return rc;
  return SECO_OK;
}

int backward(const seco_desc* d, const void* q, const void* k, const void* v, const void* o, const float* lse,
             const void* d_o, void* d_q, float* gk, float* gv, const float* w, const float* wq, int32_t n_chunks,
             int32_t wlen, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_fwd_like(d);
  if (rc) return rc;
  if ((rc = check_strides(d->g_stride, 4, d->head_dim))) return rc;
  if (!q || !k || !v || !o || !lse || !d_o || !d_q || !gk || !gv) return SECO_ERR_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(d_o) || !aligned16(d_q) ||
      !aligned16(gk) || !aligned16(gv) || !aligned16(lse))
    return SECO_ERR_ALIGN;
  const int kv_len = d->q_start + d->chunk_len;
  const int tile = d->dtype == SECO_BF16 ? kColTileBf16 : kColTileF32;

  // Chunk weights: validated here, turned into column segments (maximal runs of cache rows with one non-zero
  // weight) when the dK/dV pass is launched below.
  if (w) {
    if (n_chunks < 1 || wlen < 1) return SECO_ERR_WEIGHTS;
    if ((int64_t)n_chunks * wlen < kv_len || (int64_t)(n_chunks - 1) * wlen >= kv_len) return SECO_ERR_WEIGHTS;
    for (int i = 0; i < n_chunks; ++i)
      if (!std::isfinite(w[i])) return SECO_ERR_WEIGHTS;
  }

  // Runs of the column-weighted dQ: the same construction over wq, which must be non-negative.  A single run
  // of weight 1 over every visible row is the exact dQ and takes the dense kernel.
  SegTable dq_runs;
  std::memset(&dq_runs, 0, sizeof(dq_runs));
  bool sparse_dq = false;
  if (wq) {
    for (int i = 0; i < n_chunks; ++i)
      if (!std::isfinite(wq[i]) || wq[i] < 0.f) return SECO_ERR_WEIGHTS;
    int n = 0;
    for (int i = 0; i < n_chunks; ++i) {
      if (wq[i] == 0.f) continue;
      const int b = (int)((int64_t)i * wlen), e = (int)std::min<int64_t>((int64_t)(i + 1) * wlen, kv_len);
      if (n > 0 && dq_runs.col_end[n - 1] == b && dq_runs.weight[n - 1] == wq[i]) {
        dq_runs.col_end[n - 1] = e;
      } else {
        if (n == kMaxSegments) return SECO_ERR_TOO_LARGE;
        dq_runs.col_begin[n] = b;
        dq_runs.col_end[n] = e;
        dq_runs.weight[n] = wq[i];
        ++n;
      }
    }
    dq_runs.n = n;
    sparse_dq = !(n == 1 && dq_runs.col_begin[0] == 0 && dq_runs.col_end[0] == kv_len && dq_runs.weight[0] == 1.f);
  }

  if (!ws || ws_bytes < delta_bytes(d) + bwd_part_bytes(d) || (reinterpret_cast<uintptr_t>(ws) & 255u))
    return SECO_ERR_WORKSPACE;

  AttnParams p = make_params(d);
  p.q = q; p.k = k; p.v = v; p.o = o; p.d_o = d_o; p.d_q = d_q;
  p.lse = const_cast<float*>(lse);
  p.delta = static_cast<float*>(ws);
  p.nlse2 = d->dtype == SECO_BF16 ? reinterpret_cast<float*>(static_cast<char*>(ws) + row_stat_bytes(d)) : nullptr;
  p.gk = gk; p.gv = gv;
  p.n_splits = splits_for(d);
  p.Cpad = (d->chunk_len + 31) / 32 * 32;
  p.part = reinterpret_cast<float*>(static_cast<char*>(ws) + delta_bytes(d));
  p.tail_part = tail_part_bytes(d) ? p.part : nullptr;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool bf16 = d->dtype == SECO_BF16;
  // delta = rowsum(dO * O): the bf16 dQ kernel computes it in its prologue (and stores it for the dK/dV kernel)
  if (!bf16 && (rc = launch_delta(p, d->dtype, s))) return rc;
  const SegTable* runs_arg = sparse_dq ? &dq_runs : nullptr;
  if ((rc = bf16 ? launch_dq_bf16(p, runs_arg, s) : launch_dq_f32(p, runs_arg, s))) return rc;
  // dK/dV pass: one launch per table of at most kMaxSegments runs (no host allocation: a table is launched as soon
  // as it is full, and every argument has been validated by now)
  SegTable seg;
  std::memset(&seg, 0, sizeof(seg));
  auto flush = [&]() -> int {
    const int st = seg.n == 0 ? SECO_OK : (bf16 ? launch_dkdv_bf16(p, seg, s) : launch_dkdv_f32(p, seg, s));
    std::memset(&seg, 0, sizeof(seg));
    return st;
  };
  auto add_rows = [&](int b, int e, float wt) -> int {      // rows [b, e) with weight wt != 0
    if (seg.n > 0 && seg.col_end[seg.n - 1] == b && seg.weight[seg.n - 1] == wt) {
      seg.col_end[seg.n - 1] = e;
      seg.tile_begin[seg.n] = seg.tile_begin[seg.n - 1] + (e - seg.col_begin[seg.n - 1] + tile - 1) / tile;
      return SECO_OK;
    }
    if (seg.n == kMaxSegments) {
      const int st = flush();
      if (st) return st;
    }
    seg.col_begin[seg.n] = b;
    seg.col_end[seg.n] = e;
    seg.weight[seg.n] = wt;
    seg.tile_begin[seg.n + 1] = seg.tile_begin[seg.n] + (e - b + tile - 1) / tile;
    ++seg.n;
    return SECO_OK;
  };
  if (!w) {
    if ((rc = add_rows(0, kv_len, 1.f))) return rc;
  } else {
    for (int i = 0; i < n_chunks; ++i) {
      if (w[i] == 0.f) continue;
      const int b = (int)((int64_t)i * wlen), e = (int)std::min<int64_t>((int64_t)(i + 1) * wlen, kv_len);
      if ((rc = add_rows(b, e, w[i]))) return rc;
    }
  }
  if ((rc = flush())) return rc;
  return SECO_OK;
}


// Backward of chunk i in the transposed order: dQ of the chunk as usual, and the chunk's own gK/gV rows from the
// query rows of the chunk and of every later row handed in (their -delta and -LSE are read from row_stats, where
// the dQ kernels of their own calls left them).
int backward_gather(const seco_desc* d, const void* q_rows, const void* k, const void* v, const void* o,
                    const float* lse, const void* d_o_rows, void* d_q, float* gk, float* gv, float* row_stats,
                    int64_t stat_rows, int32_t n_later_rows, const float* w, int32_t n_w, int32_t wlen, void* ws,
                    size_t ws_bytes, void* stream) {
  int rc = check_fwd_like(d);
  if (rc) return rc;
  if (d->dtype != SECO_BF16) return SECO_ERR_DTYPE;
  if ((rc = check_strides(d->g_stride, 4, d->head_dim))) return rc;
  if (!q_rows || !k || !v || !o || !lse || !d_o_rows || !d_q || !gk || !gv || !row_stats) return SECO_ERR_NULL;
  if (!aligned16(q_rows) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(d_o_rows) ||
      !aligned16(d_q) || !aligned16(gk) || !aligned16(gv) || !aligned16(lse) || !aligned16(row_stats))
    return SECO_ERR_ALIGN;
  if (n_later_rows < 0) return SECO_ERR_RANGE;
  const int64_t rows = (int64_t)d->chunk_len + n_later_rows;
  const int64_t last = (int64_t)d->q_start + rows;
  if (last > (int64_t)1 << 30) return SECO_ERR_TOO_LARGE;
  if ((int64_t)d->batch * d->n_q_heads * ((rows + 3) / 4) > (int64_t)1 << 31) return SECO_ERR_TOO_LARGE;
  if (stat_rows < last || stat_rows % 4 != 0) return SECO_ERR_RANGE;
  if (stat_rows > (int64_t)1 << 30) return SECO_ERR_TOO_LARGE;
  // runs of query rows with one non-zero weight (weights given per chunk of wlen rows, counted from the call's
  // first row); without weights every row counts once
  RowRuns rr;
  std::memset(&rr, 0, sizeof(rr));
  if (w) {
    if (n_w < 1 || wlen < 1 || wlen % 64 != 0) return SECO_ERR_WEIGHTS;
    if ((int64_t)n_w * wlen < rows || (int64_t)(n_w - 1) * wlen >= rows) return SECO_ERR_WEIGHTS;
    for (int i = 0; i < n_w; ++i)
      if (!std::isfinite(w[i]) || w[i] < 0.f) return SECO_ERR_WEIGHTS;
    for (int i = 0; i < n_w; ++i) {
      if (w[i] == 0.f) continue;
      const int b = (int)((int64_t)i * wlen), e = (int)std::min<int64_t>((int64_t)(i + 1) * wlen, rows);
      const float lw = std::log2(w[i]);
      if (rr.n > 0 && rr.end[rr.n - 1] == b && rr.log2w[rr.n - 1] == lw) {
        rr.end[rr.n - 1] = e;
      } else {
        if (rr.n == kMaxRowRuns) return SECO_ERR_TOO_LARGE;
        rr.begin[rr.n] = b;
        rr.end[rr.n] = e;
        rr.log2w[rr.n] = lw;
        ++rr.n;
      }
    }
  }
  if (!ws || ws_bytes < delta_bytes(d) + bwd_part_bytes(d) || (reinterpret_cast<uintptr_t>(ws) & 255u))
    return SECO_ERR_WORKSPACE;

  AttnParams p = make_params(d);
  p.q = q_rows; p.k = k; p.v = v; p.o = o; p.d_o = d_o_rows; p.d_q = d_q;
  p.lse = const_cast<float*>(lse);
  p.delta = row_stats;
  p.nlse2 = row_stats + (int64_t)d->batch * d->n_q_heads * stat_rows;
  p.stat_stride = (int)stat_rows;
  p.stat_off = d->q_start;
  p.gk = gk; p.gv = gv;
  p.n_splits = splits_for(d);
  p.Cpad = (d->chunk_len + 31) / 32 * 32;
  p.part = reinterpret_cast<float*>(static_cast<char*>(ws) + delta_bytes(d));
  p.tail_part = tail_part_bytes(d) ? p.part : nullptr;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if ((rc = launch_dq_bf16(p, nullptr, s))) return rc;
  // dK/dV: the query rows are the chunk's and the later ones, the cache rows the chunk's own
  AttnParams pr = p;
  pr.C = (int)rows;
  SegTable seg;
  std::memset(&seg, 0, sizeof(seg));
  seg.n = 1;
  seg.col_begin[0] = d->q_start;
  seg.col_end[0] = d->q_start + d->chunk_len;
  seg.weight[0] = 1.f;
  seg.tile_begin[1] = (d->chunk_len + kColTileBf16 - 1) / kColTileBf16;
  return w ? launch_dkdv_rows_bf16(pr, seg, rr, s) : launch_dkdv_bf16(pr, seg, s);
}

}  // namespace
}  // namespace seco

// ---- optional per-kernel timing ---------------------------------------------------------
namespace seco {
namespace {
struct ProfRecord { int kind; hipEvent_t start, stop; };
unsigned g_prof_mask = 0;   // bit k set: kernels of kind k are timed
std::vector<ProfRecord> g_prof;
}  // namespace

ProfScope::ProfScope(KernelKind kind, hipStream_t s) : stream(s), slot(-1) {
  if (!(g_prof_mask >> (unsigned)kind & 1u)) return;
  ProfRecord r;
  r.kind = kind;
  if (hipEventCreate(&r.start) != hipSuccess) return;
  if (hipEventCreate(&r.stop) != hipSuccess) { (void)hipEventDestroy(r.start); return; }
  (void)hipEventRecord(r.start, s);
  slot = (int)g_prof.size();
  g_prof.push_back(r);
}
ProfScope::~ProfScope() {
  if (slot >= 0) (void)hipEventRecord(g_prof[slot].stop, stream);
}
}  // namespace seco

using namespace seco;

extern "C" int seco_profile_enable_kinds(uint32_t kind_mask) {
  for (ProfRecord& r : g_prof) {
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  g_prof.clear();
  g_prof_mask = kind_mask & ((1u << SECO_PROFILE_KINDS) - 1u);
  return SECO_OK;
}

extern "C" int seco_profile_set_kinds(uint32_t kind_mask) {
  g_prof_mask = kind_mask & ((1u << SECO_PROFILE_KINDS) - 1u);
  return SECO_OK;
}

extern "C" int seco_profile_enable(int on) { return seco_profile_enable_kinds(on ? ~0u : 0u); }

extern "C" int seco_profile_read(double* total_ms, int64_t* launches) {
  if (!total_ms || !launches) return SECO_ERR_NULL;
  for (int i = 0; i < SECO_PROFILE_KINDS; ++i) {
    total_ms[i] = 0.0;
    launches[i] = 0;
  }
  int rc = SECO_OK;
  for (ProfRecord& r : g_prof) {
    float ms = 0.f;
    if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess)
      rc = SECO_ERR_LAUNCH;
    total_ms[r.kind] += ms;
    launches[r.kind] += 1;
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  g_prof.clear();
  return rc;
}

extern "C" int seco_device_info(int32_t* compute_units_host, int32_t* max_clock_khz_host) {
  if (!compute_units_host || !max_clock_khz_host) return SECO_ERR_NULL;
  int dev = 0, cus = 0, khz = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev) != hipSuccess) {
    (void)hipGetLastError();
    return SECO_ERR_LAUNCH;
  }
  *compute_units_host = cus;
  *max_clock_khz_host = khz;
  return SECO_OK;
}

extern "C" size_t seco_workspace_bytes(const seco_desc* desc, int op) {
  if (check_desc(desc) != SECO_OK) return (size_t)-1;
  if (op == SECO_OP_FWD) return split_part_bytes(desc) + split_ml_bytes(desc);
  if (op == SECO_OP_BWD) return delta_bytes(desc) + bwd_part_bytes(desc);
  return (size_t)-1;
}

extern "C" int seco_launch_plan(const seco_desc* desc, int32_t n_col_tiles, int32_t* plan_host) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (!plan_host) return SECO_ERR_NULL;
  if (desc->dtype != SECO_BF16) return SECO_ERR_DTYPE;
  if (n_col_tiles < 0) return SECO_ERR_RANGE;
  const int G = desc->n_q_heads / desc->n_kv_heads;
  const SplitPlan pl = split_plan(desc->batch, desc->n_kv_heads, G, desc->chunk_len);
  const int n_splits = splits_for(desc);
  plan_host[0] = n_splits;
  plan_host[1] = n_splits > 1 ? pl.items : desc->batch * desc->n_q_heads * ((desc->chunk_len + 127) / 128);
  const TailPlan tp = tail_plan(desc->batch * desc->n_kv_heads, n_col_tiles, G, desc->chunk_len);
  plan_host[2] = tp.hs > 1 ? tp.n_tiles : 0;
  plan_host[3] = tp.hs;
  return SECO_OK;
}

extern "C" int seco_chunk_attn_fwd(const seco_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                                   void* o, float* lse, void* ws, size_t ws_bytes, void* hip_stream) {
  int rc = check_fwd_like(desc);
  if (rc) return rc;
  if (!q || !k_cache || !v_cache || !o || !lse) return SECO_ERR_NULL;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(o) || !aligned16(lse))
    return SECO_ERR_ALIGN;
  AttnParams p = make_params(desc);
  p.q = q; p.k = k_cache; p.v = v_cache; p.o_out = o; p.lse = lse;
  p.n_splits = 1;
  p.Cpad = (desc->chunk_len + 31) / 32 * 32;
  const size_t part_bytes = split_part_bytes(desc);
  if (part_bytes && ws && !(reinterpret_cast<uintptr_t>(ws) & 255u) && ws_bytes >= part_bytes + split_ml_bytes(desc)) {
    p.n_splits = splits_for(desc);
    p.part = static_cast<float*>(ws);
    p.part_ml = reinterpret_cast<float*>(static_cast<char*>(ws) + part_bytes);
  }
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  return desc->dtype == SECO_BF16 ? launch_fwd_bf16(p, s) : launch_fwd_f32(p, s);
}

extern "C" int seco_chunk_attn_bwd(const seco_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                                   const void* o, const float* lse, const void* d_o, void* d_q, float* gk, float* gv,
                                   void* ws, size_t ws_bytes, void* hip_stream) {
  return backward(desc, q, k_cache, v_cache, o, lse, d_o, d_q, gk, gv, nullptr, nullptr, 0, 0, ws, ws_bytes, hip_stream);
}

extern "C" int spaco_chunk_attn_bwd(const seco_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                                    const void* o, const float* lse, const void* d_o, void* d_q, float* gk, float* gv,
                                    const float* chunk_weight_host, int32_t n_chunks, int32_t weight_chunk_len, void* ws,
                                    size_t ws_bytes, void* hip_stream) {
  if (!chunk_weight_host) return SECO_ERR_NULL;
  return backward(desc, q, k_cache, v_cache, o, lse, d_o, d_q, gk, gv, chunk_weight_host, nullptr, n_chunks,
                  weight_chunk_len, ws, ws_bytes, hip_stream);
}

extern "C" int seco_chunk_attn_bwd_gather(const seco_desc* desc, const void* q_rows, const void* k_cache,
                                          const void* v_cache, const void* o, const float* lse, const void* d_o_rows,
                                          void* d_q, float* gk, float* gv, float* row_stats, int64_t stat_rows,
                                          int32_t n_later_rows, void* ws, size_t ws_bytes, void* hip_stream) {
  return backward_gather(desc, q_rows, k_cache, v_cache, o, lse, d_o_rows, d_q, gk, gv, row_stats, stat_rows,
                         n_later_rows, nullptr, 0, 0, ws, ws_bytes, hip_stream);
}

extern "C" int spaco_chunk_attn_bwd_gather(const seco_desc* desc, const void* q_rows, const void* k_cache,
                                           const void* v_cache, const void* o, const float* lse, const void* d_o_rows,
                                           void* d_q, float* gk, float* gv, float* row_stats, int64_t stat_rows,
                                           int32_t n_later_rows, const float* row_weight_host, int32_t n_row_chunks,
                                           int32_t weight_chunk_len, void* ws, size_t ws_bytes, void* hip_stream) {
  if (!row_weight_host) return SECO_ERR_NULL;
  return backward_gather(desc, q_rows, k_cache, v_cache, o, lse, d_o_rows, d_q, gk, gv, row_stats, stat_rows,
                         n_later_rows, row_weight_host, n_row_chunks, weight_chunk_len, ws, ws_bytes, hip_stream);
}

extern "C" int spaco_chunk_attn_bwd_sparse_dq(const seco_desc* desc, const void* q, const void* k_cache,
                                              const void* v_cache, const void* o, const float* lse, const void* d_o,
                                              void* d_q, float* gk, float* gv, const float* chunk_weight_host,
                                              const float* dq_weight_host, int32_t n_chunks, int32_t weight_chunk_len,
                                              void* ws, size_t ws_bytes, void* hip_stream) {
  if (!chunk_weight_host || !dq_weight_host) return SECO_ERR_NULL;
  return backward(desc, q, k_cache, v_cache, o, lse, d_o, d_q, gk, gv, chunk_weight_host, dq_weight_host, n_chunks,
                  weight_chunk_len, ws, ws_bytes, hip_stream);
}

// ---- seco_chunk_attn_bwd for callers that cannot allocate -------------------------------------------------------
// The workspace of the backward (row statistics, partial dQ of the short-chunk path, shared-out dK/dV tiles) lives
// in a device array of the library itself.  Each GPU the library runs on holds its own copy of the array at its
// own address, which is looked up once per device, with that device current, and used from then on; the array's
// name itself is never handed to a kernel or to a memory call.
namespace {
constexpr size_t kScratchBytes = SECO_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];   // address of `scratch` on device i, or NULL before the first call there

int scratch_address(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return SECO_ERR_LAUNCH;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return SECO_ERR_LAUNCH;
    }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return SECO_OK;
}
}  // namespace

extern "C" int seco_chunk_attn_bwd_noalloc(const seco_desc* desc, const void* q, const void* k_cache,
                                           const void* v_cache, const void* o, const float* lse, const void* d_o,
                                           void* d_q, float* gk, float* gv, void* hip_stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (delta_bytes(desc) + bwd_part_bytes(desc) > kScratchBytes) return SECO_ERR_TOO_LARGE;
  void* ws = nullptr;
  if ((rc = scratch_address(&ws))) return rc;
  // every value the kernels read from the scratch array is written earlier in the same call (row statistics by the
  // dQ kernel, partial sums by the kernels whose merge reads them), so nothing has to be cleared between calls
  return backward(desc, q, k_cache, v_cache, o, lse, d_o, d_q, gk, gv, nullptr, nullptr, 0, 0, ws, kScratchBytes,
                  hip_stream);
}

namespace {
int check_rows(const seco_desc* d, int64_t r0, int64_t r1) {
  int rc = check_desc(d);
  if (rc) return rc;
  if ((rc = check_strides(d->g_stride, 4, d->head_dim))) return rc;
  if (r0 < 0 || r1 < r0 || r1 > ((int64_t)1 << 40)) return SECO_ERR_RANGE;
  return SECO_OK;
}
}  // namespace

extern "C" int kvgrad_zero(const seco_desc* desc, float* gk, float* gv, int64_t row_begin, int64_t row_end,
                           void* hip_stream) {
  int rc = check_rows(desc, row_begin, row_end);
  if (rc) return rc;
  if ((gk && !aligned16(gk)) || (gv && !aligned16(gv))) return SECO_ERR_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  return launch_kvgrad_zero(gk, gv, desc->batch, desc->n_kv_heads, desc->head_dim, desc->g_stride, row_begin, row_end, s);
}

extern "C" int kvgrad_accumulate(const seco_desc* desc, float* dst_k, float* dst_v, const float* src_k,
                                 const float* src_v, float scale, int64_t row_begin, int64_t row_end, void* hip_stream) {
  int rc = check_rows(desc, row_begin, row_end);
  if (rc) return rc;
  if ((dst_k == nullptr) != (src_k == nullptr) || (dst_v == nullptr) != (src_v == nullptr)) return SECO_ERR_NULL;
  if ((dst_k && dst_k == src_k) || (dst_v && dst_v == src_v)) return SECO_ERR_RANGE;
  for (const void* ptr : {(const void*)dst_k, (const void*)dst_v, (const void*)src_k, (const void*)src_v})
    if (ptr && !aligned16(ptr)) return SECO_ERR_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  return launch_kvgrad_axpy(dst_k, dst_v, src_k, src_v, scale, desc->batch, desc->n_kv_heads, desc->head_dim,
                            desc->g_stride, row_begin, row_end, s);
}

// ---- cache append and gradient hand-over (appendix listing) ---------------------------------------------------------
namespace {
int check_append_like(const seco_desc* d, bool with_g) {
  int rc = check_desc(d);
  if (rc) return rc;
  const int eb = d->dtype == SECO_BF16 ? 2 : 4;
  if ((rc = check_strides(d->q_stride, eb, d->head_dim))) return rc;
  if (with_g) {
    if ((rc = check_strides(d->g_stride, 4, d->head_dim))) return rc;
    if (d->head_dim % 8 != 0) return SECO_ERR_HEAD_DIM;
  } else if ((rc = check_strides(d->kv_stride, eb, d->head_dim))) {
    return rc;
  }
  return SECO_OK;
}
}  // namespace

extern "C" int kv_append(const seco_desc* desc, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                         void* hip_stream) {
  int rc = check_append_like(desc, false);
  if (rc) return rc;
  if ((k_new == nullptr) != (k_cache == nullptr) || (v_new == nullptr) != (v_cache == nullptr)) return SECO_ERR_NULL;
  for (const void* ptr : {k_new, v_new, (const void*)k_cache, (const void*)v_cache})
    if (ptr && !aligned16(ptr)) return SECO_ERR_ALIGN;
  const int eb = desc->dtype == SECO_BF16 ? 2 : 4;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  return launch_rows_copy(k_cache, v_cache, k_new, v_new, eb, desc->batch, desc->n_kv_heads, desc->chunk_len,
                          desc->head_dim, desc->kv_stride, desc->q_stride, desc->q_start, s);
}

extern "C" int kvgrad_readout(const seco_desc* desc, const float* gk, const float* gv, void* d_k_new, void* d_v_new,
                              float scaler, void* hip_stream) {
  int rc = check_append_like(desc, true);
  if (rc) return rc;
  if ((gk == nullptr) != (d_k_new == nullptr) || (gv == nullptr) != (d_v_new == nullptr)) return SECO_ERR_NULL;
  if (!std::isfinite(scaler)) return SECO_ERR_RANGE;
  for (const void* ptr : {(const void*)gk, (const void*)gv, (const void*)d_k_new, (const void*)d_v_new})
    if (ptr && !aligned16(ptr)) return SECO_ERR_ALIGN;
  const bool bf16 = desc->dtype == SECO_BF16;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  return launch_readout(d_k_new, d_v_new, gk, gv, scaler, bf16, desc->batch, desc->n_kv_heads, desc->chunk_len,
                        desc->head_dim, desc->q_stride, desc->g_stride, desc->q_start, s);
}

// ---- rotary position embedding fused into append / read-out (not part of the paper; see seco.h) -----------------------
namespace {
int check_rope(const seco_desc* d, float base) {
  if (d->head_dim % 8 != 0) return SECO_ERR_HEAD_DIM;
  if (!std::isfinite(base) || !(base > 1.f)) return SECO_ERR_RANGE;
  return SECO_OK;
}
}  // namespace

extern "C" int kv_append_rope(const seco_desc* desc, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                              float rope_base, void* hip_stream) {
  int rc = check_append_like(desc, false);
  if (rc) return rc;
  if ((rc = check_rope(desc, rope_base))) return rc;
  if ((k_new == nullptr) != (k_cache == nullptr) || (v_new == nullptr) != (v_cache == nullptr)) return SECO_ERR_NULL;
  for (const void* ptr : {k_new, v_new, (const void*)k_cache, (const void*)v_cache})
    if (ptr && !aligned16(ptr)) return SECO_ERR_ALIGN;
  const int eb = desc->dtype == SECO_BF16 ? 2 : 4;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  (void)eb;
  // one launch: the keys rotated, the values copied (scale 1 and equal types: the conversion is the identity)
  return launch_rope_rows(k_cache, k_new, v_cache, v_new, desc->dtype, desc->dtype, desc->batch, desc->n_kv_heads,
                          desc->chunk_len, desc->head_dim, desc->kv_stride, desc->q_stride, desc->q_start, 0,
                          desc->q_start, rope_base, false, 1.f, s);
}

extern "C" int kvgrad_readout_rope(const seco_desc* desc, const float* gk, const float* gv, void* d_k_new,
                                   void* d_v_new, float scaler, float rope_base, void* hip_stream) {
  int rc = check_append_like(desc, true);
  if (rc) return rc;
  if ((rc = check_rope(desc, rope_base))) return rc;
  if ((gk == nullptr) != (d_k_new == nullptr) || (gv == nullptr) != (d_v_new == nullptr)) return SECO_ERR_NULL;
  if (!std::isfinite(scaler)) return SECO_ERR_RANGE;
  for (const void* ptr : {(const void*)gk, (const void*)gv, (const void*)d_k_new, (const void*)d_v_new})
    if (ptr && !aligned16(ptr)) return SECO_ERR_ALIGN;
  const bool bf16 = desc->dtype == SECO_BF16;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  (void)bf16;
  // one launch: the key gradient scaled and turned back, the value gradient scaled
  return launch_rope_rows(d_k_new, gk, d_v_new, gv, SECO_F32, desc->dtype, desc->batch, desc->n_kv_heads,
                          desc->chunk_len, desc->head_dim, desc->q_stride, desc->g_stride, 0, desc->q_start,
                          desc->q_start, rope_base, true, scaler, s);
}

extern "C" int rope_rotate(const seco_desc* desc, int32_t n_heads, const void* x_in, void* x_out, int64_t pos_start,
                           float rope_base, int32_t inverse, void* hip_stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  const int eb = desc->dtype == SECO_BF16 ? 2 : 4;
  if ((rc = check_strides(desc->q_stride, eb, desc->head_dim))) return rc;
  if ((rc = check_strides(desc->o_stride, eb, desc->head_dim))) return rc;
  if ((rc = check_rope(desc, rope_base))) return rc;
  if (!x_in || !x_out) return SECO_ERR_NULL;
  if (!aligned16(x_in) || !aligned16(x_out)) return SECO_ERR_ALIGN;
  if (n_heads < 1 || n_heads > 65535 || pos_start < 0 || pos_start > ((int64_t)1 << 40)) return SECO_ERR_RANGE;
  return launch_rope_rows(x_out, x_in, nullptr, nullptr, desc->dtype, desc->dtype, desc->batch, n_heads, desc->chunk_len, desc->head_dim,
                          desc->o_stride, desc->q_stride, 0, 0, pos_start, rope_base, inverse != 0, 1.f,
                          static_cast<hipStream_t>(hip_stream));
}
