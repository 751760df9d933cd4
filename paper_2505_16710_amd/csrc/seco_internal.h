// Internal declarations shared by the host entry points and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "seco.h"

namespace seco {

// Everything a kernel needs to know about one chunk call (validated by the host side).
struct AttnParams {
  const void* q;
  const void* k;
  const void* v;
  const void* o;
  const void* d_o;
  void* o_out;
  void* d_q;
  float* lse;        // [B, Hq, C] contiguous
  float* delta;      // [B, Hq, stat_stride], backward only: rowsum(dO * O); NEGATED on the bf16 path
  float* nlse2;      // bf16 backward: -LSE / scale, [B, Hq, stat_stride], written by the dQ kernel for the dK/dV kernel
  int stat_stride;   // rows per (batch, head) of delta / nlse2: C (workspace of one call), or the length of
  int stat_off;      // arrays kept for the whole sequence, in which this call's first query row sits at stat_off
  float* gk;
  float* gv;
  float* part;       // split path: partial O (forward) or partial dQ (backward), fp32 [n_splits, B, Hq, C, D]
  float* part_ml;    // split path, forward: (reference max in log2 units, sum) per partial row, [n_splits, B, Hq, C, 2]
  float* tail_part;  // dK/dV pass: sums of the column tiles divided by query head (workspace), or NULL
  int n_splits;      // > 1 selects the split path
  int Cpad;          // C rounded up to 32: rows per head in the packed row space of the split path
  int B, Hq, Hkv, D, C, q_start, G;
  float scale;
  int64_t qs[3], os[3], kvs[3], gs[3];
};

// Column segments of the dK/dV pass: a run of cache rows that share one weight.
// The table travels by value in the kernel arguments, so no device memory or
// host-to-device copy is needed for SpaCO's selection.
constexpr int kMaxSegments = 48;
struct SegTable {
  int n;
  int col_begin[kMaxSegments];
  int col_end[kMaxSegments];
  float weight[kMaxSegments];
  int tile_begin[kMaxSegments + 1];  // prefix sum of column tiles, in units of the launcher's tile width
};

// Runs of query rows of the dK/dV pass in the transposed order: rows [begin, end) relative to the call's first
// query row, begin a multiple of 64, ascending and disjoint; the probabilities of a run's rows are scaled by its
// weight (log2w = log2 of the weight).  By value in the kernel arguments, like the column segments.
constexpr int kMaxRowRuns = 24;
struct RowRuns {
  int n;
  int begin[kMaxRowRuns];
  int end[kMaxRowRuns];
  float log2w[kMaxRowRuns];
};

// Split path of the bf16 forward and dQ kernels (short chunks): the rows of the G heads of a KV head are packed
// into row tiles of 128, and the visible cache rows of a tile are divided among several workgroups.
struct SplitPlan {
  int n_mtiles;     // row tiles per (batch, KV head)
  int items;        // B * Hkv * n_mtiles
  int max_splits;   // 1: the split path is never used for this shape
};
// Compute units of the current device, asked of the device once per process (kDefaultCUs, an MI355X's 256, when
// there is no device to ask, as in host-only use of the planning calls).  Every launch-shape decision below and in the launchers counts
// workgroups against this one number; seco_device_info reports the same attribute.
constexpr int kDefaultCUs = 256;
int device_cus();

inline SplitPlan split_plan(int B, int Hkv, int G, int C) {
  SplitPlan pl;
  const int cus = device_cus();
  const int cpad = (C + 31) / 32 * 32;
  pl.n_mtiles = (G * cpad + 127) / 128;
  pl.items = B * Hkv * pl.n_mtiles;
  pl.max_splits = pl.items >= cus ? 1 : (2 * cus + pl.items - 1) / pl.items;
  if (pl.max_splits > 64) pl.max_splits = 64;
  return pl;
}
// number of splits for a call that sees kv_len cache rows: every split gets at least 4 tiles of 64 rows
inline int split_count(const SplitPlan& pl, int kv_len) {
  const int by_len = (kv_len + 63) / 64 / 4;
  const int n = pl.max_splits < by_len ? pl.max_splits : by_len;
  return n < 2 ? 1 : n;
}
int launch_fwd_merge(const AttnParams& p, hipStream_t s);   // O, LSE from the partials
int launch_dq_merge(const AttnParams& p, hipStream_t s);    // dQ = scale * sum of the partials, in split order

// Last round of the bf16 dK/dV pass.  One workgroup fills a CU, so n_units * n_ctiles column tiles run in rounds of
// one workgroup per CU; when the last round would hold at most half of that, the last n_tiles column tiles of every
// (batch, KV head) are divided among hs workgroups by query head (hs = 1: nothing is divided).  A share keeps
// at least 512 query rows, and all shares together fit one round (device_cus() shares at most, which is also what
// the workspace for their partial sums is sized for).
struct TailPlan {
  int n_tiles;
  int hs;
};
inline TailPlan tail_plan(int n_units, int n_ctiles, int G, int C) {
  TailPlan tp{0, 1};
  const int round = device_cus();
  const int64_t items = (int64_t)n_units * n_ctiles;
  const int tail = (int)(items % round);
  if (tail == 0 || tail > round / 2) return tp;
  const int n_tiles = (tail + n_units - 1) / n_units;
  for (int hs = 4; hs >= 2; hs >>= 1) {
    if (G % hs != 0 || (int64_t)n_units * n_tiles * hs > round) continue;
    if ((int64_t)C * (G / hs) < 512) continue;
    tp.n_tiles = n_tiles;
    tp.hs = hs;
    break;
  }
  return tp;
}

// fp32 reference-grade kernels (any head_dim that is a multiple of 4, up to 256)
int launch_fwd_f32(const AttnParams& p, hipStream_t s);
int launch_dq_f32(const AttnParams& p, const SegTable* dq_runs, hipStream_t s);   // dq_runs as in launch_dq_bf16
int launch_dkdv_f32(const AttnParams& p, const SegTable& seg, hipStream_t s);
constexpr int kColTileF32 = 4;     // columns per workgroup in launch_dkdv_f32

// bf16 matrix-core kernels (head_dim 128)
int launch_fwd_bf16(const AttnParams& p, hipStream_t s);
// the 4-wavefront forward kernel (its own translation unit); split: the short-chunk variant that writes partials
int launch_fwd4_bf16(const AttnParams& p, bool split, int n_mtiles, int total, hipStream_t s);
int launch_fwd4_split_bf16(const AttnParams& p, int n_mtiles, int total, hipStream_t s);
// dq_runs: NULL for all visible cache rows with weight 1; else runs of cache rows (ascending, disjoint), each with
// a positive weight (tile_begin is not used)
int launch_dq_bf16(const AttnParams& p, const SegTable* dq_runs, hipStream_t s);
int launch_dkdv_bf16(const AttnParams& p, const SegTable& seg, hipStream_t s);
// the same with the query rows taken from runs (p.C: number of rows that may be addressed from p.q / p.d_o)
int launch_dkdv_rows_bf16(const AttnParams& p, const SegTable& seg, const RowRuns& rr, hipStream_t s);
#ifndef SECO_DKDV_COLS
#define SECO_DKDV_COLS 128
#endif
constexpr int kColTileBf16 = SECO_DKDV_COLS;  // columns per workgroup in launch_dkdv_bf16

// delta[r] = sum_d dO[r,d] * O[r,d]
int launch_delta(const AttnParams& p, int dtype, hipStream_t s);

// Bandwidth-bound helpers; each takes a pair of tensors (gK and gV, keys and values) handled by one launch,
// a NULL member of the pair is skipped.
int launch_kvgrad_zero(float* ga, float* gb, int B, int H, int D, const int64_t gs[3], int64_t r0, int64_t r1,
                       hipStream_t s);
int launch_kvgrad_axpy(float* da, float* db, const float* sa, const float* sb, float scale, int B, int H, int D,
                       const int64_t gs[3], int64_t r0, int64_t r1, hipStream_t s);

// rows [r0, r0 + C) of a [B, H, *, D] array <- a [B, H, C, D] array (same element type, eb bytes per element)
int launch_rows_copy(void* da, void* db, const void* sa, const void* sb, int eb, int B, int H, int C, int D,
                     const int64_t dst_s[3], const int64_t src_s[3], int64_t r0, hipStream_t s);
// out[B, H, C, D] (bf16 or fp32) = scaler * g[rows r0 .. r0 + C) (fp32)
int launch_readout(void* oa, void* ob, const float* ga, const float* gb, float scaler, bool bf16, int B, int H, int C,
                   int D, const int64_t out_s[3], const int64_t gs[3], int64_t r0, hipStream_t s);

// out rows [out_r0, out_r0 + C) <- rotary embedding (or its inverse) of scale * in rows [in_r0, in_r0 + C), row r at
// position pos0 + r; in_kind / out_kind: SECO_F32 or SECO_BF16 (bf16 -> f32 is not needed and not provided).
// plain_out / plain_in: a second pair with the same strides and row ranges that is scaled and converted but not
// rotated, in the same launch; either pair may be NULL (skipped).
int launch_rope_rows(void* out, const void* in, void* plain_out, const void* plain_in, int in_kind, int out_kind, int B,
                     int H, int C, int D, const int64_t out_s[3], const int64_t in_s[3], int64_t out_r0, int64_t in_r0,
                     int64_t pos0, float base, bool inverse, float scale, hipStream_t s);

// Optional per-kernel timing (seco_profile_enable): a scope brackets one launch with HIP events
// on the launch stream.  Disabled by default; then a scope costs one branch.
enum KernelKind { kKernelFwd = 0, kKernelDelta, kKernelDq, kKernelDkdv, kKernelKvgrad, kKernelMerge, kKernelKinds };
struct ProfScope {
  ProfScope(KernelKind kind, hipStream_t s);
  ~ProfScope();
  hipStream_t stream;
  int slot;
};

inline int launch_status() { return hipGetLastError() == hipSuccess ? SECO_OK : SECO_ERR_LAUNCH; }

}  // namespace seco
