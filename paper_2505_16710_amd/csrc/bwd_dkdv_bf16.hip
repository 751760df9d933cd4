// dK/dV of one chunk, bf16 matrix cores, accumulated into the persistent fp32 KV-gradient
// buffers (Alg. 1 second loop; Alg. 2 with per-chunk weights):
//   gV[c] += w * sum_{heads of the group} P^T dO      gK[c] += w * s * sum_{heads} dS^T Q
//
// Column-parallel: one workgroup is the only writer of 128 cache rows of one (batch, KV head),
// so the read-modify-write of gK/gV needs no atomics and the result is deterministic.
// Each wavefront owns 32 of those cache rows: it keeps their K^T and V^T fragments and the
// dK and dV accumulators (32 x 128 fp32 each) in registers and loops over the group's query
// heads and over 32-row tiles of Q and dO, which stream through swizzled, double-buffered
// LDS shared by the four wavefronts.  Scores are computed as S = Q K^T (C layout: lane =
// cache row), so that P and dS feed dV += P^T dO and dK += dS^T Q as A operands straight from
// registers, with dO and Q delivered by the LDS transpose read.
//
// Column tiles are enumerated from a by-value segment table (runs of cache rows that share
// one non-zero weight); SpaCO's unselected chunks simply have no tiles.
#include "mfma_tiles.h"
#include "seco_internal.h"

namespace seco {
namespace {

constexpr int BQ = 32;                       // query rows per LDS tile
constexpr int kTileBytes = BQ * kRowBytes;   // 8 KiB
constexpr int kStageBytes = 2 * kTileBytes + 2 * BQ * 4;  // Q, dO, lse, delta

__global__ __launch_bounds__(256, 1) void dkdv_bf16_kernel(AttnParams p, SegTable seg, int total_items) {
  __shared__ __attribute__((aligned(16))) char smem_raw[2 * kStageBytes];
  lds_char* smem = (lds_char*)smem_raw;

  const int item = xcd_item(blockIdx.x, total_items);
  if (item < 0) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  // item -> (batch, kv head, column tile)
  const int n_ctiles = seg.tile_begin[seg.n];
  const int tile = item % n_ctiles;
  const int kvh = (item / n_ctiles) % p.Hkv, b = item / (n_ctiles * p.Hkv);
  int si = 0;
  while (si + 1 < seg.n && tile >= seg.tile_begin[si + 1]) ++si;
  const int c0 = seg.col_begin[si] + (tile - seg.tile_begin[si]) * kColTileBf16;
  const int c_end = min(c0 + kColTileBf16, seg.col_end[si]);
  const float weight = seg.weight[si];

  const int kv_len = p.q_start + p.C;
  const int n0 = c0 + wave * 32;   // first cache row of this wavefront
  const int col = n0 + l32;        // this lane's cache row in the score tile
  const __bf16* kptr = static_cast<const __bf16*>(p.k) + b * p.kvs[0] + kvh * p.kvs[1] + (int64_t)min(col, kv_len - 1) * p.kvs[2];
  const __bf16* vptr = static_cast<const __bf16*>(p.v) + b * p.kvs[0] + kvh * p.kvs[1] + (int64_t)min(col, kv_len - 1) * p.kvs[2];
  bf16x8 kf[8], vf[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    kf[t] = *reinterpret_cast<const bf16x8*>(kptr + 16 * t + 8 * g);
    vf[t] = *reinterpret_cast<const bf16x8*>(vptr + 16 * t + 8 * g);
  }

  // query-row tiles that see at least one cache row of this workgroup
  const int rt0 = max(0, c0 - p.q_start) / BQ;
  const int n_rt = (p.C + BQ - 1) / BQ - rt0;
  const int n_iter = n_rt * p.G;
  const float c = p.scale * kLog2e;

  // staging: thread owns chunks tid and tid + 256 of the 32 x 16 chunk tiles
  bf16x8 qreg[2], doreg[2];
  float stat = 0.f;
  auto fetch = [&](int it) {
    const int h = kvh * p.G + it / n_rt;
    const int r0 = (rt0 + it % n_rt) * BQ;
    const __bf16* qb = static_cast<const __bf16*>(p.q) + b * p.qs[0] + h * p.qs[1];
    const __bf16* dob = static_cast<const __bf16*>(p.d_o) + b * p.os[0] + h * p.os[1];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int cid = tid + 256 * i, r = min(r0 + (cid >> 4), p.C - 1), ch = cid & 15;
      qreg[i] = *reinterpret_cast<const bf16x8*>(qb + (int64_t)r * p.qs[2] + ch * 8);
      doreg[i] = *reinterpret_cast<const bf16x8*>(dob + (int64_t)r * p.os[2] + ch * 8);
    }
    if (tid < 64) {
      const int r = r0 + (tid & 31);
      const int64_t idx = ((int64_t)b * p.Hq + h) * p.C + min(r, p.C - 1);
      // rows past the chunk get LSE = +inf so that their probabilities vanish
      if (tid < 32) stat = r < p.C ? p.lse[idx] * kLog2e : INFINITY;
      else stat = p.delta[idx];
    }
  };
  auto stash = [&](int buf) {
    lds_char* qt = smem + buf * kStageBytes;
    lds_char* dot = qt + kTileBytes;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int cid = tid + 256 * i;
      lds_store16(qt, cid >> 4, cid & 15, qreg[i]);
      lds_store16(dot, cid >> 4, cid & 15, doreg[i]);
    }
    if (tid < 64) *reinterpret_cast<SECO_LDS float*>(qt + 2 * kTileBytes + tid * 4) = stat;
  };

  f32x16 dk[4], dv[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) dk[db][r] = dv[db][r] = 0.f;

  if (n_iter > 0) {
    fetch(0);
    stash(0);
  }
  __syncthreads();

  for (int it = 0; it < n_iter; ++it) {
    const int buf = it & 1;
    if (it + 1 < n_iter) fetch(it + 1);
    const int r0 = (rt0 + it % n_rt) * BQ;
    if (p.q_start + r0 + BQ - 1 >= n0) {  // some row of the tile sees some cache row of this wavefront
      lds_char* qt = smem + buf * kStageBytes;
      lds_char* dot = qt + kTileBytes;
      SECO_LDS float* lse_s = reinterpret_cast<SECO_LDS float*>(qt + 2 * kTileBytes);
      SECO_LDS float* delta_s = lse_s + BQ;
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
#pragma unroll
      for (int t = 0; t < 8; ++t) s = mfma(lds_row8(qt, l32, 2 * t + g), kf[t], s);
#pragma unroll
      for (int t = 0; t < 8; ++t) dp = mfma(lds_row8(dot, l32, 2 * t + g), vf[t], dp);
      const bool diag = n0 + 31 > p.q_start + r0;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int qr = 8 * (r >> 2) + 4 * g + (r & 3);
        float pr = fast_exp2(__builtin_fmaf(s[r], c, -lse_s[qr]));
        if (diag && col > p.q_start + r0 + qr) pr = 0.f;
        s[r] = pr;
        dp[r] = pr * (dp[r] - delta_s[qr]);
      }
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 pa = pack8(s, t), dsa = pack8(dp, t);
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          dv[db] = mfma(pa, lds_tr8(dot, 16 * t, db, lane), dv[db]);
          dk[db] = mfma(dsa, lds_tr8(qt, 16 * t, db, lane), dk[db]);
        }
      }
    }
    if (it + 1 < n_iter) stash(buf ^ 1);
    __syncthreads();
  }

  // exclusive read-modify-write of this workgroup's gK/gV rows
  float* gk = p.gk + b * p.gs[0] + kvh * p.gs[1];
  float* gv = p.gv + b * p.gs[0] + kvh * p.gs[1];
  const float wk = weight * p.scale;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int kvrow = n0 + 8 * (r >> 2) + 4 * g + (r & 3);
    if (kvrow < c_end) {
      float* gkr = gk + (int64_t)kvrow * p.gs[2] + l32;
      float* gvr = gv + (int64_t)kvrow * p.gs[2] + l32;
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        gkr[32 * db] += wk * dk[db][r];
        gvr[32 * db] += weight * dv[db][r];
      }
    }
  }
}

}  // namespace

int launch_dkdv_bf16(const AttnParams& p, const SegTable& seg, hipStream_t s) {
  const int tiles = seg.tile_begin[seg.n];
  if (tiles == 0) return SECO_OK;
  const int total = tiles * p.Hkv * p.B;
  {
    ProfScope prof(kKernelDkdv, s);
    hipLaunchKernelGGL(dkdv_bf16_kernel, dim3(xcd_grid(total)), dim3(256), 0, s, p, seg, total);
  }
  return launch_status();
}

}  // namespace seco
