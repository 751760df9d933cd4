// dK/dV of one chunk, bf16 matrix cores, accumulated into the persistent fp32 KV-gradient
// buffers (Alg. 1 second loop; Alg. 2 with per-chunk weights):
//   gV[c] += w * sum_{heads of the group} P^T dO      gK[c] += w * s * sum_{heads} dS^T Q
//
// Column-parallel: one workgroup is the only writer of 128 cache rows of one (batch, KV head),
// so the read-modify-write of gK/gV needs no atomics and the result is deterministic.
//
// The workgroup has 8 wavefronts: 4 column blocks of 32 cache rows x 2 roles.
//   role A ("probabilities"): keeps K^T fragments and the dV accumulator; computes
//          S = Q K^T, P = exp(S - LSE) (causal mask applied), hands P (bf16) to its partner
//          through LDS and accumulates dV += P^T dO;
//   role B ("score gradient"): keeps V^T fragments and the dK accumulator; computes
//          dP = dO V^T, dS = P * (dP - delta) and accumulates dK += dS^T Q.
// Each of the four products is computed exactly once, and a wavefront holds one 32x128 fp32
// accumulator plus one operand fragment set instead of two of each, which is what lets two
// wavefronts share a SIMD.  Role A runs one row tile ahead of role B, so the P hand-over
// costs no extra barrier: one barrier per 32-row tile.
//
// Q, dO, LSE and delta of 32 query rows stream through a three-deep ring of swizzled LDS
// stages (A reads Q of tile i+1 while B reads Q and dO of tile i and tile i+2 is landing).
// S and dP are computed in the "row = query" orientation, so P and dS sit in the C layout
// with lane = cache row and feed the second products as A operands straight from registers;
// dO and Q for those products come through the LDS transpose read.
//
// Column tiles are enumerated from a by-value segment table (runs of cache rows that share
// one non-zero weight); SpaCO's unselected chunks simply have no tiles.
#include "mfma_tiles.h"
#include "seco_internal.h"

namespace seco {
namespace {

constexpr int BQ = 32;                                     // query rows per stage
constexpr int kTileBytes = BQ * kRowBytes;                 // 8 KiB
constexpr int kStageBytes = 2 * kTileBytes + 2 * BQ * 4;   // Q, dO, lse, delta
constexpr int kStages = 3;
constexpr int kPBytes = 2048;                              // one 32x32 bf16 P tile
constexpr int kSmemBytes = kStages * kStageBytes + 2 * 4 * kPBytes;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(512, 1) void dkdv_bf16_kernel(AttnParams p, SegTable seg, int total_items) {
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];   // kSmemBytes, above the 64 KiB static limit
  lds_char* smem = (lds_char*)smem_raw;
  lds_char* pbuf = smem + kStages * kStageBytes;

  const int item = xcd_item(blockIdx.x, total_items);
  if (item < 0) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int role = wave >> 2, cb = wave & 3;
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
  const int n0 = c0 + cb * 32;     // first cache row of this wavefront
  const int col = n0 + l32;        // this lane's cache row in the score tile
  // role A holds K^T fragments, role B holds V^T fragments
  const __bf16* fptr = static_cast<const __bf16*>(role == 0 ? p.k : p.v) + b * p.kvs[0] + kvh * p.kvs[1] +
                       (int64_t)min(col, kv_len - 1) * p.kvs[2];
  bf16x8 frag[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) frag[t] = *reinterpret_cast<const bf16x8*>(fptr + 16 * t + 8 * g);

  // query-row tiles that see at least one cache row of this workgroup
  const int rt0 = max(0, c0 - p.q_start) / BQ;
  const int n_rt = (p.C + BQ - 1) / BQ - rt0;
  const int n_iter = n_rt * p.G;
  const float c = p.scale * kLog2e;
  auto row0_of = [&](int it) { return (rt0 + it % n_rt) * BQ; };
  // does any row of tile `it` see any cache row of this wavefront?
  auto live = [&](int it) { return p.q_start + row0_of(it) + BQ - 1 >= n0; };

  // staging: one 16-byte chunk of Q and one of dO per thread, LSE / delta by the first wavefront
  bf16x8 qreg, doreg;
  float stat = 0.f;
  auto fetch = [&](int it) {
    const int h = kvh * p.G + it / n_rt;
    const int r0 = row0_of(it);
    const int r = min(r0 + (tid >> 4), p.C - 1), ch = tid & 15;
    qreg = *reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(p.q) + b * p.qs[0] + h * p.qs[1] +
                                            (int64_t)r * p.qs[2] + ch * 8);
    doreg = *reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(p.d_o) + b * p.os[0] + h * p.os[1] +
                                             (int64_t)r * p.os[2] + ch * 8);
    if (tid < 64) {
      const int rr = r0 + (tid & 31);
      const int64_t idx = ((int64_t)b * p.Hq + h) * p.C + min(rr, p.C - 1);
      // rows past the chunk get LSE = +inf so that their probabilities vanish
      if (tid < 32) stat = rr < p.C ? p.lse[idx] * kLog2e : INFINITY;
      else stat = p.delta[idx];
    }
  };
  auto stash = [&](int it) {
    lds_char* qt = smem + (it % kStages) * kStageBytes;
    lds_store16(qt, tid >> 4, tid & 15, qreg);
    lds_store16(qt + kTileBytes, tid >> 4, tid & 15, doreg);
    if (tid < 64) *reinterpret_cast<SECO_LDS float*>(qt + 2 * kTileBytes + tid * 4) = stat;
  };

  f32x16 acc[4];   // role A: dV, role B: dK  (32 cache rows x 128)
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;
  bf16x8 p_cur[2] = {}, p_next[2] = {};   // role A: P of the tile being accumulated / of the next tile

  // role A: S = Q K^T for tile `it`, P = exp2(S*c - LSE) with the causal mask, as two operand halves;
  // the same values go to the partner through pbuf
  auto scores = [&](int it, bf16x8 (&out)[2]) {
    lds_char* qt = smem + (it % kStages) * kStageBytes;
    SECO_LDS float* lse_s = reinterpret_cast<SECO_LDS float*>(qt + 2 * kTileBytes);
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) s = mfma(lds_row8(qt, l32, 2 * t + g), frag[t], s);
    const int r0 = row0_of(it);
    const bool diag = n0 + 31 > p.q_start + r0;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int qr = 8 * (r >> 2) + 4 * g + (r & 3);
      float pr = fast_exp2(__builtin_fmaf(s[r], c, -lse_s[qr]));
      if (diag && col > p.q_start + r0 + qr) pr = 0.f;
      s[r] = pr;
    }
    out[0] = pack8(s, 0);
    out[1] = pack8(s, 1);
    lds_char* pb = pbuf + ((it & 1) * 4 + cb) * kPBytes;
    *reinterpret_cast<SECO_LDS bf16x8*>(pb + lane * 16) = out[0];
    *reinterpret_cast<SECO_LDS bf16x8*>(pb + 1024 + lane * 16) = out[1];
  };

  const int n_pro = min(n_iter, 2);
  for (int it = 0; it < n_pro; ++it) {
    fetch(it);
    stash(it);
  }
  __syncthreads();
  if (role == 0 && live(0)) scores(0, p_cur);
  __syncthreads();

  for (int it = 0; it < n_iter; ++it) {
    if (it + 2 < n_iter) fetch(it + 2);
    lds_char* qt = smem + (it % kStages) * kStageBytes;
    lds_char* dot = qt + kTileBytes;
    if (role == 0) {
      if (it + 1 < n_iter && live(it + 1)) scores(it + 1, p_next);
      if (live(it)) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int db = 0; db < 4; ++db) acc[db] = mfma(p_cur[t], lds_tr8(dot, 16 * t, db, lane), acc[db]);
      }
      p_cur[0] = p_next[0];
      p_cur[1] = p_next[1];
    } else if (live(it)) {
      SECO_LDS float* delta_s = reinterpret_cast<SECO_LDS float*>(qt + 2 * kTileBytes) + BQ;
      f32x16 dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) dp[r] = 0.f;
#pragma unroll
      for (int t = 0; t < 8; ++t) dp = mfma(lds_row8(dot, l32, 2 * t + g), frag[t], dp);
      lds_char* pb = pbuf + ((it & 1) * 4 + cb) * kPBytes;
      const bf16x8 ph[2] = {*reinterpret_cast<SECO_LDS bf16x8*>(pb + lane * 16),
                            *reinterpret_cast<SECO_LDS bf16x8*>(pb + 1024 + lane * 16)};
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int qr = 8 * (r >> 2) + 4 * g + (r & 3);
        dp[r] = (float)ph[r >> 3][r & 7] * (dp[r] - delta_s[qr]);
      }
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 dsa = pack8(dp, t);
#pragma unroll
        for (int db = 0; db < 4; ++db) acc[db] = mfma(dsa, lds_tr8(qt, 16 * t, db, lane), acc[db]);
      }
    }
    if (it + 2 < n_iter) stash(it + 2);
    __syncthreads();
  }

  // exclusive read-modify-write of this workgroup's gK/gV rows: role A adds dV, role B adds s * dK
  float* gbase = (role == 0 ? p.gv : p.gk) + b * p.gs[0] + kvh * p.gs[1];
  const float wf = role == 0 ? weight : weight * p.scale;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int kvrow = n0 + 8 * (r >> 2) + 4 * g + (r & 3);
    if (kvrow < c_end) {
      float* gr = gbase + (int64_t)kvrow * p.gs[2] + l32;
#pragma unroll
      for (int db = 0; db < 4; ++db) gr[32 * db] += wf * acc[db][r];
    }
  }
}

}  // namespace

int launch_dkdv_bf16(const AttnParams& p, const SegTable& seg, hipStream_t s) {
  const int tiles = seg.tile_begin[seg.n];
  if (tiles == 0) return SECO_OK;
  const int total = tiles * p.Hkv * p.B;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(dkdv_bf16_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          kSmemBytes) != hipSuccess)
    return SECO_ERR_LAUNCH;
  {
    ProfScope prof(kKernelDkdv, s);
    hipLaunchKernelGGL(dkdv_bf16_kernel, dim3(xcd_grid(total)), dim3(512), kSmemBytes, s, p, seg, total);
  }
  return launch_status();
}

}  // namespace seco
