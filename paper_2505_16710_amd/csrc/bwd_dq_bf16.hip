// dQ of one chunk, bf16 matrix cores: dQ = s * dS K over ALL visible cache rows, with
// P = exp(S - LSE), dS = P * (dO V^T - delta), delta = rowsum(dO * O) (computed in this kernel's prologue).  (SpaCO keeps dQ exact: a selected chunk's
// graph is rebuilt against every earlier cache, Alg. 2.)
//
// Same row-parallel decomposition as the forward, in the same two workgroup shapes: a workgroup
// owns 128 query rows of one head, a wavefront 32 of them; K and V tiles stream through
// swizzled, double-buffered LDS, copied global -> LDS directly one tile ahead; with KH = 2 (8 wavefronts, 128-row tiles) the two wavefronts
// of a row block take one 64-row half of every tile each and their partial dQ are added
// through LDS at the end.  Scores are again computed transposed (S^T = K Q^T, dP^T = V dO^T)
// so that LSE and delta are per-lane scalars and dS^T feeds dQ^T += K^T dS^T from registers;
// K^T comes from the same K tile through the LDS transpose read.
//
// Column-weighted dQ (SPARSE = true): the tiles are taken from a by-value table of runs of cache rows, each with
// one positive weight w, instead of from all visible rows: dQ = s * sum over the runs of w * dS K.  A tile starts
// where its run starts (not on a multiple of the tile height), rows past the run's end are masked like rows above
// the diagonal, and the weight costs nothing per element: P * w = exp2(S - (LSE - log2 w)), one logarithm per
// tile.  With every chunk sampled with probability pi and weighted 1 / pi this is an unbiased estimate of dQ
// whose cost does not grow with the number of unvisited rows.
//
// Short chunks (SPLIT = true): as in the forward, the rows of the G heads of a KV head are packed into one row
// space and the visible cache rows of a row tile are divided among n_splits workgroups; each writes its partial
// dQ (fp32, unscaled) to the workspace and dq_merge_kernel adds the partials in split order.
#include "mfma_tiles.h"
#include "seco_internal.h"

namespace seco {
namespace {

constexpr int BM = 128;
constexpr int BNW = 64;   // cache rows per wavefront and tile

// seg (SPARSE only): runs of cache rows in ascending order, each with a positive weight
template <int KH, bool SPLIT, bool SPARSE>
__global__ __launch_bounds__(256 * KH, 2) void dq_bf16_kernel(AttnParams p, SegTable seg, int n_mtiles,
                                                              int total_items) {
  static_assert(!SPLIT || KH == 1, "the split variant uses the 4-wavefront shape");
  constexpr int BN = BNW * KH;
  constexpr int kTileBytes = BN * kRowBytes;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];   // 4 * kTileBytes: [buf][K|V]
  lds_char* smem = (lds_char*)smem_raw;

  const int item = xcd_item(blockIdx.x, total_items);
  if (item < 0) return;
  // (the wavefront index through readfirstlane: the compiler then knows that it, and every tile coordinate and branch
  // condition derived from it, is uniform over the wavefront and keeps them in scalar registers)
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, g = lane >> 5;
  const int rb = wave & 3, kh = (KH == 1 && !SPARSE) ? 0 : wave >> 2;
  int b, kvh, h, mt, m0, sp = 0;              // m0: first chunk-local row of this wavefront
  if constexpr (SPLIT) {
    sp = item % p.n_splits;
    int rest = item / p.n_splits;
    mt = n_mtiles - 1 - rest % n_mtiles;
    rest /= n_mtiles;
    kvh = rest % p.Hkv;
    b = rest / p.Hkv;
    const int v0 = mt * BM + rb * 32;          // packed row: head v0 / Cpad of the group, row v0 % Cpad
    int hg = v0 / p.Cpad;
    m0 = v0 - hg * p.Cpad;
    if (hg >= p.G) {                           // past the last head of the group: idle wavefront (m0 >= C)
      hg = p.G - 1;
      m0 = p.Cpad;
    }
    h = kvh * p.G + hg;
  } else {
    const int hg = item % p.G;
    int rest = item / p.G;
    mt = n_mtiles - 1 - rest % n_mtiles;
    rest /= n_mtiles;
    kvh = rest % p.Hkv;
    b = rest / p.Hkv;
    h = kvh * p.G + hg;
    m0 = mt * BM + rb * 32;
  }

  const int kv_len = p.q_start + p.C;
  const int row = m0 + l32;
  const int crow = min(row, p.C - 1);
  const int qpos = p.q_start + row;
  const __bf16* qptr = static_cast<const __bf16*>(p.q) + b * p.qs[0] + h * p.qs[1] + (int64_t)crow * p.qs[2];
  const __bf16* doptr = static_cast<const __bf16*>(p.d_o) + b * p.os[0] + h * p.os[1] + (int64_t)crow * p.os[2];
  bf16x8 qf[8], dof[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    qf[t] = *reinterpret_cast<const bf16x8*>(qptr + 16 * t + 8 * g);
    dof[t] = *reinterpret_cast<const bf16x8*>(doptr + 16 * t + 8 * g);
  }
  const int64_t stat = ((int64_t)b * p.Hq + h) * p.C + crow;
  const float lse_c = p.lse[stat] * kLog2e;
  // delta = rowsum(dO * O) is computed here, from the dO fragments already in registers and the matching O
  // fragments: a lane holds half of its row's head_dim (the other half is in lane ^ 32).  It is also written to
  // the workspace for the dK/dV kernel that follows on the same stream, negated, together with -LSE / s (the
  // log-sum-exp in units of the unscaled dot product): the two values that kernel starts its MFMA chains from.
  float delta = 0.f;
  {
    const __bf16* optr = static_cast<const __bf16*>(p.o) + b * p.os[0] + h * p.os[1] + (int64_t)crow * p.os[2];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const bf16x8 of = *reinterpret_cast<const bf16x8*>(optr + 16 * t + 8 * g);
#pragma unroll
      for (int i = 0; i < 8; ++i) delta = __builtin_fmaf((float)of[i], (float)dof[t][i], delta);
    }
    delta += __shfl_xor(delta, 32);
    if (kh == 0 && sp == 0 && g == 0 && row < p.C) {
      const int64_t kept = ((int64_t)b * p.Hq + h) * p.stat_stride + p.stat_off + crow;
      p.delta[kept] = -delta;
      p.nlse2[kept] = -p.lse[stat] / p.scale;
    }
  }
  const float c = p.scale * kLog2e;

  const __bf16* kbase = static_cast<const __bf16*>(p.k) + b * p.kvs[0] + kvh * p.kvs[1];
  const __bf16* vbase = static_cast<const __bf16*>(p.v) + b * p.kvs[0] + kvh * p.kvs[1];
  int wg_kv_end;                               // columns any row of the workgroup sees
  if constexpr (SPLIT) {
    int rows_end = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int v = mt * BM + r * 32, hh = v / p.Cpad, mm = v - hh * p.Cpad;
      if (hh < p.G && mm < p.C) rows_end = max(rows_end, min(mm + 32, p.C));
    }
    wg_kv_end = rows_end ? p.q_start + rows_end : 0;
  } else {
    wg_kv_end = p.q_start + min((mt + 1) * BM, p.C);
  }
  // SPARSE: position in the run table = (run, first cache row of the tile, end of the run clipped to the rows
  // this workgroup sees); runs that start at or past that limit have no tiles
  struct Cur { int si, col, end; };
  auto run_at = [&](int si) { return Cur{si, seg.col_begin[si], min(seg.col_end[si], wg_kv_end)}; };
  auto advance = [&](Cur x) {
    x.col += BN;
    if (x.col >= x.end && x.si + 1 < seg.n) x = run_at(x.si + 1);
    return x;
  };
  int n_tiles = (wg_kv_end + BN - 1) / BN;
  if constexpr (SPARSE) {
    n_tiles = 0;
    for (int si = 0; si < seg.n; ++si) {
      const int len = min(seg.col_end[si], wg_kv_end) - seg.col_begin[si];
      if (len > 0) n_tiles += (len + BN - 1) / BN;
    }
  }
  const int wave_kv_end = m0 < p.C ? p.q_start + min(m0 + 32, p.C) : 0;
  int n_begin = 0, n_end = n_tiles;            // tiles of this workgroup
  if constexpr (SPLIT) {
    const int per = (n_tiles + p.n_splits - 1) / p.n_splits;
    n_begin = sp * per;
    n_end = min(n_tiles, n_begin + per);       // may be empty: the partial written below is then all zero
  }

  // asynchronous global -> LDS copy of one K and one V tile: each wavefront copies 4 groups of 4 rows of each.
  // The per-lane byte offsets inside a tile never change; a tile that lies entirely inside the cache is copied
  // from a scalar base address with no vector arithmetic, the last (ragged) one with clamped per-lane addresses.
  uint32_t lane_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) lane_off[i] = dma_lane_offset(4 * (wave + 4 * KH * i), p.kvs[2] * 2, lane);
  const uint32_t lds_wave = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem + wave * 4 * kRowBytes);
  auto copy_tile = [&](int col, int buf) {      // col: first cache row of the tile
    if (col + BN <= kv_len) {
      const __bf16* kt_src = kbase + (int64_t)col * p.kvs[2];
      const __bf16* vt_src = vbase + (int64_t)col * p.kvs[2];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t dst = lds_wave + buf * 2 * kTileBytes + i * (16 * KH * kRowBytes);
        dma16_sbase(kt_src, lane_off[i], dst);
        dma16_sbase(vt_src, lane_off[i], dst + kTileBytes);
      }
    } else {
      lds_char* kt = smem + buf * 2 * kTileBytes;
      lds_char* vt = kt + kTileBytes;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int r = 4 * (wave + 4 * KH * i);
        const int64_t off = (int64_t)min(col + r + (lane >> 4), kv_len - 1) * p.kvs[2];
        dma4rows(kt, r, kbase + off, lane);
        dma4rows(vt, r, vbase + off, lane);
      }
    }
  };

  // lane-dependent parts of the LDS operand addresses (constant for the whole kernel)
  int r_off[8];
  TrOff t_off[4];
  // (dense variants: the wavefront's half of the tile, for KH = 2, is part of the per-lane offsets, so that a tile's
  // base is a compile-time constant in the unrolled loop below)
  const int half_off = SPARSE ? 0 : kh * BNW * kRowBytes;
#pragma unroll
  for (int t = 0; t < 8; ++t) r_off[t] = row8_lane_off(l32, 2 * t + g) + half_off;
#pragma unroll
  for (int db = 0; db < 4; ++db) {
    t_off[db] = tr8_lane_off(db, lane);
    t_off[db].lo += half_off;
    t_off[db].hi += half_off;
  }

  f32x16 dq[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[db][r] = 0.f;

  Cur cur{0, n_begin * BN, 0};
  if constexpr (SPARSE) {
    cur = run_at(0);
    for (int i = 0; i < n_begin && i < n_tiles; ++i) cur = advance(cur);
  }
  Cur nxt = cur;
  if (n_begin < n_end) copy_tile(cur.col, 0);
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    settle(qf[t]);
    settle(dof[t]);
  }
  dma_wait_all();
  __syncthreads();

  if constexpr (SPARSE) {
    for (int n = n_begin; n < n_end; ++n) {
      const int buf = (n - n_begin) & 1;
#include "bwd_dq_tile_step.inc"
    }
  } else {
    for (int n0 = n_begin; n0 < n_end; n0 += 2) {
      {
        constexpr int buf = 0;
        const int n = n0;
#include "bwd_dq_tile_step.inc"
      }
      if (n0 + 1 >= n_end) break;
      {
        constexpr int buf = 1;
        const int n = n0 + 1;
#include "bwd_dq_tile_step.inc"
      }
    }
  }

  if (KH == 2) {
    // add the partial dQ of the two column halves of each row block through LDS
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    lds_char* slot = smem + rb * (16 * 1024);
    if (kh == 1) {
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          f32x4 v = {dq[db][4 * r4], dq[db][4 * r4 + 1], dq[db][4 * r4 + 2], dq[db][4 * r4 + 3]};
          *reinterpret_cast<SECO_LDS f32x4*>(slot + ((db * 4 + r4) * 64 + lane) * 16) = v;
        }
    }
    __syncthreads();
    if (kh == 1) return;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const f32x4 v = *reinterpret_cast<SECO_LDS f32x4*>(slot + ((db * 4 + r4) * 64 + lane) * 16);
#pragma unroll
        for (int i = 0; i < 4; ++i) dq[db][4 * r4 + i] += v[i];
      }
  }

  if constexpr (SPLIT) {
    if (row < p.C) {
      typedef float f32x4 __attribute__((ext_vector_type(4)));
      float* po = p.part + ((int64_t)sp * p.B * p.Hq * p.C + stat) * kHeadDim;   // row < C: stat is this row's index
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const f32x4 v = {dq[db][4 * r4], dq[db][4 * r4 + 1], dq[db][4 * r4 + 2], dq[db][4 * r4 + 3]};
          *reinterpret_cast<f32x4*>(po + 32 * db + 8 * r4 + 4 * g) = v;
        }
    }
    return;
  }

  if (row < p.C) {
    __bf16* out = static_cast<__bf16*>(p.d_q) + b * p.qs[0] + h * p.qs[1] + (int64_t)row * p.qs[2];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        bf16x4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = (__bf16)(dq[db][4 * r4 + i] * p.scale);
        *reinterpret_cast<bf16x4*>(out + 32 * db + 8 * r4 + 4 * g) = v;
      }
  }
}

template <int KH, bool SPLIT, bool SPARSE>
int launch_kh(const AttnParams& p, const SegTable& seg, int n_mtiles, int total, hipStream_t s) {
  constexpr int smem = 4 * BNW * KH * kRowBytes;
  auto kern = dq_bf16_kernel<KH, SPLIT, SPARSE>;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem) !=
      hipSuccess)
    return SECO_ERR_LAUNCH;
  {
    ProfScope prof(kKernelDq, s);
    hipLaunchKernelGGL(kern, dim3(xcd_grid(total)), dim3(256 * KH), smem, s, p, seg, n_mtiles, total);
  }
  return launch_status();
}

}  // namespace

// runs == nullptr: all visible cache rows, weight 1
int launch_dq_bf16(const AttnParams& p, const SegTable* runs, hipStream_t s) {
  SegTable none = {};
  const SegTable& seg = runs ? *runs : none;
  if (p.n_splits > 1) {
    const SplitPlan plan = split_plan(p.B, p.Hkv, p.G, p.C);
    const int total = plan.items * p.n_splits;
    int rc = runs ? launch_kh<1, true, true>(p, seg, plan.n_mtiles, total, s)
                  : launch_kh<1, true, false>(p, seg, plan.n_mtiles, total, s);
    return rc ? rc : launch_dq_merge(p, s);
  }
  const int n_mtiles = (p.C + BM - 1) / BM;
  const int total = p.B * p.Hq * n_mtiles;
  if (total < 2 * device_cus())
    return runs ? launch_kh<2, false, true>(p, seg, n_mtiles, total, s) : launch_kh<2, false, false>(p, seg, n_mtiles, total, s);
  return runs ? launch_kh<1, false, true>(p, seg, n_mtiles, total, s) : launch_kh<1, false, false>(p, seg, n_mtiles, total, s);
}

}  // namespace seco
