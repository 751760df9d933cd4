// Forward of one chunk, bf16 matrix cores, 4-wavefront workgroups (Eq. 1 at the attention layer): the shape used
// when a call has at least two row tiles per CU, and by the split path of short chunks.  Decomposition and
// register layout are those of the 8-wavefront kernel in fwd_bf16.hip (a workgroup owns 128 query rows of one
// head, a wavefront 32 of them; S^T = K Q^T so that a lane owns a query row; O^T += V^T P^T from registers);
// the tile pipeline differs: K tiles stream through a ring of three LDS slots and V tiles through a ring of two,
// and S of tile n+1 is computed while the exponentials of tile n are taken (the two instruction streams are
// written interleaved), so that the matrix pipe runs while the vector ALU works: 5 % faster than computing a
// tile's S, softmax and PV one after the other.  (In the 8-wavefront shape the same interleaving was slower.)
//
// Short chunks (SPLIT = true).  With chunks of 32 .. 512 rows (the sizes of the paper's chunk-size study,
// Sec. 6.3) a call has far fewer row tiles than the GPU has CUs and every tile would stream the whole cache
// alone.  The split variant therefore (a) packs the rows of the G query heads that share a KV head into one row
// space of G * roundup(C, 32) rows, so that a workgroup's K/V tiles serve several heads, and (b) divides the
// visible cache rows of a row tile among n_splits workgroups; each writes its un-normalised partial O with its
// reference maximum and sum (fp32) to the workspace, and fwd_merge_kernel combines the partials in split order.
//
// (A header: the two instantiations are compiled in translation units of their own, fwd4_bf16.hip and
// fwd4_split_bf16.hip.  Compiled in one unit with the 8-wavefront kernel, that kernel's instruction schedule comes
// out 5 % slower; and the compiler option that makes the plain instantiation 2 % faster makes the split one spill.)
#pragma once
#include "mfma_tiles.h"
#include "seco_internal.h"

namespace seco {
namespace {

constexpr int BM = 128;  // query rows per workgroup
constexpr int BNW = 64;  // cache rows per wavefront and tile
constexpr float kBig = 1099511627776.f;   // 2^40: a tile's exponentials may sum to this before the reference moves

template <bool SPLIT>
__global__ __launch_bounds__(256, 2) void fwd4_bf16_kernel(AttnParams p, int n_mtiles, int total_items) {
  constexpr int KH = 1;
  constexpr int BN = BNW * KH;                 // cache rows per tile
  constexpr int kTileBytes = BN * kRowBytes;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];   // 5 * kTileBytes: K ring (3 tiles), V ring (2 tiles)
  lds_char* smem = (lds_char*)smem_raw;

  const int item = xcd_item(blockIdx.x, total_items);
  if (item < 0) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int rb = wave, kh = 0;
  int b, kvh, h, mt, m0, sp = 0;              // m0: first chunk-local row of this wavefront
  if constexpr (SPLIT) {
    // item -> (batch, kv head, row tile of the packed row space, split)
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
    // item -> (batch, kv head, row tile (heavy first), head within the group)
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
  const int row = m0 + l32;                    // this lane's row
  const int qpos = p.q_start + row;            // its global position
  const __bf16* qptr = static_cast<const __bf16*>(p.q) + b * p.qs[0] + h * p.qs[1] + (int64_t)min(row, p.C - 1) * p.qs[2];
  bf16x8 qf[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) qf[t] = *reinterpret_cast<const bf16x8*>(qptr + 16 * t + 8 * g);

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
  const int n_tiles = (wg_kv_end + BN - 1) / BN;
  const int wave_kv_end = m0 < p.C ? p.q_start + min(m0 + 32, p.C) : 0;  // columns this wavefront sees
  int n_begin = 0, n_end = n_tiles;            // tiles of this workgroup
  // row of the partial-result arrays (computed where it is used: it would otherwise occupy registers across the loop)
  auto part_row_of = [&]() { return (int64_t)sp * p.B * p.Hq * p.C + ((int64_t)b * p.Hq + h) * p.C + row; };
  if constexpr (SPLIT) {
    const int per = (n_tiles + p.n_splits - 1) / p.n_splits;
    n_begin = sp * per;
    n_end = min(n_tiles, n_begin + per);
    if (n_begin >= n_end) {                    // nothing to do for this split: an empty partial (max = -inf)
      if (row < p.C && g == 0) {
        const int64_t part_row = part_row_of();
        p.part_ml[2 * part_row] = -INFINITY;
        p.part_ml[2 * part_row + 1] = 0.f;
      }
      return;
    }
  }

  // K tiles stream through a ring of three LDS slots, V tiles through a ring of two: while the matrix pipe works on
  // S of tile n+1 (from K slot n+1) the vector ALU turns S of tile n into probabilities, and the product with V
  // of tile n follows; K of tile n+2 and V of tile n+1 are landing meanwhile.
  // Asynchronous global -> LDS copy of one tile: each wavefront copies 4 groups of 4 rows.  The per-lane byte
  // offsets inside a tile never change; a tile that lies entirely inside the cache is copied from a scalar base
  // address with no vector arithmetic, the last (ragged) one with clamped per-lane addresses.
  // (the four copies of a wavefront are 16 * KH rows apart: the swizzle of a lane's chunk is the same in all four,
  // so one per-lane offset serves them and the row distance goes into the scalar base)
  const uint32_t lane_off = dma_lane_offset(4 * wave, p.kvs[2] * 2, lane);
  const uint32_t lds_wave = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem + wave * 4 * kRowBytes);
  constexpr int kKSlots = 3;
  lds_char* vring = smem + kKSlots * kTileBytes;
  auto copy_ring = [&](const __bf16* base, int n, int tile_index) {   // one tile of K (tile_index 0..2) or V (3..4), 4-wavefront shape
    if ((n + 1) * BN <= kv_len) {
      const __bf16* src = base + (int64_t)n * BN * p.kvs[2];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        dma16_sbase(src + (int64_t)i * (16 * KH) * p.kvs[2], lane_off, lds_wave + tile_index * kTileBytes + i * (16 * KH * kRowBytes));
    } else {
      lds_char* t = smem + tile_index * kTileBytes;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int r = 4 * (wave + 4 * KH * i);
        const int64_t off = (int64_t)min(n * BN + r + (lane >> 4), kv_len - 1) * p.kvs[2];
        dma4rows(t, r, base + off, lane);
      }
    }
  };

  f32x16 o[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c = p.scale * kLog2e;

  // S^T of this wavefront's 64 cache rows of the K tile in slot ks, both 32-row blocks
  auto scores = [&](int ks, f32x16 (&sc)[2]) {
    lds_char* kt = smem + ks * kTileBytes + kh * BNW * kRowBytes;
#pragma unroll
    for (int kvb = 0; kvb < 2; ++kvb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sc[kvb][r] = 0.f;
#pragma unroll
      for (int t = 0; t < 8; ++t) sc[kvb] = mfma(lds_row8(kt, kvb * 32 + l32, 2 * t + g), qf[t], sc[kvb]);
    }
  };
  auto causal_mask = [&](int col0, f32x16 (&sc)[2]) {
    if (col0 + BNW - 1 > p.q_start + m0) {  // reaches past this wavefront's first row
#pragma unroll
      for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kv = col0 + kvb * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
          if (kv > qpos) sc[kvb][r] = -INFINITY;
        }
    }
  };

  // One tile.  PIPE: `cur` holds S of tile n (slot ks of the K ring) on entry, `nxt` S of tile n+1 on exit;
  // otherwise S of tile n is computed here first.
  auto tile_body = [&](int n, int ks, int vs, f32x16 (&cur)[2], f32x16 (&nxt)[2]) {
    const int ks1 = ks + 1 == kKSlots ? 0 : ks + 1;
    if (n + 2 < n_end) copy_ring(kbase, n + 2, ks1 + 1 == kKSlots ? 0 : ks1 + 1);
    if (n + 1 < n_end) copy_ring(vbase, n + 1, kKSlots + (vs ^ 1));
    const int col0 = n * BN + kh * BNW;        // first cache row of this wavefront's part of the tile
    if (col0 < wave_kv_end) {
      lds_char* vt = vring + vs * kTileBytes + kh * BNW * kRowBytes;
      causal_mask(col0, cur);
      // Reference value of the row's exponentials.  A max subtraction only guards against overflow, so the
      // reference m_run is kept as it is as long as the exponentials stay representable: the (costly) row maximum
      // is computed only on a row's first visible tile and when the tile's sum of exponentials exceeds kBig = 2^40,
      // which for a whole kernel is a handful of times.  Exponentials may thus reach 2^40; bf16 and fp32 have
      // the exponent range for that, and O and the sum are rescaled together when the reference moves.
      auto tile_max = [&]() {
        float mx = cur[0][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, cur[0][r]);
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, cur[1][r]);
        return fmaxf(mx, __shfl_xor(mx, 32)) * c;
      };
      auto move_reference = [&](float m_new) {          // m_new >= m_run; exp2(-inf - x) = 0 on the first tile
        const float alpha = fast_exp2(m_run - m_new);
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
        m_run = m_new;
      };
      if (__builtin_amdgcn_ballot_w64(m_run == -INFINITY) != 0) {      // some row has seen nothing yet
        const float m_blk = tile_max();
        if (m_run == -INFINITY && m_blk != -INFINITY) m_run = m_blk;    // (o and l_run are still zero)
      }
      // a part of a tile can be fully masked for a row (only when kh > 0 or q_start is unaligned): such a row
      // has seen nothing yet and keeps m_run = -inf; use 0 so that exp2(-inf - (-inf)) never appears
      float m_use = m_run == -INFINITY ? 0.f : m_run;
      // S of the next tile is issued here, in the same straight-line code as the exponentials below, which do not
      // depend on it: the matrix pipe runs while the vector ALU works.  (On the last tile this computes on
      // whatever the slot holds; the result is never used.)
      float sum = 0.f;
      {
        lds_char* kt1 = smem + ks1 * kTileBytes + kh * BNW * kRowBytes;
#pragma unroll
        for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
          for (int r = 0; r < 16; ++r) nxt[kvb][r] = 0.f;
        // written interleaved: the i-th MFMA of the next tile's two chains, then two exponentials of this tile
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int kvb = i & 1, t = i >> 1;
          nxt[kvb] = mfma(lds_row8(kt1, kvb * 32 + l32, 2 * t + g), qf[t], nxt[kvb]);
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            const int e = 2 * i + j;
            cur[e >> 4][e & 15] = fast_exp2(__builtin_fmaf(cur[e >> 4][e & 15], c, -m_use));
            sum += cur[e >> 4][e & 15];
          }
        }
      }
      if (__builtin_amdgcn_ballot_w64(!(sum <= kBig)) != 0) {           // reference too low for this tile (rare)
        scores(ks, cur);                                                // the scores again: K of this tile is still in its slot
        causal_mask(col0, cur);
        const float m_blk = tile_max();
        if (m_blk > m_run) move_reference(m_blk);
        m_use = m_run == -INFINITY ? 0.f : m_run;
        sum = 0.f;
#pragma unroll
        for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            cur[kvb][r] = fast_exp2(__builtin_fmaf(cur[kvb][r], c, -m_use));
            sum += cur[kvb][r];
          }
      }
      l_run += sum;
#pragma unroll
      for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const bf16x8 pb = pack8(cur[kvb], t);
#pragma unroll
          for (int db = 0; db < 4; ++db) o[db] = mfma(lds_tr8(vt, kvb * 32 + 16 * t, db, lane), pb, o[db]);
        }
    }
    dma_wait_all();
    __syncthreads();
  };

  copy_ring(kbase, n_begin, 0);
  copy_ring(vbase, n_begin, kKSlots);
  if (n_begin + 1 < n_end) copy_ring(kbase, n_begin + 1, 1);
#pragma unroll
  for (int t = 0; t < 8; ++t) settle(qf[t]);
  dma_wait_all();
  __syncthreads();

  f32x16 sa[2], sb[2];
  scores(0, sa);
  int ks = 0;
  for (int n = n_begin; n < n_end; n += 2) {   // two tiles per trip: the score registers swap roles
    tile_body(n, ks, 0, sa, sb);
    ks = ks + 1 == kKSlots ? 0 : ks + 1;
    if (n + 1 < n_end) {
      tile_body(n + 1, ks, 1, sb, sa);
      ks = ks + 1 == kKSlots ? 0 : ks + 1;
    }
  }

  float l_tot = l_run + __shfl_xor(l_run, 32);
  if constexpr (SPLIT) {
    // un-normalised partial O (relative to the reference maximum m_run), fp32, plus (m_run, sum)
    if (row < p.C) {
      typedef float f32x4 __attribute__((ext_vector_type(4)));
      const int64_t part_row = part_row_of();
      float* po = p.part + part_row * kHeadDim;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const f32x4 v = {o[db][4 * r4], o[db][4 * r4 + 1], o[db][4 * r4 + 2], o[db][4 * r4 + 3]};
          *reinterpret_cast<f32x4*>(po + 32 * db + 8 * r4 + 4 * g) = v;
        }
      if (g == 0) {
        p.part_ml[2 * part_row] = m_run;
        p.part_ml[2 * part_row + 1] = l_tot;
      }
    }
    return;
  }

  if (row < p.C) {
    const float inv = 1.f / l_tot;
    __bf16* optr = static_cast<__bf16*>(p.o_out) + b * p.os[0] + h * p.os[1] + (int64_t)row * p.os[2];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        bf16x4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = (__bf16)(o[db][4 * r4 + i] * inv);
        *reinterpret_cast<bf16x4*>(optr + 32 * db + 8 * r4 + 4 * g) = v;
      }
    if (g == 0) p.lse[((int64_t)b * p.Hq + h) * p.C + row] = (m_run + __log2f(l_tot)) * kLn2;
  }
}


template <bool SPLIT>
int launch_fwd4(const AttnParams& p, int n_mtiles, int total, hipStream_t s) {
  constexpr int smem = 5 * BNW * kRowBytes;
  auto kern = fwd4_bf16_kernel<SPLIT>;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem) !=
      hipSuccess)
    return SECO_ERR_LAUNCH;
  {
    ProfScope prof(kKernelFwd, s);
    hipLaunchKernelGGL(kern, dim3(xcd_grid(total)), dim3(256), smem, s, p, n_mtiles, total);
  }
  return launch_status();
}

}  // namespace
}  // namespace seco
