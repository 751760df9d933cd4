// Forward of one chunk, bf16 matrix cores (Eq. 1 at the attention layer):
// O = softmax(s Q K^T) V over cache rows [0, q_start + C) with the causal rule
// col <= q_start + row, plus the per-row log-sum-exp.
//
// Decomposition.  A workgroup owns 128 query rows of one head; a wavefront owns 32 of them and
// keeps Q^T fragments, the running max / sum and the O^T accumulator (128 x 32, fp32) in
// registers.  K and V tiles stream through swizzled LDS tiles shared by the workgroup, copied
// global -> LDS directly ahead of their use.  Two shapes of workgroup:
//   4 wavefronts (fwd4_bf16.hip): tiles of 64 cache rows, 80 KiB of LDS -> two workgroups per CU; used when a
//       call has at least two row tiles per CU, and by the split path of short chunks;
//   8 wavefronts (this file): tiles of 128 cache rows in two buffers of a K and a V tile; wavefront (rb, kh)
//       handles row block rb and the kh-th 64-row half of every tile, and the two partial (max, sum, O) of a
//       row block are merged through LDS at the end.  One such workgroup fills a CU with two wavefronts per
//       SIMD, which is what calls with few row tiles need (a 1024-row chunk of a 32-head layer has only 256
//       row tiles for 256 CUs).
//
// The score tile is computed transposed, S^T = K Q^T, so that a lane owns one query row
// (C layout: lane = column): row max / row sum are in-lane reductions plus one exchange with
// lane^32, the rescale of O^T is a per-lane scalar, and P^T feeds the second product
// O^T += V^T P^T straight from registers.  V^T comes from the row-major V tile through the
// LDS transpose read.
#include "mfma_tiles.h"
#include "seco_internal.h"

namespace seco {
namespace {

constexpr int BM = 128;  // query rows per workgroup
constexpr int BNW = 64;  // cache rows per wavefront and tile
constexpr float kBig = 1099511627776.f;   // 2^40: a tile's exponentials may sum to this before the reference moves

// 8-wavefront shape (see the head of the file)
__global__ __launch_bounds__(512, 2) void fwd8_bf16_kernel(AttnParams p, int n_mtiles, int total_items) {
  constexpr int KH = 2;
  constexpr int BN = BNW * KH;                 // cache rows per tile
  constexpr int kTileBytes = BN * kRowBytes;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];   // 4 * kTileBytes: [buf][K|V]
  lds_char* smem = (lds_char*)smem_raw;

  const int item = xcd_item(blockIdx.x, total_items);
  if (item < 0) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int rb = wave & 3, kh = wave >> 2;
  // item -> (batch, kv head, row tile (heavy first), head within the group)
  const int hg = item % p.G;
  int rest = item / p.G;
  const int mt = n_mtiles - 1 - rest % n_mtiles;
  rest /= n_mtiles;
  const int kvh = rest % p.Hkv, b = rest / p.Hkv;
  const int h = kvh * p.G + hg;
  const int m0 = mt * BM + rb * 32;          // first chunk-local row of this wavefront

  const int kv_len = p.q_start + p.C;
  const int row = m0 + l32;                    // this lane's row
  const int qpos = p.q_start + row;            // its global position
  const __bf16* qptr = static_cast<const __bf16*>(p.q) + b * p.qs[0] + h * p.qs[1] + (int64_t)min(row, p.C - 1) * p.qs[2];
  bf16x8 qf[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) qf[t] = *reinterpret_cast<const bf16x8*>(qptr + 16 * t + 8 * g);

  const __bf16* kbase = static_cast<const __bf16*>(p.k) + b * p.kvs[0] + kvh * p.kvs[1];
  const __bf16* vbase = static_cast<const __bf16*>(p.v) + b * p.kvs[0] + kvh * p.kvs[1];

  const int wg_kv_end = p.q_start + min((mt + 1) * BM, p.C);   // columns any row of the workgroup sees
  const int n_tiles = (wg_kv_end + BN - 1) / BN;
  const int wave_kv_end = m0 < p.C ? p.q_start + min(m0 + 32, p.C) : 0;  // columns this wavefront sees
  const int n_begin = 0, n_end = n_tiles;      // tiles of this workgroup

  // asynchronous global -> LDS copy of one K and one V tile: each wavefront copies 4 groups of 4 rows of each.
  // The per-lane byte offsets inside a tile never change; a tile that lies entirely inside the cache is copied
  // from a scalar base address with no vector arithmetic, the last (ragged) one with clamped per-lane addresses.
  uint32_t lane_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) lane_off[i] = dma_lane_offset(4 * (wave + 4 * KH * i), p.kvs[2] * 2, lane);
  const uint32_t lds_wave = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem + wave * 4 * kRowBytes);
  auto copy_tile = [&](int n, int buf) {
    if ((n + 1) * BN <= kv_len) {
      const __bf16* kt_src = kbase + (int64_t)n * BN * p.kvs[2];
      const __bf16* vt_src = vbase + (int64_t)n * BN * p.kvs[2];
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
        const int64_t off = (int64_t)min(n * BN + r + (lane >> 4), kv_len - 1) * p.kvs[2];
        dma4rows(kt, r, kbase + off, lane);
        dma4rows(vt, r, vbase + off, lane);
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

  copy_tile(n_begin, 0);
#pragma unroll
  for (int t = 0; t < 8; ++t) settle(qf[t]);
  dma_wait_all();
  __syncthreads();

  for (int n = n_begin; n < n_end; ++n) {
    const int buf = (n - n_begin) & 1;
    if (n + 1 < n_end) copy_tile(n + 1, buf ^ 1);
    const int col0 = n * BN + kh * BNW;        // first cache row of this wavefront's part of the tile
    if (col0 < wave_kv_end) {
      lds_char* kt = smem + buf * 2 * kTileBytes + kh * BNW * kRowBytes;
      lds_char* vt = kt + kTileBytes;
      f32x16 s[2];
#pragma unroll
      for (int kvb = 0; kvb < 2; ++kvb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[kvb][r] = 0.f;
#pragma unroll
        for (int t = 0; t < 8; ++t) s[kvb] = mfma(lds_row8(kt, kvb * 32 + l32, 2 * t + g), qf[t], s[kvb]);
      }
      if (col0 + BNW - 1 > p.q_start + m0) {  // reaches past this wavefront's first row: causal mask
#pragma unroll
        for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int kv = col0 + kvb * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
            if (kv > qpos) s[kvb][r] = -INFINITY;
          }
      }
      // Reference value of the row's exponentials.  A max subtraction only guards against overflow, so the
      // reference m_run is kept as it is as long as the exponentials stay representable: the (costly) row maximum
      // is computed only on a row's first visible tile and when the tile's sum of exponentials exceeds kBig = 2^40,
      // which for a whole kernel is a handful of times.  Exponentials may thus reach 2^40; bf16 and fp32 have
      // the exponent range for that, and O and the sum are rescaled together when the reference moves.
      auto tile_max = [&]() {
        float mx = s[0][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[0][r]);
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[1][r]);
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
      float sum = 0.f;
      f32x16 e[2];
#pragma unroll
      for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          e[kvb][r] = fast_exp2(__builtin_fmaf(s[kvb][r], c, -m_use));
          sum += e[kvb][r];
        }
      if (__builtin_amdgcn_ballot_w64(!(sum <= kBig)) != 0) {           // reference too low for this tile (rare)
        const float m_blk = tile_max();
        if (m_blk > m_run) move_reference(m_blk);
        m_use = m_run == -INFINITY ? 0.f : m_run;
        sum = 0.f;
#pragma unroll
        for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            e[kvb][r] = fast_exp2(__builtin_fmaf(s[kvb][r], c, -m_use));
            sum += e[kvb][r];
          }
      }
#pragma unroll
      for (int kvb = 0; kvb < 2; ++kvb) s[kvb] = e[kvb];
      l_run += sum;
#pragma unroll
      for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const bf16x8 pb = pack8(s[kvb], t);
#pragma unroll
          for (int db = 0; db < 4; ++db) o[db] = mfma(lds_tr8(vt, kvb * 32 + 16 * t, db, lane), pb, o[db]);
        }
    }
    dma_wait_all();
    __syncthreads();
  }

  float l_tot = l_run + __shfl_xor(l_run, 32);
  {
    // merge the two column halves of each row block: kh = 1 publishes (m, l, O), kh = 0 combines
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    lds_char* slot = smem + rb * (17 * 1024);            // 16 KiB of O + 512 B of (m, l) per row block
    if (kh == 1) {
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          f32x4 v = {o[db][4 * r4], o[db][4 * r4 + 1], o[db][4 * r4 + 2], o[db][4 * r4 + 3]};
          *reinterpret_cast<SECO_LDS f32x4*>(slot + ((db * 4 + r4) * 64 + lane) * 16) = v;
        }
      *reinterpret_cast<SECO_LDS float*>(slot + 16384 + lane * 4) = m_run;
      *reinterpret_cast<SECO_LDS float*>(slot + 16384 + 256 + lane * 4) = l_tot;
    }
    __syncthreads();
    if (kh == 1) return;
    const float m1 = *reinterpret_cast<SECO_LDS float*>(slot + 16384 + lane * 4);
    const float l1 = *reinterpret_cast<SECO_LDS float*>(slot + 16384 + 256 + lane * 4);
    const float m = fmaxf(m_run, m1);               // finite: half 0 always sees column 0
    const float a0 = fast_exp2(m_run - m), a1 = fast_exp2(m1 - m);
    l_tot = l_tot * a0 + l1 * a1;
    m_run = m;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const f32x4 v = *reinterpret_cast<SECO_LDS f32x4*>(slot + ((db * 4 + r4) * 64 + lane) * 16);
#pragma unroll
        for (int i = 0; i < 4; ++i) o[db][4 * r4 + i] = o[db][4 * r4 + i] * a0 + v[i] * a1;
      }
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

int launch_fwd8(const AttnParams& p, int n_mtiles, int total, hipStream_t s) {
  constexpr int smem = 4 * BNW * 2 * kRowBytes;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(fwd8_bf16_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          smem) != hipSuccess)
    return SECO_ERR_LAUNCH;
  {
    ProfScope prof(kKernelFwd, s);
    hipLaunchKernelGGL(fwd8_bf16_kernel, dim3(xcd_grid(total)), dim3(512), smem, s, p, n_mtiles, total);
  }
  return launch_status();
}

}  // namespace

int launch_fwd_bf16(const AttnParams& p, hipStream_t s) {
  if (p.n_splits > 1) {
    const SplitPlan plan = split_plan(p.B, p.Hkv, p.G, p.C);
    int rc = launch_fwd4_bf16(p, true, plan.n_mtiles, plan.items * p.n_splits, s);
    return rc ? rc : launch_fwd_merge(p, s);
  }
  const int n_mtiles = (p.C + BM - 1) / BM;
  const int total = p.B * p.Hq * n_mtiles;
  // fewer row tiles than two per CU: use the 8-wavefront shape so that every SIMD still has two wavefronts
  return total < 2 * device_cus() ? launch_fwd8(p, n_mtiles, total, s) : launch_fwd4_bf16(p, false, n_mtiles, total, s);
}

}  // namespace seco
