// fp32 kernels for chunked causal attention: forward, dQ and dK/dV.
//
// These serve the fp32 configuration (small shapes, parity at 1e-4) and any
// head_dim that is a multiple of 4 up to 256.  One 64-lane wavefront owns one
// query row (forward, dQ) or one cache column (dK/dV); scores are computed one
// per lane, reduced with cross-lane shuffles, and the D-wide accumulations keep
// lane = head_dim index so that V/K/Q/dO rows are read coalesced.  No matrix
// cores: the bf16 kernels are the performance path.
#include "seco_internal.h"

namespace seco {
namespace {

constexpr int kWaves = 4;
constexpr int kMaxD = 256;
constexpr int kRegs = kMaxD / 64;

__device__ inline float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ inline float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}
// dot product of a global row (16-byte aligned, D % 4 == 0) with a vector held in LDS
__device__ inline float dot_row(const float* __restrict__ row, const float* sh, int D) {
  float acc = 0.f;
  for (int d = 0; d < D; d += 4) {
    float4 x = *reinterpret_cast<const float4*>(row + d);
    acc += x.x * sh[d] + x.y * sh[d + 1] + x.z * sh[d + 2] + x.w * sh[d + 3];
  }
  return acc;
}

// O = softmax(s Q K^T) V and LSE for one chunk; wave per query row, online softmax over 64-column blocks.
__global__ __launch_bounds__(kWaves * 64) void fwd_f32_kernel(AttnParams p) {
  __shared__ float qsh[kWaves][kMaxD];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int r = blockIdx.x * kWaves + w, h = blockIdx.y, b = blockIdx.z;
  const bool active = r < p.C;
  const int D = p.D;
  if (active) {
    const float* q = static_cast<const float*>(p.q) + b * p.qs[0] + h * p.qs[1] + (int64_t)r * p.qs[2];
    for (int d = lane; d < D; d += 64) qsh[w][d] = q[d];
  }
  __syncthreads();
  if (!active) return;
  const int g = h / p.G;
  const float* K = static_cast<const float*>(p.k) + b * p.kvs[0] + g * p.kvs[1];
  const float* V = static_cast<const float*>(p.v) + b * p.kvs[0] + g * p.kvs[1];
  const int last = p.q_start + r;  // last visible column
  float m = -INFINITY, l = 0.f, acc[kRegs] = {0.f, 0.f, 0.f, 0.f};
  for (int c0 = 0; c0 <= last; c0 += 64) {
    const int c = c0 + lane;
    const bool vis = c <= last;
    float s = -INFINITY;
    if (vis) s = p.scale * dot_row(K + (int64_t)c * p.kvs[2], qsh[w], D);
    const float m_new = fmaxf(m, wave_max(s));
    const float pe = vis ? __expf(s - m_new) : 0.f;
    const float alpha = __expf(m - m_new);  // exp(-inf) = 0 on the first block
    l = l * alpha + wave_sum(pe);
#pragma unroll
    for (int i = 0; i < kRegs; ++i) acc[i] *= alpha;
    const int nc = min(64, last - c0 + 1);
    for (int cc = 0; cc < nc; ++cc) {
      const float pc = __shfl(pe, cc);
      const float* vrow = V + (int64_t)(c0 + cc) * p.kvs[2];
#pragma unroll
      for (int i = 0; i < kRegs; ++i) {
        const int d = lane + 64 * i;
        if (d < D) acc[i] += pc * vrow[d];
      }
    }
    m = m_new;
  }
  float* o = static_cast<float*>(p.o_out) + b * p.os[0] + h * p.os[1] + (int64_t)r * p.os[2];
  const float inv = 1.f / l;
#pragma unroll
  for (int i = 0; i < kRegs; ++i) {
    const int d = lane + 64 * i;
    if (d < D) o[d] = acc[i] * inv;
  }
  if (lane == 0) p.lse[((int64_t)b * p.Hq + h) * p.C + r] = m + __logf(l);
}

// dQ = s * sum over the runs of cache rows in `seg` of w * dS K (one run with weight 1 over all visible rows: the
// exact dQ); wave per query row.
__global__ __launch_bounds__(kWaves * 64) void dq_f32_kernel(AttnParams p, SegTable seg) {
  __shared__ float qsh[kWaves][kMaxD];
  __shared__ float dosh[kWaves][kMaxD];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int r = blockIdx.x * kWaves + w, h = blockIdx.y, b = blockIdx.z;
  const bool active = r < p.C;
  const int D = p.D;
  if (active) {
    const float* q = static_cast<const float*>(p.q) + b * p.qs[0] + h * p.qs[1] + (int64_t)r * p.qs[2];
    const float* d_o = static_cast<const float*>(p.d_o) + b * p.os[0] + h * p.os[1] + (int64_t)r * p.os[2];
    for (int d = lane; d < D; d += 64) {
      qsh[w][d] = q[d];
      dosh[w][d] = d_o[d];
    }
  }
  __syncthreads();
  if (!active) return;
  const int g = h / p.G;
  const float* K = static_cast<const float*>(p.k) + b * p.kvs[0] + g * p.kvs[1];
  const float* V = static_cast<const float*>(p.v) + b * p.kvs[0] + g * p.kvs[1];
  const int64_t row = ((int64_t)b * p.Hq + h) * p.C + r;
  const float lse = p.lse[row], delta = p.delta[row];
  const int last = p.q_start + r;
  float acc[kRegs] = {0.f, 0.f, 0.f, 0.f};
  for (int si = 0; si < seg.n; ++si) {
    const int run_last = min(last, seg.col_end[si] - 1);   // last column of the run this row sees
    const float wt = seg.weight[si];
    for (int c0 = seg.col_begin[si]; c0 <= run_last; c0 += 64) {
      const int c = c0 + lane;
      float ds = 0.f;
      if (c <= run_last) {
        const float s = p.scale * dot_row(K + (int64_t)c * p.kvs[2], qsh[w], D);
        const float dp = dot_row(V + (int64_t)c * p.kvs[2], dosh[w], D);
        ds = wt * (__expf(s - lse) * (dp - delta));
      }
      const int nc = min(64, run_last - c0 + 1);
      for (int cc = 0; cc < nc; ++cc) {
        const float dsc = __shfl(ds, cc);
        const float* krow = K + (int64_t)(c0 + cc) * p.kvs[2];
#pragma unroll
        for (int i = 0; i < kRegs; ++i) {
          const int d = lane + 64 * i;
          if (d < D) acc[i] += dsc * krow[d];
        }
      }
    }
  }
  float* dq = static_cast<float*>(p.d_q) + b * p.qs[0] + h * p.qs[1] + (int64_t)r * p.qs[2];
#pragma unroll
  for (int i = 0; i < kRegs; ++i) {
    const int d = lane + 64 * i;
    if (d < D) dq[d] = p.scale * acc[i];
  }
}

// gK[c] += w * s * sum_h dS^T Q, gV[c] += w * sum_h P^T dO; wave per cache column, exclusive owner.
__global__ __launch_bounds__(kWaves * 64) void dkdv_f32_kernel(AttnParams p, SegTable seg) {
  __shared__ float ksh[kWaves][kMaxD];
  __shared__ float vsh[kWaves][kMaxD];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int tile = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  int si = 0;
  while (si + 1 < seg.n && tile >= seg.tile_begin[si + 1]) ++si;
  const int c = seg.col_begin[si] + (tile - seg.tile_begin[si]) * kColTileF32 + w;
  const bool active = c < seg.col_end[si];
  const float weight = seg.weight[si];
  const int D = p.D;
  if (active) {
    const float* krow = static_cast<const float*>(p.k) + b * p.kvs[0] + g * p.kvs[1] + (int64_t)c * p.kvs[2];
    const float* vrow = static_cast<const float*>(p.v) + b * p.kvs[0] + g * p.kvs[1] + (int64_t)c * p.kvs[2];
    for (int d = lane; d < D; d += 64) {
      ksh[w][d] = krow[d];
      vsh[w][d] = vrow[d];
    }
  }
  __syncthreads();
  if (!active) return;
  float dk[kRegs] = {0.f, 0.f, 0.f, 0.f}, dv[kRegs] = {0.f, 0.f, 0.f, 0.f};
  const int r_first = max(0, c - p.q_start);  // rows that see column c
  for (int hh = 0; hh < p.G; ++hh) {
    const int h = g * p.G + hh;
    const float* Q = static_cast<const float*>(p.q) + b * p.qs[0] + h * p.qs[1];
    const float* dO = static_cast<const float*>(p.d_o) + b * p.os[0] + h * p.os[1];
    const int64_t row0 = ((int64_t)b * p.Hq + h) * p.C;
    for (int r0 = r_first; r0 < p.C; r0 += 64) {
      const int r = r0 + lane;
      float pr = 0.f, ds = 0.f;
      if (r < p.C) {
        const float s = p.scale * dot_row(Q + (int64_t)r * p.qs[2], ksh[w], D);
        const float dp = dot_row(dO + (int64_t)r * p.os[2], vsh[w], D);
        pr = __expf(s - p.lse[row0 + r]);
        ds = pr * (dp - p.delta[row0 + r]);
      }
      const int nr = min(64, p.C - r0);
      for (int rr = 0; rr < nr; ++rr) {
        const float pb = __shfl(pr, rr), dsb = __shfl(ds, rr);
        const float* qrow = Q + (int64_t)(r0 + rr) * p.qs[2];
        const float* dorow = dO + (int64_t)(r0 + rr) * p.os[2];
#pragma unroll
        for (int i = 0; i < kRegs; ++i) {
          const int d = lane + 64 * i;
          if (d < D) {
            dv[i] += pb * dorow[d];
            dk[i] += dsb * qrow[d];
          }
        }
      }
    }
  }
  float* gk = p.gk + b * p.gs[0] + g * p.gs[1] + (int64_t)c * p.gs[2];
  float* gv = p.gv + b * p.gs[0] + g * p.gs[1] + (int64_t)c * p.gs[2];
#pragma unroll
  for (int i = 0; i < kRegs; ++i) {
    const int d = lane + 64 * i;
    if (d < D) {
      gk[d] += weight * (p.scale * dk[i]);
      gv[d] += weight * dv[i];
    }
  }
}

}  // namespace

int launch_fwd_f32(const AttnParams& p, hipStream_t s) {
  dim3 grid((p.C + kWaves - 1) / kWaves, p.Hq, p.B);
  {
    ProfScope prof(kKernelFwd, s);
    hipLaunchKernelGGL(fwd_f32_kernel, grid, dim3(kWaves * 64), 0, s, p);
  }
  return launch_status();
}

int launch_dq_f32(const AttnParams& p, const SegTable* dq_runs, hipStream_t s) {
  SegTable all = {};
  all.n = 1;
  all.col_end[0] = p.q_start + p.C;
  all.weight[0] = 1.f;
  dim3 grid((p.C + kWaves - 1) / kWaves, p.Hq, p.B);
  {
    ProfScope prof(kKernelDq, s);
    hipLaunchKernelGGL(dq_f32_kernel, grid, dim3(kWaves * 64), 0, s, p, dq_runs ? *dq_runs : all);
  }
  return launch_status();
}

int launch_dkdv_f32(const AttnParams& p, const SegTable& seg, hipStream_t s) {
  const int tiles = seg.tile_begin[seg.n];
  if (tiles == 0) return SECO_OK;
  dim3 grid(tiles, p.Hkv, p.B);
  {
    ProfScope prof(kKernelDkdv, s);
    hipLaunchKernelGGL(dkdv_f32_kernel, grid, dim3(kWaves * 64), 0, s, p, seg);
  }
  return launch_status();
}

}  // namespace seco
