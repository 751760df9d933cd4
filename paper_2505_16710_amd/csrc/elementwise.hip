// Bandwidth-bound helpers: KV-gradient buffer zero / axpy (the gradient relay of the
// paper's appendix listing, "grad + base * scaler") and the softmax-gradient row term
// delta = rowsum(dO * O); and the merge steps of the split forward / dQ kernels (short chunks).
#include "seco_internal.h"

namespace seco {
namespace {

// Rows [r0, r1) of a [B, H, N, D] fp32 buffer, one float4 per thread-iteration.
// Work item index -> (b, h, row, d4); consecutive threads touch consecutive 16-byte words of a row.
// blockIdx.y selects the tensor (gK or gV): both are handled by one launch.
template <bool kAxpy>
__global__ __launch_bounds__(256) void kvgrad_kernel(float* __restrict__ dst_a, float* __restrict__ dst_b,
                                                     const float* __restrict__ src_a, const float* __restrict__ src_b,
                                                     float scale, int H, int d4, int64_t gs0, int64_t gs1, int64_t gs2,
                                                     int64_t r0, int64_t nrows, int64_t total) {
  float* __restrict__ dst = blockIdx.y ? dst_b : dst_a;
  const float* __restrict__ src = blockIdx.y ? src_b : src_a;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t dd = i % d4;
    int64_t t = i / d4;
    const int64_t row = t % nrows;
    t /= nrows;
    const int64_t h = t % H, b = t / H;
    const int64_t off = b * gs0 + h * gs1 + (r0 + row) * gs2 + dd * 4;
    float4* d = reinterpret_cast<float4*>(dst + off);
    if (kAxpy) {
      const float4 x = *reinterpret_cast<const float4*>(src + off);
      float4 y = *d;
      y.x += scale * x.x;
      y.y += scale * x.y;
      y.z += scale * x.z;
      y.w += scale * x.w;
      *d = y;
    } else {
      *d = make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
}

__device__ inline float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// One wavefront per row; 16-byte loads; fp32 accumulation; cross-lane tree reduction.
template <bool kBf16>
__global__ __launch_bounds__(256) void delta_kernel(AttnParams p) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t nrows = (int64_t)p.B * p.Hq * p.C;
  if (row >= nrows) return;
  const int r = row % p.C;
  const int h = (row / p.C) % p.Hq;
  const int b = row / ((int64_t)p.C * p.Hq);
  const int64_t off = b * p.os[0] + h * p.os[1] + (int64_t)r * p.os[2];
  float acc = 0.f;
  if (kBf16) {
    const uint4* o = reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(p.o) + off);
    const uint4* g = reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(p.d_o) + off);
    for (int i = lane; i < p.D / 8; i += 64) {
      const uint4 a = o[i], c = g[i];
      acc += bf16_lo(a.x) * bf16_lo(c.x) + bf16_hi(a.x) * bf16_hi(c.x);
      acc += bf16_lo(a.y) * bf16_lo(c.y) + bf16_hi(a.y) * bf16_hi(c.y);
      acc += bf16_lo(a.z) * bf16_lo(c.z) + bf16_hi(a.z) * bf16_hi(c.z);
      acc += bf16_lo(a.w) * bf16_lo(c.w) + bf16_hi(a.w) * bf16_hi(c.w);
    }
  } else {
    const float4* o = reinterpret_cast<const float4*>(static_cast<const float*>(p.o) + off);
    const float4* g = reinterpret_cast<const float4*>(static_cast<const float*>(p.d_o) + off);
    for (int i = lane; i < p.D / 4; i += 64) {
      const float4 a = o[i], c = g[i];
      acc += a.x * c.x + a.y * c.y + a.z * c.z + a.w * c.w;
    }
  }
#pragma unroll
  for (int s = 32; s > 0; s >>= 1) acc += __shfl_xor(acc, s);
  if (lane == 0) p.delta[row] = acc;
}

// Merge of the split forward: the 32 threads of a row (thread = 4 consecutive head_dim elements) combine the
// n_splits (<= 64) partial rows in split order,
//   M = max m_s,  L = sum l_s 2^(m_s - M),  O = sum o_s 2^(m_s - M) / L,  LSE = (M + log2 L) ln 2.
// Lane i of the row's group loads (m, l) of splits i and i + 32 once; max, sum and the per-split weights then
// travel by cross-lane shuffles.  A partial with m_s = -inf is empty (nothing was written for its O): weight 0,
// its O is not read.
__global__ __launch_bounds__(256) void fwd_merge_kernel(AttnParams p) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t R = (int64_t)p.B * p.Hq * p.C;
  const int64_t rowid = min(i >> 5, R - 1);      // surplus threads of the last block repeat the last row, no store
  const bool live = (i >> 5) < R;
  const int l32 = (int)(i & 31);
  float m0 = -INFINITY, m1 = -INFINITY, s0 = 0.f, s1 = 0.f;
  if (l32 < p.n_splits) {
    m0 = p.part_ml[2 * (l32 * R + rowid)];
    s0 = p.part_ml[2 * (l32 * R + rowid) + 1];
  }
  if (l32 + 32 < p.n_splits) {
    m1 = p.part_ml[2 * ((l32 + 32) * R + rowid)];
    s1 = p.part_ml[2 * ((l32 + 32) * R + rowid) + 1];
  }
  float M = fmaxf(m0, m1);
#pragma unroll
  for (int sh = 16; sh > 0; sh >>= 1) M = fmaxf(M, __shfl_xor(M, sh, 32));
  const float w0 = m0 == -INFINITY ? 0.f : exp2f(m0 - M);
  const float w1 = m1 == -INFINITY ? 0.f : exp2f(m1 - M);
  float L = w0 * s0 + w1 * s1;
#pragma unroll
  for (int sh = 16; sh > 0; sh >>= 1) L += __shfl_xor(L, sh, 32);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int sp = 0; sp < p.n_splits; ++sp) {
    const float w = __shfl(sp < 32 ? w0 : w1, sp & 31, 32);
    if (w == 0.f) continue;
    const float4 x = *reinterpret_cast<const float4*>(p.part + (sp * R + rowid) * 128 + 4 * l32);
    acc.x += w * x.x;
    acc.y += w * x.y;
    acc.z += w * x.z;
    acc.w += w * x.w;
  }
  if (!live) return;
  const float inv = 1.f / L;
  const int row = (int)(rowid % p.C);
  const int h = (int)((rowid / p.C) % p.Hq);
  const int b = (int)(rowid / ((int64_t)p.C * p.Hq));
  typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
  const bf16x4 v = {(__bf16)(acc.x * inv), (__bf16)(acc.y * inv), (__bf16)(acc.z * inv), (__bf16)(acc.w * inv)};
  *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(p.o_out) + b * p.os[0] + h * p.os[1] + (int64_t)row * p.os[2] + 4 * l32) = v;
  if (l32 == 0) p.lse[rowid] = (M + log2f(L)) * 0.6931471805599453f;
}

// Merge of the split dQ: dQ = scale * (sum of the partials in split order), rounded to bf16.
__global__ __launch_bounds__(256) void dq_merge_kernel(AttnParams p) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t R = (int64_t)p.B * p.Hq * p.C;
  const int64_t rowid = i >> 5;
  if (rowid >= R) return;
  const int d4 = (int)(i & 31);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int sp = 0; sp < p.n_splits; ++sp) {
    const float4 x = *reinterpret_cast<const float4*>(p.part + (sp * R + rowid) * 128 + 4 * d4);
    acc.x += x.x;
    acc.y += x.y;
    acc.z += x.z;
    acc.w += x.w;
  }
  const int row = (int)(rowid % p.C);
  const int h = (int)((rowid / p.C) % p.Hq);
  const int b = (int)(rowid / ((int64_t)p.C * p.Hq));
  typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
  const bf16x4 v = {(__bf16)(acc.x * p.scale), (__bf16)(acc.y * p.scale), (__bf16)(acc.z * p.scale), (__bf16)(acc.w * p.scale)};
  *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(p.d_q) + b * p.qs[0] + h * p.qs[1] + (int64_t)row * p.qs[2] + 4 * d4) = v;
}

// Row-range copy into the cache: work item = 16 bytes; consecutive threads walk along a row.
__global__ __launch_bounds__(256) void rows_copy_kernel(uint4* __restrict__ dst_a, uint4* __restrict__ dst_b,
                                                        const uint4* __restrict__ src_a, const uint4* __restrict__ src_b,
                                                        int H, int C, int v16, int64_t ds0, int64_t ds1, int64_t ds2,
                                                        int64_t ss0, int64_t ss1, int64_t ss2, int64_t r0, int64_t total) {
  // strides arrive in units of 16 bytes; blockIdx.y selects the tensor (keys or values)
  uint4* __restrict__ dst = blockIdx.y ? dst_b : dst_a;
  const uint4* __restrict__ src = blockIdx.y ? src_b : src_a;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t dd = i % v16;
    int64_t t = i / v16;
    const int64_t row = t % C;
    t /= C;
    const int64_t h = t % H, b = t / H;
    dst[b * ds0 + h * ds1 + (r0 + row) * ds2 + dd] = src[b * ss0 + h * ss1 + row * ss2 + dd];
  }
}

// Read-out of KV-gradient rows: work item = 8 consecutive floats of a row (32 bytes in, 16 or 32 bytes out).
template <bool kBf16>
__global__ __launch_bounds__(256) void readout_kernel(void* __restrict__ out_a, void* __restrict__ out_b,
                                                      const float* __restrict__ g_a, const float* __restrict__ g_b,
                                                      float scaler, int H, int C, int d8, int64_t os0, int64_t os1,
                                                      int64_t os2, int64_t gs0, int64_t gs1, int64_t gs2, int64_t r0,
                                                      int64_t total) {
  void* __restrict__ out = blockIdx.y ? out_b : out_a;
  const float* __restrict__ g = blockIdx.y ? g_b : g_a;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t dd = i % d8;
    int64_t t = i / d8;
    const int64_t row = t % C;
    t /= C;
    const int64_t h = t % H, b = t / H;
    const float4* src = reinterpret_cast<const float4*>(g + b * gs0 + h * gs1 + (r0 + row) * gs2 + dd * 8);
    float4 a = src[0], c = src[1];
    a.x *= scaler; a.y *= scaler; a.z *= scaler; a.w *= scaler;
    c.x *= scaler; c.y *= scaler; c.z *= scaler; c.w *= scaler;
    const int64_t off = b * os0 + h * os1 + row * os2 + dd * 8;
    if (kBf16) {
      typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
      const bf16x8 v = {(__bf16)a.x, (__bf16)a.y, (__bf16)a.z, (__bf16)a.w, (__bf16)c.x, (__bf16)c.y, (__bf16)c.z, (__bf16)c.w};
      *reinterpret_cast<bf16x8*>(static_cast<__bf16*>(out) + off) = v;
    } else {
      float4* d = reinterpret_cast<float4*>(static_cast<float*>(out) + off);
      d[0] = a;
      d[1] = c;
    }
  }
}

int grid_for(int64_t total) {
  const int64_t blocks = (total + 255) / 256;
  return (int)(blocks < 65536 ? blocks : 65536);  // grid-stride loop covers the rest
}

}  // namespace

// The launchers take a pair of tensors (gK and gV, keys and values); a NULL member is skipped.
int launch_kvgrad_zero(float* ga, float* gb, int B, int H, int D, const int64_t gs[3], int64_t r0, int64_t r1,
                       hipStream_t s) {
  const int64_t total = (int64_t)B * H * (r1 - r0) * (D / 4);
  if (!ga) { ga = gb; gb = nullptr; }
  if (total == 0 || !ga) return SECO_OK;
  {
    ProfScope prof(kKernelKvgrad, s);
    hipLaunchKernelGGL(kvgrad_kernel<false>, dim3(grid_for(total), gb ? 2 : 1), dim3(256), 0, s, ga, gb, nullptr, nullptr,
                       0.f, H, D / 4, gs[0], gs[1], gs[2], r0, r1 - r0, total);
  }
  return launch_status();
}

int launch_kvgrad_axpy(float* da, float* db, const float* sa, const float* sb, float scale, int B, int H, int D,
                       const int64_t gs[3], int64_t r0, int64_t r1, hipStream_t s) {
  const int64_t total = (int64_t)B * H * (r1 - r0) * (D / 4);
  if (!da) { da = db; sa = sb; db = nullptr; sb = nullptr; }
  if (total == 0 || !da) return SECO_OK;
  {
    ProfScope prof(kKernelKvgrad, s);
    hipLaunchKernelGGL(kvgrad_kernel<true>, dim3(grid_for(total), db ? 2 : 1), dim3(256), 0, s, da, db, sa, sb, scale, H,
                       D / 4, gs[0], gs[1], gs[2], r0, r1 - r0, total);
  }
  return launch_status();
}

int launch_rows_copy(void* da, void* db, const void* sa, const void* sb, int eb, int B, int H, int C, int D,
                     const int64_t dst_s[3], const int64_t src_s[3], int64_t r0, hipStream_t s) {
  const int per16 = 16 / eb;                  // elements per 16-byte word; strides and D are multiples of it
  const int v16 = D / per16;
  const int64_t total = (int64_t)B * H * C * v16;
  if (!da) { da = db; sa = sb; db = nullptr; sb = nullptr; }
  if (total == 0 || !da) return SECO_OK;
  {
    ProfScope prof(kKernelKvgrad, s);
    hipLaunchKernelGGL(rows_copy_kernel, dim3(grid_for(total), db ? 2 : 1), dim3(256), 0, s, static_cast<uint4*>(da),
                       static_cast<uint4*>(db), static_cast<const uint4*>(sa), static_cast<const uint4*>(sb), H, C, v16,
                       dst_s[0] / per16, dst_s[1] / per16, dst_s[2] / per16, src_s[0] / per16, src_s[1] / per16,
                       src_s[2] / per16, r0, total);
  }
  return launch_status();
}

int launch_readout(void* oa, void* ob, const float* ga, const float* gb, float scaler, bool bf16, int B, int H, int C,
                   int D, const int64_t out_s[3], const int64_t gs[3], int64_t r0, hipStream_t s) {
  const int64_t total = (int64_t)B * H * C * (D / 8);
  if (!oa) { oa = ob; ga = gb; ob = nullptr; gb = nullptr; }
  if (total == 0 || !oa) return SECO_OK;
  {
    ProfScope prof(kKernelKvgrad, s);
    const dim3 grid(grid_for(total), ob ? 2 : 1);
    if (bf16)
      hipLaunchKernelGGL(readout_kernel<true>, grid, dim3(256), 0, s, oa, ob, ga, gb, scaler, H, C, D / 8, out_s[0],
                         out_s[1], out_s[2], gs[0], gs[1], gs[2], r0, total);
    else
      hipLaunchKernelGGL(readout_kernel<false>, grid, dim3(256), 0, s, oa, ob, ga, gb, scaler, H, C, D / 8, out_s[0],
                         out_s[1], out_s[2], gs[0], gs[1], gs[2], r0, total);
  }
  return launch_status();
}

// Rotary position embedding of rows: out[b, h, r, :] = R(sign * theta(pos0 + r)) (scale * in[b, h, r, :]), pairs
// (i, i + D/2), theta_i = pos * base^(-2 i / D).  Work item = 4 consecutive i of one row (both halves); angles and
// sines in fp64, one rounding of the result.  In / out element types are template parameters so that the same
// kernel serves the cache append (storage type -> storage type, rows at r0 of the destination), the gradient
// read-out (fp32 -> storage type, rows at r0 of the source) and the plain rotation.  A second tensor pair with the
// same strides (the values of an append, the value gradient of a read-out) rides along as blockIdx.y == 1: the same
// rows, scaled and converted but not rotated, so that keys and values take one pass and one launch.
template <typename TIn, typename TOut>
__global__ __launch_bounds__(256) void rope_rows_kernel(TOut* out, const TIn* in, TOut* plain_out, const TIn* plain_in,
                                                        int H, int C,   // (out may be in)
                                                        int D, int64_t os0, int64_t os1, int64_t os2, int64_t is0,
                                                        int64_t is1, int64_t is2, int64_t out_r0, int64_t in_r0,
                                                        int64_t pos0, double log2_base, float sign, float scale,
                                                        int plain_from, int64_t total) {
  const int q4 = D / 8;                                   // groups of 4 pairs per row
  const bool plain = (int)blockIdx.y >= plain_from;       // plain_from: 1 with a rotated pair present, else 0
  if (plain) {
    out = plain_out;
    in = plain_in;
  }
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int grp = (int)(i % q4);
    int64_t t = i / q4;
    const int64_t row = t % C;
    t /= C;
    const int64_t h = t % H, b = t / H;
    const TIn* src = in + b * is0 + h * is1 + (in_r0 + row) * is2 + grp * 4;
    TOut* dst = out + b * os0 + h * os1 + (out_r0 + row) * os2 + grp * 4;
    float lo[4], hi[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      lo[j] = (float)src[j] * scale;
      hi[j] = (float)src[D / 2 + j] * scale;
    }
    if (plain) {                                          // (uniform over the workgroup)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        dst[j] = (TOut)lo[j];
        dst[D / 2 + j] = (TOut)hi[j];
      }
      continue;
    }
    const double pos = (double)(pos0 + row);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const double theta = pos * exp2(-2.0 * (double)(grp * 4 + j) / (double)D * log2_base);
      double sn, cs;
      sincos(theta, &sn, &cs);
      sn *= (double)sign;
      const double a = (double)lo[j], c = (double)hi[j];
      dst[j] = (TOut)(float)(a * cs - c * sn);
      dst[D / 2 + j] = (TOut)(float)(c * cs + a * sn);
    }
  }
}

int launch_rope_rows(void* out, const void* in, void* plain_out, const void* plain_in, int in_kind, int out_kind, int B,
                     int H, int C, int D, const int64_t out_s[3], const int64_t in_s[3], int64_t out_r0, int64_t in_r0,
                     int64_t pos0, float base, bool inverse, float scale, hipStream_t s) {
  const int64_t total = (int64_t)B * H * C * (D / 8);
  if (total == 0 || (!out && !plain_out)) return SECO_OK;
  const double l2b = log2((double)base);
  const float sign = inverse ? -1.f : 1.f;
  {
    ProfScope prof(kKernelKvgrad, s);
    // grid.y: one slice of workgroups per tensor pair present (the rotated pair first)
    const int plain_from = out ? 1 : 0;
    const dim3 grid(grid_for(total), (out ? 1u : 0u) + (plain_out ? 1u : 0u));
#define SECO_ROPE_LAUNCH(TI, TO)                                                                                       \
  hipLaunchKernelGGL((rope_rows_kernel<TI, TO>), grid, dim3(256), 0, s, static_cast<TO*>(out),                         \
                     static_cast<const TI*>(in), static_cast<TO*>(plain_out), static_cast<const TI*>(plain_in), H, C,   \
                     D, out_s[0], out_s[1], out_s[2], in_s[0], in_s[1], in_s[2], out_r0, in_r0, pos0, l2b, sign,        \
                     scale, plain_from, total)
    if (in_kind == SECO_BF16 && out_kind == SECO_BF16) SECO_ROPE_LAUNCH(__bf16, __bf16);
    else if (in_kind == SECO_F32 && out_kind == SECO_BF16) SECO_ROPE_LAUNCH(float, __bf16);
    else SECO_ROPE_LAUNCH(float, float);
#undef SECO_ROPE_LAUNCH
  }
  return launch_status();
}

int launch_fwd_merge(const AttnParams& p, hipStream_t s) {
  const int64_t threads = (int64_t)p.B * p.Hq * p.C * 32;
  {
    ProfScope prof(kKernelMerge, s);
    hipLaunchKernelGGL(fwd_merge_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, p);
  }
  return launch_status();
}

int launch_dq_merge(const AttnParams& p, hipStream_t s) {
  const int64_t threads = (int64_t)p.B * p.Hq * p.C * 32;
  {
    ProfScope prof(kKernelMerge, s);
    hipLaunchKernelGGL(dq_merge_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, p);
  }
  return launch_status();
}

int launch_delta(const AttnParams& p, int dtype, hipStream_t s) {
  const int64_t nrows = (int64_t)p.B * p.Hq * p.C;
  const unsigned blocks = (unsigned)((nrows + 3) / 4);
  if (dtype == SECO_BF16)
    {
    ProfScope prof(kKernelDelta, s);
    hipLaunchKernelGGL(delta_kernel<true>, dim3(blocks), dim3(256), 0, s, p);
  }
  else
    {
    ProfScope prof(kKernelDelta, s);
    hipLaunchKernelGGL(delta_kernel<false>, dim3(blocks), dim3(256), 0, s, p);
  }
  return launch_status();
}

}  // namespace seco
