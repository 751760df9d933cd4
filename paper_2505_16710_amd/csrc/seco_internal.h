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
  float* delta;      // [B, Hq, C] contiguous (workspace), backward only
  float* gk;
  float* gv;
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

// fp32 reference-grade kernels (any head_dim that is a multiple of 4, up to 256)
int launch_fwd_f32(const AttnParams& p, hipStream_t s);
int launch_dq_f32(const AttnParams& p, hipStream_t s);
int launch_dkdv_f32(const AttnParams& p, const SegTable& seg, hipStream_t s);
constexpr int kColTileF32 = 4;     // columns per workgroup in launch_dkdv_f32

// bf16 matrix-core kernels (head_dim 128)
int launch_fwd_bf16(const AttnParams& p, hipStream_t s);
int launch_dq_bf16(const AttnParams& p, hipStream_t s);
int launch_dkdv_bf16(const AttnParams& p, const SegTable& seg, hipStream_t s);
#ifndef SECO_DKDV_COLS
#define SECO_DKDV_COLS 128
#endif
constexpr int kColTileBf16 = SECO_DKDV_COLS;  // columns per workgroup in launch_dkdv_bf16

// delta[r] = sum_d dO[r,d] * O[r,d]
int launch_delta(const AttnParams& p, int dtype, hipStream_t s);

int launch_kvgrad_zero(float* g, int B, int H, int D, const int64_t gs[3], int64_t r0, int64_t r1, hipStream_t s);
int launch_kvgrad_axpy(float* dst, const float* src, float scale, int B, int H, int D, const int64_t gs[3],
                       int64_t r0, int64_t r1, hipStream_t s);

// Optional per-kernel timing (seco_profile_enable): a scope brackets one launch with HIP events
// on the launch stream.  Disabled by default; then a scope costs one branch.
enum KernelKind { kKernelFwd = 0, kKernelDelta, kKernelDq, kKernelDkdv, kKernelKvgrad, kKernelKinds };
struct ProfScope {
  ProfScope(KernelKind kind, hipStream_t s);
  ~ProfScope();
  hipStream_t stream;
  int slot;
};

inline int launch_status() { return hipGetLastError() == hipSuccess ? SECO_OK : SECO_ERR_LAUNCH; }

}  // namespace seco
