// The 4-wavefront forward kernel, plain instantiation (calls with at least two row tiles per CU).
#include "fwd4_kernel.h"

namespace seco {

int launch_fwd4_bf16(const AttnParams& p, bool split, int n_mtiles, int total, hipStream_t s) {
  return split ? launch_fwd4_split_bf16(p, n_mtiles, total, s) : launch_fwd4<false>(p, n_mtiles, total, s);
}

}  // namespace seco
