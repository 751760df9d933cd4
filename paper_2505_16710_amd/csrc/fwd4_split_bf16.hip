// The 4-wavefront forward kernel, split instantiation (short chunks: packed heads, cache range divided among
// workgroups, partial results to the workspace).
#include "fwd4_kernel.h"

namespace seco {

int launch_fwd4_split_bf16(const AttnParams& p, int n_mtiles, int total, hipStream_t s) {
  return launch_fwd4<true>(p, n_mtiles, total, s);
}

}  // namespace seco
