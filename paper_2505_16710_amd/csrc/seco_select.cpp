// Host-only parts of the C ABI: SpaCO chunk selection (Alg. 2, selection step: t different
// chunks of k, uniformly), the per-call chunk weight vector (Alg. 2 with the compensation
// factor of Sec. 5), and status strings.
#include <algorithm>
#include <cmath>
#include <functional>
#include <vector>

#include "seco.h"

namespace {

constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;

inline uint64_t finalise(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// SplitMix64 (Steele, Lea, Flood 2014): additive state, multiplicative-xorshift output function.
struct SplitMix64 {
  uint64_t state;
  uint64_t next() {
    state += kGolden;
    return finalise(state);
  }
  // Uniform in [0, m): reject the top (2^64 mod m) values so that every residue is equally likely.
  uint64_t below(uint64_t m) {
    const uint64_t excess = (0 - m) % m;  // 2^64 mod m
    for (;;) {
      const uint64_t u = next();
      if (excess == 0 || u < (uint64_t)(0 - excess)) return u % m;
    }
  }
};

}  // namespace

extern "C" int spaco_select_chunks(uint64_t seed, uint64_t step, int32_t k, int32_t t, int32_t* out_host) {
  if (!out_host) return SECO_ERR_NULL;
  if (k < 1 || t < 1 || t > k) return SECO_ERR_RANGE;
  SplitMix64 rng{finalise(seed ^ finalise(step + kGolden))};
  std::vector<int32_t> perm(k);
  for (int32_t i = 0; i < k; ++i) perm[i] = i;
  for (int32_t i = 0; i < t; ++i) {
    const int32_t r = i + (int32_t)rng.below((uint64_t)(k - i));
    std::swap(perm[i], perm[r]);
  }
  std::sort(perm.begin(), perm.begin() + t, std::greater<int32_t>());
  std::copy(perm.begin(), perm.begin() + t, out_host);
  return SECO_OK;
}

extern "C" int spaco_percall_weights(uint64_t seed, uint64_t step, int32_t j, int32_t t, float* w_host) {
  if (!w_host) return SECO_ERR_NULL;
  if (j < 0 || t < 0) return SECO_ERR_RANGE;
  std::fill(w_host, w_host + j + 1, 0.f);
  w_host[j] = 1.f;
  const int32_t m = std::min(t, j);
  if (m > 0) {
    std::vector<int32_t> sel(m);
    const int rc = spaco_select_chunks(seed, step * (1ull << 20) + (uint64_t)j, j, m, sel.data());
    if (rc) return rc;
    const float w = (float)((double)j / (double)m);
    for (int32_t i : sel) w_host[i] = w;
  }
  return SECO_OK;
}

extern "C" int spaco_select_bernoulli(uint64_t seed, uint64_t step, int32_t k, double q, int32_t* out_host,
                                      int32_t* n_selected_host) {
  if (!out_host || !n_selected_host) return SECO_ERR_NULL;
  if (k < 1 || !(q > 0.0) || !(q <= 1.0)) return SECO_ERR_RANGE;
  SplitMix64 rng{finalise(seed ^ finalise(step + kGolden))};
  // q * 2^64 is exact in double (a power-of-two scaling); below 1 it fits 64 bits and converts by truncation
  const bool all = q >= 1.0;
  const uint64_t threshold = all ? 0 : (uint64_t)std::ldexp(q, 64);
  int32_t n = 0;
  for (int32_t i = 0; i < k; ++i) {
    const uint64_t u = rng.next();
    if (all || u < threshold) out_host[n++] = i;
  }
  std::reverse(out_host, out_host + n);
  *n_selected_host = n;
  return SECO_OK;
}

extern "C" float spaco_compensation_factor(int32_t k, int32_t t, float cap) {
  if (k < 1 || t < 1 || t > k) return -1.f;
  const float lam = (float)((double)k / (double)t);
  return cap > 0.f && cap < lam ? cap : lam;
}

extern "C" int spaco_chunk_weights(const int32_t* selected_host, int32_t n_selected, int32_t j, float factor,
                                   float* w_host) {
  if (!w_host || (n_selected > 0 && !selected_host)) return SECO_ERR_NULL;
  if (j < 0 || n_selected < 0) return SECO_ERR_RANGE;
  for (int32_t i = 0; i < n_selected; ++i)
    if (selected_host[i] < 0) return SECO_ERR_RANGE;
  std::fill(w_host, w_host + j + 1, 0.f);
  for (int32_t i = 0; i < n_selected; ++i)
    if (selected_host[i] < j) w_host[selected_host[i]] = factor;
  w_host[j] = 1.f;
  return SECO_OK;
}

extern "C" int spaco_gather_row_weights(const int32_t* selected_host, int32_t n_selected, int32_t i, int32_t k,
                                        float factor, float* w_host) {
  if (!w_host || (n_selected > 0 && !selected_host)) return SECO_ERR_NULL;
  if (i < 0 || k <= i || n_selected < 0) return SECO_ERR_RANGE;
  for (int32_t n = 0; n < n_selected; ++n)
    if (selected_host[n] < 0) return SECO_ERR_RANGE;
  // the transpose of spaco_chunk_weights: what call m > i deposits on chunk i carries the factor iff m is selected
  std::fill(w_host, w_host + (k - i), 0.f);
  for (int32_t n = 0; n < n_selected; ++n)
    if (selected_host[n] > i && selected_host[n] < k) w_host[selected_host[n] - i] = factor;
  w_host[0] = 1.f;
  return SECO_OK;
}

extern "C" const char* seco_strerror(int status) {
  switch (status) {
    case SECO_OK: return "ok";
    case SECO_ERR_NULL: return "a required pointer is NULL";
    case SECO_ERR_SHAPE: return "invalid shape (sizes must be positive, n_q_heads a multiple of n_kv_heads, q_start >= 0)";
    case SECO_ERR_HEAD_DIM: return "head_dim not supported for this dtype";
    case SECO_ERR_DTYPE: return "unknown dtype";
    case SECO_ERR_ALIGN: return "pointer or stride breaks the 16-byte row alignment";
    case SECO_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SECO_ERR_WEIGHTS: return "chunk weights do not cover the visible cache rows or are not finite";
    case SECO_ERR_RANGE: return "argument out of range";
    case SECO_ERR_LAUNCH: return "kernel launch failed";
    case SECO_ERR_TOO_LARGE: return "size exceeds the supported 32-bit range";
    default: return "unknown status";
  }
}
