// Counter-based generator of the method's random draws: a four-level integer hash of
// (seed, stream, a, b, c) whose top 23 bits m give the uniform (m + 1/2) 2^-23 in (0,1),
// exactly representable in fp32.  The mixing function is the SplitMix64 finaliser.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ssd {

enum { STREAM_ACCEPT = 0, STREAM_BONUS = 1, STREAM_DRAFT = 2, STREAM_BACKUP = 4 };

__host__ __device__ __forceinline__ uint64_t mix64(uint64_t x) {
  x ^= x >> 30;
  x *= 0xBF58476D1CE4E5B9ull;
  x ^= x >> 27;
  x *= 0x94D049BB133111EBull;
  x ^= x >> 31;
  return x;
}

// Hash state after (seed, stream, a, b); the last level is applied per token by draw_u.
__host__ __device__ __forceinline__ uint64_t draw_prefix(uint64_t seed, uint32_t stream, uint64_t a, uint64_t b) {
  uint64_t h = mix64(seed ^ (0x9E3779B97F4A7C15ull * (uint64_t)(stream + 1)));
  h = mix64(h + a);
  h = mix64(h + b);
  return h;
}

__host__ __device__ __forceinline__ double draw_u(uint64_t prefix, uint64_t c) {
  uint64_t m = mix64(prefix + c) >> 41;
  return ((double)m + 0.5) * (1.0 / 8388608.0);
}

__device__ __forceinline__ double gumbel_from_u(double u) { return -log(-log(u)); }

}  // namespace ssd
