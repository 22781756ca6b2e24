// Device helpers shared by the decode-stage kernels (single-sentence /
// gathered decode and the union-batched decode).
#pragma once

#include "common.hpp"

namespace ci {

constexpr int kSuper = 64;  // rows of a slice handled between two barriers (<= smallest workgroup)

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// 16-byte streaming load: the weights are read once per token and never
// reused, so they are marked non-temporal.
__device__ __forceinline__ uint4 ld16_stream(const void* p) {
  const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(t[0], t[1], t[2], t[3]);
}

// Sums DEPTH per-lane values across the wave with a halving butterfly: after
// the call every lane holds the wave-wide sum of value number
// lane / (64 / DEPTH) -- for DEPTH = 8, 10 shuffles instead of 48.
template <int N, int BIT>
__device__ __forceinline__ void halve_rows(float* v, int lane) {
  if constexpr (N > 1) {
    const bool hi = (lane & BIT) != 0;
#pragma unroll
    for (int i = 0; i < N / 2; ++i) {
      const float send = hi ? v[i] : v[i + N / 2];
      const float keep = hi ? v[i + N / 2] : v[i];
      v[i] = keep + __shfl_xor(send, BIT, kWave);
    }
    halve_rows<N / 2, BIT / 2>(v, lane);
  } else {
    float r = v[0];
#pragma unroll
    for (int bit = BIT; bit >= 1; bit >>= 1) r += __shfl_xor(r, bit, kWave);
    v[0] = r;
  }
}

}  // namespace ci
