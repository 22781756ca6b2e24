// Development probe (csrc/coreinfer_dev.h): how fast a compute unit's L1 is
// filled as a function of the bytes it keeps in flight.  Every workgroup
// streams 16-byte loads over a window of the caller's buffer -- one window
// shared by all workgroups (L2 hits once it is warm) or one window per
// workgroup (sized for L2, the memory-side cache or HBM) -- with DEPTH loads
// in flight per thread.  Measures what bounds the streaming kernels of this
// library (decode GEMV: HBM misses) and the tile loads of the prefill GEMM
// (a mix of L2 hits and misses).
#include "common.hpp"
#include "coreinfer_dev.h"

namespace ci {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int DEPTH>
__global__ __launch_bounds__(512) void stream_probe_kernel(const u32x4* __restrict__ buf, uint32_t win_vecs,
                                                           int per_wg, int iters, uint32_t* __restrict__ out) {
  const size_t base = per_wg ? (size_t)blockIdx.x * win_vecs : 0;
  u32x4 r[DEPTH];
  uint32_t acc = 0;
  uint32_t pos = threadIdx.x;  // < win_vecs: the host checks blockDim.x <= win_vecs
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int s = 0; s < DEPTH; ++s) {
      r[s] = buf[base + pos];
      pos += blockDim.x;
      pos = pos >= win_vecs ? pos - win_vecs : pos;
    }
#pragma unroll
    for (int s = 0; s < DEPTH; ++s) acc ^= r[s].x ^ r[s].y ^ r[s].z ^ r[s].w;
  }
  if (threadIdx.x == 0) out[blockIdx.x] = acc;  // keeps the loads alive
}

// The load stream of a GEMM operand tile without the arithmetic: 256 threads, every load instruction
// takes 128 bytes (eight lanes) of each of 32 rows that lie `pitch` bytes apart; DEPTH such instructions
// (32 * DEPTH rows) are in flight, then the same rows 128 bytes further along, `ksteps` times, and over again.
template <int DEPTH>
__global__ __launch_bounds__(256) void tile_probe_kernel(const unsigned char* __restrict__ buf, size_t pitch,
                                                         size_t wg_stride, int ksteps, int iters,
                                                         uint32_t* __restrict__ out) {
  const unsigned char* base = buf + (size_t)blockIdx.x * wg_stride + (size_t)(threadIdx.x >> 3) * pitch +
                              (size_t)(threadIdx.x & 7) * 16;
  u32x4 r[DEPTH];
  uint32_t acc = 0;
  int k = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int s = 0; s < DEPTH; ++s)
      r[s] = *reinterpret_cast<const u32x4*>(base + (size_t)(32 * s) * pitch + (size_t)k * 128);
#pragma unroll
    for (int s = 0; s < DEPTH; ++s) acc ^= r[s].x ^ r[s].y ^ r[s].z ^ r[s].w;
    k = k + 1 == ksteps ? 0 : k + 1;
  }
  if (threadIdx.x == 0) out[blockIdx.x] = acc;
}

}  // namespace
}  // namespace ci

extern "C" int coreinfer_dev_stream_probe(const void* buf, int64_t buf_bytes, int64_t window_bytes, int per_workgroup,
                                          int workgroups, int threads, int depth, int iters, void* out, void* stream) {
  using namespace ci;
  if (!buf || !out || workgroups < 1 || workgroups > 4096 || threads < 64 || threads > 512 || threads % 64 ||
      iters < 1 || window_bytes < 16 * (int64_t)threads || window_bytes % 16 || window_bytes > ((int64_t)1 << 34))
    return CI_ERR_INVALID_ARG;
  const int64_t need = per_workgroup ? window_bytes * workgroups : window_bytes;
  if (need > buf_bytes) return CI_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(buf) % 16) return CI_ERR_BAD_LAYOUT;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const u32x4* b = static_cast<const u32x4*>(buf);
  const uint32_t wv = (uint32_t)(window_bytes / 16);
  uint32_t* o = static_cast<uint32_t*>(out);
  switch (depth) {
    case 2: hipLaunchKernelGGL((stream_probe_kernel<2>), dim3(workgroups), dim3(threads), 0, s, b, wv, per_workgroup, iters, o); break;
    case 4: hipLaunchKernelGGL((stream_probe_kernel<4>), dim3(workgroups), dim3(threads), 0, s, b, wv, per_workgroup, iters, o); break;
    case 8: hipLaunchKernelGGL((stream_probe_kernel<8>), dim3(workgroups), dim3(threads), 0, s, b, wv, per_workgroup, iters, o); break;
    case 16: hipLaunchKernelGGL((stream_probe_kernel<16>), dim3(workgroups), dim3(threads), 0, s, b, wv, per_workgroup, iters, o); break;
    default: return CI_ERR_INVALID_ARG;
  }
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

extern "C" int coreinfer_dev_tile_probe(const void* buf, int64_t buf_bytes, int64_t pitch_bytes, int shared,
                                        int workgroups, int depth, int ksteps, int iters, void* out, void* stream) {
  using namespace ci;
  if (!buf || !out || workgroups < 1 || workgroups > 4096 || iters < 1 || ksteps < 1 || pitch_bytes < 128 ||
      pitch_bytes % 16 || (depth != 4 && depth != 8 && depth != 16))
    return CI_ERR_INVALID_ARG;
  // last byte a workgroup touches: row 32 * depth - 1, k-step ksteps - 1
  const int64_t rows = 32 * (int64_t)depth;
  const int64_t span = (rows - 1) * pitch_bytes + (int64_t)ksteps * 128;
  const int64_t wg_stride = shared ? 0 : rows * pitch_bytes;
  if (pitch_bytes > ((int64_t)1 << 24) || ksteps > 4096 || wg_stride * (workgroups - 1) + span > buf_bytes)
    return CI_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(buf) % 16) return CI_ERR_BAD_LAYOUT;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const unsigned char* b = static_cast<const unsigned char*>(buf);
  uint32_t* o = static_cast<uint32_t*>(out);
  switch (depth) {
    case 4: hipLaunchKernelGGL((tile_probe_kernel<4>), dim3(workgroups), dim3(256), 0, s, b, (size_t)pitch_bytes, (size_t)wg_stride, ksteps, iters, o); break;
    case 8: hipLaunchKernelGGL((tile_probe_kernel<8>), dim3(workgroups), dim3(256), 0, s, b, (size_t)pitch_bytes, (size_t)wg_stride, ksteps, iters, o); break;
    default: hipLaunchKernelGGL((tile_probe_kernel<16>), dim3(workgroups), dim3(256), 0, s, b, (size_t)pitch_bytes, (size_t)wg_stride, ksteps, iters, o); break;
  }
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}
