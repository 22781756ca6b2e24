// Shared device / host helpers for libcoreinfer (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "coreinfer.h"

namespace ci {

constexpr int kWave = 64;

// ---- element types ---------------------------------------------------------
// VEC = elements per 16-byte global load.
struct F32 {
  using T = float;
  static constexpr int VEC = 4;
  static constexpr int BYTES = 4;
};
struct F16 {
  using T = _Float16;
  static constexpr int VEC = 8;
  static constexpr int BYTES = 2;
};
struct BF16 {
  using T = uint16_t;  // raw bits
  static constexpr int VEC = 8;
  static constexpr int BYTES = 2;
};

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t f2u(float f) { return __builtin_bit_cast(uint32_t, f); }

__device__ __forceinline__ uint4 ld16(const void* p) {
  return *reinterpret_cast<const uint4*>(p);
}

// Expand one 16-byte vector into fp32 lanes.
template <class D>
__device__ __forceinline__ void unpack(const uint4& v, float (&f)[D::VEC]);

template <>
__device__ __forceinline__ void unpack<F32>(const uint4& v, float (&f)[4]) {
  f[0] = u2f(v.x); f[1] = u2f(v.y); f[2] = u2f(v.z); f[3] = u2f(v.w);
}
template <>
__device__ __forceinline__ void unpack<F16>(const uint4& v, float (&f)[8]) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    half2_t h = __builtin_bit_cast(half2_t, w[i]);
    f[2 * i] = (float)h[0];
    f[2 * i + 1] = (float)h[1];
  }
}
template <>
__device__ __forceinline__ void unpack<BF16>(const uint4& v, float (&f)[8]) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = u2f(w[i] << 16);
    f[2 * i + 1] = u2f(w[i] & 0xffff0000u);
  }
}

template <class D>
__device__ __forceinline__ float to_float(typename D::T v);
template <> __device__ __forceinline__ float to_float<F32>(float v) { return v; }
template <> __device__ __forceinline__ float to_float<F16>(_Float16 v) { return (float)v; }
template <> __device__ __forceinline__ float to_float<BF16>(uint16_t v) { return u2f((uint32_t)v << 16); }

// fp32 -> element, round to nearest even.
template <class D>
__device__ __forceinline__ typename D::T from_float(float f);
template <> __device__ __forceinline__ float from_float<F32>(float f) { return f; }
template <> __device__ __forceinline__ _Float16 from_float<F16>(float f) { return (_Float16)f; }
template <> __device__ __forceinline__ uint16_t from_float<BF16>(float f) {
  uint32_t u = f2u(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float silu(float z) { return z / (1.0f + __expf(-z)); }

// ---- wave64 primitives -----------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}
__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}
__device__ __forceinline__ uint64_t lanemask_lt() {
  return (1ull << (threadIdx.x & 63)) - 1ull;
}

// ---- host side -------------------------------------------------------------
struct DeviceInfo {
  int cus;
};
// Compute-unit count of the current device (queried once per device).
int device_info(DeviceInfo* out);

// Development knobs (see coreinfer_dev.h).  Relaxed atomics: a sweep may change one while
// another thread is inside an entry point; each reads a consistent value of each knob.
struct Knob {
  std::atomic<int> v;
  explicit Knob(int x) : v(x) {}
  operator int() const { return v.load(std::memory_order_relaxed); }
  void operator=(int x) { v.store(x, std::memory_order_relaxed); }
};
struct Params {
  Knob decode_wgs_per_cu{1};
  Knob decode_wgs{0};        // absolute number of neuron slices per sentence (0 = per-CU rule)
  Knob decode_threads{0};    // 0 = derived from d
  Knob decode_depth{4};      // weight rows in flight per thread (4, 8 or 16)
  Knob select_wgs_per_cu{2};
  Knob select_def2_single{0};  // Def. 2 in one workgroup even where the parallel kernel applies
  Knob gemv_wgs_per_cu{4};
  Knob gemm_ring{1};         // register-ring GEMM kernel where it applies
  Knob gemm_direct{1};       // 128 x 128 tiles loaded straight into LDS instead of through the register ring
  Knob gemm_big{1};          // 256 x 256 tiles: 0 never, 1 when there are enough of them, 2 whenever the shape divides
  Knob reduce_threads{256};  // threads per reduce workgroup (64, 128, 256)
  Knob reduce_cq{8};         // column quads per reduce workgroup (4, 8, 16)
  Knob decode_nt_store{1};   // non-temporal stores for the partial sums
  Knob union_depth{8};            // union-batched decode: rows in flight per thread (8 or 16)
  Knob union_down_threads{384};   // threads (= 16-byte column vectors) per down-phase workgroup
  Knob union_up_wgs_per_cu{1};
  Knob union_down_wgs_per_cu{2};
  Knob union_super{0};            // cap on the rows between two ring drains (0: 256 or what LDS holds)
  Knob fused_depth{4};     // single-launch decode: rows in flight per thread (4, 8 or 16)
  Knob fused_threads{0};   // 0 = derived from d
  Knob fused_chunks{2};    // least number of neuron chunks
  Knob fused_chunk_size{0}; // 0 = chosen by the cost model, else neurons per chunk (used if it respects the limits)
  Knob fused_wgs{0};       // 0 = one workgroup per compute unit
  Knob fused_ablate{0};    // development builds only
  Knob fused_chunk_cost10{80};  // tenths of a ring slot that a chunk's two barriers are counted as
  Knob fused_window_slots{13};  // ring slots the exchange of a chunk needs between its publication and its use
  Knob fused_guard_us10{12}; // tenths of a microsecond after a phase's end at which its hidden values are collected
  Knob fused_aux{-1};       // ring loads: buffer loads with these cache-policy bits (0, 16), or global loads (-1 non-temporal, -2 plain)
};
Params& params();

inline int elem_bytes(int dtype) { return dtype == CI_F32 ? 4 : 2; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Raises a kernel's dynamic-LDS limit once per device.  `seen` holds one bit per device ordinal;
// a bit is set only after the call succeeded, so a failure is reported again by the next launch.
// Ordinals past 63 are not remembered (the attribute is set on every launch there).
inline int allow_dynamic_lds(std::atomic<uint64_t>& seen, const void* kernel, size_t bytes) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return CI_ERR_HIP;
  const uint64_t bit = dev < 64 ? 1ull << dev : 0;
  if (seen.load(std::memory_order_acquire) & bit) return CI_OK;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
    return CI_ERR_HIP;
  seen.fetch_or(bit, std::memory_order_release);
  return CI_OK;
}

#define CI_HIP_CHECK_LAUNCH()                          \
  do {                                                 \
    if (hipGetLastError() != hipSuccess) return CI_ERR_HIP; \
  } while (0)

// ---- launchers (one per translation unit) ----------------------------------
enum { kSelZero = 1, kSelTokens = 2, kSelFinal = 4, kSelAccumulate = 8 };
struct SelectWs {
  size_t off_thr, off_hist, off_counts, total;
};
void select_ws_layout(int64_t M, int64_t N, SelectWs* w, int64_t B = 1);
bool select_batch_ok(int64_t M, int64_t N);
// ws: laid out by select_ws_layout (may be null when only kSelZero is asked for)
int launch_select(const void* act, int act_dtype, int take_abs, int64_t M, int64_t N, int64_t ld, int64_t q_alpha,
                  int64_t K, int64_t max_count, int32_t* core_idx, int32_t* counts, void* ws, int what,
                  hipStream_t s, int B = 1, int64_t counts_stride = 0);
int launch_scatter_count(const int32_t* idx, int64_t n_idx, int64_t N, int32_t* counts, hipStream_t s);
int launch_similarity(const int32_t* a, int64_t Ka, const int32_t* b, int64_t Kb, int32_t* out, hipStream_t s);
int launch_assign_group(const int32_t* set, int64_t K, const int32_t* groups, int64_t G, int64_t Kg,
                        int32_t* best, int32_t* iu, hipStream_t s);
int launch_assign_centroid(const float* act, int64_t M, int64_t N, int64_t ld, const float* centroids,
                           int64_t G, int32_t* best, float* dist, float* feature, hipStream_t s);
// Leading dimension of an output-major compact down matrix [d, ld]: K rounded up to whole 16-byte vectors.
inline int64_t compact_down_ld(int64_t K, int dtype) {
  const int64_t v = 16 / elem_bytes(dtype);
  return (K + v - 1) / v * v;
}
int launch_compact(const void* w_up, const void* w_gate, const void* b_up, const void* w_down,
                   int down_layout, int dtype, int64_t d, int64_t N, const int32_t* core_idx,
                   int64_t K, void* w_up_c, void* w_gate_c, void* b_up_c, void* w_down_c,
                   int down_c_layout, int32_t* status, hipStream_t s);
int launch_compact_update(const void* w_up, const void* w_gate, const void* b_up, const void* w_down,
                          int down_layout, int dtype, int64_t d, int64_t N, const int32_t* new_idx,
                          int64_t K, int32_t* slot_idx, void* w_up_c, void* w_gate_c, void* b_up_c,
                          void* w_down_c, int down_c_layout, int32_t* changed, uint32_t* ws, hipStream_t s);
int decode_splits(int64_t B, int64_t K);
int launch_ffn_decode(const void* x, int64_t B, const ci_ffn_weights* w, int dtype, int act,
                      void* y, float* partial, hipStream_t s);
int launch_decode_reduce(const float* partial, const void* b_down, void* y, int n_wg, int d, int B,
                         int dtype, hipStream_t s);
size_t fused_decode_ws_bytes(int64_t K);
int fused_decode_plan(int64_t K, int64_t d, int dtype, int act, int* out);
int launch_ffn_decode_fused(const void* x, int64_t B, const ci_ffn_weights* w, int dtype, int act, void* y,
                            void* ws, hipStream_t s);
int union_up_chunks(int64_t vecs);
int launch_union_build(const int32_t* core_idx, int64_t B, int64_t K, int64_t N, int64_t cap,
                       int32_t* uidx, uint32_t* umask, int32_t* ucount, uint32_t* owners,
                       hipStream_t s);
int launch_ffn_decode_union(const void* x, int64_t B, const ci_ffn_weights* w, const int32_t* uidx,
                            const uint32_t* umask, const int32_t* ucount, int64_t cap, int dtype,
                            int act, void* y, float* ws, hipStream_t s);
// h[M, N] fp32 = act(X w^T ...) and y = W h + b by row-dot GEMVs (small M).
int launch_up_rows(const void* X, int64_t M, const void* w_up, const void* w_gate, const void* b_up,
                   int dtype, int act, int64_t d, int64_t N, float* H, float* A, hipStream_t s);
int launch_down_rows(const float* H, int64_t M, const void* w_down, const void* b_down, int dtype,
                     int64_t d, int64_t N, void* Y, hipStream_t s);
int launch_gemm_up(const void* X, int64_t M, const void* w_up, const void* w_gate, const void* b_up,
                   int dtype, int act, int64_t d, int64_t N, void* H, float* A, hipStream_t s);
int gemm_down_splits(int64_t M, int64_t d, int64_t N, int dtype);
int gemm_down_splits_max(int64_t M, int64_t d, int64_t N, int dtype);  // what the workspace is sized for
int launch_gemm_down(const void* H, int64_t M, const void* w_down, const void* b_down,
                     int down_layout, int dtype, int64_t d, int64_t N, void* Y, float* partial,
                     hipStream_t s);

}  // namespace ci
