// Dense FFN for a handful of tokens (M <= 4): the dense decode baseline that
// the sparse path of arXiv 2410.18311 (Sec. 4.2) is compared against, and the
// activation vector A(x) of Def. 1 for single tokens.  Both projections are
// row-dot GEMVs over weights in the nn.Linear layout, bandwidth bound:
//   up_rows_kernel   : H[m, n] = act(<w_up[n, :], X[m, :]> [+ b_up[n]]), fp32
//   down_rows_kernel : Y[m, j] = <w_down[j, :], H[m, :]> [+ b_down[j]]
// A workgroup owns a contiguous slice of output rows; its threads split the
// reduction dimension with 16-byte loads, reduce by wave shuffles and then
// across waves through LDS.
#include "common.hpp"

namespace ci {

namespace {

constexpr int RC = 4;  // weight rows in flight per thread

template <class D, bool SWIGLU>
__global__ __launch_bounds__(256) void up_rows_kernel(const void* __restrict__ X,
                                                      const void* __restrict__ w_up,
                                                      const void* __restrict__ w_gate,
                                                      const void* __restrict__ b_up, float* H,
                                                      float* A, int d, int N) {
  using T = typename D::T;
  constexpr int VEC = D::VEC;
  __shared__ float red[2][4][RC];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = blockIdx.y;
  const int r0 = (int)(((int64_t)blockIdx.x * N) / gridDim.x);
  const int r1 = (int)(((int64_t)(blockIdx.x + 1) * N) / gridDim.x);
  const T* x = reinterpret_cast<const T*>(X) + (size_t)m * d;
  const T* wu = reinterpret_cast<const T*>(w_up);
  const T* wg = reinterpret_cast<const T*>(w_gate);

  for (int rb = r0; rb < r1; rb += RC) {
    float su[RC], sg[RC];
#pragma unroll
    for (int j = 0; j < RC; ++j) su[j] = sg[j] = 0.f;
    for (int c = tid * VEC; c < d; c += 256 * VEC) {
      float xf[VEC];
      unpack<D>(ld16(x + c), xf);
      uint4 vu[RC], vg[RC];
#pragma unroll
      for (int j = 0; j < RC; ++j) {
        const int r = min(rb + j, r1 - 1);
        vu[j] = ld16(wu + (size_t)r * d + c);
        if (SWIGLU) vg[j] = ld16(wg + (size_t)r * d + c);
      }
#pragma unroll
      for (int j = 0; j < RC; ++j) {
        float f[VEC];
        unpack<D>(vu[j], f);
#pragma unroll
        for (int v = 0; v < VEC; ++v) su[j] = fmaf(f[v], xf[v], su[j]);
        if (SWIGLU) {
          unpack<D>(vg[j], f);
#pragma unroll
          for (int v = 0; v < VEC; ++v) sg[j] = fmaf(f[v], xf[v], sg[j]);
        }
      }
    }
#pragma unroll
    for (int j = 0; j < RC; ++j) {
      su[j] = wave_sum(su[j]);
      if (SWIGLU) sg[j] = wave_sum(sg[j]);
    }
    __syncthreads();
    if (lane == 0) {
#pragma unroll
      for (int j = 0; j < RC; ++j) {
        red[0][wave][j] = su[j];
        if (SWIGLU) red[1][wave][j] = sg[j];
      }
    }
    __syncthreads();
    if (tid < RC && rb + tid < r1) {
      const int r = rb + tid;
      float zu = red[0][0][tid] + red[0][1][tid] + red[0][2][tid] + red[0][3][tid];
      float h;
      if (SWIGLU) {
        const float zg = red[1][0][tid] + red[1][1][tid] + red[1][2][tid] + red[1][3][tid];
        h = silu(zg) * zu;
      } else {
        if (b_up) zu += to_float<D>(reinterpret_cast<const T*>(b_up)[r]);
        h = fmaxf(zu, 0.f);
      }
      if (H) H[(size_t)m * N + r] = h;
      if (A) A[(size_t)m * N + r] = fabsf(h);
    }
  }
}

template <class D>
__global__ __launch_bounds__(256) void down_rows_kernel(const float* __restrict__ H,
                                                        const void* __restrict__ w_down,
                                                        const void* __restrict__ b_down, void* Y,
                                                        int d, int N) {
  using T = typename D::T;
  constexpr int VEC = D::VEC;
  __shared__ float red[4][RC];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = blockIdx.y;
  const int r0 = (int)(((int64_t)blockIdx.x * d) / gridDim.x);
  const int r1 = (int)(((int64_t)(blockIdx.x + 1) * d) / gridDim.x);
  const float* h = H + (size_t)m * N;
  const T* w = reinterpret_cast<const T*>(w_down);

  for (int rb = r0; rb < r1; rb += RC) {
    float s[RC];
#pragma unroll
    for (int j = 0; j < RC; ++j) s[j] = 0.f;
    for (int c = tid * VEC; c < N; c += 256 * VEC) {
      float hf[VEC];
#pragma unroll
      for (int v = 0; v < VEC; v += 4) {
        const float4 t = *reinterpret_cast<const float4*>(h + c + v);
        hf[v] = t.x; hf[v + 1] = t.y; hf[v + 2] = t.z; hf[v + 3] = t.w;
      }
      uint4 vw[RC];
#pragma unroll
      for (int j = 0; j < RC; ++j) vw[j] = ld16(w + (size_t)min(rb + j, r1 - 1) * N + c);
#pragma unroll
      for (int j = 0; j < RC; ++j) {
        float f[VEC];
        unpack<D>(vw[j], f);
#pragma unroll
        for (int v = 0; v < VEC; ++v) s[j] = fmaf(f[v], hf[v], s[j]);
      }
    }
#pragma unroll
    for (int j = 0; j < RC; ++j) s[j] = wave_sum(s[j]);
    __syncthreads();
    if (lane == 0) {
#pragma unroll
      for (int j = 0; j < RC; ++j) red[wave][j] = s[j];
    }
    __syncthreads();
    if (tid < RC && rb + tid < r1) {
      const int r = rb + tid;
      float y = red[0][tid] + red[1][tid] + red[2][tid] + red[3][tid];
      if (b_down) y += to_float<D>(reinterpret_cast<const T*>(b_down)[r]);
      reinterpret_cast<T*>(Y)[(size_t)m * d + r] = from_float<D>(y);
    }
  }
}

int row_grid(int64_t rows) {
  DeviceInfo di;
  int cus = 256;
  if (device_info(&di) == CI_OK) cus = di.cus;
  int64_t g = (int64_t)cus * params().gemv_wgs_per_cu;
  if (g > (rows + RC - 1) / RC) g = (rows + RC - 1) / RC;
  return g < 1 ? 1 : (int)g;
}

template <class D>
int up_typed(const void* X, int M, const void* w_up, const void* w_gate, const void* b_up, int act,
             int d, int N, float* H, float* A, hipStream_t s) {
  dim3 grid(row_grid(N), M), block(256);
  if (act == CI_ACT_SWIGLU)
    hipLaunchKernelGGL((up_rows_kernel<D, true>), grid, block, 0, s, X, w_up, w_gate, b_up, H, A, d, N);
  else
    hipLaunchKernelGGL((up_rows_kernel<D, false>), grid, block, 0, s, X, w_up, w_gate, b_up, H, A, d, N);
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

template <class D>
int down_typed(const float* H, int M, const void* w_down, const void* b_down, int d, int N, void* Y,
               hipStream_t s) {
  dim3 grid(row_grid(d), M), block(256);
  hipLaunchKernelGGL((down_rows_kernel<D>), grid, block, 0, s, H, w_down, b_down, Y, d, N);
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

}  // namespace

int launch_up_rows(const void* X, int64_t M, const void* w_up, const void* w_gate, const void* b_up,
                   int dtype, int act, int64_t d, int64_t N, float* H, float* A, hipStream_t s) {
  switch (dtype) {
    case CI_F32: return up_typed<F32>(X, (int)M, w_up, w_gate, b_up, act, (int)d, (int)N, H, A, s);
    case CI_F16: return up_typed<F16>(X, (int)M, w_up, w_gate, b_up, act, (int)d, (int)N, H, A, s);
    case CI_BF16: return up_typed<BF16>(X, (int)M, w_up, w_gate, b_up, act, (int)d, (int)N, H, A, s);
  }
  return CI_ERR_BAD_DTYPE;
}

int launch_down_rows(const float* H, int64_t M, const void* w_down, const void* b_down, int dtype,
                     int64_t d, int64_t N, void* Y, hipStream_t s) {
  switch (dtype) {
    case CI_F32: return down_typed<F32>(H, (int)M, w_down, b_down, (int)d, (int)N, Y, s);
    case CI_F16: return down_typed<F16>(H, (int)M, w_down, b_down, (int)d, (int)N, Y, s);
    case CI_BF16: return down_typed<BF16>(H, (int)M, w_down, b_down, (int)d, (int)N, Y, s);
  }
  return CI_ERR_BAD_DTYPE;
}

}  // namespace ci
