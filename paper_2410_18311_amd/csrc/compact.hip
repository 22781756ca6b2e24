// Deploying the core neurons (Sec. 5.3 of arXiv 2410.18311): one-time gather
// of the weights that the sentence's core set S names into contiguous,
// neuron-major buffers, so that every decode token streams them linearly.
//
//   gather_rows_kernel      : out[k, :] = in[S[k], :] for up / gate / a
//                             neuron-major down matrix, 16-byte copies; also
//                             gathers the up bias and validates S.
//   gather_cols_t_kernel    : out[k, j] = in[j, S[k]] for the nn.Linear
//                             [d, N] down matrix: 64x64 tiles staged through
//                             LDS so that both the reads (along S, which is
//                             ascending) and the writes (along j) touch whole
//                             cache lines.
#include "common.hpp"

namespace ci {

namespace {

struct RowGather {
  const void* in[3];
  void* out[3];
  int n_mat;
  const void* b_in;
  void* b_out;
  int elem;  // bytes per element
};

__device__ __forceinline__ bool index_ok(const int32_t* idx, int k, int N) {
  const int n = idx[k];
  return n >= 0 && n < N && (k == 0 || idx[k - 1] < n);
}

__global__ __launch_bounds__(256) void gather_rows_kernel(RowGather g, const int32_t* __restrict__ idx,
                                                          int K, int N, int vecs_per_row,
                                                          int32_t* status) {
  const int k = blockIdx.x, mat = blockIdx.y;
  const bool ok = index_ok(idx, k, N);
  const size_t src = ok ? (size_t)idx[k] : 0;
  const uint4* in = reinterpret_cast<const uint4*>(g.in[mat]) + src * vecs_per_row;
  uint4* out = reinterpret_cast<uint4*>(g.out[mat]) + (size_t)k * vecs_per_row;
  for (int v = threadIdx.x; v < vecs_per_row; v += blockDim.x)
    out[v] = ok ? in[v] : make_uint4(0, 0, 0, 0);
  if (mat == 0 && threadIdx.x == 0) {
    if (!ok && status) *status = 1;
    if (g.b_in) {
      if (g.elem == 2)
        reinterpret_cast<uint16_t*>(g.b_out)[k] = ok ? reinterpret_cast<const uint16_t*>(g.b_in)[src] : (uint16_t)0;
      else
        reinterpret_cast<uint32_t*>(g.b_out)[k] = ok ? reinterpret_cast<const uint32_t*>(g.b_in)[src] : 0u;
    }
  }
}

template <class E>
__global__ __launch_bounds__(256) void gather_cols_t_kernel(const E* __restrict__ in, E* __restrict__ out,
                                                            const int32_t* __restrict__ idx, int K,
                                                            int N, int d) {
  __shared__ E tile[64][65];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int k0 = blockIdx.x * 64, j0 = blockIdx.y * 64;
  const int k = k0 + tx;
  bool ok = false;
  size_t n = 0;
  if (k < K) {
    ok = index_ok(idx, k, N);
    n = ok ? (size_t)idx[k] : 0;
  }
  for (int jj = ty; jj < 64; jj += 4) {
    const int j = j0 + jj;
    E v = 0;
    if (ok && j < d) v = in[(size_t)j * N + n];
    tile[jj][tx] = v;
  }
  __syncthreads();
  const int j = j0 + tx;
  for (int kk = ty; kk < 64; kk += 4) {
    if (k0 + kk < K && j < d) out[(size_t)(k0 + kk) * d + j] = tile[tx][kk];
  }
}

}  // namespace

int launch_compact(const void* w_up, const void* w_gate, const void* b_up, const void* w_down,
                   int down_layout, int dtype, int64_t d, int64_t N, const int32_t* core_idx,
                   int64_t K, void* w_up_c, void* w_gate_c, void* b_up_c, void* w_down_c,
                   int32_t* status, hipStream_t s) {
  if (K == 0) return CI_OK;
  const int e = elem_bytes(dtype);
  RowGather g;
  g.n_mat = 0;
  g.in[g.n_mat] = w_up; g.out[g.n_mat++] = w_up_c;
  if (w_gate) { g.in[g.n_mat] = w_gate; g.out[g.n_mat++] = w_gate_c; }
  if (down_layout == CI_DOWN_NEURON_MAJOR) { g.in[g.n_mat] = w_down; g.out[g.n_mat++] = w_down_c; }
  for (int i = g.n_mat; i < 3; ++i) { g.in[i] = nullptr; g.out[i] = nullptr; }
  g.b_in = b_up;
  g.b_out = b_up_c;
  g.elem = e;
  const int vecs = (int)(d * e / 16);
  hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)K, g.n_mat), dim3(256), 0, s, g, core_idx,
                     (int)K, (int)N, vecs, status);
  CI_HIP_CHECK_LAUNCH();
  if (down_layout == CI_DOWN_OUT_MAJOR) {
    dim3 grid((unsigned)((K + 63) / 64), (unsigned)((d + 63) / 64));
    if (e == 2)
      hipLaunchKernelGGL((gather_cols_t_kernel<uint16_t>), grid, dim3(256), 0, s,
                         reinterpret_cast<const uint16_t*>(w_down), reinterpret_cast<uint16_t*>(w_down_c),
                         core_idx, (int)K, (int)N, (int)d);
    else
      hipLaunchKernelGGL((gather_cols_t_kernel<uint32_t>), grid, dim3(256), 0, s,
                         reinterpret_cast<const uint32_t*>(w_down), reinterpret_cast<uint32_t*>(w_down_c),
                         core_idx, (int)K, (int)N, (int)d);
    CI_HIP_CHECK_LAUNCH();
  }
  return CI_OK;
}

}  // namespace ci
