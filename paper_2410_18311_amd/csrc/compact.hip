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
//   compact_fused_kernel    : both of the above in one launch (column tiles
//                             first) when the down matrix is [d, N].
// For the single-launch decode the down matrix is kept output-major instead,
// out [d, ld] = w_down[:, S] with the columns K .. ld-1 zero:
//   gather_cols_kernel      : out[j, k] = in[j, S[k]] from the nn.Linear
//                             [d, N] matrix: a thread holds the indices of one
//                             16-byte group of k and walks down the rows.
//   gather_rows_t_kernel    : out[j, k] = in[S[k], j] from a neuron-major
//                             [N, d] matrix, 64x64 tiles through LDS.
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

__device__ __forceinline__ void gather_row(const RowGather& g, const int32_t* __restrict__ idx, int k, int mat,
                                           int N, int vecs_per_row, int32_t* status) {
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

__global__ __launch_bounds__(256) void gather_rows_kernel(RowGather g, const int32_t* __restrict__ idx,
                                                          int N, int vecs_per_row, int32_t* status) {
  gather_row(g, idx, blockIdx.x, blockIdx.y, N, vecs_per_row, status);
}

// One 64 x 64 tile of out[k, j] = in[j, S[k]]: tile column block bk, row block bj.
template <class E>
__device__ __forceinline__ void gather_cols_tile(const E* __restrict__ in, E* __restrict__ out,
                                                 const int32_t* __restrict__ idx, int K, int N, int d, int bk,
                                                 int bj, E (*tile)[65]) {
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int k0 = bk * 64, j0 = bj * 64;
  const int k = k0 + tx;
  bool ok = false;
  size_t n = 0;
  if (k < K) {
    ok = index_ok(idx, k, N);
    n = ok ? (size_t)idx[k] : 0;
  }
  // all 16 loads of a thread in flight before the first is used
  E v[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int j = j0 + ty + 4 * i;
    const bool take = ok && j < d;
    const E t = in[take ? (size_t)j * N + n : (size_t)0];
    v[i] = take ? t : (E)0;
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) tile[ty + 4 * i][tx] = v[i];
  __syncthreads();
  const int j = j0 + tx;
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = tile[tx][ty + 4 * i];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int kk = ty + 4 * i;
    if (k0 + kk < K && j < d) out[(size_t)(k0 + kk) * d + j] = v[i];
  }
}

template <class E>
__global__ __launch_bounds__(256) void gather_cols_t_kernel(const E* __restrict__ in, E* __restrict__ out,
                                                            const int32_t* __restrict__ idx, int K,
                                                            int N, int d) {
  __shared__ E tile[64][65];
  gather_cols_tile<E>(in, out, idx, K, N, d, blockIdx.x, blockIdx.y, tile);
}

// Whole deployment with an nn.Linear ([d, N]) down matrix in one launch: the first n_col_blocks
// workgroups transpose-gather the down columns (the longer part, so it starts first), the rest copy
// rows of up / gate.  One launch instead of two, and the two streams overlap.
template <class E>
__global__ __launch_bounds__(256) void compact_fused_kernel(RowGather g, const E* __restrict__ w_down,
                                                            E* __restrict__ w_down_c,
                                                            const int32_t* __restrict__ idx, int K, int N, int d,
                                                            int vecs_per_row, int kblocks, int n_col_blocks,
                                                            int32_t* status) {
  __shared__ E tile[64][65];
  const int b = blockIdx.x;
  if (b < n_col_blocks) {
    gather_cols_tile<E>(w_down, w_down_c, idx, K, N, d, b % kblocks, b / kblocks, tile);
  } else {
    const int r = b - n_col_blocks;
    gather_row(g, idx, r % K, r / K, N, vecs_per_row, status);
  }
}

// out[j, k] = in[j, S[k]] for k < K, 0 for K <= k < ld.  A thread owns VE = 16 / sizeof(E)
// consecutive k (one 16-byte store per row) and ROWS rows; the indices stay in registers.
template <class E, int ROWS>
__global__ __launch_bounds__(256) void gather_cols_kernel(const E* __restrict__ in, E* __restrict__ out,
                                                          const int32_t* __restrict__ idx, int K, int ld,
                                                          int N, int d, int32_t* status) {
  constexpr int VE = 16 / sizeof(E);
  const int kv = blockIdx.x * 256 + threadIdx.x;  // 16-byte group along k
  const int k0 = kv * VE;
  if (k0 >= ld) return;
  uint32_t src[VE];
  bool okv[VE];
  bool bad = false;
#pragma unroll
  for (int e = 0; e < VE; ++e) {
    const int k = k0 + e;
    okv[e] = k < K && index_ok(idx, k, N);
    bad |= k < K && !okv[e];
    src[e] = okv[e] ? (uint32_t)idx[k] : 0u;
  }
  if (bad && status && blockIdx.y == 0) *status = 1;
  const int j0 = blockIdx.y * ROWS;
#pragma unroll 4
  for (int r = 0; r < ROWS; ++r) {
    const int j = j0 + r;
    if (j >= d) break;
    const E* row = in + (size_t)j * N;
    E v[VE];
#pragma unroll
    for (int e = 0; e < VE; ++e) v[e] = row[src[e]];
#pragma unroll
    for (int e = 0; e < VE; ++e) v[e] = okv[e] ? v[e] : (E)0;
    uint4 pack;
    __builtin_memcpy(&pack, v, 16);
    *reinterpret_cast<uint4*>(out + (size_t)j * ld + k0) = pack;
  }
}

// out[j, k] = in[S[k], j] (k < K; 0 up to ld): 64 k x 64 j tiles, reads along j, writes along k.
template <class E>
__global__ __launch_bounds__(256) void gather_rows_t_kernel(const E* __restrict__ in, E* __restrict__ out,
                                                            const int32_t* __restrict__ idx, int K, int ld,
                                                            int N, int d, int32_t* status) {
  __shared__ E tile[64][65];
  __shared__ int srow[64];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int k0 = blockIdx.x * 64, j0 = blockIdx.y * 64;
  if (ty == 0) {
    const int k = k0 + tx;
    int n = -1;
    if (k < K) {
      if (index_ok(idx, k, N)) n = idx[k];
      else if (status && blockIdx.y == 0) *status = 1;
    }
    srow[tx] = n;
  }
  __syncthreads();
  E v[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int n = srow[ty + 4 * i];
    const int j = j0 + tx;
    const bool take = n >= 0 && j < d;
    const E t = in[take ? (size_t)n * d + j : (size_t)0];
    v[i] = take ? t : (E)0;
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) tile[ty + 4 * i][tx] = v[i];
  __syncthreads();
  const int k = k0 + tx;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int j = j0 + ty + 4 * i;
    if (j < d && k < ld) out[(size_t)j * ld + k] = tile[tx][ty + 4 * i];
  }
}

// ---- in-place update after the core set changed ------------------------------
// flags[n]: 0 not in the new set, 1 in the new set and not yet deployed, 2 in
// the new set and already held by a row.
__global__ void delta_zero_kernel(uint32_t* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}
__global__ void delta_mark_new_kernel(const int32_t* __restrict__ new_idx, int K, int N, uint32_t* flags) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= K) return;
  const int n = new_idx[j];
  if (n >= 0 && n < N) flags[n] = 1u;
}
// keep[j] = 1 when row j's neuron stays (first row to claim it), else the row is free
__global__ void delta_mark_kept_kernel(const int32_t* __restrict__ slot_idx, int K, int N, uint32_t* flags,
                                       uint32_t* keep) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= K) return;
  const int n = slot_idx[j];
  uint32_t k = 0;
  if (n >= 0 && n < N) k = atomicCAS(&flags[n], 1u, 2u) == 1u ? 1u : 0u;
  keep[j] = k;
}
// Ordered lists of the free rows (ascending row) and of the entering neurons
// (ascending neuron); count[0] = number of pairs.  One workgroup.
__global__ __launch_bounds__(1024) void delta_pair_kernel(const int32_t* __restrict__ new_idx,
                                                          const uint32_t* __restrict__ flags,
                                                          const uint32_t* __restrict__ keep, int K, int N,
                                                          int32_t* free_list, int32_t* enter_list,
                                                          int32_t* count, int32_t* changed) {
  __shared__ int wf[16], we[16];
  __shared__ int base_f, base_e;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) { base_f = 0; base_e = 0; }
  __syncthreads();
  for (int j0 = 0; j0 < K; j0 += 1024) {
    const int j = j0 + tid;
    const bool is_free = j < K && keep[j] == 0u;
    int n = -1;
    if (j < K) n = new_idx[j];
    // entering: in the new set, not held by any row; a duplicate in new_idx counts once (its first place)
    const bool enters = j < K && n >= 0 && n < N && flags[n] == 1u && (j == 0 || new_idx[j - 1] != n);
    const uint64_t bf = __ballot(is_free), be = __ballot(enters);
    if (lane == 0) { wf[wave] = __popcll(bf); we[wave] = __popcll(be); }
    __syncthreads();
    int of = base_f, oe = base_e;
    for (int w = 0; w < wave; ++w) { of += wf[w]; oe += we[w]; }
    if (is_free) free_list[of + __popcll(bf & lanemask_lt())] = j;
    if (enters) enter_list[oe + __popcll(be & lanemask_lt())] = n;
    __syncthreads();
    if (tid == 0) {
      int tf = 0, te = 0;
      for (int w = 0; w < 16; ++w) { tf += wf[w]; te += we[w]; }
      base_f += tf; base_e += te;
    }
    __syncthreads();
  }
  if (tid == 0) {
    const int c = base_f < base_e ? base_f : base_e;
    count[0] = c;
    if (changed) changed[0] = c;
  }
}
// Row t of the pair list: the entering neuron's weights go to the free row.
__global__ __launch_bounds__(256) void delta_rows_kernel(RowGather g, const int32_t* __restrict__ free_list,
                                                         const int32_t* __restrict__ enter_list,
                                                         const int32_t* __restrict__ count,
                                                         int32_t* slot_idx, int vecs_per_row) {
  const int t = blockIdx.x, mat = blockIdx.y;
  if (t >= count[0]) return;
  const size_t dst = (size_t)free_list[t], src = (size_t)enter_list[t];
  const uint4* in = reinterpret_cast<const uint4*>(g.in[mat]) + src * vecs_per_row;
  uint4* out = reinterpret_cast<uint4*>(g.out[mat]) + dst * vecs_per_row;
  for (int v = threadIdx.x; v < vecs_per_row; v += blockDim.x) out[v] = in[v];
  if (mat == 0 && threadIdx.x == 0) {
    slot_idx[dst] = (int32_t)src;
    if (g.b_in) {
      if (g.elem == 2) reinterpret_cast<uint16_t*>(g.b_out)[dst] = reinterpret_cast<const uint16_t*>(g.b_in)[src];
      else reinterpret_cast<uint32_t*>(g.b_out)[dst] = reinterpret_cast<const uint32_t*>(g.b_in)[src];
    }
  }
}
// nn.Linear [d, N] down matrix: out[free_list[t], j] = in[j, enter_list[t]], 64 pairs x 64 j per workgroup.
template <class E>
__global__ __launch_bounds__(256) void delta_cols_t_kernel(const E* __restrict__ in, E* __restrict__ out,
                                                           const int32_t* __restrict__ free_list,
                                                           const int32_t* __restrict__ enter_list,
                                                           const int32_t* __restrict__ count, int N, int d) {
  __shared__ E tile[64][65];
  __shared__ int sdst[64];
  const int c = count[0];
  const int t0 = blockIdx.x * 64, j0 = blockIdx.y * 64;
  if (t0 >= c) return;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int t = t0 + tx;
  const bool ok = t < c;
  const size_t n = ok ? (size_t)enter_list[t] : 0;
  if (ty == 0) sdst[tx] = ok ? free_list[t] : 0;
  E v[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int j = j0 + ty + 4 * i;
    const bool take = ok && j < d;
    const E x = in[take ? (size_t)j * N + n : (size_t)0];
    v[i] = take ? x : (E)0;
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) tile[ty + 4 * i][tx] = v[i];
  __syncthreads();
  const int j = j0 + tx;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int kk = ty + 4 * i;
    if (t0 + kk < c && j < d) out[(size_t)sdst[kk] * d + j] = tile[tx][kk];
  }
}

// Output-major compact down matrix: column free_list[t] of out [d, ld] takes neuron enter_list[t],
// from in [d, N] (in_neuron_major == 0) or in [N, d].
template <class E>
__global__ __launch_bounds__(256) void delta_cols_kernel(const E* __restrict__ in, E* __restrict__ out,
                                                         const int32_t* __restrict__ free_list,
                                                         const int32_t* __restrict__ enter_list,
                                                         const int32_t* __restrict__ count, int N, int d, int ld,
                                                         int in_neuron_major) {
  const int t = blockIdx.x;
  if (t >= count[0]) return;
  const size_t dst = (size_t)free_list[t], src = (size_t)enter_list[t];
  for (int j = blockIdx.y * 256 + threadIdx.x; j < d; j += gridDim.y * 256)
    out[(size_t)j * ld + dst] = in_neuron_major ? in[src * d + j] : in[(size_t)j * N + src];
}

}  // namespace

int launch_compact_update(const void* w_up, const void* w_gate, const void* b_up, const void* w_down,
                          int down_layout, int dtype, int64_t d, int64_t N, const int32_t* new_idx,
                          int64_t K, int32_t* slot_idx, void* w_up_c, void* w_gate_c, void* b_up_c,
                          void* w_down_c, int down_c_layout, int32_t* changed, uint32_t* ws, hipStream_t s) {
  // workspace: flags [N], keep [K], free_list [K], enter_list [K], count [1]
  uint32_t* flags = ws;
  uint32_t* keep = flags + N;
  int32_t* free_list = reinterpret_cast<int32_t*>(keep + K);
  int32_t* enter_list = free_list + K;
  int32_t* count = enter_list + K;
  const unsigned gk = (unsigned)((K + 255) / 256);
  hipLaunchKernelGGL(delta_zero_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, s, flags, N);
  if (K > 0) {
    hipLaunchKernelGGL(delta_mark_new_kernel, dim3(gk), dim3(256), 0, s, new_idx, (int)K, (int)N, flags);
    hipLaunchKernelGGL(delta_mark_kept_kernel, dim3(gk), dim3(256), 0, s, slot_idx, (int)K, (int)N, flags, keep);
  }
  hipLaunchKernelGGL(delta_pair_kernel, dim3(1), dim3(1024), 0, s, new_idx, flags, keep, (int)K, (int)N,
                     free_list, enter_list, count, changed);
  CI_HIP_CHECK_LAUNCH();
  if (K == 0) return CI_OK;
  const int e = elem_bytes(dtype);
  RowGather g;
  g.n_mat = 0;
  g.in[g.n_mat] = w_up; g.out[g.n_mat++] = w_up_c;
  if (w_gate) { g.in[g.n_mat] = w_gate; g.out[g.n_mat++] = w_gate_c; }
  const bool down_as_rows = down_layout == CI_DOWN_NEURON_MAJOR && down_c_layout == CI_DOWN_NEURON_MAJOR;
  if (down_as_rows) { g.in[g.n_mat] = w_down; g.out[g.n_mat++] = w_down_c; }
  for (int i = g.n_mat; i < 3; ++i) { g.in[i] = nullptr; g.out[i] = nullptr; }
  g.b_in = b_up;
  g.b_out = b_up_c;
  g.elem = e;
  // the down columns first: the row kernel rewrites slot_idx, which nothing below reads
  if (down_c_layout == CI_DOWN_OUT_MAJOR) {
    const int ld = (int)compact_down_ld(K, dtype);
    dim3 grid((unsigned)K, (unsigned)((d + 1023) / 1024));
    const int nm = down_layout == CI_DOWN_NEURON_MAJOR ? 1 : 0;
    if (e == 2)
      hipLaunchKernelGGL((delta_cols_kernel<uint16_t>), grid, dim3(256), 0, s,
                         reinterpret_cast<const uint16_t*>(w_down), reinterpret_cast<uint16_t*>(w_down_c),
                         free_list, enter_list, count, (int)N, (int)d, ld, nm);
    else
      hipLaunchKernelGGL((delta_cols_kernel<uint32_t>), grid, dim3(256), 0, s,
                         reinterpret_cast<const uint32_t*>(w_down), reinterpret_cast<uint32_t*>(w_down_c),
                         free_list, enter_list, count, (int)N, (int)d, ld, nm);
    CI_HIP_CHECK_LAUNCH();
  } else if (down_layout == CI_DOWN_OUT_MAJOR) {
    dim3 grid((unsigned)((K + 63) / 64), (unsigned)((d + 63) / 64));
    if (e == 2)
      hipLaunchKernelGGL((delta_cols_t_kernel<uint16_t>), grid, dim3(256), 0, s,
                         reinterpret_cast<const uint16_t*>(w_down), reinterpret_cast<uint16_t*>(w_down_c),
                         free_list, enter_list, count, (int)N, (int)d);
    else
      hipLaunchKernelGGL((delta_cols_t_kernel<uint32_t>), grid, dim3(256), 0, s,
                         reinterpret_cast<const uint32_t*>(w_down), reinterpret_cast<uint32_t*>(w_down_c),
                         free_list, enter_list, count, (int)N, (int)d);
    CI_HIP_CHECK_LAUNCH();
  }
  hipLaunchKernelGGL(delta_rows_kernel, dim3((unsigned)K, g.n_mat), dim3(256), 0, s, g, free_list, enter_list,
                     count, slot_idx, (int)(d * e / 16));
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

int launch_compact(const void* w_up, const void* w_gate, const void* b_up, const void* w_down,
                   int down_layout, int dtype, int64_t d, int64_t N, const int32_t* core_idx,
                   int64_t K, void* w_up_c, void* w_gate_c, void* b_up_c, void* w_down_c,
                   int down_c_layout, int32_t* status, hipStream_t s) {
  if (K == 0) return CI_OK;
  const int e = elem_bytes(dtype);
  RowGather g;
  g.n_mat = 0;
  g.in[g.n_mat] = w_up; g.out[g.n_mat++] = w_up_c;
  if (w_gate) { g.in[g.n_mat] = w_gate; g.out[g.n_mat++] = w_gate_c; }
  if (down_layout == CI_DOWN_NEURON_MAJOR && down_c_layout == CI_DOWN_NEURON_MAJOR) {
    g.in[g.n_mat] = w_down; g.out[g.n_mat++] = w_down_c;
  }
  for (int i = g.n_mat; i < 3; ++i) { g.in[i] = nullptr; g.out[i] = nullptr; }
  g.b_in = b_up;
  g.b_out = b_up_c;
  g.elem = e;
  const int vecs = (int)(d * e / 16);
  if (down_c_layout == CI_DOWN_OUT_MAJOR) {
    // output-major compact down matrix [d, ld] first (the larger stream), then the rows of up / gate
    const int ld = (int)compact_down_ld(K, dtype);
    if (down_layout == CI_DOWN_OUT_MAJOR) {
      constexpr int ROWS = 16;
      dim3 grid((unsigned)((ld / (16 / e) + 255) / 256), (unsigned)((d + ROWS - 1) / ROWS));
      if (e == 2)
        hipLaunchKernelGGL((gather_cols_kernel<uint16_t, ROWS>), grid, dim3(256), 0, s,
                           reinterpret_cast<const uint16_t*>(w_down), reinterpret_cast<uint16_t*>(w_down_c),
                           core_idx, (int)K, ld, (int)N, (int)d, status);
      else
        hipLaunchKernelGGL((gather_cols_kernel<uint32_t, ROWS>), grid, dim3(256), 0, s,
                           reinterpret_cast<const uint32_t*>(w_down), reinterpret_cast<uint32_t*>(w_down_c),
                           core_idx, (int)K, ld, (int)N, (int)d, status);
    } else {
      dim3 grid((unsigned)((ld + 63) / 64), (unsigned)((d + 63) / 64));
      if (e == 2)
        hipLaunchKernelGGL((gather_rows_t_kernel<uint16_t>), grid, dim3(256), 0, s,
                           reinterpret_cast<const uint16_t*>(w_down), reinterpret_cast<uint16_t*>(w_down_c),
                           core_idx, (int)K, ld, (int)N, (int)d, status);
      else
        hipLaunchKernelGGL((gather_rows_t_kernel<uint32_t>), grid, dim3(256), 0, s,
                           reinterpret_cast<const uint32_t*>(w_down), reinterpret_cast<uint32_t*>(w_down_c),
                           core_idx, (int)K, ld, (int)N, (int)d, status);
    }
    CI_HIP_CHECK_LAUNCH();
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)K, g.n_mat), dim3(256), 0, s, g, core_idx,
                       (int)N, vecs, status);
    CI_HIP_CHECK_LAUNCH();
    return CI_OK;
  }
  if (down_layout == CI_DOWN_OUT_MAJOR) {
    const int kblocks = (int)((K + 63) / 64);
    const int64_t n_col = (int64_t)kblocks * ((d + 63) / 64);
    const int64_t total = n_col + K * g.n_mat;
    if (total < ((int64_t)1 << 31)) {
      if (e == 2)
        hipLaunchKernelGGL((compact_fused_kernel<uint16_t>), dim3((unsigned)total), dim3(256), 0, s, g,
                           reinterpret_cast<const uint16_t*>(w_down), reinterpret_cast<uint16_t*>(w_down_c),
                           core_idx, (int)K, (int)N, (int)d, vecs, kblocks, (int)n_col, status);
      else
        hipLaunchKernelGGL((compact_fused_kernel<uint32_t>), dim3((unsigned)total), dim3(256), 0, s, g,
                           reinterpret_cast<const uint32_t*>(w_down), reinterpret_cast<uint32_t*>(w_down_c),
                           core_idx, (int)K, (int)N, (int)d, vecs, kblocks, (int)n_col, status);
      CI_HIP_CHECK_LAUNCH();
      return CI_OK;
    }
  }
  hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)K, g.n_mat), dim3(256), 0, s, g, core_idx,
                     (int)N, vecs, status);
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
