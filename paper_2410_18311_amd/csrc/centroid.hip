// Group choice for similarity-guided prediction when the groups are K-Means
// clusters of a layer's activation (App. A.2.3 of arXiv 2410.18311): the
// prompt's feature vector (mean over its tokens of the activation rows) and
// the K-Means assignment step, the nearest centroid in Euclidean distance.
//
//   token_mean_kernel    : feature[n] = (sum_m act[m, n]) / M.  A workgroup owns
//                          64 neurons; a wave instruction covers four tokens;
//                          every lane sums its tokens in order, the 64 partial
//                          sums per neuron are added in a fixed order -- the
//                          result does not depend on scheduling.
//   centroid_dist_kernel : dist[g] = sum_n (feature[n] - centroids[g, n])^2,
//                          one workgroup per centroid, fixed summation order.
//   nearest_kernel       : best = argmin_g dist[g], ties to the lower g.
// All sums are fp32.
#include "common.hpp"

namespace ci {

namespace {

constexpr int kMeanNeurons = 64;  // neurons per workgroup of the mean kernel

template <bool VEC>
__device__ __forceinline__ void sum_tokens_of_lane(const float* __restrict__ act, int64_t ld, int M, int N,
                                                   int n0, int ts, int wave, int nw, float (&acc)[4]) {
  constexpr int UN = 8, TPW = 4;
  for (int m0 = wave * UN * TPW; m0 < M; m0 += nw * UN * TPW) {
    float v[UN][4];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int m = min(m0 + u * TPW + ts, M - 1);  // clamped: a repeated token is masked below
      const float* p = act + (size_t)m * ld;
      if (VEC) {
        const float4 q = *reinterpret_cast<const float4*>(p + n0);
        v[u][0] = q.x; v[u][1] = q.y; v[u][2] = q.z; v[u][3] = q.w;
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) v[u][c] = p[min(n0 + c, N - 1)];
      }
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      if (m0 + u * TPW + ts < M) {
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] += v[u][c];
      }
    }
  }
}

__global__ __launch_bounds__(1024) void token_mean_kernel(const float* __restrict__ act, int M, int N, int64_t ld,
                                                          int vec_ok, float* __restrict__ feature) {
  __shared__ float part[64][kMeanNeurons + 1];  // [wave * 4 + token slot][neuron]
  const int tid = threadIdx.x, nt = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
  const int quad = lane & 15, ts = lane >> 4;
  const int n0 = blockIdx.x * kMeanNeurons + quad * 4;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  if (vec_ok && n0 + 3 < N) sum_tokens_of_lane<true>(act, ld, M, N, n0, ts, wave, nw, acc);
  else sum_tokens_of_lane<false>(act, ld, M, N, n0, ts, wave, nw, acc);
#pragma unroll
  for (int c = 0; c < 4; ++c) part[wave * 4 + ts][quad * 4 + c] = acc[c];
  __syncthreads();
  if (tid < kMeanNeurons) {
    const int n = blockIdx.x * kMeanNeurons + tid;
    float sum = 0.f;
    for (int r = 0; r < nw * 4; ++r) sum += part[r][tid];
    if (n < N) feature[n] = sum / (float)M;
  }
}

// Block-wide sum in a fixed order: lanes by a shuffle tree, then the waves in index order.
__device__ __forceinline__ float block_sum_ordered(float v, float* wave_part) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_down(v, off, kWave);
  if (lane == 0) wave_part[wave] = v;
  __syncthreads();
  float t = 0.f;
  for (int w = 0; w < nw; ++w) t += wave_part[w];
  return t;
}

__global__ __launch_bounds__(256) void centroid_dist_kernel(const float* __restrict__ feature,
                                                            const float* __restrict__ centroids, int N,
                                                            float* __restrict__ dist) {
  __shared__ float wave_part[4];
  const float* c = centroids + (size_t)blockIdx.x * N;
  float acc = 0.f;
  for (int n = threadIdx.x; n < N; n += blockDim.x) {
    const float d = feature[n] - c[n];
    acc += d * d;
  }
  const float t = block_sum_ordered(acc, wave_part);
  if (threadIdx.x == 0) dist[blockIdx.x] = t;
}

// A NaN distance is never the minimum; if every distance is NaN the answer is group 0.
__global__ __launch_bounds__(1024) void nearest_kernel(const float* __restrict__ dist, int G,
                                                       int32_t* __restrict__ best) {
  __shared__ float sd[1024];
  __shared__ int sg[1024];
  float bd = __builtin_inff();
  int bg = 0x7fffffff;
  for (int g = threadIdx.x; g < G; g += blockDim.x) {
    const float d = dist[g];
    if (d < bd || (d == bd && g < bg)) { bd = d; bg = g; }  // ascending g per thread: keeps the lowest index
  }
  sd[threadIdx.x] = bd; sg[threadIdx.x] = bg;
  __syncthreads();
  for (int half = 512; half >= 1; half >>= 1) {
    if ((int)threadIdx.x < half) {
      const float d2 = sd[threadIdx.x + half];
      const int g2 = sg[threadIdx.x + half];
      if (d2 < sd[threadIdx.x] || (d2 == sd[threadIdx.x] && g2 < sg[threadIdx.x])) {
        sd[threadIdx.x] = d2; sg[threadIdx.x] = g2;
      }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) best[0] = sg[0] == 0x7fffffff ? 0 : sg[0];
}

}  // namespace

int launch_assign_centroid(const float* act, int64_t M, int64_t N, int64_t ld, const float* centroids,
                           int64_t G, int32_t* best, float* dist, float* feature, hipStream_t s) {
  const int vec_ok = ((reinterpret_cast<uintptr_t>(act) & 15u) == 0 && ld % 4 == 0) ? 1 : 0;
  const unsigned blocks = (unsigned)((N + kMeanNeurons - 1) / kMeanNeurons);
  hipLaunchKernelGGL(token_mean_kernel, dim3(blocks), dim3(1024), 0, s, act, (int)M, (int)N, ld, vec_ok, feature);
  hipLaunchKernelGGL(centroid_dist_kernel, dim3((unsigned)G), dim3(256), 0, s, feature, centroids, (int)N, dist);
  hipLaunchKernelGGL(nearest_kernel, dim3(1), dim3(1024), 0, s, dist, (int)G, best);
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

}  // namespace ci
