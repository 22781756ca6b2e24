// Sentence-wise core neuron selection (Sec. 3.1 of arXiv 2410.18311).
//
// select_kernel, one launch per sentence and layer:
//   * Def. 1 / Eq. 1 and Eq. 3.  One workgroup per prompt token (looping when
//     M exceeds the grid).  The token's N activations become integer keys
//     (the IEEE bits of a positive float are monotone in its value;
//     everything that is not > 0 becomes key 0) held in registers.  The value
//     T of the k-th largest key (k = the share alpha of the positive keys) is
//     built bit by bit, most significant first: a candidate bit stays set if
//     at least k keys are >= the candidate.  Counting is a vector compare, a
//     scalar popcount of the lane mask and one LDS exchange per step -- no
//     atomics, no cross-lane shuffles.  Keys > T are token-wise core neurons;
//     of the keys == T the lowest indices fill the remaining places (ordered
//     ballot / popcount prefix; skipped when all of them are taken).  Each
//     chosen neuron's counter is incremented: in an LDS-private packed-u16
//     histogram when the workgroup sees several tokens (flushed once with
//     integer atomics), else directly in global memory.  Integer adds commute,
//     so the counts do not depend on scheduling.
//   * Def. 2 / Eq. 2.  The workgroup that finishes last (a ticket taken after a
//     device-scope fence) selects the K neurons first in the order (count
//     descending, index ascending): the threshold count by the same bitwise
//     search, then a ballot-based ordered compaction that writes S in ascending
//     index order: position = #greater before + min(#equal before, need).
// zero_i32_kernel clears the counters and the ticket beforehand.
#include "common.hpp"

namespace ci {

namespace {

constexpr int kMaxWaves = 16;

struct SelShared {
  uint32_t wcnt[2][kMaxWaves];  // per-wave tallies, double buffered: one barrier per exchange
  uint32_t ticket;
};

// Number of lanes of this wave for which `pred` holds (wave-uniform).
__device__ __forceinline__ uint32_t wave_count(bool pred) { return (uint32_t)__popcll(__ballot(pred)); }

// Block-wide sum of one value per wave (already wave-uniform).  `phase`
// alternates between calls, so successive calls need no second barrier.
__device__ __forceinline__ uint32_t block_sum_waves(uint32_t wave_value, SelShared* sh, int& phase) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  if (lane == 0) sh->wcnt[phase][wave] = wave_value;
  __syncthreads();
  uint32_t t = 0;
  for (int w = 0; w < nw; ++w) t += sh->wcnt[phase][w];
  phase ^= 1;
  return t;
}

// Runs f(i) for i in [0, n_iter).  With ITEMS > 0 the loop is unrolled to a
// compile-time bound so that per-thread key arrays stay in registers.
template <int ITEMS, class F>
__device__ __forceinline__ void for_items(int n_iter, F f) {
  if constexpr (ITEMS > 0) {
#pragma unroll
    for (int i = 0; i < ITEMS; ++i)
      if (i < n_iter) f(i);
  } else {
    for (int i = 0; i < n_iter; ++i) f(i);
  }
}

// Largest T in [0, 2^(top_bit+1)) such that at least k keys are >= T.  On
// return ge_T = number of keys >= T (unchanged if T stays 0: the caller
// presets it to the number of valid keys).  Every thread gets the same result.
template <int ITEMS, class KeyAt>
__device__ __forceinline__ uint32_t kth_largest(KeyAt key_at, int n_iter, uint32_t k, int top_bit,
                                                SelShared* sh, int& phase, uint32_t& ge_T) {
  uint32_t T = 0;
  for (int bit = top_bit; bit >= 0; --bit) {
    const uint32_t cand = T | (1u << bit);
    uint32_t c = 0;
    for_items<ITEMS>(n_iter, [&](int i) {
      bool valid;
      const uint32_t key = key_at(i, valid);
      c += wave_count(valid && key >= cand);
    });
    c = block_sum_waves(c, sh, phase);
    if (c >= k) {
      T = cand;
      ge_T = c;
    }
  }
  return T;
}

template <int ITEMS>
__global__ __launch_bounds__(1024) void select_kernel(const float* __restrict__ act, int M, int N,
                                                      int64_t ld, int64_t q_alpha, int K,
                                                      int32_t* counts, int32_t* core_idx,
                                                      uint32_t* ticket, int privatise) {
  __shared__ SelShared sh;
  extern __shared__ uint32_t lcount[];  // [ceil(N/2)] packed u16 pairs when privatised
  const int tid = threadIdx.x, nt = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
  const int n_iter = (N + nt - 1) / nt;
  const int npair = (N + 1) / 2;
  int phase = 0;

  if (privatise) {
    for (int j = tid; j < npair; j += nt) lcount[j] = 0;
    __syncthreads();
  }

  // ------------------------------------------------ Def. 1 / Eq. 1, Eq. 3 ----
  for (int m = blockIdx.x; m < M; m += gridDim.x) {
    const float* row = act + (size_t)m * ld;
    uint32_t kc[ITEMS > 0 ? ITEMS : 1];
    uint32_t npos = 0;
    if (ITEMS > 0) {
#pragma unroll
      for (int i = 0; i < ITEMS; ++i) {
        const int e = i * nt + tid;
        uint32_t key = 0;
        if (e < N) {
          const float a = row[e];
          key = (a > 0.f) ? f2u(a) : 0u;
        }
        kc[i] = key;
      }
#pragma unroll
      for (int i = 0; i < ITEMS; ++i) npos += wave_count(kc[i] != 0);
    } else {
      for (int i = 0; i < n_iter; ++i) {
        const int e = i * nt + tid;
        npos += wave_count(e < N && row[e] > 0.f);
      }
    }
    auto key_at = [&](int i, bool& valid) -> uint32_t {
      const int e = i * nt + tid;
      valid = e < N;
      if (ITEMS > 0) return kc[ITEMS > 0 ? i : 0];  // i is a constant after unrolling
      if (!valid) return 0u;
      const float a = row[e];
      return (a > 0.f) ? f2u(a) : 0u;
    };

    const uint32_t P = block_sum_waves(npos, &sh, phase);
    const uint32_t k = (uint32_t)((q_alpha * (int64_t)P + 999999) / 1000000);  // share of the positives
    if (k == 0) continue;  // uniform: no positive activation

    // positive keys are <= 0x7f800000 (+inf): bit 30 is the top one.  k <= P, so T >= 1.
    uint32_t ge_T = 0;
    const uint32_t T = kth_largest<ITEMS>(key_at, n_iter, k, 30, &sh, phase, ge_T);
    uint32_t gt = 0;
    for_items<ITEMS>(n_iter, [&](int i) {
      bool valid;
      const uint32_t key = key_at(i, valid);
      gt += wave_count(valid && key > T);
    });
    gt = block_sum_waves(gt, &sh, phase);
    const uint32_t need = k - gt;      // how many of the keys == T belong to the top k
    const uint32_t n_eq = ge_T - gt;   // how many keys == T exist

    auto bump = [&](int e) {
      if (privatise) atomicAdd(&lcount[e >> 1], 1u << (16 * (e & 1)));
      else atomicAdd(&counts[e], 1);
    };

    const bool all_ties = (need == n_eq);  // uniform
    uint32_t base = 0;                      // ties seen in earlier iterations
    for_items<ITEMS>(n_iter, [&](int i) {
      bool valid;
      const uint32_t key = key_at(i, valid);
      const int e = i * nt + tid;
      if (valid && key > T) bump(e);
      if (all_ties) {
        if (valid && key == T) bump(e);
      } else if (base < need) {  // uniform condition
        // index order = iteration, then wave, then lane
        const bool tie = valid && key == T;
        const uint64_t bal = __ballot(tie);
        if (lane == 0) sh.wcnt[phase][wave] = (uint32_t)__popcll(bal);
        __syncthreads();
        uint32_t before = base, tot = 0;
        for (int w = 0; w < nw; ++w) {
          const uint32_t c = sh.wcnt[phase][w];
          if (w < wave) before += c;
          tot += c;
        }
        phase ^= 1;
        const uint32_t rank = before + (uint32_t)__popcll(bal & lanemask_lt());
        if (tie && rank < need) bump(e);
        base += tot;
      }
    });
  }

  if (privatise) {
    __syncthreads();
    for (int j = tid; j < npair; j += nt) {
      const uint32_t v = lcount[j];
      if (v & 0xffffu) atomicAdd(&counts[2 * j], (int)(v & 0xffffu));
      if (v >> 16) atomicAdd(&counts[2 * j + 1], (int)(v >> 16));
    }
  }

  // ------------------------------------------------ Def. 2 / Eq. 2 -----------
  // The last workgroup to arrive sees every counter update: each workgroup's
  // atomics are complete (device-scope fence) before it takes its ticket.
  __threadfence();
  __syncthreads();
  if (tid == 0) sh.ticket = atomicAdd(ticket, 1u);
  __syncthreads();
  if (sh.ticket != gridDim.x - 1) return;
  __threadfence();

  auto count_at = [&](int i, bool& valid) -> uint32_t {
    const int e = i * nt + tid;
    valid = e < N;
    if (!valid) return 0u;
    return (uint32_t)__hip_atomic_load(&counts[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  };
  uint32_t cc[ITEMS > 0 ? ITEMS : 1];
  if (ITEMS > 0) {
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      bool valid;
      cc[i] = count_at(i, valid);
    }
  }
  auto ckey_at = [&](int i, bool& valid) -> uint32_t {
    if (ITEMS > 0) {
      valid = i * nt + tid < N;
      return cc[ITEMS > 0 ? i : 0];
    }
    return count_at(i, valid);
  };

  // counts lie in [0, M]: search only the bits M can have
  const int top_bit = 31 - __clz((uint32_t)(M | 1));
  uint32_t ge_T = (uint32_t)N;  // T = 0 holds for every neuron
  const uint32_t T = kth_largest<ITEMS>(ckey_at, n_iter, (uint32_t)K, top_bit, &sh, phase, ge_T);
  uint32_t gt = 0;
  for_items<ITEMS>(n_iter, [&](int i) {
    bool valid;
    const uint32_t key = ckey_at(i, valid);
    gt += wave_count(valid && key > T);
  });
  gt = block_sum_waves(gt, &sh, phase);
  const uint32_t need = (uint32_t)K - gt;

  // ordered compaction: running totals of (#greater, #equal) over earlier iterations
  uint32_t g_base = 0, e_base = 0;
  for_items<ITEMS>(n_iter, [&](int i) {
    bool valid;
    const uint32_t key = ckey_at(i, valid);
    const bool isg = valid && key > T, ise = valid && key == T;
    const uint64_t bg = __ballot(isg), be = __ballot(ise);
    if (lane == 0) sh.wcnt[phase][wave] = ((uint32_t)__popcll(bg) << 16) | (uint32_t)__popcll(be);  // <= 64 each
    __syncthreads();
    uint32_t g_before = g_base, e_before = e_base, g_tot = 0, e_tot = 0;
    for (int w = 0; w < nw; ++w) {
      const uint32_t c = sh.wcnt[phase][w];
      if (w < wave) { g_before += c >> 16; e_before += c & 0xffffu; }
      g_tot += c >> 16;
      e_tot += c & 0xffffu;
    }
    phase ^= 1;
    g_before += (uint32_t)__popcll(bg & lanemask_lt());
    e_before += (uint32_t)__popcll(be & lanemask_lt());
    // position in the ascending output = selected neurons with a lower index
    const uint32_t pos = g_before + (e_before < need ? e_before : need);
    if (isg || (ise && e_before < need)) core_idx[pos] = i * nt + tid;
    g_base += g_tot;
    e_base += e_tot;
  });
}

__global__ void zero_i32_kernel(int32_t* p, int n, uint32_t* ticket) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
  if (i == 0) *ticket = 0;
}

template <int ITEMS>
int launch_sel(const float* act, int M, int N, int64_t ld, int64_t q_alpha, int K, int32_t* counts,
               int32_t* core_idx, uint32_t* ticket, int grid, int nt, int privatise, size_t lds,
               hipStream_t s) {
  if (lds > 48 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&select_kernel<ITEMS>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return CI_ERR_HIP;
  }
  hipLaunchKernelGGL((select_kernel<ITEMS>), dim3(grid), dim3(nt), lds, s, act, M, N, ld, q_alpha, K,
                     counts, core_idx, ticket, privatise);
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

}  // namespace

int launch_select(const float* act, int64_t M64, int64_t N64, int64_t ld, int64_t q_alpha,
                  int64_t K64, int32_t* core_idx, int32_t* counts, uint32_t* ticket, hipStream_t s) {
  const int M = (int)M64, N = (int)N64, K = (int)K64;
  DeviceInfo di;
  int rc = device_info(&di);
  if (rc != CI_OK) return rc;

  hipLaunchKernelGGL(zero_i32_kernel, dim3((N + 255) / 256), dim3(256), 0, s, counts, N, ticket);
  CI_HIP_CHECK_LAUNCH();

  const int nt = N >= 4096 ? 1024 : 256;
  const int items = (N + nt - 1) / nt;
  int grid = di.cus * params().select_wgs_per_cu;
  if (grid > M) grid = M;
  const int tokens_per_wg = (M + grid - 1) / grid;
  // private u16 counters pay off only when a workgroup sees several tokens
  // and they fit LDS
  const size_t priv_bytes = (size_t)((N + 1) / 2) * 4;
  const int privatise = (tokens_per_wg >= 2 && priv_bytes <= 128 * 1024) ? 1 : 0;
  const size_t lds = privatise ? priv_bytes : 0;

#define CI_SEL(I) launch_sel<I>(act, M, N, ld, q_alpha, K, counts, core_idx, ticket, grid, nt, privatise, lds, s)
  if (items <= 4) return CI_SEL(4);
  if (items <= 8) return CI_SEL(8);
  if (items <= 16) return CI_SEL(16);
  return CI_SEL(0);
#undef CI_SEL
}

}  // namespace ci
