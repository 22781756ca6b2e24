// Sentence-wise core neuron selection (Sec. 3.1 of arXiv 2410.18311).
//
//   token_select_kernel : Def. 1 / Eq. 1 and Eq. 3.  One workgroup per prompt
//     token (looping when M exceeds the grid).  The token's N activations are
//     turned into integer keys (the IEEE bits of a positive float are monotone
//     in its value; everything that is not > 0 becomes key 0) and kept in
//     registers.  A three-pass most-significant-digit radix select over LDS
//     histograms finds the value T of the k-th largest key, k being the share
//     alpha of the positive keys.  Every key > T is a token-wise core neuron;
//     of the keys == T the lowest indices fill the remaining places (ordered
//     ballot / popcount prefix; skipped when all of them are taken).  Each
//     chosen neuron's counter is incremented -- in an LDS-private u16
//     histogram when the workgroup handles several tokens, flushed once with
//     integer atomics, else directly in global memory.  Integer adds commute,
//     so the counts do not depend on scheduling.
//   count_topk_kernel   : Def. 2 / Eq. 2.  One workgroup.  Two-pass radix
//     select over the counts (<= 65535) finds the threshold count; neurons
//     above it plus the lowest-indexed neurons equal to it are written in
//     ascending index order through a ballot-based ordered compaction.
#include "common.hpp"

namespace ci {

namespace {

constexpr int kBins = 2048;
constexpr int kMaxWaves = 16;

struct SelShared {
  uint32_t wave_tot[kMaxWaves];
  uint32_t bin;      // chosen digit
  uint32_t above;    // keys in higher digits
  uint32_t in_bin;   // keys in the chosen digit
  uint32_t total;
};

// Block-wide sum of a per-thread value (every thread gets the result).
__device__ __forceinline__ uint32_t block_sum(uint32_t v, SelShared* sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  v = (uint32_t)wave_sum((int)v);
  __syncthreads();
  if (lane == 0) sh->wave_tot[wave] = v;
  __syncthreads();
  uint32_t t = 0;
  for (int w = 0; w < nw; ++w) t += sh->wave_tot[w];
  return t;
}

// hist[0..nbins) holds digit counts.  Finds the digit that contains the
// k-th largest key (k >= 1, k <= sum of hist) and how many keys lie in higher
// digits.  Result in sh->bin / above / in_bin, visible to all threads on
// return.  nbins must be a multiple of blockDim.x or smaller than it.
__device__ __forceinline__ void find_digit(const uint32_t* hist, int nbins, uint32_t k,
                                           SelShared* sh) {
  const int tid = threadIdx.x, nt = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
  const int per = (nbins + nt - 1) / nt;  // digits per thread, contiguous
  const int b0 = tid * per;
  uint32_t mine = 0;
  for (int j = 0; j < per; ++j) {
    const int bidx = b0 + j;
    if (bidx < nbins) mine += hist[bidx];
  }
  // inclusive suffix sum over threads (higher thread = higher digits)
  uint32_t suf = mine;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t o = __shfl_down(suf, off, kWave);
    if (lane + off < 64) suf += o;
  }
  if (lane == 0) sh->wave_tot[wave] = suf;  // total of this wave
  __syncthreads();
  uint32_t higher = 0;
  for (int w = wave + 1; w < nw; ++w) higher += sh->wave_tot[w];
  const uint32_t incl = suf + higher;  // keys in my digits and above
  const uint32_t excl = incl - mine;   // keys strictly above my digits
  if (excl < k && k <= incl) {
    uint32_t run = excl;
    for (int j = per - 1; j >= 0; --j) {
      const int bidx = b0 + j;
      if (bidx >= nbins) continue;
      const uint32_t c = hist[bidx];
      if (run + c >= k) {
        sh->bin = (uint32_t)bidx;
        sh->above = run;
        sh->in_bin = c;
        break;
      }
      run += c;
    }
  }
  __syncthreads();
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

template <int NPASS>
struct Digits;
template <>
struct Digits<3> {  // 31-bit keys (positive floats)
  static __device__ __forceinline__ int shift(int p) { return p == 0 ? 20 : (p == 1 ? 9 : 0); }
  static __device__ __forceinline__ int bits(int p) { return p == 2 ? 9 : 11; }
};
template <>
struct Digits<2> {  // 16-bit keys (counts)
  static __device__ __forceinline__ int shift(int p) { return p == 0 ? 8 : 0; }
  static __device__ __forceinline__ int bits(int) { return 8; }
};

// Most-significant-digit radix select.  On return T is the k-th largest key
// (over keys for which `live` holds), need = how many keys == T belong to the
// top k, n_eq = how many keys == T exist.  KeyAt(i, valid) yields the key of
// this thread's i-th element.
template <int NPASS, bool SKIP_ZERO, int ITEMS, class KeyAt>
__device__ __forceinline__ void radix_select(KeyAt key_at, int n_iter, uint32_t k, uint32_t* hist,
                                             SelShared* sh, uint32_t& T, uint32_t& need,
                                             uint32_t& n_eq) {
  const int tid = threadIdx.x, nt = blockDim.x;
  uint32_t prefix = 0, prefix_mask = 0;
#pragma unroll
  for (int p = 0; p < NPASS; ++p) {
    const int shift = Digits<NPASS>::shift(p), nb = 1 << Digits<NPASS>::bits(p);
    for (int j = tid; j < nb; j += nt) hist[j] = 0;
    __syncthreads();
    for_items<ITEMS>(n_iter, [&](int i) {
      bool valid;
      const uint32_t key = key_at(i, valid);
      if (valid && (!SKIP_ZERO || key != 0) && (key & prefix_mask) == prefix)
        atomicAdd(&hist[(key >> shift) & (nb - 1)], 1u);
    });
    __syncthreads();
    find_digit(hist, nb, k, sh);
    prefix |= sh->bin << shift;
    prefix_mask |= (uint32_t)(nb - 1) << shift;
    k -= sh->above;
    n_eq = sh->in_bin;
    __syncthreads();  // sh is reused by the next pass
  }
  T = prefix;
  need = k;
}

// ---------------------------------------------------------------------------
template <int ITEMS>
__global__ __launch_bounds__(1024) void token_select_kernel(const float* __restrict__ act, int M,
                                                            int N, int64_t ld, int64_t q_alpha,
                                                            int32_t* __restrict__ counts,
                                                            int privatise) {
  __shared__ uint32_t hist[kBins];
  __shared__ SelShared sh;
  extern __shared__ uint32_t lcount[];  // [ceil(N/2)] packed u16 pairs when privatised
  const int tid = threadIdx.x, nt = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
  const int n_iter = (N + nt - 1) / nt;
  const int npair = (N + 1) / 2;

  if (privatise) {
    for (int j = tid; j < npair; j += nt) lcount[j] = 0;
    __syncthreads();
  }

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
        npos += key != 0;
      }
    } else {
      for (int e = tid; e < N; e += nt) npos += row[e] > 0.f;
    }
    auto key_at = [&](int i, bool& valid) -> uint32_t {
      const int e = i * nt + tid;
      valid = e < N;
      if (ITEMS > 0) return kc[ITEMS > 0 ? i : 0];  // i is a constant after unrolling
      if (!valid) return 0u;
      const float a = row[e];
      return (a > 0.f) ? f2u(a) : 0u;
    };

    const uint32_t P = block_sum(npos, &sh);
    const uint32_t k = (uint32_t)((q_alpha * (int64_t)P + 999999) / 1000000);  // Def. 1: share of the positives
    if (k == 0) continue;  // uniform: no positive activation

    uint32_t T, need, n_eq;
    radix_select<3, true, ITEMS>(key_at, n_iter, k, hist, &sh, T, need, n_eq);

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
        __syncthreads();
        if (lane == 0) sh.wave_tot[wave] = (uint32_t)__popcll(bal);
        __syncthreads();
        uint32_t before = base, tot = 0;
        for (int w = 0; w < nw; ++w) {
          const uint32_t c = sh.wave_tot[w];
          if (w < wave) before += c;
          tot += c;
        }
        const uint32_t rank = before + (uint32_t)__popcll(bal & lanemask_lt());
        if (tie && rank < need) bump(e);
        base += tot;
      }
    });
    __syncthreads();
  }

  if (privatise) {
    __syncthreads();
    for (int j = tid; j < npair; j += nt) {
      const uint32_t v = lcount[j];
      if (v & 0xffffu) atomicAdd(&counts[2 * j], (int)(v & 0xffffu));
      if (v >> 16) atomicAdd(&counts[2 * j + 1], (int)(v >> 16));
    }
  }
}

// ---------------------------------------------------------------------------
template <int ITEMS>
__global__ __launch_bounds__(1024) void count_topk_kernel(const int32_t* __restrict__ counts, int N,
                                                          int K, int32_t* __restrict__ core_idx) {
  __shared__ uint32_t hist[256];
  __shared__ SelShared sh;
  extern __shared__ uint32_t tab[];  // [n_iter][nw][2]: (#greater, #equal) per wave-row
  const int tid = threadIdx.x, nt = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
  const int n_iter = (N + nt - 1) / nt;

  uint32_t kc[ITEMS > 0 ? ITEMS : 1];
  if (ITEMS > 0) {
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      const int e = i * nt + tid;
      kc[i] = (e < N) ? (uint32_t)counts[e] : 0u;
    }
  }
  auto key_at = [&](int i, bool& valid) -> uint32_t {
    const int e = i * nt + tid;
    valid = e < N;
    if (ITEMS > 0) return kc[ITEMS > 0 ? i : 0];
    return valid ? (uint32_t)counts[e] : 0u;
  };

  uint32_t T, need, n_eq;
  radix_select<2, false, ITEMS>(key_at, n_iter, (uint32_t)K, hist, &sh, T, need, n_eq);

  // per (iteration, wave) tallies, then an exclusive scan over them in index order
  for_items<ITEMS>(n_iter, [&](int i) {
    bool valid;
    const uint32_t key = key_at(i, valid);
    const uint64_t bg = __ballot(valid && key > T);
    const uint64_t be = __ballot(valid && key == T);
    if (lane == 0) {
      tab[(i * nw + wave) * 2 + 0] = (uint32_t)__popcll(bg);
      tab[(i * nw + wave) * 2 + 1] = (uint32_t)__popcll(be);
    }
  });
  __syncthreads();
  if (wave == 0) {
    // wave 0 scans the n_iter*nw entries: each lane takes a contiguous run
    const int n_ent = n_iter * nw;
    const int per = (n_ent + 63) / 64;
    const int e0 = lane * per;
    uint32_t sg = 0, se = 0;
    for (int j = 0; j < per; ++j) {
      if (e0 + j < n_ent) { sg += tab[(e0 + j) * 2]; se += tab[(e0 + j) * 2 + 1]; }
    }
    uint32_t pg = sg, pe = se;  // inclusive prefix over lanes
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t og = __shfl_up(pg, off, kWave), oe = __shfl_up(pe, off, kWave);
      if (lane >= off) { pg += og; pe += oe; }
    }
    uint32_t rg = pg - sg, re = pe - se;  // exclusive
    for (int j = 0; j < per; ++j) {
      if (e0 + j < n_ent) {
        const uint32_t cg = tab[(e0 + j) * 2], ce = tab[(e0 + j) * 2 + 1];
        tab[(e0 + j) * 2] = rg;
        tab[(e0 + j) * 2 + 1] = re;
        rg += cg;
        re += ce;
      }
    }
  }
  __syncthreads();
  for_items<ITEMS>(n_iter, [&](int i) {
    bool valid;
    const uint32_t key = key_at(i, valid);
    const bool gt = valid && key > T, eq = valid && key == T;
    const uint64_t bg = __ballot(gt), be = __ballot(eq);
    const uint32_t g_before = tab[(i * nw + wave) * 2] + (uint32_t)__popcll(bg & lanemask_lt());
    const uint32_t e_before = tab[(i * nw + wave) * 2 + 1] + (uint32_t)__popcll(be & lanemask_lt());
    // position in the ascending output = selected neurons with a lower index
    const uint32_t pos = g_before + (e_before < need ? e_before : need);
    if (gt || (eq && e_before < need)) core_idx[pos] = i * nt + tid;
  });
}

__global__ void zero_i32_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

template <int ITEMS>
int launch_token(const float* act, int M, int N, int64_t ld, int64_t q_alpha, int32_t* counts,
                 int grid, int nt, int privatise, size_t lds, hipStream_t s) {
  if (lds > 48 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&token_select_kernel<ITEMS>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return CI_ERR_HIP;
  }
  hipLaunchKernelGGL((token_select_kernel<ITEMS>), dim3(grid), dim3(nt), lds, s, act, M, N, ld,
                     q_alpha, counts, privatise);
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

template <int ITEMS>
int launch_topk(const int32_t* counts, int N, int K, int32_t* core_idx, int nt, size_t lds,
                hipStream_t s) {
  if (lds > 48 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&count_topk_kernel<ITEMS>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return CI_ERR_HIP;
  }
  hipLaunchKernelGGL((count_topk_kernel<ITEMS>), dim3(1), dim3(nt), lds, s, counts, N, K, core_idx);
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

}  // namespace

int launch_select(const float* act, int64_t M64, int64_t N64, int64_t ld, int64_t q_alpha,
                  int64_t K64, int32_t* core_idx, int32_t* counts, hipStream_t s) {
  const int M = (int)M64, N = (int)N64, K = (int)K64;
  DeviceInfo di;
  int rc = device_info(&di);
  if (rc != CI_OK) return rc;

  hipLaunchKernelGGL(zero_i32_kernel, dim3((N + 255) / 256), dim3(256), 0, s, counts, N);
  CI_HIP_CHECK_LAUNCH();

  const int nt = N >= 4096 ? 1024 : 256;
  const int items = (N + nt - 1) / nt;
  int grid = di.cus * params().select_wgs_per_cu;
  if (grid > M) grid = M;
  const int tokens_per_wg = (M + grid - 1) / grid;
  // private u16 counters pay off only when a workgroup sees several tokens
  // and they fit LDS next to the digit histogram
  const size_t priv_bytes = (size_t)((N + 1) / 2) * 4;
  const int privatise = (tokens_per_wg >= 2 && priv_bytes <= 128 * 1024) ? 1 : 0;
  const size_t lds = privatise ? priv_bytes : 0;

  if (items <= 4) rc = launch_token<4>(act, M, N, ld, q_alpha, counts, grid, nt, privatise, lds, s);
  else if (items <= 8) rc = launch_token<8>(act, M, N, ld, q_alpha, counts, grid, nt, privatise, lds, s);
  else if (items <= 16) rc = launch_token<16>(act, M, N, ld, q_alpha, counts, grid, nt, privatise, lds, s);
  else rc = launch_token<0>(act, M, N, ld, q_alpha, counts, grid, nt, privatise, lds, s);
  if (rc != CI_OK) return rc;

  const size_t tab_bytes = (size_t)items * (nt / 64) * 2 * sizeof(uint32_t);
  if (items <= 4) return launch_topk<4>(counts, N, K, core_idx, nt, tab_bytes, s);
  if (items <= 8) return launch_topk<8>(counts, N, K, core_idx, nt, tab_bytes, s);
  if (items <= 16) return launch_topk<16>(counts, N, K, core_idx, nt, tab_bytes, s);
  if (items <= 40) return launch_topk<40>(counts, N, K, core_idx, nt, tab_bytes, s);
  return launch_topk<0>(counts, N, K, core_idx, nt, tab_bytes, s);
}

}  // namespace ci
