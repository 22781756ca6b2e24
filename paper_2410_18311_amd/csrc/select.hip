// Sentence-wise core neuron selection (Sec. 3.1 of arXiv 2410.18311).
//
// select_kernel, one launch per sentence and layer:
//   * Def. 1 / Eq. 1 and Eq. 3.  One workgroup per prompt token (looping when
//     M exceeds the grid).  The token's N activations become integer keys
//     (the IEEE bits of a positive float are monotone in its value;
//     everything that is not > 0 becomes key 0), loaded once and kept in
//     registers.  A three-pass most-significant-digit radix select (11 + 11 +
//     9 bits) over LDS histograms finds the value T of the k-th largest key,
//     k being the share alpha of the positive keys.  The histograms are
//     replicated eight times by lane so that activations sharing an exponent
//     do not serialise on one LDS address.  Keys > T are token-wise core
//     neurons; of the keys == T the lowest indices fill the remaining places
//     (ordered ballot / popcount prefix; skipped when all of them are taken).
//     Each chosen neuron's counter is incremented: in an LDS-private
//     packed-u16 histogram when the workgroup sees several tokens (flushed
//     once with integer atomics), else directly in global memory.  Integer
//     adds commute, so the counts do not depend on scheduling.
//   * Def. 2 / Eq. 2.  The workgroup that finishes last (a ticket taken after a
//     device-scope fence) selects the K neurons first in the order (count
//     descending, index ascending): threshold count by a two-pass radix select
//     over the counts (<= 65535), then a ballot-based ordered compaction that
//     writes S ascending: position = #greater before + min(#equal before, need).
// zero_i32_kernel clears the counters and the ticket beforehand.
#include "common.hpp"

namespace ci {

namespace {

constexpr int kBins = 2048;              // largest digit: 11 bits
constexpr int kCopies = 8;               // histogram replicas, chosen by lane & 7
constexpr int kCopyStride = kBins + 8;   // words; the +8 spreads the replicas over LDS banks
constexpr int kHistWords = kCopies * kCopyStride;
constexpr int kMaxWaves = 16;

struct SelShared {
  uint32_t wave_tot[kMaxWaves];
  uint32_t bin;      // chosen digit
  uint32_t above;    // keys in higher digits
  uint32_t in_bin;   // keys in the chosen digit
  uint32_t ticket;
};

__device__ __forceinline__ uint32_t wave_count(bool pred) { return (uint32_t)__popcll(__ballot(pred)); }

// Block-wide sum of one wave-uniform value per wave (every thread gets it).
__device__ __forceinline__ uint32_t block_sum_waves(uint32_t wave_value, SelShared* sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if (lane == 0) sh->wave_tot[wave] = wave_value;
  __syncthreads();
  uint32_t t = 0;
  for (int w = 0; w < nw; ++w) t += sh->wave_tot[w];
  return t;
}

// hist holds kCopies replicas of nbins digit counts.  Finds the digit that
// contains the k-th largest key (1 <= k <= total) and how many keys lie in
// higher digits.  Result in sh->bin / above / in_bin, visible to all threads on
// return.
__device__ __forceinline__ void find_digit(const uint32_t* hist, int nbins, uint32_t k, SelShared* sh) {
  const int tid = threadIdx.x, nt = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
  const int per = (nbins + nt - 1) / nt;  // digits per thread, contiguous; higher thread = higher digits
  const int b0 = tid * per;
  auto bin_total = [&](int bidx) {
    uint32_t c = 0;
#pragma unroll
    for (int r = 0; r < kCopies; ++r) c += hist[r * kCopyStride + bidx];
    return c;
  };
  uint32_t mine = 0;
  for (int j = 0; j < per; ++j)
    if (b0 + j < nbins) mine += bin_total(b0 + j);
  uint32_t suf = mine;  // inclusive suffix sum over the wave
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t o = __shfl_down(suf, off, kWave);
    if (lane + off < 64) suf += o;
  }
  if (lane == 0) sh->wave_tot[wave] = suf;
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
      const uint32_t c = bin_total(bidx);
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

// One radix pass: histogram of the digit (key >> shift) & (nb - 1) over the
// keys that match `prefix` under `prefix_mask`, then the digit holding the
// k-th largest of them.  Updates prefix / prefix_mask / k; n_eq = keys in it.
template <int ITEMS, class KeyAt>
__device__ __forceinline__ void radix_pass(KeyAt key_at, int n_iter, int shift, int nb, uint32_t* hist,
                                           SelShared* sh, uint32_t& prefix, uint32_t& prefix_mask,
                                           uint32_t& k, uint32_t& n_eq) {
  const int tid = threadIdx.x, nt = blockDim.x;
  uint32_t* my_hist = hist + (tid & (kCopies - 1)) * kCopyStride;
  // clear the replicas (the padding words are never read)
  for (int j = tid; j < kCopies * nb; j += nt) hist[(j / nb) * kCopyStride + (j % nb)] = 0;
  __syncthreads();
  for_items<ITEMS>(n_iter, [&](int i) {
    const uint32_t key = key_at(i);
    if ((key & prefix_mask) == prefix) atomicAdd(&my_hist[(key >> shift) & (nb - 1)], 1u);
  });
  __syncthreads();
  find_digit(hist, nb, k, sh);
  prefix |= sh->bin << shift;
  prefix_mask |= (uint32_t)(nb - 1) << shift;
  k -= sh->above;
  n_eq = sh->in_bin;
  __syncthreads();  // sh is reused by the next pass
}

template <int ITEMS>
__global__ __launch_bounds__(1024) void select_kernel(const float* __restrict__ act, int M, int N,
                                                      int64_t ld, int64_t q_alpha, int K,
                                                      int32_t* counts, int32_t* core_idx,
                                                      uint32_t* ticket, int privatise, int max_count,
                                                      int debug) {
  __shared__ SelShared sh;
  extern __shared__ uint32_t dyn[];  // [kHistWords] histograms, then [ceil(N/2)] packed u16 counters
  uint32_t* hist = dyn;
  uint32_t* lcount = dyn + kHistWords;
  const int tid = threadIdx.x, nt = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
  const int n_iter = (N + nt - 1) / nt;
  const int npair = (N + 1) / 2;

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
      float av[ITEMS > 0 ? ITEMS : 1];
#pragma unroll
      for (int i = 0; i < ITEMS; ++i) {  // branch-free: all loads are issued back to back
        const int e = i * nt + tid;
        av[i] = row[e < N ? e : N - 1];
      }
#pragma unroll
      for (int i = 0; i < ITEMS; ++i) {
        const int e = i * nt + tid;
        kc[i] = (e < N && av[i] > 0.f) ? f2u(av[i]) : 0u;
      }
#pragma unroll
      for (int i = 0; i < ITEMS; ++i) npos += wave_count(kc[i] != 0);
    } else {
      for (int i = 0; i < n_iter; ++i) {
        const int e = i * nt + tid;
        npos += wave_count(e < N && row[e] > 0.f);
      }
    }
    // key of this thread's i-th element; 0 (never a candidate) past the end
    auto key_at = [&](int i) -> uint32_t {
      if (ITEMS > 0) return kc[ITEMS > 0 ? i : 0];  // i is a constant after unrolling
      const int e = i * nt + tid;
      if (e >= N) return 0u;
      const float a = row[e];
      return (a > 0.f) ? f2u(a) : 0u;
    };
    // for the histogram passes a zero key must match no prefix: map it to all-ones
    // (bit 31 set, which no prefix mask ever covers with a zero prefix... see radix_pass use)
    auto key_sel = [&](int i) -> uint32_t {
      const uint32_t key = key_at(i);
      return key != 0 ? key : 0xffffffffu;
    };

    const uint32_t P = block_sum_waves(npos, &sh);
    const uint32_t k = (uint32_t)((q_alpha * (int64_t)P + 999999) / 1000000);  // share of the positives
    if (k == 0) continue;  // uniform: no positive activation

    // 31-bit keys: digits of 11, 11 and 9 bits.  Bit 31 is part of the mask from the start,
    // so the all-ones stand-in of a zero key never matches.
    uint32_t prefix = 0, prefix_mask = 0x80000000u, need = k, n_eq = 0;
    radix_pass<ITEMS>(key_sel, n_iter, 20, 2048, hist, &sh, prefix, prefix_mask, need, n_eq);
    radix_pass<ITEMS>(key_sel, n_iter, 9, 2048, hist, &sh, prefix, prefix_mask, need, n_eq);
    radix_pass<ITEMS>(key_sel, n_iter, 0, 512, hist, &sh, prefix, prefix_mask, need, n_eq);
    const uint32_t T = prefix;  // the k-th largest key; `need` of the n_eq keys == T are in the top k

    auto bump = [&](int e) {
      if (privatise) atomicAdd(&lcount[e >> 1], 1u << (16 * (e & 1)));
      else atomicAdd(&counts[e], 1);
    };

    const bool all_ties = (need == n_eq);  // uniform
    uint32_t base = 0;                      // ties seen in earlier iterations
    for_items<ITEMS>(n_iter, [&](int i) {
      const uint32_t key = key_at(i);  // T >= 1, so elements past the end (key 0) never match
      const int e = i * nt + tid;
      if (key > T) bump(e);
      if (all_ties) {
        if (key == T) bump(e);
      } else if (base < need) {  // uniform condition
        // index order = iteration, then wave, then lane
        const bool tie = key == T;
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

  // ------------------------------------------------ Def. 2 / Eq. 2 -----------
  // The last workgroup to arrive sees every counter update: each workgroup's
  // atomics are complete (device-scope fence) before it takes its ticket.
  if (debug & 1) return;
  // Every wave first waits until its own counter updates have been performed (vmcnt(0)); the
  // barrier orders them before thread 0, whose single device-scope fence then publishes the
  // workgroup's updates before the ticket is taken.  (A fence in every wave costs far more.)
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();
  if (tid == 0) {
    __threadfence();
    sh.ticket = atomicAdd(ticket, 1u);
  }
  __syncthreads();
  if (sh.ticket != gridDim.x - 1) return;
  __threadfence();
  if (debug & 2) return;

  uint32_t cc[ITEMS > 0 ? ITEMS : 1];
  auto load_count = [&](int i) -> uint32_t {  // past the end: element N-1, masked by the callers
    const int e = i * nt + tid;
    return (uint32_t)__hip_atomic_load(&counts[e < N ? e : N - 1], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
  };
  if (ITEMS > 0) {
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) cc[i] = load_count(i);
  }
  auto ckey_valid = [&](int i, bool& valid) -> uint32_t {
    valid = i * nt + tid < N;
    return ITEMS > 0 ? cc[ITEMS > 0 ? i : 0] : load_count(i);
  };
  auto ckey_sel = [&](int i) -> uint32_t {  // all-ones (never matches) past the end
    bool valid;
    const uint32_t c = ckey_valid(i, valid);
    return valid ? c : 0xffffffffu;
  };

  // counts are <= max_count <= 65535: two 8-bit digits; the high one is skipped below 256
  uint32_t prefix = 0, prefix_mask = 0xffff0000u, need = (uint32_t)K, n_eq = 0;
  if (max_count >= 256) radix_pass<ITEMS>(ckey_sel, n_iter, 8, 256, hist, &sh, prefix, prefix_mask, need, n_eq);
  else prefix_mask |= 0xff00u;
  radix_pass<ITEMS>(ckey_sel, n_iter, 0, 256, hist, &sh, prefix, prefix_mask, need, n_eq);
  const uint32_t T = prefix;

  // ordered compaction.  pos = (#greater before) + min(#equal before, need), "before" in index
  // order = iteration, then wave, then lane.
  if constexpr (ITEMS > 0) {
    // tallies per (iteration, wave) go to a table, one wave scans it, then every thread
    // places its elements: three barriers in all
    uint32_t* tab = hist;  // [n_iter * nw], (#greater << 16) | #equal, each <= 64 before the scan
    uint64_t bgs[ITEMS], bes[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      bool valid;
      const uint32_t key = ckey_valid(i, valid);
      bgs[i] = __ballot(valid && key > T);
      bes[i] = __ballot(valid && key == T);
      if (lane == 0 && i < n_iter) tab[i * nw + wave] = ((uint32_t)__popcll(bgs[i]) << 16) | (uint32_t)__popcll(bes[i]);
    }
    __syncthreads();
    if (wave == 0) {
      // exclusive scan of the n_iter * nw entries; the two 16-bit fields cannot overflow into
      // each other because N <= 16 * 1024 here (#equal < 65536 is needed: it is <= N)
      const int n_ent = n_iter * nw;
      const int per = (n_ent + 63) / 64;
      uint32_t g_sum = 0, e_sum = 0;
      for (int j = 0; j < per; ++j) {
        const int idx = lane * per + j;
        if (idx < n_ent) { g_sum += tab[idx] >> 16; e_sum += tab[idx] & 0xffffu; }
      }
      uint32_t g_inc = g_sum, e_inc = e_sum;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t og = __shfl_up(g_inc, off, kWave), oe = __shfl_up(e_inc, off, kWave);
        if (lane >= off) { g_inc += og; e_inc += oe; }
      }
      uint32_t g_run = g_inc - g_sum, e_run = e_inc - e_sum;
      uint32_t* gtab = tab + n_ent;  // exclusive #greater / #equal prefixes, full 32 bits each
      uint32_t* etab = gtab + n_ent;
      for (int j = 0; j < per; ++j) {
        const int idx = lane * per + j;
        if (idx < n_ent) {
          const uint32_t c = tab[idx];
          gtab[idx] = g_run;
          etab[idx] = e_run;
          g_run += c >> 16;
          e_run += c & 0xffffu;
        }
      }
    }
    __syncthreads();
    const uint32_t* gtab = tab + n_iter * nw;
    const uint32_t* etab = gtab + n_iter * nw;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      if (i < n_iter) {
        const bool isg = (bgs[i] >> lane) & 1, ise = (bes[i] >> lane) & 1;
        const uint32_t g_before = gtab[i * nw + wave] + (uint32_t)__popcll(bgs[i] & lanemask_lt());
        const uint32_t e_before = etab[i * nw + wave] + (uint32_t)__popcll(bes[i] & lanemask_lt());
        const uint32_t pos = g_before + (e_before < need ? e_before : need);
        if (isg || (ise && e_before < need)) core_idx[pos] = i * nt + tid;
      }
    }
  } else {
    // large N: running totals over the iterations, two barriers per iteration
    uint32_t g_base = 0, e_base = 0;
    for (int i = 0; i < n_iter; ++i) {
      bool valid;
      const uint32_t key = ckey_valid(i, valid);
      const bool isg = valid && key > T, ise = valid && key == T;
      const uint64_t bg = __ballot(isg), be = __ballot(ise);
      __syncthreads();
      if (lane == 0) sh.wave_tot[wave] = ((uint32_t)__popcll(bg) << 16) | (uint32_t)__popcll(be);  // <= 64 each
      __syncthreads();
      uint32_t g_before = g_base, e_before = e_base, g_tot = 0, e_tot = 0;
      for (int w = 0; w < nw; ++w) {
        const uint32_t c = sh.wave_tot[w];
        if (w < wave) { g_before += c >> 16; e_before += c & 0xffffu; }
        g_tot += c >> 16;
        e_tot += c & 0xffffu;
      }
      g_before += (uint32_t)__popcll(bg & lanemask_lt());
      e_before += (uint32_t)__popcll(be & lanemask_lt());
      const uint32_t pos = g_before + (e_before < need ? e_before : need);
      if (isg || (ise && e_before < need)) core_idx[pos] = i * nt + tid;
      g_base += g_tot;
      e_base += e_tot;
    }
  }
}

__global__ void zero_i32_kernel(int32_t* p, int n, uint32_t* ticket) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
  if (i == 0 && ticket) *ticket = 0;
}

// counts[idx] += 1 for every entry of an index list (entries outside [0, N)
// are ignored).  Integer atomics: the result does not depend on the order.
__global__ void scatter_count_kernel(const int32_t* __restrict__ idx, int64_t n_idx, int N,
                                     int32_t* counts) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_idx) {
    const int n = idx[i];
    if (n >= 0 && n < N) atomicAdd(&counts[n], 1);
  }
}

// out[0] = |a ∩ b|, out[1] = |a ∪ b| for two ascending duplicate-free index
// lists (Insight-2's similarity is out[0] / out[1]).  One workgroup per list a
// (blockIdx.x picks row a + blockIdx.x * Ka and out + 2 * blockIdx.x); every
// element of a is looked up in b by binary search.
__global__ __launch_bounds__(1024) void similarity_kernel(const int32_t* __restrict__ a, int Ka,
                                                          const int32_t* __restrict__ b, int Kb,
                                                          int32_t* out) {
  __shared__ uint32_t wsum[kMaxWaves];
  a += (size_t)blockIdx.x * Ka;
  out += 2 * blockIdx.x;
  uint32_t hits = 0;
  for (int i = threadIdx.x; i < Ka; i += blockDim.x) {
    const int v = a[i];
    int lo = 0, hi = Kb;  // first position with b[pos] >= v
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (b[mid] < v) lo = mid + 1; else hi = mid;
    }
    hits += (lo < Kb && b[lo] == v);
  }
  hits = (uint32_t)wave_sum((int)hits);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = hits;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t t = 0;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += wsum[w];
    out[0] = (int32_t)t;
    out[1] = Ka + Kb - (int32_t)t;
  }
}

// best[0] = the group with the largest identical / involved ratio (compared
// exactly by cross-multiplication; 0 / 0 counts as 1; ties to the lower index).
__global__ __launch_bounds__(1024) void best_group_kernel(const int32_t* __restrict__ iu, int G,
                                                          int32_t* __restrict__ best) {
  __shared__ int64_t si[1024], su[1024];
  __shared__ int sg[1024];
  int64_t bi = -1, bu = 1;
  int bg = 0x7fffffff;
  for (int g = threadIdx.x; g < G; g += blockDim.x) {
    int64_t i = iu[2 * g], u = iu[2 * g + 1];
    if (u == 0) { i = 1; u = 1; }
    if (i * bu > bi * u) { bi = i; bu = u; bg = g; }  // strictly better only: keeps the lowest index
  }
  si[threadIdx.x] = bi; su[threadIdx.x] = bu; sg[threadIdx.x] = bg;
  __syncthreads();
  for (int half = 512; half >= 1; half >>= 1) {
    if ((int)threadIdx.x < half) {
      const int64_t i2 = si[threadIdx.x + half], u2 = su[threadIdx.x + half];
      const int g2 = sg[threadIdx.x + half];
      const int64_t l = i2 * su[threadIdx.x], r = si[threadIdx.x] * u2;
      if (l > r || (l == r && g2 < sg[threadIdx.x])) {
        si[threadIdx.x] = i2; su[threadIdx.x] = u2; sg[threadIdx.x] = g2;
      }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) best[0] = sg[0];
}

template <int ITEMS>
int launch_sel(const float* act, int M, int N, int64_t ld, int64_t q_alpha, int K, int32_t* counts,
               int32_t* core_idx, uint32_t* ticket, int grid, int nt, int privatise, size_t lds,
               int max_count, int stop, hipStream_t s) {
  static bool attr_done = false;  // raise the dynamic-LDS ceiling once (64 KB by default)
  if (!attr_done) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&select_kernel<ITEMS>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 156 * 1024) != hipSuccess)
      return CI_ERR_HIP;
    attr_done = true;
  }
  hipLaunchKernelGGL((select_kernel<ITEMS>), dim3(grid), dim3(nt), lds, s, act, M, N, ld, q_alpha, K,
                     counts, core_idx, ticket, privatise, max_count, stop);
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

}  // namespace

// The three stages of the selection, individually switchable:
//   kSelZero   clear the counters (else they are accumulated into: Eq. 3 is a sum over tokens)
//   kSelTokens Def. 1 + Eq. 3 over the M rows of act
//   kSelFinal  Def. 2 on the counters (values <= max_count)
int launch_select(const float* act, int64_t M64, int64_t N64, int64_t ld, int64_t q_alpha,
                  int64_t K64, int64_t max_count, int32_t* core_idx, int32_t* counts,
                  uint32_t* ticket, int what, hipStream_t s) {
  const int M = (what & kSelTokens) ? (int)M64 : 0, N = (int)N64, K = (int)K64;
  DeviceInfo di;
  int rc = device_info(&di);
  if (rc != CI_OK) return rc;

  if ((what & kSelZero) || (what & kSelFinal)) {
    const int nz = (what & kSelZero) ? N : 0;
    hipLaunchKernelGGL(zero_i32_kernel, dim3(nz > 0 ? (nz + 255) / 256 : 1), dim3(256), 0, s, counts, nz, ticket);
    CI_HIP_CHECK_LAUNCH();
  }
  if (!(what & (kSelTokens | kSelFinal))) return CI_OK;

  const int nt = N >= 4096 ? 1024 : 256;
  const int items = (N + nt - 1) / nt;
  int grid = di.cus * params().select_wgs_per_cu;
  if (grid > M) grid = M;
  if (grid < 1) grid = 1;
  const int tokens_per_wg = (M + grid - 1) / grid;
  // private u16 counters pay off only when a workgroup sees several tokens
  // and they fit LDS next to the digit histograms
  const size_t hist_bytes = (size_t)kHistWords * 4;
  const size_t priv_bytes = (size_t)((N + 1) / 2) * 4;
  const int privatise = (tokens_per_wg >= 2 && priv_bytes <= 88 * 1024) ? 1 : 0;
  const size_t lds = hist_bytes + (privatise ? priv_bytes : 0);
  const int stop = (what & kSelFinal) ? params().select_debug : 1;  // 1: return before the ticket
  const int mc = (int)max_count;

#define CI_SEL(I) launch_sel<I>(act, M, N, ld, q_alpha, K, counts, core_idx, ticket, grid, nt, privatise, lds, mc, stop, s)
  if (items <= 4) return CI_SEL(4);
  if (items <= 8) return CI_SEL(8);
  if (items <= 16) return CI_SEL(16);
  return CI_SEL(0);
#undef CI_SEL
}

int launch_scatter_count(const int32_t* idx, int64_t n_idx, int64_t N, int32_t* counts, hipStream_t s) {
  if (n_idx <= 0) return CI_OK;
  hipLaunchKernelGGL(scatter_count_kernel, dim3((unsigned)((n_idx + 255) / 256)), dim3(256), 0, s, idx, n_idx,
                     (int)N, counts);
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

int launch_similarity(const int32_t* a, int64_t Ka, const int32_t* b, int64_t Kb, int32_t* out, hipStream_t s) {
  hipLaunchKernelGGL(similarity_kernel, dim3(1), dim3(1024), 0, s, a, (int)Ka, b, (int)Kb, out);
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

int launch_assign_group(const int32_t* set, int64_t K, const int32_t* groups, int64_t G, int64_t Kg,
                        int32_t* best, int32_t* iu, hipStream_t s) {
  hipLaunchKernelGGL(similarity_kernel, dim3((unsigned)G), dim3(1024), 0, s, groups, (int)Kg, set, (int)K, iu);
  hipLaunchKernelGGL(best_group_kernel, dim3(1), dim3(1024), 0, s, iu, (int)G, best);
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

}  // namespace ci
