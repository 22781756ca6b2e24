// Sentence-wise core neuron selection (Sec. 3.1 of arXiv 2410.18311), three
// short launches per sentence and layer, no floating-point or counter atomics:
//
// The activation matrix may be fp32, fp16 or bf16 (the kernels that read it are
// templated on the element type; a 16-bit value is ranked through its exact
// fp32 image, and a flag makes the magnitude the ranked value).
//
// token_threshold_kernel -- Def. 1 / Eq. 1.  One workgroup of 1024 threads per
//     prompt token (looping when M exceeds the grid).  The token's N activations
//     become integer keys (the IEEE bits of a positive float are monotone in its
//     value; everything that is not > 0 gets a stand-in that matches nothing),
//     loaded once and kept in registers.  A most-significant-digit radix select
//     over LDS histograms (digits of 11 + 11 + 9 bits for fp32 inputs, the last
//     one by ranking the few keys left against each other when there are at most
//     64; 11 + 7 bits for 16-bit inputs, which have no more) finds the value T of
//     the k-th largest key, k being the share alpha of the positive keys -- their
//     number is the total of the first digit's histogram.  That histogram is
//     replicated eight times by lane so that activations sharing an exponent do
//     not serialise on one LDS address; both digits' histograms are cleared
//     while the row is still on its way from memory.  The digit that holds the
//     k-th key is found by prefix sums over threads (DPP shifts inside rows of 16
//     lanes, scalar lane reads across rows and waves).  Keys > T are token-wise
//     core neurons; of the keys == T the lowest indices fill the remaining
//     places: an ordered ballot / popcount prefix finds the index `cut` of the
//     last tie that is taken (skipped when all of them are).  The token's result
//     is the pair (T, cut): neuron n is in its core set iff key > T or (key == T
//     and n <= cut).  Nine barriers per token in the usual fp32 case (no tie
//     cut, at most 64 keys left after two digits).
// count_kernel -- Eq. 3.  Counting is a second pass over the activations by
//     neuron: a workgroup owns 64 neurons (256 when that still gives more
//     workgroups than half the compute units), walks all tokens, compares every
//     activation with its token's (T, cut) and keeps the tallies in registers
//     -- no atomics on the counters, and the counts are the same whatever the
//     scheduling.  It also adds its neurons' counts to a histogram of count
//     values.
// def2_parallel_kernel -- Def. 2 / Eq. 2 for counts below 2048 (every prompt
//     length of the workloads): each workgroup reads the threshold count off
//     the histogram, tallies the neurons before its own block, and places its
//     neurons: S ascending, position = #greater before + min(#equal before,
//     need) in the order (count descending, index ascending).
// def2_single_kernel -- the same in one workgroup for any counts up to 65535
//     (radix select over the counts, table-based ordered compaction); also
//     serves counts that come from the caller.
#include "common.hpp"

namespace ci {

namespace {

constexpr int kBins = 2048;              // largest digit: 11 bits
constexpr int kCopies = 8;               // histogram replicas, chosen by lane & 7
constexpr int kCopyStride = kBins + 8;   // words; the +8 spreads the replicas over LDS banks
constexpr int kHistWords = kCopies * kCopyStride;
constexpr int kMaxWaves = 16;
constexpr int kThreads = 1024;           // threads of the per-token and the one-workgroup Def. 2 kernels
// second digit's histogram of the per-token kernel, next to the first one so that both are cleared
// up front: fp32 keys use one replica of 2048 digits (few keys are left, spread over all digits),
// 16-bit keys eight replicas of 128 digits
constexpr int kHist2Words = kBins + 8;
constexpr int kCopyStride2 = 128 + 8;
constexpr uint32_t kNoKey = 0xffffffffu;  // stands for an activation that is not positive

// Element types the activation matrix may have; bits() gives the IEEE fp32 bits of a value (the
// conversions from the 16-bit types are exact, so ranking the bits ranks the values).
struct InF32 {
  using T = float;
  static __device__ __forceinline__ uint32_t bits(float v) { return f2u(v); }
};
struct InF16 {
  using T = _Float16;
  static __device__ __forceinline__ uint32_t bits(_Float16 v) { return f2u((float)v); }
};
struct InBF16 {
  using T = uint16_t;
  static __device__ __forceinline__ uint32_t bits(uint16_t v) { return (uint32_t)v << 16; }
};
// Key of an activation: its fp32 bits (of its magnitude when `mask` clears the sign bit) if that is
// a positive number, +inf included; else `none`.  NaN, zeros and negatives give `none`.
__device__ __forceinline__ uint32_t act_key(uint32_t bits, uint32_t mask, uint32_t none) {
  bits &= mask;
  return (bits - 1u < 0x7f800000u) ? bits : none;
}
constexpr int kCountBins = 2048;  // counts below this go to a global histogram for the parallel Def. 2
constexpr int kHistCopies = 8;    // copies of that histogram, by workgroup: atomics on one address serialise

struct SelShared {
  alignas(16) uint32_t wave_tot[kMaxWaves];  // one value per wave; the entries past the workgroup's waves stay zero
  uint32_t bin;      // chosen digit
  uint32_t above;    // keys in higher digits
  uint32_t in_bin;   // keys in the chosen digit
};
// Called once at kernel start (the first read of wave_tot comes after a barrier).
__device__ __forceinline__ void init_shared(SelShared* sh) {
  const int tid = threadIdx.x, nw = blockDim.x >> 6;
  if (tid >= nw && tid < kMaxWaves) sh->wave_tot[tid] = 0u;
}

__device__ __forceinline__ uint32_t wave_count(bool pred) { return (uint32_t)__popcll(__ballot(pred)); }

// ceil(q * n / 10^6) for q <= 10^6 and n <= 2^20 without a 64-bit division:
// x / 10^6 = (x * ceil(2^62 / 10^6)) >> 62 holds exactly for x < 7.5 * 10^12.
static_assert(CI_MAX_NEURONS <= (1 << 20), "share_ppm: the product has to stay below 7.5e12");
__device__ __forceinline__ uint32_t share_ppm(int64_t q, uint32_t n) {
  const uint64_t x = (uint64_t)q * n + 999999u;
  constexpr uint64_t kMagic = 4611686018428ull;
  const uint64_t hi = __umul64hi(x, kMagic), lo = x * kMagic;
  return (uint32_t)((hi << 2) | (lo >> 62));
}

// Inclusive prefix sum inside each row of 16 lanes: four DPP shifts (a lane whose source falls
// outside its row adds zero).  Needs all 64 lanes active.
__device__ __forceinline__ uint32_t row_prefix_incl(uint32_t v) {
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, true);  // row_shr:1
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, true);  // row_shr:2
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, true);  // row_shr:4
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, true);  // row_shr:8
  return v;
}
// Inclusive prefix sum over the lanes of a wave (lane 0 first): the rows' own prefixes, then the
// totals of the rows before, read from lanes 15, 31 and 47.
__device__ __forceinline__ uint32_t wave_prefix_incl(uint32_t v) {
  v = row_prefix_incl(v);
  const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 15);
  const uint32_t r1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 31);
  const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 47);
  const int row = (threadIdx.x & 63) >> 4;
  return v + (row >= 1 ? r0 : 0u) + (row >= 2 ? r1 : 0u) + (row >= 3 ? r2 : 0u);
}

// Thread t owns KEEP neighbouring digits counted from the top (digit nbins - 1 - (t * KEEP + j)),
// so "keys in higher digits" is a prefix sum over threads, and the totals of a thread's digits
// stay in registers for the search.  PAIR: KEEP = 2 and nbins = 2 * threads, one 8-byte read per
// replica.  KEEP = 0: any number of digits per thread, totals recomputed in the search.
template <bool FIRST, int KEEP, bool PAIR, int COPIES, int STRIDE>
__device__ __forceinline__ uint32_t find_digit_impl(const uint32_t* hist, int nbins, uint32_t k, int64_t q_alpha,
                                                    SelShared* sh) {
  int tid = threadIdx.x;
  // opaque: the addresses derived from it are computed here, not ahead of the caller's token loop
  // (where they would each occupy a register for the whole kernel)
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int per = KEEP > 0 ? KEEP : (nbins + kThreads - 1) / kThreads;
  const int o0 = tid * per;  // my first digit is nbins - 1 - o0
  auto bin_total = [&](int bidx) {
    uint32_t c = 0;
#pragma unroll
    for (int r = 0; r < COPIES; ++r) c += hist[r * STRIDE + bidx];
    return c;
  };
  uint32_t tot[KEEP > 0 ? KEEP : 1];
  uint32_t mine = 0;
  if constexpr (PAIR) {
    tot[0] = tot[1] = 0u;
#pragma unroll
    for (int r = 0; r < COPIES; ++r) {
      const uint2 pr = *reinterpret_cast<const uint2*>(hist + r * STRIDE + nbins - 2 - o0);
      tot[0] += pr.y;
      tot[1] += pr.x;
    }
    mine = tot[0] + tot[1];
  } else if constexpr (KEEP > 0) {
#pragma unroll
    for (int j = 0; j < KEEP; ++j) {
      tot[j] = (o0 + j < nbins) ? bin_total(nbins - 1 - o0 - j) : 0u;
      mine += tot[j];
    }
  } else {
    for (int j = 0; j < per; ++j)
      if (o0 + j < nbins) mine += bin_total(nbins - 1 - o0 - j);
  }
  const uint32_t incl_w = wave_prefix_incl(mine);
  if (lane == 63) sh->wave_tot[wave] = incl_w;
  __syncthreads();
  // prefix over the (at most 16) wave totals in the first row of lanes
  const uint32_t wt = sh->wave_tot[lane & (kMaxWaves - 1)];
  const uint32_t wp = row_prefix_incl(wt);
  const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)wp, kMaxWaves - 1);  // keys of all waves
  const uint32_t upto = (uint32_t)__builtin_amdgcn_readlane((int)wp, wave);
  const uint32_t own = (uint32_t)__builtin_amdgcn_readlane((int)wt, wave);
  const uint32_t before = upto - own;  // keys owned by the waves before mine
  if (FIRST) k = share_ppm(q_alpha, total);
  const uint32_t incl = incl_w + before;  // keys in my digits and above
  const uint32_t excl = incl - mine;      // keys strictly above my digits
  if (k != 0 && excl < k && k <= incl) {
    uint32_t run = excl;
    if constexpr (KEEP > 0) {
      bool found = false;
#pragma unroll
      for (int j = 0; j < KEEP; ++j) {
        const uint32_t c = tot[j];
        if (!found && run + c >= k) {
          sh->bin = (uint32_t)(nbins - 1 - o0 - j);
          sh->above = run;
          sh->in_bin = c;
          found = true;
        }
        run += c;
      }
    } else {
      for (int j = 0; j < per; ++j) {
        if (o0 + j >= nbins) break;
        const uint32_t c = bin_total(nbins - 1 - o0 - j);
        if (run + c >= k) {
          sh->bin = (uint32_t)(nbins - 1 - o0 - j);
          sh->above = run;
          sh->in_bin = c;
          break;
        }
        run += c;
      }
    }
  }
  __syncthreads();
  return k;
}

// hist holds COPIES replicas (STRIDE words apart) of nbins digit counts.  Finds the digit that
// contains the k-th largest key (1 <= k <= total) and how many keys lie in higher digits; result in
// sh->bin / above / in_bin, visible to all threads on return.  FIRST: k is not given but derived
// here as the share q_alpha of all keys in the histogram (the first digit's histogram holds every
// positive key).  Returns k; 0 means there is no key at all and nothing was written.
// For workgroups of kThreads threads; nbins is a constant at every call.
template <bool FIRST, int COPIES, int STRIDE>
__device__ __forceinline__ uint32_t find_digit(const uint32_t* hist, int nbins, uint32_t k, int64_t q_alpha,
                                               SelShared* sh) {
  if (nbins == 2 * kThreads) return find_digit_impl<FIRST, 2, true, COPIES, STRIDE>(hist, nbins, k, q_alpha, sh);
  if (nbins <= kThreads) return find_digit_impl<FIRST, 1, false, COPIES, STRIDE>(hist, nbins, k, q_alpha, sh);
  if (nbins <= 8 * kThreads) return find_digit_impl<FIRST, 8, false, COPIES, STRIDE>(hist, nbins, k, q_alpha, sh);
  return find_digit_impl<FIRST, 0, false, COPIES, STRIDE>(hist, nbins, k, q_alpha, sh);
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

// Clears COPIES replicas (STRIDE words apart) of an nb-digit histogram, 16 bytes per store (nb and
// STRIDE are multiples of 4; the padding words are never read).
template <int COPIES, int STRIDE>
__device__ __forceinline__ void clear_hist(uint32_t* hist, int nb) {
  const int q = nb >> 2;  // 16-byte pieces per replica
  int first = threadIdx.x;
  asm volatile("" : "+v"(first));  // opaque: the store addresses are not kept across the caller's loops
  for (int j = first; j < COPIES * q; j += kThreads)
    *reinterpret_cast<uint4*>(hist + (j / q) * STRIDE + (j % q) * 4) = make_uint4(0, 0, 0, 0);
}

// One radix pass: histogram of the digit (key >> shift) & (nb - 1) over the
// keys that match `prefix` under `prefix_mask`, then the digit holding the
// k-th largest of them.  Updates prefix / prefix_mask / k; n_eq = keys in it.
// CLEARED: the caller has cleared the histogram, with a barrier since.  FIRST: k comes out of the
// pass as the share q_alpha of the keys counted (0: there are none, and nothing else is updated).
// No barrier at the end: the next writes to *sh or the histogram all follow a barrier of their own.
template <int ITEMS, bool FIRST = false, bool CLEARED = false, int COPIES = kCopies, int STRIDE = kCopyStride,
          class KeyAt>
__device__ __forceinline__ void radix_pass(KeyAt key_at, int n_iter, int shift, int nb, uint32_t* hist,
                                           SelShared* sh, uint32_t& prefix, uint32_t& prefix_mask,
                                           uint32_t& k, uint32_t& n_eq, int64_t q_alpha = 0) {
  uint32_t* my_hist = hist + (threadIdx.x & (COPIES - 1)) * STRIDE;
  if (!CLEARED) {
    clear_hist<COPIES, STRIDE>(hist, nb);
    __syncthreads();
  }
  for_items<ITEMS>(n_iter, [&](int i) {
    const uint32_t key = key_at(i);
    if ((key & prefix_mask) == prefix) atomicAdd(&my_hist[(key >> shift) & (nb - 1)], 1u);
  });
  __syncthreads();
  k = find_digit<FIRST, COPIES, STRIDE>(hist, nb, k, q_alpha, sh);
  if (FIRST && k == 0) return;
  prefix |= sh->bin << shift;
  prefix_mask |= (uint32_t)(nb - 1) << shift;
  k -= sh->above;
  n_eq = sh->in_bin;
}

template <int ITEMS, bool TWO, class IN>  // TWO: registers capped so that two workgroups of 16 waves share a compute unit
__global__ __launch_bounds__(kThreads, TWO ? 8 : 4) void token_threshold_kernel(const typename IN::T* __restrict__ act,
                                                               int M, int N, int64_t ld, int64_t q_alpha,
                                                               uint32_t sign_mask, uint32_t* __restrict__ thr,
                                                               uint32_t* ghist, int ghist_words) {
  using TI = typename IN::T;
  constexpr bool kNarrow = sizeof(TI) == 2;  // the fp32 image of a 16-bit value has nothing below bit 13
  __shared__ SelShared sh;
  __shared__ uint32_t cut_s;
  constexpr int kCand = 64;
  __shared__ uint32_t cand[kCand];
  __shared__ uint32_t cand_n;
  extern __shared__ __attribute__((aligned(16))) uint32_t dyn[];  // [kHistWords + kHist2Words], cleared 16 bytes at a time
  uint32_t* hist = dyn;
  uint32_t* hist2 = dyn + kHistWords;
  constexpr int nt = kThreads, nw = kMaxWaves;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int n_iter = (N + nt - 1) / nt;
  init_shared(&sh);
  if (ghist)  // cleared here, a slice per workgroup, for the counting launch that follows
    for (int j = blockIdx.x * nt + tid; j < ghist_words; j += gridDim.x * nt) ghist[j] = 0u;

  for (int m = blockIdx.x; m < M; m += gridDim.x) {
    const TI* row = act + (size_t)m * ld;
    // the histograms of both digits are cleared while the row is on its way
    clear_hist<kCopies, kCopyStride>(hist, 2048);
    if (kNarrow) clear_hist<kCopies, kCopyStride2>(hist2, 128);
    else clear_hist<1, kCopyStride>(hist2, 2048);
    if (tid == 0) cand_n = 0;
    uint32_t kc[ITEMS > 0 ? ITEMS : 1];
    uint32_t lane_id = (uint32_t)tid;  // thread index within the workgroup
    asm volatile("" : "+v"(lane_id));
    if (ITEMS > 0) {
      // branch-free loads, issued back to back in batches (a batch bounds the registers that hold
      // values not yet turned into keys)
      constexpr int BATCH = ITEMS > 16 ? 8 : (ITEMS > 0 ? ITEMS : 1);
#pragma unroll
      for (int i0 = 0; i0 < ITEMS; i0 += BATCH) {
        TI av[BATCH];
#pragma unroll
        for (int j = 0; j < BATCH; ++j) {
          // uniform base of the item + a 32-bit lane offset (clamped inside the row); the lane
          // index is made opaque per token so that the offsets are not all computed ahead of
          // the token loop and kept in two registers each
          const int s0 = ((i0 + j) * nt < N) ? (i0 + j) * nt : 0;
          const TI* item = row + s0;
          av[j] = item[min(lane_id, (uint32_t)(N - 1 - s0))];
        }
#pragma unroll
        for (int j = 0; j < BATCH; ++j) {
          const uint32_t e = (uint32_t)((i0 + j) * nt) + lane_id;
          kc[i0 + j] = e < (uint32_t)N ? act_key(IN::bits(av[j]), sign_mask, kNoKey) : kNoKey;
        }
      }
    }
    // key of this thread's i-th element.  Elements that are not positive, and those past the end,
    // get all-ones: bit 31 is part of the prefix mask from the start, so they match no prefix, and
    // no threshold equals them
    auto key_at = [&](int i) -> uint32_t {
      if (ITEMS > 0) return kc[ITEMS > 0 ? i : 0];  // i is a constant after unrolling
      const int e = i * nt + tid;
      if (e >= N) return kNoKey;
      return act_key(IN::bits(row[e]), sign_mask, kNoKey);
    };
    auto key_sel = key_at;

    __syncthreads();  // the histograms are clear

    // 31-bit keys: digits of 11, 11 and 9 bits (16-bit inputs: 11 and 7, which is all they have).
    // Bit 31 is part of the mask from the start, so the all-ones stand-in of a zero key never
    // matches.  The first digit's histogram counts every positive key, and k -- the share alpha of
    // them -- is taken from its total.
    uint32_t prefix = 0, prefix_mask = 0x80000000u, need = 0, n_eq = 0;
    radix_pass<ITEMS, true, true>(key_sel, n_iter, 20, 2048, hist, &sh, prefix, prefix_mask, need, n_eq, q_alpha);
    if (need == 0) {  // uniform: no positive activation, nothing is selected (no key exceeds all-ones)
      if (tid == 0) { thr[2 * m] = 0xffffffffu; thr[2 * m + 1] = 0u; }
      continue;
    }
    uint32_t T;  // the k-th largest key; `need` of the n_eq keys == T are in the top k
    if constexpr (kNarrow) {
      radix_pass<ITEMS, false, true, kCopies, kCopyStride2>(key_sel, n_iter, 13, 128, hist2, &sh, prefix, prefix_mask,
                                                            need, n_eq);
      T = prefix;  // bits 13 .. 30 are all of the key
    } else {
      radix_pass<ITEMS, false, true, 1, kCopyStride>(key_sel, n_iter, 9, 2048, hist2, &sh, prefix, prefix_mask, need,
                                                     n_eq);
      if (n_eq <= kCand) {  // uniform; the usual case: after 22 bits only a few keys are left
        // the candidates go to a short list and are ranked against each other
        for_items<ITEMS>(n_iter, [&](int i) {
          const uint32_t key = key_sel(i);
          if ((key & prefix_mask) == prefix) cand[atomicAdd(&cand_n, 1u)] = key;
        });
        __syncthreads();
        if (tid < (int)n_eq) {
          const uint32_t c = cand[tid];
          uint32_t g = 0, ge = 0;
          for (uint32_t j = 0; j < n_eq; ++j) {
            g += cand[j] > c;
            ge += cand[j] >= c;
          }
          if (g < need && need <= ge) {  // equal candidates write the same three values
            sh.bin = c;
            sh.above = g;
            sh.in_bin = ge - g;
          }
        }
        __syncthreads();
        T = sh.bin;
        need -= sh.above;
        n_eq = sh.in_bin;
        // no barrier: sh and the list are written again only after barriers of the next token
      } else {
        radix_pass<ITEMS>(key_sel, n_iter, 0, 512, hist, &sh, prefix, prefix_mask, need, n_eq);
        T = prefix;
      }
    }

    // index of the last tie that is taken; ties in index order = iteration, then wave, then lane
    if (tid == 0) cut_s = 0x7fffffffu;  // all ties taken (the usual case: need == n_eq)
    if (need != n_eq) {                 // uniform
      if constexpr (ITEMS > 0) {
        // keys in registers: ties per (iteration, wave) go to LDS (the histograms are done with);
        // a row of 16 lanes then turns one iteration's 16 wave tallies into prefixes over the
        // waves and the iteration's total; every thread finds the one iteration that holds the
        // last tie taken and only that iteration is ranked lane by lane
        static_assert(ITEMS % 4 == 0, "the prefix step runs in whole waves");
        uint32_t* cnt = hist;                        // [ITEMS][16]
        uint32_t* itot = hist + ITEMS * kMaxWaves;   // [ITEMS]
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
          const uint32_t c = wave_count(kc[i] == T);  // T < 2^31, so elements without a key never match
          if (lane == 0) cnt[i * nw + wave] = c;
        }
        __syncthreads();
        if (tid < ITEMS * kMaxWaves) {
          const uint32_t c = cnt[tid];
          const uint32_t inc = row_prefix_incl(c);
          cnt[tid] = inc - c;  // ties of this iteration in the waves before
          if ((tid & (kMaxWaves - 1)) == kMaxWaves - 1) itot[tid >> 4] = inc;
        }
        __syncthreads();
        uint32_t base = 0;  // ties in earlier iterations
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
          const uint32_t t = itot[i];
          if (base < need && need <= base + t) {  // uniform: the (need - 1)-th tie lies in this iteration
            const bool tie = kc[i] == T;
            const uint64_t bal = __ballot(tie);
            const uint32_t rank = base + cnt[i * nw + wave] + (uint32_t)__popcll(bal & lanemask_lt());
            if (tie && rank == need - 1) cut_s = (uint32_t)(i * nt + tid);
          }
          base += t;
        }
      } else {
        uint32_t base = 0;                // ties seen in earlier iterations
        for_items<ITEMS>(n_iter, [&](int i) {
          if (base < need) {  // uniform condition
            const bool tie = key_at(i) == T;  // T < 2^31, so elements without a key never match
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
            if (tie && rank == need - 1) cut_s = (uint32_t)(i * nt + tid);
            base += tot;
          }
        });
      }
      __syncthreads();  // cut_s is final, and the tables in the histogram's place are done with
    }
    if (tid == 0) { thr[2 * m] = T; thr[2 * m + 1] = cut_s; }
    // no barrier: the next token clears the histograms (last read before a barrier above) and
    // thread 0 alone resets cut_s; everything else in LDS is written again only after barriers
  }
}

// Tallies of one lane's four neurons n0 .. n0+3 over its share of the tokens.  A wave instruction
// covers TPW tokens (lane / (64 / TPW) picks the token, the other lane bits the neuron quad); waves
// take batches of UN * TPW tokens in turn, UN loads per lane in flight.  VEC: one 16-byte load per
// token, else four clamped 4-byte loads (unaligned rows or the last neurons of the layer).
template <bool VEC, int TPW, class IN>
__device__ __forceinline__ void count_tokens_of_lane(const typename IN::T* __restrict__ act, int64_t ld,
                                                     const uint32_t* __restrict__ thr, int M, int N, uint32_t sign_mask,
                                                     int n0, int ts, int wave, int nw, uint32_t (&cnt)[4]) {
  using TI = typename IN::T;
  constexpr int UN = 8;
  for (int m0 = wave * UN * TPW; m0 < M; m0 += nw * UN * TPW) {
    uint32_t vb[UN][4];  // fp32 bits of the four activations
    uint32_t T[UN], cut[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int m = min(m0 + u * TPW + ts, M - 1);  // clamped: a repeated token is masked below
      const TI* p = act + (size_t)m * ld;
      if (VEC) {
        if constexpr (sizeof(TI) == 4) {
          const float4 q = *reinterpret_cast<const float4*>(p + n0);
          vb[u][0] = f2u(q.x); vb[u][1] = f2u(q.y); vb[u][2] = f2u(q.z); vb[u][3] = f2u(q.w);
        } else {
          struct alignas(8) Quad { TI e[4]; };
          const Quad q = *reinterpret_cast<const Quad*>(p + n0);
#pragma unroll
          for (int c = 0; c < 4; ++c) vb[u][c] = IN::bits(q.e[c]);
        }
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) vb[u][c] = IN::bits(p[min(n0 + c, N - 1)]);
      }
      T[u] = thr[2 * m];
      cut[u] = thr[2 * m + 1];
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const uint32_t live = (m0 + u * TPW + ts < M) ? 1u : 0u;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint32_t key = n0 + c < N ? act_key(vb[u][c], sign_mask, 0u) : 0u;
        cnt[c] += (key > T[u] || (key == T[u] && (uint32_t)(n0 + c) <= cut[u])) ? live : 0u;
      }
    }
  }
}

// Eq. 3: a workgroup owns NPW neurons and walks all tokens (NPW = 64 gives the launch four times
// the workgroups of NPW = 256: the pass is bound by vector instructions per compute unit, and the
// layers here have only 43 to 144 blocks of 256 neurons).  With `ghist` it also adds its neurons'
// final counts to the histogram of count values (integer atomics, commutative).
template <int NPW, class IN>
__global__ __launch_bounds__(1024) void count_kernel(const typename IN::T* __restrict__ act, int M, int N, int64_t ld,
                                                     uint32_t sign_mask, const uint32_t* __restrict__ thr, int vec_ok,
                                                     int32_t* counts, int accumulate, uint32_t* ghist,
                                                     int64_t counts_stride) {
  // blockIdx.y: the sentence of a batch (M rows, M thresholds, its own counters and histogram)
  act += (size_t)blockIdx.y * M * ld;
  thr += (size_t)blockIdx.y * M * 2;
  counts += (size_t)blockIdx.y * counts_stride;
  if (ghist) ghist += (size_t)blockIdx.y * kCountBins * kHistCopies;
  constexpr int TPW = 256 / NPW;   // tokens per wave instruction
  constexpr int LPR = 64 / TPW;    // lanes per token row
  __shared__ uint32_t tally[NPW];
  __shared__ uint32_t vhist[kCountBins];
  const int tid = threadIdx.x, nt = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
  const int nb = blockIdx.x;
  const int quad = lane % LPR, ts = lane / LPR;
  const int n0 = nb * NPW + quad * 4;  // this lane's four neurons
  for (int j = tid; j < NPW; j += nt) tally[j] = 0;
  __syncthreads();
  uint32_t cnt[4] = {0, 0, 0, 0};
  // rows of the last, partial block take the element-wise path as a whole (uniform per workgroup
  // would be enough; per lane keeps the full blocks' lanes on the vector path)
  if (vec_ok && n0 + 3 < N) count_tokens_of_lane<true, TPW, IN>(act, ld, thr, M, N, sign_mask, min(n0, N - 4), ts, wave, nw, cnt);
  else count_tokens_of_lane<false, TPW, IN>(act, ld, thr, M, N, sign_mask, n0, ts, wave, nw, cnt);
  // block tallies: integer adds in LDS (commutative), then one plain store per neuron
#pragma unroll
  for (int c = 0; c < 4; ++c)
    if (cnt[c]) atomicAdd(&tally[quad * 4 + c], cnt[c]);
  __syncthreads();
  // the count values cluster on a few bins: they are first tallied per workgroup in LDS, so that a
  // hot bin receives one device-scope atomic per workgroup, not one per neuron (those serialise)
  if (ghist) {
    for (int j = tid; j < kCountBins; j += nt) vhist[j] = 0;
    __syncthreads();
  }
  for (int j = tid; j < NPW; j += nt) {
    const int n = nb * NPW + j;
    if (n < N) {
      const int32_t c = (int32_t)tally[j] + (accumulate ? counts[n] : 0);
      counts[n] = c;
      if (ghist && c >= 0 && c < kCountBins) atomicAdd(&vhist[c], 1u);
    }
  }
  if (ghist) {
    __syncthreads();
    uint32_t* gcopy = ghist + (nb % kHistCopies) * kCountBins;
    for (int j = tid; j < kCountBins; j += nt)
      if (vhist[j]) atomicAdd(&gcopy[j], vhist[j]);
  }
}

// Def. 2 in parallel, for counts below kCountBins whose histogram `ghist` is known: every workgroup
// (256 threads = 256 neurons) finds the threshold count T from the histogram, tallies the neurons
// before its own that are above / at T, and places its own: position = #greater before +
// min(#equal before, need).  The tally re-reads the counts before the block (cache resident;
// N <= 65536 keeps that to a few MB in all).
__global__ __launch_bounds__(1024) void def2_parallel_kernel(const int32_t* __restrict__ counts,
                                                             const uint32_t* __restrict__ ghist, int N, int K,
                                                             int32_t* __restrict__ core_idx, int vec_ok,
                                                             int64_t counts_stride) {
  counts += (size_t)blockIdx.y * counts_stride;  // blockIdx.y: the sentence of a batch
  ghist += (size_t)blockIdx.y * kCountBins * kHistCopies;
  core_idx += (size_t)blockIdx.y * K;
  __shared__ __attribute__((aligned(16))) uint32_t wtot[4], wg[kMaxWaves], we[kMaxWaves];
  __shared__ uint32_t T_s, need_s;
  const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63, wave = tid >> 6;
  // (1) T: the count value with #(count > T) < K <= #(count >= T).  Thread t < 256 owns the eight
  // bins 2047 - 8t - j, highest first, so the keys above a bin are a prefix sum over threads.
  uint32_t bins[8], mine = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) bins[j] = 0;
  if (tid < kCountBins / 8) {
#pragma unroll
    for (int r = 0; r < kHistCopies; ++r) {
      const uint4* hp = reinterpret_cast<const uint4*>(ghist + r * kCountBins + (kCountBins - 8 - tid * 8));
      const uint4 lo = hp[0], hi = hp[1];
      bins[0] += hi.w; bins[1] += hi.z; bins[2] += hi.y; bins[3] += hi.x;
      bins[4] += lo.w; bins[5] += lo.z; bins[6] += lo.y; bins[7] += lo.x;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) mine += bins[j];
  }
  const uint32_t incl_w = wave_prefix_incl(mine);
  if (lane == 63 && wave < 4) wtot[wave] = incl_w;
  __syncthreads();
  if (tid < kCountBins / 8) {
    const uint4 w4 = *reinterpret_cast<const uint4*>(wtot);
    const uint32_t before = (wave > 0 ? w4.x : 0u) + (wave > 1 ? w4.y : 0u) + (wave > 2 ? w4.z : 0u);
    const uint32_t incl = incl_w + before, excl = incl - mine;
    if (excl < (uint32_t)K && (uint32_t)K <= incl) {
      uint32_t run = excl;
      bool found = false;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (!found && run + bins[j] >= (uint32_t)K) {
          T_s = (uint32_t)(kCountBins - 1 - tid * 8 - j);
          need_s = (uint32_t)K - run;
          found = true;
        }
        run += bins[j];
      }
    }
  }
  __syncthreads();
  const uint32_t T = T_s, need = need_s;
  // (2) neurons before this block that are above / at T: all threads, eight loads in flight each
  // (the loop is nothing but latency)
  const int before = blockIdx.x * 256;
  uint32_t g = 0, e = 0;
  if (vec_ok) {
    const int4* cv = reinterpret_cast<const int4*>(counts);
    const int nv = before / 4;
    for (int i0 = tid; i0 < nv; i0 += nt * 8) {
      int4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = cv[min(i0 + u * nt, nv - 1)];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (i0 + u * nt < nv) {
          g += ((uint32_t)v[u].x > T) + ((uint32_t)v[u].y > T) + ((uint32_t)v[u].z > T) + ((uint32_t)v[u].w > T);
          e += ((uint32_t)v[u].x == T) + ((uint32_t)v[u].y == T) + ((uint32_t)v[u].z == T) + ((uint32_t)v[u].w == T);
        }
      }
    }
  } else {
    for (int i0 = tid; i0 < before; i0 += nt * 8) {
      uint32_t v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = (uint32_t)counts[min(i0 + u * nt, before - 1)];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (i0 + u * nt < before) {
          g += v[u] > T;
          e += v[u] == T;
        }
      }
    }
  }
  // wave totals: lane 63 of the prefix sums
  g = wave_prefix_incl(g);
  e = wave_prefix_incl(e);
  // (3) this block's neurons (threads 0..255), in index order = wave, then lane
  const int n = before + tid;
  const bool valid = tid < 256 && n < N;
  const uint32_t c = valid ? (uint32_t)counts[n] : 0u;
  const bool isg = valid && c > T, ise = valid && c == T;
  const uint64_t bg = __ballot(isg), be = __ballot(ise);
  if (lane == 63) {
    wg[wave] = g;
    we[wave] = e;
    if (wave < 4) wtot[wave] = ((uint32_t)__popcll(bg) << 16) | (uint32_t)__popcll(be);
  }
  if (tid >= (nt >> 6) && tid < kMaxWaves) { wg[tid] = 0u; we[tid] = 0u; }  // waves that do not exist
  __syncthreads();
  if (tid < 256) {
    uint32_t g_before = 0, e_before = 0;
#pragma unroll
    for (int q = 0; q < kMaxWaves / 4; ++q) {
      const uint4 a = *reinterpret_cast<const uint4*>(&wg[4 * q]), b = *reinterpret_cast<const uint4*>(&we[4 * q]);
      g_before += a.x + a.y + a.z + a.w;
      e_before += b.x + b.y + b.z + b.w;
    }
    const uint4 w4 = *reinterpret_cast<const uint4*>(wtot);
    const uint32_t wt[3] = {w4.x, w4.y, w4.z};
#pragma unroll
    for (int w = 0; w < 3; ++w)
      if (w < wave) { g_before += wt[w] >> 16; e_before += wt[w] & 0xffffu; }
    g_before += (uint32_t)__popcll(bg & lanemask_lt());
    e_before += (uint32_t)__popcll(be & lanemask_lt());
    const uint32_t pos = g_before + (e_before < need ? e_before : need);
    if (isg || (ise && e_before < need)) core_idx[pos] = n;
  }
}

// Def. 2 in one workgroup (any counts up to 65535; also for counts that come from the caller).
template <int ITEMS>
__global__ __launch_bounds__(1024) void def2_single_kernel(int N, int32_t* counts, int K, int32_t* core_idx,
                                                           int max_count) {
  __shared__ SelShared sh;
  extern __shared__ __attribute__((aligned(16))) uint32_t dyn[];  // [kHistWords] histograms, cleared 16 bytes at a time
  uint32_t* hist = dyn;
  constexpr int nt = kThreads, nw = kMaxWaves;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int n_iter = (N + nt - 1) / nt;
  init_shared(&sh);

  // plain loads: all of a thread's counts are in flight at once
  auto total_count = [&](int e) -> uint32_t { return (uint32_t)counts[e]; };

  uint32_t cc[ITEMS > 0 ? ITEMS : 1];
  auto load_count = [&](int i) -> uint32_t {  // past the end: element N-1, masked by the callers
    const int e = i * nt + tid;
    return total_count(e < N ? e : N - 1);
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

  // counts are <= max_count <= 65535: one digit of 8 or 11 bits when they stay below 256 or 2048
  // (every prompt length of the workloads), else an 8-bit digit on top of an 8-bit one
  uint32_t prefix = 0, prefix_mask = 0xffff0000u, need = (uint32_t)K, n_eq = 0;
  if (max_count < 256) {
    prefix_mask |= 0xff00u;
    radix_pass<ITEMS>(ckey_sel, n_iter, 0, 256, hist, &sh, prefix, prefix_mask, need, n_eq);
  } else if (max_count < 2048) {
    prefix_mask |= 0xf800u;
    radix_pass<ITEMS>(ckey_sel, n_iter, 0, 2048, hist, &sh, prefix, prefix_mask, need, n_eq);
  } else {
    radix_pass<ITEMS>(ckey_sel, n_iter, 8, 256, hist, &sh, prefix, prefix_mask, need, n_eq);
    radix_pass<ITEMS>(ckey_sel, n_iter, 0, 256, hist, &sh, prefix, prefix_mask, need, n_eq);
  }
  const uint32_t T = prefix;

  // ordered compaction.  pos = (#greater before) + min(#equal before, need), "before" in index
  // order = iteration, then wave, then lane.
  if constexpr (ITEMS > 0) {
    // tallies per (iteration, wave) go to a table, one wave scans it, then every thread places its
    // elements (the ballots are taken again rather than kept): three barriers in all
    uint32_t* tab = hist;  // [n_iter * nw], (#greater << 16) | #equal, each <= 64 before the scan
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      bool valid;
      const uint32_t key = ckey_valid(i, valid);
      const uint64_t bg = __ballot(valid && key > T), be = __ballot(valid && key == T);
      if (lane == 0 && i < n_iter) tab[i * nw + wave] = ((uint32_t)__popcll(bg) << 16) | (uint32_t)__popcll(be);
    }
    __syncthreads();
    if (wave == 0) {
      // exclusive scan of the n_iter * nw entries (the running sums are kept in full 32 bits)
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
      uint32_t* gtab = tab + n_ent;  // exclusive #greater / #equal prefixes
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
        bool valid;
        const uint32_t key = ckey_valid(i, valid);
        const bool isg = valid && key > T, ise = valid && key == T;
        const uint64_t bg = __ballot(isg), be = __ballot(ise);
        const uint32_t g_before = gtab[i * nw + wave] + (uint32_t)__popcll(bg & lanemask_lt());
        const uint32_t e_before = etab[i * nw + wave] + (uint32_t)__popcll(be & lanemask_lt());
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

__global__ void zero_i32_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
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

template <int ITEMS, bool TWO, class IN>
int launch_threshold(const typename IN::T* act, int M, int N, int64_t ld, int64_t q_alpha, uint32_t sign_mask,
                     uint32_t* thr, uint32_t* ghist, int ghist_words, int grid, hipStream_t s) {
  static std::atomic<uint64_t> attr_seen{0};  // raise the dynamic-LDS ceiling once (64 KB by default)
  if (allow_dynamic_lds(attr_seen, reinterpret_cast<const void*>(&token_threshold_kernel<ITEMS, TWO, IN>), 156 * 1024) != CI_OK)
    return CI_ERR_HIP;
  hipLaunchKernelGGL((token_threshold_kernel<ITEMS, TWO, IN>), dim3(grid), dim3(kThreads),
                     (size_t)(kHistWords + kHist2Words) * 4, s, act,
                     M, N, ld, q_alpha, sign_mask, thr, ghist, ghist_words);
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

// Def. 1 and Eq. 3 for an activation matrix of element type IN::T.  The fp32 path has a kernel for
// every keys-per-thread step; the 16-bit types share three of them (16, 40, streaming).
template <class IN>
int launch_tokens(const void* act_v, int B, int M_each, int N, int64_t ld, int64_t q_alpha, uint32_t sign_mask,
                  uint32_t* thr, uint32_t* ghist, int32_t* counts, int64_t counts_stride, int accumulate, int nt,
                  int items, int nblocks, int cus, hipStream_t s) {
  using TI = typename IN::T;
  const TI* act = reinterpret_cast<const TI*>(act_v);
  const int M = B * M_each;  // Def. 1 treats the rows of all sentences alike
  const int ghist_words = B * kCountBins * kHistCopies;
  // more tokens than compute units and at most 16 keys per thread: two workgroups per compute
  // unit (a token round is half instruction issue, half barriers and latency; the register cap
  // this needs costs a single workgroup about 10 %, so it is not used for short prompts)
  const bool two = M > cus && items <= 16 && params().select_wgs_per_cu >= 2;
  int grid = cus * (two ? 2 : 1);
  if (grid > M) grid = M;
  if (grid < 1) grid = 1;
  int rc = CI_OK;
#define CI_THR(I, W) launch_threshold<I, W, IN>(act, M, N, ld, q_alpha, sign_mask, thr, ghist, ghist_words, grid, s)
  if constexpr (sizeof(TI) == 4) {
    if (two && items <= 8) rc = CI_THR(8, true);
    else if (two) rc = CI_THR(16, true);
    else if (items <= 4) rc = CI_THR(4, false);
    else if (items <= 8) rc = CI_THR(8, false);
    else if (items <= 16) rc = CI_THR(16, false);
    else if (items <= 24) rc = CI_THR(24, false);
    else if (items <= 32) rc = CI_THR(32, false);
    else if (items <= 36) rc = CI_THR(36, false);
    else if (items <= 40) rc = CI_THR(40, false);
    else rc = CI_THR(0, false);
  } else {
    if (two) rc = CI_THR(16, true);
    else if (items <= 16) rc = CI_THR(16, false);
    else if (items <= 40) rc = CI_THR(40, false);
    else rc = CI_THR(0, false);
  }
#undef CI_THR
  if (rc != CI_OK) return rc;
  // four activations per load: 16 bytes of fp32 or 8 bytes of a 16-bit type
  const uintptr_t quad = 4 * sizeof(TI);
  const int vec_ok = ((reinterpret_cast<uintptr_t>(act) & (quad - 1)) == 0 && ld % 4 == 0) ? 1 : 0;
  // 64 neurons per workgroup when blocks of 256 would leave more than half of the chip idle
  if (nblocks * B <= cus / 2)
    hipLaunchKernelGGL((count_kernel<64, IN>), dim3((N + 63) / 64, B), dim3(nt), 0, s, act, M_each, N, ld, sign_mask,
                       thr, vec_ok, counts, accumulate, ghist, counts_stride);
  else
    hipLaunchKernelGGL((count_kernel<256, IN>), dim3(nblocks, B), dim3(nt), 0, s, act, M_each, N, ld, sign_mask, thr,
                       vec_ok, counts, accumulate, ghist, counts_stride);
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

template <int ITEMS>
int launch_def2_single(int N, int32_t* counts, int K, int32_t* core_idx, int max_count, hipStream_t s) {
  static std::atomic<uint64_t> attr_seen{0};
  if (allow_dynamic_lds(attr_seen, reinterpret_cast<const void*>(&def2_single_kernel<ITEMS>), 156 * 1024) != CI_OK)
    return CI_ERR_HIP;
  hipLaunchKernelGGL((def2_single_kernel<ITEMS>), dim3(1), dim3(kThreads), (size_t)kHistWords * 4, s, N, counts, K,
                     core_idx, max_count);
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

size_t round256z(size_t n) { return (n + 255) / 256 * 256; }

}  // namespace

// Workspace of one selection: per-token (T, cut) pairs, the histogram of count
// values, and counters for callers that pass none.
void select_ws_layout(int64_t M, int64_t N, SelectWs* w, int64_t B) {
  w->off_thr = 0;
  w->off_hist = round256z((size_t)B * (size_t)(M > 0 ? M : 1) * 2 * sizeof(uint32_t));
  w->off_counts = w->off_hist + round256z((size_t)B * kCountBins * kHistCopies * sizeof(uint32_t));
  w->total = w->off_counts + round256z((size_t)B * (size_t)N * sizeof(int32_t));
}

// The stages of the selection, individually switchable:
//   kSelZero       clear the counters (before members are scattered into them)
//   kSelTokens     Def. 1 over the M rows of act, then Eq. 3 (kSelAccumulate: added to the counters)
//   kSelFinal      Def. 2 on the counters (values <= max_count)
// B > 1: a batch of sentences, sentence b being rows [b M, (b + 1) M) of act, with counts [B, N]
// (row stride counts_stride) and core_idx [B, K]; only for the whole selection in one go
// (kSelTokens | kSelFinal) where Def. 2 runs in parallel (select_batch_ok).
bool select_batch_ok(int64_t M, int64_t N) {
  return M < kCountBins && (N + 255) / 256 <= 256 && params().select_def2_single == 0;
}

int launch_select(const void* act, int act_dtype, int take_abs, int64_t M64, int64_t N64, int64_t ld,
                  int64_t q_alpha, int64_t K64, int64_t max_count, int32_t* core_idx, int32_t* counts, void* ws,
                  int what, hipStream_t s, int B, int64_t counts_stride) {
  const int M = (what & kSelTokens) ? (int)M64 : 0, N = (int)N64, K = (int)K64;
  DeviceInfo di;
  int rc = device_info(&di);
  if (rc != CI_OK) return rc;

  if (what & kSelZero) {
    hipLaunchKernelGGL(zero_i32_kernel, dim3((N + 255) / 256), dim3(256), 0, s, counts, N);
    CI_HIP_CHECK_LAUNCH();
  }
  if (!(what & (kSelTokens | kSelFinal))) return CI_OK;

  const int nt = N >= 4096 ? 1024 : 256;               // threads of the counting launch
  const int items = (N + kThreads - 1) / kThreads;     // keys per thread in the one-row kernels
  const int nblocks = (N + 255) / 256;
  // Def. 2 in parallel needs the histogram that the counting launch fills
  const bool parallel_final = (what & kSelTokens) && (what & kSelFinal) && !(what & kSelAccumulate) &&
                              max_count < kCountBins && nblocks <= 256 && params().select_def2_single == 0;
  if (what & kSelTokens) {
    SelectWs w;
    select_ws_layout(M, N, &w, B);
    if (B > 1 && !parallel_final) return CI_ERR_UNSUPPORTED;
    char* base = reinterpret_cast<char*>(ws);
    uint32_t* thr = reinterpret_cast<uint32_t*>(base + w.off_thr);
    uint32_t* ghist = parallel_final ? reinterpret_cast<uint32_t*>(base + w.off_hist) : nullptr;
    const uint32_t sign_mask = take_abs ? 0x7fffffffu : 0xffffffffu;
    const int acc = (what & kSelAccumulate) ? 1 : 0;
    if (act_dtype == CI_F16)
      rc = launch_tokens<InF16>(act, B, M, N, ld, q_alpha, sign_mask, thr, ghist, counts, counts_stride, acc, nt, items,
                               nblocks, di.cus, s);
    else if (act_dtype == CI_BF16)
      rc = launch_tokens<InBF16>(act, B, M, N, ld, q_alpha, sign_mask, thr, ghist, counts, counts_stride, acc, nt, items,
                               nblocks, di.cus, s);
    else
      rc = launch_tokens<InF32>(act, B, M, N, ld, q_alpha, sign_mask, thr, ghist, counts, counts_stride, acc, nt, items,
                               nblocks, di.cus, s);
    if (rc != CI_OK) return rc;
    if (parallel_final) {
      const int cvec = (reinterpret_cast<uintptr_t>(counts) & 15u) == 0 ? 1 : 0;
      hipLaunchKernelGGL(def2_parallel_kernel, dim3(nblocks, B), dim3(1024), 0, s, counts, ghist, N, K, core_idx,
                         cvec && counts_stride % 4 == 0, counts_stride);
      CI_HIP_CHECK_LAUNCH();
      return CI_OK;
    }
  }
  if (!(what & kSelFinal)) return CI_OK;
  const int mc = (int)max_count;
#define CI_DEF2(I) launch_def2_single<I>(N, counts, K, core_idx, mc, s)
  if (items <= 4) return CI_DEF2(4);
  if (items <= 8) return CI_DEF2(8);
  if (items <= 16) return CI_DEF2(16);
  if (items <= 40) return CI_DEF2(40);  // up to 40 counts per thread in registers
  return CI_DEF2(0);
#undef CI_DEF2
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
