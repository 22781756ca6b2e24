// Union-batched decode: several sentences, each with its own frozen core set,
// decode one token each against the same resident weights (the large-model
// scenario of Sec. 5.3 of arXiv 2410.18311, extended to a batch).  Instead of
// fetching every sentence's rows separately, each row of the union of the core
// sets is read ONCE and applied to the sentences that own it (a bit mask per
// row).  The result per sentence is exactly its own sparse FFN (Sec. 4.2).
//
//   union_scatter / union_count / union_place : owner masks [N] -> ascending row list + masks + count
//   union_up_kernel   : partial dots of the up (and gate) rows with every owner's x,
//                       per column chunk -> hp[chunk][matrix][row][sentence]
//   union_down_kernel : h = act(sum of chunks [+ bias]) for the owners, then
//                       y_s += h[row][s] * W_down[row, :] -> partial[s][slice][d]
//   (decode_reduce_kernel of the single-sentence path sums the slices.)
//
// The number of union rows lives in device memory: the kernels slice the rows
// themselves, so no host synchronisation separates building the union from
// using it.
#include "common.hpp"
#include "decode_common.hpp"

namespace ci {

namespace {

constexpr int SB = 8;  // sentences per batch (bits of the owner mask that the kernels look at)
constexpr int kSuperMax = 256;  // most rows of a slice between two drains of the load ring

struct UnionArgs {
  const void* x;
  const void* w_up;
  const void* w_gate;
  const void* b_up;
  const void* w_down;
  const int32_t* uidx;
  const uint32_t* umask;
  const int32_t* ucount;
  float* hp;       // [c_up][NDOT][cap][SB]
  float* partial;  // [B][n_down][d]
  int B, d, N, cap, vecs;
  int vc;  // up phase: 16-byte vectors of a row per column chunk
  int n_up, c_up, n_down, c_down;
  int ks_up, ks_down;  // most rows of a slice handled between two drains of the load ring
};

__global__ void union_zero_kernel(uint32_t* owners, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) owners[i] = 0u;
}

// owners[n] |= 1 << s for every valid member n of sentence s's list
__global__ void union_scatter_kernel(const int32_t* __restrict__ core_idx, int64_t n_idx, int64_t K,
                                     int64_t N, uint32_t* __restrict__ owners) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_idx) return;
  const int n = core_idx[i];
  if (n >= 0 && n < N) atomicOr(&owners[n], 1u << (uint32_t)(i / K));
}

// Ordered compaction of the neurons with a non-empty owner mask, in two launches over blocks of 1024
// neurons: the number of owned neurons per block, then every block adds up the blocks before it and
// places its own neurons behind them (ascending, so the result does not depend on the scheduling).
constexpr int kUnionBlock = 1024;

__global__ __launch_bounds__(kUnionBlock) void union_count_kernel(const uint32_t* __restrict__ owners, int N,
                                                                  uint32_t* __restrict__ blkcnt) {
  __shared__ int wsum[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i = blockIdx.x * kUnionBlock + tid;
  const uint32_t m = i < N ? owners[i] : 0u;
  const uint64_t bal = __ballot(m != 0u);
  if (lane == 0) wsum[wave] = __popcll(bal);
  __syncthreads();
  if (tid == 0) {
    int t = 0;
    for (int w = 0; w < 16; ++w) t += wsum[w];
    blkcnt[blockIdx.x] = (uint32_t)t;
  }
}

__global__ __launch_bounds__(kUnionBlock) void union_place_kernel(const uint32_t* __restrict__ owners, int N,
                                                                  int cap, const uint32_t* __restrict__ blkcnt,
                                                                  int32_t* __restrict__ uidx,
                                                                  uint32_t* __restrict__ umask,
                                                                  int32_t* __restrict__ ucount) {
  __shared__ int wsum[16];
  __shared__ int bsum[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int blk = blockIdx.x;
  const int i = blk * kUnionBlock + tid;
  const uint32_t m = i < N ? owners[i] : 0u;
  const uint64_t bal = __ballot(m != 0u);
  const int before = __popcll(bal & lanemask_lt());
  if (lane == 0) wsum[wave] = __popcll(bal);
  // owned neurons in the blocks before mine (at most 1024 blocks: one per thread)
  int c = tid < blk ? (int)blkcnt[tid] : 0;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) c += __shfl_xor(c, off);
  if (lane == 0) bsum[wave] = c;
  __syncthreads();
  int base = 0, own = 0;
  for (int w = 0; w < 16; ++w) {
    base += bsum[w];
    own += wsum[w];
  }
  int off = base;
  for (int w = 0; w < wave; ++w) off += wsum[w];
  const int pos = off + before;
  if (m != 0u && pos < cap) {
    uidx[pos] = i;
    umask[pos] = m;
  }
  if (blk == (int)gridDim.x - 1 && tid == 0) {
    const int total = base + own;
    ucount[0] = total < cap ? total : cap;
  }
}

__device__ __forceinline__ int union_rows_clamped(const UnionArgs& a) {
  const int k = *a.ucount;
  return k < 0 ? 0 : (k > a.cap ? a.cap : k);
}

// Stages the weight row and owner mask of each row of a super-chunk in LDS.
// Rows whose index is out of range get mask 0 and read row 0.
__device__ __forceinline__ void union_stage(const UnionArgs& a, int row0, int Rs, int* sidx,
                                            uint32_t* smask) {
  for (int r = threadIdx.x; r < Rs; r += blockDim.x) {
    const int n = a.uidx[row0 + r];
    const bool ok = n >= 0 && n < a.N;
    sidx[r] = ok ? n : 0;
    smask[r] = ok ? (a.umask[row0 + r] & ((1u << a.B) - 1u)) : 0u;
  }
}

// ---- up phase ----------------------------------------------------------------
// dot of one 16-byte vector of weights with the matching 16 bytes of x, both in
// the element type: two-element dot instructions with fp32 accumulation for the
// 16-bit types (no conversions), plain FMAs for fp32.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

template <class D>
__device__ __forceinline__ float dot16(const uint4& w, const uint4& x, float acc);
template <>
__device__ __forceinline__ float dot16<F32>(const uint4& w, const uint4& x, float acc) {
  acc = fmaf(u2f(w.x), u2f(x.x), acc);
  acc = fmaf(u2f(w.y), u2f(x.y), acc);
  acc = fmaf(u2f(w.z), u2f(x.z), acc);
  return fmaf(u2f(w.w), u2f(x.w), acc);
}
template <>
__device__ __forceinline__ float dot16<F16>(const uint4& w, const uint4& x, float acc) {
  acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w.x), __builtin_bit_cast(half2_t, x.x), acc, false);
  acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w.y), __builtin_bit_cast(half2_t, x.y), acc, false);
  acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w.z), __builtin_bit_cast(half2_t, x.z), acc, false);
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w.w), __builtin_bit_cast(half2_t, x.w), acc, false);
}
template <>
__device__ __forceinline__ float dot16<BF16>(const uint4& w, const uint4& x, float acc) {
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.x), __builtin_bit_cast(bf16x2_t, x.x), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.y), __builtin_bit_cast(bf16x2_t, x.y), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.z), __builtin_bit_cast(bf16x2_t, x.z), acc, false);
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.w), __builtin_bit_cast(bf16x2_t, x.w), acc, false);
}

// One thread owns NI 16-byte column vectors of its chunk and keeps the matching
// x values of all sentences in registers (element type, 4 registers per vector).
// DEPTH rows are in flight per thread; every ring position issues its loads
// (filler positions from x), so the outstanding-load count is the same on
// every path.  One cross-lane reduction per row serves all NI vectors.
template <class T, int NI, bool SWIGLU>
__device__ __forceinline__ void union_up_issue(int pos, int Rs, int QB, const char* __restrict__ gate,
                                               const char* __restrict__ up,
                                               const char* __restrict__ filler, size_t rowbytes,
                                               const int* sidx, const uint32_t (&coff)[NI],
                                               uint4 (&dst)[NI]) {
  const bool valid = pos < QB;
  const bool second = SWIGLU && pos >= Rs;  // gate rows first, then up rows
  int r = second ? pos - Rs : pos;
  r = r > Rs - 1 ? Rs - 1 : r;
  const char* base = (SWIGLU && !second) ? gate : up;
  const char* prow = base + (size_t)sidx[r] * rowbytes;
  prow = valid ? prow : filler;
#pragma unroll
  for (int i = 0; i < NI; ++i) dst[i] = ld16_stream(prow + coff[i]);
}

template <class D, int NI, bool SWIGLU, int DEPTH>
__global__ __launch_bounds__(512) void union_up_kernel(UnionArgs a) {
  using T = typename D::T;
  constexpr int NDOT = SWIGLU ? 2 : 1;

  extern __shared__ float smem[];
  const int tid = threadIdx.x, nt = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
  const int slice = blockIdx.x, chunk = blockIdx.y;
  const int Ku = union_rows_clamped(a);
  const int r0 = (int)(((int64_t)slice * Ku) / a.n_up);
  const int r1 = (int)(((int64_t)(slice + 1) * Ku) / a.n_up);
  const int R = r1 - r0;

  const int ks = a.ks_up;
  float* red = smem;                                              // [nw][NDOT * ks][SB]
  int* sidx = reinterpret_cast<int*>(red + nw * NDOT * ks * SB);  // [ks]
  uint32_t* smask = reinterpret_cast<uint32_t*>(sidx + ks);       // [ks]

  const size_t rowbytes = (size_t)a.d * sizeof(T);
  const char* up = reinterpret_cast<const char*>(a.w_up);
  const char* gate = reinterpret_cast<const char*>(a.w_gate);
  const char* xbase = reinterpret_cast<const char*>(a.x);

  // vectors [chunk * vc, (chunk + 1) * vc) of a row belong to this chunk
  uint32_t coff[NI];
  uint4 xq[SB][NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int local = i * nt + tid;
    const int vec = chunk * a.vc + local;
    const bool cv = local < a.vc && vec < a.vecs;
    // a column past the end re-reads column 0 with x = 0, so every load is unconditional
    coff[i] = cv ? (uint32_t)vec * 16u : 0u;
#pragma unroll
    for (int t = 0; t < SB; ++t) {
      xq[t][i] = (t < a.B && cv) ? ld16(xbase + (size_t)t * rowbytes + coff[i]) : make_uint4(0u, 0u, 0u, 0u);
    }
  }

  // super-chunks of equal size (a short last one would pay a full drain and refill of the ring)
  const int nsc = (R + ks - 1) / ks;
  const int step = nsc > 0 ? (R + nsc - 1) / nsc : 1;
  for (int s0 = 0; s0 < R; s0 += step) {
    const int Rs = min(step, R - s0);
    const int QB = NDOT * Rs;
    const int QBp = (QB + DEPTH - 1) / DEPTH * DEPTH;
    __syncthreads();  // previous super-chunk done with sidx / smask / red
    union_stage(a, r0 + s0, Rs, sidx, smask);
    __syncthreads();

    uint4 buf[DEPTH][NI];
#define CI_UISSUE(pos, slot) \
  union_up_issue<T, NI, SWIGLU>((pos), Rs, QB, gate, up, xbase, rowbytes, sidx, coff, buf[slot])
#pragma unroll
    for (int s = 0; s < DEPTH; ++s) {
      CI_UISSUE(s, s);
      __builtin_amdgcn_sched_barrier(0);
    }

    for (int g0 = 0; g0 < QBp; g0 += DEPTH) {
#pragma unroll
      for (int s = 0; s < DEPTH; ++s) {
        const int pos = g0 + s;
        int r = (SWIGLU && pos >= Rs) ? pos - Rs : pos;
        r = r > Rs - 1 ? Rs - 1 : r;
        const uint32_t m = __builtin_amdgcn_readfirstlane(pos < QB ? smask[r] : 0u);
        float p[SB];
#pragma unroll
        for (int t = 0; t < SB; ++t) {
          float sum = 0.f;
          if (m & (1u << t)) {  // uniform: only the owners' dots are computed
#pragma unroll
            for (int i = 0; i < NI; ++i) sum = dot16<D>(buf[s][i], xq[t][i], sum);
          }
          p[t] = sum;
        }
        // refill the slot as soon as it has been consumed
        __builtin_amdgcn_sched_barrier(0);
        CI_UISSUE(pos + DEPTH, s);
        __builtin_amdgcn_sched_barrier(0);
        halve_rows<SB, 32>(p, lane);  // lanes 8t .. 8t+7 now hold sentence t's wave sum
        if ((lane & 7) == 0 && pos < QB) red[((wave * NDOT * ks) + pos) * SB + (lane >> 3)] = p[0];
      }
    }
    // filler loads issued past the end are still outstanding
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
#undef CI_UISSUE
    // sum over the waves; gate rows are matrix 0, up rows matrix 1 (SwiGLU), else matrix 0
    for (int o = tid; o < QB * SB; o += nt) {
      const int q = o / SB, t = o % SB;
      float z = 0.f;
      for (int w = 0; w < nw; ++w) z += red[((w * NDOT * ks) + q) * SB + t];
      const int mat = (SWIGLU && q >= Rs) ? 1 : 0;
      const int r = q - mat * Rs;
      a.hp[(((size_t)chunk * NDOT + mat) * a.cap + (size_t)(r0 + s0 + r)) * SB + t] = z;
    }
  }
}

// ---- down phase ----------------------------------------------------------------
__device__ __forceinline__ uint4 union_down_issue(int pos, int Rs, const char* __restrict__ down,
                                                  const char* __restrict__ filler, size_t rowbytes,
                                                  const int* sidx, uint32_t coff) {
  const int r = pos > Rs - 1 ? Rs - 1 : pos;
  const char* prow = down + (size_t)sidx[r] * rowbytes;
  prow = pos < Rs ? prow : filler;
  return ld16_stream(prow + coff);
}

template <class D, bool SWIGLU, int DEPTH>
__global__ __launch_bounds__(512) void union_down_kernel(UnionArgs a) {
  using T = typename D::T;
  constexpr int VEC = D::VEC;
  constexpr int NDOT = SWIGLU ? 2 : 1;

  __shared__ float hbuf[kSuperMax * SB];
  __shared__ int sidx[kSuperMax];
  __shared__ uint32_t smask[kSuperMax];
  const int tid = threadIdx.x, nt = blockDim.x;
  const int slice = blockIdx.x, chunk = blockIdx.y;
  const int Ku = union_rows_clamped(a);
  const int r0 = (int)(((int64_t)slice * Ku) / a.n_down);
  const int r1 = (int)(((int64_t)(slice + 1) * Ku) / a.n_down);
  const int R = r1 - r0;

  const size_t rowbytes = (size_t)a.d * sizeof(T);
  const char* down = reinterpret_cast<const char*>(a.w_down);
  const char* filler = reinterpret_cast<const char*>(a.x);
  const int vec = chunk * nt + tid;
  const bool cv = vec < a.vecs;
  const uint32_t coff = cv ? (uint32_t)vec * 16u : 0u;

  float acc[SB][VEC];
#pragma unroll
  for (int t = 0; t < SB; ++t)
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[t][v] = 0.f;

  const int nsc = (R + a.ks_down - 1) / a.ks_down;
  const int step = nsc > 0 ? (R + nsc - 1) / nsc : 1;
  for (int s0 = 0; s0 < R; s0 += step) {
    const int Rs = min(step, R - s0);
    const int QBp = (Rs + DEPTH - 1) / DEPTH * DEPTH;
    __syncthreads();  // previous super-chunk done with hbuf / sidx / smask
    union_stage(a, r0 + s0, Rs, sidx, smask);
    // hidden value of (row, sentence): sum of the column chunks' partial dots
    for (int o = tid; o < Rs * SB; o += nt) {
      const int r = o / SB, t = o % SB;
      const size_t u = (size_t)(r0 + s0 + r);
      const int n = a.uidx[u];
      const bool ok = n >= 0 && n < a.N && t < a.B && ((a.umask[u] >> t) & 1u);
      float z0 = 0.f, z1 = 0.f;
      for (int c = 0; c < a.c_up; ++c) {
        z0 += a.hp[(((size_t)c * NDOT) * a.cap + u) * SB + t];
        if (SWIGLU) z1 += a.hp[(((size_t)c * NDOT + 1) * a.cap + u) * SB + t];
      }
      float h;
      if (SWIGLU) h = silu(z0) * z1;  // z0: gate, z1: up
      else {
        const float bias = (a.b_up && ok) ? to_float<D>(reinterpret_cast<const T*>(a.b_up)[n]) : 0.f;
        h = fmaxf(z0 + bias, 0.f);
      }
      hbuf[o] = ok ? h : 0.f;
    }
    __syncthreads();

    uint4 buf[DEPTH];
#define CI_DISSUE(pos) union_down_issue((pos), Rs, down, filler, rowbytes, sidx, coff)
#pragma unroll
    for (int s = 0; s < DEPTH; ++s) {
      buf[s] = CI_DISSUE(s);
      __builtin_amdgcn_sched_barrier(0);
    }
    for (int g0 = 0; g0 < QBp; g0 += DEPTH) {
#pragma unroll
      for (int s = 0; s < DEPTH; ++s) {
        const int pos = g0 + s;
        const int r = pos > Rs - 1 ? Rs - 1 : pos;
        const uint32_t m = __builtin_amdgcn_readfirstlane(pos < Rs ? smask[r] : 0u);
        float f[VEC];
        unpack<D>(buf[s], f);
        __builtin_amdgcn_sched_barrier(0);
        buf[s] = CI_DISSUE(pos + DEPTH);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < SB; ++t) {
          if (m & (1u << t)) {  // uniform
            const float hj = hbuf[r * SB + t];
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[t][v] = fmaf(hj, f[v], acc[t][v]);
          }
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
#undef CI_DISSUE
  }

  if (cv) {
    const int col = vec * VEC;
    typedef float f32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int t = 0; t < SB; ++t) {
      if (t < a.B) {
        float* out = a.partial + ((size_t)t * a.n_down + slice) * a.d + col;
#pragma unroll
        for (int v = 0; v < VEC; v += 4) {
          const f32x4 o = {acc[t][v], acc[t][v + 1], acc[t][v + 2], acc[t][v + 3]};
          __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(out + v));
        }
      }
    }
  }
}

inline size_t union_up_lds(int t_up, int ndot, int ks) {
  return (size_t)(t_up / 64) * ndot * ks * SB * sizeof(float) + 2 * (size_t)ks * sizeof(int);
}

template <class D, int NI, bool SWIGLU>
void launch_union_up(const UnionArgs& a, int t_up, hipStream_t s) {
  constexpr int NDOT = SWIGLU ? 2 : 1;
  const size_t lds = union_up_lds(t_up, NDOT, a.ks_up);
  const dim3 g(a.n_up, a.c_up);
  // about 16 loads in flight per thread
  if constexpr (NI >= 3) hipLaunchKernelGGL((union_up_kernel<D, NI, SWIGLU, 4>), g, dim3(t_up), lds, s, a);
  else if constexpr (NI == 2) hipLaunchKernelGGL((union_up_kernel<D, NI, SWIGLU, 8>), g, dim3(t_up), lds, s, a);
  else hipLaunchKernelGGL((union_up_kernel<D, NI, SWIGLU, 16>), g, dim3(t_up), lds, s, a);
}

template <class D, bool SWIGLU>
int launch_union_typed(const UnionArgs& a, int ni, int t_up, int t_down, hipStream_t s) {
  switch (ni) {
    case 1: launch_union_up<D, 1, SWIGLU>(a, t_up, s); break;
    case 2: launch_union_up<D, 2, SWIGLU>(a, t_up, s); break;
    case 3: launch_union_up<D, 3, SWIGLU>(a, t_up, s); break;
    case 4: launch_union_up<D, 4, SWIGLU>(a, t_up, s); break;
    default: return CI_ERR_UNSUPPORTED;
  }
  const dim3 gd(a.n_down, a.c_down);
  if (params().union_depth == 16)
    hipLaunchKernelGGL((union_down_kernel<D, SWIGLU, 16>), gd, dim3(t_down), 0, s, a);
  else
    hipLaunchKernelGGL((union_down_kernel<D, SWIGLU, 8>), gd, dim3(t_down), 0, s, a);
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

}  // namespace

// Column chunks of the up phase for a row of `vecs` 16-byte vectors (a
// workgroup covers at most 512 threads x 4 vectors); part of the workspace layout.
int union_up_chunks(int64_t vecs) { return (int)((vecs + 2047) / 2048); }

int launch_union_build(const int32_t* core_idx, int64_t B, int64_t K, int64_t N, int64_t cap,
                       int32_t* uidx, uint32_t* umask, int32_t* ucount, uint32_t* owners,
                       hipStream_t s) {
  hipLaunchKernelGGL(union_zero_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, s, owners, N);
  const int64_t n_idx = B * K;
  if (n_idx > 0)
    hipLaunchKernelGGL(union_scatter_kernel, dim3((unsigned)((n_idx + 255) / 256)), dim3(256), 0, s,
                       core_idx, n_idx, K, N, owners);
  const unsigned nblk = (unsigned)((N + kUnionBlock - 1) / kUnionBlock);  // <= 1024: N <= CI_MAX_NEURONS
  uint32_t* blkcnt = owners + (N + 63) / 64 * 64;
  hipLaunchKernelGGL(union_count_kernel, dim3(nblk), dim3(kUnionBlock), 0, s, owners, (int)N, blkcnt);
  hipLaunchKernelGGL(union_place_kernel, dim3(nblk), dim3(kUnionBlock), 0, s, owners, (int)N, (int)cap, blkcnt, uidx,
                     umask, ucount);
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

int launch_ffn_decode_union(const void* x, int64_t B, const ci_ffn_weights* w, const int32_t* uidx,
                            const uint32_t* umask, const int32_t* ucount, int64_t cap, int dtype,
                            int act, void* y, float* ws, hipStream_t s) {
  UnionArgs a;
  a.x = x;
  a.w_up = w->w_up;
  a.w_gate = w->w_gate;
  a.b_up = w->b_up;
  a.w_down = w->w_down;
  a.uidx = uidx;
  a.umask = umask;
  a.ucount = ucount;
  a.B = (int)B;
  a.d = (int)w->d;
  a.N = (int)w->N;
  a.cap = (int)cap;
  a.vecs = (int)(w->d / (dtype == CI_F32 ? 4 : 8));
  const int ndot = act == CI_ACT_SWIGLU ? 2 : 1;

  DeviceInfo di;
  int cus = 256;
  if (device_info(&di) == CI_OK) cus = di.cus;
  a.c_up = union_up_chunks(a.vecs);
  a.vc = (a.vecs + a.c_up - 1) / a.c_up;
  // vectors per thread: the choice that pads the chunk least, the larger one on ties (one
  // cross-lane reduction per row serves all of a thread's vectors)
  int ni = 1, t_up = 512, waste = 1 << 30;
  for (int n = 4; n >= 1; --n) {
    const int t = ((a.vc + n - 1) / n + 63) / 64 * 64;
    if (t > 512) continue;
    if (t * n - a.vc < waste) { waste = t * n - a.vc; ni = n; t_up = t; }
  }
  // down phase: column chunks of about union_down_threads vectors, evenly sized
  int want = params().union_down_threads;
  if (want < 64) want = 64;
  if (want > 512) want = 512;
  a.c_down = (a.vecs + want - 1) / want;
  const int t_down = ((a.vecs + a.c_down - 1) / a.c_down + 63) / 64 * 64;
  a.c_down = (a.vecs + t_down - 1) / t_down;
  a.n_up = cus * params().union_up_wgs_per_cu / a.c_up;
  a.n_down = cus * params().union_down_wgs_per_cu / a.c_down;
  if (a.n_up > 1024) a.n_up = 1024;
  if (a.n_down > 256) a.n_down = 256;  // bounds the partial sums of the workspace
  if (a.n_up > a.cap) a.n_up = a.cap;
  if (a.n_down > a.cap) a.n_down = a.cap;
  if (a.n_up < 1) a.n_up = 1;
  if (a.n_down < 1) a.n_down = 1;

  // rows between two drains: as many as 64 KB of LDS hold (wave sums of the up phase)
  a.ks_up = kSuperMax;
  while (a.ks_up > 64 && union_up_lds(t_up, ndot, a.ks_up) > 65536) a.ks_up >>= 1;
  a.ks_down = kSuperMax;
  const int ks_cap = params().union_super;
  if (ks_cap > 0) {
    if (a.ks_up > ks_cap) a.ks_up = ks_cap;
    if (a.ks_down > ks_cap) a.ks_down = ks_cap;
  }

  a.hp = ws;
  const size_t hp_floats = ((size_t)a.c_up * ndot * (size_t)a.cap * SB + 63) / 64 * 64;
  a.partial = ws + hp_floats;

  int rc;
  const bool sw = act == CI_ACT_SWIGLU;
  switch (dtype) {
    case CI_F32: rc = sw ? launch_union_typed<F32, true>(a, ni, t_up, t_down, s) : launch_union_typed<F32, false>(a, ni, t_up, t_down, s); break;
    case CI_F16: rc = sw ? launch_union_typed<F16, true>(a, ni, t_up, t_down, s) : launch_union_typed<F16, false>(a, ni, t_up, t_down, s); break;
    case CI_BF16: rc = sw ? launch_union_typed<BF16, true>(a, ni, t_up, t_down, s) : launch_union_typed<BF16, false>(a, ni, t_up, t_down, s); break;
    default: return CI_ERR_BAD_DTYPE;
  }
  if (rc != CI_OK) return rc;
  return launch_decode_reduce(a.partial, w->b_down, y, a.n_down, a.d, (int)B, dtype, s);
}

}  // namespace ci
