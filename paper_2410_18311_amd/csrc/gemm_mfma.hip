// Dense prefill FFN (Def. 1 of arXiv 2410.18311: the activation vector A(x)
// of every prompt token) -- the one real dense contraction of the path, so it
// runs on the matrix cores.
//
//   C[M, Nn] = A[M, Kk] * B^T   with B given as [Nn, Kk] (both operands
//   k-contiguous, the nn.Linear layout) or, for a neuron-major down matrix, as
//   [Kk, Nn].
//
// gemm_mfma_kernel (fp16 / bf16): 128x128x64 workgroup tiles, 256 threads =
// 2x2 waves, each wave a 64x64 sub-tile as 2x2 v_mfma_f32_32x32x16 tiles with
// fp32 accumulators.  Global -> register -> LDS staging with two LDS buffers,
// so the next tile's global loads are in flight during the MFMAs.  The
// epilogue is fused: bias + ReLU, or SiLU(gate)*up from two accumulator sets,
// writing the fp32 score matrix and/or the element-type hidden matrix; or
// bias + convert for the down projection.
// gemm_f32_kernel: plain fp32 FMA tiles for the fp32 element type.
#include "common.hpp"

namespace ci {

namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

enum { EPI_RELU = 0, EPI_SWIGLU = 1, EPI_LINEAR = 2 };

struct GemmArgs {
  const void* A;
  const void* B0;  // EPI_SWIGLU: gate
  const void* B1;  // EPI_SWIGLU: up
  const void* bias;
  void* out_e;     // [M, Nn] element type, may be null
  float* out_f;    // [M, Nn] fp32, may be null
  int64_t lda, ldb, ldo;
  int M, Nn, Kk;
  int k_chunk;     // k range handled by one workgroup along blockIdx.y (a multiple of the k tile)
  float* partial;  // split-K only: [gridDim.y][M][Nn] fp32 partial products (epilogue skipped)
};

template <class D>
__device__ __forceinline__ f32x16 mfma32(const uint4& a, const uint4& b, f32x16 c);
template <>
__device__ __forceinline__ f32x16 mfma32<F16>(const uint4& a, const uint4& b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
template <>
__device__ __forceinline__ f32x16 mfma32<BF16>(const uint4& a, const uint4& b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDK = BK + 8;  // LDS row stride in elements (144 bytes)

// Spreads consecutive tiles over one XCD (workgroup ids go round-robin over the
// 8 XCDs, each with its own L2), so that tiles sharing a B panel share an L2.
__device__ __forceinline__ int xcd_swizzle(int id, int n) {
  if (n % 8 != 0) return id;
  return (id % 8) * (n / 8) + id / 8;
}

// Fused epilogue shared by the two MFMA kernels.  Accumulator element v of lane
// l is C[row, col] with col = l % 32, row = 8 * (v / 4) + 4 * (l / 32) + v % 4
// inside a 32x32 tile.
template <class D, int EPI>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& g, f32x16 (&acc)[EPI == EPI_SWIGLU ? 2 : 1][2][2],
                                              int m0, int n0, int wm, int wn, int lane) {
  using T = typename D::T;
  constexpr int NB = (EPI == EPI_SWIGLU) ? 2 : 1;
  if (g.partial) {  // split-K: raw fp32 partial products, reduced by splitk_reduce_kernel
    float* part = g.partial + (size_t)blockIdx.y * g.M * g.Nn;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col = n0 + wn * 64 + j * 32 + (lane & 31);
      if (col >= g.Nn) continue;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = m0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          if (row < g.M) part[(size_t)row * g.Nn + col] = acc[0][i][j][v];
        }
    }
    return;
  }
  const T* bias = reinterpret_cast<const T*>(g.bias);
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int col = n0 + wn * 64 + j * 32 + (lane & 31);
    if (col >= g.Nn) continue;
    const float bv = bias ? to_float<D>(bias[col]) : 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (row >= g.M) continue;
        float h, score;
        if (EPI == EPI_SWIGLU) {
          h = silu(acc[0][i][j][v]) * acc[NB - 1][i][j][v];
          score = fabsf(h);
        } else if (EPI == EPI_RELU) {
          h = fmaxf(acc[0][i][j][v] + bv, 0.f);
          score = h;
        } else {
          h = acc[0][i][j][v] + bv;
          score = h;
        }
        const size_t o = (size_t)row * g.ldo + col;
        if (g.out_f) g.out_f[o] = score;
        if (g.out_e) reinterpret_cast<T*>(g.out_e)[o] = from_float<D>(h);
      }
    }
  }
}

template <class D, int EPI, bool BNN>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmArgs g) {
  using T = typename D::T;
  constexpr bool DUAL = (EPI == EPI_SWIGLU);
  constexpr int NB = DUAL ? 2 : 1;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* smem = reinterpret_cast<T*>(smem_raw);
  // per stage: A tile, then NB B tiles
  constexpr int TILE = BM * LDK;
  constexpr int STAGE = TILE * (1 + NB);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int tiles_m = (g.M + BM - 1) / BM;
  const int t = xcd_swizzle(blockIdx.x, gridDim.x);
  const int m0 = (t % tiles_m) * BM, n0 = (t / tiles_m) * BN;
  const T* A = reinterpret_cast<const T*>(g.A);
  const T* Bp[2] = {reinterpret_cast<const T*>(g.B0), reinterpret_cast<const T*>(g.B1)};

  uint4 ra[4], rb[NB][4];
  auto load_global = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int v = tid + 256 * i;
      {
        const int row = v >> 3, kc = (v & 7) * 8;
        ra[i] = make_uint4(0, 0, 0, 0);
        if (m0 + row < g.M && k0 + kc < g.Kk) ra[i] = ld16(A + (size_t)(m0 + row) * g.lda + k0 + kc);
      }
#pragma unroll
      for (int q = 0; q < NB; ++q) {
        rb[q][i] = make_uint4(0, 0, 0, 0);
        if (!BNN) {
          const int row = v >> 3, kc = (v & 7) * 8;
          if (n0 + row < g.Nn && k0 + kc < g.Kk)
            rb[q][i] = ld16(Bp[q] + (size_t)(n0 + row) * g.ldb + k0 + kc);
        } else {
          const int krow = v >> 4, nc = (v & 15) * 8;
          if (k0 + krow < g.Kk && n0 + nc < g.Nn)
            rb[q][i] = ld16(Bp[q] + (size_t)(k0 + krow) * g.ldb + n0 + nc);
        }
      }
    }
  };
  auto store_lds = [&](int stage) {
    T* sA = smem + stage * STAGE;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int v = tid + 256 * i;
      const int row = v >> 3, kc = (v & 7) * 8;
      *reinterpret_cast<uint4*>(sA + row * LDK + kc) = ra[i];
#pragma unroll
      for (int q = 0; q < NB; ++q) {
        T* sB = sA + TILE * (1 + q);
        if (!BNN) {
          *reinterpret_cast<uint4*>(sB + row * LDK + kc) = rb[q][i];
        } else {
          const int krow = v >> 4, nc = (v & 15) * 8;
          const uint32_t w[4] = {rb[q][i].x, rb[q][i].y, rb[q][i].z, rb[q][i].w};
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const uint16_t bits = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
            reinterpret_cast<uint16_t*>(sB)[(nc + e) * LDK + krow] = bits;
          }
        }
      }
    }
  };

  f32x16 acc[NB][2][2];
#pragma unroll
  for (int q = 0; q < NB; ++q)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[q][i][j][v] = 0.f;

  const int k_begin = blockIdx.y * g.k_chunk;
  const int k_end = min(g.Kk, k_begin + g.k_chunk);
  const int nk = (k_end - k_begin + BK - 1) / BK;
  load_global(k_begin);
  store_lds(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) load_global(k_begin + (kt + 1) * BK);
    const T* sA = smem + cur * STAGE;
#pragma unroll
    for (int s = 0; s < BK / 16; ++s) {
      const int koff = s * 16 + (lane >> 5) * 8;
      uint4 fa[2], fb[NB][2];
#pragma unroll
      for (int i = 0; i < 2; ++i)
        fa[i] = *reinterpret_cast<const uint4*>(sA + (wm * 64 + i * 32 + (lane & 31)) * LDK + koff);
#pragma unroll
      for (int q = 0; q < NB; ++q)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          fb[q][j] = *reinterpret_cast<const uint4*>(sA + TILE * (1 + q) +
                                                     (wn * 64 + j * 32 + (lane & 31)) * LDK + koff);
#pragma unroll
      for (int q = 0; q < NB; ++q)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[q][i][j] = mfma32<D>(fa[i], fb[q][j], acc[q][i][j]);
    }
    if (kt + 1 < nk) {
      store_lds(cur ^ 1);  // the other buffer: last read before the previous barrier
      __syncthreads();
    }
  }

  gemm_epilogue<D, EPI>(g, acc, m0, n0, wm, wn, lane);
}

// ---------------------------------------------------------------------------
// Fast path of the kernel above for k-contiguous B and a reduction length that
// is a multiple of the k tile: the global loads of the next RD k-tiles are kept
// in flight in a register ring (a tile is written to LDS only when it is about
// to be used), because one k-tile of MFMA work (~0.4 us) is far shorter than a
// memory round trip.  Every load is unconditional (rows past the edge are
// clamped: they only feed outputs that are never stored), so the number of
// outstanding loads is the same on every path and the waits are exact.
template <class D, int EPI, int RD, bool GUARD>  // RD: k-tiles in flight per thread; GUARD: nk % RD != 0 allowed
__global__ __launch_bounds__(256) void gemm_mfma_ring_kernel(GemmArgs g) {
  using T = typename D::T;
  constexpr bool DUAL = (EPI == EPI_SWIGLU);
  constexpr int NB = DUAL ? 2 : 1;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* smem = reinterpret_cast<T*>(smem_raw);
  constexpr int TILE = BM * LDK;
  constexpr int STAGE = TILE * (1 + NB);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int tiles_m = (g.M + BM - 1) / BM;
  const int t = xcd_swizzle(blockIdx.x, gridDim.x);
  const int m0 = (t % tiles_m) * BM, n0 = (t / tiles_m) * BN;
  const int k_begin = blockIdx.y * g.k_chunk;
  const int k_end = min(g.Kk, k_begin + g.k_chunk);
  const int nk = (k_end - k_begin) / BK;

  const T* pa[4];
  const T* pb[NB][4];
  int lds_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v = tid + 256 * i;
    const int row = v >> 3, kc = (v & 7) * 8;
    lds_off[i] = row * LDK + kc;
    pa[i] = reinterpret_cast<const T*>(g.A) + (size_t)min(m0 + row, g.M - 1) * g.lda + k_begin + kc;
    pb[0][i] = reinterpret_cast<const T*>(g.B0) + (size_t)min(n0 + row, g.Nn - 1) * g.ldb + k_begin + kc;
    if (DUAL) pb[NB - 1][i] = reinterpret_cast<const T*>(g.B1) + (size_t)min(n0 + row, g.Nn - 1) * g.ldb + k_begin + kc;
  }

  uint4 ra[RD][4], rb[RD][NB][4];
#define CI_GEMM_ISSUE(slot, tile)                                   \
  do {                                                              \
    const int kk_ = min((tile), nk - 1) * BK;                       \
    _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_) {              \
      ra[slot][i_] = ld16(pa[i_] + kk_);                            \
      _Pragma("unroll") for (int q_ = 0; q_ < NB; ++q_)             \
        rb[slot][q_][i_] = ld16(pb[q_][i_] + kk_);                  \
    }                                                               \
  } while (0)

  f32x16 acc[NB][2][2];
#pragma unroll
  for (int q = 0; q < NB; ++q)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[q][i][j][v] = 0.f;

#pragma unroll
  for (int r = 0; r < RD; ++r) {
    CI_GEMM_ISSUE(r, r);
    __builtin_amdgcn_sched_barrier(0);  // oldest tile first: the waits below count on this order
  }
  // tile 0: registers -> LDS stage 0, slot 0 refilled with tile RD
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    *reinterpret_cast<uint4*>(smem + lds_off[i]) = ra[0][i];
#pragma unroll
    for (int q = 0; q < NB; ++q) *reinterpret_cast<uint4*>(smem + TILE * (1 + q) + lds_off[i]) = rb[0][q][i];
  }
  __builtin_amdgcn_sched_barrier(0);
  CI_GEMM_ISSUE(0, RD);
  __builtin_amdgcn_sched_barrier(0);
  __syncthreads();

  // Software pipeline: while tile kt is multiplied out of one LDS stage, tile kt + 1 moves from its
  // register slot into the other stage and the slot is refilled with tile kt + 1 + RD -- a third of
  // the stores and loads in each of the first three MFMA k-steps.  The fragments of k-step s + 1
  // are read while k-step s is multiplied (two register sets), so a wave never waits for the LDS
  // read it has just issued; the one barrier per k-tile sits before the last k-step, whose MFMAs
  // cover the first fragment reads of the next tile.
  const int l31 = lane & 31, khalf = (lane >> 5) * 8;
  uint4 fa[2][2], fb[2][NB][2];
#define CI_RING_FRAGS(buf, base, s)                                                                 \
  do {                                                                                              \
    _Pragma("unroll") for (int i_ = 0; i_ < 2; ++i_)                                                \
      fa[buf][i_] = *reinterpret_cast<const uint4*>((base) + (wm * 64 + i_ * 32 + l31) * LDK + (s) * 16 + khalf); \
    _Pragma("unroll") for (int q_ = 0; q_ < NB; ++q_)                                               \
      _Pragma("unroll") for (int j_ = 0; j_ < 2; ++j_)                                              \
        fb[buf][q_][j_] = *reinterpret_cast<const uint4*>((base) + TILE * (1 + q_) +                \
                                                          (wn * 64 + j_ * 32 + l31) * LDK + (s) * 16 + khalf); \
  } while (0)
  CI_RING_FRAGS(0, smem, 0);

  constexpr int NP = 4 + 4 * NB;                                  // 16-byte pieces per thread and k-tile
  constexpr int kPieceLo[4] = {0, (NP + 2) / 3, (2 * NP + 2) / 3, NP};  // 3 + 3 + 2, or 4 + 4 + 4
  for (int kt0 = 0; kt0 < nk; kt0 += RD) {
#pragma unroll
    for (int r = 0; r < RD; ++r) {
      const int kt = kt0 + r;
      const int rn = (r + 1) % RD;  // slot of tile kt + 1
      const T* sA = smem + (kt & 1) * STAGE;
      T* sN = smem + ((kt + 1) & 1) * STAGE;  // last read before the barrier inside tile kt - 1
      const int kk_next = min(kt + 1 + RD, nk - 1) * BK;
#pragma unroll
      for (int s = 0; s < BK / 16; ++s) {
        if (s == BK / 16 - 1) {
          // every wave has read all fragments of this tile and stored its share of the next one
          __syncthreads();
          CI_RING_FRAGS(0, sN, 0);
        } else {
          CI_RING_FRAGS((s + 1) & 1, sA, s + 1);
#pragma unroll
          for (int p = 0; p < NP; ++p) {
            if (p < kPieceLo[s] || p >= kPieceLo[s + 1]) continue;
            if (p < 4) {
              *reinterpret_cast<uint4*>(sN + lds_off[p]) = ra[rn][p];
              ra[rn][p] = ld16(pa[p] + kk_next);
            } else {
              const int q = (p - 4) >> 2, i = (p - 4) & 3;
              *reinterpret_cast<uint4*>(sN + TILE * (1 + q) + lds_off[i]) = rb[rn][q][i];
              rb[rn][q][i] = ld16(pb[q][i] + kk_next);
            }
          }
        }
        if (!GUARD || kt < nk) {  // padding iterations (nk not a multiple of RD) skip the arithmetic only
#pragma unroll
          for (int q = 0; q < NB; ++q)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
              for (int j = 0; j < 2; ++j) acc[q][i][j] = mfma32<D>(fa[s & 1][i], fb[s & 1][q][j], acc[q][i][j]);
        }
        // one LDS or global instruction after each MFMA rather than a burst of them before the first
#pragma unroll
        for (int m = 0; m < 4 * NB; ++m) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // LDS read
          __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);  // LDS write
          __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // global load
        }
        __builtin_amdgcn_sched_barrier(0);  // keeps the k-steps (and with them the load order) apart
      }
    }
  }
#undef CI_RING_FRAGS
#undef CI_GEMM_ISSUE

  gemm_epilogue<D, EPI>(g, acc, m0, n0, wm, wn, lane);
}

// ---------------------------------------------------------------------------
// The same 128 x 128 tile with the operand tiles copied from global memory
// straight into LDS (global_load_lds_dwordx4: every lane names its own 16 source
// bytes, and the 64 pieces of a wave instruction land next to each other in
// LDS), so that no register ring, no staging store and no wait for a load sits
// in a wave's instruction stream: the k-tiles in flight live in LDS stages
// (four of 32 KB; three of 48 KB for SwiGLU), and a wave only waits, once per
// k-tile and just before the barrier, until the tile after the current one has
// landed.  As the destination cannot be padded, a tile row is 128 bytes and its
// eight 16-byte chunks are stored permuted -- chunk j of row r at position
// j ^ ((r / 2) & 7), chosen on the global side.  LDS has 64 banks of 4 bytes:
// even and odd rows lie in different halves of them, and the 16 lanes that a
// 16-byte fragment read serves per clock (16 neighbouring rows, one chunk
// each) then hit eight different positions in either half: every bank once.
// The stages are separate LDS arrays, and the waits are written out by hand:
// loads retire in order, so "at most 8 (S - 2) of my loads outstanding" means
// that every k-tile up to the next one is complete.
#define CI_GLOBAL_PTR(p) ((const void __attribute__((address_space(1)))*)(p))
#define CI_LDS_PTR(p) ((void __attribute__((address_space(3)))*)(p))
template <class D, int EPI, bool GUARD>  // GUARD: the k-tile count need not be a multiple of the stage count
__global__ __launch_bounds__(256) void gemm_mfma_direct_kernel(GemmArgs g) {
  using T = typename D::T;
  constexpr bool DUAL = (EPI == EPI_SWIGLU);
  constexpr int NB = DUAL ? 2 : 1;
  constexpr int S = DUAL ? 3 : 4;                 // LDS stages
  constexpr int TILE_B = BM * BK * 2;             // bytes of one operand tile: 128 rows of 128 bytes
  constexpr int STAGE_B = TILE_B * (1 + NB);
  constexpr int NP = 4 * (1 + NB);                // 16-byte pieces per thread and k-tile
  __shared__ __attribute__((aligned(1024))) unsigned char st0[STAGE_B], st1[STAGE_B], st2[STAGE_B], st3[DUAL ? 16 : STAGE_B];
  unsigned char* const st[4] = {st0, st1, st2, st3};

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int tiles_m = (g.M + BM - 1) / BM;
  const int t = xcd_swizzle(blockIdx.x, gridDim.x);
  const int m0 = (t % tiles_m) * BM, n0 = (t / tiles_m) * BN;
  const int k_begin = blockIdx.y * g.k_chunk;
  const int k_end = min(g.Kk, k_begin + g.k_chunk);
  const int nk = (k_end - k_begin) / BK;

  // piece i of this thread: rows 32 i + 8 wave + lane / 8 of every operand tile; the lane's chunk
  // position lane % 8 holds chunk (lane % 8) ^ ((row / 2) % 8).  Rows past the edge are clamped: they
  // only feed outputs that are never stored.
  const T* pa[4];
  const T* pb[NB][4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = 32 * i + 8 * wave + (lane >> 3);
    const int chunk = (lane & 7) ^ ((row >> 1) & 7);
    pa[i] = reinterpret_cast<const T*>(g.A) + (size_t)min(m0 + row, g.M - 1) * g.lda + k_begin + chunk * 8;
    pb[0][i] = reinterpret_cast<const T*>(g.B0) + (size_t)min(n0 + row, g.Nn - 1) * g.ldb + k_begin + chunk * 8;
    if (DUAL) pb[NB - 1][i] = reinterpret_cast<const T*>(g.B1) + (size_t)min(n0 + row, g.Nn - 1) * g.ldb + k_begin + chunk * 8;
  }
  // piece p (0 .. NP-1) of k-tile `tile` into stage base `sb`: operand p / 4, row group p % 4
#define CI_DIRECT_PIECE(sb, tile, p)                                                                  \
  do {                                                                                                \
    const int kk_ = min((tile), nk - 1) * BK;                                                         \
    const T* src_ = ((p) < 4) ? pa[(p) & 3] + kk_ : pb[((p) >> 2) - 1][(p) & 3] + kk_;                \
    __builtin_amdgcn_global_load_lds(CI_GLOBAL_PTR(src_),                                             \
                                     CI_LDS_PTR((sb) + ((p) >> 2) * TILE_B + (32 * ((p) & 3) + 8 * wave) * 128), \
                                     16, 0, 0);                                                       \
  } while (0)

  f32x16 acc[NB][2][2];
#pragma unroll
  for (int q = 0; q < NB; ++q)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[q][i][j][v] = 0.f;

  // k-tiles 0 .. S-2 on their way
#pragma unroll
  for (int r = 0; r < S - 1; ++r) {
#pragma unroll
    for (int p = 0; p < NP; ++p) CI_DIRECT_PIECE(st[r], r, p);
  }
  // fragment addresses: row l31 (+ 32 i + 64 wm) of the tile, chunk 2 s + lane / 32
  const int l31 = lane & 31, hi = lane >> 5;
  uint4 fa[2][2], fb[2][NB][2];
#define CI_DIRECT_FRAGS(buf, base, s)                                                                 \
  do {                                                                                                \
    _Pragma("unroll") for (int i_ = 0; i_ < 2; ++i_) {                                                \
      const int r_ = wm * 64 + i_ * 32 + l31;                                                         \
      fa[buf][i_] = *reinterpret_cast<const uint4*>((base) + r_ * 128 + (((2 * (s) + hi) ^ ((r_ >> 1) & 7)) << 4)); \
    }                                                                                                 \
    _Pragma("unroll") for (int q_ = 0; q_ < NB; ++q_)                                                 \
      _Pragma("unroll") for (int j_ = 0; j_ < 2; ++j_) {                                              \
        const int r_ = wn * 64 + j_ * 32 + l31;                                                       \
        fb[buf][q_][j_] = *reinterpret_cast<const uint4*>((base) + TILE_B * (1 + q_) + r_ * 128 +     \
                                                          (((2 * (s) + hi) ^ ((r_ >> 1) & 7)) << 4));        \
      }                                                                                               \
  } while (0)
  // vmcnt(NP (S - 2)) and lgkmcnt(0): the next k-tile has landed, and my fragment reads are done.
  // The barrier is the bare instruction: a fenced one would wait for every load in flight.
  constexpr int kWaitNext = 0x0070 | ((NP * (S - 2)) & 15) | (((NP * (S - 2)) >> 4) << 14);
  __builtin_amdgcn_s_waitcnt(kWaitNext);  // k-tile 0 has landed
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
  CI_DIRECT_FRAGS(0, st[0], 0);

  constexpr int kPieceLo[4] = {0, (NP + 2) / 3, (2 * NP + 2) / 3, NP};  // 3 + 3 + 2, or 4 + 4 + 4
  for (int kt0 = 0; kt0 < nk; kt0 += S) {
#pragma unroll
    for (int r = 0; r < S; ++r) {
      const int kt = kt0 + r;
      const unsigned char* sA = st[r];                  // k-tile kt
      const unsigned char* sN = st[(r + 1) % S];        // k-tile kt + 1
      unsigned char* sF = st[(r + S - 1) % S];          // free since the barrier inside k-tile kt - 1: takes k-tile kt + S - 1
#pragma unroll
      for (int s = 0; s < BK / 16; ++s) {
        if (s == BK / 16 - 1) {
          // my pieces of k-tile kt + 1 have landed; after the barrier everybody's have, and every
          // wave has read all fragments of k-tile kt
          __builtin_amdgcn_sched_barrier(0);
          __builtin_amdgcn_s_waitcnt(kWaitNext);
          __builtin_amdgcn_s_barrier();
          __builtin_amdgcn_sched_barrier(0);
          CI_DIRECT_FRAGS(0, sN, 0);
        } else {
          CI_DIRECT_FRAGS((s + 1) & 1, sA, s + 1);
#pragma unroll
          for (int p = 0; p < NP; ++p) {
            if (p < kPieceLo[s] || p >= kPieceLo[s + 1]) continue;
            CI_DIRECT_PIECE(sF, kt + S - 1, p);
          }
        }
        if (!GUARD || kt < nk) {  // padding iterations (nk not a multiple of S) skip the arithmetic only
#pragma unroll
          for (int q = 0; q < NB; ++q)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
              for (int j = 0; j < 2; ++j) acc[q][i][j] = mfma32<D>(fa[s & 1][i], fb[s & 1][q][j], acc[q][i][j]);
        }
#pragma unroll
        for (int m = 0; m < 4 * NB; ++m) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // LDS read
          __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // global load
        }
        __builtin_amdgcn_sched_barrier(0);  // keeps the k-steps (and with them the load order) apart
      }
    }
  }
#undef CI_DIRECT_FRAGS
#undef CI_DIRECT_PIECE
  __builtin_amdgcn_s_waitcnt(0x0F70);  // nothing of mine is still on its way into LDS when the workgroup ends
  gemm_epilogue<D, EPI>(g, acc, m0, n0, wm, wn, lane);
}

// ---------------------------------------------------------------------------
// Large-tile kernel for shapes that divide evenly: 256 x 256 outputs per
// workgroup (SwiGLU: 256 rows x 128 gate + the same 128 up columns), eight waves
// of 128 x 64 with 8 accumulator tiles each, two waves per SIMD.  What bounds a
// tiled MFMA kernel on this chip is LDS traffic: per k-tile a compute unit
// writes the two operand tiles once and every wave reads its fragments, and at
// 128 bytes per clock that takes about as long as the tile's MFMAs for this
// shape (1.5 times as long for 128 x 128 tiles with 64 x 64 wave tiles), so the
// LDS instructions have to issue between the MFMAs, never in a burst in front
// of them.  One k-tile ahead lives in registers; a third of it moves to the
// other LDS stage (and is re-requested for the tile after) in each of the first
// three k-steps; fragments are double-buffered; the one barrier per k-tile sits
// before the last k-step, whose MFMAs cover the first fragment reads of the next
// tile.  (Four waves of 128 x 128 read a third less from LDS and do overlap
// their own reads with their MFMAs when scheduled this way, but came out no
// faster: the stores and the barrier weigh more with one wave per SIMD.)
constexpr int GM = 256;
constexpr int LDN = 256 + 32;  // LDS row pitch of a k-major B tile (576 bytes: rows alternate bank halves)
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
constexpr int kFullChip = 256;          // compute units of an MI355X
constexpr int kBigMinWorkgroups = 160;  // below this the 128 x 128 kernel fills the chip better

template <class D, int EPI>
__device__ __forceinline__ void big_store_block(const GemmArgs& g, const f32x16& c0, const f32x16& c1,
                                                int row0, int col, int lane) {
  using T = typename D::T;
  if (g.partial) {
    float* part = g.partial + (size_t)blockIdx.y * g.M * g.Nn;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = row0 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      part[(size_t)row * g.Nn + col] = c0[v];
    }
    return;
  }
  const T* bias = reinterpret_cast<const T*>(g.bias);
  const float bv = bias ? to_float<D>(bias[col]) : 0.f;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int row = row0 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
    float h, score;
    if (EPI == EPI_SWIGLU) {
      h = silu(c0[v]) * c1[v];
      score = fabsf(h);
    } else if (EPI == EPI_RELU) {
      h = fmaxf(c0[v] + bv, 0.f);
      score = h;
    } else {
      h = c0[v] + bv;
      score = h;
    }
    const size_t o = (size_t)row * g.ldo + col;
    if (g.out_f) g.out_f[o] = score;
    if (g.out_e) reinterpret_cast<T*>(g.out_e)[o] = from_float<D>(h);
  }
}

template <class D, int EPI, bool BNN>
__global__ __launch_bounds__(512) void gemm_mfma_big_kernel(GemmArgs g) {
  using T = typename D::T;
  constexpr bool DUAL = (EPI == EPI_SWIGLU);
  constexpr int BNO = DUAL ? 128 : 256;  // output columns per workgroup
  constexpr int TILE = GM * LDK;         // one operand tile in LDS (elements)
  constexpr int STAGE = 2 * TILE;        // A rows, then 256 B rows (SwiGLU: 128 gate, 128 up)
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* smem = reinterpret_cast<T*>(smem_raw);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;  // 2 x 4 waves of 128 x 64 outputs
  const int tiles_m = g.M / GM;
  const int t = xcd_swizzle(blockIdx.x, gridDim.x);
  const int m0 = (t % tiles_m) * GM, n0 = (t / tiles_m) * BNO;
  const int k_begin = blockIdx.y * g.k_chunk;
  const int k_end = min(g.Kk, k_begin + g.k_chunk);
  const int nk = (k_end - k_begin) / BK;

  // staging: 8 16-byte pieces per thread and k-tile; piece i < 4 is A row srow + 64 i, piece
  // 4 + j is row srow + 64 j of the 256-row B image.  Uniform bases + 32-bit per-thread byte
  // offsets (an operand spans far less than 4 GB)
  const int srow = tid >> 3, kc = (tid & 7) * 8;
  const char* Ab = reinterpret_cast<const char*>(g.A) + ((size_t)m0 * g.lda + k_begin) * sizeof(T);
  // B given k-major ([Kk, Nn], a neuron-major down matrix): its tile is staged as it lies in
  // memory, [64 k][256 n] with row pitch LDN, piece j of a thread = k row tid/32 + 16 j, columns
  // 8 (tid % 32) .. + 8; the fragments then come out of LDS through transposing reads.
  static_assert(!(BNN && DUAL), "k-major B is only needed for the down projection");
  const char* B0b = BNN ? reinterpret_cast<const char*>(g.B0) + ((size_t)k_begin * g.ldb + n0) * sizeof(T)
                        : reinterpret_cast<const char*>(g.B0) + ((size_t)n0 * g.ldb + k_begin) * sizeof(T);
  const char* B1b = DUAL ? reinterpret_cast<const char*>(g.B1) + ((size_t)n0 * g.ldb + k_begin) * sizeof(T) : B0b;
  const uint32_t offA = (uint32_t)(((size_t)srow * g.lda + kc) * sizeof(T));
  const uint32_t offB = BNN ? (uint32_t)(((size_t)(tid >> 5) * g.ldb + (tid & 31) * 8) * sizeof(T))
                            : (uint32_t)(((size_t)srow * g.ldb + kc) * sizeof(T));
  const uint32_t sa = (uint32_t)(64 * g.lda * sizeof(T));
  const uint32_t sb = (uint32_t)((BNN ? 16 : 64) * g.ldb * sizeof(T));
  const uint32_t kstepB = BNN ? (uint32_t)(g.ldb * sizeof(T)) : (uint32_t)sizeof(T);  // bytes per unit of k
  const int soff = srow * LDK + kc;
  const int soffB = BNN ? (tid >> 5) * LDN + (tid & 31) * 8 : soff;

  constexpr int RD = 1;  // k-tiles held in registers ahead of the one being multiplied (2 does not fit 128 VGPRs)
  uint4 r[RD][8];
#define CI_BIG_ISSUE(slot, i, kk)                                                                  \
  do {                                                                                             \
    const uint32_t kb_ = (uint32_t)(kk) * (uint32_t)sizeof(T);                                     \
    const uint32_t kbB_ = (uint32_t)(kk) * kstepB;                                                 \
    if ((i) < 4) r[slot][i] = ld16(Ab + (offA + (uint32_t)(i) * sa + kb_));                          \
    else if (!DUAL || (i) < 6) r[slot][i] = ld16(B0b + (offB + (uint32_t)((i) - 4) * sb + kbB_));    \
    else r[slot][i] = ld16(B1b + (offB + (uint32_t)((i) - 6) * sb + kbB_));                          \
  } while (0)
#define CI_BIG_STORE(slot, i, base)                                                                \
  do {                                                                                             \
    if ((i) < 4) *reinterpret_cast<uint4*>((base) + soff + 64 * (i) * LDK) = r[slot][i];             \
    else if (BNN) *reinterpret_cast<uint4*>((base) + TILE + soffB + 16 * ((i) - 4) * LDN) = r[slot][i]; \
    else *reinterpret_cast<uint4*>((base) + TILE + soffB + 64 * ((i) - 4) * LDK) = r[slot][i];        \
  } while (0)

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // fragment rows of this wave: A rows wm*128 + 32 i; B image rows wn*64 + 32 j, or for SwiGLU the
  // gate rows wn*32 (j = 0) and the up rows 128 + wn*32 (j = 1) of the same output columns
  const int l31 = lane & 31, khalf = (lane >> 5) * 8;
  const int brow0 = DUAL ? wn * 32 + l31 : wn * 64 + l31;
  const int brow1 = DUAL ? 128 + wn * 32 + l31 : wn * 64 + 32 + l31;
  // k-major B: a transposing 64-bit LDS read hands lane 4a + b of a 16-lane group element b of the
  // 8-byte pieces that lanes a, a + 4, a + 8, a + 12 of the group point at.  With lane s of a group
  // pointing at k row s / 4, columns 4 (s % 4) .. + 4, lane L of the group receives four consecutive
  // k of column L: two such reads give the eight k of one MFMA operand (k chunk lane / 32, column
  // lane % 32).
  const int trow = 8 * (lane >> 5) + ((lane & 15) >> 2);
  const int tcol = wn * 64 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  uint4 fa[2][4], fb[2][2];
#define CI_BIG_FRAGS(buf, base, s)                                                                 \
  do {                                                                                             \
    _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_)                                               \
      fa[buf][i_] = *reinterpret_cast<const uint4*>((base) + (wm * 128 + i_ * 32 + l31) * LDK + (s) * 16 + khalf); \
    if (BNN) {                                                                                     \
      _Pragma("unroll") for (int j_ = 0; j_ < 2; ++j_) {                                           \
        const T* p_ = (base) + TILE + ((s) * 16 + trow) * LDN + tcol + j_ * 32;                    \
        const s16x4 lo_ = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p_));               \
        const s16x4 hi_ = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p_ + 4 * LDN));     \
        const s16x8 both_ = __builtin_shufflevector(lo_, hi_, 0, 1, 2, 3, 4, 5, 6, 7);             \
        fb[buf][j_] = __builtin_bit_cast(uint4, both_);                                            \
      }                                                                                            \
    } else {                                                                                       \
      fb[buf][0] = *reinterpret_cast<const uint4*>((base) + TILE + brow0 * LDK + (s) * 16 + khalf); \
      fb[buf][1] = *reinterpret_cast<const uint4*>((base) + TILE + brow1 * LDK + (s) * 16 + khalf); \
    }                                                                                              \
  } while (0)

  // prologue: tiles 0 .. RD-1 requested, tile 0 -> LDS stage 0, its slot re-requested with tile RD
#pragma unroll
  for (int q = 0; q < RD; ++q) {
    const int kkq = min(q, nk - 1) * BK;
#pragma unroll
    for (int i = 0; i < 8; ++i) CI_BIG_ISSUE(q, i, kkq);
    __builtin_amdgcn_sched_barrier(0);
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) CI_BIG_STORE(0, i, smem);
  __builtin_amdgcn_sched_barrier(0);
  {
    const int kkq = min(RD, nk - 1) * BK;
#pragma unroll
    for (int i = 0; i < 8; ++i) CI_BIG_ISSUE(0, i, kkq);
  }
  __builtin_amdgcn_sched_barrier(0);
  __syncthreads();
  CI_BIG_FRAGS(0, smem, 0);

  for (int kt0 = 0; kt0 < nk; kt0 += 2) {
#pragma unroll
    for (int par = 0; par < 2; ++par) {
      const int kt = kt0 + par;              // stage par holds tile kt
      constexpr int kNext[2] = {1 % RD, 0};
      const int slot = kNext[par];           // slot of tile kt + 1 (RD = 2: its parity; RD = 1: slot 0)
      const T* sA = smem + par * STAGE;
      T* sN = smem + (1 - par) * STAGE;
      const int kk_next = min(kt + 1 + RD, nk - 1) * BK;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        if (s == 3) {
          // every wave has read all of this tile's fragments and written its share of the next tile
          __syncthreads();
          CI_BIG_FRAGS(0, sN, 0);
        } else {
          CI_BIG_FRAGS((s + 1) & 1, sA, s + 1);
          // a third of tile kt + 1: registers -> the other stage, then re-requested with tile kt + 1 + RD
          constexpr int lo[4] = {0, 3, 6, 8};
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            if (i >= lo[s] && i < lo[s + 1]) {
              CI_BIG_STORE(slot, i, sN);
              CI_BIG_ISSUE(slot, i, kk_next);
            }
          }
        }
        if (kt < nk) {  // the padding iteration of an odd tile count skips the arithmetic only
#pragma unroll
          for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = mfma32<D>(fa[s & 1][i], fb[s & 1][j], acc[i][j]);
        }
        // within a k-step: one LDS or global instruction after each MFMA instead of a burst of them
        // before the first (the matrix pipe idles while a burst issues)
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // LDS read
          __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);  // LDS write
          __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // global load
        }
        __builtin_amdgcn_sched_barrier(0);  // keeps the k-steps (and with them the load order) apart
      }
    }
  }
#undef CI_BIG_ISSUE
#undef CI_BIG_STORE
#undef CI_BIG_FRAGS

#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row0 = m0 + wm * 128 + i * 32;
    if (DUAL) {
      big_store_block<D, EPI>(g, acc[i][0], acc[i][1], row0, n0 + wn * 32 + l31, lane);
    } else {
#pragma unroll
      for (int j = 0; j < 2; ++j)
        big_store_block<D, EPI>(g, acc[i][j], acc[i][j], row0, n0 + wn * 64 + j * 32 + l31, lane);
    }
  }
}

// ---------------------------------------------------------------------------
// fp32 element type: 64x64x16 tiles, 256 threads, 4x4 outputs per thread.
template <int EPI, bool BNN>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs g) {
  constexpr bool DUAL = (EPI == EPI_SWIGLU);
  constexpr int NB = DUAL ? 2 : 1;
  __shared__ float sA[16][68];
  __shared__ float sB[NB][16][68];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int tiles_m = (g.M + 63) / 64;
  const int m0 = (blockIdx.x % tiles_m) * 64, n0 = (blockIdx.x / tiles_m) * 64;
  const float* A = reinterpret_cast<const float*>(g.A);
  const float* Bp[2] = {reinterpret_cast<const float*>(g.B0), reinterpret_cast<const float*>(g.B1)};
  float acc[NB][4][4];
#pragma unroll
  for (int q = 0; q < NB; ++q)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[q][i][j] = 0.f;

  for (int k0 = 0; k0 < g.Kk; k0 += 16) {
    // 64 rows x 16 k: thread -> (row = tid / 4, k quad = tid % 4)
    {
      const int row = tid >> 2, kq = (tid & 3) * 4;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int k = k0 + kq + e;
        sA[kq + e][row] = (m0 + row < g.M && k < g.Kk) ? A[(size_t)(m0 + row) * g.lda + k] : 0.f;
      }
#pragma unroll
      for (int q = 0; q < NB; ++q) {
        if (!BNN) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int k = k0 + kq + e;
            sB[q][kq + e][row] = (n0 + row < g.Nn && k < g.Kk) ? Bp[q][(size_t)(n0 + row) * g.ldb + k] : 0.f;
          }
        } else {
          const int kr = tid >> 4, nq = (tid & 15) * 4;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int n = n0 + nq + e;
            sB[q][kr][nq + e] = (k0 + kr < g.Kk && n < g.Nn) ? Bp[q][(size_t)(k0 + kr) * g.ldb + n] : 0.f;
          }
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], b[NB][4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = sA[k][ty * 4 + i];
#pragma unroll
      for (int q = 0; q < NB; ++q)
#pragma unroll
        for (int j = 0; j < 4; ++j) b[q][j] = sB[q][k][tx * 4 + j];
#pragma unroll
      for (int q = 0; q < NB; ++q)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[q][i][j] = fmaf(a[i], b[q][j], acc[q][i][j]);
    }
    __syncthreads();
  }
  const float* bias = reinterpret_cast<const float*>(g.bias);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = m0 + ty * 4 + i;
    if (row >= g.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = n0 + tx * 4 + j;
      if (col >= g.Nn) continue;
      const float bv = bias ? bias[col] : 0.f;
      float h, score;
      if (EPI == EPI_SWIGLU) {
        h = silu(acc[0][i][j]) * acc[NB - 1][i][j];
        score = fabsf(h);
      } else if (EPI == EPI_RELU) {
        h = fmaxf(acc[0][i][j] + bv, 0.f);
        score = h;
      } else {
        h = acc[0][i][j] + bv;
        score = h;
      }
      const size_t o = (size_t)row * g.ldo + col;
      if (g.out_f) g.out_f[o] = score;
      if (g.out_e) reinterpret_cast<float*>(g.out_e)[o] = h;
    }
  }
}

// Y[m, n] = sum_s partial[s][m][n] + bias[n], converted to the element type.
template <class D>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial,
                                                            const void* __restrict__ bias,
                                                            void* __restrict__ out, int splits,
                                                            int M, int Nn) {
  using T = typename D::T;
  const size_t total4 = (size_t)M * Nn / 4;
  const size_t i4 = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i4 >= total4) return;
  float4 a = reinterpret_cast<const float4*>(partial)[i4];
  for (int s = 1; s < splits; ++s) {
    const float4 v = reinterpret_cast<const float4*>(partial + (size_t)s * M * Nn)[i4];
    a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
  }
  const int col = (int)((i4 * 4) % Nn);
  float o[4] = {a.x, a.y, a.z, a.w};
  if (bias) {
#pragma unroll
    for (int k = 0; k < 4; ++k) o[k] += to_float<D>(reinterpret_cast<const T*>(bias)[col + k]);
  }
  T* y = reinterpret_cast<T*>(out) + i4 * 4;
#pragma unroll
  for (int k = 0; k < 4; ++k) y[k] = from_float<D>(o[k]);
}

template <class D, int EPI, int RD, bool GUARD>
int launch_ring(const GemmArgs& g, int tiles, int splits, size_t lds, hipStream_t s) {
  static std::atomic<uint64_t> attr_seen{0};
  if (lds > 48 * 1024 && allow_dynamic_lds(attr_seen, reinterpret_cast<const void*>(&gemm_mfma_ring_kernel<D, EPI, RD, GUARD>), lds) != CI_OK)
    return CI_ERR_HIP;
  hipLaunchKernelGGL((gemm_mfma_ring_kernel<D, EPI, RD, GUARD>), dim3(tiles, splits), dim3(256), lds, s, g);
  return CI_OK;
}

template <class D, int EPI, bool BNN>
int launch_mfma(const GemmArgs& g, hipStream_t s) {
  constexpr int NB = (EPI == EPI_SWIGLU) ? 2 : 1;
  const size_t lds = (size_t)2 * BM * LDK * (1 + NB) * sizeof(typename D::T);
  static std::atomic<uint64_t> attr_seen{0};
  if (lds > 48 * 1024 && allow_dynamic_lds(attr_seen, reinterpret_cast<const void*>(&gemm_mfma_kernel<D, EPI, BNN>), lds) != CI_OK)
    return CI_ERR_HIP;
  const int tiles = ((g.M + BM - 1) / BM) * ((g.Nn + BN - 1) / BN);
  const int splits = g.partial ? (g.Kk + g.k_chunk - 1) / g.k_chunk : 1;
  const bool ring = !BNN && g.Kk % BK == 0 && g.k_chunk % BK == 0 && params().gemm_ring;
  constexpr int BNO = (EPI == EPI_SWIGLU) ? 128 : 256;
  const int big_tiles = (g.M / GM) * (g.Nn / BNO);
  const bool ring_shape = g.Kk % BK == 0 && g.k_chunk % BK == 0 && params().gemm_ring;
  // the large-tile kernel addresses an operand through a uniform base and 32-bit byte offsets; a
  // k-major B is walked along k from one base, so the whole matrix has to stay below 4 GB
  const bool offsets_fit = (size_t)GM * (size_t)g.lda * 4 + (size_t)g.Kk * 4 < ((size_t)1 << 32) &&
                           (BNN ? (size_t)g.Kk * (size_t)g.ldb * 4 : (size_t)GM * (size_t)g.ldb * 4 + (size_t)g.Kk * 4) <
                               ((size_t)1 << 32);
  const bool big = ring_shape && offsets_fit && (EPI == EPI_LINEAR || !BNN) && g.M % GM == 0 && g.Nn % BNO == 0 && g.Kk / BK >= 2 &&
                   (params().gemm_big == 2 || (params().gemm_big == 1 && big_tiles * splits >= kBigMinWorkgroups));
  if (big) {
    const size_t lds_big = (size_t)2 * 2 * GM * LDK * sizeof(typename D::T);
    static std::atomic<uint64_t> big_attr_seen{0};
    if (allow_dynamic_lds(big_attr_seen, reinterpret_cast<const void*>(&gemm_mfma_big_kernel<D, EPI, BNN && EPI == EPI_LINEAR>), lds_big) != CI_OK)
      return CI_ERR_HIP;
    hipLaunchKernelGGL((gemm_mfma_big_kernel<D, EPI, BNN && EPI == EPI_LINEAR>), dim3(big_tiles, splits), dim3(512), lds_big, s, g);
  } else if (ring && params().gemm_direct) {
    constexpr int kStages = (EPI == EPI_SWIGLU) ? 3 : 4;
    const int chunk = g.partial ? g.k_chunk : g.Kk;
    const bool even = g.Kk % chunk == 0 && (chunk / BK) % kStages == 0;  // every split's k-tile count divides
    if (even) hipLaunchKernelGGL((gemm_mfma_direct_kernel<D, EPI, false>), dim3(tiles, splits), dim3(256), 0, s, g);
    else hipLaunchKernelGGL((gemm_mfma_direct_kernel<D, EPI, true>), dim3(tiles, splits), dim3(256), 0, s, g);
  } else if (ring) {
    // deepest ring whose depth divides every split's k-tile count (no padding iterations); else the
    // guarded variant.  SwiGLU holds three operand tiles per k-tile, so its ring stays at two.
    const int chunk = g.partial ? g.k_chunk : g.Kk;
    const int nkc = (g.Kk % chunk == 0) ? chunk / BK : 0;  // 0: the splits differ in length
    int rc = CI_OK;
    if constexpr (EPI == EPI_SWIGLU) {
      rc = (nkc > 0 && nkc % 2 == 0) ? launch_ring<D, EPI, 2, false>(g, tiles, splits, lds, s)
                                     : launch_ring<D, EPI, 2, true>(g, tiles, splits, lds, s);
    } else {
      if (nkc > 0 && nkc % 4 == 0 && tiles * splits <= kFullChip)
        rc = launch_ring<D, EPI, 4, false>(g, tiles, splits, lds, s);  // one workgroup per CU: registers to spare
      else if (nkc > 0 && nkc % 3 == 0)
        rc = launch_ring<D, EPI, 3, false>(g, tiles, splits, lds, s);
      else if (nkc > 0 && nkc % 2 == 0)
        rc = launch_ring<D, EPI, 2, false>(g, tiles, splits, lds, s);
      else
        rc = launch_ring<D, EPI, 3, true>(g, tiles, splits, lds, s);
    }
    if (rc != CI_OK) return rc;
  } else {
    hipLaunchKernelGGL((gemm_mfma_kernel<D, EPI, BNN>), dim3(tiles, splits), dim3(256), lds, s, g);
  }
  CI_HIP_CHECK_LAUNCH();
  if (g.partial) {
    const size_t total4 = (size_t)g.M * g.Nn / 4;
    hipLaunchKernelGGL((splitk_reduce_kernel<D>), dim3((unsigned)((total4 + 255) / 256)), dim3(256), 0, s,
                       g.partial, g.bias, g.out_e, splits, g.M, g.Nn);
    CI_HIP_CHECK_LAUNCH();
  }
  return CI_OK;
}

template <int EPI, bool BNN>
int launch_f32(const GemmArgs& g, hipStream_t s) {
  const int tiles = ((g.M + 63) / 64) * ((g.Nn + 63) / 64);
  hipLaunchKernelGGL((gemm_f32_kernel<EPI, BNN>), dim3(tiles), dim3(256), 0, s, g);
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

template <int EPI, bool BNN>
int launch_any(int dtype, const GemmArgs& g, hipStream_t s) {
  switch (dtype) {
    case CI_F32: return launch_f32<EPI, BNN>(g, s);
    case CI_F16: return launch_mfma<F16, EPI, BNN>(g, s);
    case CI_BF16: return launch_mfma<BF16, EPI, BNN>(g, s);
  }
  return CI_ERR_BAD_DTYPE;
}

}  // namespace

int launch_gemm_up(const void* X, int64_t M, const void* w_up, const void* w_gate, const void* b_up,
                   int dtype, int act, int64_t d, int64_t N, void* H, float* A, hipStream_t s) {
  GemmArgs g;
  g.A = X;
  g.lda = d;
  g.ldb = d;
  g.ldo = N;
  g.M = (int)M;
  g.Nn = (int)N;
  g.Kk = (int)d;
  g.out_e = H;
  g.out_f = A;
  g.k_chunk = (int)d;
  g.partial = nullptr;
  if (act == CI_ACT_SWIGLU) {
    g.B0 = w_gate;
    g.B1 = w_up;
    g.bias = nullptr;
    return launch_any<EPI_SWIGLU, false>(dtype, g, s);
  }
  g.B0 = w_up;
  g.B1 = nullptr;
  g.bias = b_up;
  return launch_any<EPI_RELU, false>(dtype, g, s);
}

// Number of k splits of the down projection: few output tiles (small M) would
// leave most CUs idle, so the long reduction over N is cut into chunks.  Pure
// functions of the shape; the workspace is sized for the larger of the two.
static int down_splits_small(int64_t M, int64_t d, int64_t N) {
  const int64_t tiles = ((M + BM - 1) / BM) * ((d + BN - 1) / BN);
  int64_t s = (256 + tiles - 1) / tiles;
  const int64_t max_by_k = (N + 4 * BK - 1) / (4 * BK);  // at least four k tiles per split
  if (s > max_by_k) s = max_by_k;
  if (s > 8) s = 8;
  return s < 1 ? 1 : (int)s;
}
// Large tiles: as many k splits as bring the grid to about one workgroup per CU;
// 0 when the large-tile kernel does not apply.
static int down_splits_big(int64_t M, int64_t d, int64_t N) {
  if (M % GM != 0 || d % 256 != 0 || N % BK != 0) return 0;
  const int64_t tb = (M / GM) * (d / 256);
  if (tb >= kBigMinWorkgroups) {
    // enough tiles to fill the chip; a k split can still pay when the last round of workgroups is
    // mostly empty (576 tiles = 2.25 rounds on 256 compute units take as long as three).  Model:
    // rounds of tiles, each 1/s of a full tile's time at ~4.5 TFLOP/s per compute unit, plus the
    // fp32 partial products written and read back at ~4.5 TB/s and one more launch.
    const double t_tile = 2.0 * GM * 256 * (double)N / 4.5e12;
    const double t_one = (double)((tb + kFullChip - 1) / kFullChip) * t_tile;
    int best = 1;
    double best_t = 0.95 * t_one;  // a split has to win by 5 %
    for (int sp = 2; sp <= 8; ++sp) {
      if (N / ((int64_t)sp * BK) < 8) break;  // at least eight k tiles per split
      const int64_t rounds = (tb * sp + kFullChip - 1) / kFullChip;
      const double t = (double)rounds * t_tile / sp + 2.0 * sp * (double)M * (double)d * 4.0 / 4.5e12 + 6e-6;
      if (t < best_t) { best = sp; best_t = t; }
    }
    return best;
  }
  if (tb < 32) return 0;
  int64_t sb = (256 + tb / 2) / tb;
  const int64_t max_k = N / (8 * BK);  // at least eight k tiles per split
  if (sb > max_k) sb = max_k;
  if (sb > 8) sb = 8;
  return (sb >= 1 && tb * sb >= kBigMinWorkgroups) ? (int)sb : 0;
}
int gemm_down_splits(int64_t M, int64_t d, int64_t N, int dtype) {
  if (dtype == CI_F32) return 1;
  if (params().gemm_big == 1) {
    const int sb = down_splits_big(M, d, N);
    if (sb > 0) return sb;
  }
  return down_splits_small(M, d, N);
}
int gemm_down_splits_max(int64_t M, int64_t d, int64_t N, int dtype) {
  if (dtype == CI_F32) return 1;
  const int a = down_splits_small(M, d, N), b = down_splits_big(M, d, N);
  return a > b ? a : b;
}

int launch_gemm_down(const void* H, int64_t M, const void* w_down, const void* b_down,
                     int down_layout, int dtype, int64_t d, int64_t N, void* Y, float* partial,
                     hipStream_t s) {
  GemmArgs g;
  g.A = H;
  g.lda = N;
  g.B0 = w_down;
  g.B1 = nullptr;
  g.bias = b_down;
  g.out_e = Y;
  g.out_f = nullptr;
  g.ldo = d;
  g.M = (int)M;
  g.Nn = (int)d;
  g.Kk = (int)N;
  const int splits = gemm_down_splits(M, d, N, dtype);
  g.k_chunk = (int)N;
  g.partial = nullptr;
  if (splits > 1) {
    g.k_chunk = (int)(((N + splits - 1) / splits + BK - 1) / BK * BK);
    g.partial = partial;
  }
  if (down_layout == CI_DOWN_OUT_MAJOR) {
    g.ldb = N;
    return launch_any<EPI_LINEAR, false>(dtype, g, s);
  }
  g.ldb = d;
  return launch_any<EPI_LINEAR, true>(dtype, g, s);
}

}  // namespace ci
