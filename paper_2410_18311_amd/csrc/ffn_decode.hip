// Decode-stage FFN over the frozen core set (Sec. 4.2 of arXiv 2410.18311):
//   y = W_down_c^T act(W_up_c x [+ b]) [+ b_down]
// with all three matrices neuron-major [K, d].  HBM-bandwidth bound: every
// weight byte is read exactly once, x and the K hidden values stay on chip.
//
// Kernel 1 (ffn_decode_kernel): a workgroup owns a contiguous slice of the K
// neurons.  Phase A: all threads of the workgroup split the d columns of each
// up (and gate) row with 16-byte loads, reduce the dot products across the
// wave by shuffles and across waves through LDS, and apply bias + ReLU or
// SiLU(g)*u in fp32.  Phase B: each thread owns fixed output columns and
// accumulates h_k * W_down_c[k, :] over the slice.  The slice's partial y goes
// to partial[b][wg][d] (fp32).
// Kernel 2 (decode_reduce_kernel): sums the partials in a fixed order (so the
// result is deterministic), adds b_down, converts to the element type.
#include "common.hpp"
#include "decode_common.hpp"

namespace ci {

namespace {

struct DecodeArgs {
  const void* x;
  const void* w_up;
  const void* w_gate;
  const void* b_up;
  const void* w_down;
  const int32_t* core_idx;
  float* partial;
  int K, d, N, n_wg;
  int nt_store;
};

template <int DEPTH>
__device__ __forceinline__ float wave_sum_rows(float (&v)[DEPTH], int lane) {
  static_assert(DEPTH == 4 || DEPTH == 8 || DEPTH == 16, "ring depth");
  halve_rows<DEPTH, 32>(v, lane);
  return v[0];
}

// Weight row that super-chunk-local neuron r names (gathered: through the
// index list staged in LDS, -1 = skip; compacted: consecutive rows).
template <bool GATHER>
__device__ __forceinline__ size_t decode_row_of(int r, int row_base, const int* sidx) {
  if (GATHER) {
    const int n = sidx[r];
    return n < 0 ? (size_t)0 : (size_t)n;
  }
  return (size_t)(row_base + r);
}

// Issues the 16-byte loads of ring position `pos` into one register slot.
// Ring positions of one super-chunk of Rs neurons (QB = NDOT * Rs dot rows):
//   [0, lead)               filler so that lead + QB is a multiple of DEPTH
//   [lead, lead + QB)       rows of the gate (SwiGLU only) and up matrices -> dot with x
//   [lead + QB, NQ)         rows of the down matrix                        -> axpy into y
//   [NQ, ...)               filler
// EVERY position issues its loads, filler positions from the (cache-resident)
// x vector: with the same number of loads on every control path the compiler
// can count outstanding loads exactly and waits only for the slot it consumes.
template <class T, int NI, bool SWIGLU, bool GATHER>
__device__ __forceinline__ void decode_issue(int pos, int lead, int Rs, int QB, int NQ,
                                             const char* __restrict__ gate,
                                             const char* __restrict__ up,
                                             const char* __restrict__ down,
                                             const char* __restrict__ filler, size_t rowbytes,
                                             int row_base, const int* sidx,
                                             const uint32_t (&coff)[NI], uint4 (&dst)[NI]) {
  const int q = pos - lead;
  const bool valid = q >= 0 && pos < NQ;
  const bool is_dot = q < QB;
  const bool second = SWIGLU && q >= Rs;  // SwiGLU: gate rows first, then up rows
  int r = is_dot ? (second ? q - Rs : q) : q - QB;
  r = r < 0 ? 0 : (r > Rs - 1 ? Rs - 1 : r);
  const char* base = is_dot ? ((SWIGLU && !second) ? gate : up) : down;
  const char* prow = base + decode_row_of<GATHER>(r, row_base, sidx) * rowbytes;
  prow = valid ? prow : filler;
#pragma unroll
  for (int i = 0; i < NI; ++i) dst[i] = ld16_stream(prow + coff[i]);
}

// DEPTH rows are always in flight per thread; the loads of the down rows are
// issued while the dots are still being reduced, so the memory pipeline never
// drains at the phase boundary.
template <class D, int NI, bool SWIGLU, bool GATHER, int DEPTH>
__global__ __launch_bounds__(NI >= 4 ? 1024 : 512) void ffn_decode_kernel(DecodeArgs a) {
  using T = typename D::T;
  constexpr int VEC = D::VEC;
  constexpr int NDOT = SWIGLU ? 2 : 1;  // matrices that are dotted with x

  extern __shared__ float smem[];
  const int tid = threadIdx.x, nt = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
  const int wg = blockIdx.x, b = blockIdx.y;
#ifdef CI_FUSED_STAMPS
  unsigned long long* st = reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(a.partial) + (8 << 20));
#define CI_OSTAMP(i) do { if (tid == 0) st[wg * 8 + (i)] = __builtin_amdgcn_s_memrealtime(); } while (0)
#else
#define CI_OSTAMP(i) do { } while (0)
#endif
  CI_OSTAMP(0);
  const int r0 = (int)(((int64_t)wg * a.K) / a.n_wg);
  const int r1 = (int)(((int64_t)(wg + 1) * a.K) / a.n_wg);
  const int R = r1 - r0;

  float* red = smem;                            // [nw][NDOT * kSuper] wave partial dots
  float* hbuf = red + nw * NDOT * kSuper;       // [kSuper] hidden values
  int* sidx = reinterpret_cast<int*>(hbuf + kSuper);  // [kSuper] weight row of each slice neuron (-1: skip)

  const size_t rowbytes = (size_t)a.d * sizeof(T);
  const char* up = reinterpret_cast<const char*>(a.w_up);
  const char* gate = reinterpret_cast<const char*>(a.w_gate);
  const char* down = reinterpret_cast<const char*>(a.w_down);
  const char* xrow = reinterpret_cast<const char*>(a.x) + (size_t)b * rowbytes;

  // columns owned by this thread
  uint32_t coff[NI];
  bool cv[NI];
  uint4 xraw[NI];
  float xr[NI][VEC];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int col = (i * nt + tid) * VEC;
    cv[i] = col < a.d;
    // a column past the end re-reads column 0: its x is zeroed and it is never stored, so every
    // load is unconditional and the loop body stays free of per-lane branches
    coff[i] = cv[i] ? (uint32_t)col * sizeof(T) : 0u;
    xraw[i] = ld16(xrow + coff[i]);  // unpacked after the first weight loads are in flight
  }

  float acc[NI][VEC];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[i][v] = 0.f;

  for (int s0 = 0; s0 < R; s0 += kSuper) {
    const int Rs = min(kSuper, R - s0);
    const int QB = NDOT * Rs;
    const int lead = (DEPTH - QB % DEPTH) % DEPTH;
    const int QBp = lead + QB;  // multiple of DEPTH: the phase boundary falls between two groups
    const int NQ = QBp + Rs;

    if (GATHER) {
      __syncthreads();  // previous super-chunk done with sidx
      for (int r = tid; r < Rs; r += nt) {
        const int n = a.core_idx[(size_t)b * a.K + r0 + s0 + r];
        sidx[r] = (n >= 0 && n < a.N) ? n : -1;
      }
      __syncthreads();
    }
    const int row_base = r0 + s0;
    // up-projection bias of "my" neurons, fetched ahead of the weight stream: loads return in
    // order, so waiting for it later never drains the ring
    uint32_t bias_bits = 0;  // raw element bits; converted only where used, after phase A
    if (!SWIGLU && a.b_up && tid < Rs) {
      const T braw = reinterpret_cast<const T*>(a.b_up)[decode_row_of<GATHER>(tid, row_base, sidx)];
      if constexpr (sizeof(T) == 4) bias_bits = __builtin_bit_cast(uint32_t, braw);
      else bias_bits = (uint32_t)__builtin_bit_cast(uint16_t, braw);
    }
    uint4 buf[DEPTH][NI];
#define CI_ISSUE(pos, slot)                                                                     \
  decode_issue<T, NI, SWIGLU, GATHER>((pos), lead, Rs, QB, NQ, gate, up, down, xrow, rowbytes, \
                                      row_base, sidx, coff, buf[slot])

#pragma unroll
    for (int s = 0; s < DEPTH; ++s) CI_ISSUE(s, s);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      // opaque to the optimiser, so that the unpacking (and with it the wait for x) is not
      // hoisted above the first weight loads
      asm volatile("" : "+v"(xraw[i].x), "+v"(xraw[i].y), "+v"(xraw[i].z), "+v"(xraw[i].w));
      unpack<D>(xraw[i], xr[i]);
      if (!cv[i]) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) xr[i][v] = 0.f;
      }
    }

    // ---- phase A: dots of the gate / up rows with x ----
    for (int g0 = 0; g0 < QBp; g0 += DEPTH) {
      float p[DEPTH];
#pragma unroll
      for (int s = 0; s < DEPTH; ++s) {
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
          float f[VEC];
          unpack<D>(buf[s][i], f);
#pragma unroll
          for (int v = 0; v < VEC; ++v) sum = fmaf(f[v], xr[i][v], sum);
        }
        p[s] = sum;  // filler positions give a value that is never stored
        // keep the ring order: the slot is refilled right after it has been consumed and
        // before the next slot is waited for (the scheduler would otherwise batch the loads)
        __builtin_amdgcn_sched_barrier(0);
        CI_ISSUE(g0 + s + DEPTH, s);
        __builtin_amdgcn_sched_barrier(0);
      }
      const float tot = wave_sum_rows<DEPTH>(p, lane);
      constexpr int SH = DEPTH == 16 ? 2 : (DEPTH == 8 ? 3 : 4);  // 64 / DEPTH lanes share a row
      const int q = g0 + (lane >> SH) - lead;
      if ((lane & ((1 << SH) - 1)) == 0 && q >= 0) red[wave * NDOT * kSuper + q] = tot;
    }
    CI_OSTAMP(1);
    __syncthreads();
    CI_OSTAMP(2);

    // ---- hidden value of each neuron of the super-chunk, fp32 ----
    if (tid < Rs) {  // Rs <= kSuper <= blockDim.x
      const int r = tid;
      float z0 = 0.f, z1 = 0.f;
      for (int w = 0; w < nw; ++w) {
        z0 += red[w * NDOT * kSuper + r];
        if (SWIGLU) z1 += red[w * NDOT * kSuper + Rs + r];
      }
      float h;
      if (SWIGLU) h = silu(z0) * z1;  // z0: gate, z1: up
      else {
        // opaque: keeps the conversion (and the wait for the bias load) down here
        asm volatile("" : "+v"(bias_bits));
        float bias;
        if constexpr (sizeof(T) == 4) bias = u2f(bias_bits);
        else bias = to_float<D>(__builtin_bit_cast(T, (uint16_t)bias_bits));
        h = fmaxf(z0 + bias, 0.f);
      }
      if (GATHER && sidx[r] < 0) h = 0.f;
      hbuf[r] = h;
    }
    __syncthreads();
    CI_OSTAMP(3);

    // ---- phase B: y += h_k * W_down_c[k, :] ----
    for (int g0 = QBp; g0 < NQ; g0 += DEPTH) {
#pragma unroll
      for (int s = 0; s < DEPTH; ++s) {
        const int pos = g0 + s;
        if (pos < NQ) {  // uniform; no load inside, so the load count stays path-independent
          const float hj = hbuf[pos - QBp];
#pragma unroll
          for (int i = 0; i < NI; ++i) {
            float f[VEC];
            unpack<D>(buf[s][i], f);
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[i][v] = fmaf(hj, f[v], acc[i][v]);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
        CI_ISSUE(pos + DEPTH, s);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // the filler loads issued past the end are still outstanding: drain them here (vmcnt(0)),
    // so that the next super-chunk's first loads need not wait on these registers
    __builtin_amdgcn_s_waitcnt(0x0F70);
    // red / hbuf are rewritten only after the next super-chunk's barriers
    __syncthreads();
#undef CI_ISSUE
  }

  CI_OSTAMP(4);
  const bool NT_STORE = a.nt_store != 0;
  float* out = a.partial + ((size_t)b * a.n_wg + wg) * a.d;
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    if (cv[i]) {
      const int col = (i * nt + tid) * VEC;
#pragma unroll
      for (int v = 0; v < VEC; v += 4) {
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        const f32x4 t = {acc[i][v], acc[i][v + 1], acc[i][v + 2], acc[i][v + 3]};
        if (NT_STORE) __builtin_nontemporal_store(t, reinterpret_cast<f32x4*>(out + col + v));
        else *reinterpret_cast<f32x4*>(out + col + v) = t;
      }
    }
  }
  CI_OSTAMP(5);
}

// y[b, c] = sum_w partial[b, w, c] + b_down[c].  256 threads = CQ column quads
// (4 * CQ columns, contiguous in every partial row) x 256 / CQ groups of
// partial rows.  A thread adds up the rows of its group (all its loads in
// flight at once), the groups that share a wave are added by a butterfly over
// the lanes (every lane of a column quad ends with the same sum), the four
// waves through LDS with a single barrier.  The order of summation is fixed,
// so the result is deterministic.
template <class D, int CQ, int NT>
__global__ __launch_bounds__(NT) void decode_reduce_kernel(const float* __restrict__ partial,
                                                           const void* __restrict__ b_down,
                                                           void* __restrict__ y, int n_wg, int d) {
  using T = typename D::T;
  constexpr int G = NT / CQ;
  constexpr int NW = NT / 64;
  __shared__ float4 sm[NW][CQ];
  const int tx = threadIdx.x % CQ, ty = threadIdx.x / CQ;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = (blockIdx.x * CQ + tx) * 4;
  const int b = blockIdx.y;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  float bias[4] = {0.f, 0.f, 0.f, 0.f};
  if (c < d) {
    if (b_down && threadIdx.x < CQ) {  // requested ahead of the partial sums
#pragma unroll
      for (int k = 0; k < 4; ++k) bias[k] = to_float<D>(reinterpret_cast<const T*>(b_down)[c + k]);
    }
    const float* p = partial + (size_t)b * n_wg * d + c;
#pragma unroll 8
    for (int w = ty; w < n_wg; w += G) {
      const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + (size_t)w * d));
      s.x += u2f(t[0]); s.y += u2f(t[1]); s.z += u2f(t[2]); s.w += u2f(t[3]);
    }
  }
  // lanes tx, tx + CQ, tx + 2 CQ, ... of a wave hold the same columns
#pragma unroll
  for (int m = CQ; m < 64; m <<= 1) {
    s.x += __shfl_xor(s.x, m);
    s.y += __shfl_xor(s.y, m);
    s.z += __shfl_xor(s.z, m);
    s.w += __shfl_xor(s.w, m);
  }
  if constexpr (NW > 1) {
    if (lane < CQ) sm[wave][lane] = s;
    __syncthreads();
  }
  if (threadIdx.x < CQ && c < d) {
    float4 t = s;
    if constexpr (NW > 1) {
      t = sm[0][tx];
#pragma unroll
      for (int w = 1; w < NW; ++w) {
        const float4 v = sm[w][tx];
        t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
      }
    }
    const float o[4] = {t.x + bias[0], t.y + bias[1], t.z + bias[2], t.w + bias[3]};
    T* yo = reinterpret_cast<T*>(y) + (size_t)b * d + c;
#pragma unroll
    for (int k = 0; k < 4; ++k) yo[k] = from_float<D>(o[k]);
  }
}

template <class D>
int launch_reduce_typed(const float* partial, const void* b_down, void* y, int n_wg, int d, int B,
                        hipStream_t s) {
  const int rt = params().reduce_threads;
#define CI_REDUCE(CQ_, NT_)                                                                              \
  hipLaunchKernelGGL((decode_reduce_kernel<D, CQ_, NT_>), dim3((d + 4 * CQ_ - 1) / (4 * CQ_), B), dim3(NT_), 0, s, \
                     partial, b_down, y, n_wg, d)
  switch (params().reduce_cq) {
    case 4:
      if (rt == 64) CI_REDUCE(4, 64); else if (rt == 128) CI_REDUCE(4, 128); else CI_REDUCE(4, 256);
      break;
    case 16:
      if (rt == 64) CI_REDUCE(16, 64); else if (rt == 128) CI_REDUCE(16, 128); else CI_REDUCE(16, 256);
      break;
    default:
      if (rt == 64) CI_REDUCE(8, 64); else if (rt == 128) CI_REDUCE(8, 128); else if (rt == 512) CI_REDUCE(8, 512);
      else if (rt == 1024) CI_REDUCE(8, 1024); else CI_REDUCE(8, 256);
  }
#undef CI_REDUCE
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

template <class D, int NI, bool SWIGLU, bool GATHER>
int launch_depth(const DecodeArgs& a, dim3 grid, dim3 block, size_t lds, hipStream_t s) {
  int depth = params().decode_depth;
  if (NI >= 4) depth = 4;                 // 1024-thread workgroups: 128 VGPRs
  if (NI == 3 && depth > 8) depth = 8;
  switch (depth) {
    case 4: hipLaunchKernelGGL((ffn_decode_kernel<D, NI, SWIGLU, GATHER, 4>), grid, block, lds, s, a); break;
    case 16: hipLaunchKernelGGL((ffn_decode_kernel<D, NI, SWIGLU, GATHER, 16>), grid, block, lds, s, a); break;
    default: hipLaunchKernelGGL((ffn_decode_kernel<D, NI, SWIGLU, GATHER, 8>), grid, block, lds, s, a); break;
  }
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

template <class D, bool SWIGLU, bool GATHER>
int launch_typed(const DecodeArgs& a, int B, int nt, int ni, const void* b_down, void* y,
                 hipStream_t s) {
  if (a.n_wg > 0) {
    const int nw = nt / 64;
    const size_t lds = (size_t)((SWIGLU ? 2 : 1) * nw + 2) * kSuper * sizeof(float);
    dim3 grid(a.n_wg, B), block(nt);
    int rc;
    switch (ni) {
      case 1: rc = launch_depth<D, 1, SWIGLU, GATHER>(a, grid, block, lds, s); break;
      case 2: rc = launch_depth<D, 2, SWIGLU, GATHER>(a, grid, block, lds, s); break;
      case 3: rc = launch_depth<D, 3, SWIGLU, GATHER>(a, grid, block, lds, s); break;
      case 4: rc = launch_depth<D, 4, SWIGLU, GATHER>(a, grid, block, lds, s); break;
      default: return CI_ERR_UNSUPPORTED;
    }
    if (rc != CI_OK) return rc;
  }
  return launch_reduce_typed<D>(a.partial, b_down, y, a.n_wg, a.d, B, s);
}

// Workgroup width for a row of `vecs` 16-byte vectors: NI loads per thread
// and row.  Up to three loads the workgroup has at most 512 threads (the
// register ring needs the 256-VGPR budget); four loads cover d up to 32768.
inline void pick_shape(int vecs, int* nt, int* ni) {
  for (int n = (vecs <= 64 ? 1 : 2); n <= 4; ++n) {
    const int t = ((vecs + n - 1) / n + 63) / 64 * 64;
    if (t <= (n >= 4 ? 1024 : 512)) { *nt = t; *ni = n; return; }
  }
  *nt = 1024;
  *ni = (vecs + 1023) / 1024;
}

template <class D>
int launch_dtype(const DecodeArgs& a, int B, int act, const void* b_down, void* y, hipStream_t s) {
  const int vecs = (a.d + D::VEC - 1) / D::VEC;
  int nt, ni;
  pick_shape(vecs, &nt, &ni);
  const int want = params().decode_threads / 64 * 64;  // tuning override, if it fits the bounds
  if (want >= 64) {
    const int n = (vecs + want - 1) / want;
    if (n <= 4 && want <= (n >= 4 ? 1024 : 512)) { nt = want; ni = n; }
  }
  const bool gather = a.core_idx != nullptr;
  if (act == CI_ACT_SWIGLU)
    return gather ? launch_typed<D, true, true>(a, B, nt, ni, b_down, y, s)
                  : launch_typed<D, true, false>(a, B, nt, ni, b_down, y, s);
  return gather ? launch_typed<D, false, true>(a, B, nt, ni, b_down, y, s)
                : launch_typed<D, false, false>(a, B, nt, ni, b_down, y, s);
}

}  // namespace

// Number of neuron slices (workgroups) per sentence.  Bounded by 1024 so the
// workspace size does not depend on the device.
int decode_splits(int64_t B, int64_t K) {
  if (K <= 0) return 0;
  DeviceInfo di;
  int cus = 256;
  if (device_info(&di) == CI_OK) cus = di.cus;
  int64_t n = ((int64_t)cus * params().decode_wgs_per_cu + B - 1) / B;
  if (params().decode_wgs > 0) n = params().decode_wgs;
  if (n > 1024) n = 1024;
  if (n > K) n = K;
  if (n < 1) n = 1;
  return (int)n;
}

int launch_decode_reduce(const float* partial, const void* b_down, void* y, int n_wg, int d, int B,
                         int dtype, hipStream_t s) {
  switch (dtype) {
    case CI_F32: return launch_reduce_typed<F32>(partial, b_down, y, n_wg, d, B, s);
    case CI_F16: return launch_reduce_typed<F16>(partial, b_down, y, n_wg, d, B, s);
    case CI_BF16: return launch_reduce_typed<BF16>(partial, b_down, y, n_wg, d, B, s);
  }
  return CI_ERR_BAD_DTYPE;
}

int launch_ffn_decode(const void* x, int64_t B, const ci_ffn_weights* w, int dtype, int act,
                      void* y, float* partial, hipStream_t s) {
  DecodeArgs a;
  a.x = x;
  a.w_up = w->w_up;
  a.w_gate = w->w_gate;
  a.b_up = w->b_up;
  a.w_down = w->w_down;
  a.core_idx = w->core_idx;
  a.partial = partial;
  a.K = (int)w->K;
  a.d = (int)w->d;
  a.N = (int)w->N;
  a.n_wg = decode_splits(B, w->K);
  a.nt_store = params().decode_nt_store;
  switch (dtype) {
    case CI_F32: return launch_dtype<F32>(a, (int)B, act, w->b_down, y, s);
    case CI_F16: return launch_dtype<F16>(a, (int)B, act, w->b_down, y, s);
    case CI_BF16: return launch_dtype<BF16>(a, (int)B, act, w->b_down, y, s);
  }
  return CI_ERR_BAD_DTYPE;
}

}  // namespace ci
