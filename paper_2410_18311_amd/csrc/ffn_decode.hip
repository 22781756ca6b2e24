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

namespace ci {

namespace {

constexpr int kSuper = 128;  // rows of a slice handled between two barriers

struct DecodeArgs {
  const void* x;
  const void* w_up;
  const void* w_gate;
  const void* b_up;
  const void* w_down;
  const int32_t* core_idx;
  float* partial;
  int K, d, N, n_wg;
};

template <class D, int NI, bool SWIGLU, bool GATHER>
__global__ __launch_bounds__(1024) void ffn_decode_kernel(DecodeArgs a) {
  using T = typename D::T;
  constexpr int VEC = D::VEC;
  // rows in flight per thread: at most 16 sixteen-byte loads outstanding
  constexpr int RCB = NI <= 2 ? 8 : 4;            // phase B
  constexpr int RCA = SWIGLU ? RCB / 2 : RCB;     // phase A (two matrices when gated)

  extern __shared__ float smem[];
  const int tid = threadIdx.x, nt = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
  const int wg = blockIdx.x, b = blockIdx.y;
  const int r0 = (int)(((int64_t)wg * a.K) / a.n_wg);
  const int r1 = (int)(((int64_t)(wg + 1) * a.K) / a.n_wg);
  const int R = r1 - r0;

  float* red_u = smem;                         // [nw][kSuper]
  float* red_g = red_u + nw * kSuper;          // [nw][kSuper] (SwiGLU only)
  float* hbuf = SWIGLU ? red_g + nw * kSuper : red_g;  // [kSuper]

  const int32_t* idx = GATHER ? a.core_idx + (size_t)b * a.K + r0 : nullptr;
  const size_t rowbytes = (size_t)a.d * sizeof(T);
  const char* up = reinterpret_cast<const char*>(a.w_up);
  const char* gate = reinterpret_cast<const char*>(a.w_gate);
  const char* down = reinterpret_cast<const char*>(a.w_down);

  // Row of the weight matrices that slice-local neuron r names; `ok` is false
  // for a gathered index outside [0, N) (it then contributes nothing).
  auto row_of = [&](int r, bool& ok) -> size_t {
    if (GATHER) {
      int n = idx[r];
      ok = (n >= 0) && (n < a.N);
      return ok ? (size_t)n : (size_t)0;
    }
    ok = true;
    return (size_t)(r0 + r);
  };

  // columns owned by this thread
  int col[NI];
  bool cv[NI];
  float xr[NI][VEC];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    col[i] = (i * nt + tid) * VEC;
    cv[i] = col[i] < a.d;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (cv[i]) v = ld16(reinterpret_cast<const T*>(a.x) + (size_t)b * a.d + col[i]);
    unpack<D>(v, xr[i]);
  }

  float acc[NI][VEC];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[i][v] = 0.f;

  for (int s0 = 0; s0 < R; s0 += kSuper) {
    const int Rs = min(kSuper, R - s0);

    // ---- phase A: z_k = <W_up_c[k, :], x> (and the gate's) ----
    for (int rb = 0; rb < Rs; rb += RCA) {
      uint4 wu[RCA][NI];
      uint4 wgt[SWIGLU ? RCA : 1][NI];
#pragma unroll
      for (int j = 0; j < RCA; ++j) {
        const int r = s0 + min(rb + j, Rs - 1);
        bool ok;
        const size_t row = row_of(r, ok);
        const char* pu = up + row * rowbytes;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
          wu[j][i] = make_uint4(0, 0, 0, 0);
          if (cv[i]) wu[j][i] = ld16(pu + (size_t)col[i] * sizeof(T));
        }
        if (SWIGLU) {
          const char* pg = gate + row * rowbytes;
#pragma unroll
          for (int i = 0; i < NI; ++i) {
            wgt[j][i] = make_uint4(0, 0, 0, 0);
            if (cv[i]) wgt[j][i] = ld16(pg + (size_t)col[i] * sizeof(T));
          }
        }
      }
      float pu_[RCA], pg_[RCA];
#pragma unroll
      for (int j = 0; j < RCA; ++j) {
        float su = 0.f, sg = 0.f;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
          float f[VEC];
          unpack<D>(wu[j][i], f);
#pragma unroll
          for (int v = 0; v < VEC; ++v) su = fmaf(f[v], xr[i][v], su);
          if (SWIGLU) {
            unpack<D>(wgt[j][i], f);
#pragma unroll
            for (int v = 0; v < VEC; ++v) sg = fmaf(f[v], xr[i][v], sg);
          }
        }
        pu_[j] = wave_sum(su);
        if (SWIGLU) pg_[j] = wave_sum(sg);
      }
      if (lane == 0) {
#pragma unroll
        for (int j = 0; j < RCA; ++j) {
          if (rb + j < Rs) {
            red_u[wave * kSuper + rb + j] = pu_[j];
            if (SWIGLU) red_g[wave * kSuper + rb + j] = pg_[j];
          }
        }
      }
    }
    __syncthreads();

    // ---- hidden value of each neuron of the slice, fp32 ----
    for (int r = tid; r < Rs; r += nt) {
      float zu = 0.f, zg = 0.f;
      for (int w = 0; w < nw; ++w) {
        zu += red_u[w * kSuper + r];
        if (SWIGLU) zg += red_g[w * kSuper + r];
      }
      bool ok;
      const size_t row = row_of(s0 + r, ok);
      float h;
      if (SWIGLU) {
        h = silu(zg) * zu;
      } else {
        if (a.b_up) zu += to_float<D>(reinterpret_cast<const T*>(a.b_up)[row]);
        h = fmaxf(zu, 0.f);
      }
      hbuf[r] = ok ? h : 0.f;
    }
    __syncthreads();

    // ---- phase B: y += h_k * W_down_c[k, :] ----
    for (int rb = 0; rb < Rs; rb += RCB) {
      uint4 wd[RCB][NI];
#pragma unroll
      for (int j = 0; j < RCB; ++j) {
        const int r = s0 + min(rb + j, Rs - 1);
        bool ok;
        const size_t row = row_of(r, ok);
        const char* pd = down + row * rowbytes;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
          wd[j][i] = make_uint4(0, 0, 0, 0);
          if (cv[i]) wd[j][i] = ld16(pd + (size_t)col[i] * sizeof(T));
        }
      }
#pragma unroll
      for (int j = 0; j < RCB; ++j) {
        const float hj = (rb + j < Rs) ? hbuf[rb + j] : 0.f;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
          float f[VEC];
          unpack<D>(wd[j][i], f);
#pragma unroll
          for (int v = 0; v < VEC; ++v) acc[i][v] = fmaf(hj, f[v], acc[i][v]);
        }
      }
    }
    // the next super-chunk's phase A writes red_*, its h pass writes hbuf only
    // after the barrier that follows phase A, which every thread reaches after
    // finishing the reads above.
  }

  float* out = a.partial + ((size_t)b * a.n_wg + wg) * a.d;
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    if (cv[i]) {
#pragma unroll
      for (int v = 0; v < VEC; v += 4)
        *reinterpret_cast<float4*>(out + col[i] + v) =
            make_float4(acc[i][v], acc[i][v + 1], acc[i][v + 2], acc[i][v + 3]);
    }
  }
}

// y[b, c] = sum_w partial[b, w, c] + b_down[c]; 256 threads = 16 column
// quads x 16 partial groups; fixed summation order.
template <class D>
__global__ __launch_bounds__(256) void decode_reduce_kernel(const float* __restrict__ partial,
                                                            const void* __restrict__ b_down,
                                                            void* __restrict__ y, int n_wg, int d) {
  using T = typename D::T;
  __shared__ float4 sm[16][17];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int c = (blockIdx.x * 16 + tx) * 4;
  const int b = blockIdx.y;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (c < d) {
    const float* p = partial + (size_t)b * n_wg * d + c;
    for (int w = ty; w < n_wg; w += 16) {
      const float4 v = *reinterpret_cast<const float4*>(p + (size_t)w * d);
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
  }
  sm[ty][tx] = s;
  __syncthreads();
  if (ty == 0 && c < d) {
    float4 t = sm[0][tx];
#pragma unroll
    for (int k = 1; k < 16; ++k) {
      const float4 v = sm[k][tx];
      t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
    }
    float o[4] = {t.x, t.y, t.z, t.w};
    if (b_down) {
#pragma unroll
      for (int k = 0; k < 4; ++k) o[k] += to_float<D>(reinterpret_cast<const T*>(b_down)[c + k]);
    }
    T* yo = reinterpret_cast<T*>(y) + (size_t)b * d + c;
#pragma unroll
    for (int k = 0; k < 4; ++k) yo[k] = from_float<D>(o[k]);
  }
}

template <class D, bool SWIGLU, bool GATHER>
int launch_typed(const DecodeArgs& a, int B, int nt, int ni, const void* b_down, void* y,
                 hipStream_t s) {
  if (a.n_wg > 0) {
    const int nw = nt / 64;
    const size_t lds = (size_t)((SWIGLU ? 2 : 1) * nw + 1) * kSuper * sizeof(float);
    dim3 grid(a.n_wg, B), block(nt);
    switch (ni) {
      case 1: hipLaunchKernelGGL((ffn_decode_kernel<D, 1, SWIGLU, GATHER>), grid, block, lds, s, a); break;
      case 2: hipLaunchKernelGGL((ffn_decode_kernel<D, 2, SWIGLU, GATHER>), grid, block, lds, s, a); break;
      case 3: hipLaunchKernelGGL((ffn_decode_kernel<D, 3, SWIGLU, GATHER>), grid, block, lds, s, a); break;
      case 4: hipLaunchKernelGGL((ffn_decode_kernel<D, 4, SWIGLU, GATHER>), grid, block, lds, s, a); break;
      default: return CI_ERR_UNSUPPORTED;
    }
    CI_HIP_CHECK_LAUNCH();
  }
  dim3 rgrid((a.d + 63) / 64, B);
  hipLaunchKernelGGL((decode_reduce_kernel<D>), rgrid, dim3(256), 0, s, a.partial, b_down, y,
                     a.n_wg, a.d);
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

template <class D>
int launch_dtype(const DecodeArgs& a, int B, int act, const void* b_down, void* y, hipStream_t s) {
  // threads per workgroup: aim at two 16-byte loads per thread and row
  int nt = params().decode_threads;
  if (nt <= 0) {
    const int vecs = (a.d + D::VEC - 1) / D::VEC;
    nt = ((vecs + 1) / 2 + 63) / 64 * 64;
  }
  nt = nt < 64 ? 64 : (nt > 1024 ? 1024 : nt / 64 * 64);
  const int ni = (a.d + nt * D::VEC - 1) / (nt * D::VEC);
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
  if (n > 1024) n = 1024;
  if (n > K) n = K;
  if (n < 1) n = 1;
  return (int)n;
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
  switch (dtype) {
    case CI_F32: return launch_dtype<F32>(a, (int)B, act, w->b_down, y, s);
    case CI_F16: return launch_dtype<F16>(a, (int)B, act, w->b_down, y, s);
    case CI_BF16: return launch_dtype<BF16>(a, (int)B, act, w->b_down, y, s);
  }
  return CI_ERR_BAD_DTYPE;
}

}  // namespace ci
