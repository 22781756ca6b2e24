// Decode-stage FFN over the frozen core set (Sec. 4.2 of arXiv 2410.18311) in
// ONE launch, for compact buffers whose down matrix is kept output-major:
//   w_up_c, w_gate_c [K, d]   (rows of the core neurons)
//   w_down_o         [d, ldk] (w_down[:, S]: one row per output, K core columns)
//   y = w_down_o act(w_up_c x [+ b]) [+ b_down]
// Every weight byte is read exactly once and nothing but y is written to HBM:
// there are no partial output vectors and no second kernel.
//
// Work split.  The K neurons are cut into C >= 2 chunks.  Workgroup w
//   phase A(i): computes the hidden values of ITS share of chunk i (rows of
//               w_up_c / w_gate_c dotted with x) and publishes them,
//   phase B(i): adds chunk i's contribution to ITS d / n_wg outputs (row
//               segments of w_down_o dotted with the chunk's hidden values,
//               which all workgroups produced in A(i)).
// The order is A(0) .. A(C-1), B(0) .. B(C-1): B(i) uses hidden values that
// were published C - 1 phases earlier, so in the normal case they are there
// long before they are needed and no workgroup waits for another.
//
// Waves.  All waves but the last two are COMPUTE waves: they do nothing but
// stream weight rows through a register ring (DEPTH rows in flight per thread,
// a slot refilled right after it has been consumed) and dot them with a
// register resident vector (x in A, the chunk's hidden values in B); the ring
// never drains between phases, the loads of the next phase are issued one
// group ahead by a cursor that walks the same (phase, group) sequence.  Where a
// chunk's row segment of w_down_o is narrower than the workgroup, several
// output rows are dotted side by side by sets of waves.  The last two waves
// are SERVICE waves: at the end of A(i) the first of them sums the compute
// waves' partial dots, applies bias and activation and publishes the
// workgroup's hidden values; both then collect the whole chunk (everybody's
// values) into LDS, from where the compute waves take their 16-byte position
// at the start of B(i); at the end of B(i) the first folds the compute waves'
// partial outputs into the workgroup's outputs and, after the last phase,
// writes y.  The two kinds of waves meet only at the workgroup barrier that
// ends each phase.
//
// Exchange of the hidden values.  Each value is one 8-byte word {tag, fp32
// bits} written with a single device-scope store; tag = epoch + 1, where the
// epoch word lives in the workspace and is bumped once per call (by workgroup
// 0, after every workgroup has read it: it cannot finish before all values are
// published).  A reader accepts a word only if it carries the call's tag, so a
// word is its own "ready" flag: no fences, no read-modify-write atomics, no
// counters to reset, and replaying the launch from a HIP graph works because
// the epoch advances on the device.  The workspace must have been zeroed once
// before its first use.  The service wave first reads a chunk with ordinary
// (cacheable) loads -- the 32 workgroups behind one L2 then fetch it from
// memory once -- and polls only the words that do not carry the tag yet, with
// device-scope loads, a bounded number of times; if the bound is hit (another
// launch holding compute units so that the grid is not co-resident) the error
// word is set and zeros are used, so every wave always exits.
#include <algorithm>

#include "common.hpp"
#include "decode_common.hpp"

namespace ci {

namespace {

constexpr int kServiceWaves = 2;  // waves per workgroup that publish and collect hidden values

struct FusedArgs {
  const void* x;
  const void* w_up;
  const void* w_gate;
  const void* b_up;
  const void* w_down;  // [d, ldk]
  const void* b_down;
  void* y;
  uint32_t* hdr;               // [0] epoch, [1] error
  unsigned long long* hws;     // {tag, fp32 bits} per neuron
  int K, d, ldk, n_wg;
  int C, S;                    // chunks; neurons per chunk (the last chunk takes the rest: S - VEC < rest <= hcap)
  int hcap;                    // neurons the largest chunk holds, rounded up to whole 16-byte positions
  int rmax;                    // most outputs a workgroup owns
  int spin_limit;
  int guard_ticks;             // 10 ns ticks after a phase's end before the service waves collect its hidden values
#ifdef CI_FUSED_STAMPS
  unsigned long long* stamps;  // development build: 100 MHz time stamps
  int ablate;                  // development build: 1 = A phases only, 2 = B phases only (outputs are then wrong)
#endif
};

#ifdef CI_FUSED_STAMPS
// [8 calls][256 workgroups][compute wave 0 | service wave][32 stamps]
#define CI_STAMP(i)                                                                                      \
  do {                                                                                                   \
    if ((threadIdx.x & 63) == 0 && (wave == 0 || wave == nwc))                                           \
      a.stamps[(((size_t)(stamp_slot & 7u) * 256 + wg) * 2 + (wave == nwc)) * 32 + (i)] =                \
          __builtin_amdgcn_s_memrealtime();                                                              \
  } while (0)
#else
#define CI_STAMP(i) do { } while (0)
#endif

// One phase as the issuing or the consuming side sees it (all fields uniform).
struct Phase {
  int ngroups;         // ring groups
  int Q;               // ring items: NDOT * Ra rows (A), or ceil(R / RG) sets of RG rows (B)
  int rows;            // rows to dot: NDOT * Ra (A) or R, the outputs of this workgroup (B)
  int RG, PBw;         // B: RG rows are dotted side by side, each by PBw waves (A: 1 row by all waves)
  int Ra;              // A: neurons of this workgroup in the chunk
  int lim;             // 16-byte positions of a row that exist (others re-read position 0)
  int row0;            // A: first neuron (row of w_up_c); B: first output (row of w_down_o)
  const char* b0;      // A, SwiGLU: first gate row
  const char* b1;      // A: first up row; B: first row segment
  uint32_t stride;     // bytes between consecutive rows (< 2^23)
};

template <int DEPTH>
__device__ __forceinline__ float wave_rows(float (&v)[DEPTH], int lane) {
  static_assert(DEPTH == 4 || DEPTH == 8 || DEPTH == 16, "ring depth");
  halve_rows<DEPTH, 32>(v, lane);
  return v[0];
}

// B phases, one load per thread and row (NI == 1): a chunk row segment has Pn 16-byte positions, often far
// fewer than the workgroup has compute lanes.  So PBw = ceil(Pn / 64) waves take one row and the
// nwc / PBw such wave sets work on RG different rows at the same time (one ring item = RG rows).
template <class D, bool SWIGLU, int DEPTH, int NI>
__device__ __forceinline__ void describe(const FusedArgs& a, int ph, int wg, int nwc, Phase* p) {
  using T = typename D::T;
  constexpr int VEC = D::VEC;
  constexpr int NDOT = SWIGLU ? 2 : 1;
  const bool isB = ph >= a.C;
  const int i = isB ? ph - a.C : ph;
  const int k0 = i * a.S;
  const int Kc = i == a.C - 1 ? a.K - k0 : a.S;
  if (!isB) {
    // wg * Kc < 2^32: a chunk holds at most kSuper neurons per workgroup
    const int ra0 = k0 + (int)(((uint32_t)wg * (uint32_t)Kc) / (uint32_t)a.n_wg);
    const int ra1 = k0 + (int)(((uint32_t)(wg + 1) * (uint32_t)Kc) / (uint32_t)a.n_wg);
    p->Ra = ra1 - ra0;
    p->Q = NDOT * p->Ra;
    p->rows = p->Q;
    p->RG = 1;
    p->PBw = nwc;
    p->ngroups = (p->Q + DEPTH - 1) / DEPTH;
#ifdef CI_FUSED_STAMPS
    if (a.ablate == 2) p->ngroups = 0;
#endif
    p->lim = a.d / VEC;
    p->row0 = ra0;
    p->stride = (uint32_t)a.d * (uint32_t)sizeof(T);
    p->b0 = reinterpret_cast<const char*>(a.w_gate) + (size_t)ra0 * p->stride;
    p->b1 = reinterpret_cast<const char*>(a.w_up) + (size_t)ra0 * p->stride;
  } else {
    const int c0 = (int)(((uint32_t)wg * (uint32_t)a.d) / (uint32_t)a.n_wg);  // d <= 2^15, wg < 2^16
    const int c1 = (int)(((uint32_t)(wg + 1) * (uint32_t)a.d) / (uint32_t)a.n_wg);
    const int R = c1 - c0;
    const int Pn = (Kc + VEC - 1) / VEC;
    p->Ra = 0;
    p->PBw = NI == 1 ? max((Pn + 63) >> 6, 1) : nwc;
    p->RG = 1;
    for (int t = 2 * p->PBw; t <= nwc; t += p->PBw) ++p->RG;  // nwc / PBw
    p->rows = R;
    p->Q = (R + p->RG - 1) / p->RG;
    p->ngroups = (R > 0 && Pn > 0) ? (p->Q + DEPTH - 1) / DEPTH : 0;
#ifdef CI_FUSED_STAMPS
    if (a.ablate == 1) p->ngroups = 0;
#endif
    p->lim = Pn;
    p->row0 = c0;
    p->stride = (uint32_t)a.ldk * (uint32_t)sizeof(T);
    p->b0 = nullptr;
    p->b1 = reinterpret_cast<const char*>(a.w_down) + ((size_t)c0 * a.ldk + k0) * sizeof(T);
  }
}

// LDS: red  [2][nwc][NDOT * kSuper]  wave partial dots of an A phase (double-buffered by phase parity),
//      yred [2][nwc][rmax]           wave partial outputs of a B phase (double-buffered by phase parity),
//      ysum [rmax]                   this workgroup's outputs, summed over the B phases (service wave 0 only),
//      hbuf [2][hcap]                a chunk's hidden values (by chunk parity)
__host__ __device__ __forceinline__ int lds_red_floats(int nwc, int ndot) { return 2 * nwc * ndot * kSuper; }
__host__ __device__ __forceinline__ int lds_yred_floats(int nwc, int rmax) {
  return (2 * nwc * rmax + rmax + 3) & ~3;  // yred and ysum; keeps hbuf 16-byte aligned
}

// ---- the service wave ---------------------------------------------------------
// After barrier b (the end of phase b), b < C: publishes this workgroup's hidden values of chunk b.
// Then collects into LDS every chunk j that has been published (j <= b, j < C) and whose buffer
// (chunk parity) the compute waves no longer read (j < 2, or B(j - 2) has ended: b >= C + j - 2).
// B(j) starts after barrier C + j - 1, which this wave reaches only when chunk j is in LDS.
template <class D, bool SWIGLU, int DEPTH, int NI>
__device__ __forceinline__ void service_wave(const FusedArgs& a, float* smem, int nwc, int sv, int lane, int wg,
                                             uint32_t tag) {
  using T = typename D::T;
  constexpr int VEC = D::VEC;
  constexpr int NDOT = SWIGLU ? 2 : 1;
  float* red = smem;
  const float* yred = smem + lds_red_floats(nwc, NDOT);
  float* ysum = smem + lds_red_floats(nwc, NDOT) + 2 * nwc * a.rmax;
  float* hbuf = smem + lds_red_floats(nwc, NDOT) + lds_yred_floats(nwc, a.rmax);
  const int hcap = a.hcap;  // floats per chunk buffer
  const int nph = 2 * a.C;
  int failed = 0;
  if (sv == 0)
    for (int r = lane; r < a.rmax; r += 64) ysum[r] = 0.f;
  int fetched = 0;  // chunks [0, fetched) are (or have been) in LDS
  __builtin_amdgcn_s_setprio(3);  // few instructions, all on the critical path of the next phase
#ifdef CI_FUSED_STAMPS
  const int wave = nwc + sv;
  const uint32_t stamp_slot = tag - 1u;
#endif
  const __amdgpu_buffer_rsrc_t hrsrc = __builtin_amdgcn_make_buffer_rsrc(a.hws, 0, 0x7fffffff, 0x00020000);
  for (int b = 0; b < nph; ++b) {
    Phase p;
    describe<D, SWIGLU, DEPTH, NI>(a, b, wg, nwc, &p);
    // the up bias of "my" neuron of this chunk, asked for before the wait at the barrier
    float bias = 0.f;
    if (!SWIGLU && sv == 0 && b < a.C && a.b_up && lane < p.Ra)
      bias = to_float<D>(reinterpret_cast<const T*>(a.b_up)[p.row0 + lane]);
    __syncthreads();  // end of phase b
    const unsigned long long t_barrier = __builtin_amdgcn_s_memrealtime();
    CI_STAMP(2 + b);
    if (sv == 0 && b < a.C && lane < p.Ra) {
      // ---- hidden values of this workgroup's neurons of chunk b: fp32, published with the tag ----
      const float* redp = red + (b & 1) * nwc * NDOT * kSuper;
      float z0 = 0.f, z1 = 0.f;
      for (int w = 0; w < nwc; ++w) {
        z0 += redp[w * NDOT * kSuper + lane];
        if (SWIGLU) z1 += redp[w * NDOT * kSuper + p.Ra + lane];
      }
      const float h = SWIGLU ? silu(z0) * z1 : fmaxf(z0 + bias, 0.f);  // z0: gate (SwiGLU), z1: up
      const unsigned long long word = ((unsigned long long)f2u(h) << 32) | (unsigned long long)tag;
      __hip_atomic_store(a.hws + p.row0 + lane, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (sv == 0 && b >= a.C && p.ngroups > 0) {
      // ---- end of a B phase: this chunk's share of the workgroup's outputs.  Row r was item r / RG
      // of the wave set r % RG; its PBw waves each hold a partial sum. ----
      const float* yp = yred + (b & 1) * nwc * a.rmax;
      for (int r = lane; r < p.rows; r += 64) {
        const int q = r / p.RG, rg = r - q * p.RG;
        float t = 0.f;
        for (int wp = 0; wp < p.PBw; ++wp) t += yp[(rg * p.PBw + wp) * a.rmax + q];
        ysum[r] += t;
      }
    }
    // red and yred are double-buffered by phase parity: a buffer is rewritten two phases later, after
    // the next barrier, which this wave reaches only after it has read the buffer
    while (fetched < a.C && fetched <= b && (fetched < 2 || b >= a.C + fetched - 2)) {
      const int j = fetched;
      // The other workgroups publish at about the same time as this one; asking right away would
      // mostly find words that are not there yet (and leave incomplete lines in the L2 for the
      // workgroups behind it).  So this wave first lets `guard` ticks of the 100 MHz clock pass
      // since the barrier.
      if (b + 1 < nph) {
        for (int spins = 0; spins < a.spin_limit; ++spins) {
          if ((long long)(__builtin_amdgcn_s_memrealtime() - t_barrier) >= (long long)a.guard_ticks) break;
          __builtin_amdgcn_s_sleep(2);
        }
      }
      const int k0 = j * a.S;
      const int kc = j == a.C - 1 ? a.K - k0 : a.S;
      float* dst = hbuf + (j & 1) * hcap;
      const uint32_t boff = (uint32_t)k0 * 8u;  // byte offset of the chunk's first word
      // Two words per 16-byte load, UNR loads per lane in flight, the service waves taking alternate
      // kilobytes.  A vector with a word that does not carry the tag is read again, a bounded number
      // of times.
      constexpr int UNR = 16;
      for (int v0 = 0; v0 * 2 < hcap; v0 += 64 * UNR * kServiceWaves) {
        uint4 t[UNR];
        uint32_t need = 0;  // bit u: vector u still has a word without the tag
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
          const int v = v0 + (u * kServiceWaves + sv) * 64 + lane;
          if (v * 2 < kc) need |= 1u << u;
          t[u] = make_uint4(0, 0, 0, 0);
        }
        for (int pass = 0; __any(need != 0); ++pass) {
          if (pass > a.spin_limit) { failed = 1; break; }
          if (pass > 0) __builtin_amdgcn_s_sleep(8);
#pragma unroll
          for (int u = 0; u < UNR; ++u) {
            if (need & (1u << u)) {
              const int v = v0 + (u * kServiceWaves + sv) * 64 + lane;
              // first an ordinary load: behind one L2 the chunk then comes from the memory side once,
              // not once per workgroup; after that device-scope loads, which never see a line that an
              // L2 cached before all its words were written
              const u32x4 r = pass == 0 ? __builtin_amdgcn_raw_buffer_load_b128(hrsrc, (int)(boff + (uint32_t)v * 16u), 0, 0)
                                        : __builtin_amdgcn_raw_buffer_load_b128(hrsrc, (int)(boff + (uint32_t)v * 16u), 0,
                                                                                16 /* device scope */);
              t[u] = make_uint4(r[0], r[1], r[2], r[3]);
            }
          }
#pragma unroll
          for (int u = 0; u < UNR; ++u) {
            const int v = v0 + (u * kServiceWaves + sv) * 64 + lane;
            if (t[u].x == tag && (v * 2 + 1 >= kc || t[u].z == tag)) need &= ~(1u << u);
          }
#ifdef CI_FUSED_STAMPS
          if (sv == 0 && v0 == 0 && pass < 5) {
            const unsigned long long mm = __ballot(need != 0);  // depends on the loaded words
            if (lane == 0) {
              a.stamps[(((size_t)(stamp_slot & 7u) * 256 + wg) * 2 + 1) * 32 + 20 + j * 5 + pass] =
                  __builtin_amdgcn_s_memrealtime() + (mm == 0x123456789abcdefull);
              if (pass == 0) a.stamps[(((size_t)(stamp_slot & 7u) * 256 + wg) * 2 + 0) * 32 + 20 + j] = (unsigned long long)__popcll(mm);
            }
          }
#endif
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
          const int v = v0 + (u * kServiceWaves + sv) * 64 + lane;
          const int k = v * 2;
          if (k + 1 < hcap) {
            const float h0 = (k < kc && t[u].x == tag) ? u2f(t[u].y) : 0.f;  // zero past the chunk's last neuron
            const float h1 = (k + 1 < kc && t[u].z == tag) ? u2f(t[u].w) : 0.f;
            *reinterpret_cast<float2*>(dst + k) = make_float2(h0, h1);
          }
        }
      }
      CI_STAMP(16 + j);
      ++fetched;
    }
  }
  if (failed && lane == 0) __hip_atomic_store(a.hdr + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (sv == 0) {
    // ---- the workgroup's outputs ----
    const int c0 = (int)(((uint32_t)wg * (uint32_t)a.d) / (uint32_t)a.n_wg);
    const int c1 = (int)(((uint32_t)(wg + 1) * (uint32_t)a.d) / (uint32_t)a.n_wg);
    for (int r = lane; r < c1 - c0; r += 64) {
      float t = ysum[r];
      if (a.b_down) t += to_float<D>(reinterpret_cast<const T*>(a.b_down)[c0 + r]);
      reinterpret_cast<T*>(a.y)[c0 + r] = from_float<D>(t);
    }
    CI_STAMP(31);
    // every workgroup has read the epoch: this one could not have collected its last chunk otherwise
    if (wg == 0 && lane == 0) __hip_atomic_store(a.hdr, tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// AUX: cache policy of the ring loads.  >= 0: buffer instruction bits (2 = non-temporal, 16 = device
// scope); -1: non-temporal global loads; -2: plain global loads.
template <class D, int NI, bool SWIGLU, int DEPTH, int AUX>
__global__ __launch_bounds__(1024) void ffn_decode_fused_kernel(FusedArgs a) {
  using T = typename D::T;
  constexpr int VEC = D::VEC;
  constexpr int NDOT = SWIGLU ? 2 : 1;
  constexpr int SH = DEPTH == 16 ? 2 : (DEPTH == 8 ? 3 : 4);  // 64 / DEPTH lanes share a row

  extern __shared__ float smem[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // in a scalar register: row addresses depend on it
  const int nwc = (blockDim.x >> 6) - kServiceWaves;  // compute waves
  const int ntc = nwc * 64;               // compute threads
  const int wg = blockIdx.x;
  const int nph = 2 * a.C;

  // the call's tag; the epoch word is rewritten only after every workgroup has published with it
  const uint32_t tag = __hip_atomic_load(a.hdr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u;
  if (wave >= nwc) {
    service_wave<D, SWIGLU, DEPTH, NI>(a, smem, nwc, wave - nwc, lane, wg, tag);
    return;
  }
#ifdef CI_FUSED_STAMPS
  const uint32_t stamp_slot = tag - 1u;  // the last eight calls are kept
#endif
  CI_STAMP(0);

  float* red = smem;
  float* yred = red + lds_red_floats(nwc, NDOT);
  const float* hbuf = yred + lds_yred_floats(nwc, a.rmax);
  const int hcap = a.hcap;

  const char* xrow = reinterpret_cast<const char*>(a.x);
  int pidx[NI];
  uint4 xraw[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    pidx[i] = i * ntc + tid;
    // a position past the end re-reads position 0 (its vector entry is zeroed below)
    xraw[i] = ld16(xrow + (pidx[i] * VEC < a.d ? (size_t)pidx[i] * 16 : (size_t)0));
  }

  // ---- issue side: one group ahead of the consuming side ----
  // Per group and wave (all in scalar registers): item s of the group reads
  // (s < isel ? ibase0 : ibase1) + s * istride when s < ivalid, x otherwise; a lane adds ioffv, 16 times
  // its position in the row (0 when it has none), which changes only from phase to phase.
  Phase ip;
  int iph = -1, ig = 0;
  ip.ngroups = 0;
  const char* ibase0 = xrow;
  const char* ibase1 = xrow;
  uint32_t istride = 0;
  int isel = 0, ivalid = 0, irg = 0;
  uint32_t ioffv[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) ioffv[i] = 0;
  auto issue_advance = [&]() {
    ++ig;
    while (ig >= ip.ngroups && iph < nph) {
      ++iph;
      ig = 0;
      if (iph < nph) {
        describe<D, SWIGLU, DEPTH, NI>(a, iph, wg, nwc, &ip);
        // this wave's row set and this lane's position for the whole phase
        int wp = wave;
        irg = 0;
        if (iph >= a.C && NI == 1)
          while (wp >= ip.PBw) { wp -= ip.PBw; ++irg; }
#pragma unroll
        for (int i = 0; i < NI; ++i) {
          const int pos = (iph >= a.C && NI == 1) ? wp * 64 + lane : pidx[i];
          ioffv[i] = (pos < ip.lim && irg < ip.RG) ? (uint32_t)pos * 16u : 0u;
        }
      } else {
        ip.ngroups = 0;
      }
    }
    ivalid = 0;
    if (iph < nph) {
      const bool isB = iph >= a.C;
      const int r0 = ig * DEPTH * ip.RG + irg;  // this wave's first row of the group
      istride = ip.stride * (uint32_t)ip.RG;
      ivalid = irg < ip.RG ? max(min((ip.rows - r0 + ip.RG - 1) / ip.RG, DEPTH), 0) : 0;
      const size_t goff = (size_t)r0 * ip.stride;
      // SwiGLU A phase: rows [0, Ra) come from the gate matrix, rows [Ra, 2 Ra) from the up matrix
      isel = (SWIGLU && !isB) ? max(min(ip.Ra - r0, DEPTH), 0) : 0;
      ibase0 = ip.b0 + goff;
      ibase1 = ip.b1 + goff - ((SWIGLU && !isB) ? (size_t)ip.Ra * ip.stride : (size_t)0);
    }
  };
  uint4 buf[DEPTH][NI];
  // Loads of ring position s of the issue cursor's group into slot s.  Every position issues
  // exactly NI 16-byte loads (past the end: of x, which is cache resident) with one and the same
  // instruction and no branch around it, so the number of loads in flight is the same on every
  // path and the waits can be counted exactly.  Only the base address (scalar) and the lane's
  // offset differ: a row of w_gate_c / w_up_c, a row segment of w_down_o, or x.
  auto issue = [&](int s) {
    const bool valid = s < ivalid;
    const char* rowp = ((SWIGLU && s < isel) ? ibase0 : ibase1) + (uint32_t)s * istride;
    const char* base = valid ? rowp : xrow;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const uint32_t off = valid ? ioffv[i] : 0u;
      if constexpr (AUX >= 0) {
        const __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(base), 0, 0x7fffffff, 0x00020000);
        const u32x4 t = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, AUX);
        buf[s][i] = make_uint4(t[0], t[1], t[2], t[3]);
      } else if constexpr (AUX == -1) {
        buf[s][i] = ld16_stream(base + off);
      } else {
        buf[s][i] = ld16(base + off);
      }
    }
  };

  issue_advance();  // to the first group that exists
#pragma unroll
  for (int s = 0; s < DEPTH; ++s) {
    issue(s);
    __builtin_amdgcn_sched_barrier(0);  // in slot order, as the loop refills them
  }
  issue_advance();
  CI_STAMP(1);

  // the vector the rows are dotted with: x during the A phases, a chunk's hidden values during B
  float vr[NI][VEC];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    // opaque to the optimiser, so that the unpacking (and with it the wait for x) is not hoisted
    // above the first weight loads
    asm volatile("" : "+v"(xraw[i].x), "+v"(xraw[i].y), "+v"(xraw[i].z), "+v"(xraw[i].w));
    unpack<D>(xraw[i], vr[i]);
    if (pidx[i] * VEC >= a.d) {
#pragma unroll
      for (int v = 0; v < VEC; ++v) vr[i][v] = 0.f;
    }
  }

  // ---- consuming side: ONE loop over all groups of all phases ----
  // Its first part (dots + refills) is a single basic block that owns the ring registers, so they
  // are never copied and never waited for as a whole; everything with control flow comes after it.
  Phase cp;
  int ph = -1, g = 0;
  cp.ngroups = 0;
  bool cact = true;  // this wave has rows in the current phase
  // moves to the next group; a phase that ends meets the service waves at the barrier, and a B phase
  // that begins takes its hidden values out of LDS
  auto consume_advance = [&]() {
    ++g;
    while (g >= cp.ngroups && ph < nph) {
      if (ph >= 0) {
        __syncthreads();  // end of phase ph
        CI_STAMP(2 + ph);
      }
      ++ph;
      g = 0;
      if (ph < nph) {
        describe<D, SWIGLU, DEPTH, NI>(a, ph, wg, nwc, &cp);
        cact = true;
        if (ph >= a.C) {
          const float* hb = hbuf + ((ph - a.C) & 1) * hcap;
          int wp = wave, rg = 0;
          if (NI == 1)
            while (wp >= cp.PBw) { wp -= cp.PBw; ++rg; }
          cact = rg < cp.RG;
#pragma unroll
          for (int i = 0; i < NI; ++i) {
            const int pos = NI == 1 ? wp * 64 + lane : pidx[i];
            const bool have = cact && pos < cp.lim;  // the chunk's tail is zero-filled by the service waves
#pragma unroll
            for (int v = 0; v < VEC; v += 4) {
              const float4 t = *reinterpret_cast<const float4*>(hb + (have ? pos * VEC + v : 0));
              vr[i][v] = have ? t.x : 0.f;
              vr[i][v + 1] = have ? t.y : 0.f;
              vr[i][v + 2] = have ? t.z : 0.f;
              vr[i][v + 3] = have ? t.w : 0.f;
            }
          }
        }
      } else {
        cp.ngroups = 0;
      }
    }
  };
  consume_advance();  // to the first group that exists
#ifdef CI_FUSED_STAMPS
  int gcount = 0;
#endif

  while (ph < nph) {
    const bool isB = ph >= a.C;
    float p[DEPTH];
#pragma unroll
    for (int s = 0; s < DEPTH; ++s) {
      float sum = 0.f;
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        float f[VEC];
        unpack<D>(buf[s][i], f);
#pragma unroll
        for (int v = 0; v < VEC; ++v) sum = fmaf(f[v], vr[i][v], sum);
      }
      p[s] = sum;  // positions past the last row give values that are never stored
      // keep the ring order: the slot is refilled right after it has been consumed and before the
      // next slot is waited for (the dot must not sink below the refill, and the scheduler would
      // otherwise batch the loads)
      asm volatile("" : "+v"(p[s]));
      __builtin_amdgcn_sched_barrier(0);
      issue(s);
      __builtin_amdgcn_sched_barrier(0);
    }
    const float tot = wave_rows<DEPTH>(p, lane);
    const int q = g * DEPTH + (lane >> SH);
    if ((lane & ((1 << SH) - 1)) == 0 && q < cp.Q && cact) {
      if (isB) yred[((ph & 1) * nwc + wave) * a.rmax + q] = tot;
      else red[(ph & 1) * nwc * NDOT * kSuper + wave * NDOT * kSuper + q] = tot;
    }
#ifdef CI_FUSED_STAMPS
    if (tid == 0 && gcount < 96)
      a.stamps[(size_t)8 * 256 * 64 + (size_t)wg * 96 + gcount] = __builtin_amdgcn_s_memrealtime();
    ++gcount;
#endif
    issue_advance();
    consume_advance();
  }

  // the last phase's barrier has been passed: service wave 0 folds the last partial outputs and writes y
}

// Chooses the chunk size S (and with it the number of chunks C = ceil(K / S)) of a launch.
// Limits per chunk (cap): one 16-byte position per load of a compute thread, kSuper neurons per
// workgroup, two chunks of fp32 hidden values in 48 KB of LDS.  Among the sizes that respect them the
// one with the fewest ring slots on the critical path wins:
//   A phase of a chunk of Kc neurons: NDOT * ceil(Kc / n_wg) rows, rounded up to whole groups;
//   B phase: ceil(R / RG) items, RG = nwc / ceil(Pn / 64) rows side by side, rounded up likewise;
//   + chunk_cost slots per chunk for its two barriers;
//   + the slots by which the time between a chunk's publication and its use (the phases in between)
//     falls short of window_slots, the time the exchange needs.
// Candidates: multiples of U = n_wg * DEPTH / NDOT (every workgroup then owns whole groups of A rows),
// and equal splits of K in whole positions.  K too small to split: one empty chunk and the rest.
void plan_chunks(int K, int d, int n_wg, int ndot, int depth, int vec, int ni, int nwc, int64_t cap, int* C_out,
                 int* S_out, int* hcap_out) {
  const int R = (d + n_wg - 1) / n_wg;
  const double chunk_cost = params().fused_chunk_cost10 / 10.0;
  const int window_slots = params().fused_window_slots;
  const int min_chunks = params().fused_chunks > 2 ? (int)params().fused_chunks : 2;
  auto round_up = [](int64_t v, int64_t m) { return (v + m - 1) / m * m; };
  auto slots = [&](int64_t Kc, int64_t* sa, int64_t* sb) {
    *sa = round_up(ndot * ((Kc + n_wg - 1) / n_wg), depth);
    const int64_t Pn = (Kc + vec - 1) / vec;
    int64_t rg = 1;
    if (ni == 1) rg = std::max<int64_t>(1, nwc / std::max<int64_t>((Pn + 63) / 64, 1));
    *sb = round_up((R + rg - 1) / rg, depth);
  };
  int64_t U = (int64_t)n_wg * depth / ndot;
  while (U % vec) U *= 2;
  double best = -1.0;
  int64_t best_S = 0, best_C = 0;
  auto consider = [&](int64_t S) {
    if (S <= 0 || S >= K || S > cap || S % vec) return;
    const int64_t C = (K + S - 1) / S, last = K - (C - 1) * S;
    if (C < min_chunks || C > 4096 || last > cap) return;
    int64_t a0, b0, a1, b1;
    slots(S, &a0, &b0);
    slots(last, &a1, &b1);
    double cost = (double)((C - 1) * (a0 + b0) + a1 + b1) + chunk_cost * (double)C;
    // window of chunk j: the A phases after A(j) and the B phases before B(j)
    for (int64_t j = 0; j < C; ++j) {
      const int64_t after_a = (C - 2 - j >= 0 ? (C - 2 - j) * a0 : 0) + (j < C - 1 ? a1 : 0);
      const int64_t before_b = j * b0;
      if (after_a + before_b < window_slots) cost += (double)(window_slots - after_a - before_b);
    }
    if (best < 0 || cost < best - 1e-9) { best = cost; best_S = S; best_C = C; }
  };
  const int forced = params().fused_chunk_size;
  if (forced > 0) consider(forced);
  if (best < 0)
    for (int64_t S = U; S <= cap; S += U) consider(S);
  if (forced <= 0 || best < 0)
    for (int64_t C = min_chunks; C <= min_chunks + 6; ++C) consider(round_up((K + C - 1) / C, vec));
  if (best < 0) {
    // larger minimum number of chunks than the aligned sizes allow, or K below two positions
    for (int64_t C = min_chunks; C <= 4096 && best < 0; ++C) consider(round_up((K + C - 1) / C, vec));
  }
  if (best < 0) { best_S = 0; best_C = 2; }  // an empty chunk and one with everything (K <= vec)
  *C_out = (int)best_C;
  *S_out = (int)best_S;
  const int64_t last = K - (best_C - 1) * best_S;
  *hcap_out = (int)round_up(std::max<int64_t>(best_S, last), vec);
}

template <class D, int NI, bool SWIGLU, int DEPTH>
int launch_aux(const FusedArgs& a, int nt, size_t lds, hipStream_t s) {
  switch (params().fused_aux) {
    case -1: hipLaunchKernelGGL((ffn_decode_fused_kernel<D, NI, SWIGLU, DEPTH, -1>), dim3(a.n_wg), dim3(nt), lds, s, a); break;
    case -2: hipLaunchKernelGGL((ffn_decode_fused_kernel<D, NI, SWIGLU, DEPTH, -2>), dim3(a.n_wg), dim3(nt), lds, s, a); break;
    case 16: hipLaunchKernelGGL((ffn_decode_fused_kernel<D, NI, SWIGLU, DEPTH, 16>), dim3(a.n_wg), dim3(nt), lds, s, a); break;
    default: hipLaunchKernelGGL((ffn_decode_fused_kernel<D, NI, SWIGLU, DEPTH, 0>), dim3(a.n_wg), dim3(nt), lds, s, a); break;
  }
  CI_HIP_CHECK_LAUNCH();
  return CI_OK;
}

template <class D, int NI, bool SWIGLU>
int launch_depth(const FusedArgs& a, int nt, size_t lds, hipStream_t s) {
  int depth = params().fused_depth;
  if (NI >= 2) depth = 4;                 // 128 VGPRs at 1024 threads
  if (depth == 8) return launch_aux<D, NI, SWIGLU, 8>(a, nt, lds, s);
  return launch_aux<D, NI, SWIGLU, 4>(a, nt, lds, s);
}

// The launch shape of a call: loads per thread and row (ni), compute threads (ntc), chunks.
template <class D>
int plan_dtype(FusedArgs& a, int act, int* ni_out, int* ntc_out) {
  constexpr int VEC = D::VEC;
  const int vecs = a.d / VEC;
  // one 16-byte load per compute thread and row up to 896 threads (14 waves + the service waves),
  // more loads per thread beyond
  int ni = (vecs + 895) / 896;
  if (ni == 3) ni = 4;
  if (ni > 4) return CI_ERR_UNSUPPORTED;
  int ntc = ((vecs + ni - 1) / ni + 63) / 64 * 64;
  const int want = params().fused_threads / 64 * 64;
  if (want >= 64 && want <= 896 && (vecs + want - 1) / want <= 4 && (vecs + want - 1) / want != 3) {
    ntc = want;
    ni = (vecs + want - 1) / want;
  }
  const int nwc = ntc / 64;
  // Chunks: all but the last hold S neurons, the last takes the rest.  S is chosen by counting ring
  // slots (see plan_chunks).
  const bool swiglu = act == CI_ACT_SWIGLU;
  const int depth = ni >= 2 ? 4 : (params().fused_depth == 8 ? 8 : 4);
  a.rmax = (a.d + a.n_wg - 1) / a.n_wg;
  // two chunk buffers of fp32 hidden values must fit into what the other arrays leave of 64 KB of LDS
  const int64_t lds_left = 16384 - lds_red_floats(nwc, swiglu ? 2 : 1) - lds_yred_floats(nwc, a.rmax);
  if (lds_left < 2 * VEC) return CI_ERR_UNSUPPORTED;
  const int64_t cap = std::min<int64_t>(std::min<int64_t>(std::min<int64_t>((int64_t)ntc * ni * VEC, (int64_t)kSuper * a.n_wg),
                                                          6144), lds_left / 2 / VEC * VEC);
  plan_chunks(a.K, a.d, a.n_wg, swiglu ? 2 : 1, depth, VEC, ni, nwc, cap, &a.C, &a.S, &a.hcap);
  a.spin_limit = 1 << 16;
  // the service waves start collecting a chunk this long after it was published here, by which time the
  // other workgroups have published too
  a.guard_ticks = params().fused_guard_us10 * 10;
  *ni_out = ni;
  *ntc_out = ntc;
  return CI_OK;
}

template <class D>
int launch_dtype(FusedArgs a, int act, hipStream_t s) {
  int ni = 0, ntc = 0;
  const int rc = plan_dtype<D>(a, act, &ni, &ntc);
  if (rc != CI_OK) return rc;
  const int nwc = ntc / 64;
  const bool swiglu = act == CI_ACT_SWIGLU;
  const size_t lds = ((size_t)lds_red_floats(nwc, swiglu ? 2 : 1) + (size_t)lds_yred_floats(nwc, a.rmax) +
                      (size_t)2 * a.hcap) * sizeof(float);
  if (lds > 64 * 1024) return CI_ERR_UNSUPPORTED;
  const int nt = ntc + 64 * kServiceWaves;
  switch (ni) {
    case 1: return swiglu ? launch_depth<D, 1, true>(a, nt, lds, s) : launch_depth<D, 1, false>(a, nt, lds, s);
    case 2: return swiglu ? launch_depth<D, 2, true>(a, nt, lds, s) : launch_depth<D, 2, false>(a, nt, lds, s);
    default: return swiglu ? launch_depth<D, 4, true>(a, nt, lds, s) : launch_depth<D, 4, false>(a, nt, lds, s);
  }
}

int device_cus() {
  DeviceInfo di;
  return device_info(&di) == CI_OK ? di.cus : 256;
}

}  // namespace

// Workspace of the single-launch decode: a 256-byte header and one 8-byte word per neuron.
size_t fused_decode_ws_bytes(int64_t K) { return 256 + ((size_t)K + 16) * 8; }

// Development aid: the launch shape the single-launch decode would use.  out[0..4] = chunks, neurons
// per chunk, compute waves, loads per thread and row, workgroups.
int fused_decode_plan(int64_t K, int64_t d, int dtype, int act, int* out) {
  FusedArgs a = {};
  a.K = (int)K;
  a.d = (int)d;
  const int cus = device_cus();
  const int want_wgs = params().fused_wgs;
  a.n_wg = want_wgs > 0 && want_wgs < cus ? want_wgs : cus;
  int ni = 0, ntc = 0, rc;
  switch (dtype) {
    case CI_F32: rc = plan_dtype<F32>(a, act, &ni, &ntc); break;
    case CI_F16: rc = plan_dtype<F16>(a, act, &ni, &ntc); break;
    case CI_BF16: rc = plan_dtype<BF16>(a, act, &ni, &ntc); break;
    default: return CI_ERR_BAD_DTYPE;
  }
  if (rc != CI_OK) return rc;
  out[0] = a.C; out[1] = a.S; out[2] = ntc / 64; out[3] = ni; out[4] = a.n_wg;
  return CI_OK;
}

int launch_ffn_decode_fused(const void* x, int64_t B, const ci_ffn_weights* w, int dtype, int act, void* y,
                            void* ws, hipStream_t s) {
  const int cus = device_cus();
  FusedArgs a;
  a.w_up = w->w_up;
  a.w_gate = w->w_gate;
  a.b_up = act == CI_ACT_SWIGLU ? nullptr : w->b_up;
  a.w_down = w->w_down;
  a.b_down = w->b_down;
  a.hdr = reinterpret_cast<uint32_t*>(ws);
  a.hws = reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(ws) + 256);
#ifdef CI_FUSED_STAMPS
  a.stamps = reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(ws) + (1 << 20));  // needs K < 2^17 - 64
  a.ablate = params().fused_ablate;
#endif
  a.K = (int)w->K;
  a.d = (int)w->d;
  a.ldk = (int)w->ld_down;
  const int want_wgs = params().fused_wgs;
  a.n_wg = want_wgs > 0 ? want_wgs : cus;
  if (a.n_wg > cus) a.n_wg = cus;  // the grid must be co-resident: one workgroup per compute unit
  const size_t eb = (size_t)elem_bytes(dtype);
  // the sentences of a batch share the exchange buffer, so they run one after the other
  for (int64_t b = 0; b < B; ++b) {
    a.x = reinterpret_cast<const char*>(x) + (size_t)b * w->d * eb;
    a.y = reinterpret_cast<char*>(y) + (size_t)b * w->d * eb;
    int rc;
    switch (dtype) {
      case CI_F32: rc = launch_dtype<F32>(a, act, s); break;
      case CI_F16: rc = launch_dtype<F16>(a, act, s); break;
      case CI_BF16: rc = launch_dtype<BF16>(a, act, s); break;
      default: return CI_ERR_BAD_DTYPE;
    }
    if (rc != CI_OK) return rc;
  }
  return CI_OK;
}

}  // namespace ci
