// C ABI of libcoreinfer: argument validation (host only, before any HIP
// call) and dispatch to the kernel launchers.
#include <math.h>
#include <string.h>

#include <mutex>

#include <algorithm>

#include "common.hpp"
#include "coreinfer_dev.h"

namespace ci {

Params& params() {
  static Params p;
  return p;
}

int device_info(DeviceInfo* out) {
  static std::mutex mu;
  static int cached_cus[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return CI_ERR_HIP;
  if (dev < 0 || dev >= 64) return CI_ERR_HIP;
  std::lock_guard<std::mutex> lock(mu);
  if (cached_cus[dev] == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
      return CI_ERR_HIP;
    cached_cus[dev] = cus;
  }
  out->cus = cached_cus[dev];
  return CI_OK;
}

namespace {

bool dtype_ok(int dt) { return dt == CI_F32 || dt == CI_F16 || dt == CI_BF16; }
bool act_ok(int a) { return a == CI_ACT_RELU || a == CI_ACT_SWIGLU; }
bool layout_ok(int l) { return l == CI_DOWN_OUT_MAJOR || l == CI_DOWN_NEURON_MAJOR; }
int vec_of(int dt) { return dt == CI_F32 ? 4 : 8; }
size_t round256(size_t n) { return (n + 255) / 256 * 256; }

// parts per million of a keep fraction; 0 if the fraction is not in (0, 1]
int64_t fraction_ppm(double frac) {
  if (!(frac > 0.0) || !(frac <= 1.0)) return 0;
  const int64_t q = (int64_t)floor(frac * 1e6 + 0.5);
  return q < 1 ? 0 : q;
}
int64_t keep(int64_t q, int64_t n) { return (q * n + 999999) / 1000000; }

constexpr int64_t kMaxSplits = 1024;

}  // namespace
}  // namespace ci

using namespace ci;

extern "C" {

const char* coreinfer_strerror(int status) {
  switch (status) {
    case CI_OK: return "ok";
    case CI_ERR_INVALID_ARG: return "invalid argument";
    case CI_ERR_BAD_DTYPE: return "unknown dtype or activation";
    case CI_ERR_BAD_LAYOUT: return "bad layout or alignment";
    case CI_ERR_WORKSPACE: return "workspace missing or too small";
    case CI_ERR_HIP: return "HIP runtime error";
    case CI_ERR_UNSUPPORTED: return "unsupported configuration";
  }
  return "unknown status";
}

int coreinfer_version(void) { return 2; }

int coreinfer_dev_fused_plan(int64_t K, int64_t d, int dtype, int act, int* out) {
  if (!out || K < 1 || d < 1 || d > (1 << 15)) return CI_ERR_INVALID_ARG;
  if (act != CI_ACT_RELU && act != CI_ACT_SWIGLU) return CI_ERR_INVALID_ARG;
  return fused_decode_plan(K, d, dtype, act, out);
}

// Development hook (coreinfer_dev.h), not part of the installed interface: launch-shape
// parameters for tuning sweeps.  Returns CI_ERR_INVALID_ARG for unknown names.
int coreinfer_dev_set_param(const char* name, int value) {
  if (!name) return CI_ERR_INVALID_ARG;
  Params& p = params();
  if (!strcmp(name, "decode_wgs_per_cu") && value >= 1 && value <= 16) p.decode_wgs_per_cu = value;
  else if (!strcmp(name, "decode_wgs") && value >= 0 && value <= 1024) p.decode_wgs = value;
  else if (!strcmp(name, "decode_threads") && value >= 0 && value <= 1024) p.decode_threads = value;
  else if (!strcmp(name, "decode_depth") && (value == 4 || value == 8 || value == 16)) p.decode_depth = value;
  else if (!strcmp(name, "reduce_cq") && (value == 4 || value == 8 || value == 16)) p.reduce_cq = value;
  else if (!strcmp(name, "reduce_threads") && (value == 64 || value == 128 || value == 256 || value == 512 || value == 1024)) p.reduce_threads = value;
  else if (!strcmp(name, "decode_nt_store") && (value == 0 || value == 1)) p.decode_nt_store = value;
  else if (!strcmp(name, "fused_depth") && (value == 4 || value == 8)) p.fused_depth = value;
  else if (!strcmp(name, "fused_threads") && value >= 0 && value <= 1024) p.fused_threads = value;
  else if (!strcmp(name, "fused_chunks") && value >= 2 && value <= 64) p.fused_chunks = value;
  else if (!strcmp(name, "fused_chunk_size") && value >= 0 && value <= 6144) p.fused_chunk_size = value;
  else if (!strcmp(name, "fused_wgs") && value >= 0 && value <= 1024) p.fused_wgs = value;
  else if (!strcmp(name, "fused_guard_us10") && value >= 0 && value <= 1000) p.fused_guard_us10 = value;
  else if (!strcmp(name, "fused_chunk_cost10") && value >= 0 && value <= 1000) p.fused_chunk_cost10 = value;
  else if (!strcmp(name, "fused_window_slots") && value >= 0 && value <= 1000) p.fused_window_slots = value;
  else if (!strcmp(name, "fused_ablate") && value >= 0 && value <= 2) p.fused_ablate = value;
  else if (!strcmp(name, "fused_aux") && (value == -1 || value == -2 || value == 0 || value == 16)) p.fused_aux = value;
  else if (!strcmp(name, "select_def2_single") && (value == 0 || value == 1)) p.select_def2_single = value;
  else if (!strcmp(name, "select_wgs_per_cu") && value >= 1 && value <= 8) p.select_wgs_per_cu = value;
  else if (!strcmp(name, "gemm_ring") && (value == 0 || value == 1)) p.gemm_ring = value;
  else if (!strcmp(name, "gemm_direct") && (value == 0 || value == 1)) p.gemm_direct = value;
  else if (!strcmp(name, "gemm_big") && value >= 0 && value <= 2) p.gemm_big = value;
  else if (!strcmp(name, "gemv_wgs_per_cu") && value >= 1 && value <= 32) p.gemv_wgs_per_cu = value;
  else if (!strcmp(name, "union_depth") && (value == 8 || value == 16)) p.union_depth = value;
  else if (!strcmp(name, "union_down_threads") && value >= 64 && value <= 512) p.union_down_threads = value;
  else if (!strcmp(name, "union_up_wgs_per_cu") && value >= 1 && value <= 8) p.union_up_wgs_per_cu = value;
  else if (!strcmp(name, "union_down_wgs_per_cu") && value >= 1 && value <= 16) p.union_down_wgs_per_cu = value;
  else if (!strcmp(name, "union_super") && (value == 0 || (value >= 16 && value <= 256))) p.union_super = value;
  else return CI_ERR_INVALID_ARG;
  return CI_OK;
}

int coreinfer_keep_count(double frac, int64_t n, int64_t* k) {
  if (!k || n < 0 || n > ((int64_t)1 << 40)) return CI_ERR_INVALID_ARG;
  const int64_t q = fraction_ppm(frac);
  if (q == 0) return CI_ERR_INVALID_ARG;
  *k = keep(q, n);
  return CI_OK;
}

int coreinfer_select_workspace_size(int64_t M, int64_t N, size_t* bytes) {
  if (!bytes || M < 1 || M > CI_MAX_TOKENS || N < 1 || N > CI_MAX_NEURONS) return CI_ERR_INVALID_ARG;
  SelectWs w;
  select_ws_layout(M, N, &w);
  *bytes = w.total;
  return CI_OK;
}

namespace {
// counters inside the workspace, for callers that pass none
int32_t* ws_counts(void* ws, int64_t M, int64_t N) {
  SelectWs w;
  select_ws_layout(M, N, &w);
  return reinterpret_cast<int32_t*>(reinterpret_cast<char*>(ws) + w.off_counts);
}
}  // namespace

int coreinfer_select(const float* act, int64_t M, int64_t N, int64_t ld, double alpha, double beta,
                     int32_t* core_idx, int32_t* counts, void* ws, size_t ws_bytes, void* stream) {
  size_t need = 0;
  if (coreinfer_select_workspace_size(M, N, &need) != CI_OK) return CI_ERR_INVALID_ARG;
  if (!act || !core_idx) return CI_ERR_INVALID_ARG;
  const int64_t qa = fraction_ppm(alpha), qb = fraction_ppm(beta);
  if (qa == 0 || qb == 0) return CI_ERR_INVALID_ARG;
  if (ld < N) return CI_ERR_BAD_LAYOUT;
  if ((reinterpret_cast<uintptr_t>(act) & 3u) || (reinterpret_cast<uintptr_t>(core_idx) & 3u) ||
      (reinterpret_cast<uintptr_t>(counts) & 3u))
    return CI_ERR_BAD_LAYOUT;
  if (!ws || ws_bytes < need) return CI_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) & 15u) return CI_ERR_BAD_LAYOUT;
  int32_t* cnt = counts ? counts : ws_counts(ws, M, N);
  return launch_select(act, CI_F32, 0, M, N, ld, qa, keep(qb, N), M, core_idx, cnt, ws, kSelTokens | kSelFinal,
                       (hipStream_t)stream);
}

int coreinfer_select_batch_workspace_size(int64_t B, int64_t M, int64_t N, size_t* bytes) {
  if (!bytes || B < 1 || B > 65535 || M < 1 || M > CI_MAX_TOKENS || N < 1 || N > CI_MAX_NEURONS ||
      B * M > (int64_t)CI_MAX_TOKENS * 64)
    return CI_ERR_INVALID_ARG;
  SelectWs w;
  select_ws_layout(M, N, &w, B);
  *bytes = w.total;
  return CI_OK;
}

int coreinfer_select_batch(const float* act, int64_t B, int64_t M, int64_t N, int64_t ld, double alpha, double beta,
                           int32_t* core_idx, int32_t* counts, void* ws, size_t ws_bytes, void* stream) {
  size_t need = 0;
  if (coreinfer_select_batch_workspace_size(B, M, N, &need) != CI_OK) return CI_ERR_INVALID_ARG;
  if (!act || !core_idx) return CI_ERR_INVALID_ARG;
  const int64_t qa = fraction_ppm(alpha), qb = fraction_ppm(beta);
  if (qa == 0 || qb == 0) return CI_ERR_INVALID_ARG;
  if (ld < N) return CI_ERR_BAD_LAYOUT;
  if ((reinterpret_cast<uintptr_t>(act) & 3u) || (reinterpret_cast<uintptr_t>(core_idx) & 3u) ||
      (reinterpret_cast<uintptr_t>(counts) & 3u))
    return CI_ERR_BAD_LAYOUT;
  if (!ws || ws_bytes < need) return CI_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) & 15u) return CI_ERR_BAD_LAYOUT;
  const int64_t K = keep(qb, N);
  SelectWs w;
  select_ws_layout(M, N, &w, B);
  int32_t* cnt = counts ? counts : reinterpret_cast<int32_t*>(reinterpret_cast<char*>(ws) + w.off_counts);
  if (B == 1 || select_batch_ok(M, N))
    return launch_select(act, CI_F32, 0, M, N, ld, qa, K, M, core_idx, cnt, ws, kSelTokens | kSelFinal,
                         (hipStream_t)stream, (int)B, N);
  // one sentence after the other; a sentence's thresholds and histogram fit the front of the batch's workspace
  for (int64_t b = 0; b < B; ++b) {
    const int rc = launch_select(act + (size_t)b * M * ld, CI_F32, 0, M, N, ld, qa, K, M, core_idx + b * K, cnt + b * N,
                                 ws, kSelTokens | kSelFinal, (hipStream_t)stream);
    if (rc != CI_OK) return rc;
  }
  return CI_OK;
}

int coreinfer_select_hidden(const void* hidden, int dtype, int act, int64_t M, int64_t N, int64_t ld, double alpha,
                            double beta, int32_t* core_idx, int32_t* counts, void* ws, size_t ws_bytes,
                            void* stream) {
  if (!dtype_ok(dtype) || !act_ok(act)) return CI_ERR_BAD_DTYPE;
  size_t need = 0;
  if (coreinfer_select_workspace_size(M, N, &need) != CI_OK) return CI_ERR_INVALID_ARG;
  if (!hidden || !core_idx) return CI_ERR_INVALID_ARG;
  const int64_t qa = fraction_ppm(alpha), qb = fraction_ppm(beta);
  if (qa == 0 || qb == 0) return CI_ERR_INVALID_ARG;
  if (ld < N) return CI_ERR_BAD_LAYOUT;
  const uintptr_t elem = dtype == CI_F32 ? 4 : 2;
  if ((reinterpret_cast<uintptr_t>(hidden) & (elem - 1)) || (reinterpret_cast<uintptr_t>(core_idx) & 3u) ||
      (reinterpret_cast<uintptr_t>(counts) & 3u))
    return CI_ERR_BAD_LAYOUT;
  if (!ws || ws_bytes < need) return CI_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) & 15u) return CI_ERR_BAD_LAYOUT;
  int32_t* cnt = counts ? counts : ws_counts(ws, M, N);
  return launch_select(hidden, dtype, act == CI_ACT_SWIGLU ? 1 : 0, M, N, ld, qa, keep(qb, N), M, core_idx, cnt, ws,
                       kSelTokens | kSelFinal, (hipStream_t)stream);
}

int coreinfer_count_tokens(const float* act, int64_t M, int64_t N, int64_t ld, double alpha,
                           int32_t* counts, int accumulate, void* ws, size_t ws_bytes, void* stream) {
  size_t need = 0;
  if (coreinfer_select_workspace_size(M, N, &need) != CI_OK) return CI_ERR_INVALID_ARG;
  if (!act || !counts) return CI_ERR_INVALID_ARG;
  const int64_t qa = fraction_ppm(alpha);
  if (qa == 0) return CI_ERR_INVALID_ARG;
  if (ld < N) return CI_ERR_BAD_LAYOUT;
  if ((reinterpret_cast<uintptr_t>(act) & 3u) || (reinterpret_cast<uintptr_t>(counts) & 3u)) return CI_ERR_BAD_LAYOUT;
  if (!ws || ws_bytes < need) return CI_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) & 15u) return CI_ERR_BAD_LAYOUT;
  return launch_select(act, CI_F32, 0, M, N, ld, qa, 1, M, nullptr, counts, ws,
                       kSelTokens | (accumulate ? kSelAccumulate : 0), (hipStream_t)stream);
}

int coreinfer_count_select(const int32_t* counts, int64_t N, int64_t max_count, double beta,
                           int32_t* core_idx, void* ws, size_t ws_bytes, void* stream) {
  if (!counts || !core_idx || N < 1 || N > CI_MAX_NEURONS || max_count < 0 || max_count > CI_MAX_TOKENS)
    return CI_ERR_INVALID_ARG;
  const int64_t qb = fraction_ppm(beta);
  if (qb == 0) return CI_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(counts) & 3u) || (reinterpret_cast<uintptr_t>(core_idx) & 3u)) return CI_ERR_BAD_LAYOUT;
  if (!ws || ws_bytes < 256) return CI_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) & 15u) return CI_ERR_BAD_LAYOUT;
  // Def. 2 alone runs in one workgroup and needs no scratch
  return launch_select(nullptr, CI_F32, 0, 0, N, N, 1, keep(qb, N), max_count, core_idx, const_cast<int32_t*>(counts),
                       nullptr, kSelFinal, (hipStream_t)stream);
}

int coreinfer_group_select(const int32_t* core_sets, int64_t G, int64_t K, int64_t N, double gamma,
                           int32_t* core_idx, int32_t* counts, void* ws, size_t ws_bytes, void* stream) {
  size_t need = 0;
  if (G < 1 || G > CI_MAX_TOKENS || coreinfer_select_workspace_size(G, N, &need) != CI_OK) return CI_ERR_INVALID_ARG;
  if (!core_sets || !core_idx || K < 0 || K > N) return CI_ERR_INVALID_ARG;
  const int64_t qg = fraction_ppm(gamma);
  if (qg == 0) return CI_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(core_sets) & 3u) || (reinterpret_cast<uintptr_t>(core_idx) & 3u) ||
      (reinterpret_cast<uintptr_t>(counts) & 3u))
    return CI_ERR_BAD_LAYOUT;
  if (!ws || ws_bytes < need) return CI_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) & 15u) return CI_ERR_BAD_LAYOUT;
  int32_t* cnt = counts ? counts : ws_counts(ws, G, N);
  hipStream_t s = (hipStream_t)stream;
  // clear the counters, count the groups' members, then Def. 2 with gamma on the counters
  int rc = launch_select(nullptr, CI_F32, 0, 0, N, N, 1, 1, G, nullptr, cnt, nullptr, kSelZero, s);
  if (rc != CI_OK) return rc;
  rc = launch_scatter_count(core_sets, G * K, N, cnt, s);
  if (rc != CI_OK) return rc;
  return launch_select(nullptr, CI_F32, 0, 0, N, N, 1, keep(qg, N), G, core_idx, cnt, nullptr, kSelFinal, s);
}

int coreinfer_core_similarity(const int32_t* set_a, int64_t Ka, const int32_t* set_b, int64_t Kb,
                              int32_t* out, void* stream) {
  if (!out || Ka < 0 || Kb < 0 || Ka > CI_MAX_NEURONS || Kb > CI_MAX_NEURONS) return CI_ERR_INVALID_ARG;
  if ((Ka > 0 && !set_a) || (Kb > 0 && !set_b)) return CI_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(set_a) & 3u) || (reinterpret_cast<uintptr_t>(set_b) & 3u) ||
      (reinterpret_cast<uintptr_t>(out) & 3u))
    return CI_ERR_BAD_LAYOUT;
  return launch_similarity(set_a, Ka, set_b, Kb, out, (hipStream_t)stream);
}

int coreinfer_assign_group(const int32_t* set, int64_t K, const int32_t* group_sets, int64_t G, int64_t Kg,
                           int32_t* best, int32_t* inter_union, void* stream) {
  if (!best || !inter_union || G < 1 || G > CI_MAX_TOKENS || K < 0 || Kg < 0 || K > CI_MAX_NEURONS ||
      Kg > CI_MAX_NEURONS)
    return CI_ERR_INVALID_ARG;
  if ((K > 0 && !set) || (Kg > 0 && !group_sets)) return CI_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(set) & 3u) || (reinterpret_cast<uintptr_t>(group_sets) & 3u) ||
      (reinterpret_cast<uintptr_t>(best) & 3u) || (reinterpret_cast<uintptr_t>(inter_union) & 3u))
    return CI_ERR_BAD_LAYOUT;
  return launch_assign_group(set, K, group_sets, G, Kg, best, inter_union, (hipStream_t)stream);
}

int coreinfer_assign_centroid_workspace_size(int64_t N, size_t* bytes) {
  if (!bytes || N < 1 || N > CI_MAX_NEURONS) return CI_ERR_INVALID_ARG;
  *bytes = round256((size_t)N * sizeof(float));
  return CI_OK;
}

int coreinfer_assign_centroid(const float* act, int64_t M, int64_t N, int64_t ld, const float* centroids,
                              int64_t G, int32_t* best, float* dist, void* ws, size_t ws_bytes, void* stream) {
  size_t need = 0;
  if (coreinfer_assign_centroid_workspace_size(N, &need) != CI_OK) return CI_ERR_INVALID_ARG;
  if (M < 1 || M > CI_MAX_TOKENS || G < 1 || G > CI_MAX_TOKENS) return CI_ERR_INVALID_ARG;
  if (!act || !centroids || !best || !dist) return CI_ERR_INVALID_ARG;
  if (ld < N) return CI_ERR_BAD_LAYOUT;
  if ((reinterpret_cast<uintptr_t>(act) & 3u) || (reinterpret_cast<uintptr_t>(centroids) & 3u) ||
      (reinterpret_cast<uintptr_t>(best) & 3u) || (reinterpret_cast<uintptr_t>(dist) & 3u))
    return CI_ERR_BAD_LAYOUT;
  if (!ws || ws_bytes < need) return CI_ERR_WORKSPACE;
  if (!aligned16(ws)) return CI_ERR_BAD_LAYOUT;
  return launch_assign_centroid(act, M, N, ld, centroids, G, best, dist, reinterpret_cast<float*>(ws),
                                (hipStream_t)stream);
}

int coreinfer_compact_down_ld(int64_t K, int dtype, int64_t* ld) {
  if (!dtype_ok(dtype)) return CI_ERR_BAD_DTYPE;
  if (!ld || K < 0 || K > CI_MAX_NEURONS) return CI_ERR_INVALID_ARG;
  *ld = compact_down_ld(K, dtype);
  return CI_OK;
}

int coreinfer_compact_preferred_layout(int64_t K, int64_t d, int dtype, int act, int* down_c_layout) {
  if (!dtype_ok(dtype) || !act_ok(act)) return CI_ERR_BAD_DTYPE;
  if (!down_c_layout || K < 0 || K > CI_MAX_NEURONS || d < 1 || d > CI_MAX_DMODEL) return CI_ERR_INVALID_ARG;
  *down_c_layout = CI_DOWN_NEURON_MAJOR;
  if (K < 1 || d % vec_of(dtype) != 0) return CI_OK;
  int plan[5];
  if (fused_decode_plan(K, d, dtype, act, plan) != CI_OK) return CI_OK;
  // Measured on MI355X (OPT-6.7B / Llama-2-7B / Llama-2-13B shapes): the two paths are within 2 % of
  // each other; the single launch wins from about 120 MB of weights per token on, where its fixed
  // cost (the exchange of the hidden values between the workgroups) is spread over more bytes.
  const double bytes = (double)(act == CI_ACT_SWIGLU ? 3 : 2) * (double)K * (double)d * (double)elem_bytes(dtype);
  if (bytes >= 120e6) *down_c_layout = CI_DOWN_OUT_MAJOR;
  return CI_OK;
}

int coreinfer_compact(const void* w_up, const void* w_gate, const void* b_up, const void* w_down,
                      int down_layout, int dtype, int act, int64_t d, int64_t N,
                      const int32_t* core_idx, int64_t K, void* w_up_c, void* w_gate_c,
                      void* b_up_c, void* w_down_c, int down_c_layout, int32_t* status, void* stream) {
  if (!dtype_ok(dtype) || !act_ok(act)) return CI_ERR_BAD_DTYPE;
  if (!layout_ok(down_layout) || !layout_ok(down_c_layout)) return CI_ERR_BAD_LAYOUT;
  if (d < 1 || d > CI_MAX_DMODEL || N < 1 || N > CI_MAX_NEURONS || K < 0 || K > N) return CI_ERR_INVALID_ARG;
  if (!w_up || !w_down || !w_up_c || !w_down_c || (K > 0 && !core_idx)) return CI_ERR_INVALID_ARG;
  if ((act == CI_ACT_SWIGLU) != (w_gate != nullptr) || (w_gate != nullptr) != (w_gate_c != nullptr))
    return CI_ERR_INVALID_ARG;
  if ((b_up != nullptr) != (b_up_c != nullptr)) return CI_ERR_INVALID_ARG;
  if (act == CI_ACT_SWIGLU && b_up) return CI_ERR_INVALID_ARG;  // gated FFNs carry no up bias here
  if (d % vec_of(dtype) != 0) return CI_ERR_BAD_LAYOUT;
  if (!aligned16(w_up) || !aligned16(w_gate) || !aligned16(w_down) || !aligned16(w_up_c) ||
      !aligned16(w_gate_c) || !aligned16(w_down_c))
    return CI_ERR_BAD_LAYOUT;
  return launch_compact(w_up, w_gate, b_up, w_down, down_layout, dtype, d, N, core_idx, K, w_up_c,
                        w_gate_c, b_up_c, w_down_c, down_c_layout, status, (hipStream_t)stream);
}

int coreinfer_compact_update_workspace_size(int64_t N, int64_t K, size_t* bytes) {
  if (!bytes || N < 1 || N > CI_MAX_NEURONS || K < 0 || K > N) return CI_ERR_INVALID_ARG;
  *bytes = round256(((size_t)N + 3 * (size_t)K + 64) * sizeof(uint32_t));
  return CI_OK;
}

int coreinfer_compact_update(const void* w_up, const void* w_gate, const void* b_up, const void* w_down,
                             int down_layout, int dtype, int act, int64_t d, int64_t N,
                             const int32_t* new_idx, int64_t K, int32_t* slot_idx, void* w_up_c,
                             void* w_gate_c, void* b_up_c, void* w_down_c, int down_c_layout,
                             int32_t* changed, void* ws, size_t ws_bytes, void* stream) {
  if (!dtype_ok(dtype) || !act_ok(act)) return CI_ERR_BAD_DTYPE;
  if (!layout_ok(down_layout) || !layout_ok(down_c_layout)) return CI_ERR_BAD_LAYOUT;
  if (d < 1 || d > CI_MAX_DMODEL) return CI_ERR_INVALID_ARG;
  size_t need = 0;
  if (coreinfer_compact_update_workspace_size(N, K, &need) != CI_OK) return CI_ERR_INVALID_ARG;
  if (!w_up || !w_down || !w_up_c || !w_down_c || (K > 0 && (!new_idx || !slot_idx))) return CI_ERR_INVALID_ARG;
  if ((act == CI_ACT_SWIGLU) != (w_gate != nullptr) || (w_gate != nullptr) != (w_gate_c != nullptr))
    return CI_ERR_INVALID_ARG;
  if ((b_up != nullptr) != (b_up_c != nullptr)) return CI_ERR_INVALID_ARG;
  if (act == CI_ACT_SWIGLU && b_up) return CI_ERR_INVALID_ARG;
  if (d % vec_of(dtype) != 0) return CI_ERR_BAD_LAYOUT;
  if (!aligned16(w_up) || !aligned16(w_gate) || !aligned16(w_down) || !aligned16(w_up_c) ||
      !aligned16(w_gate_c) || !aligned16(w_down_c) || (reinterpret_cast<uintptr_t>(new_idx) & 3u) ||
      (reinterpret_cast<uintptr_t>(slot_idx) & 3u) || (reinterpret_cast<uintptr_t>(changed) & 3u))
    return CI_ERR_BAD_LAYOUT;
  if (!ws || ws_bytes < need) return CI_ERR_WORKSPACE;
  if (!aligned16(ws)) return CI_ERR_BAD_LAYOUT;
  return launch_compact_update(w_up, w_gate, b_up, w_down, down_layout, dtype, d, N, new_idx, K, slot_idx,
                               w_up_c, w_gate_c, b_up_c, w_down_c, down_c_layout, changed,
                               reinterpret_cast<uint32_t*>(ws), (hipStream_t)stream);
}

int coreinfer_ffn_decode_workspace_size(int64_t B, int64_t K, int64_t d, size_t* bytes) {
  if (!bytes || B < 1 || B > 65535 || K < 0 || K > CI_MAX_NEURONS || d < 1 || d > CI_MAX_DMODEL)
    return CI_ERR_INVALID_ARG;
  // two-launch path: fp32 partial outputs of the neuron slices; single-launch path: a header and
  // one 8-byte word per neuron.  One size serves both, so the caller need not know the path.
  const int64_t splits = K < kMaxSplits ? K : kMaxSplits;
  const size_t two = round256((size_t)B * (size_t)splits * (size_t)d * sizeof(float)) + 256;
  const size_t one = round256(fused_decode_ws_bytes(K));
  *bytes = std::max(two, one);
  return CI_OK;
}

namespace {

// Argument checks common to the decode entry points (everything but the workspace).
int decode_check(const void* x, int64_t B, const ci_ffn_weights* w, int dtype, int act, void* y) {
  if (!w) return CI_ERR_INVALID_ARG;
  if (!dtype_ok(dtype) || !act_ok(act)) return CI_ERR_BAD_DTYPE;
  if (!layout_ok(w->down_layout)) return CI_ERR_BAD_LAYOUT;
  size_t need = 0;
  if (coreinfer_ffn_decode_workspace_size(B, w->K, w->d, &need) != CI_OK) return CI_ERR_INVALID_ARG;
  if (!x || !y) return CI_ERR_INVALID_ARG;
  if (w->K > 0 && (!w->w_up || !w->w_down)) return CI_ERR_INVALID_ARG;
  if (w->K > 0 && (act == CI_ACT_SWIGLU) != (w->w_gate != nullptr)) return CI_ERR_INVALID_ARG;
  if (act == CI_ACT_SWIGLU && w->b_up) return CI_ERR_INVALID_ARG;
  if (w->core_idx && (w->N < 1 || w->N > CI_MAX_NEURONS)) return CI_ERR_INVALID_ARG;
  if (w->d % vec_of(dtype) != 0) return CI_ERR_BAD_LAYOUT;
  const bool out_major = w->down_layout == CI_DOWN_OUT_MAJOR;
  if (out_major && w->core_idx) return CI_ERR_BAD_LAYOUT;  // gathered rows need the neuron-major matrix
  if (out_major && w->K > 0 && (w->ld_down < w->K || w->ld_down % vec_of(dtype) != 0 || w->ld_down > CI_MAX_NEURONS))
    return CI_ERR_BAD_LAYOUT;
  if (!aligned16(x) || !aligned16(y) || !aligned16(w->w_up) || !aligned16(w->w_gate) ||
      !aligned16(w->w_down) || (reinterpret_cast<uintptr_t>(w->core_idx) & 3u))
    return CI_ERR_BAD_LAYOUT;
  return CI_OK;
}

// Scratch of coreinfer_ffn_decode_static: device memory that belongs to the library, one copy per
// GPU the library runs on, held until the process ends.  Two parts that are never mixed: the tagged
// words of the single-launch path (zero when the module is loaded, which is all that path asks
// for: a call's tag is one more than the epoch the last call left) and the partial outputs of the
// two-launch path.
constexpr size_t kStaticWords = (size_t)1 << 20;     // header + 8 bytes per neuron: K <= 131024
constexpr size_t kStaticPartial = (size_t)16 << 20;  // B * slices * d fp32 partial outputs
static __device__ __align__(256) unsigned char scratch[kStaticWords + kStaticPartial];

// The array's address on the current device.  `scratch` itself is a host-side stand-in, not a device
// address: only the pointer obtained here may be handed to kernels and copies.
int static_scratch(unsigned char** out) {
  static std::mutex mu;
  static unsigned char* ptr[64] = {nullptr};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return CI_ERR_HIP;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    unsigned char* p = nullptr;
    if (hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)) != hipSuccess || !p) return CI_ERR_HIP;
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return CI_OK;
}

}  // namespace

int coreinfer_ffn_decode(const void* x, int64_t B, const ci_ffn_weights* w, int dtype, int act,
                         void* y, void* ws, size_t ws_bytes, void* stream) {
  const int rc = decode_check(x, B, w, dtype, act, y);
  if (rc != CI_OK) return rc;
  size_t need = 0;
  if (coreinfer_ffn_decode_workspace_size(B, w->K, w->d, &need) != CI_OK) return CI_ERR_INVALID_ARG;
  if (!ws || ws_bytes < need) return CI_ERR_WORKSPACE;
  if (!aligned16(ws)) return CI_ERR_BAD_LAYOUT;
  if (w->down_layout == CI_DOWN_OUT_MAJOR && w->K > 0)
    return launch_ffn_decode_fused(x, B, w, dtype, act, y, ws, (hipStream_t)stream);
  return launch_ffn_decode(x, B, w, dtype, act, y, reinterpret_cast<float*>(ws), (hipStream_t)stream);
}

int coreinfer_ffn_decode_static(const void* x, int64_t B, const ci_ffn_weights* w, int dtype, int act,
                                void* y, int32_t* status_out, void* stream) {
  const int rc = decode_check(x, B, w, dtype, act, y);
  if (rc != CI_OK) return rc;
  if (reinterpret_cast<uintptr_t>(status_out) & 3u) return CI_ERR_BAD_LAYOUT;
  const bool single = w->down_layout == CI_DOWN_OUT_MAJOR && w->K > 0;
  // what THIS call needs (not the device-independent bound of coreinfer_ffn_decode_workspace_size)
  const size_t need = single ? fused_decode_ws_bytes(w->K)
                             : (size_t)B * (size_t)decode_splits(B, w->K) * (size_t)w->d * sizeof(float);
  if (need > (single ? kStaticWords : kStaticPartial)) return CI_ERR_WORKSPACE;
  unsigned char* base = nullptr;
  const int rs = static_scratch(&base);
  if (rs != CI_OK) return rs;
  hipStream_t s = (hipStream_t)stream;
  if (!single) {
    const int rl = launch_ffn_decode(x, B, w, dtype, act, y, reinterpret_cast<float*>(base + kStaticWords), s);
    if (rl != CI_OK || !status_out) return rl;
    // the two-launch path has no bounded waits: nothing to report.  A copy, not a memset: callers may
    // be under graph capture, and base + 8 is a word of the header that no kernel writes.
    return hipMemcpyAsync(status_out, base + 8, sizeof(int32_t), hipMemcpyDeviceToDevice, s) == hipSuccess ? CI_OK
                                                                                                         : CI_ERR_HIP;
  }
  const int rl = launch_ffn_decode_fused(x, B, w, dtype, act, y, base, s);
  if (rl != CI_OK || !status_out) return rl;
  return hipMemcpyAsync(status_out, base + 4, sizeof(int32_t), hipMemcpyDeviceToDevice, s) == hipSuccess ? CI_OK
                                                                                                       : CI_ERR_HIP;
}

int coreinfer_ffn_decode_status(const void* ws, int32_t* status_out, void* stream) {
  if (!ws || !status_out) return CI_ERR_INVALID_ARG;
  if (!aligned16(ws) || (reinterpret_cast<uintptr_t>(status_out) & 3u)) return CI_ERR_BAD_LAYOUT;
  if (hipMemcpyAsync(status_out, reinterpret_cast<const char*>(ws) + 4, sizeof(int32_t), hipMemcpyDeviceToDevice,
                     (hipStream_t)stream) != hipSuccess)
    return CI_ERR_HIP;
  return CI_OK;
}

int coreinfer_union_workspace_size(int64_t N, size_t* bytes) {
  if (!bytes || N < 1 || N > CI_MAX_NEURONS) return CI_ERR_INVALID_ARG;
  // owner masks [N] and the number of owned neurons per block of 1024
  *bytes = round256(((size_t)(N + 63) / 64 * 64 + 1024) * sizeof(uint32_t));
  return CI_OK;
}

int coreinfer_union_build(const int32_t* core_idx, int64_t B, int64_t K, int64_t N, int64_t max_rows,
                          int32_t* union_idx, uint32_t* union_mask, int32_t* union_count, void* ws,
                          size_t ws_bytes, void* stream) {
  size_t need = 0;
  if (coreinfer_union_workspace_size(N, &need) != CI_OK) return CI_ERR_INVALID_ARG;
  if (B < 1 || B > CI_MAX_UNION_SENTENCES || K < 0 || K > N) return CI_ERR_INVALID_ARG;
  if ((K > 0 && !core_idx) || !union_idx || !union_mask || !union_count) return CI_ERR_INVALID_ARG;
  const int64_t worst = B * K < N ? B * K : N;  // the union cannot have more rows than this
  if (max_rows < 1 || max_rows < worst || max_rows > CI_MAX_NEURONS) return CI_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(core_idx) & 3u) || (reinterpret_cast<uintptr_t>(union_idx) & 3u) ||
      (reinterpret_cast<uintptr_t>(union_mask) & 3u) || (reinterpret_cast<uintptr_t>(union_count) & 3u))
    return CI_ERR_BAD_LAYOUT;
  if (!ws || ws_bytes < need) return CI_ERR_WORKSPACE;
  if (!aligned16(ws)) return CI_ERR_BAD_LAYOUT;
  return launch_union_build(core_idx, B, K, N, max_rows, union_idx, union_mask, union_count,
                            reinterpret_cast<uint32_t*>(ws), (hipStream_t)stream);
}

int coreinfer_ffn_decode_union_workspace_size(int64_t B, int64_t max_rows, int64_t d, int dtype, int act,
                                              size_t* bytes) {
  if (!dtype_ok(dtype) || !act_ok(act)) return CI_ERR_BAD_DTYPE;
  if (!bytes || B < 1 || B > CI_MAX_UNION_SENTENCES || max_rows < 1 || max_rows > CI_MAX_NEURONS ||
      d < 1 || d > CI_MAX_DMODEL)
    return CI_ERR_INVALID_ARG;
  if (d % vec_of(dtype) != 0) return CI_ERR_BAD_LAYOUT;
  const int64_t chunks = union_up_chunks(d / vec_of(dtype));
  const int64_t ndot = act == CI_ACT_SWIGLU ? 2 : 1;
  // partial dots [chunks][ndot][max_rows][8] and partial sums [B][<= 256 slices][d], fp32
  const size_t hp = ((size_t)chunks * ndot * (size_t)max_rows * 8 + 63) / 64 * 64;
  *bytes = round256((hp + (size_t)B * 256 * (size_t)d) * sizeof(float)) + 256;
  return CI_OK;
}

int coreinfer_ffn_decode_union(const void* x, int64_t B, const ci_ffn_weights* w,
                               const int32_t* union_idx, const uint32_t* union_mask,
                               const int32_t* union_count, int64_t max_rows, int dtype, int act,
                               void* y, void* ws, size_t ws_bytes, void* stream) {
  if (!w) return CI_ERR_INVALID_ARG;
  size_t need = 0;
  const int rc = coreinfer_ffn_decode_union_workspace_size(B, max_rows, w->d, dtype, act, &need);
  if (rc != CI_OK) return rc;
  if (!x || !y || !union_idx || !union_mask || !union_count) return CI_ERR_INVALID_ARG;
  if (!w->w_up || !w->w_down || w->N < 1 || w->N > CI_MAX_NEURONS) return CI_ERR_INVALID_ARG;
  if ((act == CI_ACT_SWIGLU) != (w->w_gate != nullptr)) return CI_ERR_INVALID_ARG;
  if (act == CI_ACT_SWIGLU && w->b_up) return CI_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(y) || !aligned16(w->w_up) || !aligned16(w->w_gate) ||
      !aligned16(w->w_down) || (reinterpret_cast<uintptr_t>(union_idx) & 3u) ||
      (reinterpret_cast<uintptr_t>(union_mask) & 3u) || (reinterpret_cast<uintptr_t>(union_count) & 3u))
    return CI_ERR_BAD_LAYOUT;
  if (!ws || ws_bytes < need) return CI_ERR_WORKSPACE;
  if (!aligned16(ws)) return CI_ERR_BAD_LAYOUT;
  return launch_ffn_decode_union(x, B, w, union_idx, union_mask, union_count, max_rows, dtype, act, y,
                                 reinterpret_cast<float*>(ws), (hipStream_t)stream);
}

int coreinfer_ffn_dense_workspace_size(int64_t M, int64_t d, int64_t N, int dtype, size_t* bytes) {
  if (!dtype_ok(dtype)) return CI_ERR_BAD_DTYPE;
  if (!bytes || M < 1 || M > CI_MAX_TOKENS || d < 1 || d > CI_MAX_DMODEL || N < 1 || N > CI_MAX_NEURONS)
    return CI_ERR_INVALID_ARG;
  // hidden matrix H [M, N]: fp32 on the row-dot path (M <= 4), element type
  // on the matrix-core path; plus the decode partials for a neuron-major down.
  size_t b = round256((size_t)M * (size_t)N * sizeof(float));
  if (M <= 4) {
    b += round256((size_t)M * (size_t)(N < kMaxSplits ? N : kMaxSplits) * (size_t)d * sizeof(float));
  } else {
    const int splits = gemm_down_splits_max(M, d, N, dtype);  // split-K partial products of Y
    if (splits > 1) b += round256((size_t)splits * (size_t)M * (size_t)d * sizeof(float));
  }
  *bytes = b + 256;
  return CI_OK;
}

int coreinfer_ffn_dense(const void* X, int64_t M, const void* w_up, const void* w_gate,
                        const void* b_up, const void* w_down, const void* b_down, int down_layout,
                        int dtype, int act, int64_t d, int64_t N, void* Y, float* A, void* ws,
                        size_t ws_bytes, void* stream) {
  if (!dtype_ok(dtype) || !act_ok(act)) return CI_ERR_BAD_DTYPE;
  if (!layout_ok(down_layout)) return CI_ERR_BAD_LAYOUT;
  size_t need = 0;
  if (coreinfer_ffn_dense_workspace_size(M, d, N, dtype, &need) != CI_OK) return CI_ERR_INVALID_ARG;
  if (!X || !w_up || (!Y && !A) || (Y && !w_down)) return CI_ERR_INVALID_ARG;
  if ((act == CI_ACT_SWIGLU) != (w_gate != nullptr)) return CI_ERR_INVALID_ARG;
  if (act == CI_ACT_SWIGLU && b_up) return CI_ERR_INVALID_ARG;
  if (d % vec_of(dtype) != 0 || N % vec_of(dtype) != 0) return CI_ERR_BAD_LAYOUT;
  if (!aligned16(X) || !aligned16(w_up) || !aligned16(w_gate) || !aligned16(w_down) ||
      !aligned16(Y) || !aligned16(A))
    return CI_ERR_BAD_LAYOUT;
  if (!ws || ws_bytes < need) return CI_ERR_WORKSPACE;
  if (!aligned16(ws)) return CI_ERR_BAD_LAYOUT;
  hipStream_t s = (hipStream_t)stream;

  if (M <= 4) {
    float* H = reinterpret_cast<float*>(ws);
    if (down_layout == CI_DOWN_NEURON_MAJOR && Y) {
      // all three matrices are neuron-major: this is the decode kernel with S = all neurons
      if (A) {
        int rc = launch_up_rows(X, M, w_up, w_gate, b_up, dtype, act, d, N, nullptr, A, s);
        if (rc != CI_OK) return rc;
      }
      ci_ffn_weights w;
      w.w_up = w_up; w.w_gate = w_gate; w.b_up = b_up; w.w_down = w_down; w.b_down = b_down;
      w.core_idx = nullptr; w.K = N; w.d = d; w.N = N;
      w.ld_down = 0; w.down_layout = CI_DOWN_NEURON_MAJOR;
      float* partial = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) +
                                                round256((size_t)M * (size_t)N * sizeof(float)));
      return launch_ffn_decode(X, M, &w, dtype, act, Y, partial, s);
    }
    int rc = launch_up_rows(X, M, w_up, w_gate, b_up, dtype, act, d, N, Y ? H : nullptr, A, s);
    if (rc != CI_OK || !Y) return rc;
    return launch_down_rows(H, M, w_down, b_down, dtype, d, N, Y, s);
  }
  void* H = Y ? ws : nullptr;
  int rc = launch_gemm_up(X, M, w_up, w_gate, b_up, dtype, act, d, N, H, A, s);
  if (rc != CI_OK || !Y) return rc;
  float* partial = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) +
                                            round256((size_t)M * (size_t)N * sizeof(float)));
  return launch_gemm_down(H, M, w_down, b_down, down_layout, dtype, d, N, Y, partial, s);
}

int coreinfer_ffn_dense_hidden_workspace_size(int64_t M, int64_t d, int64_t N, int dtype, size_t* bytes) {
  if (!dtype_ok(dtype)) return CI_ERR_BAD_DTYPE;
  if (!bytes || M < 1 || M > CI_MAX_TOKENS || d < 1 || d > CI_MAX_DMODEL || N < 1 || N > CI_MAX_NEURONS)
    return CI_ERR_INVALID_ARG;
  const int splits = gemm_down_splits_max(M, d, N, dtype);  // split-K partial products of Y
  *bytes = (splits > 1 ? round256((size_t)splits * (size_t)M * (size_t)d * sizeof(float)) : 0) + 256;
  return CI_OK;
}

int coreinfer_ffn_dense_hidden(const void* X, int64_t M, const void* w_up, const void* w_gate, const void* b_up,
                               const void* w_down, const void* b_down, int down_layout, int dtype, int act,
                               int64_t d, int64_t N, void* Y, void* H, void* ws, size_t ws_bytes, void* stream) {
  if (!dtype_ok(dtype) || !act_ok(act)) return CI_ERR_BAD_DTYPE;
  if (!layout_ok(down_layout)) return CI_ERR_BAD_LAYOUT;
  size_t need = 0;
  if (coreinfer_ffn_dense_hidden_workspace_size(M, d, N, dtype, &need) != CI_OK) return CI_ERR_INVALID_ARG;
  if (!X || !w_up || !H || (Y && !w_down)) return CI_ERR_INVALID_ARG;
  if ((act == CI_ACT_SWIGLU) != (w_gate != nullptr)) return CI_ERR_INVALID_ARG;
  if (act == CI_ACT_SWIGLU && b_up) return CI_ERR_INVALID_ARG;
  if (d % vec_of(dtype) != 0 || N % vec_of(dtype) != 0) return CI_ERR_BAD_LAYOUT;
  if (!aligned16(X) || !aligned16(w_up) || !aligned16(w_gate) || !aligned16(w_down) || !aligned16(Y) ||
      !aligned16(H))
    return CI_ERR_BAD_LAYOUT;
  if (!ws || ws_bytes < need) return CI_ERR_WORKSPACE;
  if (!aligned16(ws)) return CI_ERR_BAD_LAYOUT;
  hipStream_t s = (hipStream_t)stream;
  int rc = launch_gemm_up(X, M, w_up, w_gate, b_up, dtype, act, d, N, H, nullptr, s);
  if (rc != CI_OK || !Y) return rc;
  return launch_gemm_down(H, M, w_down, b_down, down_layout, dtype, d, N, Y, reinterpret_cast<float*>(ws), s);
}

}  // extern "C"
