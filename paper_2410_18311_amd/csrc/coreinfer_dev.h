/*
 * coreinfer_dev.h -- development hook of libcoreinfer.so, NOT part of the
 * installed interface (it is not in include/): launch-shape parameters for
 * tuning sweeps and for tests that run the alternative kernels.  No setting
 * changes what a call computes or makes it skip an output.
 *
 * Names and ranges:
 *   "decode_wgs_per_cu" (1..16), "decode_wgs" (0 = use the per-CU rule, else the
 *   number of neuron slices per sentence, up to 1024), "decode_threads" (0 =
 *   derive from d, else a multiple of 64 up to 1024), "decode_depth" (4, 8 or 16
 *   weight rows in flight per thread), "reduce_cq" (4, 8, 16 column quads per
 *   reduction workgroup), "reduce_threads" (64 .. 1024, a power of two: threads per reduction
 *   workgroup), "decode_nt_store" (0/1): two-launch decode;
 *   "fused_depth" (4, 8), "fused_threads" (0 or a multiple of 64 up to 896),
 *   "fused_chunks" (least number of neuron chunks, 2..64),
 *   "fused_chunk_size" (0 = cost model, else neurons per chunk, a multiple of the
 *   elements per 16 bytes; ignored where it breaks a limit), "fused_wgs" (0 = one
 *   workgroup per compute unit, else fewer), "fused_chunk_cost10" and
 *   "fused_window_slots" (weights of the chunk-size cost model, 0..1000),
 *   "fused_guard_us10" (tenths of a microsecond between a chunk's publication
 *   and its collection, 0..1000), "fused_aux" (cache policy of the weight
 *   loads: -1 non-temporal, -2 plain, 0 / 16 buffer loads without / with device
 *   scope), "fused_ablate" (timing builds only): single-launch decode;
 *   "select_wgs_per_cu" (1..8; 1 keeps the per-token kernel at one workgroup per
 *   compute unit also for prompts longer than the chip has compute units),
 *   "select_def2_single" (0/1: 1 runs Def. 2 in one workgroup even where the
 *   parallel kernel applies);
 *   "gemv_wgs_per_cu" (1..32), "gemm_ring" (0/1: pipelined 128 x 128 GEMM kernels),
 *   "gemm_direct" (0/1: those tiles loaded straight into LDS, else through a
 *   register ring), "gemm_big" (0 never, 1 when the grid is large enough, 2
 *   whenever the shape divides: the 256 x 256-tile GEMM kernel);
 *   "union_depth" (8, 16), "union_down_threads" (64..512), "union_up_wgs_per_cu"
 *   (1..8), "union_down_wgs_per_cu" (1..16), "union_super" (0 = default, 16..256:
 *   cap on the rows between two drains of the load ring): union-batched decode.
 * Unknown name or value out of range: CI_ERR_INVALID_ARG.  The values are
 * relaxed atomics: a call that runs while one is being changed sees the old or
 * the new value of that parameter.  A workspace size must be queried under the
 * setting the call will run with.
 */
#ifndef COREINFER_DEV_H_
#define COREINFER_DEV_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

int coreinfer_dev_set_param(const char* name, int value);

/* The launch shape the single-launch decode would use for K core neurons of a
 * layer with model width d under the current settings: out[0..4] = chunks,
 * neurons per chunk, compute waves per workgroup, 16-byte loads per thread and
 * row, workgroups.  Host arrays; CI_ERR_UNSUPPORTED where that path does not
 * apply. */
int coreinfer_dev_fused_plan(int64_t K, int64_t d, int dtype, int act, int* out);

/* Measurement aid: `workgroups` workgroups of `threads` threads (a multiple of
 * 64 up to 512) each stream 16-byte loads, `depth` (2, 4, 8, 16) in flight per
 * thread, `iters` * depth per thread in all, round and round over a window of
 * `window_bytes` (a multiple of 16, at least 16 * threads) of the device buffer
 * `buf` (16-byte aligned, `buf_bytes` long): the same window for all
 * (`per_workgroup` = 0) or consecutive windows, one each (then window_bytes *
 * workgroups <= buf_bytes).  `out`: device, 4 * workgroups bytes, receives a
 * checksum.  Asynchronous on `stream`; the caller times it. */
int coreinfer_dev_stream_probe(const void* buf, int64_t buf_bytes, int64_t window_bytes, int per_workgroup,
                               int workgroups, int threads, int depth, int iters, void* out, void* stream);

/* Measurement aid: the load stream of a GEMM operand tile without the
 * arithmetic.  Workgroups of 256 threads; a load instruction takes 128 bytes
 * of each of 32 rows `pitch_bytes` apart, `depth` (4, 8, 16) instructions = 32 *
 * depth rows in flight, then the same rows 128 bytes further along, `ksteps`
 * times (ksteps * 128 <= pitch_bytes keeps the rows apart), round and round for
 * `iters` steps.  `shared` != 0: every workgroup reads the same rows; else
 * workgroup w reads rows [32 * depth * w, 32 * depth * (w + 1)).  Everything it
 * touches must lie inside `buf` (checked). */
int coreinfer_dev_tile_probe(const void* buf, int64_t buf_bytes, int64_t pitch_bytes, int shared,
                             int workgroups, int depth, int ksteps, int iters, void* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* COREINFER_DEV_H_ */
