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
 *   reduction workgroup), "decode_nt_store" (0/1): two-launch decode;
 *   "fused_depth" (4, 8, 16), "fused_threads" (0 or a multiple of 64 up to 1024),
 *   "fused_chunks" (2..64), "fused_wgs" (0 = one workgroup per compute unit, else
 *   fewer): single-launch decode;
 *   "select_wgs_per_cu" (1..8; 1 keeps the per-token kernel at one workgroup per
 *   compute unit also for prompts longer than the chip has compute units),
 *   "select_def2_single" (0/1: 1 runs Def. 2 in one workgroup even where the
 *   parallel kernel applies);
 *   "gemv_wgs_per_cu" (1..32), "gemm_ring" (0/1: pipelined 128 x 128 GEMM kernels),
 *   "gemm_direct" (0/1: those tiles loaded straight into LDS, else through a
 *   register ring), "gemm_big" (0 never, 1 when the grid is large enough, 2
 *   whenever the shape divides: the 256 x 256-tile GEMM kernel);
 *   "union_depth" (8, 16), "union_down_threads" (64..512), "union_up_wgs_per_cu"
 *   (1..8), "union_down_wgs_per_cu" (1..16): union-batched decode.
 * Unknown name or value out of range: CI_ERR_INVALID_ARG.  The values are
 * relaxed atomics: a call that runs while one is being changed sees the old or
 * the new value of that parameter.  A workspace size must be queried under the
 * setting the call will run with.
 */
#ifndef COREINFER_DEV_H_
#define COREINFER_DEV_H_

#ifdef __cplusplus
extern "C" {
#endif

int coreinfer_dev_set_param(const char* name, int value);

#ifdef __cplusplus
}
#endif
#endif /* COREINFER_DEV_H_ */
