/*
 * coreinfer.h -- C ABI of libcoreinfer.so: the data-parallel hot path of
 * CoreInfer (arXiv 2410.18311) for one AMD MI355X (gfx950).
 *
 * The path has two halves.
 *   Prefill (once per sentence and FFN layer): the dense FFN produces the
 *   activation matrix A (one row per prompt token); coreinfer_select turns it
 *   into the sentence-wise core neuron set S (Sec. 3.1, Def. 1-2, Eq. 1-3);
 *   coreinfer_compact gathers the weights of S into contiguous buffers
 *   (Sec. 5.3, "deploying the necessary neurons during pre-filling").
 *   Decode (every generated token): coreinfer_ffn_decode runs the FFN over
 *   the frozen set S only (Sec. 4.1 stability-guided prediction; Sec. 4.2).
 *
 * Conventions, valid for every entry point unless stated otherwise:
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  The
 *     library allocates and frees nothing; scratch memory is the caller's
 *     workspace, sized by the matching *_workspace_size query (a pure host
 *     function that needs no GPU).  Inputs are never modified.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is enqueued on it; no call synchronises the device, so outputs
 *     are valid only after the caller synchronises the stream.
 *   - Arguments are validated on the host before any HIP call.  The return
 *     value is CI_OK (0) or a negative ci_status; coreinfer_strerror names it.
 *     No exception crosses the boundary.
 *   - Matrices are row-major and dense (leading dimension = row length) unless
 *     an `ld` argument says otherwise.  Weights use the nn.Linear convention of
 *     the models the paper runs: w_up, w_gate are [N, d]; w_down is [d, N]
 *     (CI_DOWN_OUT_MAJOR) or its transpose [N, d] (CI_DOWN_NEURON_MAJOR).
 *   - d = d_model, N = d_ff (neurons per layer), M = prompt tokens,
 *     K = |S|, B = sentences decoded together.
 *   - Element types: CI_F32, CI_F16 (IEEE half), CI_BF16.  Every sum is
 *     accumulated in fp32.  The decode entry points and the scores A handed
 *     to the selection keep the hidden activations in fp32 (Sec. 5, "Models":
 *     fp16 parameters, fp32 intermediate activations); the two places that
 *     round them to the element type say so (the Y of coreinfer_ffn_dense for
 *     M > 4, and the H of coreinfer_ffn_dense_hidden).
 *   - Pointers must be 16-byte aligned, and d must be a multiple of
 *     16 / sizeof(element) (8 for 16-bit types, 4 for fp32); otherwise
 *     CI_ERR_BAD_LAYOUT.
 *   - Calls are deterministic: the same bits in give the same bits out.
 */
#ifndef COREINFER_H_
#define COREINFER_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CI_OK = 0,
  CI_ERR_INVALID_ARG = -1, /* null pointer, size out of range, fraction outside (0,1] */
  CI_ERR_BAD_DTYPE = -2,   /* dtype / activation enum not recognised               */
  CI_ERR_BAD_LAYOUT = -3,  /* alignment, leading dimension or layout enum          */
  CI_ERR_WORKSPACE = -4,   /* workspace null or smaller than the query says        */
  CI_ERR_HIP = -5,         /* a HIP runtime call or kernel launch failed           */
  CI_ERR_UNSUPPORTED = -6  /* valid request that this build does not implement     */
} ci_status;

typedef enum { CI_F32 = 0, CI_F16 = 1, CI_BF16 = 2 } ci_dtype;
typedef enum { CI_ACT_RELU = 0, CI_ACT_SWIGLU = 1 } ci_act;
typedef enum { CI_DOWN_OUT_MAJOR = 0, CI_DOWN_NEURON_MAJOR = 1 } ci_down_layout;

/* Upper limits accepted by the entry points. */
#define CI_MAX_TOKENS 65535     /* M: counts fit 16 bits                */
#define CI_MAX_NEURONS 1048576  /* N                                   */
#define CI_MAX_DMODEL 32768     /* d                                   */
#define CI_MAX_UNION_SENTENCES 8 /* sentences of a union-batched decode */

/* Human-readable name of a status code (static storage, never NULL). */
const char* coreinfer_strerror(int status);

/* Library ABI version (increases when a signature changes). */
int coreinfer_version(void);

/*
 * Size of "the top `frac` share of n items", the rule every selection below
 * uses: k = ceil(q * n / 10^6) with q = floor(frac * 10^6 + 0.5), in integer
 * arithmetic (Def. 1 and Def. 2 leave the rounding open; this is the smallest
 * set that covers at least the fraction).  Host-only, needs no GPU; lets the
 * caller size core_idx without a device round trip.
 * frac outside (0, 1] (or below 1e-6), n < 0 or k == NULL: CI_ERR_INVALID_ARG.
 */
int coreinfer_keep_count(double frac, int64_t n, int64_t* k);

/*
 * Sentence-wise core neuron selection for one FFN layer of one sentence
 * (Sec. 3.1; Fig. 1 "top-k selection ... top-k commonly activated").
 *
 *   act      [M, N] fp32, row stride ld >= N elements: A, the activation of
 *            every neuron for every prompt token (ReLU output, or
 *            |SiLU(gate)*up| for gated FFNs).
 *   step 1   (Def. 1 / Eq. 1) per token m: P = #{a > 0};
 *            C_m = the keep_count(alpha, P) largest positive entries,
 *            equal values resolved towards the lower neuron index.
 *            NaN and values <= 0 are never selected.
 *   step 2   (Eq. 3) counts[n] = #{m : n in C_m}.
 *   step 3   (Def. 2 / Eq. 2) S = the K = keep_count(beta, N) neurons that
 *            come first in the order (count descending, index ascending).
 *   core_idx [K] int32 out: S in ascending index order.
 *   counts   [N] int32 out, may be NULL (then it lives in the workspace).
 *   ws       at least coreinfer_select_workspace_size(M, N) bytes.
 * Limits: 1 <= M <= CI_MAX_TOKENS, 1 <= N <= CI_MAX_NEURONS.
 */
int coreinfer_select_workspace_size(int64_t M, int64_t N, size_t* bytes);
int coreinfer_select(const float* act, int64_t M, int64_t N, int64_t ld,
                     double alpha, double beta,
                     int32_t* core_idx, int32_t* counts,
                     void* ws, size_t ws_bytes, void* stream);

/*
 * The same selection for B sentences at once (independent sentences batched,
 * each with its own core set): sentence b is rows [b M, (b + 1) M) of
 * act [B M, N]; core_idx [B, K] and counts [B, N] (may be NULL) hold its
 * results, exactly those of coreinfer_select on its rows.  One set of launches
 * serves all sentences where Def. 2 runs in parallel (M < 2048 and
 * N <= 65536); otherwise the sentences are taken one after the other.
 * ws: at least coreinfer_select_batch_workspace_size(B, M, N) bytes.
 * Limits: 1 <= B <= 65535, B * M <= CI_MAX_TOKENS * 64.
 */
int coreinfer_select_batch_workspace_size(int64_t B, int64_t M, int64_t N, size_t* bytes);
int coreinfer_select_batch(const float* act, int64_t B, int64_t M, int64_t N, int64_t ld,
                           double alpha, double beta, int32_t* core_idx, int32_t* counts,
                           void* ws, size_t ws_bytes, void* stream);

/*
 * The same selection on the hidden matrix as the FFN holds it, in the layer's
 * element type, so that no fp32 copy of the activations has to be written for
 * it (Sec. 1 calls the prefill-stage selection free of extra cost; Def. 1
 * ranks "the activation", and a 16-bit model holds 16-bit activations).
 *   hidden [M, N] of `dtype` (row stride ld >= N elements), as written by
 *   coreinfer_ffn_dense_hidden: max(z, 0) for CI_ACT_RELU, SiLU(gate) * up for
 *   CI_ACT_SWIGLU.  The value ranked is the element itself for CI_ACT_RELU and
 *   its magnitude for CI_ACT_SWIGLU; 16-bit values are compared exactly (their
 *   fp32 images).  Everything else -- keep counts, ties towards the lower
 *   index, outputs, workspace, limits -- as for coreinfer_select; with
 *   CI_F32 / CI_ACT_RELU the two calls are the same.  Equal activations are far
 *   more frequent among 16-bit values; they are resolved towards the lower
 *   neuron index like any other tie.
 */
int coreinfer_select_hidden(const void* hidden, int dtype, int act, int64_t M, int64_t N, int64_t ld,
                            double alpha, double beta, int32_t* core_idx, int32_t* counts, void* ws,
                            size_t ws_bytes, void* stream);

/*
 * The two halves of coreinfer_select as separate calls, for callers that keep
 * running counts while a sentence grows (Fig. 1 names a "stability estimation"
 * that decides how the set is updated but does not specify it; Eq. 3 is a sum
 * over tokens, so counts of new tokens simply add to the old ones):
 *   coreinfer_count_tokens  steps 1-2 of coreinfer_select over the M rows of
 *                           act; counts [N] is overwritten unless
 *                           accumulate != 0, in which case it is added to;
 *                           ws: coreinfer_select_workspace_size(M, N) bytes.
 *   coreinfer_count_select  step 3 on given counts (every value must lie in
 *                           [0, max_count], max_count <= CI_MAX_TOKENS);
 *                           core_idx [keep_count(beta, N)] ascending;
 *                           ws: at least 256 bytes.
 */
int coreinfer_count_tokens(const float* act, int64_t M, int64_t N, int64_t ld, double alpha,
                           int32_t* counts, int accumulate, void* ws, size_t ws_bytes, void* stream);
int coreinfer_count_select(const int32_t* counts, int64_t N, int64_t max_count, double beta,
                           int32_t* core_idx, void* ws, size_t ws_bytes, void* stream);

/*
 * Similarity-guided prediction, group step (Sec. 4.1): the core neurons of a
 * semantic group are the top gamma share of neurons that appear most often in
 * the core sets of the group's sentences.
 *   core_sets [G, K] int32: the G sentences' core sets (any order; entries
 *             outside [0, N) are ignored);  counts[n] = #{g : n in set g}
 *             (out, may be NULL);  core_idx [keep_count(gamma, N)] ascending,
 *             ties towards the lower index as in coreinfer_select.
 *   ws: at least coreinfer_select_workspace_size(G, N) bytes.  G <= CI_MAX_TOKENS.
 * How sentences are grouped (labels, K-Means; App. A.2.3) is outside this library.
 */
int coreinfer_group_select(const int32_t* core_sets, int64_t G, int64_t K, int64_t N, double gamma,
                           int32_t* core_idx, int32_t* counts, void* ws, size_t ws_bytes, void* stream);

/*
 * Core-neuron similarity of two sets (Sec. 3.2, Insight-2: identical neurons
 * over all neurons involved).  set_a [Ka], set_b [Kb]: ascending, duplicate
 * free.  out [2] int32 (device): out[0] = |a and b|, out[1] = |a or b|; the
 * similarity is out[0] / out[1] (1 if both are empty).
 */
int coreinfer_core_similarity(const int32_t* set_a, int64_t Ka, const int32_t* set_b, int64_t Kb,
                              int32_t* out, void* stream);

/*
 * Similarity-guided prediction, choosing the group (Sec. 4.1 says only "once
 * the input sentence's group is determined"; the rule here is a reading): the
 * group whose core set is most similar to the prompt's own core set under the
 * metric above.  set [K] and every row of group_sets [G, Kg]: ascending,
 * duplicate free.  Out (device): inter_union [G, 2] int32 as for
 * coreinfer_core_similarity, best [1] int32 = the group with the largest
 * identical / involved ratio, compared exactly; equal ratios go to the lower
 * index; two empty sets count as ratio 1.  G <= CI_MAX_TOKENS.
 */
int coreinfer_assign_group(const int32_t* set, int64_t K, const int32_t* group_sets, int64_t G, int64_t Kg,
                           int32_t* best, int32_t* inter_union, void* stream);

/*
 * Similarity-guided prediction, choosing the group when the groups are K-Means
 * clusters of one layer's activation (App. A.2.3): the K-Means assignment
 * step.  The prompt's feature vector is the mean over its M tokens of the
 * activation rows act [M, N] (fp32, row stride ld >= N; the same matrix that
 * coreinfer_select ranks) -- the paper does not say how a sentence's tokens
 * are summarised, this is a reading.  centroids [G, N] fp32, row-major.
 * Out (device): dist [G] fp32 = squared Euclidean distance of the feature to
 * every centroid; best [1] int32 = the nearest centroid, equal distances going
 * to the lower index (a NaN distance is never nearest; group 0 if all are).
 * All sums in fp32, in an order that does not depend on scheduling.
 *   ws: at least coreinfer_assign_centroid_workspace_size(N) bytes (holds the
 *       feature vector, N floats from its start, readable after the call).
 * Limits: 1 <= M <= CI_MAX_TOKENS, 1 <= N <= CI_MAX_NEURONS, 1 <= G <= CI_MAX_TOKENS.
 */
int coreinfer_assign_centroid_workspace_size(int64_t N, size_t* bytes);
int coreinfer_assign_centroid(const float* act, int64_t M, int64_t N, int64_t ld, const float* centroids,
                              int64_t G, int32_t* best, float* dist, void* ws, size_t ws_bytes, void* stream);

/*
 * Deploy the core neurons (Sec. 5.3): gather rows S of w_up (and w_gate),
 * entries S of b_up and columns S of w_down into contiguous buffers:
 *   w_up_c   [K, d] = w_up[S, :]        w_gate_c [K, d] = w_gate[S, :]
 *   b_up_c   [K]    = b_up[S]
 *   w_down_c, by down_c_layout:
 *     CI_DOWN_NEURON_MAJOR  [K, d]  = (w_down[:, S])^T
 *     CI_DOWN_OUT_MAJOR     [d, ld] = w_down[:, S], ld = K rounded up to whole
 *                           16-byte vectors (coreinfer_compact_down_ld); the
 *                           columns K .. ld-1 are written as zeros.  This is
 *                           the layout the single-launch decode reads.
 * w_gate / w_gate_c must be non-NULL exactly when act == CI_ACT_SWIGLU;
 * b_up / b_up_c are both NULL or both non-NULL, and NULL for CI_ACT_SWIGLU
 * (the gated FFNs of the paper's models have no biases; CI_ERR_INVALID_ARG).
 * core_idx [K] must be strictly ascending with values in [0, N); an entry that
 * violates this yields an all-zero row / column and sets *status (device
 * int32, may be NULL; the caller zeroes it beforehand) to 1 -- it never causes
 * an out-of-bounds access.  Output buffers are caller-allocated and must not
 * overlap the inputs.  With CI_DOWN_OUT_MAJOR b_up_c holds ld elements (the
 * entries K .. ld-1 are left as they are).
 *
 * coreinfer_compact_preferred_layout names, in *down_c_layout (host), the
 * layout of w_down_c that decodes faster for K core neurons of a layer of width
 * d: both are correct for every shape; small layers decode faster through the
 * neuron-major path (two launches), large ones through the output-major path
 * (one launch), and where the single-launch path does not apply
 * (coreinfer_ffn_decode would return CI_ERR_UNSUPPORTED) the answer is
 * CI_DOWN_NEURON_MAJOR.
 */
int coreinfer_compact_down_ld(int64_t K, int dtype, int64_t* ld);
int coreinfer_compact_preferred_layout(int64_t K, int64_t d, int dtype, int act, int* down_c_layout);
int coreinfer_compact(const void* w_up, const void* w_gate, const void* b_up,
                      const void* w_down, int down_layout, int dtype, int act,
                      int64_t d, int64_t N, const int32_t* core_idx, int64_t K,
                      void* w_up_c, void* w_gate_c, void* b_up_c, void* w_down_c,
                      int down_c_layout, int32_t* status, void* stream);

/*
 * Re-deploying after the core set changed (Fig. 1 names a stability estimation
 * that decides "how to update" the set but gives no rule; this call rewrites
 * as little as possible).  The compact buffers written by coreinfer_compact
 * (or by an earlier update) are changed in place so that they hold exactly the
 * neurons of new_idx: a neuron that stays keeps its row; the rows of neurons
 * that left, in ascending row order, take the neurons that entered, in
 * ascending neuron order.  Only those rows are copied.
 *   new_idx [K] int32 ascending, duplicate free, the new core set (same K as
 *   the buffers).  slot_idx [K] int32, in/out: the neuron held by each row;
 *   after coreinfer_compact it equals that call's core_idx.  The decode entry
 *   point does not care about the order of the rows.  changed [1] int32
 *   (device, may be NULL): number of rows rewritten.  Weights, layouts
 *   (down_c_layout names the layout of w_down_c: rows or columns are rewritten
 *   accordingly) and dtypes as for coreinfer_compact.
 *   ws: coreinfer_compact_update_workspace_size.
 */
int coreinfer_compact_update_workspace_size(int64_t N, int64_t K, size_t* bytes);
int coreinfer_compact_update(const void* w_up, const void* w_gate, const void* b_up, const void* w_down,
                             int down_layout, int dtype, int act, int64_t d, int64_t N,
                             const int32_t* new_idx, int64_t K, int32_t* slot_idx, void* w_up_c,
                             void* w_gate_c, void* b_up_c, void* w_down_c, int down_c_layout,
                             int32_t* changed, void* ws, size_t ws_bytes, void* stream);

/*
 * Weights of one FFN layer as the decode kernel reads them.
 *   core_idx == NULL: compacted -- the buffers written by coreinfer_compact;
 *                     K rows each, shared by all B inputs.  down_layout says
 *                     how w_down_c was written: CI_DOWN_NEURON_MAJOR [K, d], or
 *                     CI_DOWN_OUT_MAJOR [d, ld_down].
 *   core_idx != NULL: gathered -- the resident dense weights, all neuron-major
 *                     (w_up, w_gate, w_down are [N, d], b_up is [N];
 *                     down_layout must be CI_DOWN_NEURON_MAJOR);
 *                     core_idx is [B, K], row b naming sentence b's core set.
 *                     Entries outside [0, N) contribute nothing.
 */
typedef struct {
  const void* w_up;        /* [K, d] or [N, d]                          */
  const void* w_gate;      /* same shape; NULL unless CI_ACT_SWIGLU     */
  const void* b_up;        /* [K] or [N]; may be NULL; NULL for SwiGLU  */
  const void* w_down;      /* [K, d] / [N, d], or [d, ld_down]          */
  const void* b_down;      /* [d]; may be NULL                          */
  const int32_t* core_idx; /* NULL (compacted) or [B, K] (gathered)     */
  int64_t K;               /* core neurons per sentence                 */
  int64_t d;               /* d_model                                   */
  int64_t N;               /* rows of the resident weights (gathered)   */
  int64_t ld_down;         /* row length of an output-major w_down (>= K, whole 16-byte vectors;
                              the columns K .. ld_down-1 must hold finite values, e.g. the zeros
                              coreinfer_compact writes: they are multiplied by zero) */
  int32_t down_layout;     /* ci_down_layout of w_down                  */
} ci_ffn_weights;

/*
 * Decode-stage FFN over the frozen core set (Sec. 4.2):
 *   ReLU:    y = w_down_c^T max(w_up_c x + b_up_c, 0) + b_down
 *   SwiGLU:  y = w_down_c^T (SiLU(w_gate_c x) * (w_up_c x)) + b_down
 * x [B, d] in, y [B, d] out, element type `dtype`; K = 0 gives y = b_down.
 * b_up with CI_ACT_SWIGLU: CI_ERR_INVALID_ARG.
 * ws: at least coreinfer_ffn_decode_workspace_size(B, K, d) bytes.
 *
 * Two kernel paths, chosen by the layout of the compact down matrix:
 *   CI_DOWN_NEURON_MAJOR (and every gathered call): neuron slices produce fp32
 *     partial outputs in ws, a second launch sums them in a fixed order.  ws
 *     needs no initialisation.
 *   CI_DOWN_OUT_MAJOR: one launch, no partial outputs; the hidden values cross
 *     workgroups through ws as self-validating words.  For this path ws must
 *     have been ZEROED ONCE (hipMemsetAsync) before its first use and must not
 *     be written by anything else afterwards; every call leaves it ready for
 *     the next one, also when replayed from a HIP graph.  A workspace that has
 *     served a neuron-major or gathered call (which fills it with partial sums)
 *     must be zeroed again before an output-major call.  The launch needs one workgroup per compute unit resident at
 *     the same time; if other work keeps compute units busy for long, a
 *     workgroup gives up waiting after a bounded number of polls, the call's
 *     output is then unspecified and the int32 at ws + 4 is set to 1 (it is 0
 *     otherwise; coreinfer_ffn_decode_status copies it out).
 * Calls that share a workspace must not overlap in time.
 */
int coreinfer_ffn_decode_workspace_size(int64_t B, int64_t K, int64_t d, size_t* bytes);
int coreinfer_ffn_decode(const void* x, int64_t B, const ci_ffn_weights* w,
                         int dtype, int act, void* y,
                         void* ws, size_t ws_bytes, void* stream);
/* Enqueues a copy of the workspace's error word (see above) to *status_out, a
 * device int32; valid after the stream has been synchronised. */
int coreinfer_ffn_decode_status(const void* ws, int32_t* status_out, void* stream);

/*
 * coreinfer_ffn_decode for callers that cannot allocate device memory or have
 * none to pass: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, same kernels and same results as
 * coreinfer_ffn_decode, but the workspace is a static array inside the library
 * (17 MiB of device memory on every GPU the library runs on, held until the
 * process ends); the call allocates nothing.  Limits: output-major compact
 * buffers: K <= 131024; neuron-major and gathered calls: B * slices * d * 4
 * bytes <= 16 MiB, slices = min(K, compute units / B) (e.g. B = 8, d = 9216 on
 * 256 compute units needs 9 MiB).  Beyond them: CI_ERR_WORKSPACE, nothing is
 * launched.  status_out: NULL, or a device int32 that receives the call's error
 * word (0, or 1 if a single-launch call gave up waiting; see above) by a copy
 * enqueued after the kernels.
 * All calls on one GPU share that GPU's array: calls that overlap in time on
 * one GPU (different streams, different host threads) race and give wrong
 * results; calls on one stream are fine.  Nothing needs zeroing by the caller.
 */
int coreinfer_ffn_decode_static(const void* x, int64_t B, const ci_ffn_weights* w,
                                int dtype, int act, void* y, int32_t* status_out, void* stream);

/*
 * Union-batched decode.  Several sentences, each with its own frozen core set
 * (stability-guided prediction, Sec. 4.1), decode one token each against the
 * same resident weights (the large-model scenario of Sec. 5.3).  Each row of
 * the UNION of the core sets is read once and applied to the sentences that
 * own it; per sentence the result is exactly the sparse FFN of Sec. 4.2 over
 * its own set, i.e. what coreinfer_ffn_decode computes with core_idx = [B, K].
 *
 * coreinfer_union_build: core_idx [B, K] int32 (device; any order, entries
 *   outside [0, N) are ignored, duplicates allowed), B <= CI_MAX_UNION_SENTENCES.
 *   Out (device, caller-owned): union_idx [max_rows] int32, ascending, the
 *   neurons in at least one set; union_mask [max_rows] uint32, bit s set iff
 *   sentence s owns the row; union_count [1] int32, the number of rows.
 *   max_rows >= min(N, B*K) (CI_ERR_INVALID_ARG otherwise).  Entries past
 *   union_count are left untouched.  ws: coreinfer_union_workspace_size(N) bytes.
 *
 * coreinfer_ffn_decode_union: x [B, d], y [B, d] of `dtype`; w->w_up,
 *   w->w_gate (SwiGLU), w->b_up, w->b_down as for the gathered decode: the full
 *   resident matrices, w_up / w_gate [N, d], w_down NEURON-MAJOR [N, d];
 *   w->core_idx, w->K, w->ld_down and w->down_layout are ignored.  union_idx / union_mask / union_count as
 *   written by coreinfer_union_build with the same max_rows; the row count is
 *   read on the device, so no host synchronisation is needed between the two
 *   calls.  ws: coreinfer_ffn_decode_union_workspace_size bytes, 16-byte aligned.
 *   Deterministic (fixed summation order).  Errors as for coreinfer_ffn_decode.
 */
int coreinfer_union_workspace_size(int64_t N, size_t* bytes);
int coreinfer_union_build(const int32_t* core_idx, int64_t B, int64_t K, int64_t N, int64_t max_rows,
                          int32_t* union_idx, uint32_t* union_mask, int32_t* union_count, void* ws,
                          size_t ws_bytes, void* stream);
int coreinfer_ffn_decode_union_workspace_size(int64_t B, int64_t max_rows, int64_t d, int dtype, int act,
                                              size_t* bytes);
int coreinfer_ffn_decode_union(const void* x, int64_t B, const ci_ffn_weights* w,
                               const int32_t* union_idx, const uint32_t* union_mask,
                               const int32_t* union_count, int64_t max_rows, int dtype, int act,
                               void* y, void* ws, size_t ws_bytes, void* stream);

/*
 * Dense FFN over all N neurons (Def. 1: the activation vector A(x) of every
 * prompt token; with M = 1 also the dense decode baseline).
 *   ReLU:    H = max(X w_up^T + b_up, 0),           A = H
 *   SwiGLU:  H = SiLU(X w_gate^T) * (X w_up^T),     A = |H|
 *   Y = H w_down^T + b_down
 * X [M, d]; Y [M, d] (element type `dtype`, may be NULL); A [M, N] fp32 (may
 * be NULL); at least one of Y, A must be given.  b_up may be NULL and must be
 * NULL for CI_ACT_SWIGLU (CI_ERR_INVALID_ARG).  For Y, H is rounded to
 * `dtype` before the second product when M > 4 (matrix-core path).
 * ws: at least coreinfer_ffn_dense_workspace_size(M, d, N, dtype) bytes.
 */
int coreinfer_ffn_dense_workspace_size(int64_t M, int64_t d, int64_t N, int dtype, size_t* bytes);
int coreinfer_ffn_dense(const void* X, int64_t M,
                        const void* w_up, const void* w_gate, const void* b_up,
                        const void* w_down, const void* b_down, int down_layout,
                        int dtype, int act, int64_t d, int64_t N,
                        void* Y, float* A,
                        void* ws, size_t ws_bytes, void* stream);

/*
 * Dense FFN that hands out the hidden matrix instead of fp32 scores: the
 * prefill pass for coreinfer_select_hidden.  H [M, N] (caller-allocated, of
 * `dtype`, 16-byte aligned) receives max(X w_up^T + b_up, 0) or
 * SiLU(X w_gate^T) * (X w_up^T), rounded once from the fp32 accumulator; Y
 * (nullable) = H w_down^T + b_down as in coreinfer_ffn_dense.  No fp32 matrix
 * of size M x N is written.  Arguments, layouts and errors as for
 * coreinfer_ffn_dense; the workspace only holds split partial products of Y.
 */
int coreinfer_ffn_dense_hidden_workspace_size(int64_t M, int64_t d, int64_t N, int dtype, size_t* bytes);
int coreinfer_ffn_dense_hidden(const void* X, int64_t M, const void* w_up, const void* w_gate,
                               const void* b_up, const void* w_down, const void* b_down, int down_layout,
                               int dtype, int act, int64_t d, int64_t N, void* Y, void* H, void* ws,
                               size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* COREINFER_H_ */
