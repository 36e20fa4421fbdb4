/*
 * knnsoftmax.h -- C ABI of the KNN-softmax output layer for extreme classification on one MI355X (gfx950).
 *
 * Method: "Large-Scale Training System for 100-Million Classification at Alibaba" (KDD'20), Section 3.2
 * "KNN Softmax" (Algorithm 1: KNN graph-based active classes selection; Section 3.2.2: graph building by
 * linear search; Section 3.1 steps 3-6: fc forward, softmax, backward, local weight update of the
 * model-parallel fc layer; Section 3.1: 16-bit compute copy + fp32 copy for the parameter update).
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers, row-major, 16-byte aligned, owned by the caller.  The library
 *     allocates nothing and keeps no state between calls; temporary storage comes from the caller's
 *     workspace `ws` (device memory, 256-byte aligned, at least *_workspace(...) bytes; its contents are
 *     undefined on entry and on exit).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue work:
 *     there is no host synchronisation inside a call, so outputs are valid once the stream has drained.
 *   - Return value: a ks_status for argument-level problems, detected on the host before any launch.
 *   - Data-dependent problems (a label or a class id out of range, ...) cannot be seen from the host; they
 *     set KS_DEV_* bits (atomic OR) in the caller's device word *dev_status, which the caller zeroes
 *     beforehand.  dev_status may be NULL (nothing is reported).  When a bit is set the outputs are
 *     unspecified, but no access leaves the caller's buffers.
 *   - bf16 values are passed as uint16_t bit patterns.  "Class id" is int32.
 *   - Results are deterministic: no floating-point atomics are used anywhere.
 */
#ifndef KNNSOFTMAX_H
#define KNNSOFTMAX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KS_OK = 0,
    KS_INVALID_ARG = 1,        /* NULL required pointer, non-positive size, D % 32 != 0, K + 1 > M, B > M, ... */
    KS_UNSUPPORTED = 2,        /* size beyond what the kernels support (K > 128 or K > C - 1 in the graph build) */
    KS_WORKSPACE_TOO_SMALL = 3,
    KS_HIP_ERROR = 4           /* a launch failed; hipGetLastError() had the details */
} ks_status;

/* bits of *dev_status */
#define KS_DEV_BAD_LABEL 1          /* a label outside [0, C) */
#define KS_DEV_BAD_GRAPH_ID 2       /* a neighbour id outside [-1, C) */
#define KS_DEV_BAD_INDEX 4          /* apply_weight_grad: an index outside [0, C) (that row is skipped) */
#define KS_DEV_IDX_NOT_SORTED 8     /* apply_weight_grad: idx_sorted_unique was promised but does not hold */
#define KS_DEV_BAD_COUNT 16         /* a device-side count (n, n_active) outside [0, n_max]; a compressed-graph list
                                       longer than promised or outside its array; a flat array too short */
#define KS_DEV_RANGE 32             /* KS_FLAG_UNIT_ROWS was promised but a sample's exponentials overflowed or all vanished */

/* bits of the `flags` argument of the softmax entry points */
#define KS_FLAG_UNIT_ROWS 1u        /* every row of W_bf16 and X_bf16 has L2 norm <= 1 (up to rounding) */
#define KS_FLAG_PAD_RANDOM 2u       /* knn_select_active_csr: fill the active list up to M with randomly drawn classes */
#define KS_FLAG_TRUSTED_LIST 4u     /* the calls that take a selection made earlier: the list is the unmodified output of this
                                       library's selection for the same C and M; it is used where it lies, without the
                                       validating copy (a broken promise may read outside W) */

#define KS_DTYPE_BF16 0
#define KS_DTYPE_FP32 1

/* Largest K the graph build supports, and the limits of the selection. */
#define KS_MAX_GRAPH_K 128

const char *ks_version(void);

/* ------------------------------------------------------------------------------------------------------
 * knn_graph_build -- Section 3.2.2: exact K nearest neighbours of every class-weight row among all rows,
 * by linear search with inner-product similarity; a 16-bit matrix-core pass recalls k' > K candidates per
 * row, which are then re-ranked exactly (the paper's two-precision scheme).
 *
 *   W      [C, D]  class weights (normally L2-normalised rows; used as given), dtype KS_DTYPE_BF16 or _FP32
 *   graph  [C, K]  out: row i = the K ids j != i with the largest similarity, in descending similarity,
 *                  ties to the lowest id
 *   sims   [C, K]  out, may be NULL: the similarities of those neighbours (fp32 rounding of the fp64 value)
 *
 * Similarity used for ranking = sum over d ascending of (double)W[i,d] * (double)W[j,d], accumulated
 * sequentially in fp64; two similarities tie only when these fp64 values are equal.  The result is exact:
 * a row whose recall cannot be certified from the matrix-core pass' error bound is redone by exhaustive
 * fp64 search inside the same call.
 * Requires 2 <= C < 2^31, D % 32 == 0, 1 <= K <= min(C - 1, KS_MAX_GRAPH_K).
 * ---------------------------------------------------------------------------------------------------- */
size_t knn_graph_build_workspace(int64_t C, int D, int K, int dtype);
int knn_graph_build(const void *W, int dtype, int64_t C, int D, int K, int32_t *graph, float *sims,
                    void *ws, size_t ws_bytes, int32_t *dev_status, void *stream);

/* knn_graph_build_plan -- how knn_graph_build divides the linear search of Section 3.2.2 when it computes every
 * similarity once and uses it for both rows of the pair (large C; D = 128, 256 or 512; K <= 64).  Host-only, no GPU
 * work; for tests and tools.
 *   n_workgroups [1]   out (host): workgroups of that pass, 0 when this problem takes the plain pass
 *   out          [12]  out (host), may be NULL: for `workgroup` in [0, *n_workgroups):
 *                      [0] its block of 256 resident rows (rows 256 b .. 256 b + 255), or -1: none;
 *                      [1 + 2 p], [2 + 2 p], p = 0..4: streamed rows [first, end) of its five ranges (end <= first:
 *                      empty); range 0 is the 768-row super-block that holds its own block;
 *                      [11] bit k set: inside range 0 it pairs its rows with block k of that super-block (its own
 *                      block is always searched, for its own rows only)
 * Every pair of different blocks is paired by exactly one workgroup: inside range 0 as [11] says, in ranges 1..4
 * with every row.  Returns KS_OK, or KS_INVALID_ARG / KS_UNSUPPORTED as knn_graph_build would. */
int knn_graph_build_plan(int64_t C, int D, int K, int dtype, int workgroup, int32_t *n_workgroups, int32_t *out);

/* ------------------------------------------------------------------------------------------------------
 * knn_select_active -- Algorithm 1 without its random fill-up branch: the de-duplicated union of the
 * labels' neighbour lists, each list headed by the label itself; when more than M classes remain, the M
 * with the best ranking score are kept (score of a class = its smallest position in any contributing list,
 * the label itself having position 0; ties to the lowest class id).  Entries -1 in `graph` are empty.
 *
 *   labels      [B]     class ids in [0, C)
 *   graph       [C, K]  neighbour lists (K may be 0, graph then unused)
 *   active_idx  [M]     out: the active class ids in ascending order; entries >= *n_active are -1
 *   n_active    [1]     out (device): number of active classes, 1 <= *n_active <= M
 *   target_pos  [B]     out: position of labels[i] in active_idx
 * Requires B <= M and K + 1 <= M (every label and a whole list always fit).
 * This is the first stage of knn_softmax_fwd_bwd, exported on its own.
 * ---------------------------------------------------------------------------------------------------- */
size_t knn_select_workspace(int64_t C, int B, int K, int M);
int knn_select_active(const int32_t *labels, const int32_t *graph, int64_t C, int B, int K, int M,
                      int32_t *active_idx, int32_t *n_active, int32_t *target_pos,
                      void *ws, size_t ws_bytes, int32_t *dev_status, void *stream);

/* ------------------------------------------------------------------------------------------------------
 * knn_select_active_static -- knn_select_active for callers that cannot allocate device memory or bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments (without ws / ws_bytes), same kernels, same results bit for bit; the scratch memory the kernels need
 * (the staging array of the candidates, or the score table of the large-C path) is a device array of
 * KS_SELECT_STATIC_BYTES that is part of the library's code object: every GPU the library runs on holds its own
 * copy from the first call on that GPU until the process ends.  The call allocates nothing and frees nothing.
 *
 * Limit: knn_select_workspace(C, B, K, M) <= KS_SELECT_STATIC_BYTES, else KS_UNSUPPORTED (nothing is launched).
 * All calls on one GPU share the one array: calls that overlap in time on the same GPU (different streams or
 * threads) race with each other; calls on one stream are ordered and safe.  Nothing in the array has to
 * survive between calls and nothing has to be zero on entry (the kernels write every word before reading it).
 * ---------------------------------------------------------------------------------------------------- */
#define KS_SELECT_STATIC_BYTES (2u << 20)
int knn_select_active_static(const int32_t *labels, const int32_t *graph, int64_t C, int B, int K, int M,
                             int32_t *active_idx, int32_t *n_active, int32_t *target_pos,
                             int32_t *dev_status, void *stream);

/* ------------------------------------------------------------------------------------------------------
 * knn_gather_rows -- W_active of Algorithm 1 as a dense matrix: out[a, :] = W_bf16[active_idx[a], :] for
 * a < *n_active.  (knn_softmax_fwd_bwd gathers inside its matrix kernels and does not call this; it is
 * exported for callers that want the rows, and to measure the gather on its own.)
 *   out [M, D] bf16; rows >= *n_active are not written.
 * ---------------------------------------------------------------------------------------------------- */
int knn_gather_rows(const uint16_t *W_bf16, const int32_t *active_idx, const int32_t *n_active, int M,
                    int64_t C, int D, uint16_t *out, int32_t *dev_status, void *stream);

/* ------------------------------------------------------------------------------------------------------
 * knn_softmax_fwd_bwd -- one step of the KNN-softmax layer on this GPU's classes (Section 3.2; Section 3.1
 * steps 3-5): selection as in knn_select_active, then on the active columns only
 *     Z_ia  = scale * <X_i, W[active_idx[a]]>                         (fc forward, bf16 in, fp32 accumulate)
 *     loss_i = logsumexp_a(Z_ia) - Z_{i,target_pos[i]},  loss_mean = mean_i loss_i      (softmax + CE)
 *     dZ_ia = (grad_scale / B) * (softmax(Z_i)_a - [a == target_pos[i]])                (softmax backward)
 *     dX_i  = scale * sum_a dZ_ia W[active_idx[a]]                                      (fc backward)
 *     dW_active[a] = scale * sum_i dZ_ia X_i
 * X and W rows are used as given (callers pass L2-normalised rows); gradients are with respect to them.
 * grad_scale (loss scaling) multiplies the gradients only, not the reported losses.
 *
 * flags: 0, or KS_FLAG_UNIT_ROWS when the caller normalises the rows of W and X as the paper does (Section
 * 3.2: the fc layer works on normalised weights and features).  All logits then lie in [-scale, scale], and
 * for scale <= 40 the library evaluates the softmax against that fixed bound in a single sweep over the
 * active rows instead of a statistics sweep followed by a gradient sweep.  The result is the same function
 * of the inputs (the bound only shifts the exponent range), also when some norms exceed 1; should a
 * sample's exponentials overflow or all underflow, KS_DEV_RANGE is raised and the outputs are unspecified.
 *
 *   W_bf16 [C, D], X_bf16 [B, D], labels [B], graph [C, K]           inputs
 *   active_idx [M], n_active [1], target_pos [B]                     out, as in knn_select_active
 *   loss_per_sample [B] fp32, loss_mean [1] fp32                     out
 *   dX [B, D] fp32                                                   out
 *   dW_active [M, D] fp32                                            out; rows >= *n_active are not written
 * Requires D % 32 == 0, B <= M, K + 1 <= M, C < 2^31.
 * ---------------------------------------------------------------------------------------------------- */
size_t knn_softmax_workspace(int64_t C, int D, int B, int K, int M);
int knn_softmax_fwd_bwd(const uint16_t *W_bf16, const uint16_t *X_bf16, const int32_t *labels,
                        const int32_t *graph, int64_t C, int D, int B, int K, int M, float scale,
                        float grad_scale, uint32_t flags, int32_t *active_idx, int32_t *n_active,
                        int32_t *target_pos, float *loss_per_sample, float *loss_mean, float *dX,
                        float *dW_active, void *ws, size_t ws_bytes, int32_t *dev_status, void *stream);

/* knn_softmax_fwd_bwd_update -- the whole step of the layer in one call: knn_softmax_fwd_bwd followed by the
 * weight update of Section 3.1 step 6 (apply_weight_grad with idx = active_idx, idx_sorted_unique), with the
 * same results bit for bit:
 *     W_master[active_idx[a], :] += alpha * dW_active[a, :],   W_bf16[same rows] = bf16 of the new values.
 * For D % 64 == 0 the update runs inside the kernel that produces dW_active, so the gradient does not travel
 * through memory; dW_active may then be NULL (not stored).  Otherwise dW_active is required and the two steps
 * run one after the other.  W_bf16 is read by the forward pass and updated at the end of the call. */
int knn_softmax_fwd_bwd_update(float *W_master, uint16_t *W_bf16, const uint16_t *X_bf16, const int32_t *labels,
                               const int32_t *graph, int64_t C, int D, int B, int K, int M, float scale,
                               float grad_scale, float alpha, uint32_t flags, int32_t *active_idx, int32_t *n_active,
                               int32_t *target_pos, float *loss_per_sample, float *loss_mean, float *dX,
                               float *dW_active, void *ws, size_t ws_bytes, int32_t *dev_status, void *stream);

/* knn_softmax_fwd_bwd_update_selected -- the step without its first stage: the active list comes in as
 * computed by an earlier knn_select_active (or knn_select_active_csr) call.  Algorithm 1 only reads the labels and
 * the graph, so a training loop can run the selection of batch n + 1 on a second stream while the contractions of
 * batch n run (Section 3.2.1 asks for the active classes to be fetched quickly: here the fetch leaves the
 * critical path altogether).  Everything else as in knn_softmax_fwd_bwd_update, with the same results bit for bit.
 *
 *   active_idx [M], n_active [1], target_pos [B]     in (device): the outputs of the selection
 *   W_master                                         may be NULL: no update (then dW_active is required)
 * The list is validated on the device before use: ids outside [0, C) raise KS_DEV_BAD_INDEX, a count outside
 * [0, M] KS_DEV_BAD_COUNT, target positions at or beyond the count KS_DEV_BAD_LABEL; the outputs are then
 * unspecified, but every access stays in bounds.  Target positions must lie in [0, *n_active), as the selection
 * on a GPU that owns all classes produces them (a node of a sharded layer uses the split-softmax calls below).
 * With KS_FLAG_TRUSTED_LIST the caller promises that the three arrays are what knn_select_active (or the _next call
 * below) wrote for this C and M, unmodified: they are then read in place, nothing is validated or copied (one small
 * launch less), and ids out of range would be read out of bounds.
 * Requires D % 32 == 0, B <= M. */
size_t knn_softmax_selected_workspace(int64_t C, int D, int B, int M);
int knn_softmax_fwd_bwd_update_selected(float *W_master, uint16_t *W_bf16, const uint16_t *X_bf16,
                                        const int32_t *active_idx, const int32_t *n_active, const int32_t *target_pos,
                                        int64_t C, int D, int B, int M, float scale, float grad_scale, float alpha,
                                        uint32_t flags, float *loss_per_sample, float *loss_mean, float *dX,
                                        float *dW_active, void *ws, size_t ws_bytes, int32_t *dev_status, void *stream);

/* knn_softmax_fwd_bwd_update_selected_next -- knn_softmax_fwd_bwd_update_selected for this batch AND Algorithm 1
 * (knn_select_active) for the NEXT batch in the same launches: the selection needs only the next batch's labels and the
 * graph (Section 3.2.1), so it runs as extra workgroups of the step's own dX and dW launches, on compute units those
 * leave idle -- no second stream, no dependency between streams, and the selection is off the step's critical path.
 * A training loop calls knn_select_active once for its first batch and this from then on.
 *
 *   labels_next [B] int32, graph [C, K] int32        in (device): the next batch's labels; the graph as in knn_select_active
 *   active_idx_next [M], n_active_next [1], target_pos_next [B]   out (device): exactly what knn_select_active writes for
 *                       labels_next (bit for bit).  They MAY be the buffers this call's active_idx / n_active /
 *                       target_pos came in: the call copies its own list before the selection starts (not with
 *                       KS_FLAG_TRUSTED_LIST, which reads the list in place: then they must be other buffers, else
 *                       KS_INVALID_ARG -- a loop alternates between two sets).
 *   everything else     as in knn_softmax_fwd_bwd_update_selected, with the same results bit for bit
 * Requires K + 1 <= M besides that call's conditions.  When D is not a multiple of 64, or C exceeds the 393,216 classes
 * whose bitmap one workgroup holds, the selection runs after the step as launches of its own (same results).
 * Workspace: knn_softmax_selected_next_workspace. */
size_t knn_softmax_selected_next_workspace(int64_t C, int D, int B, int K, int M);
int knn_softmax_fwd_bwd_update_selected_next(float *W_master, uint16_t *W_bf16, const uint16_t *X_bf16,
                                             const int32_t *active_idx, const int32_t *n_active,
                                             const int32_t *target_pos, int64_t C, int D, int B, int M, float scale,
                                             float grad_scale, float alpha, uint32_t flags, float *loss_per_sample,
                                             float *loss_mean, float *dX, float *dW_active, const int32_t *labels_next,
                                             const int32_t *graph, int K, int32_t *active_idx_next,
                                             int32_t *n_active_next, int32_t *target_pos_next, void *ws, size_t ws_bytes,
                                             int32_t *dev_status, void *stream);

/* Measurement aid: knn_softmax_fwd_bwd (W_master == NULL) or knn_softmax_fwd_bwd_update with one hipEvent_t
 * recorded on `stream` at each stage boundary, so that a caller can time the stages of a step without a profiler.
 * events[0..KS_N_PHASE_EVENTS) are created by the caller (hipEventCreate); event k is recorded: 0 at entry, 1
 * after the selection, 2 after the first sweep over the active rows (softmax statistics; with KS_FLAG_UNIT_ROWS
 * the only sweep, which also writes the exponentials), 3 after the per-sample combine and the loss mean, 4 after
 * the second sweep (logit gradient; nothing with KS_FLAG_UNIT_ROWS), 5 after the dX partial GEMM, 6 after the dX
 * reduction, 7 after the dW GEMM (and the update, if any).  Same results as the entry points it stands for. */
#define KS_N_PHASE_EVENTS 8
int knn_softmax_fwd_bwd_profiled(float *W_master, uint16_t *W_bf16, const uint16_t *X_bf16, const int32_t *labels,
                                 const int32_t *graph, int64_t C, int D, int B, int K, int M, float scale,
                                 float grad_scale, float alpha, uint32_t flags, int32_t *active_idx,
                                 int32_t *n_active, int32_t *target_pos, float *loss_per_sample, float *loss_mean,
                                 float *dX, float *dW_active, void *ws, size_t ws_bytes, int32_t *dev_status,
                                 void *stream, void **events, int n_events);

/* ------------------------------------------------------------------------------------------------------
 * full_softmax_fwd_bwd -- the full-softmax layer the paper compares against (Section 3.2, Table 3): the
 * same computation with every class active (active_idx = 0..C-1, no graph).  dW is dense [C, D].
 * ---------------------------------------------------------------------------------------------------- */
size_t full_softmax_workspace(int64_t C, int D, int B);
int full_softmax_fwd_bwd(const uint16_t *W_bf16, const uint16_t *X_bf16, const int32_t *labels, int64_t C,
                         int D, int B, float scale, float grad_scale, uint32_t flags, float *loss_per_sample,
                         float *loss_mean, float *dX, float *dW, void *ws, size_t ws_bytes,
                         int32_t *dev_status, void *stream);

/* ------------------------------------------------------------------------------------------------------
 * apply_weight_grad -- Section 3.1 step 6: the model-parallel fc layer updates its weights from the local
 * gradient; the fp32 copy is updated and the 16-bit compute copy refreshed from it (Section 3.1, mixed
 * precision).  For every class c that occurs in idx[0 .. n):
 *     W_master[c, :] += alpha * sum_{p : idx[p] == c} dW[p, :]        (sum in ascending p)
 *     W_bf16[c, :]    = bf16(W_master[c, :])                          (round to nearest even)
 * Rows that do not occur are not touched.  alpha folds -learning_rate and 1/grad_scale.
 *
 *   idx [n_max] class ids; may repeat (e.g. the concatenated active lists of several accumulated
 *               micro-batches) unless idx_sorted_unique != 0, which promises strictly ascending ids (true
 *               for active_idx of one step) and selects the single-pass kernel; a broken promise sets
 *               KS_DEV_IDX_NOT_SORTED.
 *   n   [1]     device count of valid entries (NULL = n_max)
 *   dW  [n_max, D] fp32 gradient rows
 * Requires D % 4 == 0.
 * ---------------------------------------------------------------------------------------------------- */
size_t apply_weight_grad_workspace(int64_t C, int D, int n_max, int idx_sorted_unique);
int apply_weight_grad(float *W_master, uint16_t *W_bf16, const int32_t *idx, const int32_t *n, int n_max,
                      const float *dW, float alpha, int64_t C, int D, int idx_sorted_unique,
                      void *ws, size_t ws_bytes, int32_t *dev_status, void *stream);

/* ------------------------------------------------------------------------------------------------------
 * The softmax split over the nodes of the model-parallel layer -- Section 3.1, steps 3 to 5: every node
 * computes the logits of its own classes for the whole (gathered) batch; the softmax needs each sample's maximum
 * and sum of exponentials over all nodes, which the nodes exchange (a tiny message, Section 3.3.1); then every node
 * forms the gradient of its own logits, its weight gradient and its contribution to the feature gradient.
 * This is one node's half of it, in two calls around the exchange:
 *
 * knn_softmax_fwd_stats: logits of the active classes (active_idx, n_active, target_pos as written by
 *   knn_select_active or knn_select_active_csr: local ids, target_pos = -1 for a sample whose class another node
 *   owns) and per sample
 *     row_max [B], row_sumexp [B]:  a pair with  sum_a exp(z_ia - row_max_i) = row_sumexp_i, not necessarily
 *                  the maximum itself: where the one-sweep softmax runs (KS_FLAG_UNIT_ROWS, D = 128, 256 or 512,
 *                  scale <= 40) row_max = scale for every sample on every node, so that combining the nodes
 *                  comes down to ADDING their sums; otherwise the pair is normalised to row_sumexp = 1.  A node
 *                  without active classes gives (-infinity, 0)
 *     target_logit [B]:  z of the sample's own class, 0 where target_pos < 0
 *   The caller combines the nodes p:  M_i = max_p row_max,  S_i = sum_p row_sumexp * exp(row_max - M_i),
 *   T_i = sum_p target_logit.
 * knn_softmax_bwd_from_stats: with global_max = M, global_sumexp = S, global_target_logit = T:
 *     loss_per_sample_i = M_i + log S_i - T_i (the same on every node), loss_mean;
 *     dZ_ia = (grad_scale / B) * (exp(z_ia - M_i) / S_i - [a == target_pos[i]]);
 *     dX [B, D] = scale * dZ * W_active  -- THIS NODE'S CONTRIBUTION, to be summed over the nodes;
 *     dW_active [M, D] = scale * dZ^T * X  (rows >= n_active not written), for apply_weight_grad.
 * Same arguments (W, X, selection, scale, flags, B, M) in both calls, and the SAME workspace, untouched in between:
 * with KS_FLAG_UNIT_ROWS the first call leaves the exponentials there and the second call makes no second sweep.
 * B is the gathered batch (the mean and grad_scale / B refer to it).  An active_idx entry outside [0, C) sets
 * KS_DEV_BAD_INDEX (and is replaced by row 0), a target_pos >= n_active sets KS_DEV_BAD_LABEL (treated as -1).
 * Requires D % 64 == 0 (KS_UNSUPPORTED otherwise), B <= M not required.  Tolerances as knn_softmax_fwd_bwd.
 * Both calls take KS_FLAG_TRUSTED_LIST (the list is the unmodified output of this library's selection: read in place, no
 * validating copy).
 *
 * knn_softmax_bwd_from_stats_next: the same second call, and in its launches knn_select_active_csr for the NEXT batch
 * (labels_next .. target_pos_next: that call's arguments, select_flags = its flags; C is its C_loc) -- the selection needs
 * only the next batch's labels and the node's compressed graph, so it runs as extra workgroups of the dX and dW launches
 * and leaves the node's critical path (Section 3.2.1).  Outputs exactly as knn_select_active_csr writes them; they may be
 * the buffers this call's list came in, except with KS_FLAG_TRUSTED_LIST.  Requires B <= M and K_max + 1 <= M.  Nodes of
 * more than 393,216 classes run the selection after the step instead.  Workspace: knn_softmax_split_next_workspace,
 * passed to both calls of a step.
 * ---------------------------------------------------------------------------------------------------- */
size_t knn_softmax_split_workspace(int64_t C, int D, int B, int M);
int knn_softmax_fwd_stats(const uint16_t *W_bf16, const uint16_t *X_bf16, const int32_t *active_idx,
                          const int32_t *n_active, const int32_t *target_pos, int64_t C, int D, int B, int M,
                          float scale, uint32_t flags, float *row_max, float *row_sumexp, float *target_logit,
                          void *ws, size_t ws_bytes, int32_t *dev_status, void *stream);
int knn_softmax_bwd_from_stats(const uint16_t *W_bf16, const uint16_t *X_bf16, const int32_t *active_idx,
                               const int32_t *n_active, const int32_t *target_pos, const float *global_max,
                               const float *global_sumexp, const float *global_target_logit, int64_t C, int D, int B,
                               int M, float scale, float grad_scale, uint32_t flags, float *loss_per_sample,
                               float *loss_mean, float *dX, float *dW_active, void *ws, size_t ws_bytes,
                               int32_t *dev_status, void *stream);
size_t knn_softmax_split_next_workspace(int64_t C, int D, int B, int K_max, int M);
int knn_softmax_bwd_from_stats_next(const uint16_t *W_bf16, const uint16_t *X_bf16, const int32_t *active_idx,
                                    const int32_t *n_active, const int32_t *target_pos, const float *global_max,
                                    const float *global_sumexp, const float *global_target_logit, int64_t C, int D, int B,
                                    int M, float scale, float grad_scale, uint32_t flags, float *loss_per_sample,
                                    float *loss_mean, float *dX, float *dW_active, const int32_t *labels_next,
                                    const int32_t *counts, const int64_t *offsets, const int32_t *flat, int64_t flat_len,
                                    int64_t Cg, int64_t c0, int K_max, uint32_t select_flags, uint64_t pad_seed,
                                    int32_t *active_idx_next, int32_t *n_active_next, int32_t *n_found_next,
                                    int32_t *target_pos_next, void *ws, size_t ws_bytes, int32_t *dev_status, void *stream);

/* ------------------------------------------------------------------------------------------------------
 * knn_graph_update -- one hop of the distributed graph build of Section 3.2.2 (the shards of W travel from
 * node to node; every node searches each visiting shard and keeps the best K so far for its own rows).
 *   W_local [C_loc, D]  the node's rows (dtype as knn_graph_build); their ids in the whole problem are
 *                       local_offset + row
 *   W_visit [C_vis, D]  the visiting shard, ids visit_offset + row (the node's own shard visits too, once)
 *   graph   [C_loc, K]  in/out: the lists so far, ids of the whole problem in rank order, -1 = empty slot
 *                       (a build starts from all -1)
 *   sims    [C_loc, K]  in/out, fp64: canonical similarities of the entries (exact; fp32 would lose the order
 *                       of near-ties between hops); -infinity in empty slots on output
 * After the call each row's list holds the best K of (list so far) U (visiting rows) by (canonical similarity
 * descending, id ascending) -- the same order and arithmetic as knn_graph_build -- the row itself excluded; a
 * visiting row that is in the list already is ignored, so a shard that visits twice changes nothing.  After
 * every shard has visited, the lists equal the graph knn_graph_build computes on the whole W.
 * Requires D % 32 == 0, K <= KS_MAX_GRAPH_K, all ids < 2^31.  Workspace: knn_graph_update_workspace.
 * ---------------------------------------------------------------------------------------------------- */
size_t knn_graph_update_workspace(int64_t C_loc, int64_t C_vis, int D, int K, int dtype);
int knn_graph_update(const void *W_local, const void *W_visit, int dtype, int64_t C_loc, int64_t C_vis, int D, int K,
                     int64_t local_offset, int64_t visit_offset, int32_t *graph, double *sims, void *ws,
                     size_t ws_bytes, int32_t *dev_status, void *stream);

/* ------------------------------------------------------------------------------------------------------
 * One node of the sharded layer -- Section 3.2.3 (graph compression, quick access) and the fill-up branch of
 * Algorithm 1.  The node owns the classes [c0, c0 + C_loc) of a problem with Cg classes; labels and the dense
 * graph carry ids of the whole problem, everything the node produces carries local ids (global id - c0).
 *
 * knn_graph_compress -- (i) of Section 3.2.3: for every class g of the whole problem keep only the neighbours the
 *   node owns, in the order of g's list, as local ids; the lists are laid end to end:
 *     graph  [Cg, K]   dense graph, global ids, -1 = empty slot
 *     counts [Cg]      out: length of g's compressed list
 *     offsets[Cg + 1]  out: running sum of the counts (offsets[Cg] = total length)
 *     flat   [flat_capacity] out: the lists; NULL = counts and offsets only (read offsets[Cg], allocate, call
 *                      again).  A capacity below the total sets KS_DEV_BAD_COUNT; lists that do not fit are not
 *                      written.
 * knn_select_active_csr -- Algorithm 1 on the compressed graph ((ii) of Section 3.2.3: a sample finds its list at
 *   offsets[label]):
 *     labels [B]       global ids.  A sample whose class the node owns contributes that class at list position 0;
 *                      entry j of its class's compressed list counts as position j + 1 (ranking for the cut to M
 *                      as in knn_select_active: smallest position first, ties to the lowest local id)
 *     K_max            upper bound of the list lengths (K of the dense graph); a longer list, or one that does
 *                      not lie inside flat[0 .. flat_len), sets KS_DEV_BAD_COUNT and is not read
 *     flags            KS_FLAG_PAD_RANDOM: when fewer than M classes are found the list is filled up to
 *                      min(M, C_loc) with classes drawn without replacement from those not chosen.  The k-th
 *                      draw (k = 0, 1, ...) is x_7 of: b = number of bits of the smallest power of two >= C_loc
 *                      (at least 1), all arithmetic modulo 2^b, s1 = (b+1)/2, s2 = max(1, b/3),
 *                        x_0 = k + lo32(pad_seed), x_1 = x_0 * 0x9E3779B1, x_2 = x_1 ^ (x_1 >> s1),
 *                        x_3 = x_2 * 0x85EBCA6B,   x_4 = x_3 ^ (x_3 >> s2), x_5 = x_4 * 0xC2B2AE35,
 *                        x_6 = x_5 ^ (x_5 >> s1),  x_7 = x_6 + hi32(pad_seed);
 *                      draws >= C_loc or already in the list are passed over.  (The paper says only "random
 *                      sample"; a caller changes pad_seed from step to step.)
 *     active_idx [M]   out: ascending local ids, -1 beyond n_active;  n_found [1] (may be NULL): classes found by
 *                      the lists, before the fill-up
 *     target_pos [B]   out: position of the sample's class in active_idx, -1 if another node owns the class
 *   Requires B <= M and K_max + 1 <= M.  Workspace: knn_select_active_csr_workspace.
 * ---------------------------------------------------------------------------------------------------- */
size_t knn_graph_compress_workspace(int64_t Cg, int K);
int knn_graph_compress(const int32_t *graph, int64_t Cg, int K, int64_t c0, int64_t C_loc, int32_t *counts,
                       int64_t *offsets, int32_t *flat, int64_t flat_capacity, void *ws, size_t ws_bytes,
                       int32_t *dev_status, void *stream);
size_t knn_select_active_csr_workspace(int64_t C_loc, int B, int K_max, int M);
int knn_select_active_csr(const int32_t *labels, const int32_t *counts, const int64_t *offsets, const int32_t *flat,
                          int64_t flat_len, int64_t Cg, int64_t c0, int64_t C_loc, int B, int K_max, int M,
                          uint32_t flags, uint64_t pad_seed, int32_t *active_idx, int32_t *n_active, int32_t *n_found,
                          int32_t *target_pos, void *ws, size_t ws_bytes, int32_t *dev_status, void *stream);

/* ------------------------------------------------------------------------------------------------------
 * Normalisation inside the layer -- Section 3.2.3 (GPU pipeline, step 2): the graph and the softmax work on normalised W and X,
 * and the normalisation itself runs on the GPU.  The layer keeps W un-normalised in fp32 (W_master), its
 * contractions read the normalised 16-bit copy W_hat = W / |W| (row-wise L2 norm; pass it wherever an entry
 * point above takes W_bf16, with KS_FLAG_UNIT_ROWS), and a gradient g with respect to a normalised row is
 * brought back to the row v itself through
 *     dv = (g - v_hat <v_hat, g>) / |v|,       v_hat = v / |v|.
 * Row reductions are taken in fp64.  A zero row has inv_norm 0, a zero normalised row and a zero gradient.
 *
 * knn_normalize_rows:  V [n, D] (dtype KS_DTYPE_*) ->  V_hat_bf16 [n, D] = bf16(fp32(V / |V|)) and
 *     inv_norm [n] = 1 / |V| (either output may be NULL, not both).  Used for X every step and for W once,
 *     when the layer is set up.
 * knn_norm_backward_rows:  dV [n, D] fp32 from V [n, D] (dtype) and G [n, D] fp32 (the gradient with respect
 *     to V / |V|, e.g. dX of knn_softmax_fwd_bwd); dV may alias G.
 * apply_weight_grad_normalized -- Section 3.1 step 6 with the normalisation folded in.  dW_hat [n_max, D] is
 *     the gradient with respect to the NORMALISED rows (dW_active of knn_softmax_fwd_bwd run on W_hat).  For
 *     every class c that occurs in idx[0 .. n):  g = sum of its rows of dW_hat (ascending p);
 *         W_master[c, :] += alpha * (g - w_hat <w_hat, g>) / |w|          (w = the row before the update)
 *         inv_norm[c]     = 1 / |W_master[c, :]|                          (the row after the update)
 *         W_hat_bf16[c,:] = bf16(fp32(W_master[c, :] * inv_norm[c]))
 *     W_hat_bf16 and inv_norm may be NULL.  idx, n, idx_sorted_unique, dev_status as for apply_weight_grad;
 *     the general path needs the workspace of apply_weight_grad_normalized_workspace (sort keys plus one
 *     summed gradient row per position).
 * All three require D % 4 == 0 and return KS_INVALID_ARG otherwise; all pointers are device pointers.
 * ---------------------------------------------------------------------------------------------------- */
int knn_normalize_rows(const void *V, int dtype, int64_t n, int D, uint16_t *V_hat_bf16, float *inv_norm,
                       void *stream);
int knn_norm_backward_rows(const void *V, int dtype, const float *G, int64_t n, int D, float *dV, void *stream);
size_t apply_weight_grad_normalized_workspace(int64_t C, int D, int n_max, int idx_sorted_unique);
int apply_weight_grad_normalized(float *W_master, uint16_t *W_hat_bf16, float *inv_norm, const int32_t *idx,
                                 const int32_t *n, int n_max, const float *dW_hat, float alpha, int64_t C, int D,
                                 int idx_sorted_unique, void *ws, size_t ws_bytes, int32_t *dev_status,
                                 void *stream);

/* ------------------------------------------------------------------------------------------------------
 * Measurement aids for the roofline report: what the chip sustains on the two resources the kernels are priced
 * against (the nominal peaks are 2.5 PFLOP/s of dense bf16 matrix work and 8 TB/s of HBM traffic).
 *   ks_peak_mfma  launches a loop of independent 32x32x16 bf16 matrix instructions on registers only;
 *                 *flops (host, may be NULL) receives the number of floating-point operations of the launch;
 *                 out (device) needs workgroups * 256 floats
 *   ks_peak_copy  launches a streaming copy of `bytes` (multiple of 16) from src to dst (device, 16-byte aligned);
 *                 the traffic of the launch is 2 * bytes
 * The caller times the launches with events on `stream` and divides.
 * ---------------------------------------------------------------------------------------------------- */
int ks_peak_mfma(float *out, int workgroups, int iters, double *flops, void *stream);
int ks_peak_copy(const void *src, void *dst, size_t bytes, int workgroups, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* KNNSOFTMAX_H */
