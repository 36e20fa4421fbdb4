/*
 * grad_topk.h -- C ABI of the layer-wise top-k selection for gradient sparsification on one MI355X (gfx950).
 *
 * Method: "Large-Scale Training System for 100-Million Classification at Alibaba" (KDD'20), Section 3.3.2
 * "Efficient layer-wise top-k sparsification" and its figure on divide-and-conquer top-k selection: the top-k
 * of a large gradient tensor is found exactly in two steps -- the tensor is cut into M chunks whose top-k are
 * taken side by side, then the top-k of the M*k survivors -- and tensors are grouped so that one launch serves
 * many layers.  Part of the same shared library as knnsoftmax.h; the conventions stated there hold here too
 * (device pointers unless marked HOST, caller-owned memory, nothing allocated, calls only enqueue work on
 * `stream`, ks_status return values).
 *
 * Definition of the result (what the paper leaves open is fixed as follows).  Of tensor t, the k[t] elements
 * of largest magnitude |g|, magnitudes compared as the 31-bit patterns of |g| (the numeric order for finite
 * values and infinities; NaN patterns rank above infinity; +0 and -0 are equal); among equal magnitudes the
 * lowest index wins.  They are emitted in descending magnitude, equal magnitudes in ascending index, so the
 * output is unique and independent of M.
 */
#ifndef GRAD_TOPK_H
#define GRAD_TOPK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KS_TOPK_MAX_K 4096 /* largest k per tensor */

/* ------------------------------------------------------------------------------------------------------
 * grad_topk_plan -- host-side planning for a group of T tensors stored back to back (Section 3.3.2: "grouping
 * tensors"): cuts every tensor into chunks and lays out the selection steps and the survivors' buffer.  No
 * device work.  The plan depends only on the sizes, so it is made once per model.
 *
 *   offsets  HOST [T + 1]  tensor t is g[offsets[t] .. offsets[t+1]) of the flat gradient array; ascending,
 *                          every tensor has 1 <= n[t] < 2^31 elements
 *   k        HOST [T]      elements to select from tensor t, 1 <= k[t] <= min(n[t], KS_TOPK_MAX_K)
 *   chunks   0: tensor t is cut into M[t] = ceil(n[t] / 32,768) chunks;  > 0: M[t] = min(chunks, n[t]) for every
 *            tensor (for tests and sweeps); chunks are consecutive ranges of ceil(n / M) elements
 *   plan     HOST [plan_capacity] out, may be NULL: the plan, a flat int64 array that the caller also copies to
 *            device memory as it is
 * The paper's method has two steps (top-k of every chunk, then top-k of the M*k survivors).  Here one workgroup
 * performs one selection, and no selection gets more than 32,768 items: where M * k exceeds that, the survivors
 * are first reduced in groups of floor(32,768 / k) chunks, and so on -- a tree of exact selections with the
 * paper's two steps as its smallest case, one launch per level for the whole group of tensors ("plain tree").
 * With chunks == 0, a tensor of several chunks whose k is small for its size goes a shorter way, in three steps
 * whatever its size: (1) a threshold, the r-th largest magnitude of 4,096 evenly spaced elements, r >= 16 chosen so
 * that about 4 k elements of the tensor are expected at or above it; (2) every chunk hands on its elements at or
 * above the threshold (one pass, no selection: the chunks of the paper's first step hand on k elements each,
 * whatever the rest of the tensor holds); (3) the final selection over what arrived.  The number that arrives is an
 * order statistic's count (n / 4,096 times a Gamma(r) variable for any values), fewer than k for about one tensor in
 * 100,000; it is checked in step (3), and if it is below k or beyond 32,768 (long runs of one magnitude), the
 * workgroup of step (3) runs the tensor's plain tree itself.  The output is the same bits on every way.
 * Returns the number of int64 words of the plan (written only if plan != NULL and plan_capacity suffices), or
 * the negative of a ks_status for bad arguments.  Plan words a caller may read: [1] = T, [2] = steps launched
 * (workgroups of 1,024 threads; a chunk of step (2) is four workgroups of 256), [3] = workspace in 8-byte words,
 * [4] = sum of k, [5] = elements in all, [6] = levels (launches per call, plus one when [29] > 0), [7] = step records
 * in all (the plain trees behind the shorter ways included), [29] = chunks that take step (2);
 * per tensor t at [32 + 4 t]: n, k, chunks, steps.
 * ---------------------------------------------------------------------------------------------------- */
int64_t grad_topk_plan(const int64_t *offsets, const int32_t *k, int T, int chunks, int64_t *plan, int64_t plan_capacity);

/* Bytes of device workspace grad_topk_select needs for this plan (HOST pointer); 0 for a plan it does not accept. */
size_t grad_topk_workspace(const int64_t *plan_host);

/* ------------------------------------------------------------------------------------------------------
 * grad_topk_select -- Section 3.3.2: the selection itself, one launch per level of the plan for the whole group
 * (plain tree: first level one workgroup per chunk of a tensor, last level one workgroup that writes its output;
 * the three steps described above: thresholds, then all chunks in a launch of their own, then the final steps,
 * beside which the tensors of a single chunk run).
 *
 *   g          [offsets[T]]  the gradient tensors, fp32, back to back as planned (4-byte aligned is enough)
 *   plan_dev   the plan in device memory;  plan_host  HOST: the same words (launch geometry is read from it)
 *   out_idx    [sum k]  out: indices within the tensor; tensor t's part starts at sum(k[0..t))
 *   out_val    [sum k]  out: the signed values g[idx]
 * Returns KS_INVALID_ARG for NULL pointers or a plan that was not produced by grad_topk_plan,
 * KS_WORKSPACE_TOO_SMALL, KS_HIP_ERROR.
 * ---------------------------------------------------------------------------------------------------- */
int grad_topk_select(const float *g, const int64_t *plan_dev, const int64_t *plan_host, int32_t *out_idx, float *out_val,
                     void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif
