/*
 * CPU oracle for the layer-wise top-k selection of gradient sparsification (paper: Section 3.3, subsection
 * on efficient layer-wise top-k sparsification, and its figure "divide and conquer top-k selection").
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT: plain and slow, shares no code with the HIP library, called
 * only from tests, from the smoke check and from the benchmark's CPU-baseline leg.
 *
 * What is computed.  The paper's method is exact ("without any approximation"), so the result has a plain
 * definition, written out in orc_topk_abs: of a tensor g[0..n), the k elements of largest magnitude.
 * orc_topk_dc states the paper's two steps (top-k of each of M chunks, then top-k of the M*k survivors) on top
 * of that definition; tests pin that both give the same answer for every M.
 *
 * Readings taken where the paper is silent:
 *   - "top-k" of a gradient tensor is by magnitude (deep gradient compression, which the paper builds on,
 *     keeps the largest |g|);
 *   - magnitudes are compared as the 31-bit patterns of |g| (for finite values and infinities this is the
 *     numeric order; NaN patterns rank above infinity; +0 and -0 are equal);
 *   - among equal magnitudes the lowest index wins; the selection is emitted in descending magnitude, equal
 *     magnitudes in ascending index, so the result is unique;
 *   - the chunks of the two-step method are M consecutive ranges of ceil(n / M) elements (the last one
 *     shorter); a chunk shorter than k contributes all of its elements.
 * Pins (tests/test_oracle_pins.py): a stable library argsort of -|g|, closed forms (alternating ramp,
 * constant tensor, signed zeros), brute-force repeated maximum on tiny inputs, equality of the two-step
 * method with the definition for all M, k = n (a full sort).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_BAD_ARG 1

typedef struct {
    uint32_t mag; /* bit pattern of |g| */
    int32_t idx;
} orc_item;

static uint32_t magnitude_bits(float v) {
    uint32_t u;
    memcpy(&u, &v, 4);
    return u & 0x7FFFFFFFu;
}

/* larger magnitude first; equal magnitudes: lower index first */
static int cmp_item(const void *a, const void *b) {
    const orc_item *x = (const orc_item *)a, *y = (const orc_item *)b;
    if (x->mag != y->mag) return x->mag > y->mag ? -1 : 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

/* The definition: sort all (|g_i|, i) and keep the first k.  out_idx [k], out_val [k] (the signed values). */
int orc_topk_abs(const float *g, int64_t n, int k, int32_t *out_idx, float *out_val) {
    if (!g || n < 1 || n > INT32_MAX || k < 1 || k > n || !out_idx || !out_val) return ORC_BAD_ARG;
    orc_item *it = (orc_item *)malloc((size_t)n * sizeof(orc_item));
    if (!it) return ORC_BAD_ARG;
    for (int64_t i = 0; i < n; ++i) {
        it[i].mag = magnitude_bits(g[i]);
        it[i].idx = (int32_t)i;
    }
    qsort(it, (size_t)n, sizeof(orc_item), cmp_item);
    for (int r = 0; r < k; ++r) {
        out_idx[r] = it[r].idx;
        out_val[r] = g[it[r].idx];
    }
    free(it);
    return ORC_OK;
}

/* The paper's two steps.  Step 1: the tensor is cut into M chunks and the top-k of every chunk is taken (all
 * of a chunk that has fewer than k elements).  Step 2: the top-k of the survivors. */
int orc_topk_dc(const float *g, int64_t n, int k, int M, int32_t *out_idx, float *out_val) {
    if (!g || n < 1 || n > INT32_MAX || k < 1 || k > n || M < 1 || M > n || !out_idx || !out_val) return ORC_BAD_ARG;
    const int64_t len = (n + M - 1) / M;
    orc_item *surv = (orc_item *)malloc((size_t)M * (size_t)k * sizeof(orc_item));
    orc_item *it = (orc_item *)malloc((size_t)len * sizeof(orc_item));
    if (!surv || !it) {
        free(surv);
        free(it);
        return ORC_BAD_ARG;
    }
    int64_t n_surv = 0;
    for (int m = 0; m < M; ++m) {
        const int64_t a = (int64_t)m * len, b = a + len < n ? a + len : n;
        if (a >= b) break;
        for (int64_t i = a; i < b; ++i) {
            it[i - a].mag = magnitude_bits(g[i]);
            it[i - a].idx = (int32_t)i;
        }
        qsort(it, (size_t)(b - a), sizeof(orc_item), cmp_item);
        const int64_t keep = b - a < k ? b - a : k;
        memcpy(surv + n_surv, it, (size_t)keep * sizeof(orc_item));
        n_surv += keep;
    }
    qsort(surv, (size_t)n_surv, sizeof(orc_item), cmp_item);
    for (int r = 0; r < k; ++r) {
        out_idx[r] = surv[r].idx;
        out_val[r] = g[surv[r].idx];
    }
    free(surv);
    free(it);
    return ORC_OK;
}

/* A group of tensors stored back to back (layer-wise selection: every tensor has its own k): tensor t is
 * g[offsets[t] .. offsets[t+1]), its selection goes to out[out_offsets[t] .. +k[t]) with out_offsets the
 * running sum of k.  M[t] == 0 selects the definition, otherwise the two-step method with M[t] chunks. */
int orc_topk_group(const float *g, const int64_t *offsets, const int32_t *k, const int32_t *M, int T, int32_t *out_idx,
                   float *out_val) {
    if (!g || !offsets || !k || T < 1 || !out_idx || !out_val) return ORC_BAD_ARG;
    int64_t *oo = (int64_t *)malloc((size_t)(T + 1) * sizeof(int64_t));
    if (!oo) return ORC_BAD_ARG;
    oo[0] = 0;
    for (int t = 0; t < T; ++t) oo[t + 1] = oo[t] + k[t];
    int rc = ORC_OK;
#pragma omp parallel for schedule(dynamic, 1)
    for (int t = 0; t < T; ++t) {
        const int64_t n = offsets[t + 1] - offsets[t];
        const int r = (M && M[t] > 0) ? orc_topk_dc(g + offsets[t], n, k[t], M[t], out_idx + oo[t], out_val + oo[t])
                                      : orc_topk_abs(g + offsets[t], n, k[t], out_idx + oo[t], out_val + oo[t]);
        if (r != ORC_OK) {
#pragma omp critical
            rc = r;
        }
    }
    free(oo);
    return rc;
}
