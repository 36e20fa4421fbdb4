/*
 * CPU oracle for the KNN-softmax output layer (paper: "Large-Scale Training System for 100-Million
 * Classification at Alibaba", Section 3.2 "KNN Softmax", Algorithm 1, Section 3.1 steps 3-6).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, obviously-correct statement of
 * what the GPU path must compute: fp32 storage of inputs, every accumulation in fp64, no blocking, no
 * fusion, no BLAS.  It shares no code with the HIP library and is only called from tests, from the
 * smoke check and from the benchmark's CPU-baseline leg.
 *
 * Every function below is pinned by tests that do not go through this file's own formulas
 * (full-softmax equality when K spans all classes, a library cross-entropy in fp64, closed forms,
 * finite differences, set-based selection, argsort-based neighbour search, dense index_add).
 *
 * Readings taken where the paper is silent (each is also listed in the design notes):
 *   - logits are scale * <x, w> with the scale given by the caller; no margin;
 *   - X and W are used as given (callers pass L2-normalised rows); gradients are w.r.t. the given rows;
 *   - neighbour lists hold K classes other than the class itself; selection always adds the label
 *     itself with rank 0 (same set as the paper's lists, in which the class itself is ranked first);
 *   - "ranking score" used to cut the set down to M = best (smallest) position of the class in any
 *     contributing list, ties to the lowest class id; the active list is emitted in ascending id;
 *   - similarity for ranking neighbours = sum over d ascending of (double)w_id * (double)w_jd;
 *     ties go to the lowest class id; lists are in descending similarity;
 *   - loss is the mean over the batch; grad_scale multiplies gradients only;
 *   - the weight update is W[c] += alpha * (sum of the gradient rows addressed to c).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <limits.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_BAD_ARG 1
#define ORC_BAD_LABEL 2
#define ORC_BAD_GRAPH_ID 3

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------------------------------------
 * Section 3.2.2 (graph building by linear search): similarity of two weight rows is their inner
 * product.  Canonical arithmetic: fp64, one term at a time, d ascending.
 * ------------------------------------------------------------------------------------------- */
static double row_similarity(const float *wi, const float *wj, int D) {
    double acc = 0.0;
    for (int d = 0; d < D; ++d) acc += (double)wi[d] * (double)wj[d];
    return acc;
}

/* is candidate (s, j) ranked before (t, k)?  higher similarity first, then lower class id */
static int ranks_before(double s, int32_t j, double t, int32_t k) {
    if (s > t) return 1;
    if (s < t) return 0;
    return j < k;
}

/*
 * Brute-force K nearest neighbours (Section 3.2.2: "linear search", exact) of the rows listed in
 * `rows` (or of every row when rows == NULL) among all C rows of W, the row itself excluded.
 * graph_out [n_rows, K] int32, sims_out [n_rows, K] fp64 (may be NULL), both in rank order.
 */
int orc_graph_bruteforce(const float *W, int64_t C, int D, int K, const int32_t *rows, int64_t n_rows,
                         int32_t *graph_out, double *sims_out) {
    if (!W || !graph_out || C < 2 || D < 1 || K < 1 || K > C - 1) return ORC_BAD_ARG;
    if (!rows) n_rows = C;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 4) reduction(| : bad)
    for (int64_t r = 0; r < n_rows; ++r) {
        int64_t i = rows ? rows[r] : r;
        if (i < 0 || i >= C) { bad = 1; continue; }
        double *best_s = (double *)malloc(sizeof(double) * (size_t)K);
        int32_t *best_j = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
        int n = 0;
        for (int64_t j = 0; j < C; ++j) {
            if (j == i) continue;
            double s = row_similarity(W + i * D, W + j * D, D);
            if (n == K && !ranks_before(s, (int32_t)j, best_s[K - 1], best_j[K - 1])) continue;
            /* insert into the sorted list of the best so far */
            int pos = (n < K) ? n : K - 1;
            while (pos > 0 && ranks_before(s, (int32_t)j, best_s[pos - 1], best_j[pos - 1])) {
                best_s[pos] = best_s[pos - 1];
                best_j[pos] = best_j[pos - 1];
                --pos;
            }
            best_s[pos] = s;
            best_j[pos] = (int32_t)j;
            if (n < K) ++n;
        }
        for (int k = 0; k < K; ++k) {
            graph_out[r * K + k] = best_j[k];
            if (sims_out) sims_out[r * K + k] = best_s[k];
        }
        free(best_s);
        free(best_j);
    }
    return bad ? ORC_BAD_ARG : ORC_OK;
}

/*
 * One hop of the distributed graph build (Section 3.2.2: the weight shards travel from node to node, every
 * node searches each visiting shard and keeps its rows' best K so far).  The node owns C_loc rows W_local whose
 * ids in the whole problem start at local_offset; W_visit holds C_vis rows with ids from visit_offset.
 * graph [C_loc, K] / sims [C_loc, K] are the lists so far (ids of the whole problem in rank order, -1 = empty
 * slot, sims = canonical fp64 similarities) and are updated in place to the best K of (list so far) U (visiting
 * rows), the row itself excluded, a visiting row already in the list ignored.  Empty slots get -1 / -infinity.
 */
typedef struct { double s; int32_t id; } sim_id;
static int cmp_sim_id(const void *a, const void *b) {
    const sim_id *x = (const sim_id *)a, *y = (const sim_id *)b;
    if (ranks_before(x->s, x->id, y->s, y->id)) return -1;
    if (ranks_before(y->s, y->id, x->s, x->id)) return 1;
    return 0;
}
int orc_graph_update(const float *W_local, int64_t C_loc, const float *W_visit, int64_t C_vis, int D, int K,
                     int64_t local_offset, int64_t visit_offset, int32_t *graph, double *sims) {
    if (!W_local || !W_visit || !graph || !sims || C_loc < 1 || C_vis < 1 || D < 1 || K < 1) return ORC_BAD_ARG;
    if (local_offset < 0 || visit_offset < 0 || local_offset + C_loc > INT32_MAX || visit_offset + C_vis > INT32_MAX)
        return ORC_BAD_ARG;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < C_loc; ++i) {
        sim_id *u = (sim_id *)malloc(sizeof(sim_id) * (size_t)(C_vis + K));
        int64_t n = 0;
        for (int k = 0; k < K; ++k)
            if (graph[i * K + k] >= 0) { u[n].s = sims[i * K + k]; u[n].id = graph[i * K + k]; ++n; }
        const int64_t n_old = n;
        for (int64_t j = 0; j < C_vis; ++j) {
            const int64_t id = visit_offset + j;
            if (id == local_offset + i) continue;
            int known = 0;
            for (int64_t e = 0; e < n_old; ++e) known |= (u[e].id == id);
            if (known) continue;
            u[n].s = row_similarity(W_local + i * D, W_visit + j * D, D);
            u[n].id = (int32_t)id;
            ++n;
        }
        qsort(u, (size_t)n, sizeof(sim_id), cmp_sim_id);
        for (int k = 0; k < K; ++k) {
            graph[i * K + k] = k < n ? u[k].id : -1;
            sims[i * K + k] = k < n ? u[k].s : -INFINITY;
        }
        free(u);
    }
    return ORC_OK;
}

/* ---------------------------------------------------------------------------------------------
 * Algorithm 1 (KNN graph-based active classes selection), without the random fill-up branch:
 * the union of the labels' neighbour lists (each list headed by the label itself), duplicates
 * removed; when more than M classes remain, the M with the best ranking score are kept.
 *   active [M]   ascending class ids, first *n_active valid, the rest set to -1
 *   target_pos[B] position of label i inside active
 * Graph entries equal to -1 are empty slots.
 * ------------------------------------------------------------------------------------------- */
typedef struct { int32_t score; int32_t cls; } scored_class;

static int cmp_scored(const void *a, const void *b) {
    const scored_class *x = (const scored_class *)a, *y = (const scored_class *)b;
    if (x->score != y->score) return x->score < y->score ? -1 : 1;
    return (x->cls > y->cls) - (x->cls < y->cls);
}
static int cmp_i32(const void *a, const void *b) {
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

int orc_select_active(const int32_t *labels, int B, const int32_t *G, int64_t C, int K, int M,
                      int32_t *active, int32_t *n_active, int32_t *target_pos) {
    if (!labels || !G || !active || !n_active || !target_pos) return ORC_BAD_ARG;
    if (B < 1 || C < 1 || K < 0 || M < 1 || B > M || K + 1 > M) return ORC_BAD_ARG;
    int32_t *score = (int32_t *)malloc(sizeof(int32_t) * (size_t)C);
    for (int64_t c = 0; c < C; ++c) score[c] = INT32_MAX; /* INT32_MAX = not a candidate */
    int rc = ORC_OK;
    for (int i = 0; i < B && rc == ORC_OK; ++i) {
        int32_t y = labels[i];
        if (y < 0 || y >= C) { rc = ORC_BAD_LABEL; break; }
        score[y] = 0; /* the class itself heads its own list */
        for (int k = 0; k < K; ++k) {
            int32_t c = G[(int64_t)y * K + k];
            if (c == -1) continue;
            if (c < -1 || c >= C) { rc = ORC_BAD_GRAPH_ID; break; }
            if (k + 1 < score[c]) score[c] = k + 1;
        }
    }
    if (rc != ORC_OK) { free(score); return rc; }
    int64_t n_unique = 0;
    for (int64_t c = 0; c < C; ++c) n_unique += (score[c] != INT32_MAX);
    scored_class *u = (scored_class *)malloc(sizeof(scored_class) * (size_t)(n_unique ? n_unique : 1));
    int64_t n = 0;
    for (int64_t c = 0; c < C; ++c)
        if (score[c] != INT32_MAX) { u[n].score = score[c]; u[n].cls = (int32_t)c; ++n; }
    int64_t A = n_unique;
    if (n_unique > M) { /* keep the M best-scored classes */
        qsort(u, (size_t)n_unique, sizeof(scored_class), cmp_scored);
        A = M;
    }
    for (int64_t a = 0; a < A; ++a) active[a] = u[a].cls;
    qsort(active, (size_t)A, sizeof(int32_t), cmp_i32);
    for (int64_t a = A; a < M; ++a) active[a] = -1;
    *n_active = (int32_t)A;
    for (int i = 0; i < B; ++i) {
        target_pos[i] = -1;
        for (int64_t a = 0; a < A; ++a)
            if (active[a] == labels[i]) { target_pos[i] = (int32_t)a; break; }
        if (target_pos[i] < 0) rc = ORC_BAD_ARG; /* cannot happen when B <= M */
    }
    free(u);
    free(score);
    return rc;
}

/* ---------------------------------------------------------------------------------------------
 * Compressed graph of one node (Section 3.2.3): the node that owns the classes [c0, c0 + C_loc) keeps, for every
 * class g of the whole problem, only those neighbours of g that it owns, in the order of g's list, as ids local to
 * the node; the lists, now of different lengths, are laid end to end (flat) with counts[g] entries starting at
 * offsets[g] (offsets = running sum of the counts, offsets[Cg] = total).  Entries -1 of the dense graph are empty
 * slots.  flat may be NULL (counts and offsets only).
 * ------------------------------------------------------------------------------------------- */
int orc_graph_compress(const int32_t *G, int64_t Cg, int K, int64_t c0, int64_t C_loc, int32_t *counts,
                       int64_t *offsets, int32_t *flat) {
    if (!G || !counts || !offsets || Cg < 1 || K < 0 || c0 < 0 || C_loc < 1 || c0 + C_loc > Cg) return ORC_BAD_ARG;
    int64_t run = 0;
    for (int64_t g = 0; g < Cg; ++g) {
        offsets[g] = run;
        int32_t n = 0;
        for (int k = 0; k < K; ++k) {
            const int32_t c = G[g * K + k];
            if (c == -1) continue;
            if (c < -1 || c >= Cg) return ORC_BAD_GRAPH_ID;
            if (c >= c0 && c < c0 + C_loc) {
                if (flat) flat[run + n] = (int32_t)(c - c0);
                ++n;
            }
        }
        counts[g] = n;
        run += n;
    }
    offsets[Cg] = run;
    return ORC_OK;
}

/* The order in which classes are drawn for the random fill-up of Algorithm 1: the k-th draw, k = 0, 1, ..., is
 * class pad_draw(k) where pad_draw is a keyed one-to-one map of [0, 2^b) onto itself, 2^b the smallest power of
 * two >= C_loc (every step below is one-to-one on b-bit numbers: adding a constant, multiplying by an odd
 * constant, xor with a right shift of itself).  Draws >= C_loc or already in the set are passed over, so the
 * fill-up is a sample without replacement of the classes not chosen.  The paper only says "random sample"; the
 * map is this build's choice, implemented on both sides from this description. */
static int pad_bits(int64_t C_loc) {
    int b = 1;
    while (((int64_t)1 << b) < C_loc) ++b;
    return b;
}
static uint32_t pad_draw(uint32_t k, int b, uint64_t seed) {
    const uint32_t mask = b >= 32 ? 0xFFFFFFFFu : (((uint32_t)1 << b) - 1u);
    const int s1 = (b + 1) / 2, s2 = b / 3 > 0 ? b / 3 : 1;
    uint32_t x = (k + (uint32_t)seed) & mask;
    x = (x * 0x9E3779B1u) & mask;
    x ^= x >> s1;
    x = (x * 0x85EBCA6Bu) & mask;
    x ^= x >> s2;
    x = (x * 0xC2B2AE35u) & mask;
    x ^= x >> s1;
    x = (x + (uint32_t)(seed >> 32)) & mask;
    return x;
}
int orc_pad_draws(int64_t C_loc, uint64_t seed, int64_t n, uint32_t *out) { /* the first n draws, for tests */
    if (C_loc < 1 || C_loc > ((int64_t)1 << 31) || !out) return ORC_BAD_ARG;
    const int b = pad_bits(C_loc);
    for (int64_t k = 0; k < n; ++k) out[k] = pad_draw((uint32_t)k, b, seed);
    return ORC_OK;
}

/* Algorithm 1 on a node of the sharded layer: labels are ids of the whole problem, the neighbour lists come from
 * the node's compressed graph, the result holds ids local to the node.
 *   - sample i contributes its own class at list position 0 if the node owns it, and entry j of the compressed
 *     list of its class at position j + 1; a class's score is its smallest position; duplicates are removed;
 *   - more than M classes found: the M best scores are kept, ties to the lowest local id;
 *   - fewer than M found and pad != 0: filled up to min(M, C_loc) by the draws of pad_draw (see above);
 *   - active: ascending local ids, -1 beyond n_active; n_found = classes found before the fill-up (capped at M);
 *   - target_pos[i] = position of sample i's class in the active list, -1 if another node owns the class. */
int orc_select_active_csr(const int32_t *labels, int B, const int32_t *counts, const int64_t *offsets,
                          const int32_t *flat, int64_t Cg, int64_t c0, int64_t C_loc, int M, int pad, uint64_t seed,
                          int32_t *active, int32_t *n_active, int32_t *n_found, int32_t *target_pos) {
    if (!labels || !counts || !offsets || !active || !n_active || !target_pos) return ORC_BAD_ARG;
    if (B < 1 || Cg < 1 || c0 < 0 || C_loc < 1 || c0 + C_loc > Cg || M < 1 || B > M) return ORC_BAD_ARG;
    int32_t *score = (int32_t *)malloc(sizeof(int32_t) * (size_t)C_loc);
    for (int64_t c = 0; c < C_loc; ++c) score[c] = INT32_MAX;
    for (int i = 0; i < B; ++i) {
        const int32_t y = labels[i];
        if (y < 0 || y >= Cg) { free(score); return ORC_BAD_LABEL; }
        if (y >= c0 && y < c0 + C_loc) score[y - c0] = 0;
        if (counts[y] < 0 || counts[y] + 1 > M) { free(score); return ORC_BAD_ARG; }
        for (int32_t j = 0; j < counts[y]; ++j) {
            const int32_t c = flat[offsets[y] + j];
            if (c == -1) continue;
            if (c < -1 || c >= C_loc) { free(score); return ORC_BAD_GRAPH_ID; }
            if (j + 1 < score[c]) score[c] = j + 1;
        }
    }
    int64_t n_unique = 0;
    for (int64_t c = 0; c < C_loc; ++c) n_unique += (score[c] != INT32_MAX);
    scored_class *u = (scored_class *)malloc(sizeof(scored_class) * (size_t)(n_unique ? n_unique : 1));
    int64_t n = 0;
    for (int64_t c = 0; c < C_loc; ++c)
        if (score[c] != INT32_MAX) { u[n].score = score[c]; u[n].cls = (int32_t)c; ++n; }
    int64_t A = n_unique;
    if (n_unique > M) {
        qsort(u, (size_t)n_unique, sizeof(scored_class), cmp_scored);
        A = M;
    }
    for (int64_t a = 0; a < A; ++a) active[a] = u[a].cls;
    if (n_found) *n_found = (int32_t)A;
    if (pad && A < M) {
        const int64_t want = M < C_loc ? M : C_loc;
        const int b = pad_bits(C_loc);
        for (uint64_t k = 0; A < want && k < ((uint64_t)1 << b); ++k) {
            const uint32_t c = pad_draw((uint32_t)k, b, seed);
            if ((int64_t)c >= C_loc || score[c] != INT32_MAX) continue;
            score[c] = INT32_MAX - 1; /* drawn */
            active[A++] = (int32_t)c;
        }
    }
    qsort(active, (size_t)A, sizeof(int32_t), cmp_i32);
    for (int64_t a = A; a < M; ++a) active[a] = -1;
    *n_active = (int32_t)A;
    for (int i = 0; i < B; ++i) {
        target_pos[i] = -1;
        const int64_t y = (int64_t)labels[i] - c0;
        if (y < 0 || y >= C_loc) continue;
        for (int64_t a = 0; a < A; ++a)
            if (active[a] == y) { target_pos[i] = (int32_t)a; break; }
    }
    free(u);
    free(score);
    return ORC_OK;
}

/* ---------------------------------------------------------------------------------------------
 * Softmax stage on the active classes (Section 3.2: fc forward, softmax forward, softmax backward,
 * fc backward; standard softmax with cross-entropy restricted to the selected columns).
 *   Z_ia   = scale * sum_d X_id * W[active[a], d]
 *   lse_i  = max_a Z_ia + log sum_a exp(Z_ia - max)
 *   loss_i = lse_i - Z_{i, target_pos[i]},  loss = mean_i loss_i
 *   P_ia   = exp(Z_ia - lse_i),  dZ_ia = (grad_scale / B) * (P_ia - [a == target_pos[i]])
 *   dX_id  = scale * sum_a dZ_ia * W[active[a], d]
 *   dWA_ad = scale * sum_i dZ_ia * X_id
 * Outputs are fp64.  P_out [B, A] and lse_out [B] are optional (NULL to skip).
 * ------------------------------------------------------------------------------------------- */
int orc_knn_softmax_fwd_bwd(const float *W, const float *X, const int32_t *active, int A,
                            const int32_t *target_pos, int B, int D, double scale, double grad_scale,
                            double *loss_i, double *loss_mean, double *dX, double *dWA,
                            double *P_out, double *lse_out) {
    if (!W || !X || !active || !target_pos || !loss_i || !loss_mean || !dX || !dWA) return ORC_BAD_ARG;
    if (A < 1 || B < 1 || D < 1) return ORC_BAD_ARG;
    double *dZ = (double *)malloc(sizeof(double) * (size_t)B * (size_t)A);
    if (!dZ) return ORC_BAD_ARG;
    const double g = grad_scale / (double)B;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < B; ++i) {
        double *z = dZ + (size_t)i * A; /* holds Z_i first, then dZ_i */
        for (int a = 0; a < A; ++a) {
            const float *w = W + (int64_t)active[a] * D;
            double acc = 0.0;
            for (int d = 0; d < D; ++d) acc += (double)X[(size_t)i * D + d] * (double)w[d];
            z[a] = scale * acc;
        }
        double m = z[0];
        for (int a = 1; a < A; ++a) if (z[a] > m) m = z[a];
        double sum = 0.0;
        for (int a = 0; a < A; ++a) sum += exp(z[a] - m);
        double lse = m + log(sum);
        loss_i[i] = lse - z[target_pos[i]];
        if (lse_out) lse_out[i] = lse;
        for (int a = 0; a < A; ++a) {
            double p = exp(z[a] - lse);
            if (P_out) P_out[(size_t)i * A + a] = p;
            z[a] = g * (p - (a == target_pos[i] ? 1.0 : 0.0));
        }
    }
    double tot = 0.0;
    for (int i = 0; i < B; ++i) tot += loss_i[i];
    *loss_mean = tot / (double)B;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < B; ++i) {
        double *out = dX + (size_t)i * D;
        for (int d = 0; d < D; ++d) out[d] = 0.0;
        for (int a = 0; a < A; ++a) {
            const float *w = W + (int64_t)active[a] * D;
            double dz = dZ[(size_t)i * A + a];
            for (int d = 0; d < D; ++d) out[d] += dz * (double)w[d];
        }
        for (int d = 0; d < D; ++d) out[d] *= scale;
    }
#pragma omp parallel for schedule(static)
    for (int a = 0; a < A; ++a) {
        double *out = dWA + (size_t)a * D;
        for (int d = 0; d < D; ++d) out[d] = 0.0;
        for (int i = 0; i < B; ++i) {
            double dz = dZ[(size_t)i * A + a];
            for (int d = 0; d < D; ++d) out[d] += dz * (double)X[(size_t)i * D + d];
        }
        for (int d = 0; d < D; ++d) out[d] *= scale;
    }
    free(dZ);
    return ORC_OK;
}

/* ---------------------------------------------------------------------------------------------
 * The softmax of the model-parallel layer, one node's part (Section 3.1, steps 3-5: every node holds the logits
 * of its own classes; the softmax needs each sample's maximum and sum of exponentials over ALL nodes, which the
 * nodes exchange; then every node forms the gradient of its own logits).
 *
 * orc_softmax_node_stats: for the node's active columns, per sample
 *     m_i = max_a Z_ia,   l_i = sum_a exp(Z_ia - m_i),   t_i = Z_{i, target_pos[i]}  (0 if target_pos[i] < 0:
 *     another node owns the sample's class).
 * Combining nodes p:  M_i = max_p m_i^p,  S_i = sum_p l_i^p exp(m_i^p - M_i),  T_i = sum_p t_i^p.
 * orc_softmax_node_bwd: with the combined (M, S, T):
 *     loss_i = M_i + log S_i - T_i,   dZ_ia = (grad_scale / B) (exp(Z_ia - M_i) / S_i - [a == target_pos[i]]),
 *     dX (this node's contribution, to be summed over the nodes) and dWA as in orc_knn_softmax_fwd_bwd.
 * ------------------------------------------------------------------------------------------- */
int orc_softmax_node_stats(const float *W, const float *X, const int32_t *active, int A, const int32_t *target_pos, int B,
                           int D, double scale, double *m_out, double *l_out, double *t_out) {
    if (!W || !X || !active || !target_pos || !m_out || !l_out || !t_out || A < 1 || B < 1 || D < 1) return ORC_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < B; ++i) {
        double *z = (double *)malloc(sizeof(double) * (size_t)A);
        for (int a = 0; a < A; ++a) {
            const float *w = W + (int64_t)active[a] * D;
            double acc = 0.0;
            for (int d = 0; d < D; ++d) acc += (double)X[(size_t)i * D + d] * (double)w[d];
            z[a] = scale * acc;
        }
        double m = z[0];
        for (int a = 1; a < A; ++a) if (z[a] > m) m = z[a];
        double l = 0.0;
        for (int a = 0; a < A; ++a) l += exp(z[a] - m);
        m_out[i] = m;
        l_out[i] = l;
        t_out[i] = (target_pos[i] >= 0 && target_pos[i] < A) ? z[target_pos[i]] : 0.0;
        free(z);
    }
    return ORC_OK;
}

int orc_softmax_node_bwd(const float *W, const float *X, const int32_t *active, int A, const int32_t *target_pos, int B,
                         int D, double scale, double grad_scale, const double *Mg, const double *Sg, const double *Tg,
                         double *loss_i, double *loss_mean, double *dX, double *dWA) {
    if (!W || !X || !active || !target_pos || !Mg || !Sg || !Tg || !loss_i || !loss_mean || !dX || !dWA) return ORC_BAD_ARG;
    if (A < 1 || B < 1 || D < 1) return ORC_BAD_ARG;
    double *dZ = (double *)malloc(sizeof(double) * (size_t)B * (size_t)A);
    if (!dZ) return ORC_BAD_ARG;
    const double g = grad_scale / (double)B;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < B; ++i) {
        double *z = dZ + (size_t)i * A;
        for (int a = 0; a < A; ++a) {
            const float *w = W + (int64_t)active[a] * D;
            double acc = 0.0;
            for (int d = 0; d < D; ++d) acc += (double)X[(size_t)i * D + d] * (double)w[d];
            z[a] = scale * acc;
        }
        loss_i[i] = Mg[i] + log(Sg[i]) - Tg[i];
        for (int a = 0; a < A; ++a) z[a] = g * (exp(z[a] - Mg[i]) / Sg[i] - (a == target_pos[i] ? 1.0 : 0.0));
    }
    double tot = 0.0;
    for (int i = 0; i < B; ++i) tot += loss_i[i];
    *loss_mean = tot / (double)B;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < B; ++i) {
        double *out = dX + (size_t)i * D;
        for (int d = 0; d < D; ++d) out[d] = 0.0;
        for (int a = 0; a < A; ++a) {
            const float *w = W + (int64_t)active[a] * D;
            const double dz = dZ[(size_t)i * A + a];
            for (int d = 0; d < D; ++d) out[d] += dz * (double)w[d];
        }
        for (int d = 0; d < D; ++d) out[d] *= scale;
    }
#pragma omp parallel for schedule(static)
    for (int a = 0; a < A; ++a) {
        double *out = dWA + (size_t)a * D;
        for (int d = 0; d < D; ++d) out[d] = 0.0;
        for (int i = 0; i < B; ++i) {
            const double dz = dZ[(size_t)i * A + a];
            for (int d = 0; d < D; ++d) out[d] += dz * (double)X[(size_t)i * D + d];
        }
        for (int d = 0; d < D; ++d) out[d] *= scale;
    }
    free(dZ);
    return ORC_OK;
}

/*
 * Full softmax over all C classes (the baseline the paper compares against; Section 3.2 claims the
 * KNN variant equals it on the selected columns).  Written separately from the function above on
 * purpose: dense columns, label used directly, dense dW [C, D].
 */
int orc_full_softmax_fwd_bwd(const float *W, const float *X, const int32_t *labels, int64_t C, int B, int D,
                             double scale, double grad_scale, double *loss_i, double *loss_mean,
                             double *dX, double *dW) {
    if (!W || !X || !labels || !loss_i || !loss_mean || !dX || !dW) return ORC_BAD_ARG;
    double *P = (double *)malloc(sizeof(double) * (size_t)B * (size_t)C);
    if (!P) return ORC_BAD_ARG;
    const double g = grad_scale / (double)B;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < B; ++i) {
        double *z = P + (size_t)i * C;
        double m = -INFINITY;
        for (int64_t c = 0; c < C; ++c) {
            double acc = 0.0;
            for (int d = 0; d < D; ++d) acc += (double)X[(size_t)i * D + d] * (double)W[c * D + d];
            z[c] = scale * acc;
            if (z[c] > m) m = z[c];
        }
        double sum = 0.0;
        for (int64_t c = 0; c < C; ++c) sum += exp(z[c] - m);
        double lse = m + log(sum);
        loss_i[i] = lse - z[labels[i]];
        for (int64_t c = 0; c < C; ++c) z[c] = exp(z[c] - lse);
    }
    double tot = 0.0;
    for (int i = 0; i < B; ++i) tot += loss_i[i];
    *loss_mean = tot / (double)B;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < B; ++i) {
        for (int d = 0; d < D; ++d) {
            double acc = 0.0;
            for (int64_t c = 0; c < C; ++c) {
                double dz = g * (P[(size_t)i * C + c] - (c == labels[i] ? 1.0 : 0.0));
                acc += dz * (double)W[c * D + d];
            }
            dX[(size_t)i * D + d] = scale * acc;
        }
    }
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < C; ++c) {
        for (int d = 0; d < D; ++d) {
            double acc = 0.0;
            for (int i = 0; i < B; ++i) {
                double dz = g * (P[(size_t)i * C + c] - (c == labels[i] ? 1.0 : 0.0));
                acc += dz * (double)X[(size_t)i * D + d];
            }
            dW[c * D + d] = scale * acc;
        }
    }
    free(P);
    return ORC_OK;
}

/* ---------------------------------------------------------------------------------------------
 * Local weight update of the model-parallel fc layer (Section 3.1 step 6; fp32 copy of the
 * parameters is the one updated, the 16-bit copy is refreshed from it):
 *   for every class c named in idx: Wm[c,:] += alpha * sum_{p: idx[p]==c} dW[p,:]
 * the sum taken in ascending p in fp64, the result stored as fp32; then Wb[c,:] = bf16(Wm[c,:])
 * by round-to-nearest-even.  Rows not named in idx are not touched.
 * ------------------------------------------------------------------------------------------- */
static uint16_t f32_to_bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u); /* NaN stays NaN */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

int orc_apply_weight_grad(float *Wm, uint16_t *Wb, const int32_t *idx, int n, const float *dW, double alpha,
                          int64_t C, int D) {
    if (!Wm || !idx || !dW || n < 0 || D < 1) return ORC_BAD_ARG;
    for (int p = 0; p < n; ++p) if (idx[p] < 0 || idx[p] >= C) return ORC_BAD_LABEL;
    int32_t *slot = (int32_t *)malloc(sizeof(int32_t) * (size_t)C);
    for (int64_t c = 0; c < C; ++c) slot[c] = -1;
    int n_distinct = 0;
    for (int p = 0; p < n; ++p) if (slot[idx[p]] < 0) slot[idx[p]] = n_distinct++;
    double *sum = (double *)calloc((size_t)(n_distinct ? n_distinct : 1) * (size_t)D, sizeof(double));
    for (int p = 0; p < n; ++p) { /* ascending p */
        double *s = sum + (size_t)slot[idx[p]] * D;
        for (int d = 0; d < D; ++d) s[d] += (double)dW[(size_t)p * D + d];
    }
    for (int p = 0; p < n; ++p) {
        int32_t c = idx[p];
        if (slot[c] < 0) continue; /* already applied */
        const double *s = sum + (size_t)slot[c] * D;
        for (int d = 0; d < D; ++d) {
            float w = (float)((double)Wm[(int64_t)c * D + d] + alpha * s[d]);
            Wm[(int64_t)c * D + d] = w;
            if (Wb) Wb[(int64_t)c * D + d] = f32_to_bf16_rne(w);
        }
        slot[c] = -1;
    }
    free(sum);
    free(slot);
    return ORC_OK;
}

/* ---------------------------------------------------------------------------------------------
 * Normalisation of the rows of W and X inside the layer (Section 3.2.3: the GPU pipeline normalises
 * W and X; Section 3.2: "normalization strategy").  With v_hat = v / |v| the layer works on the
 * normalised rows; a gradient g with respect to v_hat becomes, with respect to v,
 *     dv = (g - v_hat <v_hat, g>) / |v|                (the Jacobian of v -> v / |v| is symmetric).
 * A zero row stays zero and receives a zero gradient.
 * ------------------------------------------------------------------------------------------- */
int orc_normalize_rows(const float *V, int64_t n, int D, float *V_hat, uint16_t *V_hat_bf16, float *inv_norm) {
    if (!V || n < 0 || D < 1) return ORC_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const float *v = V + i * D;
        double s = 0.0;
        for (int d = 0; d < D; ++d) s += (double)v[d] * (double)v[d];
        const double inv = s > 0.0 ? 1.0 / sqrt(s) : 0.0;
        if (inv_norm) inv_norm[i] = (float)inv;
        for (int d = 0; d < D; ++d) {
            const float h = (float)((double)v[d] * inv);
            if (V_hat) V_hat[i * D + d] = h;
            if (V_hat_bf16) V_hat_bf16[i * D + d] = f32_to_bf16_rne(h);
        }
    }
    return ORC_OK;
}

int orc_norm_backward(const float *V, const double *G, int64_t n, int D, double *dV) {
    if (!V || !G || !dV || n < 0 || D < 1) return ORC_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const float *v = V + i * D;
        const double *g = G + i * D;
        double s = 0.0;
        for (int d = 0; d < D; ++d) s += (double)v[d] * (double)v[d];
        if (!(s > 0.0)) {
            for (int d = 0; d < D; ++d) dV[i * D + d] = 0.0;
            continue;
        }
        const double inv = 1.0 / sqrt(s);
        double dot = 0.0; /* <v_hat, g> */
        for (int d = 0; d < D; ++d) dot += (double)v[d] * inv * g[d];
        for (int d = 0; d < D; ++d) dV[i * D + d] = (g[d] - (double)v[d] * inv * dot) * inv;
    }
    return ORC_OK;
}

/* Weight update of the layer that keeps W un-normalised in fp32 and works on its normalised 16-bit copy
 * (Section 3.1 step 6 with the normalisation of Section 3.2.3 folded in).  dW_hat[p,:] is the gradient
 * with respect to the NORMALISED row of class idx[p].  For every class c that occurs in idx:
 *     g = sum of its rows of dW_hat (ascending p, fp64);  dw = (g - w_hat <w_hat, g>) / |w|  with the
 *     current master row;  W[c,:] += alpha * dw (stored fp32);  then, from the stored row,
 *     inv_norm[c] = 1 / |W[c,:]|  and  W_hat_bf16[c,:] = bf16(fp32(W[c,:] * inv_norm)).
 * Rows not named in idx are not touched. */
int orc_apply_weight_grad_normalized(float *Wm, uint16_t *W_hat_bf16, float *inv_norm, const int32_t *idx, int n,
                                     const float *dW_hat, double alpha, int64_t C, int D) {
    if (!Wm || !idx || !dW_hat || n < 0 || D < 1) return ORC_BAD_ARG;
    for (int p = 0; p < n; ++p) if (idx[p] < 0 || idx[p] >= C) return ORC_BAD_LABEL;
    int32_t *slot = (int32_t *)malloc(sizeof(int32_t) * (size_t)C);
    for (int64_t c = 0; c < C; ++c) slot[c] = -1;
    int n_distinct = 0;
    for (int p = 0; p < n; ++p) if (slot[idx[p]] < 0) slot[idx[p]] = n_distinct++;
    double *sum = (double *)calloc((size_t)(n_distinct ? n_distinct : 1) * (size_t)D, sizeof(double));
    for (int p = 0; p < n; ++p) { /* ascending p */
        double *s = sum + (size_t)slot[idx[p]] * D;
        for (int d = 0; d < D; ++d) s[d] += (double)dW_hat[(size_t)p * D + d];
    }
    for (int p = 0; p < n; ++p) {
        const int32_t c = idx[p];
        if (slot[c] < 0) continue; /* already applied */
        const double *g = sum + (size_t)slot[c] * D;
        float *w = Wm + (int64_t)c * D;
        double ss = 0.0;
        for (int d = 0; d < D; ++d) ss += (double)w[d] * (double)w[d];
        if (ss > 0.0) {
            const double inv = 1.0 / sqrt(ss);
            double dot = 0.0;
            for (int d = 0; d < D; ++d) dot += (double)w[d] * inv * g[d];
            for (int d = 0; d < D; ++d) {
                const double dw = (g[d] - (double)w[d] * inv * dot) * inv;
                w[d] = (float)((double)w[d] + alpha * dw);
            }
        }
        double s2 = 0.0;
        for (int d = 0; d < D; ++d) s2 += (double)w[d] * (double)w[d];
        const double inv2 = s2 > 0.0 ? 1.0 / sqrt(s2) : 0.0;
        if (inv_norm) inv_norm[c] = (float)inv2;
        if (W_hat_bf16)
            for (int d = 0; d < D; ++d) W_hat_bf16[(int64_t)c * D + d] = f32_to_bf16_rne((float)((double)w[d] * inv2));
        slot[c] = -1;
    }
    free(sum);
    free(slot);
    return ORC_OK;
}
