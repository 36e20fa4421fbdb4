// Active-class selection (Algorithm 1 of the paper, without the random fill-up branch) on the GPU.
//
// Data structure: a table score[C] (int32) indexed by class id.  Marking a candidate is an integer
// atomicMin of its list position into the table, so duplicates collapse by construction and the
// result does not depend on the order of the atomics.  The ascending active list is then a stream
// compaction of the table; the cut to M classes is a threshold on the score (found from a histogram
// over list positions) plus a quota of the lowest ids at the threshold score.
//
// Where the candidates come from is a template parameter: the dense [C, K] graph of a GPU that owns all classes, or
// the compressed graph of one node of the sharded layer (Section 3.2.3: per class of the whole problem only the
// neighbours this node owns, as local ids, lists of different lengths laid end to end and found through a
// running sum of their lengths).  The random fill-up of Algorithm 1 is an optional last stage of both.
#include "ks_select.h"
#include <mutex>

#define SEL_NT 256
#define SEL_PER 8
#define SEL_SEG (SEL_NT * SEL_PER) /* classes per block in the table passes */
#define SEL_NONE 0x7fffffff
#define SEL_LDS_BINS 2048

struct SelPlan {
    int r_star;    // classes with score < r_star are all kept
    int quota;     // number of classes with score == r_star that are kept (lowest ids)
    int n_active;
    int n_unique;
    int n_found;   // classes found by the lists (capped at M), before the fill-up
};

struct SelWs {
    int32_t *score;    // [C]      min list position per class, later: position in the active list
    int32_t *hist;     // [K + 1]  number of distinct classes per score
    int32_t *blk_cnt;  // [nblk*2] per table block: (#score < r_star, #score == r_star)
    int32_t *blk_base; // [nblk*2] exclusive prefixes of the kept counts / of the == r_star counts
    SelPlan *plan;
    int nblk;
};

static SelWs sel_carve(void *ws, int64_t C, int K) {
    KsArena ar(ws);
    SelWs w;
    w.nblk = (int)ks_ceil_div(C, SEL_SEG);
    w.score = ar.take<int32_t>((size_t)C);
    w.hist = ar.take<int32_t>((size_t)K + 1);
    w.blk_cnt = ar.take<int32_t>((size_t)w.nblk * 2);
    w.blk_base = ar.take<int32_t>((size_t)w.nblk * 2);
    w.plan = ar.take<SelPlan>(1);
    return w;
}

size_t ks_select_ws_bytes(int64_t C, int B, int K) {
    if (C <= (int64_t)SEL1_MAX_WORDS_HOST * 32) return ks_align_up((size_t)B * (K + 1) * sizeof(int32_t), 256);
    KsArena ar(nullptr);
    ar.take<int32_t>((size_t)C);
    ar.take<int32_t>((size_t)K + 1);
    size_t nblk = (size_t)ks_ceil_div(C, SEL_SEG);
    ar.take<int32_t>(nblk * 2);
    ar.take<int32_t>(nblk * 2);
    ar.take<SelPlan>(1);
    return ar.off;
}

__global__ void __launch_bounds__(SEL_NT) sel_init_kernel(int32_t *score, int64_t C, int32_t *hist, int K) {
    int64_t t = (int64_t)blockIdx.x * SEL_NT + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * SEL_NT;
    for (int64_t c = t; c < C; c += stride) score[c] = SEL_NONE;
    for (int64_t r = t; r <= K; r += stride) hist[r] = 0;
}

// one thread per (sample i, list position r): r = 0 is the label itself, r >= 1 is column r-1 of its list
template <class Src>
__global__ void __launch_bounds__(SEL_NT) sel_mark_kernel(Src src, int B, int K, int32_t *score, int32_t *dev_status) {
    int64_t t = (int64_t)blockIdx.x * SEL_NT + threadIdx.x;
    if (t >= (int64_t)B * (K + 1)) return;
    int i = (int)(t / (K + 1)), r = (int)(t % (K + 1));
    const int32_t c = src.cand(i, r, dev_status);
    if (c >= 0) atomicMin(&score[c], r);
}

__global__ void __launch_bounds__(SEL_NT)
sel_hist_kernel(const int32_t *__restrict__ score, int64_t C, int K, int32_t *hist) {
    __shared__ int32_t lh[SEL_LDS_BINS];
    const bool use_lds = (K + 1) <= SEL_LDS_BINS;
    if (use_lds) {
        for (int r = threadIdx.x; r <= K; r += SEL_NT) lh[r] = 0;
        __syncthreads();
    }
    int64_t c0 = (int64_t)blockIdx.x * SEL_SEG;
    for (int e = 0; e < SEL_PER; ++e) {
        int64_t c = c0 + (int64_t)e * SEL_NT + threadIdx.x;
        if (c < C) {
            int32_t r = score[c];
            if (r != SEL_NONE) {
                if (use_lds) atomicAdd(&lh[r], 1);
                else atomicAdd(&hist[r], 1);
            }
        }
    }
    if (use_lds) {
        __syncthreads();
        for (int r = threadIdx.x; r <= K; r += SEL_NT)
            if (lh[r]) atomicAdd(&hist[r], lh[r]);
    }
}

// single block: find the score threshold for the cut to M
__global__ void __launch_bounds__(1024) sel_plan_kernel(const int32_t *__restrict__ hist, int K, int M, SelPlan *plan) {
    __shared__ int sh[1024 / 64 + 1];
    __shared__ int s_rstar, s_quota;
    if (threadIdx.x == 0) { s_rstar = K + 1; s_quota = 0; }
    __syncthreads();
    int carry = 0;
    for (int r0 = 0; r0 <= K; r0 += 1024) {
        int r = r0 + threadIdx.x;
        int v = (r <= K) ? hist[r] : 0;
        int tot;
        int ex = ks_block_escan<1024>(v, sh, &tot) + carry; // classes with score < r
        // the unique r at which the running count first exceeds M
        if (r <= K && ex <= M && ex + v > M) { s_rstar = r; s_quota = M - ex; }
        carry += tot;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        plan->r_star = s_rstar;
        plan->quota = s_quota;
        plan->n_unique = carry;
        plan->n_active = carry < M ? carry : M;
        plan->n_found = plan->n_active;
    }
}

// single block, after the plan: random fill-up when fewer than M classes were found.  Drawn classes get the score
// K (any score below the cut), so the compaction that follows emits them with the rest.
__global__ void __launch_bounds__(1024) sel_pad_kernel(int32_t *score, int64_t C, int K, int M, SelPad pad, SelPlan *plan) {
    __shared__ int sh[1024 / 64 + 1];
    const int found = plan->n_unique;
    const int64_t want = M < C ? M : C;
    if (found >= want) return;
    const int need = (int)(want - found);
    const uint64_t n_draws = (uint64_t)1 << pad.b;
    int got = 0;
    for (uint64_t k0 = 0; got < need && k0 < n_draws; k0 += 1024 * 8) {
        uint32_t cs[8];
        int valid = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint64_t k = k0 + (uint64_t)threadIdx.x * 8 + e;
            const uint32_t c = k < n_draws ? sel_pad_draw((uint32_t)k, pad) : 0xFFFFFFFFu;
            cs[e] = (c < (uint64_t)C && score[c] == SEL_NONE) ? c : 0xFFFFFFFFu;
            valid += cs[e] != 0xFFFFFFFFu;
        }
        int tot;
        int ex = ks_block_escan<1024>(valid, sh, &tot);
        const int room = need - got;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (cs[e] != 0xFFFFFFFFu) {
                if (ex < room) score[cs[e]] = K;
                ++ex;
            }
        got += tot < room ? tot : room;
        __syncthreads();
    }
    if (threadIdx.x == 0) plan->n_active = found + got;
}

__global__ void __launch_bounds__(SEL_NT)
sel_count_kernel(const int32_t *__restrict__ score, int64_t C, const SelPlan *plan, int32_t *blk_cnt) {
    __shared__ int s_lt[SEL_NT / 64], s_eq[SEL_NT / 64];
    const int r_star = plan->r_star;
    int lt = 0, eq = 0;
    int64_t c0 = (int64_t)blockIdx.x * SEL_SEG + (int64_t)threadIdx.x * SEL_PER;
    for (int e = 0; e < SEL_PER; ++e) {
        int64_t c = c0 + e;
        if (c < C) {
            int32_t r = score[c];
            lt += (r < r_star);
            eq += (r == r_star);
        }
    }
    lt = ks_wave_sum_i(lt);
    eq = ks_wave_sum_i(eq);
    if ((threadIdx.x & 63) == 0) { s_lt[threadIdx.x >> 6] = lt; s_eq[threadIdx.x >> 6] = eq; }
    __syncthreads();
    if (threadIdx.x == 0) {
        int a = 0, b = 0;
        for (int w = 0; w < SEL_NT / 64; ++w) { a += s_lt[w]; b += s_eq[w]; }
        blk_cnt[2 * blockIdx.x] = a;
        blk_cnt[2 * blockIdx.x + 1] = b;
    }
}

// single block: exclusive prefixes over table blocks of (#kept, #score == r_star)
__global__ void __launch_bounds__(1024)
sel_scan_kernel(const int32_t *__restrict__ blk_cnt, int nblk, const SelPlan *plan, int32_t *blk_base) {
    __shared__ int sh[1024 / 64 + 1];
    const int quota = plan->quota;
    int carry_eq = 0, carry_keep = 0;
    for (int b0 = 0; b0 < nblk; b0 += 1024) {
        int b = b0 + threadIdx.x;
        int lt = (b < nblk) ? blk_cnt[2 * b] : 0;
        int eq = (b < nblk) ? blk_cnt[2 * b + 1] : 0;
        int tot_eq;
        int ex_eq = ks_block_escan<1024>(eq, sh, &tot_eq) + carry_eq;
        int rem = quota - ex_eq;                                   // quota left when this block starts
        int keep_eq = rem <= 0 ? 0 : (rem < eq ? rem : eq);
        int tot_keep;
        int ex_keep = ks_block_escan<1024>(lt + keep_eq, sh, &tot_keep) + carry_keep;
        if (b < nblk) { blk_base[2 * b] = ex_keep; blk_base[2 * b + 1] = ex_eq; }
        carry_eq += tot_eq;
        carry_keep += tot_keep;
    }
}

// compaction: writes the ascending active list and turns score[c] into the position of c (or -1)
__global__ void __launch_bounds__(SEL_NT)
sel_emit_kernel(int32_t *score, int64_t C, const SelPlan *plan, const int32_t *__restrict__ blk_base, int M,
                int32_t *active_idx) {
    __shared__ int sh[SEL_NT / 64 + 1];
    const int r_star = plan->r_star, quota = plan->quota;
    const int64_t c0 = (int64_t)blockIdx.x * SEL_SEG + (int64_t)threadIdx.x * SEL_PER;
    int32_t r[SEL_PER];
    int eq = 0;
    for (int e = 0; e < SEL_PER; ++e) {
        int64_t c = c0 + e;
        r[e] = (c < C) ? score[c] : SEL_NONE;
        eq += (r[e] == r_star);
    }
    int tot;
    int eq_rank = ks_block_escan<SEL_NT>(eq, sh, &tot) + blk_base[2 * blockIdx.x + 1];
    int keep = 0;
    unsigned mask = 0;
    for (int e = 0; e < SEL_PER; ++e) {
        bool k = r[e] < r_star;
        if (r[e] == r_star) { k = eq_rank < quota; ++eq_rank; }
        if (k) { mask |= 1u << e; ++keep; }
    }
    int pos = ks_block_escan<SEL_NT>(keep, sh, &tot) + blk_base[2 * blockIdx.x];
    for (int e = 0; e < SEL_PER; ++e) {
        int64_t c = c0 + e;
        if (c >= C) break;
        if (mask & (1u << e)) {
            if (pos < M) active_idx[pos] = (int32_t)c; // pos < M always holds; the test keeps stores in bounds
            score[c] = pos;
            ++pos;
        } else {
            score[c] = -1;
        }
    }
}

template <class Src>
__global__ void __launch_bounds__(SEL_NT)
sel_finish_kernel(Src src, const int32_t *__restrict__ score, int B, int M, const SelPlan *plan, int32_t *active_idx,
                  int32_t *n_active, int32_t *n_found, int32_t *target_pos) {
    int t = blockIdx.x * SEL_NT + threadIdx.x;
    const int n = plan->n_active;
    if (t == 0) {
        *n_active = n;
        if (n_found) *n_found = plan->n_found;
    }
    if (t < B) {
        const int32_t y = src.cand(t, 0, nullptr);
        const int32_t none = Src::kForeignLabels ? -1 : 0; // in range even for broken inputs (those are flagged)
        int32_t p = y >= 0 ? score[y] : none;
        target_pos[t] = (p >= 0 && p < n) ? p : none;
    }
    if (t >= n && t < M) active_idx[t] = -1;
}

// ------------------------------------------------------------------------------------------------
// Whole selection inside a workgroup when the class bitmap fits in LDS (C <= SEL1_MAX_WORDS * 32):
// candidates are marked in an LDS bitmap (duplicates collapse in the atomic OR), the ascending list is the
// bitmap read out in order, positions are prefix popcounts.  Only when more than M classes are marked
// is the list-position order needed; then the bitmap is rebuilt position by position (r = 0, 1, ...)
// until adding the classes first seen at position r would exceed M; of those, the lowest ids fill up.
// SEL1_GRID workgroups all do this same LDS work and differ only in which slice of the outputs they
// write: the global stores and their latency are spread over several compute units with no
// synchronisation between workgroups.
// ------------------------------------------------------------------------------------------------
// Stage 1 (many workgroups, so that the scattered reads of the neighbour lists are spread over the chip):
// validated candidates, list-position-major: cand[r * B + i] = class at position r of sample i's list
// (r = 0: the label itself), or -1 for an empty or invalid entry.
template <class Src>
__global__ void __launch_bounds__(SEL_NT)
sel_fetch_kernel(Src src, int B, int K, int32_t *__restrict__ cand, int32_t *dev_status) {
    const int64_t t = (int64_t)blockIdx.x * SEL_NT + threadIdx.x;
    if (t >= (int64_t)B * (K + 1)) return;
    const int i = (int)(t / (K + 1)), r = (int)(t % (K + 1));
    cand[(int64_t)r * B + i] = src.cand(i, r, dev_status);
}

__global__ void __launch_bounds__(SEL1_NT)
sel_single_kernel(const int32_t *__restrict__ cand, int64_t C, int B, int K, int M, int foreign_labels, SelPad pad,
                  int32_t *__restrict__ active_idx, int32_t *__restrict__ n_active, int32_t *__restrict__ n_found,
                  int32_t *__restrict__ target_pos) {
    __shared__ uint32_t lds[sel1_lds_words(SEL1_NT)];
    sel1_body<SEL1_NT>(lds, cand, C, B, K, M, foreign_labels, pad, active_idx, n_active, n_found, target_pos, (int)gridDim.x,
                       (int)blockIdx.x);
}

template <class Src>
static int sel_launch(const Src &src, int64_t C, int B, int K, int M, SelPad pad, int32_t *active_idx, int32_t *n_active,
                      int32_t *n_found, int32_t *target_pos, void *ws, int32_t *dev_status, hipStream_t st) {
    const int64_t n_cand = (int64_t)B * (K + 1);
    if ((uintptr_t)ws & 15) return KS_INVALID_ARG; // the staging array is read in 16-byte pieces
    if (C <= (int64_t)SEL1_MAX_WORDS * 32) {
        int32_t *cand = (int32_t *)ws;
        hipLaunchKernelGGL(sel_fetch_kernel<Src>, dim3((unsigned)ks_ceil_div(n_cand, SEL_NT)), dim3(SEL_NT), 0, st, src, B, K,
                           cand, dev_status);
        hipLaunchKernelGGL(sel_single_kernel, dim3(SEL1_GRID), dim3(SEL1_NT), 0, st, cand, C, B, K, M,
                           (int)Src::kForeignLabels, pad, active_idx, n_active, n_found, target_pos);
        KS_LAUNCH_CHECK();
        return KS_OK;
    }
    SelWs w = sel_carve(ws, C, K);
    int fill_blocks = (int)(ks_ceil_div(C, SEL_NT) < 2048 ? ks_ceil_div(C, SEL_NT) : 2048);
    hipLaunchKernelGGL(sel_init_kernel, dim3(fill_blocks), dim3(SEL_NT), 0, st, w.score, C, w.hist, K);
    hipLaunchKernelGGL(sel_mark_kernel<Src>, dim3((unsigned)ks_ceil_div(n_cand, SEL_NT)), dim3(SEL_NT), 0, st, src, B, K,
                       w.score, dev_status);
    hipLaunchKernelGGL(sel_hist_kernel, dim3(w.nblk), dim3(SEL_NT), 0, st, w.score, C, K, w.hist);
    hipLaunchKernelGGL(sel_plan_kernel, dim3(1), dim3(1024), 0, st, w.hist, K, M, w.plan);
    if (pad.on) hipLaunchKernelGGL(sel_pad_kernel, dim3(1), dim3(1024), 0, st, w.score, C, K, M, pad, w.plan);
    hipLaunchKernelGGL(sel_count_kernel, dim3(w.nblk), dim3(SEL_NT), 0, st, w.score, C, w.plan, w.blk_cnt);
    hipLaunchKernelGGL(sel_scan_kernel, dim3(1), dim3(1024), 0, st, w.blk_cnt, w.nblk, w.plan, w.blk_base);
    hipLaunchKernelGGL(sel_emit_kernel, dim3(w.nblk), dim3(SEL_NT), 0, st, w.score, C, w.plan, w.blk_base, M,
                       active_idx);
    int fin = B > M ? B : M;
    hipLaunchKernelGGL(sel_finish_kernel<Src>, dim3((unsigned)ks_ceil_div(fin, SEL_NT)), dim3(SEL_NT), 0, st, src, w.score,
                       B, M, w.plan, active_idx, n_active, n_found, target_pos);
    KS_LAUNCH_CHECK();
    return KS_OK;
}

int ks_select_launch(const int32_t *labels, const int32_t *graph, int64_t C, int B, int K, int M,
                     int32_t *active_idx, int32_t *n_active, int32_t *target_pos, void *ws,
                     int32_t *dev_status, hipStream_t st) {
    SelDense src{labels, graph, C, K};
    return sel_launch(src, C, B, K, M, sel_pad_make(0, C, 0), active_idx, n_active, nullptr, target_pos, ws, dev_status, st);
}

extern "C" size_t knn_select_workspace(int64_t C, int B, int K, int M) {
    (void)M;
    if (C < 1 || K < 0) return 0;
    return ks_select_ws_bytes(C, B, K);
}

extern "C" int knn_select_active(const int32_t *labels, const int32_t *graph, int64_t C, int B, int K, int M,
                                 int32_t *active_idx, int32_t *n_active, int32_t *target_pos, void *ws,
                                 size_t ws_bytes, int32_t *dev_status, void *stream) {
    if (!labels || !active_idx || !n_active || !target_pos || !ws) return KS_INVALID_ARG;
    if (C < 1 || C >= (int64_t)1 << 31 || B < 1 || K < 0 || M < 1) return KS_INVALID_ARG;
    if (K > 0 && !graph) return KS_INVALID_ARG;
    if (B > M || (int64_t)K + 1 > M) return KS_INVALID_ARG;
    if (ws_bytes < ks_select_ws_bytes(C, B, K)) return KS_WORKSPACE_TOO_SMALL;
    return ks_select_launch(labels, graph, C, B, K, M, active_idx, n_active, target_pos, ws, dev_status,
                            (hipStream_t)stream);
}

// ------------------------------------------------------------------------------------------------
// The selection for callers that cannot allocate: its scratch memory is this file-scope device array.  In host
// code the array's name is only a handle of the symbol; the address of each GPU's copy is asked for once per
// device (hipGetSymbolAddress, with that device current) and kept.
// ------------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[KS_SELECT_STATIC_BYTES];
#define KS_MAX_DEVICES 64
static void *g_scratch_ptr[KS_MAX_DEVICES];
static std::mutex g_scratch_mutex;

static int sel_scratch_for_current_device(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= KS_MAX_DEVICES) return KS_HIP_ERROR;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return KS_HIP_ERROR;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return KS_OK;
}

extern "C" int knn_select_active_static(const int32_t *labels, const int32_t *graph, int64_t C, int B, int K, int M,
                                        int32_t *active_idx, int32_t *n_active, int32_t *target_pos, int32_t *dev_status,
                                        void *stream) {
    if (!labels || !active_idx || !n_active || !target_pos) return KS_INVALID_ARG;
    if (C < 1 || C >= (int64_t)1 << 31 || B < 1 || K < 0 || M < 1) return KS_INVALID_ARG;
    if (K > 0 && !graph) return KS_INVALID_ARG;
    if (B > M || (int64_t)K + 1 > M) return KS_INVALID_ARG;
    if (ks_select_ws_bytes(C, B, K) > (size_t)KS_SELECT_STATIC_BYTES) return KS_UNSUPPORTED;
    void *ptr = nullptr;
    const int rc = sel_scratch_for_current_device(&ptr);
    if (rc != KS_OK) return rc;
    return ks_select_launch(labels, graph, C, B, K, M, active_idx, n_active, target_pos, ptr, dev_status,
                            (hipStream_t)stream);
}

extern "C" size_t knn_select_active_csr_workspace(int64_t C_loc, int B, int K_max, int M) {
    (void)M;
    if (C_loc < 1 || K_max < 0 || B < 1) return 0;
    return ks_select_ws_bytes(C_loc, B, K_max);
}

extern "C" int knn_select_active_csr(const int32_t *labels, const int32_t *counts, const int64_t *offsets,
                                     const int32_t *flat, int64_t flat_len, int64_t Cg, int64_t c0, int64_t C_loc, int B,
                                     int K_max, int M, uint32_t flags, uint64_t pad_seed, int32_t *active_idx,
                                     int32_t *n_active, int32_t *n_found, int32_t *target_pos, void *ws, size_t ws_bytes,
                                     int32_t *dev_status, void *stream) {
    if (!labels || !counts || !offsets || !active_idx || !n_active || !target_pos || !ws) return KS_INVALID_ARG;
    if (Cg < 1 || Cg >= (int64_t)1 << 31 || c0 < 0 || C_loc < 1 || c0 + C_loc > Cg) return KS_INVALID_ARG;
    if (B < 1 || K_max < 0 || M < 1 || flat_len < 0) return KS_INVALID_ARG;
    if (flat_len > 0 && !flat) return KS_INVALID_ARG;
    if (B > M || (int64_t)K_max + 1 > M) return KS_INVALID_ARG;
    if (flags & ~(uint32_t)KS_FLAG_PAD_RANDOM) return KS_INVALID_ARG;
    if (ws_bytes < ks_select_ws_bytes(C_loc, B, K_max)) return KS_WORKSPACE_TOO_SMALL;
    SelCsr src{labels, counts, offsets, flat, Cg, c0, C_loc, flat_len, K_max};
    return sel_launch(src, C_loc, B, K_max, M, sel_pad_make((flags & KS_FLAG_PAD_RANDOM) != 0, C_loc, pad_seed), active_idx,
                      n_active, n_found, target_pos, ws, dev_status, (hipStream_t)stream);
}

// ------------------------------------------------------------------------------------------------
// Graph compression (Section 3.2.3 (i)): per class of the whole problem the neighbours this node owns.
// Three launches: list lengths and their sums per block of classes; running sum over the blocks; offsets and the
// lists themselves.
// ------------------------------------------------------------------------------------------------
#define GC_NT 256
#define GC_SEG (GC_NT * 4) /* classes per block */

#define GC_COLS 32               /* list entries staged per pass */
#define GC_LD (GC_COLS + 1)      /* LDS row stride (odd: lanes reading their own rows hit different banks) */

// Calls f(c) on lane l for every entry c of row g0 + l, in list order (rows past Cg and columns past K read as -1).
// The 64 rows of a wavefront are contiguous in memory: they are loaded 128 bytes per row at a time, coalesced,
// staged in the wavefront's part of LDS and read back row-wise.  Uniform trip counts: every thread of the block
// must call it.
template <class F>
__device__ __forceinline__ void gc_for_rows(const int32_t *__restrict__ graph, int64_t Cg, int K, int64_t g0, int32_t *lds,
                                            F f) {
    const int lane = threadIdx.x & 63;
    int32_t *mine = lds + (threadIdx.x >> 6) * 64 * GC_LD;
    for (int kc = 0; kc < K; kc += GC_COLS) {
        const int kn = K - kc < GC_COLS ? K - kc : GC_COLS;
        for (int t = lane; t < 64 * GC_COLS; t += 64) {
            const int r = t / GC_COLS, j = t % GC_COLS;
            int32_t v = -1;
            if (j < kn && g0 + r < Cg) v = graph[(g0 + r) * K + kc + j];
            mine[r * GC_LD + j] = v;
        }
        __syncthreads();
        for (int j = 0; j < kn; ++j) f(mine[lane * GC_LD + j]);
        __syncthreads();
    }
}

__global__ void __launch_bounds__(GC_NT)
gc_count_kernel(const int32_t *__restrict__ graph, int64_t Cg, int K, int64_t c0, int64_t C_loc, int32_t *__restrict__ counts,
                int64_t *__restrict__ blk_sum, int32_t *dev_status) {
    __shared__ int s_w[GC_NT / 64];
    __shared__ int32_t s_rows[(GC_NT / 64) * 64 * GC_LD];
    int local = 0;
    const int64_t c1 = c0 + C_loc;
    for (int e = 0; e < 4; ++e) {
        const int64_t g = (int64_t)blockIdx.x * GC_SEG + (int64_t)e * GC_NT + threadIdx.x;
        int n = 0;
        bool bad = false;
        gc_for_rows(graph, Cg, K, g - (threadIdx.x & 63), s_rows, [&](int32_t c) {
            bad |= (c < -1 || c >= Cg);
            n += (c >= c0 && c < c1);
        });
        if (bad) ks_flag(dev_status, KS_DEV_BAD_GRAPH_ID);
        if (g < Cg) {
            counts[g] = n;
            local += n;
        }
    }
    local = ks_wave_sum_i(local);
    if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = local;
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t t = 0;
        for (int w = 0; w < GC_NT / 64; ++w) t += s_w[w];
        blk_sum[blockIdx.x] = t;
    }
}

// single block: blk_sum -> exclusive running sum in place; the total goes to offsets[Cg]
__global__ void __launch_bounds__(1024) gc_scan_kernel(int64_t *blk_sum, int nblk, int64_t *offsets, int64_t Cg,
                                                       int64_t flat_capacity, int check_capacity, int32_t *dev_status) {
    __shared__ int64_t s_w[1024 / 64];
    __shared__ int64_t s_carry;
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    for (int b0 = 0; b0 < nblk; b0 += 1024) {
        const int b = b0 + threadIdx.x;
        const int64_t v = b < nblk ? blk_sum[b] : 0;
        int64_t inc = v; // inclusive scan inside the wavefront
        for (int o = 1; o < 64; o <<= 1) {
            const int lo = __shfl_up((int)(uint32_t)inc, o, 64), hi = __shfl_up((int)(inc >> 32), o, 64);
            if ((threadIdx.x & 63) >= o) inc += ((int64_t)hi << 32) | (uint32_t)lo;
        }
        if ((threadIdx.x & 63) == 63) s_w[threadIdx.x >> 6] = inc;
        __syncthreads();
        int64_t base = s_carry;
        for (int w = 0; w < (int)(threadIdx.x >> 6); ++w) base += s_w[w];
        if (b < nblk) blk_sum[b] = base + inc - v;
        __syncthreads();
        if (threadIdx.x == 1023) s_carry = base + inc;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        offsets[Cg] = s_carry;
        if (check_capacity && s_carry > flat_capacity) ks_flag(dev_status, KS_DEV_BAD_COUNT);
    }
}

__global__ void __launch_bounds__(GC_NT)
gc_fill_kernel(const int32_t *__restrict__ graph, int64_t Cg, int K, int64_t c0, int64_t C_loc,
               const int32_t *__restrict__ counts, const int64_t *__restrict__ blk_base, int64_t *__restrict__ offsets,
               int32_t *__restrict__ flat, int64_t flat_capacity) {
    __shared__ int sh[GC_NT / 64 + 1];
    __shared__ int32_t s_rows[(GC_NT / 64) * 64 * GC_LD];
    int64_t base = blk_base[blockIdx.x];
    const int64_t c1 = c0 + C_loc;
    for (int e = 0; e < 4; ++e) {
        const int64_t g = (int64_t)blockIdx.x * GC_SEG + (int64_t)e * GC_NT + threadIdx.x;
        const int n = g < Cg ? counts[g] : 0;
        int tot;
        const int64_t off = base + ks_block_escan<GC_NT>(n, sh, &tot);
        base += tot;
        if (g < Cg) offsets[g] = off;
        if (!flat) continue; // uniform over the block
        // a list that does not fit the array is not written (the scan has flagged the short array)
        const int64_t end = (g < Cg && off + n <= flat_capacity) ? off + n : off;
        int64_t o = off;
        gc_for_rows(graph, Cg, K, g - (threadIdx.x & 63), s_rows, [&](int32_t c) {
            if (c >= c0 && c < c1 && o < end) flat[o++] = (int32_t)(c - c0);
        });
    }
}

// ------------------------------------------------------------------------------------------------
// The same two passes for list lengths that divide 64 (K = 32 and 64 in every workload): one lane per list ENTRY
// instead of one lane per list.  The rows of a block are one contiguous run of GC_SEG * K entries, read with fully
// coalesced loads; a list occupies K consecutive lanes, so its length is a population count over its part of a
// wavefront ballot, and an entry's place in the compressed list is the count of the kept entries before it in
// that part -- list order is preserved.
// ------------------------------------------------------------------------------------------------
#define GC_UNROLL 4

__global__ void __launch_bounds__(GC_NT)
gc_count_entries_kernel(const int32_t *__restrict__ graph, int64_t Cg, int K, int64_t c0, int64_t C_loc,
                        int32_t *__restrict__ counts, int64_t *__restrict__ blk_sum, int32_t *dev_status) {
    __shared__ int s_w[GC_NT / 64];
    const int lane = threadIdx.x & 63;
    const int64_t c1 = c0 + C_loc;
    const int64_t e0 = (int64_t)blockIdx.x * GC_SEG * K, e_end = Cg * K; // entries of this block start at e0
    const int n_it = GC_SEG * K / GC_NT;                               // (K divides 64, GC_SEG is a multiple of GC_NT)
    const int lk = __builtin_ctz((unsigned)K);                          // K is a power of two here
    const int sub = lane >> lk << lk;                                    // first lane of this lane's list
    const uint64_t gmask = (K == 64 ? ~0ull : ((1ull << K) - 1ull)) << sub;
    int local = 0;
    bool bad = false;
    for (int it = 0; it < n_it; it += GC_UNROLL) {
        int32_t c[GC_UNROLL];
#pragma unroll
        for (int u = 0; u < GC_UNROLL; ++u) {
            const int64_t e = e0 + (int64_t)(it + u) * GC_NT + threadIdx.x;
            c[u] = (it + u < n_it && e < e_end) ? graph[e] : -1;
        }
#pragma unroll
        for (int u = 0; u < GC_UNROLL; ++u) {
            if (it + u >= n_it) break; // uniform
            const int64_t e = e0 + (int64_t)(it + u) * GC_NT + threadIdx.x;
            bad |= (c[u] < -1 || c[u] >= Cg);
            const bool keep = c[u] >= c0 && c[u] < c1;
            const uint64_t m = __ballot(keep);
            if (lane == sub && e < e_end) counts[e >> lk] = __popcll(m & gmask);
            local += keep ? 1 : 0;
        }
    }
    if (bad) ks_flag(dev_status, KS_DEV_BAD_GRAPH_ID);
    local = ks_wave_sum_i(local);
    if (lane == 0) s_w[threadIdx.x >> 6] = local;
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t t = 0;
        for (int w = 0; w < GC_NT / 64; ++w) t += s_w[w];
        blk_sum[blockIdx.x] = t;
    }
}

__global__ void __launch_bounds__(GC_NT)
gc_fill_entries_kernel(const int32_t *__restrict__ graph, int64_t Cg, int K, int64_t c0, int64_t C_loc,
                       const int32_t *__restrict__ counts, const int64_t *__restrict__ blk_base, int64_t *__restrict__ offsets,
                       int32_t *__restrict__ flat, int64_t flat_capacity) {
    __shared__ int sh[GC_NT / 64 + 1];
    __shared__ int s_off[GC_SEG + 1]; // start of every list of the block, relative to the block's first entry
    const int lane = threadIdx.x & 63;
    const int64_t base = blk_base[blockIdx.x];
    const int64_t c1 = c0 + C_loc;
    const int64_t g0 = (int64_t)blockIdx.x * GC_SEG;
    {   // offsets of the block's lists: thread t owns lists 4 t .. 4 t + 3
        int n[4], mine = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int64_t g = g0 + threadIdx.x * 4 + q;
            n[q] = g < Cg ? counts[g] : 0;
            mine += n[q];
        }
        int tot;
        int run = ks_block_escan<GC_NT>(mine, sh, &tot);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int64_t g = g0 + threadIdx.x * 4 + q;
            s_off[threadIdx.x * 4 + q] = run;
            if (g < Cg) offsets[g] = base + run;
            run += n[q];
        }
        if (threadIdx.x == GC_NT - 1) s_off[GC_SEG] = run;
    }
    __syncthreads();
    if (!flat) return;
    const int64_t e0 = g0 * K, e_end = Cg * K;
    const int n_it = GC_SEG * K / GC_NT;
    const int lk = __builtin_ctz((unsigned)K); // K is a power of two here
    const int sub = lane >> lk << lk;
    const uint64_t below = ((1ull << lane) - 1ull) & ((K == 64 ? ~0ull : ((1ull << K) - 1ull)) << sub); // earlier lanes of this list
    for (int it = 0; it < n_it; it += GC_UNROLL) {
        int32_t c[GC_UNROLL];
#pragma unroll
        for (int u = 0; u < GC_UNROLL; ++u) {
            const int64_t e = e0 + (int64_t)(it + u) * GC_NT + threadIdx.x;
            c[u] = (it + u < n_it && e < e_end) ? graph[e] : -1;
        }
#pragma unroll
        for (int u = 0; u < GC_UNROLL; ++u) {
            if (it + u >= n_it) break; // uniform
            const int f = (it + u) * GC_NT + (int)threadIdx.x; // entry within the block
            const bool keep = c[u] >= c0 && c[u] < c1;
            const uint64_t m = __ballot(keep);
            if (keep) {
                const int row = f >> lk;
                const int64_t off = base + s_off[row], end = base + s_off[row + 1];
                // a list that does not fit the array is not written (the scan has flagged the short array)
                if (end <= flat_capacity) flat[off + __popcll(m & below)] = (int32_t)(c[u] - c0);
            }
        }
    }
}

extern "C" size_t knn_graph_compress_workspace(int64_t Cg, int K) {
    if (Cg < 1 || K < 0) return 0;
    return ks_align_up((size_t)ks_ceil_div(Cg, GC_SEG) * sizeof(int64_t), 256);
}

extern "C" int knn_graph_compress(const int32_t *graph, int64_t Cg, int K, int64_t c0, int64_t C_loc, int32_t *counts,
                                  int64_t *offsets, int32_t *flat, int64_t flat_capacity, void *ws, size_t ws_bytes,
                                  int32_t *dev_status, void *stream) {
    if (!graph || !counts || !offsets || !ws) return KS_INVALID_ARG;
    if (Cg < 1 || Cg >= (int64_t)1 << 31 || K < 1 || c0 < 0 || C_loc < 1 || c0 + C_loc > Cg) return KS_INVALID_ARG;
    if (flat && flat_capacity < 0) return KS_INVALID_ARG;
    if (ws_bytes < knn_graph_compress_workspace(Cg, K)) return KS_WORKSPACE_TOO_SMALL;
    const int nblk = (int)ks_ceil_div(Cg, GC_SEG);
    int64_t *blk = (int64_t *)ws;
    hipStream_t st = (hipStream_t)stream;
    const bool by_entry = K <= 64 && 64 % K == 0; // a list is a whole number of lists per wavefront
    if (by_entry)
        hipLaunchKernelGGL(gc_count_entries_kernel, dim3(nblk), dim3(GC_NT), 0, st, graph, Cg, K, c0, C_loc, counts, blk,
                           dev_status);
    else
        hipLaunchKernelGGL(gc_count_kernel, dim3(nblk), dim3(GC_NT), 0, st, graph, Cg, K, c0, C_loc, counts, blk, dev_status);
    hipLaunchKernelGGL(gc_scan_kernel, dim3(1), dim3(1024), 0, st, blk, nblk, offsets, Cg, flat_capacity, flat != nullptr,
                       dev_status);
    if (by_entry)
        hipLaunchKernelGGL(gc_fill_entries_kernel, dim3(nblk), dim3(GC_NT), 0, st, graph, Cg, K, c0, C_loc, counts, blk,
                           offsets, flat, flat_capacity);
    else
        hipLaunchKernelGGL(gc_fill_kernel, dim3(nblk), dim3(GC_NT), 0, st, graph, Cg, K, c0, C_loc, counts, blk, offsets, flat,
                           flat_capacity);
    KS_LAUNCH_CHECK();
    return KS_OK;
}
