// Internal interface of the selection stage (see ks_select.hip), and the device code of the single-workgroup selection,
// which also runs as extra workgroups of the step's own launches (the selection of the NEXT batch, ks_softmax.hip).
#pragma once
#include "ks_common.h"

size_t ks_select_ws_bytes(int64_t C, int B, int K);
// Enqueues the selection kernels on `st`.  Arguments must already be validated.
int ks_select_launch(const int32_t *labels, const int32_t *graph, int64_t C, int B, int K, int M,
                     int32_t *active_idx, int32_t *n_active, int32_t *target_pos, void *ws,
                     int32_t *dev_status, hipStream_t st);

#define SEL1_MAX_WORDS_HOST 12288 /* classes / 32 up to which the single-workgroup path is used */
#define SEL1_NT 1024
#define SEL1_GRID 32
#define SEL1_MAX_WORDS SEL1_MAX_WORDS_HOST
#define SEL1_FIRST_WORDS 257 /* one bit per sample of batches up to 8,192 (+ one word so that a clear loop may run over) */
// LDS words of the single-workgroup selection with nt threads: three bitmaps / prefix arrays, the first-of-its-label
// bits, the block scan's partial sums and one counter
__host__ __device__ constexpr int sel1_lds_words(int nt) { return 3 * SEL1_MAX_WORDS + SEL1_FIRST_WORDS + nt / 64 + 2; }

// candidate at list position r of sample i (r = 0: the sample's own class), as an id in [0, C), or -1
struct SelDense {
    const int32_t *labels, *graph;
    int64_t C;
    int K;
    static constexpr bool kForeignLabels = false; // a label this GPU does not own is an error
    __device__ __forceinline__ int32_t cand(int i, int r, int32_t *dev_status) const {
        const int32_t y = labels[i];
        if (y < 0 || y >= C) {
            if (r == 0) ks_flag(dev_status, KS_DEV_BAD_LABEL);
            return -1;
        }
        if (r == 0) return y;
        int32_t c = graph[(int64_t)y * K + (r - 1)];
        if (c < -1 || c >= C) {
            ks_flag(dev_status, KS_DEV_BAD_GRAPH_ID);
            c = -1;
        }
        return c;
    }
};
struct SelCsr {
    const int32_t *labels, *counts;
    const int64_t *offsets;
    const int32_t *flat;
    int64_t Cg, c0, C, flat_len; // classes of the whole problem; first class and number of classes of this node
    int K;                       // upper bound of the list lengths
    static constexpr bool kForeignLabels = true; // labels of other nodes' classes have no target here
    __device__ __forceinline__ int32_t cand(int i, int r, int32_t *dev_status) const {
        const int32_t y = labels[i];
        if (y < 0 || y >= Cg) {
            if (r == 0) ks_flag(dev_status, KS_DEV_BAD_LABEL);
            return -1;
        }
        if (r == 0) {
            const int64_t l = (int64_t)y - c0;
            return (l >= 0 && l < C) ? (int32_t)l : -1;
        }
        const int32_t n = counts[y];
        if (r - 1 >= n) return -1;
        const int64_t off = offsets[y];
        if (n > K || off < 0 || off + n > flat_len) { // a list longer than promised or outside the array: not read
            if (r == 1) ks_flag(dev_status, KS_DEV_BAD_COUNT);
            return -1;
        }
        int32_t c = flat[off + (r - 1)];
        if (c < -1 || c >= C) {
            ks_flag(dev_status, KS_DEV_BAD_GRAPH_ID);
            c = -1;
        }
        return c;
    }
};

// k-th draw of the random fill-up: a keyed one-to-one map of [0, 2^b) onto itself (adding a constant, multiplying
// by an odd constant and xor with a right shift of itself are each one-to-one on b-bit numbers), 2^b the smallest
// power of two >= C.  Draws >= C or already in the set are passed over: a sample without replacement of the
// classes not chosen (Algorithm 1 only says "random sample").
struct SelPad {
    int on, b;
    uint32_t mask, s_lo, s_hi;
};
inline SelPad sel_pad_make(int on, int64_t C, uint64_t seed) {
    SelPad p;
    p.on = on;
    p.b = 1;
    while (((int64_t)1 << p.b) < C) ++p.b;
    p.mask = p.b >= 32 ? 0xFFFFFFFFu : ((1u << p.b) - 1u);
    p.s_lo = (uint32_t)seed;
    p.s_hi = (uint32_t)(seed >> 32);
    return p;
}
__device__ __forceinline__ uint32_t sel_pad_draw(uint32_t k, const SelPad &p) {
    const int s1 = (p.b + 1) >> 1, s2 = p.b / 3 > 0 ? p.b / 3 : 1;
    uint32_t x = (k + p.s_lo) & p.mask;
    x = (x * 0x9E3779B1u) & p.mask;
    x ^= x >> s1;
    x = (x * 0x85EBCA6Bu) & p.mask;
    x ^= x >> s2;
    x = (x * 0xC2B2AE35u) & p.mask;
    x ^= x >> s1;
    return (x + p.s_hi) & p.mask;
}

// exclusive prefix over the words of a bitmap: pre[w] = number of set bits in words < w; returns the total
template <int NT>
__device__ __forceinline__ int sel1_prefix(const uint32_t *bm, int nw, int *pre, int *sh) {
    const int per = (nw + NT - 1) / NT;
    const int w0 = threadIdx.x * per;
    int local = 0;
    for (int w = w0; w < w0 + per && w < nw; ++w) local += __popc(bm[w]);
    int total;
    int run = ks_block_escan<NT>(local, sh, &total);
    for (int w = w0; w < w0 + per && w < nw; ++w) {
        pre[w] = run;
        run += __popc(bm[w]);
    }
    __syncthreads();
    return total;
}

// The whole selection by one workgroup of NT threads (see ks_select.hip for the method).  `lds` has sel1_lds_words(NT)
// words.  The G workgroups that call this with g = 0 .. G - 1 all do the same LDS work and write a G-th of the outputs
// each.  A __device__ function so that the workgroups may be those of a kernel of their own or extra workgroups of
// another launch.
template <int NT>
__device__ __forceinline__ void sel1_body(uint32_t *lds, const int32_t *__restrict__ cand, int64_t C, int B, int K, int M,
                                          int foreign_labels, SelPad pad, int32_t *__restrict__ active_idx,
                                          int32_t *__restrict__ n_active, int32_t *__restrict__ n_found,
                                          int32_t *__restrict__ target_pos, const int G, const int g) {
    uint32_t *bm = lds, *eq = lds + SEL1_MAX_WORDS;
    int *pre = (int *)(lds + 2 * SEL1_MAX_WORDS);
    uint32_t *s_first = lds + 3 * SEL1_MAX_WORDS;
    int *sh = (int *)(s_first + SEL1_FIRST_WORDS);
    int &s_new = sh[NT / 64 + 1];
    const int nw = (int)((C + 31) >> 5);
    const int tid = threadIdx.x;
    for (int w = tid; w < nw; w += NT) bm[w] = 0u;
    __syncthreads();
    // optimistic pass: every candidate, whatever its list position (sixteen loads in flight per thread: the
    // round trips to L2 are what this phase costs)
    const int64_t n_cand = (int64_t)B * (K + 1);
    const int64_t n_vec = n_cand >> 2; // the staging array is 256-byte aligned: whole 16-byte pieces, then a tail
    // Samples with the same label have the same list, and with skewed labels half of the batch are repeats: only the
    // first sample of a label (whichever thread marks the label first) has its list marked.  s_first holds one bit
    // per sample; for batch sizes that are a power of two, so that a 16-byte piece of the staging array holds four
    // samples of one list position and the sample index is a mask away.
    const bool dedup = B >= 4 && (B & (B - 1)) == 0 && B <= SEL1_FIRST_WORDS * 32;
    int64_t v_begin = 0;
    if (dedup) {
        for (int w = tid; w < B / 32 + 1; w += NT) s_first[w] = 0u;
        __syncthreads();
        for (int i = tid; i < B; i += NT) {
            const int32_t c = cand[i]; // list position 0: the label (or -1: a class of another node, whose list still counts)
            bool first = true;
            if (c >= 0) first = !(atomicOr(&bm[c >> 5], 1u << (c & 31)) & (1u << (c & 31)));
            if (first) atomicOr(&s_first[i >> 5], 1u << (i & 31));
        }
        __syncthreads();
        v_begin = B >> 2; // the labels are done
    }
    for (int64_t t0 = v_begin; t0 < n_vec; t0 += (int64_t)NT * 8) {
        int4 c[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int64_t t = t0 + (int64_t)e * NT + tid;
            c[e] = t < n_vec ? ((const int4 *)cand)[t] : make_int4(-1, -1, -1, -1);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            uint32_t f4 = 0xFu; // which of the four samples are the first of their label
            if (dedup) {
                const int i0 = (int)(((t0 + (int64_t)e * NT + tid) << 2) & (B - 1));
                f4 = s_first[i0 >> 5] >> (i0 & 31);
            }
            if (c[e].x >= 0 && (f4 & 1u)) atomicOr(&bm[c[e].x >> 5], 1u << (c[e].x & 31));
            if (c[e].y >= 0 && (f4 & 2u)) atomicOr(&bm[c[e].y >> 5], 1u << (c[e].y & 31));
            if (c[e].z >= 0 && (f4 & 4u)) atomicOr(&bm[c[e].z >> 5], 1u << (c[e].z & 31));
            if (c[e].w >= 0 && (f4 & 8u)) atomicOr(&bm[c[e].w >> 5], 1u << (c[e].w & 31));
        }
    }
    for (int64_t t = n_vec * 4 + tid; t < n_cand; t += NT) {
        const int32_t c = cand[t];
        if (c >= 0) atomicOr(&bm[c >> 5], 1u << (c & 31));
    }
    __syncthreads();
    int total = sel1_prefix<NT>(bm, nw, pre, sh);
    if (total > M) {
        // the cut bites: rebuild the bitmap in list-position order
        for (int w = tid; w < nw; w += NT) { bm[w] = 0u; eq[w] = 0u; }
        __syncthreads();
        int cum = 0, quota = 0;
        for (int r = 0; r <= K; ++r) {
            if (tid == 0) s_new = 0;
            __syncthreads();
            int local_new = 0;
            for (int i = tid; i < B; i += NT) {
                const int c = cand[(int64_t)r * B + i];
                if (c < 0) continue;
                const uint32_t bit = 1u << (c & 31);
                if (bm[c >> 5] & bit) continue; // already in with a better position
                if (!(atomicOr(&eq[c >> 5], bit) & bit)) ++local_new;
            }
            local_new = ks_wave_sum_i(local_new);
            if ((tid & 63) == 0 && local_new) atomicAdd(&s_new, local_new);
            __syncthreads();
            const int total_new = s_new;
            if (cum + total_new > M) { // classes first seen at position r do not all fit: r is the cut score
                quota = M - cum;
                break;
            }
            for (int i = tid; i < B; i += NT) { // commit position r
                const int c = cand[(int64_t)r * B + i];
                if (c < 0) continue;
                const uint32_t bit = 1u << (c & 31);
                if (eq[c >> 5] & bit) {
                    atomicOr(&bm[c >> 5], bit);
                    atomicAnd(&eq[c >> 5], ~bit);
                }
            }
            cum += total_new;
            __syncthreads();
        }
        // eq holds the classes whose best position is the cut score; the `quota` lowest ids of them are kept
        sel1_prefix<NT>(eq, nw, pre, sh);
        const int per = (nw + NT - 1) / NT;
        for (int w = tid * per; w < tid * per + per && w < nw; ++w) {
            uint32_t e = eq[w], keep = 0u;
            int left = quota - pre[w];
            while (left > 0 && e) {
                keep |= e & (0u - e);
                e &= e - 1;
                --left;
            }
            bm[w] |= keep;
        }
        __syncthreads();
        total = sel1_prefix<NT>(bm, nw, pre, sh);
    }
    const int found = total < M ? total : M;
    const int64_t want = M < C ? M : C;
    if (pad.on && total < want) {
        // random fill-up: the first draws that are classes of this GPU and not in the bitmap yet (the draws are
        // distinct, so marking one cannot change the test of another)
        const int need = (int)(want - total);
        const uint32_t n_draws = 1u << pad.b; // b <= 19 here
        int got = 0;
        for (uint32_t k0 = 0; got < need && k0 < n_draws; k0 += NT * 8) {
            uint32_t cs[8];
            int valid = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t k = k0 + (uint32_t)tid * 8 + e;
                const uint32_t c = k < n_draws ? sel_pad_draw(k, pad) : 0xFFFFFFFFu;
                cs[e] = (c < (uint64_t)C && !(bm[c >> 5] & (1u << (c & 31)))) ? c : 0xFFFFFFFFu;
                valid += cs[e] != 0xFFFFFFFFu;
            }
            int tot;
            int ex = ks_block_escan<NT>(valid, sh, &tot);
            const int room = need - got;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (cs[e] != 0xFFFFFFFFu) {
                    if (ex < room) atomicOr(&bm[cs[e] >> 5], 1u << (cs[e] & 31));
                    ++ex;
                }
            got += tot < room ? tot : room;
            __syncthreads();
        }
        total = sel1_prefix<NT>(bm, nw, pre, sh);
    }
    // Every workgroup of the grid has built the same bitmap and prefix (redundantly: it is LDS work, and it
    // spares a grid-wide synchronisation); each writes its share of the outputs.
    { // read the bitmap out in ascending order: this workgroup's slice of the words, one word per thread
        const int per_g = (nw + G - 1) / G;
        const int w_end = (g + 1) * per_g < nw ? (g + 1) * per_g : nw;
        for (int w = g * per_g + tid; w < w_end; w += NT) {
            uint32_t e = bm[w];
            int pos = pre[w];
            while (e) {
                const int b = __ffs(e) - 1;
                if (pos < M) active_idx[pos] = w * 32 + b; // pos < M always holds; the test keeps the store in bounds
                ++pos;
                e &= e - 1;
            }
        }
    }
    const int n = total < M ? total : M;
    for (int a = n + g * NT + tid; a < M; a += G * NT) active_idx[a] = -1;
    const int none = foreign_labels ? -1 : 0; // in range even for broken inputs (those are flagged)
    for (int i = g * NT + tid; i < B; i += G * NT) {
        const int32_t y = cand[i]; // list position 0: the sample's own class, -1 if it is not one of this GPU's
        int p = none;
        if (y >= 0 && y < C) p = pre[y >> 5] + __popc(bm[y >> 5] & ((1u << (y & 31)) - 1u));
        target_pos[i] = (p >= 0 && p < n) ? p : none;
    }
    if (g == 0 && tid == 0) {
        *n_active = n;
        if (n_found) *n_found = found;
    }
}


// The selection of the NEXT batch as extra workgroups of the step's launches (nsel == 0: none): `nfetch` blocks of
// `fetch_nt` threads stage the candidates (they ride along with the dX launch), `nsel` workgroups select (with the dW
// launch, which leaves compute units idle).  The candidates come from the dense graph of a GPU that owns all classes
// or from the compressed graph of one node (csr_source), then with that selection's fill-up if asked for.
struct KsSelNext {
    int nsel, nfetch;
    int csr_source;
    SelDense dense;
    SelCsr csr;
    SelPad pad;
    int64_t C; // classes the bitmap covers (all classes, or the node's)
    int B, K, M;
    int32_t *cand;
    int32_t *active_idx, *n_active, *n_found, *target_pos;
    int32_t *dev_status;
};
template <int NT> __device__ __forceinline__ void ks_sel_next_fetch(const KsSelNext &s, int block) {
    const int64_t t = (int64_t)block * NT + threadIdx.x;
    if (t >= (int64_t)s.B * (s.K + 1)) return;
    const int i = (int)(t / (s.K + 1)), r = (int)(t % (s.K + 1));
    s.cand[(int64_t)r * s.B + i] = s.csr_source ? s.csr.cand(i, r, s.dev_status) : s.dense.cand(i, r, s.dev_status);
}
template <int NT> __device__ __forceinline__ void ks_sel_next_select(const KsSelNext &s, uint32_t *lds, int g) {
    sel1_body<NT>(lds, s.cand, s.C, s.B, s.K, s.M, s.csr_source, s.pad, s.active_idx, s.n_active, s.n_found, s.target_pos,
                  s.nsel, g);
}
