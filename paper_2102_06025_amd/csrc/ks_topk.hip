// Layer-wise top-k selection for gradient sparsification (Section 3.3.2: divide-and-conquer top-k selection,
// tensors grouped into one launch).
//
// Every step of the method is the same workgroup-level routine, tk_select: the exact top-k of a list of items that
// sits in global memory (first step: a chunk of a gradient tensor; later steps: the survivors of several chunks).
// An item is the 64-bit word  (bits of |g|) << 32 | (0xFFFFFFFF - index) : larger word = larger magnitude, equal
// magnitudes ordered by ascending index, all words distinct, so "top-k" is unique and no step depends on the
// order in which it finds its input.
//
// tk_select (1,024 threads) is a radix selection on the item word, most significant digits first:
//   1. histogram of the current digit in LDS over the items that share the prefix found so far (first level:
//      all items, on the 14 bits of exponent and leading mantissa, in the 64 KB of the still unused sort array;
//      later levels 11 bits); a descending scan finds the bin in which the k-th largest item falls;
//   2. as soon as the items above that bin and the items in it fit the LDS array (8,192 words) they are collected
//      in one more pass over the list -- for gradient-like data after the first level, so the list is read twice;
//   3. the selection goes on inside the boundary bin, now in LDS, down to the item that closes the top-k;
//   4. a step that is not the last one of its tensor hands its survivors on unsorted; the last step orders its k
//      survivors (2,048 buckets over their range, then ranks inside the buckets), which are the output.
// Tensors with long runs of one magnitude (constant, mostly zero) are caught where they would hurt: wavefronts
// merge their histogram adds when all lanes hit one bin, and a chunk whose k-th magnitude is shared by more items
// than LDS holds takes the first of them in index order instead of resolving 32 index bits level by level.
// The passes wait on memory (a workgroup has its list to itself) and on instruction issue, not on bandwidth:
// 16-byte loads, the next batch requested before the current one is worked on, 32-bit arithmetic per item, and
// a plan that cuts tensors so that no step has more than 32,768 items: a tensor of more than about 260,000
// elements at k = 4,096 goes through more than the paper's two steps (a tree of selections instead of chunks +
// one final selection), still without any approximation.
// Tensors of several chunks whose k is small for their size take a shorter way (tk_threshold, tk_filter_kernel): a
// threshold from a sample lets every chunk hand on only what can still matter, in one pass and without a selection of its
// own; the plain tree of selections stays behind as what the final step falls back on when the sample misled.
// Everything is integer work: the result is bit-exact and deterministic.
#include <vector>
#include "ks_common.h"
#include "../../include/grad_topk.h"

#define TK_NT 1024 /* one workgroup per compute unit: its passes wait on memory, and more threads have more loads in flight */
#define TK_BINS 2048
#define TK_CAP 8192
#define TK_LEAF 32768      /* largest chunk of a tensor */
#define TK_NODE_CAP 32768  /* largest input of a later step */
#define TK_MAX_LEVELS 10
#define TK_MAGIC 0x6B706F74646172ll /* "gradtopk" cut to seven bytes */
#define TK_HEADER 32        /* words before the tensor records: [0..7] see grad_topk.h, [8 + 2 l], [9 + 2 l] first node and nodes of level l,
                               [28], [29] the sampled paths' filter steps (first node, count; they come first in level 1),
                               [30], [31] their final steps (first in level 2) */
#define TK_TENSOR 4        /* words per tensor record: n, k, chunks, steps */
#define TK_NODE 12         /* words per step ("node") record */
#define TK_SAMPLE 4096     /* elements of a tensor that its threshold is taken from (the sampled path, see tk_threshold) */
#define TK_SAMPLE_RANK 16  /* the threshold is at least the TK_SAMPLE_RANK-th largest of the sample */

// node record (int64 words)
enum { TK_N_SRC = 0, TK_N_ITEMS, TK_N_K, TK_N_OUT, TK_N_FLAGS, TK_N_FIRST, TK_N_GBEGIN, TK_N_GN, TK_N_AUX, TK_N_FB_FIRST, TK_N_FB_COUNT };
#define TK_F_LEAF 1  /* reads gradients (src = element offset in g); otherwise items (src = offset in the workspace) */
#define TK_F_FINAL 2 /* writes the tensor's output (out = offset in out_idx / out_val); otherwise items (workspace) */
// The sampled path of a tensor of several chunks (three steps whatever its size):
#define TK_F_THRESH 4   /* finds the tensor's threshold from a sample; aux = two workspace words: threshold, then count | overflow */
#define TK_F_FILTER 8   /* a chunk: the items at or above the threshold go to the tensor's list (out), counted in aux + 1 */
#define TK_F_COUNTED 16 /* final step over that list: its length is read from aux + 1; fb_first / fb_count = the steps of
                           the tensor's plain tree (node indices), which this workgroup runs itself if the sample misled */

struct TkShared {
    uint64_t sort[TK_CAP];
    uint32_t hist[TK_BINS];
    uint32_t wave_sum[TK_NT / 64];
    uint32_t b_star, above, count, count_tie, kmin, kmax;
    uint16_t cnt16[TK_BINS];
};

// step 1 reads a chunk of a gradient tensor; index of item i within the tensor = first + i
struct TkSrcGrad {
    static constexpr int VEC = 4; // items per 16-byte load
    static constexpr bool ORDERED = true; // the list is in ascending index order: of equal magnitudes the first ones win
    const float *g;
    uint32_t first;
    __device__ __forceinline__ uint32_t key(int i) const { return __float_as_uint(g[i]) & 0x7FFFFFFFu; }
    __device__ __forceinline__ uint32_t aux(int i) const { return 0xFFFFFFFFu - (first + (uint32_t)i); }
    __device__ __forceinline__ uint64_t item(int i) const { return ((uint64_t)key(i) << 32) | aux(i); }
    __device__ __forceinline__ int head() const { return (int)(((16u - ((uint32_t)(uintptr_t)g & 15u)) & 15u) >> 2); }
    __device__ __forceinline__ uint4 loadv(int i) const { return *(const uint4 *)(g + i); }
    // item e of the vector that starts at item i (e is a constant after unrolling)
    __device__ __forceinline__ uint32_t key_of(const uint4 &v, int e) const {
        return (e == 0 ? v.x : (e == 1 ? v.y : (e == 2 ? v.z : v.w))) & 0x7FFFFFFFu;
    }
    __device__ __forceinline__ uint32_t aux_of(const uint4 &, int i, int e) const { return aux(i + e); }
    __device__ __forceinline__ void unpack(const uint4 &v, int i, uint32_t (&k)[VEC], uint32_t (&a)[VEC]) const {
        k[0] = v.x & 0x7FFFFFFFu, k[1] = v.y & 0x7FFFFFFFu, k[2] = v.z & 0x7FFFFFFFu, k[3] = v.w & 0x7FFFFFFFu;
#pragma unroll
        for (int e = 0; e < VEC; ++e) a[e] = aux(i + e);
    }
};
// step 2 reads the survivors
struct TkSrcItems {
    static constexpr int VEC = 2;
    static constexpr bool ORDERED = false;
    const uint64_t *c;
    __device__ __forceinline__ uint32_t key(int i) const { return ((const uint32_t *)c)[2 * (int64_t)i + 1]; }
    __device__ __forceinline__ uint32_t aux(int i) const { return ((const uint32_t *)c)[2 * (int64_t)i]; }
    __device__ __forceinline__ uint64_t item(int i) const { return c[i]; }
    __device__ __forceinline__ int head() const { return ((uint32_t)(uintptr_t)c & 15u) ? 1 : 0; }
    __device__ __forceinline__ uint4 loadv(int i) const { return *(const uint4 *)(c + i); }
    __device__ __forceinline__ uint32_t key_of(const uint4 &v, int e) const { return e == 0 ? v.y : v.w; }
    __device__ __forceinline__ uint32_t aux_of(const uint4 &v, int, int e) const { return e == 0 ? v.x : v.z; }
    __device__ __forceinline__ void unpack(const uint4 &v, int, uint32_t (&k)[VEC], uint32_t (&a)[VEC]) const {
        a[0] = v.x, k[0] = v.y, a[1] = v.z, k[1] = v.w;
    }
};

// The list a workgroup selects from: n items behind a source, read in 16-byte vectors (plus up to three items
// before the first and after the last whole vector).  Every pass of the selection streams the list from memory
// (from L2 after the first).  A workgroup has its list to itself, so the passes are bound by memory latency: U
// loads per thread are in flight, and the next batch is requested before the current one is worked on.
template <class Src> struct TkList {
    static constexpr int V = Src::VEC;
    static constexpr bool ORDERED = Src::ORDERED;
    Src src;
    int n, head, nq, tail0;

    __device__ __forceinline__ void init(const Src &s, int n_) {
        src = s;
        n = n_;
        head = src.head(); // items before the first 16-byte boundary
        if (head > n) head = n;
        nq = (n - head) / V;
        tail0 = head + nq * V;
    }
    template <int U> __device__ __forceinline__ void load(uint4 (&v)[U], int qb) const {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int q = qb + u * TK_NT + (int)threadIdx.x;
            v[u] = q < nq ? src.loadv(head + q * V) : make_uint4(0u, 0u, 0u, 0u);
        }
    }
    // f(v, qb): v[u] is vector qb + u * TK_NT + threadIdx.x of the list (zero beyond nq), U vectors at a time
    template <int U, class F> __device__ __forceinline__ void batches(F f) const {
        uint4 cur[U], nxt[U];
        load<U>(cur, 0);
        for (int qb = 0; qb < nq; qb += U * TK_NT) {
            const bool more = qb + U * TK_NT < nq;
            if (more) load<U>(nxt, qb + U * TK_NT);
            f(cur, qb);
            if (more) {
#pragma unroll
                for (int u = 0; u < U; ++u) cur[u] = nxt[u];
            }
        }
    }
    // the up to 2 V - 2 items outside the whole vectors: thread t gets one of them (valid) or none
    __device__ __forceinline__ bool edge_item(uint32_t *key, uint32_t *aux) const {
        const int tid = threadIdx.x;
        const int i = tid < head ? tid : tail0 + (tid - head);
        const bool valid = i < n;
        *key = valid ? src.key(i) : 0u;
        *aux = valid ? src.aux(i) : 0u;
        return valid;
    }
    // One pass: f(key, aux, valid) for every item (key = magnitude bits, aux = low word of the item), called by all
    // threads together, so f may use wavefront-wide operations; lanes without an item call it with valid = false.
    template <class F> __device__ __forceinline__ void scan(F f) const {
        uint32_t ekey, eaux;
        const bool evalid = edge_item(&ekey, &eaux); // requested first, used last
        batches<4>([&](const uint4 (&v)[4], int qb) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int q = qb + u * TK_NT + (int)threadIdx.x;
                uint32_t key[V], aux[V];
                src.unpack(v[u], head + q * V, key, aux);
#pragma unroll
                for (int e = 0; e < V; ++e) f(key[e], aux[e], q < nq);
            }
        });
        f(ekey, eaux, evalid);
    }
};

// histogram update for the lanes in play; when all of them hit the same bin (lists of equal values: a constant or
// mostly-zero tensor), one lane adds for all instead of 64 atomics serialising on one address
__device__ __forceinline__ void tk_hist_add(bool in_play, uint32_t bin, uint32_t *hist) {
    const uint64_t act = __builtin_amdgcn_ballot_w64(in_play);
    if (act == 0ull) return;
    const int first = __builtin_ctzll(act);
    const uint32_t b0 = (uint32_t)__shfl((int)bin, first, 64);
    if (__builtin_amdgcn_ballot_w64(in_play && bin == b0) == act) {
        if ((int)(threadIdx.x & 63) == first) atomicAdd(&hist[b0], (uint32_t)__builtin_popcountll(act));
    } else if (in_play) {
        atomicAdd(&hist[bin], 1u);
    }
}

// exclusive prefix sum of v over the workgroup in thread order (all threads call)
__device__ __forceinline__ uint32_t tk_block_exclusive_scan(uint32_t v, TkShared &sh, uint32_t *total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = __shfl_up(inc, o, 64);
        if (lane >= o) inc += up;
    }
    __syncthreads(); // wave_sum may still be read from the previous call
    if (lane == 63) sh.wave_sum[wave] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < TK_NT / 64; ++w) {
        const uint32_t s = sh.wave_sum[w];
        if (w < wave) base += s;
        tot += s;
    }
    if (total) *total = tot;
    return base + inc - v;
}

// append `item` to an LDS array for the lanes with sel set (slot = base[dir * position], position from *counter):
// one LDS atomic per wavefront, not per item
__device__ __forceinline__ void tk_append(bool sel, uint64_t item, uint64_t *base_ptr, uint32_t *counter, int dir) {
    const uint64_t m = __builtin_amdgcn_ballot_w64(sel);
    if (m == 0ull) return;
    const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
    uint32_t base = 0u;
    if (sel && rank == 0u) base = atomicAdd(counter, (uint32_t)__builtin_popcountll(m));
    base = (uint32_t)__shfl((int)base, __builtin_ctzll(m), 64);
    if (sel && base + rank < TK_CAP) base_ptr[dir * (int)(base + rank)] = item; // always inside: the caller has counted
}

// bitonic sort of a[0 .. S) in descending order, S a power of two >= 2
__device__ __forceinline__ void tk_sort_desc(uint64_t *a, int S) {
    for (int size = 2; size <= S; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int p = threadIdx.x; p < (S >> 1); p += TK_NT) {
                const int i = 2 * p - (p & (stride - 1)), j = i + stride;
                const uint64_t x = a[i], y = a[j];
                const bool desc = (i & size) == 0;
                if ((x < y) == desc) {
                    a[i] = y;
                    a[j] = x;
                }
            }
            __syncthreads();
        }
    }
}

__device__ __forceinline__ int tk_pow2_ceil(int v) {
    int S = 2;
    while (S < v) S <<= 1;
    return S;
}

// The bin of hist[0 .. nb) (an LDS array) in which the need-th largest counted item falls, bins taken in descending order:
// returns it, the number of items in higher bins (*above) and in the bin itself (*in_bin).  All threads call.
__device__ __forceinline__ uint32_t tk_find_bin(const uint32_t *hist, int nb, uint32_t need, TkShared &sh, uint32_t *above, uint32_t *in_bin) {
    const int tid = threadIdx.x;
    const int per = nb / TK_NT > 0 ? nb / TK_NT : 1; // thread t owns bins nb-1 - t*per ... downwards (per = 2^j)
    const int top = nb - 1 - tid * per;
    uint32_t own = 0;
    if (tid * per < nb) // (summed in rotated order: with 32 bins per thread a straight walk would put all lanes on one bank)
        for (int q = 0; q < per; ++q) own += hist[top - ((q + tid) & (per - 1))];
    if (tid == 0) sh.b_star = sh.above = 0u; // (always overwritten below: at least `need` items were counted)
    uint32_t run = tk_block_exclusive_scan(own, sh, nullptr);
    if (tid * per < nb && run < need && need <= run + own) { // exactly one thread: the bin is among its own
        for (int q = 0; q < per; ++q) {
            const uint32_t h = hist[top - q];
            if (need <= run + h) {
                sh.b_star = (uint32_t)(top - q);
                sh.above = run;
                break;
            }
            run += h;
        }
    }
    __syncthreads();
    const uint32_t b_star = sh.b_star;
    *above = sh.above;
    *in_bin = hist[b_star];
    __syncthreads();
    return b_star;
}

// digit positions of the radix selection on the 64-bit item: level l covers bits [tk_lo(l), tk_lo(l - 1))
// (the first level has 14 bits: its histogram has the 64 KB of the sort array, which is still free, to itself, and
// 16,384 bins keep the LDS atomics of gradient-like data apart -- with 2,048 bins they serialise on a few dozen bins)
__device__ __forceinline__ int tk_lo(int lev) { return lev == 0 ? 49 : (lev == 1 ? 38 : (lev == 2 ? 32 : (lev == 3 ? 21 : (lev == 4 ? 10 : 0)))); }
#define TK_BINS0 (2 * TK_CAP) /* bins of the first level: the sort array as 32-bit counters */

// Collect pass: items with (item >> lo) > P go to sh.sort from the front (counter sh.count), items with
// (item >> lo) == P from the back (counter sh.count_tie).  A thread counts its items of a batch first, the
// wavefront's counts are summed by shuffles, and one LDS atomic per wavefront and batch reserves the slots.
template <class List> __device__ __forceinline__ void tk_collect(const List &list, int lo, uint64_t P, TkShared &sh) {
    const int tid = threadIdx.x, lane = tid & 63;
    constexpr int V = List::V, U = 4; // U * V <= 32 flag bits (eight vectors at a time cost more registers than a lane has)
    uint32_t ekey, eaux;
    const bool evalid = list.edge_item(&ekey, &eaux); // requested first, used last
    // The comparison is made on the magnitude alone when the digit boundary lies in it (lo >= 32, the usual case):
    // 32-bit operations, a few instructions per item -- these passes are bound by instruction issue, not by memory.
    const bool narrow = lo >= 32;
    const uint32_t P32 = (uint32_t)P;
    const int sh32 = narrow ? lo - 32 : 0;
    list.template batches<U>([&](const uint4 (&v)[U], int qb) {
        uint32_t fa = 0u, ft = 0u; // this thread's items above the bin / in the bin
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int q = qb + u * TK_NT + tid;
            if (q < list.nq) {
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    const uint32_t key = list.src.key_of(v[u], e);
                    bool above, equal;
                    if (narrow) {
                        const uint32_t d = key >> sh32;
                        above = d > P32;
                        equal = d == P32;
                    } else {
                        const uint64_t d = (((uint64_t)key << 32) | list.src.aux_of(v[u], list.head + q * V, e)) >> lo;
                        above = d > P;
                        equal = d == P;
                    }
                    fa |= (above ? 1u : 0u) << (u * V + e);
                    ft |= (equal ? 1u : 0u) << (u * V + e);
                }
            }
        }
        const uint32_t mine = (uint32_t)__builtin_popcount(fa) | ((uint32_t)__builtin_popcount(ft) << 16);
        uint32_t inc = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t up = __shfl_up(inc, o, 64);
            if (lane >= o) inc += up;
        }
        const uint32_t tot = (uint32_t)__shfl((int)inc, 63, 64);
        if (tot == 0u) return; // nothing of this batch is kept by this wavefront
        uint32_t base_a = 0u, base_t = 0u;
        if (lane == 63) {
            if (tot & 0xFFFFu) base_a = atomicAdd(&sh.count, tot & 0xFFFFu);
            if (tot >> 16) base_t = atomicAdd(&sh.count_tie, tot >> 16);
        }
        uint32_t pa = (uint32_t)__shfl((int)base_a, 63, 64) + ((inc - mine) & 0xFFFFu);
        uint32_t pt = (uint32_t)__shfl((int)base_t, 63, 64) + ((inc - mine) >> 16);
        const uint32_t any = fa | ft;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (((any >> (u * V)) & ((1u << V) - 1u)) == 0u) continue; // most vectors hold nothing to keep
            const int q = qb + u * TK_NT + tid;
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const int j = u * V + e;
                if ((any >> j) & 1u) {
                    const uint64_t item = ((uint64_t)list.src.key_of(v[u], e) << 32) | list.src.aux_of(v[u], list.head + q * V, e);
                    if ((fa >> j) & 1u) {
                        if (pa < TK_CAP) sh.sort[pa] = item; // always inside: the caller has counted
                        ++pa;
                    } else {
                        if (pt < TK_CAP) sh.sort[TK_CAP - 1 - pt] = item;
                        ++pt;
                    }
                }
            }
        }
    });
    {
        const uint64_t item = ((uint64_t)ekey << 32) | eaux;
        tk_append(evalid && (item >> lo) > P, item, sh.sort, &sh.count, 1);
        tk_append(evalid && (item >> lo) == P, item, sh.sort + TK_CAP - 1, &sh.count_tie, -1);
    }
}

// sh.sort[0 .. k) in any order -> descending order.  Items are spread over up to 2,048 buckets by their distance from
// the smallest one (histogram, descending prefix, scatter into the upper half of the array), then every item
// counts the larger items of its bucket: its rank.  Buckets are small
// for anything but pathological inputs (which take the bitonic sort instead).  k <= TK_CAP / 2.
__device__ void tk_order(int k, TkShared &sh) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint64_t *grouped = sh.sort + TK_CAP / 2;
    // largest and smallest item
    uint64_t mx = 0ull, mn = ~0ull;
    for (int i = tid; i < k; i += TK_NT) {
        const uint64_t x = sh.sort[i];
        mx = x > mx ? x : mx;
        mn = x < mn ? x : mn;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint64_t a = __shfl_xor((unsigned long long)mx, o, 64), b = __shfl_xor((unsigned long long)mn, o, 64);
        mx = a > mx ? a : mx;
        mn = b < mn ? b : mn;
    }
    if (lane == 0) {
        grouped[2 * wave] = mx;
        grouped[2 * wave + 1] = mn;
    }
    __syncthreads();
    for (int w = 0; w < TK_NT / 64; ++w) {
        const uint64_t a = grouped[2 * w], b = grouped[2 * w + 1];
        mx = a > mx ? a : mx;
        mn = b < mn ? b : mn;
    }
    __syncthreads();
    // bucket = distance from the smallest item, scaled so that the largest item lands in the last bucket (bits of the
    // items themselves would not do: neighbours on either side of a power of two differ in every bit)
    const uint64_t range = mx - mn;
    const int bits = range ? 64 - __builtin_clzll(range) : 0;
    const int shift = bits > 11 ? bits - 11 : 0;
    for (int b = tid; b < TK_BINS; b += TK_NT) sh.hist[b] = 0u;
    __syncthreads();
    for (int i = tid; i < k; i += TK_NT) atomicAdd(&sh.hist[(uint32_t)((sh.sort[i] - mn) >> shift)], 1u);
    __syncthreads();
    // descending exclusive prefix: bucket b starts at the number of items in higher buckets; keep the counts
    constexpr int per = TK_BINS / TK_NT;
    uint32_t cnt[per], own = 0, big = 0;
#pragma unroll
    for (int q = 0; q < per; ++q) {
        cnt[q] = sh.hist[TK_BINS - 1 - (tid * per + q)];
        own += cnt[q];
        big = cnt[q] > big ? cnt[q] : big;
    }
    uint32_t run = tk_block_exclusive_scan(own, sh, nullptr);
#pragma unroll
    for (int q = 0; q < per; ++q) {
        const int b = TK_BINS - 1 - (tid * per + q);
        sh.hist[b] = run;               // start of the bucket; the scatter below advances it to the bucket's end
        sh.cnt16[b] = (uint16_t)cnt[q];
        run += cnt[q];
    }
    const bool pathological = __syncthreads_or(big > 1024u);
    if (pathological) {
        const int S = tk_pow2_ceil(k);
        for (int i = k + tid; i < S; i += TK_NT) sh.sort[i] = 0ull;
        __syncthreads();
        tk_sort_desc(sh.sort, S);
        return;
    }
    for (int i = tid; i < k; i += TK_NT) {
        const uint64_t x = sh.sort[i];
        grouped[atomicAdd(&sh.hist[(uint32_t)((x - mn) >> shift)], 1u)] = x;
    }
    __syncthreads();
    for (int i = tid; i < k; i += TK_NT) {
        const uint64_t x = grouped[i];
        const uint32_t b = (uint32_t)((x - mn) >> shift);
        const int end = (int)sh.hist[b], begin = end - (int)sh.cnt16[b];
        int rank = 0;
        for (int j = begin; j < end; ++j) rank += grouped[j] > x ? 1 : 0;
        sh.sort[begin + rank] = x;
    }
    __syncthreads();
}

// Exact top-k of src's items 0 .. n-1.  On return sh.sort[0 .. min(n, k)) holds them; in descending order if
// `sorted` is asked for, otherwise in no particular order.
template <class List> __device__ __forceinline__ void tk_select(const List &list, int k, TkShared &sh, bool sorted) {
    const int tid = threadIdx.x;
    const int n = list.n;
    if (n <= k) { // everything survives
        for (int i = tid; i < n; i += TK_NT) sh.sort[i] = list.src.item(i);
        __syncthreads();
        if (sorted) tk_order(n, sh);
        return;
    }
    // Items in play: (item >> hi) == prefix.  `need` of them are still to be taken, `taken` items lie above them.
    uint64_t prefix = 0, P = 0;
    uint32_t need = (uint32_t)k, taken = 0, in_bin = 0, above = 0;
    int hi = 63, lo = 63, lev = 0;
    bool ordered = false, settled = false;
    for (;; ++lev) { // passes over the list in memory, until the boundary bin fits the LDS array beside the items above it
        lo = tk_lo(lev);
        const int nb = 1 << (hi - lo);
        uint32_t *hist = lev == 0 ? (uint32_t *)sh.sort : sh.hist;
        for (int b = tid; b < nb; b += TK_NT) hist[b] = 0u;
        __syncthreads();
        const uint32_t bin_mask = (uint32_t)(nb - 1);
        if (lev == 0) { // all items are in play, the digit lies in the magnitude
            // Stretches of one value -- a constant or mostly-zero tensor -- would send all 64 atomics of an instruction to
            // one address; they show in the first vector of a batch, and then the wavefront merges its adds.
            // (If all of the list turns out to be one value, the magnitude is settled after this pass.)
            uint32_t ekey, eaux;
            const bool evalid = list.edge_item(&ekey, &eaux);
            uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
            bool mixed = false;
            if (tid == 0) {
                sh.kmin = 0xFFFFFFFFu;
                sh.kmax = 0u;
            }
            list.template batches<4>([&](const uint4 (&v)[4], int qb) {
                const uint32_t b0 = list.src.key_of(v[0], 0) >> 17, b1 = list.src.key_of(v[0], List::V - 1) >> 17;
                const uint32_t w0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)b0);
                const bool one_value = __builtin_amdgcn_ballot_w64(b0 == w0 && b1 == w0) == __builtin_amdgcn_ballot_w64(true);
                if (one_value) {
#pragma unroll
                    for (int u = 0; u < 4; ++u)
#pragma unroll
                        for (int e = 0; e < List::V; ++e) {
                            const bool valid = qb + u * TK_NT + tid < list.nq;
                            const uint32_t key = list.src.key_of(v[u], e);
                            tk_hist_add(valid, key >> 17, hist);
                            kmin = valid && key < kmin ? key : kmin;
                            kmax = valid && key > kmax ? key : kmax;
                        }
                } else {
                    mixed = true;
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        if (qb + u * TK_NT + tid < list.nq) {
#pragma unroll
                            for (int e = 0; e < List::V; ++e) atomicAdd(&hist[list.src.key_of(v[u], e) >> 17], 1u);
                        }
                    }
                }
            });
            if (evalid) {
                atomicAdd(&hist[ekey >> 17], 1u);
                kmin = ekey < kmin ? ekey : kmin;
                kmax = ekey > kmax ? ekey : kmax;
            }
            const bool uniform = __syncthreads_and(!mixed) != 0; // (also orders the initialisation of sh.kmin / sh.kmax)
            if (List::ORDERED && uniform) {
                if (kmin <= kmax) {
                    atomicMin(&sh.kmin, kmin);
                    atomicMax(&sh.kmax, kmax);
                }
            }
            settled = List::ORDERED && uniform;
        } else {
            list.scan([&](uint32_t key, uint32_t aux, bool valid) {
                const uint64_t item = ((uint64_t)key << 32) | aux;
                tk_hist_add(valid && (item >> hi) == prefix, (uint32_t)(item >> lo) & bin_mask, hist);
            });
        }
        __syncthreads();
        const uint32_t b_star = tk_find_bin(hist, nb, need, sh, &above, &in_bin);
        P = (prefix << (hi - lo)) | b_star;
        taken += above;
        need -= above;
        prefix = P;
        hi = lo;
        if (taken + in_bin <= TK_CAP || lo == 0) break; // (at lo == 0 the bin holds one item: items are distinct)
        if (lev == 0 && settled && sh.kmin == sh.kmax) { // one magnitude throughout: nothing lies above it
            P = sh.kmin;
            lo = hi = 32;
            ordered = true;
            break;
        }
        if (List::ORDERED && lo == 32) { // the magnitude is settled and more items share it than LDS holds
            ordered = true;
            break;
        }
    }
    if (ordered) {
        // Chunks of constant or mostly-zero tensors: the items above the magnitude T, then the first `need` items
        // equal to T in list order (= ascending index) -- one pass each instead of three more levels.
        const uint32_t T = (uint32_t)P;
        if (tid == 0) sh.count = 0u;
        __syncthreads();
        list.scan([&](uint32_t key, uint32_t aux, bool valid) {
            tk_append(valid && key > T, ((uint64_t)key << 32) | aux, sh.sort, &sh.count, 1);
        });
        uint32_t done = 0; // equal items seen so far (the same in every thread)
        auto place = [&](uint32_t flags, int i0) { // this thread's items i0 + e with bit e of flags set equal T
            uint32_t tot;
            uint32_t rank = done + tk_block_exclusive_scan((uint32_t)__builtin_popcount(flags), sh, &tot);
#pragma unroll
            for (int e = 0; e < List::V; ++e) {
                if ((flags >> e) & 1u) {
                    if (rank < need) sh.sort[taken + rank] = list.src.item(i0 + e);
                    ++rank;
                }
            }
            done += tot;
        };
        place(tid < list.head && list.src.key(tid) == T ? 1u : 0u, tid);
        for (int qb = 0; qb < list.nq && done < need; qb += TK_NT) {
            const int q = qb + tid;
            uint32_t flags = 0u;
            if (q < list.nq) {
                const uint4 v = list.src.loadv(list.head + q * List::V);
#pragma unroll
                for (int e = 0; e < List::V; ++e) flags |= (list.src.key_of(v, e) == T ? 1u : 0u) << e;
            }
            place(flags, list.head + q * List::V);
        }
        if (done < need) place(list.tail0 + tid < n && list.src.key(list.tail0 + tid) == T ? 1u : 0u, list.tail0 + tid);
        __syncthreads(); // sh.sort[0 .. k) is the top-k
        if (sorted) tk_order(k, sh);
        return;
    }
    if (tid == 0) sh.count = sh.count_tie = 0u;
    __syncthreads();
    tk_collect(list, lo, P, sh);
    __syncthreads();
    // The boundary bin now lies in sh.sort[TK_CAP - in_bin, TK_CAP); `need` of its items belong to the top-k.  The
    // selection goes on there, level by level, until the bin in play is needed whole; its members are then
    // recognised by (item >> lo) >= P.
    uint64_t *tie = sh.sort + TK_CAP - in_bin;
    const int n_tie = (int)in_bin;
    while (need < in_bin) {
        ++lev;
        lo = tk_lo(lev);
        const int nb = 1 << (hi - lo);
        for (int b = tid; b < nb; b += TK_NT) sh.hist[b] = 0u;
        __syncthreads();
        const uint32_t bin_mask = (uint32_t)(nb - 1);
        for (int i0 = 0; i0 < n_tie; i0 += TK_NT) {
            const int i = i0 + tid;
            const uint64_t item = i < n_tie ? tie[i] : 0ull;
            tk_hist_add(i < n_tie && (item >> hi) == prefix, (uint32_t)(item >> lo) & bin_mask, sh.hist);
        }
        __syncthreads();
        const uint32_t b_star = tk_find_bin(sh.hist, nb, need, sh, &above, &in_bin);
        P = (prefix << (hi - lo)) | b_star;
        need -= above; // the items above the new bin are taken: they satisfy (item >> lo) > P
        prefix = P;
        hi = lo;
        // at lo == 0 the bin holds a single item, so need == in_bin == 1 and the loop ends
    }
    // move the chosen members of the boundary bin up behind the items above it; the target range may reach into the
    // bin's own place at the end of the array, so the bin is read into registers first
    uint64_t mv[TK_CAP / TK_NT];
#pragma unroll
    for (int q = 0; q < TK_CAP / TK_NT; ++q) {
        const int i = q * TK_NT + tid;
        mv[q] = i < n_tie ? tie[i] : 0ull;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < TK_CAP / TK_NT; ++q) {
        const int i = q * TK_NT + tid;
        tk_append(i < n_tie && (mv[q] >> lo) >= P, mv[q], sh.sort, &sh.count, 1);
    }
    __syncthreads(); // sh.sort[0 .. k) is the top-k
    if (sorted) tk_order(k, sh);
}

// ------------------------------------------------------------------------------------------------
// The sampled path.  The paper's chunks hand on k items each, whatever the rest of the tensor looks like: 72 chunks of
// the largest tensor pass 170,000 items for 2,359 places.  A threshold that is known to lie below the tensor's k-th
// largest magnitude lets a chunk hand on only what can still matter, in ONE pass and without a selection of its own.
// Such a threshold comes from a sample: the r-th largest of TK_SAMPLE evenly spaced elements, r chosen so that about
// four times k elements of the tensor lie at or above it.  That count is n / TK_SAMPLE times a Gamma(r) variable
// whatever the values are (an order statistic of a sample), r >= 16: fewer than k for one tensor in 100,000.  It is
// not guaranteed, so it is checked: the final step sees how many items came, and if they are fewer than k, or more than
// a step can take (long runs of one magnitude), its workgroup runs the tensor's plain tree of selections itself.  The
// result is the same bits either way.
// ------------------------------------------------------------------------------------------------
__device__ void tk_threshold(const float *__restrict__ gt, uint32_t n, int r, uint64_t *aux, TkShared &sh) {
    // The r-th largest of the sampled magnitudes, to 22 of their 31 bits (two histogram levels of 11 bits; the threshold is
    // the lower edge of the bin it falls in, so a few more elements than r lie at or above it -- sorting the sample
    // took five times as long as everything else in this step).
    const int tid = threadIdx.x;
    uint32_t key[TK_SAMPLE / TK_NT];
#pragma unroll
    for (int q = 0; q < TK_SAMPLE / TK_NT; ++q) {
        const uint32_t idx = (uint32_t)(((uint64_t)(q * TK_NT + tid) * n) / TK_SAMPLE);
        key[q] = __float_as_uint(gt[idx]) & 0x7FFFFFFFu;
    }
    for (int b = tid; b < TK_BINS; b += TK_NT) sh.hist[b] = 0u;
    __syncthreads();
#pragma unroll
    for (int q = 0; q < TK_SAMPLE / TK_NT; ++q) atomicAdd(&sh.hist[key[q] >> 20], 1u);
    __syncthreads();
    uint32_t above, in_bin;
    const uint32_t b1 = tk_find_bin(sh.hist, TK_BINS, (uint32_t)r, sh, &above, &in_bin);
    for (int b = tid; b < TK_BINS; b += TK_NT) sh.hist[b] = 0u;
    __syncthreads();
#pragma unroll
    for (int q = 0; q < TK_SAMPLE / TK_NT; ++q)
        if ((key[q] >> 20) == b1) atomicAdd(&sh.hist[(key[q] >> 9) & (TK_BINS - 1)], 1u);
    __syncthreads();
    const uint32_t b2 = tk_find_bin(sh.hist, TK_BINS, (uint32_t)r - above, sh, &above, &in_bin);
    if (tid == 0) {
        aux[0] = (b1 << 20) | (b2 << 9);
        aux[1] = 0ull; // items of the tensor's list so far (low word), overflow mark (high word)
    }
}

// A chunk on the sampled path: its items with magnitude bits >= the tensor's threshold are appended to the tensor's
// list.  One pass over memory and almost nothing to keep (about 130 of 32,768 elements), so what matters is how many
// loads are in flight on a compute unit: four small workgroups per chunk, each with its whole piece requested at once.
#define TK_FILTER_NT 256
#define TK_FILTER_PIECES 4
#define TK_FILTER_CAP 2048 /* items a piece may keep (its share of what a chunk's array would hold) */
__global__ void __launch_bounds__(TK_FILTER_NT)
tk_filter_kernel(const float *__restrict__ g, const int64_t *__restrict__ plan, uint64_t *cand, int first_node) {
    __shared__ uint64_t kept[TK_FILTER_CAP];
    __shared__ uint32_t s_cnt, s_base;
    const int T_ = (int)plan[1];
    const int64_t *rec = plan + TK_HEADER + (int64_t)T_ * TK_TENSOR + (int64_t)(first_node + (int)blockIdx.x / TK_FILTER_PIECES) * TK_NODE;
    const int piece = (int)blockIdx.x % TK_FILTER_PIECES, tid = threadIdx.x;
    const int n = (int)rec[TK_N_ITEMS];
    const int per = ((n + TK_FILTER_PIECES - 1) / TK_FILTER_PIECES + 3) & ~3; // elements per piece, whole 16-byte vectors
    const int begin = piece * per, end = begin + per < n ? begin + per : n;
    uint64_t *aux = cand + rec[TK_N_AUX];
    const uint32_t thr = (uint32_t)aux[0];
    const float *p = g + rec[TK_N_SRC];
    const uint32_t first = (uint32_t)rec[TK_N_FIRST];
    if (tid == 0) s_cnt = 0u;
    __syncthreads();
    auto take = [&](uint32_t bits, int i) { // element i of the chunk
        const uint32_t key = bits & 0x7FFFFFFFu;
        if (key >= thr) {
            const uint32_t slot = atomicAdd(&s_cnt, 1u);
            if (slot < TK_FILTER_CAP) kept[slot] = ((uint64_t)key << 32) | (0xFFFFFFFFu - (first + (uint32_t)i));
        }
    };
    if (begin < end) {
        // elements before the first and after the last whole aligned vector one by one, the vectors eight per thread at once
        const int mis = (int)(((uintptr_t)(p + begin) & 15u) >> 2);
        int v0 = begin + ((4 - mis) & 3);
        if (v0 > end) v0 = end;
        const int nvec = (end - v0) >> 2, v1 = v0 + nvec * 4;
        for (int i = begin + tid; i < v0; i += TK_FILTER_NT) take(__float_as_uint(p[i]), i);
        for (int i = v1 + tid; i < end; i += TK_FILTER_NT) take(__float_as_uint(p[i]), i);
        for (int q0 = 0; q0 < nvec; q0 += 8 * TK_FILTER_NT) {
            uint4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int q = q0 + u * TK_FILTER_NT + tid;
                v[u] = q < nvec ? *(const uint4 *)(p + v0 + 4 * q) : make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int q = q0 + u * TK_FILTER_NT + tid;
                if (q < nvec) {
                    take(v[u].x, v0 + 4 * q);
                    take(v[u].y, v0 + 4 * q + 1);
                    take(v[u].z, v0 + 4 * q + 2);
                    take(v[u].w, v0 + 4 * q + 3);
                }
            }
        }
    }
    __syncthreads();
    const uint32_t cnt = s_cnt;
    uint32_t *aux32 = (uint32_t *)(aux + 1); // [0] items of the tensor's list so far, [1] overflow mark
    if (cnt > TK_FILTER_CAP) { // a run of one magnitude at the threshold: the final step will take the plain tree
        if (tid == 0) atomicOr(&aux32[1], 1u);
        return;
    }
    if (cnt == 0u) return;
    if (tid == 0) s_base = atomicAdd(&aux32[0], cnt);
    __syncthreads();
    const uint32_t base = s_base;
    if (base + cnt > TK_NODE_CAP) {
        if (tid == 0) atomicOr(&aux32[1], 1u);
        return;
    }
    uint64_t *region = cand + rec[TK_N_OUT];
    for (uint32_t i = tid; i < cnt; i += TK_FILTER_NT) region[base + i] = kept[i];
}

// one step: a selection (from a chunk of gradients or from survivors), or the threshold of a sampled path
// (returns true when it was the final step of a sampled path and the sample had misled: nothing is written then)
__device__ __forceinline__ bool tk_run_node(const int64_t *__restrict__ rec, const float *__restrict__ g, uint64_t *cand,
                                            int32_t *__restrict__ out_idx, float *__restrict__ out_val, TkShared &sh) {
    const int flags = (int)rec[TK_N_FLAGS];
    if (flags & TK_F_THRESH) {
        tk_threshold(g + rec[TK_N_GBEGIN], (uint32_t)rec[TK_N_GN], (int)rec[TK_N_K], cand + rec[TK_N_AUX], sh);
        return false;
    }
    int n = (int)rec[TK_N_ITEMS];
    const int k = (int)rec[TK_N_K];
    if (flags & TK_F_COUNTED) {
        uint32_t *aux32 = (uint32_t *)(cand + rec[TK_N_AUX] + 1);
        const uint32_t cnt = aux32[0], overflow = aux32[1];
        if (overflow != 0u || cnt < (uint32_t)k || cnt > (uint32_t)TK_NODE_CAP) return true; // the sample misled
        n = (int)cnt;
    }
    const bool final_step = flags & TK_F_FINAL;
    if (flags & TK_F_LEAF) {
        TkSrcGrad src;
        src.g = g + rec[TK_N_SRC];
        src.first = (uint32_t)rec[TK_N_FIRST];
        TkList<TkSrcGrad> list;
        list.init(src, n);
        tk_select(list, k, sh, final_step);
    } else {
        TkSrcItems src;
        src.c = cand + rec[TK_N_SRC];
        TkList<TkSrcItems> list;
        list.init(src, n);
        tk_select(list, k, sh, final_step);
    }
    const int keep = n < k ? n : k; // (a final step has n >= k)
    const int64_t o = rec[TK_N_OUT];
    if (final_step) {
        const float *gt = g + rec[TK_N_GBEGIN];
        const uint32_t gn = (uint32_t)rec[TK_N_GN];
        for (int r = threadIdx.x; r < keep; r += TK_NT) {
            const uint32_t idx = 0xFFFFFFFFu - (uint32_t)sh.sort[r];
            out_idx[o + r] = (int32_t)idx;
            out_val[o + r] = idx < gn ? gt[idx] : 0.f; // (always inside: items carry indices of this tensor)
        }
    } else {
        for (int r = threadIdx.x; r < keep; r += TK_NT) cand[o + r] = sh.sort[r];
    }
    return false;
}

// The plain tree of a tensor whose sample misled, run by the workgroup of the sampled path's final step: its steps one
// after the other (each reads what the one before wrote).  Out of line: it is hardly ever run, and inlined its loop
// costs the steps that are run their registers.
__device__ __noinline__ void tk_plain_tree(const int64_t *nodes, const int64_t *fin, const float *g, uint64_t *cand, int32_t *out_idx,
                                           float *out_val, TkShared &sh) {
    const int64_t *rec = nodes + fin[TK_N_FB_FIRST] * TK_NODE;
    for (int64_t s = 0; s < fin[TK_N_FB_COUNT]; ++s, rec += TK_NODE) {
        tk_run_node(rec, g, cand, out_idx, out_val, sh);
        __threadfence_block();
        __syncthreads();
    }
}

// one step of the tree: one workgroup per node of the level
__global__ void __launch_bounds__(TK_NT)
tk_node_kernel(const float *__restrict__ g, const int64_t *__restrict__ plan, uint64_t *cand, int32_t *__restrict__ out_idx,
               float *__restrict__ out_val, int first_node) {
    __shared__ TkShared sh;
    const int T = (int)plan[1];
    const int64_t *nodes = plan + TK_HEADER + (int64_t)T * TK_TENSOR;
    const int64_t *rec = nodes + (int64_t)(first_node + blockIdx.x) * TK_NODE;
    if (tk_run_node(rec, g, cand, out_idx, out_val, sh)) tk_plain_tree(nodes, rec, g, cand, out_idx, out_val, sh);
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
struct TkNode {
    int64_t src, items, k, out, flags, first, gbegin, gn;
    int level;              // launch it belongs to; -1: a step of a plain tree that only a sampled path's final step may run
    int64_t aux;            // sampled path: the tensor's two workspace words
    int64_t fb_first, fb_count, tensor;
};

static int64_t tk_plan_build(const int64_t *offsets, const int32_t *k, int T, int chunks, int64_t *plan, int64_t plan_capacity);

extern "C" int64_t grad_topk_plan(const int64_t *offsets, const int32_t *k, int T, int chunks, int64_t *plan,
                                  int64_t plan_capacity) {
    if (!offsets || !k || T < 1 || chunks < 0) return -(int64_t)KS_INVALID_ARG;
    try {
        return tk_plan_build(offsets, k, T, chunks, plan, plan_capacity);
    } catch (...) { // out of host memory while laying out the plan: nothing may escape through the C ABI
        return -(int64_t)KS_UNSUPPORTED;
    }
}

// rank of the sampled path's threshold in the sample, or 0 when the tensor takes the plain tree: about four times k
// elements of the tensor are then expected at or above the threshold, and three times that expectation must fit the
// final step's input and, per chunk, the array a chunk's workgroup collects in
static int tk_sample_rank(int64_t n, int64_t k, int64_t M, int chunks) {
    if (chunks != 0 || M < 2 || n <= 8 * TK_SAMPLE) return 0;
    int64_t r = (4 * k * TK_SAMPLE + n - 1) / n;
    if (r < TK_SAMPLE_RANK) r = TK_SAMPLE_RANK;
    const int64_t expect = r * n / TK_SAMPLE;
    if (r > TK_SAMPLE / 8 || 3 * expect > TK_NODE_CAP || 3 * expect / M > TK_CAP) return 0;
    return (int)r;
}

static int64_t tk_plan_build(const int64_t *offsets, const int32_t *k, int T, int chunks, int64_t *plan, int64_t plan_capacity) {
    std::vector<TkNode> nodes;
    std::vector<int64_t> tensors;
    int64_t cand = 0, out = 0;
    int n_levels = 0;
    for (int t = 0; t < T; ++t) {
        const int64_t n = offsets[t + 1] - offsets[t];
        if (n < 1 || n >= ((int64_t)1 << 31) || k[t] < 1 || k[t] > n) return -(int64_t)KS_INVALID_ARG;
        if (k[t] > KS_TOPK_MAX_K) return -(int64_t)KS_UNSUPPORTED;
        int64_t M = chunks > 0 ? (chunks < n ? (int64_t)chunks : n) : (n + TK_LEAF - 1) / TK_LEAF;
        const int64_t chunk = (n + M - 1) / M;
        M = (n + chunk - 1) / chunk; // no empty chunks
        const int rank = tk_sample_rank(n, k[t], M, chunks);
        // the plain tree.  The lists of the current level: (offset, items) of each; level 0 = the chunks of the tensor
        std::vector<TkNode> cur, tree;
        for (int64_t j = 0; j < M; ++j) {
            TkNode nd = {offsets[t] + j * chunk, (j + 1) * chunk < n ? chunk : n - j * chunk, k[t], 0, TK_F_LEAF, j * chunk, offsets[t], n, 0,
                         0, 0, 0, t};
            cur.push_back(nd);
        }
        int level = 0;
        for (;;) {
            if (cur.size() == 1) { // the last step of the tensor
                cur[0].flags |= TK_F_FINAL;
                cur[0].out = out;
                tree.push_back(cur[0]);
                break;
            }
            // the nodes of this level hand their survivors on, back to back in the workspace
            int64_t total = 0;
            for (auto &nd : cur) {
                nd.out = cand + total;
                total += nd.items < nd.k ? nd.items : nd.k;
                tree.push_back(nd);
            }
            // next level: as few steps as the input limit allows (at least two lists each)
            int64_t G = TK_NODE_CAP / k[t];
            if (G < 2) G = 2;
            if (total <= TK_NODE_CAP) G = (int64_t)cur.size();
            std::vector<TkNode> next;
            for (size_t a = 0; a < cur.size(); a += (size_t)G) {
                const size_t b = a + (size_t)G < cur.size() ? a + (size_t)G : cur.size();
                int64_t items = 0;
                for (size_t c = a; c < b; ++c) items += cur[c].items < cur[c].k ? cur[c].items : cur[c].k;
                TkNode nd = {cur[a].out, items, k[t], 0, 0, 0, offsets[t], n, level + 1, 0, 0, 0, t};
                next.push_back(nd);
            }
            cand += total;
            cur.swap(next);
            ++level;
            if (level >= TK_MAX_LEVELS) return -(int64_t)KS_UNSUPPORTED;
        }
        int steps = level + 1;
        if (rank > 0) {
            // the sampled path in front: threshold, one filter per chunk, final step; the plain tree stays in the plan
            // for the final step's workgroup to fall back on
            for (auto &nd : tree) nd.level = -1;
            const int64_t aux = cand, region = cand + 2;
            cand += 2 + TK_NODE_CAP;
            TkNode th = {0, n, rank, 0, TK_F_THRESH, 0, offsets[t], n, 0, aux, 0, 0, t};
            nodes.push_back(th);
            for (int64_t j = 0; j < M; ++j) {
                TkNode nd = {offsets[t] + j * chunk, (j + 1) * chunk < n ? chunk : n - j * chunk, k[t], region, TK_F_LEAF | TK_F_FILTER,
                             j * chunk, offsets[t], n, 1, aux, 0, 0, t};
                nodes.push_back(nd);
            }
            TkNode fin = {region, TK_NODE_CAP, k[t], out, TK_F_FINAL | TK_F_COUNTED, 0, offsets[t], n, 2, aux, 0, (int64_t)tree.size(), t};
            nodes.push_back(fin);
            steps = 3;
        }
        for (auto &nd : tree) nodes.push_back(nd);
        if (steps > n_levels) n_levels = steps;
        tensors.push_back(n);
        tensors.push_back(k[t]);
        tensors.push_back(M);
        tensors.push_back(steps);
        out += k[t];
    }
    // Tensors of one step are independent of everything else: with sampled paths in the plan they run beside those
    // paths' final steps (the launch that otherwise has the fewest workgroups) instead of beside the thresholds.
    bool sampled = false;
    for (const TkNode &nd : nodes) sampled = sampled || (nd.flags & TK_F_THRESH);
    if (sampled)
        for (TkNode &nd : nodes)
            if (nd.level == 0 && (nd.flags & TK_F_LEAF) && (nd.flags & TK_F_FINAL)) nd.level = n_levels - 1;
    int64_t n_launched = 0;
    for (const TkNode &nd : nodes) n_launched += nd.level >= 0;
    const int64_t n_nodes = (int64_t)nodes.size();
    if (n_nodes >= ((int64_t)1 << 31)) return -(int64_t)KS_UNSUPPORTED;
    const int64_t words = TK_HEADER + (int64_t)T * TK_TENSOR + n_nodes * TK_NODE;
    if (!plan || plan_capacity < words) return words;
    for (int64_t i = 0; i < TK_HEADER; ++i) plan[i] = 0;
    plan[0] = TK_MAGIC;
    plan[1] = T;
    plan[2] = n_launched;
    plan[3] = cand > 0 ? cand : 1;
    plan[4] = out;
    plan[5] = offsets[T] - offsets[0];
    plan[6] = n_levels;
    plan[7] = n_nodes;
    for (size_t i = 0; i < tensors.size(); ++i) plan[TK_HEADER + (int64_t)i] = tensors[i];
    int64_t *nrec = plan + TK_HEADER + (int64_t)T * TK_TENSOR;
    int64_t w = 0;
    auto put = [&](const TkNode &nd) {
        int64_t *r = nrec + w * TK_NODE;
        for (int q = 0; q < TK_NODE; ++q) r[q] = 0;
        r[TK_N_SRC] = nd.src;
        r[TK_N_ITEMS] = nd.items;
        r[TK_N_K] = nd.k;
        r[TK_N_OUT] = nd.out;
        r[TK_N_FLAGS] = nd.flags;
        r[TK_N_FIRST] = nd.first;
        r[TK_N_GBEGIN] = nd.gbegin;
        r[TK_N_GN] = nd.gn;
        r[TK_N_AUX] = nd.aux;
        r[TK_N_FB_COUNT] = nd.fb_count;
        ++w;
    };
    for (int lev = 0; lev < n_levels; ++lev) { // launched nodes level by level, tensors in order inside a level; the filter
        plan[8 + 2 * lev] = w;                 // and final steps of the sampled paths first in theirs (kernels of their own)
        const int64_t special = lev == 1 ? TK_F_FILTER : (lev == 2 ? TK_F_COUNTED : 0);
        for (const TkNode &nd : nodes)
            if (nd.level == lev && (nd.flags & special)) put(nd);
        if (special) {
            plan[lev == 1 ? 28 : 30] = plan[8 + 2 * lev];
            plan[lev == 1 ? 29 : 31] = w - plan[8 + 2 * lev];
        }
        for (const TkNode &nd : nodes)
            if (nd.level == lev && !(nd.flags & special)) put(nd);
        plan[9 + 2 * lev] = w - plan[8 + 2 * lev];
    }
    // then the plain trees behind sampled paths, tensor by tensor, each in the order of its levels
    std::vector<int64_t> fb_first((size_t)T, 0);
    for (int t = 0; t < T; ++t) {
        fb_first[(size_t)t] = w;
        for (const TkNode &nd : nodes)
            if (nd.level < 0 && nd.tensor == t) put(nd);
    }
    for (int64_t i = 0; i < n_launched; ++i) { // the final steps of the sampled paths learn where their trees are
        int64_t *r = nrec + i * TK_NODE;
        if (r[TK_N_FLAGS] & TK_F_COUNTED) {
            for (int t = 0; t < T; ++t)
                if (offsets[t] == r[TK_N_GBEGIN] && r[TK_N_GN] == offsets[t + 1] - offsets[t]) r[TK_N_FB_FIRST] = fb_first[(size_t)t];
        }
    }
    return words;
}

static bool tk_plan_ok(const int64_t *p) {
    return p && p[0] == TK_MAGIC && p[1] >= 1 && p[2] >= p[1] && p[3] >= 1 && p[4] >= 1 && p[6] >= 1 && p[6] <= TK_MAX_LEVELS &&
           p[7] >= p[2] && p[29] >= 0 && p[31] >= 0 && p[29] <= p[2] && p[31] <= p[2];
}

extern "C" size_t grad_topk_workspace(const int64_t *plan_host) {
    if (!tk_plan_ok(plan_host)) return 0;
    return ks_align_up((size_t)plan_host[3] * sizeof(uint64_t), 256);
}

extern "C" int grad_topk_select(const float *g, const int64_t *plan_dev, const int64_t *plan_host, int32_t *out_idx,
                                float *out_val, void *ws, size_t ws_bytes, void *stream) {
    if (!g || !plan_dev || !out_idx || !out_val || !ws || !tk_plan_ok(plan_host)) return KS_INVALID_ARG;
    if (ws_bytes < grad_topk_workspace(plan_host)) return KS_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)stream;
    uint64_t *cand = (uint64_t *)ws;
    for (int lev = 0; lev < (int)plan_host[6]; ++lev) {
        int64_t first = plan_host[8 + 2 * lev], count = plan_host[9 + 2 * lev];
        if (lev == 1 && plan_host[29] > 0) { // the chunks of the sampled paths
            hipLaunchKernelGGL(tk_filter_kernel, dim3((unsigned)(plan_host[29] * TK_FILTER_PIECES)), dim3(TK_FILTER_NT), 0, st, g,
                               plan_dev, cand, (int)first);
            first += plan_host[29];
            count -= plan_host[29];
        }
        if (count < 1) continue;
        hipLaunchKernelGGL(tk_node_kernel, dim3((unsigned)count), dim3(TK_NT), 0, st, g, plan_dev, cand, out_idx, out_val,
                           (int)first);
    }
    KS_LAUNCH_CHECK();
    return KS_OK;
}
