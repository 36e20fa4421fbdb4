// Layer-wise top-k selection for gradient sparsification (Section 3.3.2: divide-and-conquer top-k selection,
// tensors grouped into one launch).
//
// Both steps of the method are the same workgroup-level routine, tk_select: the exact top-k of a list of items
// that sits in global memory (step 1: a chunk of a gradient tensor; step 2: the survivors of all chunks of a
// tensor).  An item is the 64-bit word  (bits of |g|) << 32 | (0xFFFFFFFF - index) : larger word = larger
// magnitude, equal magnitudes ordered by ascending index, all words distinct, so "top-k" is unique.
//
// tk_select (512 threads):
//   1. histogram of the top 11 bits of the magnitude (sign dropped: exponent and three mantissa bits) in LDS;
//      a descending scan finds the bin b in which the k-th largest item falls;
//   2. if the items above b plus the items in b fit the LDS sort array (8,192 words), they are all collected and
//      sorted there (bitonic, descending): the first k words are the answer, already in output order.  For
//      gradient-like data this is the path taken: the list is read twice (it sits in L2 after the first pass);
//   3. otherwise the bin is refined by two more histogram passes over the next 11 and the last 9 bits, restricted
//      to the items that share the prefix found so far, until the candidates fit -- or until the k-th magnitude
//      itself is known exactly and still has too many equals (constant or mostly-zero tensors): then the items
//      above it are collected, and of the equal ones the first in list order, which is ascending index order in
//      both steps (the survivors of a chunk are stored sorted, chunks in order).
// Everything is integer work: the result is bit-exact and deterministic.
#include "ks_common.h"
#include "../../include/grad_topk.h"

#define TK_NT 512
#define TK_BINS 2048
#define TK_CAP 8192
#define TK_MIN_CHUNK 8192
#define TK_MAX_AUTO_CHUNKS 256
#define TK_MAGIC 0x6B706F74646172ll /* "gradtopk" cut to seven bytes */
#define TK_HEADER 8
#define TK_RECORD 8

// plan record of a tensor (int64 words)
enum { TK_R_BEGIN = 0, TK_R_N, TK_R_K, TK_R_M, TK_R_CHUNK, TK_R_CAND_OFF, TK_R_OUT_OFF, TK_R_KC };

struct TkShared {
    uint64_t sort[TK_CAP];
    uint32_t hist[TK_BINS];
    uint32_t wave_sum[TK_NT / 64];
    uint32_t b_star, above, count;
};

// step 1 reads a chunk of a gradient tensor; index of item i within the tensor = first + i
struct TkSrcGrad {
    const float *g;
    uint32_t first;
    __device__ __forceinline__ uint32_t key(int i) const { return __float_as_uint(g[i]) & 0x7FFFFFFFu; }
    __device__ __forceinline__ uint64_t item(int i) const { return ((uint64_t)key(i) << 32) | (0xFFFFFFFFu - (first + (uint32_t)i)); }
};
// step 2 reads the survivors
struct TkSrcItems {
    const uint64_t *c;
    __device__ __forceinline__ uint32_t key(int i) const { return ((const uint32_t *)c)[2 * (int64_t)i + 1]; }
    __device__ __forceinline__ uint64_t item(int i) const { return c[i]; }
};

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

// append `item` to sh.sort for the lanes with sel set: one LDS atomic per wavefront, not per item
__device__ __forceinline__ void tk_append(bool sel, uint64_t item, TkShared &sh) {
    const uint64_t m = __builtin_amdgcn_ballot_w64(sel);
    if (m == 0ull) return;
    const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
    uint32_t base = 0u;
    if (sel && rank == 0u) base = atomicAdd(&sh.count, (uint32_t)__builtin_popcountll(m));
    base = (uint32_t)__shfl((int)base, __builtin_ctzll(m), 64);
    if (sel && base + rank < TK_CAP) sh.sort[base + rank] = item; // always inside: the caller has counted
}

// bitonic sort of sh.sort[0 .. S) in descending order, S a power of two >= 2
__device__ __forceinline__ void tk_sort_desc(TkShared &sh, int S) {
    for (int size = 2; size <= S; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int p = threadIdx.x; p < (S >> 1); p += TK_NT) {
                const int i = 2 * p - (p & (stride - 1)), j = i + stride;
                const uint64_t a = sh.sort[i], b = sh.sort[j];
                const bool desc = (i & size) == 0;
                if ((a < b) == desc) {
                    sh.sort[i] = b;
                    sh.sort[j] = a;
                }
            }
            __syncthreads();
        }
    }
}

// Exact top-k of src's items 0 .. n-1.  On return sh.sort[0 .. min(n, k)) holds them in descending order.
template <class Src> __device__ void tk_select(const Src &src, int n, int k, TkShared &sh, bool presorted) {
    const int tid = threadIdx.x;
    int count;
    if (n <= k) { // everything survives
        for (int i = tid; i < n; i += TK_NT) sh.sort[i] = src.item(i);
        count = n;
        if (presorted) {
            __syncthreads();
            return;
        }
    } else {
        // items in play: (key >> hi) == prefix.  `need` of them are still to be taken, `taken` lie above them.
        uint32_t prefix = 0, need = (uint32_t)k, taken = 0, P = 0, in_bin = 0;
        int hi = 31, lo = 31;
        bool fits = false;
        for (int lev = 0; lev < 3 && !fits; ++lev) {
            lo = lev == 0 ? 20 : (lev == 1 ? 9 : 0);
            const int nb = 1 << (hi - lo);
            for (int b = tid; b < nb; b += TK_NT) sh.hist[b] = 0u;
            if (tid == 0) sh.b_star = sh.above = 0u; // (always overwritten below: at least `need` items are in play)
            __syncthreads();
            for (int i0 = 0; i0 < n; i0 += 4 * TK_NT) {
                uint32_t key[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = i0 + u * TK_NT + tid;
                    key[u] = i < n ? src.key(i) : 0xFFFFFFFFu; // bit 31 set: never in play
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if ((key[u] >> hi) == prefix) atomicAdd(&sh.hist[(key[u] >> lo) & (uint32_t)(nb - 1)], 1u);
            }
            __syncthreads();
            // thread t owns bins nb-1 - t*per ... downwards: scan in descending bin order
            const int per = nb / TK_NT > 0 ? nb / TK_NT : 1;
            uint32_t own = 0;
            if (tid * per < nb)
                for (int q = 0; q < per; ++q) own += sh.hist[nb - 1 - (tid * per + q)];
            uint32_t run = tk_block_exclusive_scan(own, sh, nullptr);
            if (tid * per < nb) {
                for (int q = 0; q < per; ++q) {
                    const int b = nb - 1 - (tid * per + q);
                    const uint32_t h = sh.hist[b];
                    if (run < need && need <= run + h) { // exactly one bin
                        sh.b_star = (uint32_t)b;
                        sh.above = run;
                    }
                    run += h;
                }
            }
            __syncthreads();
            const uint32_t b_star = sh.b_star, above = sh.above;
            in_bin = sh.hist[b_star];
            P = (prefix << (hi - lo)) | b_star;
            taken += above;
            need -= above;
            fits = taken + in_bin <= TK_CAP;
            prefix = P;
            hi = lo;
            __syncthreads();
        }
        if (tid == 0) sh.count = 0u;
        __syncthreads();
        if (fits) { // everything at or above the boundary bin: (key >> lo) >= P
            for (int i0 = 0; i0 < n; i0 += 4 * TK_NT) {
                uint32_t key[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = i0 + u * TK_NT + tid;
                    key[u] = i < n ? src.key(i) : 0u;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = i0 + u * TK_NT + tid;
                    const bool sel = i < n && (key[u] >> lo) >= P;
                    tk_append(sel, sel ? src.item(i) : 0ull, sh);
                }
            }
            count = (int)(taken + in_bin);
        } else {
            // lo == 0: P is the k-th magnitude itself and more items equal it than the sort array holds.
            // Larger ones first (any order), then the first `need` equal ones in list order.
            for (int i0 = 0; i0 < n; i0 += TK_NT) {
                const int i = i0 + tid;
                const bool sel = i < n && src.key(i) > P;
                tk_append(sel, sel ? src.item(i) : 0ull, sh);
            }
            uint32_t done = 0; // equal items placed so far (uniform over the workgroup)
            for (int i0 = 0; i0 < n && done < need; i0 += TK_NT) {
                const int i = i0 + tid;
                const bool eq = i < n && src.key(i) == P;
                uint32_t tot;
                const uint32_t rank = done + tk_block_exclusive_scan(eq ? 1u : 0u, sh, &tot);
                if (eq && rank < need) sh.sort[taken + rank] = src.item(i);
                done += tot;
            }
            count = k;
        }
    }
    __syncthreads();
    int S = 2;
    while (S < count) S <<= 1;
    for (int i = count + tid; i < S; i += TK_NT) sh.sort[i] = 0ull; // below every item
    __syncthreads();
    tk_sort_desc(sh, S);
}

// step 1: one workgroup per chunk
__global__ void __launch_bounds__(TK_NT)
tk_chunk_kernel(const float *__restrict__ g, const int64_t *__restrict__ plan, uint64_t *__restrict__ cand) {
    __shared__ TkShared sh;
    const int T = (int)plan[1];
    const int64_t w = plan[TK_HEADER + (int64_t)T * TK_RECORD + blockIdx.x];
    const int t = (int)(w >> 32), j = (int)(w & 0xFFFFFFFFll);
    const int64_t *rec = plan + TK_HEADER + (int64_t)t * TK_RECORD;
    const int64_t n = rec[TK_R_N], chunk = rec[TK_R_CHUNK];
    const int k = (int)rec[TK_R_K], kc = (int)rec[TK_R_KC];
    const int64_t a = (int64_t)j * chunk;
    const int len = (int)((a + chunk < n ? a + chunk : n) - a);
    TkSrcGrad src;
    src.g = g + rec[TK_R_BEGIN] + a;
    src.first = (uint32_t)a;
    tk_select(src, len, k, sh, false);
    const int keep = len < k ? len : k;
    uint64_t *out = cand + rec[TK_R_CAND_OFF] + (int64_t)j * kc;
    for (int r = threadIdx.x; r < keep; r += TK_NT) out[r] = sh.sort[r];
}

// step 2: one workgroup per tensor
__global__ void __launch_bounds__(TK_NT)
tk_final_kernel(const float *__restrict__ g, const int64_t *__restrict__ plan, const uint64_t *__restrict__ cand,
                int32_t *__restrict__ out_idx, float *__restrict__ out_val) {
    __shared__ TkShared sh;
    const int t = blockIdx.x;
    const int64_t *rec = plan + TK_HEADER + (int64_t)t * TK_RECORD;
    const int64_t n = rec[TK_R_N], chunk = rec[TK_R_CHUNK], M = rec[TK_R_M];
    const int k = (int)rec[TK_R_K], kc = (int)rec[TK_R_KC];
    const int64_t last_len = n - (M - 1) * chunk;
    const int n_cand = (int)((M - 1) * kc + (last_len < k ? last_len : k));
    TkSrcItems src;
    src.c = cand + rec[TK_R_CAND_OFF];
    tk_select(src, n_cand, k, sh, M == 1); // a single chunk's survivors are the answer, already in order
    const float *gt = g + rec[TK_R_BEGIN];
    const int64_t o = rec[TK_R_OUT_OFF];
    for (int r = threadIdx.x; r < k; r += TK_NT) {
        const uint32_t idx = 0xFFFFFFFFu - (uint32_t)sh.sort[r];
        out_idx[o + r] = (int32_t)idx;
        out_val[o + r] = gt[idx];
    }
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
extern "C" int64_t grad_topk_plan(const int64_t *offsets, const int32_t *k, int T, int chunks, int64_t *plan,
                                  int64_t plan_capacity) {
    if (!offsets || !k || T < 1 || chunks < 0) return -(int64_t)KS_INVALID_ARG;
    int64_t W1 = 0;
    for (int pass = 0; pass < 2; ++pass) {
        int64_t cand = 0, out = 0, w = 0;
        for (int t = 0; t < T; ++t) {
            const int64_t n = offsets[t + 1] - offsets[t];
            if (n < 1 || n >= ((int64_t)1 << 31) || k[t] < 1 || k[t] > n) return -(int64_t)KS_INVALID_ARG;
            if (k[t] > KS_TOPK_MAX_K) return -(int64_t)KS_UNSUPPORTED;
            int64_t M;
            if (chunks > 0) {
                M = chunks < n ? chunks : n;
            } else {
                M = 1;
                while (M < TK_MAX_AUTO_CHUNKS && (M + 1) * (M + 1) * (int64_t)k[t] <= n) ++M;                   // floor(sqrt(n / k))
                if ((2 * M + 1) * (2 * M + 1) * (int64_t)k[t] <= 4 * n) ++M;            // to nearest
                if (M > n / TK_MIN_CHUNK) M = n / TK_MIN_CHUNK;
                if (M > TK_MAX_AUTO_CHUNKS) M = TK_MAX_AUTO_CHUNKS;
                if (M < 1) M = 1;
            }
            const int64_t chunk = (n + M - 1) / M;
            M = (n + chunk - 1) / chunk; // no empty chunks
            const int64_t kc = k[t] < chunk ? k[t] : chunk;
            if (pass == 1) {
                int64_t *rec = plan + TK_HEADER + (int64_t)t * TK_RECORD;
                rec[TK_R_BEGIN] = offsets[t];
                rec[TK_R_N] = n;
                rec[TK_R_K] = k[t];
                rec[TK_R_M] = M;
                rec[TK_R_CHUNK] = chunk;
                rec[TK_R_CAND_OFF] = cand;
                rec[TK_R_OUT_OFF] = out;
                rec[TK_R_KC] = kc;
                for (int64_t j = 0; j < M; ++j) plan[TK_HEADER + (int64_t)T * TK_RECORD + w + j] = ((int64_t)t << 32) | j;
            }
            cand += M * kc;
            out += k[t];
            w += M;
        }
        if (w >= ((int64_t)1 << 31)) return -(int64_t)KS_UNSUPPORTED;
        if (pass == 0) {
            W1 = w;
            const int64_t words = TK_HEADER + (int64_t)T * TK_RECORD + W1;
            if (!plan || plan_capacity < words) return words;
        } else {
            plan[0] = TK_MAGIC;
            plan[1] = T;
            plan[2] = W1;
            plan[3] = cand;
            plan[4] = out;
            plan[5] = offsets[T] - offsets[0];
            plan[6] = plan[7] = 0;
        }
    }
    return TK_HEADER + (int64_t)T * TK_RECORD + W1;
}

static bool tk_plan_ok(const int64_t *p) { return p && p[0] == TK_MAGIC && p[1] >= 1 && p[2] >= p[1] && p[3] >= 1 && p[4] >= 1; }

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
    hipLaunchKernelGGL(tk_chunk_kernel, dim3((unsigned)plan_host[2]), dim3(TK_NT), 0, st, g, plan_dev, cand);
    hipLaunchKernelGGL(tk_final_kernel, dim3((unsigned)plan_host[1]), dim3(TK_NT), 0, st, g, plan_dev, cand, out_idx, out_val);
    KS_LAUNCH_CHECK();
    return KS_OK;
}
