// Exact KNN graph of the class-weight rows (paper Section 3.2.2: linear search with inner-product
// similarity; 16-bit matrix-core pass that recalls k' > K candidates, then an exact re-rank).
//
//   prepare   bf16 copy of W when the input is fp32; row norms and their maximum (for the error bound)
//   recall    each workgroup owns a block of rows (256 in the sweep kernel) and passes all rows of W by them: bf16
//             MFMA tiles of similarities; an element that beats its row's threshold is appended to that row's candidate
//             buffer; a full buffer is cut back to its k' best by a wavefront (a bitwise search for the
//             k'-th largest key), which also raises the threshold.  The C x C similarities are never stored.
//             Large problems (D = 128, 256, 512, K <= 64) take the variant that computes every similarity once and
//             uses it for both rows of the pair, with thresholds fixed beforehand from a sample of the rows (gr_sym_*).
//   re-rank   one wavefront per row: canonical fp64 similarity of the k' candidates, exact order
//             (similarity descending, id ascending), first K written out.  The row is certified when
//             the K-th exact similarity exceeds the recall threshold by more than the error bound of the
//             matrix-core pass; otherwise the row goes to the exhaustive list.
//   exhaustive  uncertified rows are searched over all C columns in canonical fp64 arithmetic.
// Every decision that reaches the output is taken on the canonical fp64 similarity, so the lists are
// exact and do not depend on scheduling.
#include "ks_gemm.h"
#include "ks_gemm_async.h"
#include "ks_gemm_soe.h"

typedef KsTile<128, 128, 64, 2, 2> TileR;       // generic recall tile (any D % 32 == 0)
typedef KsATile<256, 256, 2, 4, 2> TileRA;      // asynchronous recall tile (D % 64 == 0)

#define GR_NT 256
#define GR_FB_BLOCKS 64   /* workgroups (and fp64 scratch rows) of the exhaustive pass */
#define GR_MAX_D 4096     /* the exhaustive pass keeps one row in LDS as fp64 */

__device__ __forceinline__ uint32_t gr_orderable(float f) {
    const uint32_t u = __float_as_uint(f); // negative: all bits flipped; otherwise: the sign bit set
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
}
__device__ __forceinline__ float gr_unorder(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

// The two sides of a recall pass: the rows whose neighbours are searched (resident in the workgroups) and the rows
// that are searched (streamed past them).  The graph build searches W in W; one hop of the distributed build
// searches the node's rows in a visiting shard.
struct GrPair {
    const uint16_t *R; // [Cr, D]
    int64_t Cr;
    const uint16_t *S; // [Cs, D]
    int64_t Cs;
    int64_t self;      // streamed row i + self is resident row i itself and is skipped
};

struct GrParams {
    int kprime; // candidates kept per row by the recall pass (48, 64, 128 or 256)
    int cap;    // candidate buffer entries per row (256 or 512)
};
// The recall pass keeps k' > K candidates so that the K-th exact similarity clears the recall threshold by more than
// the error bound of the 16-bit pass.  With fp32 rows that bound is dominated by their rounding to bf16 (0.4 % of
// |w_i||w_j|) and k' = 2 K gives the margin; with bf16 rows only the fp32 accumulation is left (D * 2^-23), orders
// of magnitude below the spacing of neighbouring similarities, and k' = 1.5 K is kept: the number of candidates a
// row collects during the sweep, and with it the epilogue's work, grows in proportion to k'.
static GrParams gr_params(int K, int D, int dtype = KS_DTYPE_FP32) {
    GrParams p;
    if (K <= 32) { p.kprime = dtype == KS_DTYPE_BF16 ? 48 : 64; p.cap = 256; }
    else if (K <= 64) { p.kprime = 128; p.cap = 256; }
    else { p.kprime = 256; p.cap = 512; }
    if (D % 64 == 0 && !(D == 128 || D == 256 || D == 512))
        p.cap = 512; // the 256 x 256 asynchronous recall kernel appends up to 256 candidates per row and tile
    return p;
}

// ------------------------------------------------------------------------------------------------
// prepare
// ------------------------------------------------------------------------------------------------
template <typename IN> struct GrElem;
template <> struct GrElem<uint16_t> {
    static __device__ __forceinline__ float f(uint16_t v) { return ks_bf2f(v); }
};
template <> struct GrElem<float> {
    static __device__ __forceinline__ float f(float v) { return v; }
};

// one wavefront per row: squared norm in fp32 (only used for the error bound, with slack), optional bf16 copy
template <typename IN>
__global__ void __launch_bounds__(GR_NT)
gr_prepare_kernel(const IN *__restrict__ W, int64_t C, int D, uint16_t *__restrict__ Wb, float *__restrict__ norms,
                  uint32_t *maxnorm_bits) {
    const int64_t i = (int64_t)blockIdx.x * (GR_NT / 64) + (threadIdx.x >> 6);
    if (i >= C) return;
    const int lane = threadIdx.x & 63;
    float s = 0.f;
    if (sizeof(IN) == 2 && D % 8 == 0) { // 16-byte loads (the sum is only used for the error bound, with slack)
        for (int d = lane * 8; d < D; d += 512) {
            const uint4 v = *(const uint4 *)((const uint16_t *)W + i * D + d);
            const uint32_t w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float lo = __uint_as_float(w4[e] << 16), hi = __uint_as_float(w4[e] & 0xFFFF0000u);
                s = fmaf(lo, lo, s);
                s = fmaf(hi, hi, s);
            }
            if (Wb) *(uint4 *)(Wb + i * D + d) = v;
        }
    } else {
        for (int d = lane; d < D; d += 64) {
            float v = GrElem<IN>::f(W[i * D + d]);
            s += v * v;
            if (Wb) Wb[i * D + d] = (uint16_t)ks_f2bf(v);
        }
    }
    s = ks_wave_sum(s);
    if (lane == 0) {
        float nrm = sqrtf(s);
        norms[i] = nrm;
        // non-negative floats order like their bit patterns.  The running maximum is read first: one atomic
        // per row on a single address would serialise the whole kernel in the L2
        const uint32_t bits = __float_as_uint(nrm);
        if (bits > __atomic_load_n(maxnorm_bits, __ATOMIC_RELAXED)) atomicMax(maxnorm_bits, bits);
    }
}

__global__ void gr_zero_kernel(uint32_t *maxnorm_bits, int32_t *fb_count) {
    *maxnorm_bits = 0u;
    *fb_count = 0;
}

// Cut the candidate buffer of one row back to its kprime best (in no particular order: the exact stage ranks them
// anyway) and make the kprime-th best value the row's new threshold; updates cnt/thr in LDS.  One wavefront per row.
// The kprime-th largest key is found by a bitwise search -- rounds of "how many keys are >= this prefix", each a
// compare per key, a wavefront ballot and a population count -- which is an order of magnitude cheaper than sorting
// the keys across the lanes (the keys are distinct: value bits above, inverted row id below; empty slots are 0).
// The 32 value bits are searched first; the id bits only when several keys share the kprime-th value.
// Requires kprime <= number of keys.
template <int E> __device__ __forceinline__ int gr_count_hi_ge(const uint64_t (&val)[E], uint32_t t) {
    int c = 0;
#pragma unroll
    for (int r = 0; r < E; ++r) c += __popcll(__ballot((uint32_t)(val[r] >> 32) >= t));
    return c;
}
template <int E> __device__ __forceinline__ int gr_count_lo_ge(const uint64_t (&val)[E], uint32_t hi, uint32_t t) {
    int c = 0;
#pragma unroll
    for (int r = 0; r < E; ++r) c += __popcll(__ballot((uint32_t)(val[r] >> 32) == hi && (uint32_t)val[r] >= t));
    return c;
}
template <int E>
__device__ __forceinline__ void gr_compact_row(uint64_t *__restrict__ cand_row, int *cnt, uint32_t *thr, int kprime) {
    const int lane = threadIdx.x & 63;
    const int n = *cnt;
    uint64_t val[E];
#pragma unroll
    for (int r = 0; r < E; ++r) {
        int idx = r * 64 + lane;
        val[r] = idx < n ? cand_row[idx] : 0ull; // 0 is below every real key
    }
    uint32_t t_hi = 0; // every decision below is uniform over the wavefront
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t c = t_hi | (1u << bit);
        if (gr_count_hi_ge<E>(val, c) >= kprime) t_hi = c;
    }
    uint64_t t = (uint64_t)t_hi << 32;
    if (gr_count_hi_ge<E>(val, t_hi) != kprime) { // keys of equal value straddle the cut: the ids decide
        const int need = kprime - (t_hi == 0xFFFFFFFFu ? 0 : gr_count_hi_ge<E>(val, t_hi + 1u));
        uint32_t t_lo = 0;
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t c = t_lo | (1u << bit);
            if (gr_count_lo_ge<E>(val, t_hi, c) >= need) t_lo = c;
        }
        t |= t_lo;
    }
    // t is the kprime-th largest key: exactly kprime keys are >= t; they move to the front of the buffer
    int base = 0;
#pragma unroll
    for (int r = 0; r < E; ++r) {
        const uint64_t m = __ballot(val[r] >= t);
        if (val[r] >= t) cand_row[base + __popcll(m & ((1ull << lane) - 1ull))] = val[r];
        base += __popcll(m);
    }
    if (lane == 0) {
        *cnt = kprime;
        *thr = (uint32_t)(t >> 32);
    }
}

// ------------------------------------------------------------------------------------------------
// recall pass
// ------------------------------------------------------------------------------------------------
template <class T, int E>
__global__ void __launch_bounds__(T::NT)
gr_recall_kernel(GrPair pr, int D, int kprime, uint64_t *__restrict__ cand, int32_t *__restrict__ cnt_out,
                 uint32_t *__restrict__ thr_out) {
    const int64_t C = pr.Cr;
    constexpr int CAP = E * 64;
    __shared__ __attribute__((aligned(16))) uint16_t lds[T::LDS_ELEMS];
    __shared__ int s_cnt[T::BM];
    __shared__ uint32_t s_thr[T::BM];
    const int wave = threadIdx.x >> 6;
    const int64_t row0 = (int64_t)blockIdx.x * T::BM;
    for (int m = threadIdx.x; m < T::BM; m += T::NT) { s_cnt[m] = 0; s_thr[m] = 0u; }
    __syncthreads();

    KsRowLoader<T::BM, T::BK, T::NT> al;
    al.init(pr.R, D, nullptr, (int)row0, (int)C, D);
    const int n_col_blocks = (int)((pr.Cs + T::BN - 1) / T::BN);
    const int nk = (D + T::BK - 1) / T::BK;
    for (int J = 0; J < n_col_blocks; ++J) {
        KsRowLoader<T::BN, T::BK, T::NT> bl;
        bl.init(pr.S, D, nullptr, J * T::BN, (int)pr.Cs, D);
        f32x16_t acc[T::FM][T::FN];
        ks_tile_clear<T>(acc);
        ks_gemm_mainloop<T>(al, bl, 0, nk, lds, acc);
        ks_tile_foreach<T>(acc, [&](int m, int n, float v) {
            const int64_t i = row0 + m, j = (int64_t)J * T::BN + n;
            if (i < C && j < pr.Cs && j != i + pr.self) {
                const uint32_t hi = gr_orderable(v);
                if (hi > s_thr[m]) {
                    int slot = atomicAdd(&s_cnt[m], 1);
                    if (slot < CAP) // always true: a buffer is cut back before it can overflow
                        cand[i * CAP + slot] = ((uint64_t)hi << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)j);
                }
            }
        });
        __syncthreads();
        for (int m = wave; m < T::BM; m += T::NT / 64) {
            if (s_cnt[m] > CAP - T::BN) gr_compact_row<E>(cand + (row0 + m) * CAP, &s_cnt[m], &s_thr[m], kprime);
        }
        __syncthreads();
    }
    for (int m = wave; m < T::BM; m += T::NT / 64) {
        if (row0 + m < C) {
            if (s_cnt[m] > kprime) gr_compact_row<E>(cand + (row0 + m) * CAP, &s_cnt[m], &s_thr[m], kprime);
        }
    }
    __syncthreads();
    for (int m = threadIdx.x; m < T::BM; m += T::NT) {
        if (row0 + m < C) { cnt_out[row0 + m] = s_cnt[m]; thr_out[row0 + m] = s_thr[m]; }
    }
}

// ------------------------------------------------------------------------------------------------
// recall pass on the asynchronous engine (D % 64 == 0): 256 rows per workgroup, 256-column blocks.
// The k-tiles of the whole sweep form one stream: the first k-tile of the next column block is already
// on its way into LDS while the current block's similarities are filtered.
// ------------------------------------------------------------------------------------------------
template <class T, int E>
__global__ void __launch_bounds__(T::NT)
gr_recall_async_kernel(GrPair pr, int D, int kprime, uint64_t *__restrict__ cand, int32_t *__restrict__ cnt_out,
                       uint32_t *__restrict__ thr_out) {
    const int64_t C = pr.Cr;
    constexpr int CAP = E * 64;
    static_assert(T::STAGES == 2 && CAP >= 256 + T::BN, "recall tile");
    __shared__ __attribute__((aligned(16))) uint16_t lds[T::LDS_ELEMS];
    __shared__ int s_cnt[T::BM];
    __shared__ uint32_t s_thr[T::BM];
    const int wave = threadIdx.x >> 6;
    const int64_t row0 = (int64_t)blockIdx.x * T::BM;
    for (int m = threadIdx.x; m < T::BM; m += T::NT) { s_cnt[m] = 0; s_thr[m] = 0u; }
    __syncthreads();

    KsARows<T::BM, T::NW> ar;
    KsARows<T::BN, T::NW> br;
    ar.init(pr.R, D, nullptr, (int)row0, (int)C);
    br.init(pr.S, D, nullptr, 0, (int)pr.Cs);
    const int nJ = (int)((pr.Cs + T::BN - 1) / T::BN), nk = D / 64;
    // stream position of the next tile to load
    int ld_J = 0, ld_kt = 0;
    auto issue_next = [&](int stage) {
        uint16_t *st = lds + stage * T::STAGE_ELEMS;
        ar.issue(ld_kt * 64, st);
        br.issue(ld_kt * 64, st + T::BM * 64);
        if (++ld_kt == nk) {
            ld_kt = 0;
            ++ld_J;
            if (ld_J < nJ) br.init(pr.S, D, nullptr, ld_J * T::BN, (int)pr.Cs);
        }
    };
    issue_next(0);
    int stage = 0;
    for (int J = 0; J < nJ; ++J) {
        f32x16_t acc[T::FM][T::FN];
        ks_a_clear<T>(acc);
        for (int kt = 0; kt < nk; ++kt) {
            ks_wait_vmcnt<0>();
            ks_barrier_nofence();
            if (ld_J < nJ) issue_next(stage ^ 1);
            ks_a_tile_mma<T>(lds + stage * T::STAGE_ELEMS, acc);
            stage ^= 1;
        }
        ks_a_foreach<T>(acc, [&](int m, int n, float v) {
            const int64_t i = row0 + m, j = (int64_t)J * T::BN + n;
            if (i < C && j < pr.Cs && j != i + pr.self) {
                const uint32_t hi = gr_orderable(v);
                if (hi > s_thr[m]) {
                    int slot = atomicAdd(&s_cnt[m], 1);
                    if (slot < CAP) // always true: a buffer is cut back before it can overflow
                        cand[i * CAP + slot] = ((uint64_t)hi << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)j);
                }
            }
        });
        __syncthreads();
        for (int m = wave; m < T::BM; m += T::NW) {
            if (s_cnt[m] > CAP - T::BN) gr_compact_row<E>(cand + (row0 + m) * CAP, &s_cnt[m], &s_thr[m], kprime);
        }
        __syncthreads();
    }
    for (int m = wave; m < T::BM; m += T::NW) {
        if (row0 + m < C) {
            if (s_cnt[m] > kprime) gr_compact_row<E>(cand + (row0 + m) * CAP, &s_cnt[m], &s_thr[m], kprime);
        }
    }
    __syncthreads();
    for (int m = threadIdx.x; m < T::BM; m += T::NT) {
        if (row0 + m < C) { cnt_out[row0 + m] = s_cnt[m]; thr_out[row0 + m] = s_thr[m]; }
    }
}

// ------------------------------------------------------------------------------------------------
// recall pass as a stationary-operand sweep (D = 128, 256 or 512): a workgroup keeps the MFMA fragments
// of its 256 rows in registers and streams every row of W past them, 96 rows at a time.  A lane owns one
// of the 256 rows in the accumulators, so the row's threshold is a register and most elements cost one
// max operation; only groups of four elements whose maximum beats the threshold are looked at one by one.
// ------------------------------------------------------------------------------------------------
#define GR_SOE_STAGES 6
// Candidate buffers of the sweep kernel below.  Two lanes of a wavefront share a row of the graph (they hold
// different streamed rows of it), so each appends to its own half of the row's buffer and counts in a register:
// an append is a store and an increment, with no atomic operation and nothing to wait for.
// Cuts the two halves (n0 and n1 keys) back to the kprime largest keys and returns the value bits of the smallest
// key kept (0 when nothing was dropped); survivors go half and half to the two halves, or -- for the final call --
// to the front of the buffer.  One wavefront per row.
template <int E>
__device__ __forceinline__ uint32_t gr_compact_halves(uint64_t *__restrict__ cand_row, int n0, int n1, int kprime,
                                                       bool final_layout, int *n_kept) {
    constexpr int HALF = E * 32;
    const int lane = threadIdx.x & 63;
    uint64_t val[E];
#pragma unroll
    for (int r = 0; r < E; ++r) {
        const int idx = r * 64 + lane;
        const bool valid = idx < HALF ? idx < n0 : idx - HALF < n1;
        val[r] = valid ? cand_row[idx] : 0ull; // 0 is below every real key
    }
    const int n = n0 + n1;
    uint64_t t = 1ull; // keeps every real key
    if (n > kprime) {
        uint32_t t_hi = 0; // every decision below is uniform over the wavefront
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t c = t_hi | (1u << bit);
            if (gr_count_hi_ge<E>(val, c) >= kprime) t_hi = c;
        }
        t = (uint64_t)t_hi << 32;
        if (gr_count_hi_ge<E>(val, t_hi) != kprime) { // keys of equal value straddle the cut: the ids decide
            const int need = kprime - (t_hi == 0xFFFFFFFFu ? 0 : gr_count_hi_ge<E>(val, t_hi + 1u));
            uint32_t t_lo = 0;
            for (int bit = 31; bit >= 0; --bit) {
                const uint32_t c = t_lo | (1u << bit);
                if (gr_count_lo_ge<E>(val, t_hi, c) >= need) t_lo = c;
            }
            t |= t_lo;
        }
    }
    const int kept = n > kprime ? kprime : n;
    const int first = final_layout ? kept : (kept + 1) / 2; // keys that go to the first half
    int base = 0;
#pragma unroll
    for (int r = 0; r < E; ++r) {
        const uint64_t m = __ballot(val[r] >= t);
        if (val[r] >= t) {
            const int q = base + __popcll(m & ((1ull << lane) - 1ull));
            cand_row[q < first ? q : HALF + (q - first)] = val[r];
        }
        base += __popcll(m);
    }
    *n_kept = kept;
    return n > kprime ? (uint32_t)(t >> 32) : 0u;
}

template <int KT, int E>
__global__ void __launch_bounds__(512)
gr_recall_soe_kernel(GrPair pr, int D, int kprime, uint64_t *__restrict__ cand, int32_t *__restrict__ cnt_out,
                      uint32_t *thr_out, const uint32_t *thr_init) {
    const int64_t C = pr.Cr;
    typedef KsSoe<KT, 96, GR_SOE_STAGES, 2> CFG;
    constexpr int CAP = E * 64, HALF = CAP / 2;
    constexpr int LIMIT = HALF - CFG::FM * 16; // a lane appends at most FM * 16 keys per chunk
    static_assert(LIMIT >= 64, "room for half of the largest kprime of this buffer size");
    __shared__ __attribute__((aligned(16))) uint16_t lds[CFG::LDS_ELEMS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t row0 = (int64_t)blockIdx.x * CFG::RES;
    const int col = ks_soe_col();
    const int gi = (int)row0 + col; // C < 2^31
    const int Ci = (int)C;
    const int64_t self0 = row0 + pr.self; // streamed rows [self0, self0 + RES) are this workgroup's own rows
    // A wavefront's accumulators hold 32 of the 256 rows, two lanes per row (lane and lane + 32 hold different streamed
    // rows), so the candidate buffers of those rows are written by that wavefront alone: it also cuts them back
    // itself, the counts and the thresholds live in registers, and the epilogue needs no barrier and no atomics.
    // an append is a store at a 32-bit slot number behind one base address of the workgroup: the count of the lane's
    // half plus a constant of the lane
    uint64_t *const wg_cand = cand + row0 * CAP;
    const uint32_t my_base = (uint32_t)(col * CAP + (lane >> 5) * HALF);
    int my_cnt = 0;
    uint32_t th = 0u; // value bits of the row's threshold; 0 = nothing dropped yet: everything passes
    float thf = gi >= Ci ? INFINITY : -INFINITY; // rows beyond C never pass
    if (thr_init && gi < Ci) { // the caller knows that nothing at or below this value is wanted (may be thr_out itself)
        th = thr_init[gi];
        if (th != 0u) thf = gr_unorder(th);
    }
    auto cut_back = [&](bool final_layout) {
        ks_wait_vmcnt<0>(); // the appended candidates have left this wavefront before it reads them back
        asm volatile("" ::: "memory");
        for (int m = 0; m < 32; ++m) {
            const int n0 = __builtin_amdgcn_readlane(my_cnt, m), n1 = __builtin_amdgcn_readlane(my_cnt, m + 32);
            if (final_layout ? (row0 + wave * 32 + m < C) : (n0 > LIMIT || n1 > LIMIT)) {
                int kept;
                const uint32_t t = gr_compact_halves<E>(cand + (row0 + wave * 32 + m) * CAP, n0, n1, kprime, final_layout, &kept);
                if ((lane & 31) == m) {
                    my_cnt = final_layout ? kept : (lane < 32 ? (kept + 1) / 2 : kept / 2);
                    if (t != 0u) { th = t; thf = gr_unorder(t); }
                }
            }
        }
        asm volatile("" ::: "memory");
    };
    auto epi = [&](int c0, int rows_here, f32x16_t (&acc)[CFG::FM]) {
        // elements that need more than the threshold test: the tail of the last chunk, and the diagonal
        const bool special = rows_here < CFG::CH || ((int64_t)c0 < self0 + CFG::RES && (int64_t)c0 + CFG::CH > self0);
        constexpr int GROUP = 4; // elements per threshold test (2 .. 16 measured alike)
        // compiled twice: nearly all chunks are plain (all rows real, none of them the row itself)
        auto elements = [&](auto is_special) __attribute__((always_inline)) {
            constexpr bool SPECIAL = decltype(is_special)::value;
#pragma unroll
            for (int fm = 0; fm < CFG::FM; ++fm) {
#pragma unroll
                for (int q = 0; q < 16 / GROUP; ++q) { // GROUP elements at a time: most groups have none that passes
                    float bm = acc[fm][q * GROUP];
#pragma unroll
                    for (int e = 1; e < GROUP; ++e) bm = fmaxf(bm, acc[fm][q * GROUP + e]);
                    if (bm > thf) {
#pragma unroll
                        for (int e = 0; e < GROUP; ++e) {
                            const int r = q * GROUP + e;
                            const float v = acc[fm][r];
                            if (v > thf) {
                                const int lr = ks_soe_row(fm, r, lane);
                                const int j = c0 + lr;
                                if (SPECIAL && (lr >= rows_here || (int64_t)j == (int64_t)gi + pr.self)) continue;
                                // (my_cnt < HALF: a buffer is cut back before it can overflow; the mask keeps the
                                // store inside the lane's half whatever happens)
                                wg_cand[my_base + ((uint32_t)my_cnt & (uint32_t)(HALF - 1))] =
                                    ((uint64_t)gr_orderable(v) << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)j);
                                ++my_cnt;
                            }
                        }
                    }
                }
            }
        };
        if (special) elements(std::true_type());
        else elements(std::false_type());
        if (__any(my_cnt > LIMIT)) cut_back(false); // a buffer could overflow in the next chunk
    };
    ks_soe_sweep<CFG>(pr.R, D, (int)row0, (int)C, pr.S, D, nullptr, 0, (int)pr.Cs, (int)pr.Cs, lds, epi);
    cut_back(true); // at most kprime keys per row, at the front of its buffer
    if (lane < 32 && gi < Ci) { cnt_out[gi] = my_cnt; thr_out[gi] = th; }
}

// ------------------------------------------------------------------------------------------------
// recall pass that computes every similarity ONCE (W searched in W, D = 128, 256 or 512, k' <= 64).
//
// The similarity matrix is symmetric, so the tile of a workgroup's 256 resident rows against a streamed row j holds,
// for every resident row i, a candidate for BOTH lists: j for row i (the "resident side", a lane's own row, as in the
// kernel above) and i for row j (the "stream side").  Each unordered pair of 256-row blocks is given to exactly one
// workgroup, which halves the MFMA work of the pass.  What it takes:
//
//  * thresholds known in advance.  A row that is streamed past hundreds of workgroups cannot keep a running
//    threshold, so a first pass (the kernel above, on every 32nd row of W only) finds for each row the 12th largest
//    similarity to that sample.  The number of rows of all of W at or above it is 32 times a Gamma(12) variable
//    whatever the distribution of the rows (it is an order statistic of a uniform sample): 384 on average, beyond
//    1,100 or below k' (then 12 of the row's k' best would have to be in the sample) for less than one row in a
//    million.  Both sides test against these fixed thresholds and the buffers are sized for those counts; nothing is
//    cut back during the sweep.  A row that does end up with too many or too few candidates is caught by the
//    re-rank's certificate like any other uncertain row.
//  * who takes which pair.  Rows are cut into blocks of 256 (a workgroup's resident rows), super-blocks of 768 rows
//    (three blocks = eight 96-row chunks, so that every streamed range starts on a chunk boundary) and groups of up
//    to 10 super-blocks.  On each level the members form a ring and a member takes the following half of the ring
//    (gr_sym_succ): a workgroup streams its own super-block (its own block for the resident side only, the blocks it
//    takes there for both sides), then the super-blocks it takes inside its group, then all rows of the groups its
//    group takes.  The 30 workgroups of a group sit on one XCD and stream the same long ranges at the same pace, so
//    a streamed row is fetched from memory once per group.
//  * the stream side's candidates.  A hit for streamed row j is a record (j, i, similarity): a wavefront collects them
//    in LDS and appends them, with one atomic per batch, to the log of j's super-block; gr_sym_scatter_kernel (one
//    workgroup per super-block, row counters in LDS) then moves them into the rows' buffers.  In the sweep the
//    thresholds of the streamed rows are scalar registers (an accumulator register holds one streamed row across the
//    lanes); the two halves of a wavefront hold different rows (j and j + 4), so the test is against the smaller of
//    the two thresholds (gr_sym_prep_kernel stores these minima) and the scatter kernel applies the row's own.
//  * gr_sym_select_kernel cuts every row's candidates (two resident-side halves and the stream side) to the k' best,
//    in the layout the re-rank expects.  A row whose buffers or log overflowed gets a threshold no similarity
//    exceeds: its certificate fails and the exhaustive pass computes it.
// ------------------------------------------------------------------------------------------------
#define GR_SYM_CAP 2048          /* candidate slots per row: two resident-side halves, then the stream side */
#define GR_SYM_Q 512             /* slots of each resident-side half */
#define GR_SYM_SCAP 1024         /* slots of the stream side */
#define GR_SYM_SB 768            /* rows of a super-block */
#define GR_SYM_LOGCAP (768 * 384) /* records per super-block log (expected: 768 rows * 192 stream-side hits, plus a tenth) */
#define GR_SYM_STAGE 192         /* records a wavefront collects in LDS between two appends to a log */
#define GR_SYM_RATIO 32          /* rows of W per sampled row */
#define GR_SYM_RANK 12           /* the threshold of a row: its GR_SYM_RANK-th largest similarity to the sample */
#define GR_SYM_MAX_GROUP 10      /* super-blocks per group at most: 30 workgroups, about the compute units of an XCD */

// rows of W sampled by the first pass: one of every `ratio` consecutive rows, at a position that varies from one run
// of `ratio` rows to the next
__device__ __forceinline__ int64_t gr_sym_sample_row(int64_t s, int ratio, int64_t C) {
    const int64_t r = s * ratio + (int64_t)(((uint32_t)s * 2654435761u) >> 16) % ratio;
    return r < C ? r : C - 1;
}
// members of a ring of n that member x takes: the next gr_sym_succ(n, x) ones.  Every unordered pair is taken once:
// for even n the opposite member is taken by the lower of the two.
__host__ __device__ __forceinline__ int gr_sym_succ(int n, int x) {
    return (n & 1) ? (n - 1) / 2 : (x < n / 2 ? n / 2 : n / 2 - 1);
}
__host__ __device__ __forceinline__ int gr_sym_group_sbs(int64_t C) { // super-blocks per group
    const int nsb = (int)((C + GR_SYM_SB - 1) / GR_SYM_SB);
    const int gs = nsb / 16;
    return gs < 1 ? 1 : (gs > GR_SYM_MAX_GROUP ? GR_SYM_MAX_GROUP : gs);
}

__global__ void __launch_bounds__(GR_NT)
gr_sym_sample_kernel(const uint16_t *__restrict__ W, int64_t C, int D, int ratio, int64_t n_sample,
                     uint16_t *__restrict__ Ws) {
    const int64_t s = (int64_t)blockIdx.x * (GR_NT / 64) + (threadIdx.x >> 6);
    if (s >= n_sample) return;
    const uint4 *src = (const uint4 *)(W + gr_sym_sample_row(s, ratio, C) * D);
    uint4 *dst = (uint4 *)(Ws + s * D);
    for (int q = threadIdx.x & 63; q < D / 8; q += 64) dst[q] = src[q];
}

// thr_sample[i]: value bits of the GR_SYM_RANK-th largest similarity of row i to the sample (0: the sample had fewer rows).
// Row i takes every similarity at or above it: thf[i] is the next float below, and tbits[i] its key, so that "v > thf"
// is the test and "key value <= tbits" holds for everything that fails it.  Rows at and beyond C never pass.  Also
// clears the counters of the logs and of the second-chance list.
__global__ void __launch_bounds__(GR_NT)
gr_sym_prep_kernel(const uint32_t *__restrict__ thr_sample, int64_t C, int64_t Cpad, float *__restrict__ thf,
                   uint32_t *__restrict__ tbits, int32_t *__restrict__ logcnt, int nsb, int32_t *second_count) {
    const int64_t i = (int64_t)blockIdx.x * GR_NT + threadIdx.x;
    if (i < nsb) logcnt[i] = 0;
    if (i == 0) *second_count = 0;
    if (i >= Cpad) return;
    if (i >= C) {
        thf[i] = INFINITY;
        return;
    }
    const uint32_t lowest = gr_orderable(-INFINITY), t = thr_sample[i];
    const uint32_t bits = t > lowest + 1u ? t - 1u : lowest;
    thf[i] = gr_unorder(bits);
    tbits[i] = bits;
}

// The plan of the sweep, made by a small kernel beforehand (the sweep kernel has no registers to spare for the
// arithmetic).  Per workgroup GR_SYM_PLAN words: [0] the resident block or -1, [1] the block's place in the ring of its
// super-block's blocks (place | members << 4 | members it takes << 8), [2] the number of chunks it streams; and a table
// of those chunks (first row, rows): its own super-block, then the super-blocks it takes in its group (two ranges: the
// ring wraps), then the groups its group takes (likewise).
#define GR_SYM_PLAN 4
struct GrSymRanges {
    int block;          // resident block, or -1: the workgroup has none
    int ring;           // place | members << 4 | members taken << 8 in the ring of its super-block's blocks
    int first[5], end[5]; // streamed rows [first, end) of the five ranges; empty: end <= first
};
__host__ __device__ inline GrSymRanges gr_sym_ranges(int wg, int C, int GS) {
    GrSymRanges out;
    const int NB = (C + 255) / 256, NSB = (C + GR_SYM_SB - 1) / GR_SYM_SB, NG = (NSB + GS - 1) / GS;
    const int BPG = GS * (GR_SYM_SB / 256); // blocks per group
    // the workgroups of a group are those that one XCD receives in a row (workgroups are dealt to the eight XCDs in turn)
    const int g = (wg >> 3) / BPG * 8 + (wg & 7);
    const int block = g * BPG + (wg >> 3) % BPG;
    out.block = -1;
    out.ring = 0;
    for (int part = 0; part < 5; ++part) out.first[part] = out.end[part] = 0;
    if (g >= NG || block >= NB) return out;
    const int sb = block * 256 / GR_SYM_SB, own0 = sb * GR_SYM_SB, own1 = own0 + GR_SYM_SB < C ? own0 + GR_SYM_SB : C;
    const int kb = (block * 256 - own0) / 256, n_b = (own1 - own0 + 255) / 256;
    const int gsb0 = g * GS, n_sb = (gsb0 + GS < NSB ? gsb0 + GS : NSB) - gsb0, s_loc = sb - gsb0;
    const int succ_s = gr_sym_succ(n_sb, s_loc), succ_g = gr_sym_succ(NG, g);
    out.block = block;
    out.ring = kb | (n_b << 4) | (gr_sym_succ(n_b, kb) << 8);
    for (int part = 0; part < 5; ++part) {
        int b = 0, e = 0; // in super-blocks
        if (part == 0) { b = sb; e = sb + 1; }
        else if (part == 1) { b = sb + 1; e = gsb0 + (s_loc + succ_s < n_sb - 1 ? s_loc + succ_s : n_sb - 1) + 1; }
        else if (part == 2) { b = gsb0; e = gsb0 + (s_loc + succ_s - n_sb) + 1; }
        else if (part == 3) { b = (g + 1) * GS; e = ((g + succ_g < NG - 1 ? g + succ_g : NG - 1) + 1) * GS; }
        else { b = 0; e = (g + succ_g - NG + 1) * GS; }
        if (e > NSB) e = NSB;
        if (e <= b) continue;
        const long long e_row = (long long)e * GR_SYM_SB;
        out.first[part] = b * GR_SYM_SB;
        out.end[part] = e_row < C ? (int)e_row : C;
    }
    return out;
}
__global__ void __launch_bounds__(GR_NT)
gr_sym_plan_kernel(int C, int GS, int32_t *__restrict__ plan, int2 *__restrict__ chunks, int chunks_stride) {
    const int wg = blockIdx.x;
    int32_t *out = plan + (int64_t)wg * GR_SYM_PLAN;
    int2 *tab = chunks + (int64_t)wg * chunks_stride;
    const GrSymRanges r = gr_sym_ranges(wg, C, GS);
    int n_chunks = 0;
    for (int part = 0; part < 5; ++part) {
        if (r.end[part] <= r.first[part]) continue;
        const int n = (r.end[part] - r.first[part] + 95) / 96;
        for (int c = threadIdx.x; c < n; c += GR_NT) {
            const int first = r.first[part] + c * 96;
            if (n_chunks + c < chunks_stride) tab[n_chunks + c] = make_int2(first, r.end[part] - first < 96 ? r.end[part] - first : 96);
        }
        n_chunks += n;
    }
    if (threadIdx.x == 0) {
        out[0] = r.block;
        out[1] = r.ring;
        out[2] = n_chunks < chunks_stride ? n_chunks : chunks_stride; // (the stride is sized for the longest plan)
    }
}

// Element r (0 .. 15, different from lane to lane) of a lane's 16 accumulator values: a binary tree of selects on the
// bits of r.  (As assembly: written as conditional expressions the compiler turns the tree into a table in scratch
// memory that it indexes with r.  The s_nop after each compare: a select must not read a mask that one of the two
// instructions before it has written.)
__device__ __forceinline__ float gr_sym_pick16(const f32x16_t &a, int r) {
    float b0, b1, b2, b3, b4, b5, b6, b7, c0, c1, c2, c3, d0, d1, v;
    asm("v_and_b32 %8, 1, %25\n\tv_cmp_ne_u32 vcc, 0, %8\n\ts_nop 1\n\t"
        "v_cndmask_b32 %0, %9, %10, vcc\n\tv_cndmask_b32 %1, %11, %12, vcc\n\t"
        "v_cndmask_b32 %2, %13, %14, vcc\n\tv_cndmask_b32 %3, %15, %16, vcc\n\t"
        "v_cndmask_b32 %4, %17, %18, vcc\n\tv_cndmask_b32 %5, %19, %20, vcc\n\t"
        "v_cndmask_b32 %6, %21, %22, vcc\n\tv_cndmask_b32 %7, %23, %24, vcc"
        : "=&v"(b0), "=&v"(b1), "=&v"(b2), "=&v"(b3), "=&v"(b4), "=&v"(b5), "=&v"(b6), "=&v"(b7), "=&v"(v)
        : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7]), "v"(a[8]), "v"(a[9]),
          "v"(a[10]), "v"(a[11]), "v"(a[12]), "v"(a[13]), "v"(a[14]), "v"(a[15]), "v"(r)
        : "vcc");
    asm("v_and_b32 %4, 2, %13\n\tv_cmp_ne_u32 vcc, 0, %4\n\ts_nop 1\n\t"
        "v_cndmask_b32 %0, %5, %6, vcc\n\tv_cndmask_b32 %1, %7, %8, vcc\n\t"
        "v_cndmask_b32 %2, %9, %10, vcc\n\tv_cndmask_b32 %3, %11, %12, vcc"
        : "=&v"(c0), "=&v"(c1), "=&v"(c2), "=&v"(c3), "=&v"(v)
        : "v"(b0), "v"(b1), "v"(b2), "v"(b3), "v"(b4), "v"(b5), "v"(b6), "v"(b7), "v"(r)
        : "vcc");
    asm("v_and_b32 %2, 4, %7\n\tv_cmp_ne_u32 vcc, 0, %2\n\ts_nop 1\n\t"
        "v_cndmask_b32 %0, %3, %4, vcc\n\tv_cndmask_b32 %1, %5, %6, vcc"
        : "=&v"(d0), "=&v"(d1), "=&v"(v)
        : "v"(c0), "v"(c1), "v"(c2), "v"(c3), "v"(r)
        : "vcc");
    asm("v_and_b32 %0, 8, %3\n\tv_cmp_ne_u32 vcc, 0, %0\n\ts_nop 1\n\tv_cndmask_b32 %0, %1, %2, vcc"
        : "=&v"(v)
        : "v"(d0), "v"(d1), "v"(r)
        : "vcc");
    return v;
}

// a stream-side hit: similarity v of a streamed row (given by its place in its super-block) with resident row `other`
__device__ __forceinline__ uint2 gr_sym_record(int j_in_sb, int other, float v) {
    return make_uint2(gr_orderable(v), ((uint32_t)other << 10) | (uint32_t)j_in_sb);
}

template <int KT>
__global__ void __launch_bounds__(512)
gr_recall_sym_kernel(const uint16_t *__restrict__ W, int C, int D, const int32_t *__restrict__ plan,
                     const int2 *__restrict__ chunks, int chunks_stride, const float *__restrict__ thf_row,
                     uint64_t *__restrict__ cand, int32_t *__restrict__ cnt_res,
                     uint2 *__restrict__ log, int32_t *logcnt) {
    typedef KsSoe<KT, 96, GR_SOE_STAGES, 2> CFG;
    constexpr int CAP = GR_SYM_CAP, Q = GR_SYM_Q, SB = GR_SYM_SB;
    static_assert(SB % CFG::CH == 0 && SB % CFG::RES == 0 && CFG::RES == 256, "super-blocks are whole chunks and whole blocks");
    __shared__ __attribute__((aligned(16))) uint16_t lds[CFG::LDS_ELEMS];
    __shared__ uint2 s_stage[CFG::NW][GR_SYM_STAGE];
    __shared__ __attribute__((aligned(16))) float s_thr[8][CFG::CH]; // the streamed rows' thresholds of the chunks in flight
    const int lane = threadIdx.x & 63;
    const int32_t *my_plan = plan + (int64_t)blockIdx.x * GR_SYM_PLAN;
    const int block = my_plan[0];
    if (block < 0) return;
    const int row0 = block * CFG::RES;
    const int sb_own = row0 / SB;
    const int ring = my_plan[1];
    const float thf = row0 + ks_soe_col() < C ? thf_row[row0 + ks_soe_col()] : INFINITY;
    uint64_t *const wg_cand = cand + (int64_t)row0 * CAP;
    int my_cnt = 0;
    // stream side: records collected by this wavefront, and the super-block they belong to
    int staged = 0, cur_sb = sb_own;
    auto my_stage = [&]() __attribute__((always_inline)) { return s_stage[__builtin_amdgcn_readfirstlane(threadIdx.x >> 6)]; };
    auto flush = [&]() {
        if (staged > 0) {
            int base = 0;
            if (lane == 0) base = atomicAdd(&logcnt[cur_sb], staged);
            base = __builtin_amdgcn_readfirstlane(base);
            uint2 *dst = log + (int64_t)cur_sb * GR_SYM_LOGCAP;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // the records written by the other lanes are in LDS
            for (int q = lane; q < staged; q += 64)
                if (base + q < GR_SYM_LOGCAP) dst[base + q] = my_stage()[q];
            asm volatile("" ::: "memory");
            staged = 0;
        }
    };
    // all lanes call it together with the ballot m of `hit`; the lanes that hit add the record (j, own row, v)
    auto push = [&](uint64_t m, bool hit, int j, float v) __attribute__((always_inline)) {
        const int n = __popcll(m);
        if (staged + n > GR_SYM_STAGE) flush();
        if (hit) my_stage()[staged + __popcll(m & ((1ull << lane) - 1ull))] = gr_sym_record(j - cur_sb * SB, row0 + ks_soe_col(), v);
        staged = __builtin_amdgcn_readfirstlane(staged + n);
    };
    auto append_res = [&](int j, float v) __attribute__((always_inline)) {
        // (the mask keeps the store inside the lane's half; a count beyond Q marks the row as overflowed)
        const uint32_t my_base = (uint32_t)(ks_soe_col() * CAP + (lane >> 5) * Q);
        wg_cand[my_base + ((uint32_t)my_cnt & (uint32_t)(Q - 1))] = ((uint64_t)gr_orderable(v) << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)j);
        ++my_cnt;
    };
    // The thresholds of a chunk's rows travel to LDS beside its rows: requested by wavefront 0 when the chunk's loads begin.
    // The loads run up to STAGES - 1 pipeline stages ahead of the MFMAs and a chunk of D = 128 is a single stage, so up to
    // seven chunks lie between the request and the epilogue that reads it: eight slots.
    static_assert(GR_SOE_STAGES - 1 + 2 <= 8, "slots for the chunks in flight");
    auto side = [&](int first, int c) __attribute__((always_inline)) {
        static_assert(CFG::CH == 96, "64 + 32 lanes");
        __builtin_amdgcn_global_load_lds(KS_GPTR(thf_row + first + lane), KS_LPTR(&s_thr[c & 7][0]), 4, 0, 0);
        if (lane < 32) __builtin_amdgcn_global_load_lds(KS_GPTR(thf_row + first + 64 + lane), KS_LPTR(&s_thr[c & 7][64]), 4, 0, 0);
    };
    int epi_chunk = 0; // chunks seen by the epilogue: the slot of their thresholds
    auto epi = [&](int c0, int rows_here, f32x16_t (&acc)[CFG::FM]) {
        const float *thr_chunk = s_thr[epi_chunk & 7];
        ++epi_chunk;
        const int sb = c0 / SB; // uniform; a chunk lies in one super-block
        if (sb != cur_sb) { flush(); cur_sb = sb; }
        if (rows_here == CFG::CH && sb != sb_own) {
            // plain chunk: all rows real, both sides wanted for every element
            const bool real_row = row0 + ks_soe_col() < C;
#pragma unroll
            for (int fm = 0; fm < CFG::FM; ++fm) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float a0 = acc[fm][4 * q], a1 = acc[fm][4 * q + 1], a2 = acc[fm][4 * q + 2], a3 = acc[fm][4 * q + 3];
                    if (fmaxf(fmaxf(a0, a1), fmaxf(a2, a3)) > thf) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float v = acc[fm][4 * q + e];
                            if (v > thf) append_res(c0 + ks_soe_row(fm, 4 * q + e, lane), v);
                        }
                    }
                }
                // Stream side.  An accumulator register holds ONE streamed row in the lanes 0..31 and the row four further
                // on in the lanes 32..63.  (Testing against the smaller of the two thresholds, held in a scalar register,
                // and sorting out the surplus later was tried: the number of records then depends on how well
                // neighbouring rows match; a tight cluster row beside a lone one got four times its share, the logs
                // overflowed and every row went to the exhaustive pass.  With the exact test the counts depend on
                // nothing but the sample.)
                // Every instruction here runs once per chunk and fragment, so there are few: a lane's hits become a bit
                // mask with a compare and an add-with-carry per element and half (bit 15 - r for element r); nearly always
                // no lane has more than one hit, and then a lane picks its element with a binary tree of selects and the
                // slots come from one ballot.
                // (a lane reads the four thresholds of its own rows from LDS: rows 8 q + e in the lanes 0..31, 8 q + 4 + e
                // in the lanes 32..63)
                uint32_t hm = 0u;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x4_t t4 = *(const f32x4_t *)(thr_chunk + fm * 32 + 8 * q + 4 * (lane >> 5));
                    // (the four compares first: a vector instruction must not read a mask that one of the two
                    // instructions before it has written)
                    uint64_t k0, k1, k2, k3;
                    asm("v_cmp_lt_f32 %1, %5, %9\n\tv_cmp_lt_f32 %2, %6, %10\n\tv_cmp_lt_f32 %3, %7, %11\n\t"
                        "v_cmp_lt_f32 %4, %8, %12\n\t"
                        "v_addc_co_u32 %0, vcc, %0, %0, %1\n\tv_addc_co_u32 %0, vcc, %0, %0, %2\n\t"
                        "v_addc_co_u32 %0, vcc, %0, %0, %3\n\tv_addc_co_u32 %0, vcc, %0, %0, %4"
                        : "+v"(hm), "=&s"(k0), "=&s"(k1), "=&s"(k2), "=&s"(k3)
                        : "v"(t4[0]), "v"(t4[1]), "v"(t4[2]), "v"(t4[3]), "v"(acc[fm][4 * q]), "v"(acc[fm][4 * q + 1]),
                          "v"(acc[fm][4 * q + 2]), "v"(acc[fm][4 * q + 3])
                        : "vcc");
                }
                if (!real_row) hm = 0u;
                const uint64_t any = __ballot(hm != 0u);
                if (any != 0ull) {
                    if (__ballot((hm & (hm - 1u)) != 0u) == 0ull) {
                        const int n = __popcll(any);
                        if (staged + n > GR_SYM_STAGE) flush();
                        if (hm != 0u) {
                            const int r = 15 - __builtin_ctz(hm);
                            const float v = gr_sym_pick16(acc[fm], r);
                            const int lr = fm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                            my_stage()[staged + __popcll(any & ((1ull << lane) - 1ull))] = gr_sym_record(c0 - sb * SB + lr, row0 + ks_soe_col(), v);
                        }
                        staged = __builtin_amdgcn_readfirstlane(staged + n);
                    } else { // a lane with several hits: row by row
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const bool hit = (hm >> (15 - r)) & 1u;
                            const uint64_t m = __ballot(hit);
                            if (m != 0ull) push(m, hit, c0 + ks_soe_row(fm, r, lane), acc[fm][r]);
                        }
                    }
                }
            }
        } else {
            // the workgroup's own super-block (which side is wanted depends on the streamed row's block) or a ragged end
            // (the lane number goes through an opaque copy: otherwise the compiler computes the 48 row numbers and what
            // follows from them once, before the sweep, and keeps them in registers that the sweep does not have)
            int lane_here = lane;
            asm volatile("" : "+v"(lane_here));
            const int gi = row0 + (threadIdx.x >> 6) * 32 + (lane_here & 31);
            const int own0 = sb_own * SB, kb = ring & 15, n_b = (ring >> 4) & 15, succ_b = ring >> 8;
#pragma unroll
            for (int fm = 0; fm < CFG::FM; ++fm) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int lr = ks_soe_row(fm, 4 * q + e, lane_here);
                        const int j = c0 + lr;
                        const float v = acc[fm][4 * q + e];
                        bool res_side = lr < rows_here, str_side = lr < rows_here;
                        if (sb == sb_own) {
                            int dd = (j - own0) / CFG::RES - kb; // ring distance from this block to the streamed row's block
                            if (dd < 0) dd += n_b;
                            const bool taken = dd >= 1 && dd <= succ_b;
                            res_side = res_side && ((dd == 0 && j != gi) || taken);
                            str_side = str_side && taken;
                        }
                        if (res_side && v > thf) append_res(j, v);
                        float t = INFINITY;
                        if (str_side && gi < C) t = thf_row[j];
                        const uint64_t m = __ballot(v > t);
                        if (m != 0ull) push(m, v > t, j, v);
                    }
                    asm volatile("" ::: "memory"); // one group at a time: no pile of threshold loads in flight
                }
            }
        }
    };
    ks_soe_sweep<CFG>(W, D, row0, C, W, D, nullptr, 0, 0, C, lds, epi, nullptr, 0, KsSoeNoPost(),
                      chunks + (int64_t)blockIdx.x * chunks_stride, my_plan[2], side);
    flush();
    if (row0 + ks_soe_col() < C) cnt_res[2 * (row0 + ks_soe_col()) + (lane >> 5)] = my_cnt;
}

// the stream-side records of a super-block go to the rows they belong to; one workgroup per super-block
__global__ void __launch_bounds__(1024)
gr_sym_scatter_kernel(const uint2 *__restrict__ log, const int32_t *__restrict__ logcnt, int C, const uint32_t *__restrict__ tbits,
                      uint64_t *__restrict__ cand, int32_t *__restrict__ cnt_str) {
    __shared__ int s_cnt[GR_SYM_SB];
    __shared__ uint32_t s_tb[GR_SYM_SB];
    const int sb = blockIdx.x, row0 = sb * GR_SYM_SB;
    for (int r = threadIdx.x; r < GR_SYM_SB; r += 1024) {
        s_cnt[r] = 0;
        s_tb[r] = row0 + r < C ? tbits[row0 + r] : 0xFFFFFFFFu;
    }
    __syncthreads();
    const int n_raw = logcnt[sb], n = n_raw < GR_SYM_LOGCAP ? n_raw : GR_SYM_LOGCAP;
    const uint2 *src = log + (int64_t)sb * GR_SYM_LOGCAP;
    for (int q0 = 0; q0 < n; q0 += 4 * 1024) { // four records per thread in flight
        uint2 rec[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int q = q0 + u * 1024 + (int)threadIdx.x;
            rec[u] = q < n ? src[q] : make_uint2(0u, 0xFFFFFFFFu); // (place 1023 of a super-block: dropped below)
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int jl = (int)(rec[u].y & 1023u); // (checked all the same: it becomes an address)
            const uint32_t other = rec[u].y >> 10;
            if (jl >= GR_SYM_SB || row0 + jl >= C || other >= (uint32_t)C) continue;
            if (rec[u].x <= s_tb[jl]) continue;  // passed its neighbour's threshold in the sweep's test, not its own
            const int slot = atomicAdd(&s_cnt[jl], 1);
            if (slot < GR_SYM_SCAP)
                cand[(int64_t)(row0 + jl) * GR_SYM_CAP + 2 * GR_SYM_Q + slot] = ((uint64_t)rec[u].x << 32) | (uint32_t)(0xFFFFFFFFu - other);
        }
    }
    __syncthreads();
    for (int r = threadIdx.x; r < GR_SYM_SB; r += 1024)
        if (row0 + r < C) cnt_str[row0 + r] = n_raw > GR_SYM_LOGCAP ? 0x7FFFFFFF : s_cnt[r]; // a lost record: all rows overflow
}

// k' best of a row's candidates to the front of its buffer; one wavefront per row
__global__ void __launch_bounds__(GR_NT)
gr_sym_select_kernel(int64_t C, int kprime, uint64_t *__restrict__ cand, const int32_t *__restrict__ cnt_res,
                     const int32_t *__restrict__ cnt_str, const uint32_t *__restrict__ tbits, int32_t *__restrict__ cnt_out,
                     uint32_t *__restrict__ thr_out, int32_t *__restrict__ cnt_all) {
    constexpr int E = GR_SYM_CAP / 64, Q = GR_SYM_Q;
    const int64_t i = (int64_t)blockIdx.x * (GR_NT / 64) + (threadIdx.x >> 6);
    if (i >= C) return;
    const int lane = threadIdx.x & 63;
    uint64_t *row = cand + i * GR_SYM_CAP;
    const int r0 = cnt_res[2 * i], r1 = cnt_res[2 * i + 1], rs = cnt_str[i];
    const bool overflow = r0 > Q || r1 > Q || rs > GR_SYM_SCAP;
    const int n0 = r0 < Q ? r0 : Q, n1 = r1 < Q ? r1 : Q, ns = rs < GR_SYM_SCAP ? rs : GR_SYM_SCAP;
    const int n = n0 + n1 + ns, nreg = (n + 63) >> 6;
    uint64_t val[E];
#pragma unroll
    for (int r = 0; r < E; ++r) {
        val[r] = 0ull; // below every real key
        if (r < nreg) {
            const int idx = r * 64 + lane;
            if (idx < n) val[r] = row[idx < n0 ? idx : (idx < n0 + n1 ? Q + (idx - n0) : 2 * Q + (idx - n0 - n1))];
        }
    }
    auto count_hi = [&](uint32_t t) {
        int c = 0;
#pragma unroll
        for (int r = 0; r < E; ++r)
            if (r < nreg) c += __popcll(__ballot((uint32_t)(val[r] >> 32) >= t));
        return c;
    };
    auto count_lo = [&](uint32_t hi, uint32_t t) {
        int c = 0;
#pragma unroll
        for (int r = 0; r < E; ++r)
            if (r < nreg) c += __popcll(__ballot((uint32_t)(val[r] >> 32) == hi && (uint32_t)val[r] >= t));
        return c;
    };
    uint64_t t = 1ull; // keeps every real key
    if (n > kprime) {
        uint32_t t_hi = 0;
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t c = t_hi | (1u << bit);
            if (count_hi(c) >= kprime) t_hi = c;
        }
        t = (uint64_t)t_hi << 32;
        if (count_hi(t_hi) != kprime) { // keys of equal value straddle the cut: the ids decide
            const int need = kprime - (t_hi == 0xFFFFFFFFu ? 0 : count_hi(t_hi + 1u));
            uint32_t t_lo = 0;
            for (int bit = 31; bit >= 0; --bit) {
                const uint32_t c = t_lo | (1u << bit);
                if (count_lo(t_hi, c) >= need) t_lo = c;
            }
            t |= t_lo;
        }
    }
    // the k' best to the front, the other candidates behind them (gr_sym_second_kernel may need them: a row whose k'
    // best do not certify its K-th neighbour is ranked again over everything the sweep found for it)
    const int kept = n > kprime ? kprime : n;
    int base = 0, rest = kept;
#pragma unroll
    for (int r = 0; r < E; ++r) {
        if (r < nreg) {
            const bool real = r * 64 + lane < n, keep = real && val[r] >= t;
            const uint64_t m = __ballot(keep), m2 = __ballot(real && !keep);
            const uint64_t below = (1ull << lane) - 1ull;
            if (keep) row[base + __popcll(m & below)] = val[r];
            else if (real) row[rest + __popcll(m2 & below)] = val[r];
            base += __popcll(m);
            rest += __popcll(m2);
        }
    }
    if (lane == 0) {
        cnt_all[i] = n;
        cnt_out[i] = kept;
        // what was left out is at or below the k'-th key if the cut dropped something, else at or below the row's
        // fixed threshold; after an overflow nothing is known about it
        thr_out[i] = overflow ? 0xFFFFFFFFu : (n > kprime ? (uint32_t)(t >> 32) : tbits[i]);
    }
}

// ------------------------------------------------------------------------------------------------
// canonical similarity: sum over d ascending of (double)a_d * (double)b_d, one fused multiply-add per
// term (the product of two fp32 or bf16 values is exact in fp64, so this equals multiply-then-add)
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ double gr_canon(const uint16_t *__restrict__ a, const uint16_t *__restrict__ b, int D) {
    double acc = 0.0;
    int d = 0;
    // whole 128-byte lines of b at a time: callers give every lane a row of its own, so a line that is only
    // partly consumed is evicted before the lane comes back to it and is fetched again
    for (; d + 64 <= D; d += 64) {
        uint4 vb[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) vb[q] = *(const uint4 *)(b + d + q * 8);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const uint4 va = *(const uint4 *)(a + d + q * 8);
            const uint32_t wa[4] = {va.x, va.y, va.z, va.w}, wb[4] = {vb[q].x, vb[q].y, vb[q].z, vb[q].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc = __builtin_fma((double)__uint_as_float(wa[e] << 16), (double)__uint_as_float(wb[e] << 16), acc);
                acc = __builtin_fma((double)__uint_as_float(wa[e] & 0xFFFF0000u),
                                    (double)__uint_as_float(wb[e] & 0xFFFF0000u), acc);
            }
        }
    }
    for (; d < D; d += 8) {
        uint4 va = *(const uint4 *)(a + d), vb = *(const uint4 *)(b + d);
        const uint32_t wa[4] = {va.x, va.y, va.z, va.w}, wb[4] = {vb.x, vb.y, vb.z, vb.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc = __builtin_fma((double)__uint_as_float(wa[e] << 16), (double)__uint_as_float(wb[e] << 16), acc);
            acc = __builtin_fma((double)__uint_as_float(wa[e] & 0xFFFF0000u), (double)__uint_as_float(wb[e] & 0xFFFF0000u),
                                acc);
        }
    }
    return acc;
}
__device__ __forceinline__ double gr_canon(const float *__restrict__ a, const float *__restrict__ b, int D) {
    double acc = 0.0;
    for (int d = 0; d < D; d += 4) {
        float4 va = *(const float4 *)(a + d), vb = *(const float4 *)(b + d);
        acc = __builtin_fma((double)va.x, (double)vb.x, acc);
        acc = __builtin_fma((double)va.y, (double)vb.y, acc);
        acc = __builtin_fma((double)va.z, (double)vb.z, acc);
        acc = __builtin_fma((double)va.w, (double)vb.w, acc);
    }
    return acc;
}

__device__ __forceinline__ bool gr_ranks_before(double s, int32_t j, double t, int32_t k) {
    return s > t || (s == t && j < k);
}

// ------------------------------------------------------------------------------------------------
// exact re-rank of the recalled candidates; one wavefront per row; kprime <= 256 (4 slots per lane)
// ------------------------------------------------------------------------------------------------
template <typename IN>
__global__ void __launch_bounds__(GR_NT)
gr_rerank_kernel(const IN *__restrict__ W, int64_t C, int D, int K, int cap, const uint64_t *__restrict__ cand,
                 const int32_t *__restrict__ cnt, const uint32_t *__restrict__ thr, const float *__restrict__ norms,
                 const uint32_t *__restrict__ maxnorm_bits, float gamma, int32_t *__restrict__ graph,
                 float *__restrict__ sims, int32_t *fb_count, int32_t *__restrict__ fb_rows) {
    const int64_t i = (int64_t)blockIdx.x * (GR_NT / 64) + (threadIdx.x >> 6);
    if (i >= C) return;
    const int lane = threadIdx.x & 63;
    const int n = cnt[i];
    if (n < K && lane == 0) fb_rows[atomicAdd(fb_count, 1)] = (int32_t)i; // no K-th candidate to certify
    double s[4];
    int32_t id[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int q = t * 64 + lane;
        s[t] = -INFINITY;
        id[t] = 0x7FFFFFFF;
        if (q < n) {
            const uint32_t j = 0xFFFFFFFFu - (uint32_t)cand[i * cap + q];
            if (j < (uint32_t)C) { // always true for keys written by the recall pass
                id[t] = (int32_t)j;
                s[t] = gr_canon(W + i * D, W + (int64_t)j * D, D);
            }
        }
    }
    int rank[4] = {0, 0, 0, 0};
    const int slots = (n + 63) >> 6;
    for (int t2 = 0; t2 < slots; ++t2) {
        double s2 = t2 == 0 ? s[0] : (t2 == 1 ? s[1] : (t2 == 2 ? s[2] : s[3]));
        int32_t id2 = t2 == 0 ? id[0] : (t2 == 1 ? id[1] : (t2 == 2 ? id[2] : id[3]));
        for (int src = 0; src < 64; ++src) {
            const double os = __shfl(s2, src, 64);
            const int32_t oid = __shfl(id2, src, 64);
            if (t2 * 64 + src < n) {
#pragma unroll
                for (int t = 0; t < 4; ++t) rank[t] += gr_ranks_before(os, oid, s[t], id[t]) ? 1 : 0;
            }
        }
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int q = t * 64 + lane;
        if (q < n && rank[t] < K) {
            graph[i * K + rank[t]] = id[t];
            if (sims) sims[i * K + rank[t]] = (float)s[t];
            if (rank[t] == K - 1) {
                // certificate: nothing that was dropped can reach the K-th exact similarity
                const uint32_t th = thr[i];
                bool certified = (th == 0u); // nothing was ever dropped
                if (!certified) {
                    const double eps = (double)gamma * (double)norms[i] * (double)__uint_as_float(*maxnorm_bits);
                    certified = s[t] > (double)gr_unorder(th) + eps;
                }
                if (!certified) fb_rows[atomicAdd(fb_count, 1)] = (int32_t)i;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// exhaustive fp64 search for the rows on the list
// ------------------------------------------------------------------------------------------------
template <typename IN>
__global__ void __launch_bounds__(GR_NT)
gr_exhaustive_kernel(const IN *__restrict__ W, int64_t C, int D, int K, const int32_t *__restrict__ fb_count,
                     const int32_t *__restrict__ fb_rows, double *__restrict__ scratch, int32_t *__restrict__ graph,
                     float *__restrict__ sims) {
    __shared__ double red_s[GR_NT];
    __shared__ int32_t red_j[GR_NT];
    __shared__ __attribute__((aligned(16))) IN row_i[GR_MAX_D];
    int n_fb = *fb_count;
    if (n_fb > C) n_fb = (int)C;
    double *my = scratch + (int64_t)blockIdx.x * C;
    for (int e = blockIdx.x; e < n_fb; e += gridDim.x) {
        const int64_t i = fb_rows[e];
        for (int d = threadIdx.x; d < D; d += GR_NT) row_i[d] = W[i * D + d];
        __syncthreads();
        for (int64_t j = threadIdx.x; j < C; j += GR_NT) my[j] = gr_canon(row_i, W + j * D, D);
        __syncthreads();
        double prev_s = INFINITY;
        int32_t prev_j = -1;
        for (int r = 0; r < K; ++r) {
            double best_s = -INFINITY;
            int32_t best_j = 0x7FFFFFFF;
            for (int64_t j = threadIdx.x; j < C; j += GR_NT) {
                if (j == i) continue;
                const double sj = my[j];
                if (gr_ranks_before(prev_s, prev_j, sj, (int32_t)j) && gr_ranks_before(sj, (int32_t)j, best_s, best_j)) {
                    best_s = sj;
                    best_j = (int32_t)j;
                }
            }
            red_s[threadIdx.x] = best_s;
            red_j[threadIdx.x] = best_j;
            __syncthreads();
            for (int o = GR_NT / 2; o > 0; o >>= 1) {
                if (threadIdx.x < o) {
                    if (gr_ranks_before(red_s[threadIdx.x + o], red_j[threadIdx.x + o], red_s[threadIdx.x], red_j[threadIdx.x])) {
                        red_s[threadIdx.x] = red_s[threadIdx.x + o];
                        red_j[threadIdx.x] = red_j[threadIdx.x + o];
                    }
                }
                __syncthreads();
            }
            prev_s = red_s[0];
            prev_j = red_j[0];
            if (threadIdx.x == 0) {
                graph[i * K + r] = prev_j;
                if (sims) sims[i * K + r] = (float)prev_s;
            }
            __syncthreads();
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Second chance for rows that the re-rank could not certify, after the pass that computes every similarity once: that pass
// leaves ALL rows above the row's fixed threshold in its buffer (some 400), not only the k' best, so the row is ranked
// again over all of them, and the certificate is taken against the fixed threshold, which lies far below the K-th
// neighbour.  It is what keeps tight clusters cheap: with hundreds of neighbours 2e-6 apart no k' of a few dozen
// spans the error bound, and the exhaustive search costs such a row 30 ms.  One wavefront per row; rows that still
// fail (a buffer overflowed; ties at the fixed threshold) go to the exhaustive list.
// ------------------------------------------------------------------------------------------------
template <typename IN>
__global__ void __launch_bounds__(GR_NT)
gr_sym_second_kernel(const IN *__restrict__ W, int64_t C, int D, int K, const uint64_t *__restrict__ cand,
                     const int32_t *__restrict__ cnt_all, const uint32_t *__restrict__ thr, const uint32_t *__restrict__ tbits,
                     const float *__restrict__ norms, const uint32_t *__restrict__ maxnorm_bits, float gamma,
                     const int32_t *__restrict__ list_count, const int32_t *__restrict__ list_rows, int32_t *__restrict__ graph,
                     float *__restrict__ sims, int32_t *fb_count, int32_t *__restrict__ fb_rows) {
    __shared__ double s_s[GR_NT / 64][GR_SYM_CAP];
    __shared__ int32_t s_id[GR_NT / 64][GR_SYM_CAP];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t n_list = *list_count;
    if (n_list > C) n_list = C;
    for (int64_t e0 = (int64_t)blockIdx.x * (GR_NT / 64); e0 < n_list; e0 += (int64_t)gridDim.x * (GR_NT / 64)) {
        const int64_t e = e0 + wave;
        const int64_t i = e < n_list ? list_rows[e] : -1;
        const bool usable = i >= 0 && thr[i] != 0xFFFFFFFFu; // (an overflowed buffer does not hold everything above the threshold)
        const int n = usable ? (cnt_all[i] < GR_SYM_CAP ? cnt_all[i] : GR_SYM_CAP) : 0;
        int n_valid = 0;
        for (int q0 = 0; q0 < n; q0 += 64) {
            const int q = q0 + lane;
            double sv = -INFINITY;
            int32_t id = 0x7FFFFFFF;
            if (q < n) {
                const uint32_t j = 0xFFFFFFFFu - (uint32_t)cand[i * GR_SYM_CAP + q];
                if (j < (uint32_t)C && (int64_t)j != i) { // always true for keys written by the recall pass
                    id = (int32_t)j;
                    sv = gr_canon(W + i * D, W + (int64_t)j * D, D);
                }
                s_s[wave][q] = sv;
                s_id[wave][q] = id;
            }
            n_valid += __popcll(__ballot(id != 0x7FFFFFFF));
        }
        __syncthreads();
        bool certified = usable && n_valid >= K;
        if (certified) {
            for (int q = lane; q < n; q += 64) {
                const double sv = s_s[wave][q];
                const int32_t id = s_id[wave][q];
                if (id == 0x7FFFFFFF) continue;
                int rank = 0;
                for (int p = 0; p < n && rank < K; ++p) rank += gr_ranks_before(s_s[wave][p], s_id[wave][p], sv, id) ? 1 : 0;
                if (rank < K) {
                    graph[i * K + rank] = id;
                    if (sims) sims[i * K + rank] = (float)sv;
                    if (rank == K - 1) {
                        const double eps = (double)gamma * (double)norms[i] * (double)__uint_as_float(*maxnorm_bits);
                        if (!(sv > (double)gr_unorder(tbits[i]) + eps)) certified = false;
                    }
                }
            }
        }
        if (i >= 0 && __ballot(!certified) != 0ull && lane == 0) fb_rows[atomicAdd(fb_count, 1)] = (int32_t)i;
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
struct GrWs {
    uint16_t *Wb;
    float *norms;
    uint32_t *maxnorm;
    uint64_t *cand;
    int32_t *cnt;
    uint32_t *thr;
    int32_t *fb_count;
    int32_t *fb_rows;
    double *scratch;
    // the pass that computes every similarity once (gr_sym_*), when it is used
    uint16_t *Ws;      // sampled rows
    float *thf;        // fixed thresholds
    uint32_t *tbits;
    int32_t *cnt_res, *cnt_str, *cnt_all, *logcnt, *plan;
    int32_t *second_count, *second_rows; // rows for gr_sym_second_kernel
    int2 *chunks;
    uint2 *log;
};

static unsigned gr_sym_grid(int64_t C) { // workgroups of the sweep: whole groups, dealt to the eight XCDs
    const int nsb = (int)ks_ceil_div(C, GR_SYM_SB), GS = gr_sym_group_sbs(C), NG = (nsb + GS - 1) / GS;
    return (unsigned)((NG + 7) / 8) * (unsigned)(GS * 3) * 8u;
}
static int gr_sym_chunks_stride(int64_t C) { // chunks a workgroup streams at most: half of all groups, half of its own, a spare
    const int64_t nsb = ks_ceil_div(C, GR_SYM_SB), GS = gr_sym_group_sbs(C), NG = ks_ceil_div(nsb, GS);
    return (int)(((NG / 2) * GS + GS / 2 + 2) * (GR_SYM_SB / 96));
}
// The pass that computes every similarity once pays off for problems of more than a few thousand rows.  A row's fixed
// threshold leaves 32 * Gamma(12) candidates (384 on average, fewer than 64 for one row in 10^7), which serves K <= 64:
// a row with fewer than k' candidates keeps them all and is certified against its fixed threshold.  A row id has 22
// bits in the stream side's records.
static bool gr_use_sym(int64_t C, int D, const GrParams &p) {
    return (D == 128 || D == 256 || D == 512) && p.kprime <= 128 && C >= 6144 && C <= ((int64_t)1 << 22);
}

static GrWs gr_carve(void *ws, int64_t C, int D, int K, int dtype, size_t *total) {
    KsArena ar(ws);
    GrParams p = gr_params(K, D);
    const GrParams pd = gr_params(K, D, dtype);
    const bool sym = gr_use_sym(C, D, pd);
    GrWs w;
    w.Wb = dtype == KS_DTYPE_FP32 ? ar.take<uint16_t>((size_t)C * D) : nullptr;
    w.norms = ar.take<float>((size_t)C);
    w.maxnorm = ar.take<uint32_t>(1);
    w.cand = ar.take<uint64_t>((size_t)C * (sym ? GR_SYM_CAP : p.cap));
    w.cnt = ar.take<int32_t>((size_t)C);
    w.thr = ar.take<uint32_t>((size_t)C);
    w.fb_count = ar.take<int32_t>(1);
    w.fb_rows = ar.take<int32_t>((size_t)C);
    w.scratch = ar.take<double>((size_t)GR_FB_BLOCKS * C);
    w.Ws = nullptr; w.thf = nullptr; w.tbits = nullptr; w.cnt_res = w.cnt_str = w.cnt_all = w.logcnt = w.plan = w.second_count = w.second_rows = nullptr; w.chunks = nullptr; w.log = nullptr;
    if (sym) {
        const int64_t nsb = ks_ceil_div(C, GR_SYM_SB), Cpad = nsb * GR_SYM_SB + 96;
        w.Ws = ar.take<uint16_t>((size_t)(C / GR_SYM_RATIO) * D);
        w.thf = ar.take<float>((size_t)Cpad);
        w.tbits = ar.take<uint32_t>((size_t)C);
        w.cnt_res = ar.take<int32_t>((size_t)C * 2);
        w.cnt_str = ar.take<int32_t>((size_t)C);
        w.cnt_all = ar.take<int32_t>((size_t)C);
        w.second_count = ar.take<int32_t>(1);
        w.second_rows = ar.take<int32_t>((size_t)C);
        w.logcnt = ar.take<int32_t>((size_t)nsb);
        w.plan = ar.take<int32_t>((size_t)gr_sym_grid(C) * GR_SYM_PLAN);
        w.chunks = ar.take<int2>((size_t)gr_sym_grid(C) * gr_sym_chunks_stride(C));
        w.log = ar.take<uint2>((size_t)nsb * GR_SYM_LOGCAP);
    }
    if (total) *total = ar.off;
    return w;
}

static int gr_check(int64_t C, int D, int K, int dtype) {
    if (dtype != KS_DTYPE_BF16 && dtype != KS_DTYPE_FP32) return KS_INVALID_ARG;
    if (C < 2 || C >= (int64_t)1 << 31 || D < 32 || D % 32 != 0 || K < 1) return KS_INVALID_ARG;
    if (K > KS_MAX_GRAPH_K || K > C - 1 || D > GR_MAX_D) return KS_UNSUPPORTED;
    return KS_OK;
}

extern "C" int knn_graph_build_plan(int64_t C, int D, int K, int dtype, int workgroup, int32_t *n_workgroups, int32_t *out) {
    if (!n_workgroups) return KS_INVALID_ARG;
    int rc = gr_check(C, D, K, dtype);
    if (rc != KS_OK) return rc;
    *n_workgroups = 0;
    if (!gr_use_sym(C, D, gr_params(K, D, dtype))) return KS_OK;
    *n_workgroups = (int32_t)gr_sym_grid(C);
    if (!out) return KS_OK;
    if (workgroup < 0 || workgroup >= *n_workgroups) return KS_INVALID_ARG;
    const GrSymRanges r = gr_sym_ranges(workgroup, (int)C, gr_sym_group_sbs(C));
    out[0] = r.block;
    for (int part = 0; part < 5; ++part) { out[1 + 2 * part] = r.first[part]; out[2 + 2 * part] = r.end[part]; }
    // which of the (up to three) 256-row blocks of its own super-block it pairs with: bit k = block k of that super-block
    int mask = 0;
    if (r.block >= 0) {
        const int kb = r.ring & 15, n_b = (r.ring >> 4) & 15, succ_b = r.ring >> 8;
        for (int k = 0; k < n_b; ++k) {
            const int dd = (k - kb + n_b) % n_b;
            if (dd >= 1 && dd <= succ_b) mask |= 1 << k;
        }
    }
    out[11] = mask;
    return KS_OK;
}

extern "C" size_t knn_graph_build_workspace(int64_t C, int D, int K, int dtype) {
    if (gr_check(C, D, K, dtype) != KS_OK) return 0;
    size_t total = 0;
    gr_carve(nullptr, C, D, K, dtype, &total);
    return total;
}

template <typename IN>
static void gr_launch_exact(const IN *W, int64_t C, int D, int K, const GrParams &p, const GrWs &w, float gamma,
                            int32_t *graph, float *sims, hipStream_t st, bool second_chance) {
    // (after the pass that computes every similarity once, uncertified rows get a second chance before the exhaustive list)
    hipLaunchKernelGGL(gr_rerank_kernel<IN>, dim3((unsigned)ks_ceil_div(C, GR_NT / 64)), dim3(GR_NT), 0, st, W, C, D, K, p.cap,
                       w.cand, w.cnt, w.thr, w.norms, w.maxnorm, gamma, graph, sims, second_chance ? w.second_count : w.fb_count,
                       second_chance ? w.second_rows : w.fb_rows);
    if (second_chance)
        hipLaunchKernelGGL(gr_sym_second_kernel<IN>, dim3(1024), dim3(GR_NT), 0, st, W, C, D, K, w.cand, w.cnt_all, w.thr, w.tbits,
                           w.norms, w.maxnorm, gamma, w.second_count, w.second_rows, graph, sims, w.fb_count, w.fb_rows);
    hipLaunchKernelGGL(gr_exhaustive_kernel<IN>, dim3(GR_FB_BLOCKS), dim3(GR_NT), 0, st, W, C, D, K, w.fb_count, w.fb_rows,
                       w.scratch, graph, sims);
}

// thr_init (optional, honoured by the sweep kernel only, may be `thr`): per row the value bits of a similarity at or below
// which no candidate is wanted
static void gr_launch_recall(const GrPair &pr, int D, const GrParams &p, uint64_t *cand, int32_t *cnt, uint32_t *thr,
                             hipStream_t st, const uint32_t *thr_init = nullptr) {
    const int64_t C = pr.Cr;
    if (D == 128 || D == 256 || D == 512) {
        const unsigned nb = (unsigned)ks_ceil_div(C, 256);
#define GR_SOE_LAUNCH(KT)                                                                                                   \
    do {                                                                                                                    \
        if (p.cap == 256)                                                                                                   \
            hipLaunchKernelGGL((gr_recall_soe_kernel<KT, 4>), dim3(nb), dim3(512), 0, st, pr, D, p.kprime, cand, cnt, thr,  \
                               thr_init);                                                                                   \
        else                                                                                                                \
            hipLaunchKernelGGL((gr_recall_soe_kernel<KT, 8>), dim3(nb), dim3(512), 0, st, pr, D, p.kprime, cand, cnt, thr,  \
                               thr_init);                                                                                   \
    } while (0)
        if (D == 512) GR_SOE_LAUNCH(8);
        else if (D == 256) GR_SOE_LAUNCH(4);
        else GR_SOE_LAUNCH(2);
#undef GR_SOE_LAUNCH
    } else if (D % 64 == 0) {
        hipLaunchKernelGGL((gr_recall_async_kernel<TileRA, 8>), dim3((unsigned)ks_ceil_div(C, TileRA::BM)), dim3(TileRA::NT), 0,
                           st, pr, D, p.kprime, cand, cnt, thr);
    } else {
        const unsigned recall_blocks = (unsigned)ks_ceil_div(C, TileR::BM);
        if (p.cap == 256)
            hipLaunchKernelGGL((gr_recall_kernel<TileR, 4>), dim3(recall_blocks), dim3(TileR::NT), 0, st, pr, D, p.kprime, cand,
                               cnt, thr);
        else
            hipLaunchKernelGGL((gr_recall_kernel<TileR, 8>), dim3(recall_blocks), dim3(TileR::NT), 0, st, pr, D, p.kprime, cand,
                               cnt, thr);
    }
}

// W searched in W with every similarity computed once: thresholds from a sample, the sweep, the stream side's records
// to their rows, the cut to k'
static void gr_launch_recall_sym(const uint16_t *Wb, int64_t C, int D, int K, const GrParams &p, const GrWs &w, hipStream_t st) {
    const int ratio = GR_SYM_RATIO;
    const int64_t n_sample = C / ratio;
    const int nsb = (int)ks_ceil_div(C, GR_SYM_SB);
    const int64_t Cpad = (int64_t)nsb * GR_SYM_SB + 96;
    hipLaunchKernelGGL(gr_sym_sample_kernel, dim3((unsigned)ks_ceil_div(n_sample, GR_NT / 64)), dim3(GR_NT), 0, st, Wb, C, D, ratio,
                       n_sample, w.Ws);
    // the sample is searched with the kernel of the plain pass: GR_SYM_RANK kept, no row is "the row itself" (the
    // sample may hold it; it counts like any other row)
    GrParams ps = p;
    ps.kprime = GR_SYM_RANK;
    ps.cap = 256;
    const GrPair pr{Wb, C, w.Ws, n_sample, -((int64_t)1 << 40)};
    gr_launch_recall(pr, D, ps, w.cand, w.cnt, w.thr, st);
    hipLaunchKernelGGL(gr_sym_prep_kernel, dim3((unsigned)ks_ceil_div(Cpad, GR_NT)), dim3(GR_NT), 0, st, w.thr, C, Cpad, w.thf,
                       w.tbits, w.logcnt, nsb, w.second_count);
    const unsigned grid = gr_sym_grid(C);
    const int stride = gr_sym_chunks_stride(C);
    hipLaunchKernelGGL(gr_sym_plan_kernel, dim3(grid), dim3(GR_NT), 0, st, (int)C, gr_sym_group_sbs(C), w.plan, w.chunks, stride);
    if (D == 512)
        hipLaunchKernelGGL((gr_recall_sym_kernel<8>), dim3(grid), dim3(512), 0, st, Wb, (int)C, D, w.plan, w.chunks, stride, w.thf, w.cand,
                           w.cnt_res, w.log, w.logcnt);
    else if (D == 256)
        hipLaunchKernelGGL((gr_recall_sym_kernel<4>), dim3(grid), dim3(512), 0, st, Wb, (int)C, D, w.plan, w.chunks, stride, w.thf, w.cand,
                           w.cnt_res, w.log, w.logcnt);
    else
        hipLaunchKernelGGL((gr_recall_sym_kernel<2>), dim3(grid), dim3(512), 0, st, Wb, (int)C, D, w.plan, w.chunks, stride, w.thf, w.cand,
                           w.cnt_res, w.log, w.logcnt);
    hipLaunchKernelGGL(gr_sym_scatter_kernel, dim3((unsigned)nsb), dim3(1024), 0, st, w.log, w.logcnt, (int)C, w.tbits, w.cand,
                       w.cnt_str);
    // (Handing the re-rank only K + 8 candidates of bf16 rows saves it 0.6 of 5.2 ms at the headline size, and costs rows
    // of tight clusters their certificate: with neighbours 2e-5 apart, eight of them span less than the error bound for
    // four rows in ten, and an uncertified row costs a millisecond.)
    const int kept = p.kprime;
    hipLaunchKernelGGL(gr_sym_select_kernel, dim3((unsigned)ks_ceil_div(C, GR_NT / 64)), dim3(GR_NT), 0, st, C, kept, w.cand,
                       w.cnt_res, w.cnt_str, w.tbits, w.cnt, w.thr, w.cnt_all);
}

// error bound of the recall pass relative to |w_i||w_j|: fp32 accumulation of D exact bf16 products
// (2^-23 per addition allows for truncating adders), plus the bf16 rounding of both rows (2 * 2^-9,
// rounded up to 2^-7.9) when the input is fp32; a small slack covers the fp32 norms themselves
static float gr_gamma(int D, int dtype) {
    float gamma = (float)D * 1.1920929e-7f * 1.01f;
    if (dtype == KS_DTYPE_FP32) gamma += 0.0042f;
    return gamma;
}

extern "C" int knn_graph_build(const void *W, int dtype, int64_t C, int D, int K, int32_t *graph, float *sims, void *ws,
                               size_t ws_bytes, int32_t *dev_status, void *stream) {
    (void)dev_status;
    if (!W || !graph || !ws) return KS_INVALID_ARG;
    int rc = gr_check(C, D, K, dtype);
    if (rc != KS_OK) return rc;
    size_t need = 0;
    GrWs w = gr_carve(ws, C, D, K, dtype, &need);
    if (ws_bytes < need) return KS_WORKSPACE_TOO_SMALL;
    const GrParams p = gr_params(K, D, dtype);
    hipStream_t st = (hipStream_t)stream;

    hipLaunchKernelGGL(gr_zero_kernel, dim3(1), dim3(1), 0, st, w.maxnorm, w.fb_count);
    const unsigned row_blocks = (unsigned)ks_ceil_div(C, GR_NT / 64);
    const uint16_t *Wb;
    if (dtype == KS_DTYPE_FP32) {
        hipLaunchKernelGGL(gr_prepare_kernel<float>, dim3(row_blocks), dim3(GR_NT), 0, st, (const float *)W, C, D, w.Wb,
                           w.norms, w.maxnorm);
        Wb = w.Wb;
    } else {
        hipLaunchKernelGGL(gr_prepare_kernel<uint16_t>, dim3(row_blocks), dim3(GR_NT), 0, st, (const uint16_t *)W, C, D,
                           (uint16_t *)nullptr, w.norms, w.maxnorm);
        Wb = (const uint16_t *)W;
    }
    GrParams pe = p; // what the exact stage reads
    const bool sym = gr_use_sym(C, D, p);
    if (sym) {
        gr_launch_recall_sym(Wb, C, D, K, p, w, st);
        pe.cap = GR_SYM_CAP;
    } else {
        const GrPair pr{Wb, C, Wb, C, 0};
        gr_launch_recall(pr, D, p, w.cand, w.cnt, w.thr, st);
    }
    const float gamma = gr_gamma(D, dtype);
    if (dtype == KS_DTYPE_FP32) gr_launch_exact<float>((const float *)W, C, D, K, pe, w, gamma, graph, sims, st, sym);
    else gr_launch_exact<uint16_t>((const uint16_t *)W, C, D, K, pe, w, gamma, graph, sims, st, sym);
    KS_LAUNCH_CHECK();
    return KS_OK;
}

// ------------------------------------------------------------------------------------------------
// One hop of the distributed graph build (Section 3.2.2: the shards of W travel from node to node, each node
// searches every visiting shard and keeps its rows' best K so far).  Recall pass of the node's rows against the
// visiting rows as above; then per row an exact merge of the recalled candidates with the list so far, on
// (canonical fp64 similarity descending, id of the whole problem ascending), with the same certificate; rows
// that fail it are merged against every visiting row.
// ------------------------------------------------------------------------------------------------
#define GR_NO_ID 0x7FFFFFFF

// one wavefront per row; k' <= 256 candidates (slots 0..3) + K <= 128 list entries (slots 4, 5) per lane
template <typename IN>
__global__ void __launch_bounds__(GR_NT)
gr_merge_kernel(const IN *__restrict__ Wl, int64_t C_loc, const IN *__restrict__ Wv, int64_t C_vis, int D, int K, int cap,
                const uint64_t *__restrict__ cand, const int32_t *__restrict__ cnt, const uint32_t *__restrict__ thr,
                const float *__restrict__ norms, const uint32_t *__restrict__ maxnorm_bits, float gamma, int64_t local_offset,
                int64_t visit_offset, int32_t *__restrict__ graph, double *__restrict__ sims, int32_t *fb_count,
                int32_t *__restrict__ fb_rows) {
    const int64_t i = (int64_t)blockIdx.x * (GR_NT / 64) + (threadIdx.x >> 6);
    if (i >= C_loc) return;
    const int lane = threadIdx.x & 63;
    const int n = cnt[i];
    double s[6];
    int32_t id[6];
#pragma unroll
    for (int t = 4; t < 6; ++t) { // the list so far
        const int e = (t - 4) * 64 + lane;
        s[t] = -INFINITY;
        id[t] = GR_NO_ID;
        if (e < K) {
            const int32_t g = graph[i * K + e];
            if (g >= 0) {
                id[t] = g;
                s[t] = sims[i * K + e];
            }
        }
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) { // the recalled candidates
        const int q = t * 64 + lane;
        s[t] = -INFINITY;
        id[t] = GR_NO_ID;
        if (q < n) {
            const uint32_t j = 0xFFFFFFFFu - (uint32_t)cand[i * cap + q];
            if (j < (uint64_t)C_vis) { // always true for keys written by the recall pass
                id[t] = (int32_t)(visit_offset + j);
                s[t] = gr_canon(Wl + i * D, Wv + (int64_t)j * D, D);
            }
        }
    }
    // a visiting row that is in the list already (a shard seen twice) is not a new candidate
    const int list_slots = (K + 63) >> 6;
    for (int t2 = 0; t2 < list_slots; ++t2) {
        const int32_t mine = t2 == 0 ? id[4] : id[5];
        for (int src = 0; src < 64; ++src) {
            const int32_t oid = __shfl(mine, src, 64);
            if (oid == GR_NO_ID) continue;
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (id[t] == oid) {
                    id[t] = GR_NO_ID;
                    s[t] = -INFINITY;
                }
        }
    }
    int rank[6] = {0, 0, 0, 0, 0, 0};
    int n_valid = 0;
    const int cand_slots = (n + 63) >> 6;
#pragma unroll
    for (int t2 = 0; t2 < 6; ++t2) {
        if (t2 < 4 ? t2 >= cand_slots : t2 - 4 >= list_slots) continue; // uniform over the wavefront
        n_valid += __popcll(__ballot(id[t2] != GR_NO_ID));
        for (int src = 0; src < 64; ++src) {
            const double os = __shfl(s[t2], src, 64);
            const int32_t oid = __shfl(id[t2], src, 64);
            if (oid == GR_NO_ID) continue;
#pragma unroll
            for (int t = 0; t < 6; ++t) rank[t] += gr_ranks_before(os, oid, s[t], id[t]) ? 1 : 0;
        }
    }
    bool certified = true;
#pragma unroll
    for (int t = 0; t < 6; ++t) {
        if (id[t] != GR_NO_ID && rank[t] < K) {
            graph[i * K + rank[t]] = id[t];
            sims[i * K + rank[t]] = s[t];
            if (rank[t] == K - 1) {
                // certificate: no visiting row that the recall pass dropped can reach the K-th exact similarity
                const uint32_t th = thr[i];
                if (th != 0u) {
                    const double eps = (double)gamma * (double)norms[i] * (double)__uint_as_float(*maxnorm_bits);
                    certified = s[t] > (double)gr_unorder(th) + eps;
                }
            }
        }
    }
    for (int e = n_valid + lane; e < K; e += 64) { // fewer than K known so far: empty slots
        graph[i * K + e] = -1;
        sims[i * K + e] = -INFINITY;
    }
    if (n_valid < K && thr[i] != 0u) certified = false; // cannot happen (something was dropped, so k' >= K were kept)
    if (__ballot(!certified) != 0ull && lane == 0) fb_rows[atomicAdd(fb_count, 1)] = (int32_t)i;
}

// A row whose list is full needs no visiting row whose similarity cannot reach the list's last entry: the recall pass
// starts from that entry's similarity, lowered by more than twice the recall's error bound (a visiting row that ties
// the entry exactly is still recalled, and the certificate of the merge -- new K-th similarity above threshold + bound
// -- holds when nothing new comes in).  0: no threshold (the list has empty slots).
__global__ void __launch_bounds__(GR_NT)
gr_hop_threshold_kernel(int64_t C_loc, int K, const int32_t *__restrict__ graph, const double *__restrict__ sims,
                        const float *__restrict__ norms, const uint32_t *__restrict__ maxnorm_bits, float gamma,
                        uint32_t *__restrict__ thr) {
    const int64_t i = (int64_t)blockIdx.x * GR_NT + threadIdx.x;
    if (i >= C_loc) return;
    uint32_t t = 0u;
    if (graph[i * K + K - 1] >= 0) {
        const double eps = (double)gamma * (double)norms[i] * (double)__uint_as_float(*maxnorm_bits);
        const double want = sims[i * K + K - 1] - 2.5 * eps;
        float f = (float)want;
        if ((double)f > want) f = nextafterf(f, -INFINITY); // rounded down
        if (f == f && f > -INFINITY) t = gr_orderable(f);
    }
    thr[i] = t;
}

// rows on the list: every visiting row in canonical fp64 arithmetic, merged with the row's list
template <typename IN>
__global__ void __launch_bounds__(GR_NT)
gr_exhaustive_merge_kernel(const IN *__restrict__ Wl, int64_t C_loc, const IN *__restrict__ Wv, int64_t C_vis, int D, int K,
                           int64_t local_offset, int64_t visit_offset, const int32_t *__restrict__ fb_count,
                           const int32_t *__restrict__ fb_rows, double *__restrict__ scratch, int32_t *__restrict__ graph,
                           double *__restrict__ sims) {
    __shared__ double red_s[GR_NT];
    __shared__ int32_t red_j[GR_NT];
    __shared__ __attribute__((aligned(16))) IN row_i[GR_MAX_D];
    __shared__ double l_s[KS_MAX_GRAPH_K], o_s[KS_MAX_GRAPH_K];
    __shared__ int32_t l_id[KS_MAX_GRAPH_K], o_id[KS_MAX_GRAPH_K];
    int n_fb = *fb_count;
    if (n_fb > C_loc) n_fb = (int)C_loc;
    double *my = scratch + (int64_t)blockIdx.x * C_vis;
    for (int e = blockIdx.x; e < n_fb; e += gridDim.x) {
        const int64_t i = fb_rows[e];
        for (int d = threadIdx.x; d < D; d += GR_NT) row_i[d] = Wl[i * D + d];
        for (int k = threadIdx.x; k < K; k += GR_NT) {
            l_id[k] = graph[i * K + k];
            l_s[k] = sims[i * K + k];
        }
        __syncthreads();
        for (int64_t j = threadIdx.x; j < C_vis; j += GR_NT) my[j] = gr_canon(row_i, Wv + j * D, D);
        __syncthreads();
        // the row itself and visiting rows that are in the list already are no candidates (-inf marks them: the
        // similarity of real rows is finite)
        if (threadIdx.x == 0) {
            const int64_t js = local_offset + i - visit_offset;
            if (js >= 0 && js < C_vis) my[js] = -INFINITY;
        }
        for (int k = threadIdx.x; k < K; k += GR_NT) {
            const int64_t jl = (int64_t)l_id[k] - visit_offset;
            if (l_id[k] >= 0 && jl >= 0 && jl < C_vis) my[jl] = -INFINITY;
        }
        __syncthreads();
        double prev_s = INFINITY;
        int32_t prev_j = -1;
        for (int r = 0; r < K; ++r) {
            double best_s = -INFINITY;
            int32_t best_j = GR_NO_ID;
            for (int64_t j = threadIdx.x; j < C_vis; j += GR_NT) {
                const double sj = my[j];
                if (sj == -INFINITY) continue;
                const int32_t gj = (int32_t)(visit_offset + j);
                if (gr_ranks_before(prev_s, prev_j, sj, gj) && gr_ranks_before(sj, gj, best_s, best_j)) {
                    best_s = sj;
                    best_j = gj;
                }
            }
            for (int k = threadIdx.x; k < K; k += GR_NT) {
                if (l_id[k] < 0) continue;
                if (gr_ranks_before(prev_s, prev_j, l_s[k], l_id[k]) && gr_ranks_before(l_s[k], l_id[k], best_s, best_j)) {
                    best_s = l_s[k];
                    best_j = l_id[k];
                }
            }
            red_s[threadIdx.x] = best_s;
            red_j[threadIdx.x] = best_j;
            __syncthreads();
            for (int o = GR_NT / 2; o > 0; o >>= 1) {
                if (threadIdx.x < o) {
                    if (gr_ranks_before(red_s[threadIdx.x + o], red_j[threadIdx.x + o], red_s[threadIdx.x], red_j[threadIdx.x])) {
                        red_s[threadIdx.x] = red_s[threadIdx.x + o];
                        red_j[threadIdx.x] = red_j[threadIdx.x + o];
                    }
                }
                __syncthreads();
            }
            prev_s = red_s[0];
            prev_j = red_j[0];
            if (threadIdx.x == 0) {
                o_id[r] = prev_j == GR_NO_ID ? -1 : prev_j;
                o_s[r] = prev_j == GR_NO_ID ? -INFINITY : prev_s;
            }
            __syncthreads();
            if (prev_j == GR_NO_ID) { // nothing left: the remaining slots are empty
                for (int k = r + 1 + threadIdx.x; k < K; k += GR_NT) { o_id[k] = -1; o_s[k] = -INFINITY; }
                break;
            }
        }
        __syncthreads();
        for (int k = threadIdx.x; k < K; k += GR_NT) {
            graph[i * K + k] = o_id[k];
            sims[i * K + k] = o_s[k];
        }
        __syncthreads();
    }
}

struct GrUpWs {
    uint16_t *Wlb, *Wvb;
    float *norms_l, *norms_v;
    uint32_t *maxnorm_l, *maxnorm_v;
    uint64_t *cand;
    int32_t *cnt;
    uint32_t *thr;
    int32_t *fb_count;
    int32_t *fb_rows;
    double *scratch;
};
static GrUpWs gr_up_carve(void *ws, int64_t C_loc, int64_t C_vis, int D, int K, int dtype, size_t *total) {
    KsArena ar(ws);
    GrParams p = gr_params(K, D);
    GrUpWs w;
    w.Wlb = dtype == KS_DTYPE_FP32 ? ar.take<uint16_t>((size_t)C_loc * D) : nullptr;
    w.Wvb = dtype == KS_DTYPE_FP32 ? ar.take<uint16_t>((size_t)C_vis * D) : nullptr;
    w.norms_l = ar.take<float>((size_t)C_loc);
    w.norms_v = ar.take<float>((size_t)C_vis);
    w.maxnorm_l = ar.take<uint32_t>(1);
    w.maxnorm_v = ar.take<uint32_t>(1);
    w.cand = ar.take<uint64_t>((size_t)C_loc * p.cap);
    w.cnt = ar.take<int32_t>((size_t)C_loc);
    w.thr = ar.take<uint32_t>((size_t)C_loc);
    w.fb_count = ar.take<int32_t>(1);
    w.fb_rows = ar.take<int32_t>((size_t)C_loc);
    w.scratch = ar.take<double>((size_t)GR_FB_BLOCKS * C_vis);
    if (total) *total = ar.off;
    return w;
}
static int gr_up_check(int64_t C_loc, int64_t C_vis, int D, int K, int dtype, int64_t lo, int64_t vo) {
    if (dtype != KS_DTYPE_BF16 && dtype != KS_DTYPE_FP32) return KS_INVALID_ARG;
    if (C_loc < 1 || C_vis < 1 || D < 32 || D % 32 != 0 || K < 1 || lo < 0 || vo < 0) return KS_INVALID_ARG;
    if (lo + C_loc >= (int64_t)1 << 31 || vo + C_vis >= (int64_t)1 << 31) return KS_INVALID_ARG;
    if (K > KS_MAX_GRAPH_K || D > GR_MAX_D) return KS_UNSUPPORTED;
    return KS_OK;
}

extern "C" size_t knn_graph_update_workspace(int64_t C_loc, int64_t C_vis, int D, int K, int dtype) {
    if (gr_up_check(C_loc, C_vis, D, K, dtype, 0, 0) != KS_OK) return 0;
    size_t total = 0;
    gr_up_carve(nullptr, C_loc, C_vis, D, K, dtype, &total);
    return total;
}

template <typename IN>
static void gr_up_prepare(const IN *W, int64_t C, int D, uint16_t *Wb, float *norms, uint32_t *maxnorm, hipStream_t st) {
    hipLaunchKernelGGL(gr_prepare_kernel<IN>, dim3((unsigned)ks_ceil_div(C, GR_NT / 64)), dim3(GR_NT), 0, st, W, C, D, Wb, norms,
                       maxnorm);
}
template <typename IN>
static void gr_up_exact(const IN *Wl, int64_t C_loc, const IN *Wv, int64_t C_vis, int D, int K, const GrParams &p,
                        const GrUpWs &w, float gamma, int64_t lo, int64_t vo, int32_t *graph, double *sims, hipStream_t st) {
    hipLaunchKernelGGL(gr_merge_kernel<IN>, dim3((unsigned)ks_ceil_div(C_loc, GR_NT / 64)), dim3(GR_NT), 0, st, Wl, C_loc, Wv,
                       C_vis, D, K, p.cap, w.cand, w.cnt, w.thr, w.norms_l, w.maxnorm_v, gamma, lo, vo, graph, sims, w.fb_count,
                       w.fb_rows);
    hipLaunchKernelGGL(gr_exhaustive_merge_kernel<IN>, dim3(GR_FB_BLOCKS), dim3(GR_NT), 0, st, Wl, C_loc, Wv, C_vis, D, K, lo, vo,
                       w.fb_count, w.fb_rows, w.scratch, graph, sims);
}

extern "C" int knn_graph_update(const void *W_local, const void *W_visit, int dtype, int64_t C_loc, int64_t C_vis, int D, int K,
                                int64_t local_offset, int64_t visit_offset, int32_t *graph, double *sims, void *ws,
                                size_t ws_bytes, int32_t *dev_status, void *stream) {
    (void)dev_status;
    if (!W_local || !W_visit || !graph || !sims || !ws) return KS_INVALID_ARG;
    int rc = gr_up_check(C_loc, C_vis, D, K, dtype, local_offset, visit_offset);
    if (rc != KS_OK) return rc;
    size_t need = 0;
    GrUpWs w = gr_up_carve(ws, C_loc, C_vis, D, K, dtype, &need);
    if (ws_bytes < need) return KS_WORKSPACE_TOO_SMALL;
    const GrParams p = gr_params(K, D, dtype);
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(gr_zero_kernel, dim3(1), dim3(1), 0, st, w.maxnorm_l, w.fb_count);
    hipLaunchKernelGGL(gr_zero_kernel, dim3(1), dim3(1), 0, st, w.maxnorm_v, w.fb_count);
    const uint16_t *Rl, *Sv;
    if (dtype == KS_DTYPE_FP32) {
        gr_up_prepare<float>((const float *)W_local, C_loc, D, w.Wlb, w.norms_l, w.maxnorm_l, st);
        gr_up_prepare<float>((const float *)W_visit, C_vis, D, w.Wvb, w.norms_v, w.maxnorm_v, st);
        Rl = w.Wlb;
        Sv = w.Wvb;
    } else {
        gr_up_prepare<uint16_t>((const uint16_t *)W_local, C_loc, D, nullptr, w.norms_l, w.maxnorm_l, st);
        gr_up_prepare<uint16_t>((const uint16_t *)W_visit, C_vis, D, nullptr, w.norms_v, w.maxnorm_v, st);
        Rl = (const uint16_t *)W_local;
        Sv = (const uint16_t *)W_visit;
    }
    const GrPair pr{Rl, C_loc, Sv, C_vis, local_offset - visit_offset};
    const float gamma = gr_gamma(D, dtype);
    hipLaunchKernelGGL(gr_hop_threshold_kernel, dim3((unsigned)ks_ceil_div(C_loc, GR_NT)), dim3(GR_NT), 0, st, C_loc, K, graph, sims,
                       w.norms_l, w.maxnorm_v, gamma, w.thr);
    gr_launch_recall(pr, D, p, w.cand, w.cnt, w.thr, st, w.thr);
    if (dtype == KS_DTYPE_FP32)
        gr_up_exact<float>((const float *)W_local, C_loc, (const float *)W_visit, C_vis, D, K, p, w, gamma, local_offset,
                           visit_offset, graph, sims, st);
    else
        gr_up_exact<uint16_t>((const uint16_t *)W_local, C_loc, (const uint16_t *)W_visit, C_vis, D, K, p, w, gamma,
                              local_offset, visit_offset, graph, sims, st);
    KS_LAUNCH_CHECK();
    return KS_OK;
}
