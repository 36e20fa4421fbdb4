// Stationary-operand MFMA sweep for gfx950 (bf16 in, fp32 accumulate).
//
// Computes, chunk by chunk, the products  C[m][n] = sum_k S[m][k] * R[n][k]  of a long list of "streamed"
// rows S (m) with a block of 256 "resident" rows R (n), both stored with k contiguous, for a depth
// K = 64 * KT that is small enough to keep the resident block's MFMA fragments in registers for the whole
// sweep (KT <= 8).  Only the streamed rows travel through LDS (global_load_lds, several CH-row x 64-k tiles
// in flight), so each byte fetched from L2 feeds 256 multiply-adds instead of the 128 of a tile engine that
// streams both operands, and the chunk size can be cut at any multiple of 32, which lets callers split the
// streamed rows evenly over the chip.
//
// Workgroup = EIGHT wavefronts, two per SIMD; wavefront w owns resident rows [32 w, 32 w + 32): one 32-column
// MFMA block, 128 registers of fragments for K = 512, so a lane stays within 256 registers and a SIMD holds two
// wavefronts.  While one of them waits (for a barrier, for its fragments, in its epilogue's exponentials and
// stores) the other one's MFMAs keep the matrix pipe busy.  The price is LDS traffic: every wavefront reads the
// whole streamed tile for half as many MFMAs as with four wavefronts of 64 resident rows.  Measured against that
// four-wavefront layout: 1.18 instead of 1.00 PFLOP/s on a plain sweep, the softmax sweep of the headline shape
// 34 instead of 40 us, the graph's recall pass 214 instead of 296 ms.
//
// MFMA orientation: streamed rows are the MFMA rows, resident rows the MFMA columns, so in the accumulator a
// lane owns ONE resident row (column lane % 32) and 16 streamed rows per 32-row block: reductions along the
// streamed rows for a fixed resident row (softmax statistics per sample, running thresholds per graph row) are
// lane-local.  Streamed tiles are loaded by wavefronts 0..3 (CH / 32 eight-row instructions each per k-tile).
//
// After every chunk (all KT k-tiles of CH streamed rows) the caller's epilogue functor gets the
// accumulators; the loads of the next chunk are already in flight at that point.
#pragma once
#include <type_traits>
#include "ks_gemm_async.h"

template <int KT_, int CH_, int STAGES_, int KSUB_ = 1> struct KsSoe {
    static constexpr int KT = KT_, STAGES = STAGES_, KSUB = KSUB_;
    static constexpr int NW = 8, NT = 512, CH = CH_, RES = 256;
    static constexpr int FM = CH / 32;
    static constexpr int LW = 4;       // wavefronts that issue the stream loads: 0..3, one per SIMD (see the sweep)
    static constexpr int NI = CH / 32; // load instructions per loading wavefront per k-tile (8 rows each)
    static constexpr int STAGE_ELEMS = KSUB * CH * 64;
    static constexpr int LDS_ELEMS = STAGES * STAGE_ELEMS;
    static_assert(KT >= 1 && KT <= 8 && KT % KSUB == 0 && STAGES >= 2 && (STAGES - 2) * NI * KSUB <= 63 && CH % 32 == 0 &&
                      LW <= NW,
                  "sweep shape");
};

// Row of the streamed chunk that accumulator element (fm, r) of this lane belongs to.
__device__ __forceinline__ int ks_soe_row(int fm, int r, int lane) { return fm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }
// Resident row (inside the workgroup's block of 256) of this lane's accumulator column.
__device__ __forceinline__ int ks_soe_col() { return (threadIdx.x >> 6) * 32 + (threadIdx.x & 31); }

// Sweep.  R: resident operand (rows r_row0 .. r_row0+255, rows >= r_limit redirected to r_limit-1).
// S: streamed operand; streamed row index g in [s_begin, s_end) maps to memory row gidx ? gidx[g'] : g'
// with g' = min(g, s_clamp - 1).  epi(chunk_first_row, rows_in_chunk, acc) is called once per chunk by all
// threads; it may use barriers (all threads call it) but must not touch the stream stages in `lds`.
// lidx / lidx_cap: optional LDS array of the caller's in which the sweep keeps its part of the gather list
// (used when the sweep's rows, rounded up to whole chunks, fit).  Without it the list is read from global
// memory once per chunk, and waiting for that read means waiting for every stream load issued before it:
// the wait counter of vector-memory instructions is shared.
//
// ctab / ctab_n: optional table of chunks (first streamed row, rows) that replaces the single range [s_begin, s_end):
// the sweep then visits ctab_n chunks that may lie anywhere (the same table for all threads; no gather list with it).
//
// post(chunk_first_row, rows_in_chunk): optional second half of a chunk's epilogue, for global stores.  The
// sweep tells that a stage has landed by counting outstanding vector-memory instructions, and stores count
// too: stores issued at the end of a chunk make the very next wait sit out their round trip.  post() for
// chunk c is therefore called inside chunk c+1, right after the loads that follow its first barrier have been
// issued: the next wait comes a whole stage of MFMAs later, when most of the stores have completed.  (Letting
// that wait tolerate the stores as well, and sparing the wavefronts that load nothing the wait altogether, was
// measured and gains nothing.)  The last chunk's post() runs after the sweep.  epi() leaves what post() needs
// in LDS of the caller's.
struct KsSoeNoPost {
    __device__ __forceinline__ void operator()(int, int) const {}
};
// side(chunk_first_row, chunk_index): optional, called by wavefront 0 when the loads of a chunk begin to be requested (up
// to two chunks before its epilogue): the place for a small asynchronous load of per-row data that the epilogue will
// want in LDS (global_load_lds; it is older than the chunk's stream loads, so the waits that cover those cover it).
struct KsSoeNoSide {
    __device__ __forceinline__ void operator()(int, int) const {}
};
template <class P> struct KsSoeHasPost { static constexpr bool value = true; };
template <> struct KsSoeHasPost<KsSoeNoPost> { static constexpr bool value = false; };
template <class CFG, class Epi, class Post = KsSoeNoPost, class Side = KsSoeNoSide>
__device__ __forceinline__ void ks_soe_sweep(const uint16_t *__restrict__ R, int64_t ldr, int r_row0, int r_limit,
                                              const uint16_t *__restrict__ S, int64_t lds_ld, const int32_t *__restrict__ gidx,
                                              int s_begin, int s_end, int s_clamp, uint16_t *lds, Epi &epi,
                                              int32_t *lidx = nullptr, int lidx_cap = 0, Post post = Post(),
                                              const int2 *__restrict__ ctab = nullptr, int ctab_n = 0, Side side = Side()) {
    constexpr int KT = CFG::KT, ST = CFG::STAGES, NI = CFG::NI, FM = CFG::FM;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    // ---- resident fragments: staged through LDS (coalesced row loads), then kept in registers ----------------
    bf16x8_t bres[KT * 4];
    {
        static_assert(CFG::LDS_ELEMS >= 2 * CFG::RES * 64, "the stream stages double as staging for the resident block");
        KsARows<CFG::RES, CFG::NW> rr;
        rr.init(R, ldr, nullptr, r_row0, r_limit);
        const int r31 = lane & 31, khalf = lane >> 5, swz = (lane >> 1) & 7;
        // up to four k-tiles in flight (the stream stages hold that many 256-row tiles): one memory round trip for the
        // first four instead of one per k-tile
        constexpr int NS = CFG::LDS_ELEMS / (CFG::RES * 64) >= 4 ? 4 : 2;
        constexpr int RNI = KsARows<CFG::RES, CFG::NW>::NI;
#pragma unroll
        for (int s = 0; s < NS; ++s)
            if (s < KT) rr.issue(s * 64, lds + s * CFG::RES * 64);
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            const int issued_tiles = (NS + (kt > 0 ? kt - 1 : 0)) < KT ? (NS + (kt > 0 ? kt - 1 : 0)) : KT;
            const int later = issued_tiles - (kt + 1); // k-tiles issued after this one (compile-time: the loop is unrolled)
            if (later >= 3) ks_wait_vmcnt<3 * RNI>();
            else if (later == 2) ks_wait_vmcnt<2 * RNI>();
            else if (later == 1) ks_wait_vmcnt<1 * RNI>();
            else ks_wait_vmcnt<0>();
            __builtin_amdgcn_s_waitcnt(0xC07F); // the fragment reads of k-tile kt-1 have returned: its slot may be reused
            ks_barrier_nofence();               // k-tile kt is in LDS
            if (kt > 0 && kt - 1 + NS < KT) rr.issue((kt - 1 + NS) * 64, lds + ((kt - 1) % NS) * CFG::RES * 64);
            const uint16_t *st = lds + (kt % NS) * CFG::RES * 64;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                bres[kt * 4 + kk] = *(const bf16x8_t *)(st + (wave * 32 + r31) * 64 + (((kk * 2 + khalf) ^ swz) * 8));
        }
    }

    // ---- stream state ---------------------------------------------------------------------------------------
    const int n_chunks = ctab ? ctab_n : (s_end - s_begin + CFG::CH - 1) / CFG::CH;
    auto chunk_first = [&](int c) __attribute__((always_inline)) { return ctab ? ctab[c].x : s_begin + c * CFG::CH; };
    auto chunk_rows = [&](int c) __attribute__((always_inline)) {
        if (ctab) return ctab[c].y;
        return (s_end - (s_begin + c * CFG::CH)) < CFG::CH ? (s_end - (s_begin + c * CFG::CH)) : CFG::CH;
    };
    const int n_tiles = n_chunks * (KT / CFG::KSUB); // pipeline stages in the whole sweep
    const bool use_lidx = gidx && lidx && n_chunks * CFG::CH <= lidx_cap;
    if (use_lidx) {
        for (int i = threadIdx.x; i < n_chunks * CFG::CH; i += CFG::NT) {
            int g = s_begin + i;
            if (g >= s_clamp) g = s_clamp - 1;
            lidx[i] = gidx[g];
        }
    }
    __builtin_amdgcn_s_waitcnt(0xC07F); // the fragment reads have returned before the stages are reused
    __syncthreads();                    // (also publishes the gather list)
    const bool loader = wave < CFG::LW;
    const uint16_t *ptr[NI]; // row pointers (k = 0, swizzled chunk) of the chunk being issued (loading wavefronts)
    // (table entries are read one chunk before they are needed, on the issue side and on the compute side: the wait for
    // a scalar load at the point of use would sit in the middle of the stream)
    int ahead_first = ctab && n_chunks > 0 ? ctab[0].x : 0; // first row of the next chunk whose loads will be set up
    auto chunk_ptrs = [&](int c) __attribute__((always_inline)) {
        const int first = ctab ? ahead_first : chunk_first(c);
        if (ctab) ahead_first = ctab[c + 1 < n_chunks ? c + 1 : c].x;
        if (wave == 0) side(first, c);
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int row = (j * CFG::LW + wave) * 8 + (lane >> 3);
            int64_t src;
            if (use_lidx) {
                src = lidx[c * CFG::CH + row];
            } else {
                int g = first + row;
                if (g >= s_clamp) g = s_clamp - 1;
                src = gidx ? (int64_t)gidx[g] : (int64_t)g;
            }
            ptr[j] = S + src * lds_ld + (((lane & 7) ^ ((row >> 1) & 7)) * 8);
        }
    };
    int is_c = 0, is_kt = 0, is_stage = 0, issued = 0; // position of the next tile to issue
    auto issue_one = [&]() __attribute__((always_inline)) { // one stage = KSUB consecutive k-tiles of the current chunk
        uint16_t *st = lds + is_stage * CFG::STAGE_ELEMS;
        if (loader) {
#pragma unroll
            for (int u = 0; u < CFG::KSUB; ++u)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    __builtin_amdgcn_global_load_lds(KS_GPTR(ptr[j] + (is_kt + u) * 64),
                                                     KS_LPTR(st + u * CFG::CH * 64 + (j * CFG::LW + wave) * 8 * 64), 16, 0, 0);
        }
        ++issued;
        if (++is_stage == ST) is_stage = 0;
        is_kt += CFG::KSUB;
        if (is_kt == KT) {
            is_kt = 0;
            ++is_c;
            if (is_c < n_chunks && loader) chunk_ptrs(is_c);
        }
    };
    if (n_chunks > 0 && loader) chunk_ptrs(0);
#pragma unroll
    for (int s = 0; s < ST - 1; ++s)
        if (issued < n_tiles) issue_one();

    // ---- sweep -------------------------------------------------------------------------------------------
    const int r31 = lane & 31, khalf = lane >> 5, swz = (lane >> 1) & 7;
    int stage = 0, done = 0;
    int2 ct_next = ctab && n_chunks > 0 ? ctab[0] : make_int2(0, 0);
    for (int c = 0; c < n_chunks; ++c) {
        const int2 ct = ct_next;
        if (ctab) ct_next = ctab[c + 1 < n_chunks ? c + 1 : c];
        const int rows_here = ctab ? ct.y : chunk_rows(c);
        f32x16_t acc[FM];
        // All k-tiles of one chunk.  FULL: the chunk has all CH rows -- the common case, compiled without a branch
        // between the MFMAs (a branch ends the basic block, and the wait for the fragment reads that the compiler
        // places at the start of the next one also waits for the reads issued ahead for the next k-step).
        // Otherwise 32-row blocks that hold no real row are skipped.
        auto chunk = [&](auto full) __attribute__((always_inline)) {
            constexpr bool FULL = decltype(full)::value;
            const int fm_cnt = (rows_here + 31) >> 5; // 32-row blocks of this chunk that hold real rows
            if (!FULL) {
#pragma unroll
                for (int fm = 0; fm < FM; ++fm)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[fm][r] = 0.f;
            }
#pragma unroll
            for (int kt0 = 0; kt0 < KT; kt0 += CFG::KSUB) {
                // stage `done` must have landed; the stages issued after it may still be in flight.  (Wavefronts that
                // load nothing only have the stores of their epilogues outstanding, which this wait also covers.)
                if (issued - done - 1 >= ST - 2) ks_wait_vmcnt<(ST - 2) * NI * CFG::KSUB>();
                else ks_wait_vmcnt<0>();
                ks_barrier_nofence();
                if (kt0 == 0 && c > 0 && KsSoeHasPost<Post>::value) post(chunk_first(c - 1), chunk_rows(c - 1));
#pragma unroll
                for (int u = 0; u < CFG::KSUB; ++u) {
                    const int kt = kt0 + u;
                    const uint16_t *st = lds + stage * CFG::STAGE_ELEMS + u * CFG::CH * 64;
                    bf16x8_t a0[FM], a1[FM];
#pragma unroll
                    for (int fm = 0; fm < FM; ++fm)
                        a0[fm] = *(const bf16x8_t *)(st + (fm * 32 + r31) * 64 + ((khalf ^ swz) * 8));
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) {
                        bf16x8_t(&cur)[FM] = (kk & 1) ? a1 : a0;
                        bf16x8_t(&nxt)[FM] = (kk & 1) ? a0 : a1;
                        __builtin_amdgcn_sched_barrier(0);
                        // The wait for this k-step's fragments goes HERE, before the next k-step's reads are issued:
                        // placed at their first use, after those reads, it would wait for them as well.
#pragma unroll
                        for (int fm = 0; fm < FM; ++fm) asm volatile("" ::"v"(cur[fm]));
                        __builtin_amdgcn_sched_barrier(0);
                        if (kk + 1 < 4) {
#pragma unroll
                            for (int fm = 0; fm < FM; ++fm)
                                nxt[fm] = *(const bf16x8_t *)(st + (fm * 32 + r31) * 64 + ((((kk + 1) * 2 + khalf) ^ swz) * 8));
                        }
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int fm = 0; fm < FM; ++fm) {
                            if (FULL) {
                                const f32x16_t zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                                acc[fm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur[fm], bres[kt * 4 + kk],
                                                                                   (kt == 0 && kk == 0) ? zero : acc[fm], 0, 0, 0);
                            } else if (fm < fm_cnt) {
                                acc[fm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur[fm], bres[kt * 4 + kk], acc[fm], 0, 0, 0);
                            }
                        }
                    }
                }
                // The next stage's loads go out HERE, after this stage's MFMAs, not right after the barrier: issuing a
                // load blocks a wavefront until the memory pipeline takes it (about 70 clocks each), and of the two
                // wavefronts of a SIMD the lower one gets the matrix pipe first, is done half a stage before the
                // other and would only wait at the next barrier -- the loading wavefronts 0..3 are those.  (The slot
                // they fill held the previous stage, which every wavefront left before this stage's barrier.)
                if (issued < n_tiles) issue_one();
                if (++stage == ST) stage = 0;
                ++done;
            }
        };
        if (rows_here == CFG::CH) chunk(std::true_type());
        else chunk(std::false_type());
        // a chunk of a single stage has no barrier between post() of the previous chunk (which reads what epi() left
        // in LDS) and this chunk's epi(): a wavefront that runs ahead must not overwrite what another still reads
        if (KT / CFG::KSUB < 2 && KsSoeHasPost<Post>::value) ks_barrier_nofence();
        epi(ctab ? ct.x : chunk_first(c), rows_here, acc);
    }
    ks_barrier_nofence();
    if (n_chunks > 0 && KsSoeHasPost<Post>::value) post(chunk_first(n_chunks - 1), chunk_rows(n_chunks - 1));
}
