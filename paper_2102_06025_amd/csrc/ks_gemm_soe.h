// Stationary-operand MFMA sweep for gfx950 (bf16 in, fp32 accumulate).
//
// Computes, chunk by chunk, the products  C[m][n] = sum_k S[m][k] * R[n][k]  of a long list of "streamed"
// rows S (m) with a block of 256 "resident" rows R (n), both stored with k contiguous, for a depth
// K = 64 * KT that is small enough to keep the resident block's MFMA fragments in registers for the whole
// sweep (KT <= 8: 256 VGPRs per lane).  Only the streamed rows travel through LDS (global_load_lds, several
// 128-row x 64-k tiles in flight), so each byte fetched from L2 feeds 256 multiply-adds instead of the
// 128 of a tile engine that streams both operands, and the chunk size (128 streamed rows) can be cut
// at any multiple of 32, which lets callers split the streamed rows evenly over the chip.
//
// Workgroup = 4 wavefronts; wavefront w owns resident rows [64 w, 64 w + 64) (two 32-column MFMA blocks),
// every wavefront reads the whole streamed tile from LDS.  MFMA orientation: streamed rows are the MFMA
// rows, resident rows the MFMA columns, so in the accumulator a lane owns ONE resident row (column
// lane % 32 of block fn) and 16 streamed rows per 32-row block: reductions along the streamed rows for a
// fixed resident row (softmax statistics per sample, running thresholds per graph row) are lane-local.
//
// After every chunk (all KT k-tiles of 128 streamed rows) the caller's epilogue functor gets the
// accumulators; the loads of the next chunk are already in flight at that point.
#pragma once
#include "ks_gemm_async.h"

template <int KT_, int CH_, int STAGES_, int KSUB_ = 1> struct KsSoe {
    static constexpr int KT = KT_, STAGES = STAGES_;
    static constexpr int KSUB = KSUB_;         // 64-wide k-tiles per pipeline stage (one barrier per stage)
    static constexpr int NW = 4, NT = 256;
    static constexpr int CH = CH_;             // streamed rows per chunk (96 or 128: the accumulators must fit beside
                                               // the resident fragments in the 512 registers of a lane)
    static constexpr int RES = 256;            // resident rows per workgroup
    static constexpr int FM = CH / 32, FN = 2; // accumulator blocks per wave
    static constexpr int NI = CH / (8 * NW);   // load instructions per wave per tile
    static constexpr int STAGE_ELEMS = KSUB * CH * 64;
    static constexpr int LDS_ELEMS = STAGES * STAGE_ELEMS;
    static_assert(KT >= 1 && KT <= 8 && KT % KSUB == 0 && STAGES >= 2 && (STAGES - 2) * NI * KSUB <= 63 && CH % 32 == 0,
                  "sweep shape");
};

// Row of the streamed chunk that accumulator element (fm, r) of this lane belongs to.
__device__ __forceinline__ int ks_soe_row(int fm, int r, int lane) { return fm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }
// Resident row (inside the workgroup's block of 256) of accumulator block fn of this lane.
__device__ __forceinline__ int ks_soe_col(int fn) { return (threadIdx.x >> 6) * 64 + fn * 32 + (threadIdx.x & 31); }

// Sweep.  R: resident operand (rows r_row0 .. r_row0+255, rows >= r_limit redirected to r_limit-1).
// S: streamed operand; streamed row index g in [s_begin, s_end) maps to memory row gidx ? gidx[g'] : g'
// with g' = min(g, s_clamp - 1).  epi(chunk_first_row, rows_in_chunk, acc) is called once per chunk by all
// threads; it may use barriers (all threads call it) but must not touch the stream stages in `lds`.
// lidx / lidx_cap: optional LDS array of the caller's in which the sweep keeps its part of the gather list
// (used when the sweep's rows, rounded up to whole chunks, fit).  Without it the list is read from global
// memory once per chunk, and waiting for that read means waiting for every stream load issued before it:
// the wait counter of vector-memory instructions is shared.
//
// post(chunk_first_row, rows_in_chunk): optional second half of a chunk's epilogue, for global stores.  The
// sweep tells that a stage has landed by counting outstanding vector-memory instructions, and stores count
// too: stores issued at the end of a chunk make the very next wait sit out their round trip.  post() for
// chunk c is therefore called inside chunk c+1, right after the loads of its first stage's successor have
// been issued (the wait after that still lets exactly those loads and the stores be outstanding, and by
// then a whole stage of MFMAs has passed), and after the sweep for the last chunk.  epi() leaves what
// post() needs in LDS of the caller's.
struct KsSoeNoPost {
    __device__ __forceinline__ void operator()(int, int) const {}
};
template <class CFG, class Epi, class Post = KsSoeNoPost>
__device__ __forceinline__ void ks_soe_sweep(const uint16_t *__restrict__ R, int64_t ldr, int r_row0, int r_limit,
                                             const uint16_t *__restrict__ S, int64_t lds_ld, const int32_t *__restrict__ gidx,
                                             int s_begin, int s_end, int s_clamp, uint16_t *lds, Epi &epi,
                                             int32_t *lidx = nullptr, int lidx_cap = 0, Post post = Post()) {
    constexpr int KT = CFG::KT, ST = CFG::STAGES, NI = CFG::NI, FM = CFG::FM;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    // ---- resident fragments: staged through LDS (coalesced row loads), then kept in registers ----------------
    bf16x8_t bres[2][KT * 4];
    {
        static_assert(CFG::LDS_ELEMS >= 2 * CFG::RES * 64, "the stream stages double as staging for the resident block");
        KsARows<CFG::RES, CFG::NW> rr;
        rr.init(R, ldr, nullptr, r_row0, r_limit);
        const int r31 = lane & 31, khalf = lane >> 5, swz = (lane >> 1) & 7;
        rr.issue(0, lds);
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            ks_wait_vmcnt<0>();
            ks_barrier_nofence(); // k-tile kt is in LDS; everyone is done reading k-tile kt-1
            if (kt + 1 < KT) rr.issue((kt + 1) * 64, lds + ((kt + 1) & 1) * CFG::RES * 64);
            const uint16_t *st = lds + (kt & 1) * CFG::RES * 64;
#pragma unroll
            for (int fn = 0; fn < 2; ++fn)
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    bres[fn][kt * 4 + kk] =
                        *(const bf16x8_t *)(st + (wave * 64 + fn * 32 + r31) * 64 + (((kk * 2 + khalf) ^ swz) * 8));
        }
    }

    // ---- stream state ---------------------------------------------------------------------------------------
    const int n_chunks = (s_end - s_begin + CFG::CH - 1) / CFG::CH;
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
    const int chunk_slot = (lane & 7) ^ 0; // 16-byte slot of this lane inside a 128-byte LDS row
    const uint16_t *ptr[NI];               // row pointers (k = 0, swizzled chunk) of the chunk being issued
    auto chunk_ptrs = [&](int c) {
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int row = (j * CFG::NW + wave) * 8 + (lane >> 3);
            int64_t src;
            if (use_lidx) {
                src = lidx[c * CFG::CH + row];
            } else {
                int g = s_begin + c * CFG::CH + row;
                if (g >= s_clamp) g = s_clamp - 1;
                src = gidx ? (int64_t)gidx[g] : (int64_t)g;
            }
            ptr[j] = S + src * lds_ld + ((chunk_slot ^ ((row >> 1) & 7)) * 8);
        }
    };
    int is_c = 0, is_kt = 0, is_stage = 0, issued = 0; // position of the next tile to issue
    auto issue_one = [&]() { // one stage = KSUB consecutive k-tiles of the current chunk
        uint16_t *st = lds + is_stage * CFG::STAGE_ELEMS;
#pragma unroll
        for (int u = 0; u < CFG::KSUB; ++u)
#pragma unroll
            for (int j = 0; j < NI; ++j)
                __builtin_amdgcn_global_load_lds(KS_GPTR(ptr[j] + (is_kt + u) * 64),
                                                 KS_LPTR(st + u * CFG::CH * 64 + (j * CFG::NW + wave) * 8 * 64), 16, 0, 0);
        ++issued;
        if (++is_stage == ST) is_stage = 0;
        is_kt += CFG::KSUB;
        if (is_kt == KT) {
            is_kt = 0;
            ++is_c;
            if (is_c < n_chunks) chunk_ptrs(is_c);
        }
    };
    if (n_chunks > 0) chunk_ptrs(0);
#pragma unroll
    for (int s = 0; s < ST - 1; ++s)
        if (issued < n_tiles) issue_one();

    // ---- sweep -------------------------------------------------------------------------------------------
    const int r31 = lane & 31, khalf = lane >> 5, swz = (lane >> 1) & 7;
    int stage = 0, done = 0;
    for (int c = 0; c < n_chunks; ++c) {
        const int rows_here = (s_end - (s_begin + c * CFG::CH)) < CFG::CH ? (s_end - (s_begin + c * CFG::CH)) : CFG::CH;
        const int fm_cnt = (rows_here + 31) >> 5; // 32-row blocks of this chunk that hold real rows
        f32x16_t acc[FM][2];
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
#pragma unroll
            for (int fn = 0; fn < 2; ++fn)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[fm][fn][r] = 0.f;
#pragma unroll
        for (int kt0 = 0; kt0 < KT; kt0 += CFG::KSUB) {
            // stage `done` must have landed; the stages issued after it may still be in flight
            if (issued - done - 1 >= ST - 2) ks_wait_vmcnt<(ST - 2) * NI * CFG::KSUB>();
            else ks_wait_vmcnt<0>();
            ks_barrier_nofence();
            if (issued < n_tiles) issue_one();
            if (kt0 == 0 && c > 0) {
                const int pc0 = s_begin + (c - 1) * CFG::CH;
                post(pc0, (s_end - pc0) < CFG::CH ? (s_end - pc0) : CFG::CH);
            }
#pragma unroll
            for (int u = 0; u < CFG::KSUB; ++u) {
                const int kt = kt0 + u;
                const uint16_t *st = lds + stage * CFG::STAGE_ELEMS + u * CFG::CH * 64;
                bf16x8_t a0[FM], a1[FM];
#pragma unroll
                for (int fm = 0; fm < FM; ++fm) a0[fm] = *(const bf16x8_t *)(st + (fm * 32 + r31) * 64 + ((khalf ^ swz) * 8));
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    bf16x8_t(&cur)[FM] = (kk & 1) ? a1 : a0;
                    bf16x8_t(&nxt)[FM] = (kk & 1) ? a0 : a1;
                    __builtin_amdgcn_sched_barrier(0);
                    if (kk + 1 < 4) {
#pragma unroll
                        for (int fm = 0; fm < FM; ++fm)
                            nxt[fm] = *(const bf16x8_t *)(st + (fm * 32 + r31) * 64 + ((((kk + 1) * 2 + khalf) ^ swz) * 8));
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int fm = 0; fm < FM; ++fm) {
                        if (fm < fm_cnt) {
                            acc[fm][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur[fm], bres[0][kt * 4 + kk], acc[fm][0], 0, 0, 0);
                            acc[fm][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur[fm], bres[1][kt * 4 + kk], acc[fm][1], 0, 0, 0);
                        }
                    }
                }
            }
            if (++stage == ST) stage = 0;
            ++done;
        }
        epi(s_begin + c * CFG::CH, rows_here, acc);
    }
    ks_barrier_nofence();
    if (n_chunks > 0) {
        const int pc0 = s_begin + (n_chunks - 1) * CFG::CH;
        post(pc0, s_end - pc0);
    }
}
