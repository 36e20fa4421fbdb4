// bf16 MFMA tile engine for gfx950, alternating version: a 256 x 256 x 64 tile engine whose eight wavefronts work as
// two groups of four that take turns.  Wavefront w and wavefront w + 4 share a SIMD; group 0 (wavefronts 0-3) owns
// the upper 128 rows of the output tile, group 1 (wavefronts 4-7) the lower 128.  Time is cut into phases that end
// with a workgroup barrier.  In every phase one group is in its MEMORY part -- it requests the direct-to-LDS loads
// of the next k-tile and reads ALL fragments of its current k-tile from LDS into registers -- while the other group
// is in its MATRIX part: 32 MFMAs on operands that are already in registers.  Then they swap.  On each SIMD the
// matrix pipe therefore always has one wavefront issuing back-to-back MFMAs, and the back-pressure of the load
// requests, the LDS round trips and the barrier skew of one group fall into the matrix time of the other.  (In the
// plain pipeline of ks_gemm_async.h all wavefronts are in the same part at the same time: loads, fragment reads and
// MFMAs of a k-tile each take about as long as the others, and only partly overlap.)
//
// Schedule, k-tiles t = 0 .. n-1, phases p = 0 .. 2n:
//     group 0:  memory part of tile t in phase 2t,      matrix part of tile t in phase 2t + 1
//     group 1:  memory part of tile t in phase 2t + 1,  matrix part of tile t in phase 2t + 2
// LDS holds two stages (tile t in stage t & 1).  Who loads what is chosen so that every load has two phases to land
// and never overwrites data still to be read:
//     group 0 requests, at the start of phase 2t, its own half of A (upper 128 rows) and the WHOLE B tile of tile
//         t + 1: stage (t + 1) & 1 held tile t - 1, whose A upper half group 0 read in phase 2t - 2 and whose B tile
//         group 1 read last, in phase 2t - 1;
//     group 1 requests, at the start of phase 2t + 1, its half of A (lower 128 rows) of tile t + 1, which only itself
//         read before (tile t - 1, phase 2t - 1).
// A group waits for its own requests (s_waitcnt vmcnt(0)) at the end of its matrix part, one to two phases after
// issuing them; the barrier that follows publishes them to the other group.  Fragment reads are complete
// (lgkmcnt(0)) before the barrier that ends a memory part, so a stage is never overwritten under a read.
//
// All LDS fragment reads are issued from inline assembly: the compiler cannot tell a read of one stage from the
// asynchronous writes into the other and would otherwise wait for every load in flight before each read.
//
// Operand forms as in ks_gemm_async.h: "rows" (k contiguous in memory, tile kept as [rows][64] with the 16-byte
// chunk c of row r in slot c ^ ((r >> 1) & 7)) or "k-major" (element (k, c) at base[src(k) * ld + c], tile kept as
// [64 k][W] with chunk c of k-row k in slot c ^ ((k & 3) << 2), fragments by the transposing read).  A k-major A
// tile is kept as two half tiles of 128 columns, one per group.
#pragma once
#include "ks_gemm_async.h"

struct KsPP {
    static constexpr int BM = 256, BN = 256, BK = 64, NW = 8, NT = 512, FM = 4, FN = 2;
    static constexpr int A_ELEMS = BM * 64, B_ELEMS = BN * 64, STAGE_ELEMS = A_ELEMS + B_ELEMS, LDS_ELEMS = 2 * STAGE_ELEMS;
    // the names the helpers of ks_gemm_async.h expect of a tile type
    static constexpr int WAVES_M = 2, WAVES_N = 4, WM = 128, WN = 64, STAGES = 2;
};

__device__ __forceinline__ ks_u32x4 ks_ds_read_b128(const uint16_t *p) {
    const uint32_t addr = (uint32_t)(uintptr_t)(const uint16_t __attribute__((address_space(3))) *)p;
    ks_u32x4 v;
    asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr));
    return v;
}

// ---- loaders of one group (four wavefronts; w4 = wavefront index inside the group) ---------------------------
// ROWS rows, k contiguous.  Rows at or beyond row_limit are redirected to the last valid row.
template <int ROWS> struct KsPRows {
    static constexpr int NI = ROWS / 32;
    const uint16_t *ptr[NI];
    __device__ __forceinline__ void init(const uint16_t *base, int64_t ld, const int32_t *gidx, int row0, int row_limit) {
        const int lane = threadIdx.x & 63, w4 = (threadIdx.x >> 6) & 3;
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int row = (j * 4 + w4) * 8 + (lane >> 3);
            int gr = row0 + row;
            if (gr >= row_limit) gr = row_limit - 1;
            const int64_t src = gidx ? (int64_t)gidx[gr] : (int64_t)gr;
            ptr[j] = base + src * ld + (((lane & 7) ^ ((row >> 1) & 7)) * 8);
        }
    }
    // lds: where row 0 of these ROWS rows sits in the stage
    __device__ __forceinline__ void issue(int k0, uint16_t *lds) const {
        const int w4 = __builtin_amdgcn_readfirstlane((threadIdx.x >> 6) & 3);
#pragma unroll
        for (int j = 0; j < NI; ++j)
            __builtin_amdgcn_global_load_lds(KS_GPTR(ptr[j] + k0), KS_LPTR(lds + (j * 4 + w4) * 8 * 64), 16, 0, 0);
    }
};

// k-major tile of W columns ([64 k][W] in LDS).  k-rows at or beyond k_limit are redirected to k_limit - 1 (the other
// operand must be zero there), columns beyond col_limit to the last 8 valid ones; src(k) through an optional gather
// list in LDS (lidx[k - k_first]).
template <int W> struct KsPKmaj {
    static constexpr int CPR = W / 8, RPI = 64 / CPR, NI = 64 / (RPI * 4);
    static_assert(W == 128 || W == 256, "k-major tile width");
    const uint16_t *base;
    const int32_t *lidx;
    int64_t ld;
    int k_limit, k_first, col_base, col_lim8;
    __device__ __forceinline__ void init(const uint16_t *base_, int64_t ld_, const int32_t *lidx_, int col0, int col_limit,
                                         int k_limit_, int k_first_) {
        base = base_; ld = ld_; lidx = lidx_; k_limit = k_limit_; k_first = k_first_;
        col_base = col0;
        col_lim8 = col_limit - 8;
    }
    __device__ __forceinline__ void issue(int k0, uint16_t *lds) const {
        const int lane = threadIdx.x & 63;
        const int w4 = __builtin_amdgcn_readfirstlane((threadIdx.x >> 6) & 3);
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int k = (j * 4 + w4) * RPI + lane / CPR;
            int col = col_base + (((lane % CPR) ^ ((k & 3) << 2)) * 8);
            if (col > col_lim8) col = col_lim8;
            int kg = k0 + k;
            if (kg >= k_limit) kg = k_limit - 1;
            const int64_t src = lidx ? (int64_t)lidx[kg - k_first] : (int64_t)kg;
            __builtin_amdgcn_global_load_lds(KS_GPTR(base + src * ld + col), KS_LPTR(lds + (j * 4 + w4) * RPI * W), 16, 0, 0);
        }
    }
};

// all fragments of one k-tile for one wavefront: 4 k-steps x (4 A + 2 B) fragments = 96 registers
struct KsPFrags {
    bf16x8_t a[4][KsPP::FM], b[4][KsPP::FN];
};

template <bool AK, bool BK>
__device__ __forceinline__ void ks_pp_read_frags(KsPFrags &f, const uint16_t *st) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = wave >> 2, wn = wave & 3;
    const uint16_t *stA = st, *stB = st + KsPP::A_ELEMS;
    const int r = lane & 31, khalf = lane >> 5, swz = (lane >> 1) & 7;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const int co = ((kk * 2 + khalf) ^ swz) * 8;
#pragma unroll
        for (int fm = 0; fm < KsPP::FM; ++fm) {
            if (AK) f.a[kk][fm] = ks_a_frag_kmaj<128>(stA + g * 64 * 128, fm, kk);
            else f.a[kk][fm] = __builtin_bit_cast(bf16x8_t, ks_ds_read_b128(stA + (g * 128 + fm * 32 + r) * 64 + co));
        }
#pragma unroll
        for (int fn = 0; fn < KsPP::FN; ++fn) {
            if (BK) f.b[kk][fn] = ks_a_frag_kmaj<256>(stB, wn * 2 + fn, kk);
            else f.b[kk][fn] = __builtin_bit_cast(bf16x8_t, ks_ds_read_b128(stB + (wn * 64 + fn * 32 + r) * 64 + co));
        }
    }
    // every read has returned before the barrier that lets the other group overwrite the stage
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
        for (int fm = 0; fm < KsPP::FM; ++fm) asm volatile("" : "+v"(f.a[kk][fm]));
#pragma unroll
        for (int fn = 0; fn < KsPP::FN; ++fn) asm volatile("" : "+v"(f.b[kk][fn]));
    }
}

__device__ __forceinline__ void ks_pp_mma(const KsPFrags &f, f32x16_t (&acc)[KsPP::FM][KsPP::FN]) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
#pragma unroll
        for (int fm = 0; fm < KsPP::FM; ++fm)
#pragma unroll
            for (int fn = 0; fn < KsPP::FN; ++fn)
                acc[fm][fn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[kk][fm], f.b[kk][fn], acc[fm][fn], 0, 0, 0);
}

// Main loop over k-tiles [kt0, kt1) (k0 = kt * 64); every thread of the workgroup calls it with the same range.
// ah: loader of this wavefront's group's half of A (rows form: KsPRows<128>, k-major: KsPKmaj<128>), initialised by
// the caller for its own group; bl: loader of the whole B tile (KsPRows<256> / KsPKmaj<256>), used by group 0 only.
// Ends with a barrier: LDS is free on return.
template <bool AK, bool BK, class AH, class BL>
__device__ __forceinline__ void ks_pp_mainloop(const AH &ah, const BL &bl, int kt0, int kt1, uint16_t *lds,
                                               f32x16_t (&acc)[KsPP::FM][KsPP::FN]) {
    const int g = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 8)); // group of this wavefront
    const int n = kt1 - kt0;
    if (n <= 0) return;
    // where this group's half of A sits inside a stage
    const int a_off = AK ? g * 64 * 128 : g * 128 * 64;
    auto request = [&](int t) __attribute__((always_inline)) { // this group's share of the loads of tile t
        uint16_t *st = lds + (t & 1) * KsPP::STAGE_ELEMS;
        ah.issue((kt0 + t) * 64, st + a_off);
        if (g == 0) bl.issue((kt0 + t) * 64, st + KsPP::A_ELEMS);
    };
    request(0);
    ks_wait_vmcnt<0>();
    ks_barrier_nofence();
    KsPFrags f;
    if (g == 0) {
        for (int t = 0; t < n; ++t) {
            if (t + 1 < n) request(t + 1);
            __builtin_amdgcn_sched_barrier(0);
            ks_pp_read_frags<AK, BK>(f, lds + (t & 1) * KsPP::STAGE_ELEMS);
            __builtin_amdgcn_sched_barrier(0);
            ks_barrier_nofence();
            __builtin_amdgcn_sched_barrier(0);
            ks_pp_mma(f, acc);
            __builtin_amdgcn_sched_barrier(0);
            ks_wait_vmcnt<0>();
            ks_barrier_nofence();
        }
        ks_barrier_nofence(); // phase 2n: group 1's last matrix part
    } else {
        ks_barrier_nofence(); // phase 0: group 0's first memory part
        for (int t = 0; t < n; ++t) {
            if (t + 1 < n) request(t + 1);
            __builtin_amdgcn_sched_barrier(0);
            ks_pp_read_frags<AK, BK>(f, lds + (t & 1) * KsPP::STAGE_ELEMS);
            __builtin_amdgcn_sched_barrier(0);
            ks_barrier_nofence();
            __builtin_amdgcn_sched_barrier(0);
            ks_pp_mma(f, acc);
            __builtin_amdgcn_sched_barrier(0);
            ks_wait_vmcnt<0>();
            ks_barrier_nofence();
        }
    }
}
