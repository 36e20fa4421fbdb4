// bf16 MFMA tile engine for gfx950, asynchronous version: operand tiles go from global memory straight
// into LDS (global_load_lds_dwordx4, no staging registers), several k-tiles in flight.
//
// Both operands must be stored with k contiguous ("row = m or n, k fast"), 16-byte aligned rows, and the
// k range handed to the main loop must be readable and finite for every row that is loaded (callers pad
// k with zeros in memory); rows beyond the operand's row limit are redirected to the last valid row, so
// the corresponding accumulator rows/columns hold finite garbage that the epilogue must not store.
//
// LDS layout of one operand tile: [ROWS][64] bf16, unpadded; the 16-byte chunk c of row r sits in slot
// c ^ ((r >> 1) & 7) of that row.  One wave-wide load instruction fills 8 consecutive rows (lane l: row
// l/8, slot l%8), so each lane fetches global chunk  slot ^ ((row >> 1) & 7)  of its row; the 16-byte
// fragment reads of 16 consecutive rows at one k offset then hit 16 distinct bank groups.
//
// Pipeline: STAGES LDS buffers.  Iteration t: wait until this wave's loads of tile t have landed
// (s_waitcnt vmcnt(N) with the number of younger loads), workgroup barrier (everyone's part of tile t
// is in LDS and everyone is done reading tile t-1), issue the loads of tile t+STAGES-1 into the buffer
// tile t-1 used, MFMAs of tile t with register double-buffered fragments.
#pragma once
#include "ks_common.h"

#define KS_GPTR(p) ((const void __attribute__((address_space(1))) *)(p))
#define KS_LPTR(p) ((void __attribute__((address_space(3))) *)(p))

template <int BM_, int BN_, int WAVES_M_, int WAVES_N_, int STAGES_> struct KsATile {
    static constexpr int BM = BM_, BN = BN_, BK = 64, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, STAGES = STAGES_;
    static constexpr int NW = WAVES_M * WAVES_N, NT = NW * 64;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int FM = WM / 32, FN = WN / 32;
    static constexpr int NI_A = BM / (8 * NW), NI_B = BN / (8 * NW); // load instructions per wave per tile
    static constexpr int STAGE_ELEMS = (BM + BN) * 64;
    static constexpr int LDS_ELEMS = STAGES * STAGE_ELEMS;
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0 && WM % 32 == 0 && WN % 32 == 0, "tile shape");
    static_assert((STAGES - 2) * (NI_A + NI_B) <= 63, "vmcnt range");
};

// s_waitcnt vmcnt(n) only (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt_hi[15:14])
template <int N> __device__ __forceinline__ void ks_wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}
// workgroup barrier without the memory fence of __syncthreads() (which would drain the loads in flight);
// the empty asm statements keep the compiler from moving LDS accesses across it
__device__ __forceinline__ void ks_barrier_nofence() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// per-lane global pointers (k = 0) of the rows this lane loads, one per load instruction
template <int ROWS, int NW> struct KsARows {
    static constexpr int NI = ROWS / (8 * NW);
    const uint16_t *ptr[NI];
    __device__ __forceinline__ void init(const uint16_t *base, int64_t ld, const int32_t *gidx, int row0, int row_limit) {
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int row = (j * NW + wave) * 8 + (lane >> 3);
            int gr = row0 + row;
            if (gr >= row_limit) gr = row_limit - 1; // row_limit >= 1
            const int64_t src = gidx ? (int64_t)gidx[gr] : (int64_t)gr;
            const int chunk = (lane & 7) ^ ((row >> 1) & 7);
            ptr[j] = base + src * ld + chunk * 8;
        }
    }
    // enqueue this wave's loads of the k-tile starting at element k0 into the tile at `lds`
    __device__ __forceinline__ void issue(int k0, uint16_t *lds) const {
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
#pragma unroll
        for (int j = 0; j < NI; ++j)
            __builtin_amdgcn_global_load_lds(KS_GPTR(ptr[j] + k0), KS_LPTR(lds + (j * NW + wave) * 8 * 64), 16, 0, 0);
    }
    // the j-th of them alone (j is a compile-time constant after unrolling)
    __device__ __forceinline__ void issue_one(int j, int k0, uint16_t *lds) const {
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        __builtin_amdgcn_global_load_lds(KS_GPTR(ptr[j] + k0), KS_LPTR(lds + (j * NW + wave) * 8 * 64), 16, 0, 0);
    }
};

// ---------------------------------------------------------------------------------------------
// Operand stored k-major: element (k, c) at base[src(k) * ld + c] (c = the operand's m or n index, fast in
// memory).  The tile is kept in LDS as it is, [64 k-rows][W columns], and the MFMA fragments (8
// consecutive k per lane) are produced by the transposing LDS read ds_read_b64_tr_b16: inside each group
// of 16 lanes, lane 4r+q supplies the address of 4 consecutive columns of k-row r, and lane i receives
// column i of those four k-rows.  16-byte chunk c of k-row k sits in slot c ^ ((k & 3) << 2), so that
// the four k-rows touched by one read fall on different bank groups.
// Rows k >= k_limit are redirected to row k_limit-1 (the other operand must be zero there); columns
// beyond col_limit are redirected to the last 8 valid columns.  src(k) goes through an optional gather
// list that the caller has staged in LDS for its k range (so that no global load sits between the
// asynchronous tile loads and their counted waits).
// ---------------------------------------------------------------------------------------------
template <int W, int NW> struct KsAKmaj {
    static constexpr int CPR = W / 8;            // 16-byte chunks per k-row
    static constexpr int RPI = 64 / CPR;         // k-rows per wave-wide load instruction
    static constexpr int NI = CPR / NW;          // load instructions per wave per tile
    static_assert(CPR % NW == 0 && NI >= 1 && (W == 128 || W == 256), "k-major tile shape");
    const uint16_t *base;
    const int32_t *lidx;  // gather list of the caller's k range, staged in LDS (or nullptr: no gather)
    int64_t ld;
    int k_limit, k_first, col_base, col_lim8;
    int kloc[NI];         // k-row (tile local) of this lane for each instruction

    // lidx_[k - k_first_] = source row of k, for every k this loader will be asked for (k < k_limit_)
    __device__ __forceinline__ void init(const uint16_t *base_, int64_t ld_, const int32_t *lidx_, int col0, int col_limit,
                                         int k_limit_, int k_first_) {
        base = base_; ld = ld_; lidx = lidx_; k_limit = k_limit_; k_first = k_first_;
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
        for (int j = 0; j < NI; ++j) kloc[j] = (j * NW + wave) * RPI + lane / CPR;
        col_base = col0;
        col_lim8 = col_limit - 8;
    }
    __device__ __forceinline__ void issue(int k0, uint16_t *lds) const {
        const int lane = threadIdx.x & 63;
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        // every source row first (the gather list is read from LDS in one batch, with one wait), then the loads
        // back to back: a list read between two loads would cost its LDS latency once per load
        int src[NI];
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            int kg = k0 + kloc[j];
            if (kg >= k_limit) kg = k_limit - 1;
            src[j] = kg;
        }
        if (lidx) {
#pragma unroll
            for (int j = 0; j < NI; ++j) src[j] = lidx[src[j] - k_first];
        }
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int k = kloc[j];
            // the slot this lane fills (lane % CPR) holds chunk slot ^ ((k & 3) << 2) of k-row k
            int col = col_base + (((lane % CPR) ^ ((k & 3) << 2)) * 8);
            if (col > col_lim8) col = col_lim8;
            __builtin_amdgcn_global_load_lds(KS_GPTR(base + (int64_t)src[j] * ld + col), KS_LPTR(lds + (j * NW + wave) * RPI * W), 16, 0, 0);
        }
    }
    __device__ __forceinline__ void issue_one(int j, int k0, uint16_t *lds) const {
        const int lane = threadIdx.x & 63;
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const int k = kloc[j];
        int col = col_base + (((lane % CPR) ^ ((k & 3) << 2)) * 8);
        if (col > col_lim8) col = col_lim8;
        int kg = k0 + k;
        if (kg >= k_limit) kg = k_limit - 1;
        const int64_t src = lidx ? (int64_t)lidx[kg - k_first] : (int64_t)kg;
        __builtin_amdgcn_global_load_lds(KS_GPTR(base + src * ld + col), KS_LPTR(lds + (j * NW + wave) * RPI * W), 16, 0, 0);
    }
};

// The transposing LDS read as inline assembly.  Through the compiler's builtin every such read is preceded by
// s_waitcnt vmcnt(0): the compiler cannot tell it apart from the buffer the asynchronous loads in flight are
// writing and waits for all of them, which serialises the loads of tile t+1 with the MFMAs of tile t.  As
// assembly the read is invisible to that logic; the price is that its completion has to be waited for by hand
// (ks_a_wait_frags) before the registers are used.
typedef uint32_t ks_u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t ks_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ ks_u32x2 ks_ds_read_tr16_b64(const uint16_t *p) {
    const uint32_t addr = (uint32_t)(uintptr_t)(const uint16_t __attribute__((address_space(3))) *)p;
    ks_u32x2 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(v) : "v"(addr));
    return v;
}

// fragment of a k-major tile: 8 consecutive k (k-step kk) of column block `cb` (32 columns)
template <int W>
__device__ __forceinline__ bf16x8_t ks_a_frag_kmaj(const uint16_t *tile, int cb32, int kk) {
    const int lane = threadIdx.x & 63;
    const int g = lane >> 4, r = (lane >> 2) & 3, q = lane & 3;
    const int kb = kk * 16 + (g >> 1) * 8 + r;
    const int chunk = cb32 * 4 + (g & 1) * 2 + (q >> 1);
    // k & 3 == r for both halves (kb + 4 has the same low bits)
    const int off = ((chunk ^ (r << 2)) * 8) + (q & 1) * 4;
    const ks_u32x2 lo = ks_ds_read_tr16_b64(tile + kb * W + off);
    const ks_u32x2 hi = ks_ds_read_tr16_b64(tile + (kb + 4) * W + off);
    const ks_u32x4 both = {lo.x, lo.y, hi.x, hi.y};
    return __builtin_bit_cast(bf16x8_t, both);
}

template <class T> struct KsAFrags {
    bf16x8_t a[T::FM], b[T::FN];
};

// fragments of k-step kk; AK / BK say whether the operand tile is k-major
template <class T, bool AK, bool BK>
__device__ __forceinline__ void ks_a_load_frags(KsAFrags<T> &f, const uint16_t *stA, const uint16_t *stB, int kk) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / T::WAVES_N, wn = wave % T::WAVES_N;
    const int r = lane & 31, khalf = lane >> 5, swz = (lane >> 1) & 7;
    const int co = ((kk * 2 + khalf) ^ swz) * 8;
#pragma unroll
    for (int fm = 0; fm < T::FM; ++fm) {
        if (AK) f.a[fm] = ks_a_frag_kmaj<T::BM>(stA, wm * T::FM + fm, kk);
        else f.a[fm] = *(const bf16x8_t *)(stA + (wm * T::WM + fm * 32 + r) * 64 + co);
    }
#pragma unroll
    for (int fn = 0; fn < T::FN; ++fn) {
        if (BK) f.b[fn] = ks_a_frag_kmaj<T::BN>(stB, wn * T::FN + fn, kk);
        else f.b[fn] = *(const bf16x8_t *)(stB + (wn * T::WN + fn * 32 + r) * 64 + co);
    }
}

// LDS instructions of one fragment set (a k-major fragment takes two reads)
template <class T, bool AK, bool BK> struct KsAFragCount {
    static constexpr int N = (AK ? 2 : 1) * T::FM + (BK ? 2 : 1) * T::FN;
    static_assert(N <= 15, "lgkmcnt range");
};
// Wait until at most YOUNGER LDS instructions issued after this fragment set's reads are outstanding, and tie
// the set's registers to the wait so that nothing using them is scheduled above it.  Only needed when some
// read was issued from assembly (k-major operands); the compiler looks after the reads it knows.
template <class T, bool AK, bool BK, int YOUNGER>
__device__ __forceinline__ void ks_a_wait_frags(KsAFrags<T> &f) {
    if (!AK && !BK) return;
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(YOUNGER));
#pragma unroll
    for (int fm = 0; fm < T::FM; ++fm) asm volatile("" : "+v"(f.a[fm]));
#pragma unroll
    for (int fn = 0; fn < T::FN; ++fn) asm volatile("" : "+v"(f.b[fn]));
}

template <class T>
__device__ __forceinline__ void ks_a_mma(const KsAFrags<T> &f, f32x16_t (&acc)[T::FM][T::FN]) {
#pragma unroll
    for (int fm = 0; fm < T::FM; ++fm)
#pragma unroll
        for (int fn = 0; fn < T::FN; ++fn)
            acc[fm][fn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[fm], f.b[fn], acc[fm][fn], 0, 0, 0);
}

// MFMAs of one k-tile held in the stage at `st` (A tile first, then B tile).  Register double buffering
// of the fragments; the scheduling barriers keep the compiler from collapsing it (the reads of step
// kk+1 are in flight while the MFMAs of step kk issue).
template <class T, bool AK = false, bool BK = false>
__device__ __forceinline__ void ks_a_tile_mma(const uint16_t *st, f32x16_t (&acc)[T::FM][T::FN]) {
    const uint16_t *stA = st, *stB = st + T::BM * 64;
    constexpr int N = KsAFragCount<T, AK, BK>::N; // the reads of one set: what may stay outstanding behind the set in use
    KsAFrags<T> f0, f1;
    __builtin_amdgcn_sched_barrier(0);
    ks_a_load_frags<T, AK, BK>(f0, stA, stB, 0);
    __builtin_amdgcn_sched_barrier(0);
    ks_a_load_frags<T, AK, BK>(f1, stA, stB, 1);
    __builtin_amdgcn_sched_barrier(0);
    ks_a_wait_frags<T, AK, BK, N>(f0);
    ks_a_mma<T>(f0, acc);
    __builtin_amdgcn_sched_barrier(0);
    ks_a_load_frags<T, AK, BK>(f0, stA, stB, 2);
    __builtin_amdgcn_sched_barrier(0);
    ks_a_wait_frags<T, AK, BK, N>(f1);
    ks_a_mma<T>(f1, acc);
    __builtin_amdgcn_sched_barrier(0);
    ks_a_load_frags<T, AK, BK>(f1, stA, stB, 3);
    __builtin_amdgcn_sched_barrier(0);
    ks_a_wait_frags<T, AK, BK, N>(f0);
    ks_a_mma<T>(f0, acc);
    __builtin_amdgcn_sched_barrier(0);
    ks_a_wait_frags<T, AK, BK, 0>(f1);
    ks_a_mma<T>(f1, acc);
}

// Main loop over k-tiles [kt0, kt1) (k0 = kt * 64).  All threads of the workgroup must call it with the
// same range.  Ends with a barrier, so the LDS can be reused at once.  AR / BR are KsARows (k contiguous)
// or KsAKmaj (k-major) loaders; AK / BK tell the fragment reader which.
template <class T, bool AK = false, bool BK = false, class AR, class BR>
__device__ __forceinline__ void ks_a_mainloop(AR &ar, BR &br, int kt0, int kt1, uint16_t *lds,
                                              f32x16_t (&acc)[T::FM][T::FN]) {
    constexpr int S = T::STAGES;
    constexpr int PER_TILE = T::NI_A + T::NI_B;
    static_assert(S == 2 || (!AK && !BK), "k-major loaders issue their gather-index loads in between: two stages only");
#pragma unroll
    for (int s = 0; s < S - 1; ++s) {
        if (kt0 + s < kt1) {
            uint16_t *st = lds + s * T::STAGE_ELEMS;
            ar.issue((kt0 + s) * 64, st);
            br.issue((kt0 + s) * 64, st + T::BM * 64);
        }
    }
    int stage = 0;
    for (int kt = kt0; kt < kt1; ++kt) {
        // loads younger than tile kt: tiles kt+1 .. kt+S-2 when they all exist
        if (S > 2 && kt + S - 2 < kt1) ks_wait_vmcnt<(S - 2) * PER_TILE>();
        else ks_wait_vmcnt<0>();
        ks_barrier_nofence();
        if (kt + S - 1 < kt1) {
            int ns = stage + S - 1;
            if (ns >= S) ns -= S;
            uint16_t *st = lds + ns * T::STAGE_ELEMS;
            ar.issue((kt + S - 1) * 64, st);
            br.issue((kt + S - 1) * 64, st + T::BM * 64);
        }
        ks_a_tile_mma<T, AK, BK>(lds + stage * T::STAGE_ELEMS, acc);
        if (++stage == S) stage = 0;
    }
    ks_barrier_nofence();
}

// ---------------------------------------------------------------------------------------------
// Main loop with the loads of the next k-tile INTERLEAVED with the MFMAs of the current one.  A wavefront that
// requests a direct-to-LDS load stalls until the vector-memory pipeline of the compute unit accepts it, and that
// pipeline takes a 1 KB request about every 32 clocks: the 64 requests of a 256 x 256 x 64 k-tile keep it busy for
// as long as the k-tile's MFMAs keep the matrix pipes busy.  Requested in one burst after the barrier (ks_a_mainloop)
// all eight wavefronts sit in that queue first and compute afterwards: the two times add up.  Here each wavefront
// requests one load every few MFMAs, over the first SPREAD of the k-tile's four k-steps (the rest of the k-tile is
// left for the last loads to land): while one wavefront of a SIMD waits to get a request accepted, the other one's
// MFMAs run.  Two stages only: the loads of tile t + 1 go out during tile t.
// ---------------------------------------------------------------------------------------------
template <class T, int KK, int SLOTS, class Issue>
__device__ __forceinline__ void ks_a_mma_il(const KsAFrags<T> &f, f32x16_t (&acc)[T::FM][T::FN], bool do_load, Issue &issue) {
    constexpr int NL = T::NI_A + T::NI_B, PER = T::FM * T::FN;
#pragma unroll
    for (int fm = 0; fm < T::FM; ++fm)
#pragma unroll
        for (int fn = 0; fn < T::FN; ++fn) {
            constexpr int dummy = 0;
            (void)dummy;
            const int idx = KK * PER + fm * T::FN + fn; // constant after unrolling
#pragma unroll
            for (int q = 0; q < NL; ++q)
                if (q * SLOTS / NL == idx) {
                    __builtin_amdgcn_sched_barrier(0);
                    if (do_load) issue(q);
                    __builtin_amdgcn_sched_barrier(0);
                }
            acc[fm][fn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[fm], f.b[fn], acc[fm][fn], 0, 0, 0);
        }
}

template <class T, bool AK, bool BK, int SPREAD, class Issue>
__device__ __forceinline__ void ks_a_tile_mma_il(const uint16_t *st, f32x16_t (&acc)[T::FM][T::FN], bool do_load, Issue &issue) {
    const uint16_t *stA = st, *stB = st + T::BM * 64;
    constexpr int N = KsAFragCount<T, AK, BK>::N;
    constexpr int SLOTS = SPREAD * T::FM * T::FN;
    KsAFrags<T> f0, f1;
    __builtin_amdgcn_sched_barrier(0);
    ks_a_load_frags<T, AK, BK>(f0, stA, stB, 0);
    __builtin_amdgcn_sched_barrier(0);
    ks_a_load_frags<T, AK, BK>(f1, stA, stB, 1);
    __builtin_amdgcn_sched_barrier(0);
    ks_a_wait_frags<T, AK, BK, N>(f0);
    ks_a_mma_il<T, 0, SLOTS>(f0, acc, do_load, issue);
    __builtin_amdgcn_sched_barrier(0);
    ks_a_load_frags<T, AK, BK>(f0, stA, stB, 2);
    __builtin_amdgcn_sched_barrier(0);
    ks_a_wait_frags<T, AK, BK, N>(f1);
    ks_a_mma_il<T, 1, SLOTS>(f1, acc, do_load, issue);
    __builtin_amdgcn_sched_barrier(0);
    ks_a_load_frags<T, AK, BK>(f1, stA, stB, 3);
    __builtin_amdgcn_sched_barrier(0);
    ks_a_wait_frags<T, AK, BK, N>(f0);
    ks_a_mma_il<T, 2, SLOTS>(f0, acc, do_load, issue);
    __builtin_amdgcn_sched_barrier(0);
    ks_a_wait_frags<T, AK, BK, 0>(f1);
    ks_a_mma_il<T, 3, SLOTS>(f1, acc, do_load, issue);
}

template <class T, bool AK = false, bool BK = false, int SPREAD = 3, class AR, class BR>
__device__ __forceinline__ void ks_a_mainloop_il(AR &ar, BR &br, int kt0, int kt1, uint16_t *lds,
                                                 f32x16_t (&acc)[T::FM][T::FN]) {
    static_assert(T::STAGES == 2 && SPREAD >= 1 && SPREAD <= 4, "two stages");
    if (kt0 >= kt1) return;
    ar.issue(kt0 * 64, lds);
    br.issue(kt0 * 64, lds + T::BM * 64);
    int stage = 0;
    for (int kt = kt0; kt < kt1; ++kt) {
        ks_wait_vmcnt<0>();
        ks_barrier_nofence();
        uint16_t *nst = lds + (stage ^ 1) * T::STAGE_ELEMS;
        const int k0n = (kt + 1) * 64;
        auto issue = [&](int q) __attribute__((always_inline)) {
            if (q < T::NI_A) ar.issue_one(q, k0n, nst);
            else br.issue_one(q - T::NI_A, k0n, nst + T::BM * 64);
        };
        ks_a_tile_mma_il<T, AK, BK, SPREAD>(lds + stage * T::STAGE_ELEMS, acc, kt + 1 < kt1, issue);
        stage ^= 1;
    }
    ks_barrier_nofence();
}

template <class T, class F>
__device__ __forceinline__ void ks_a_foreach(const f32x16_t (&acc)[T::FM][T::FN], F f) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wm0 = (wave / T::WAVES_N) * T::WM, wn0 = (wave % T::WAVES_N) * T::WN;
#pragma unroll
    for (int fm = 0; fm < T::FM; ++fm)
#pragma unroll
        for (int fn = 0; fn < T::FN; ++fn)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int m = wm0 + fm * 32 + 8 * (r / 4) + 4 * (lane >> 5) + (r & 3);
                int n = wn0 + fn * 32 + (lane & 31);
                f(m, n, acc[fm][fn][r]);
            }
}

// Row-wise hand-out of the accumulator tile.  A lane of the MFMA result holds single elements of many rows, and a
// vector-memory instruction that moves 4 bytes per lane keeps the address unit busy as long as one that moves 16:
// element-wise stores run at a quarter of the rate of row-wise ones.  So the tile goes through LDS (free once the
// main loop is done) in WAVES_M slabs of BM / WAVES_M rows: ks_a_stage_slab writes slab p (the wavefronts that own
// it), and after a barrier every thread reads 16-byte pieces of whole rows with ks_a_slab_quad.  Columns are
// XOR-swizzled by 32 on every other group of four rows (the two half-wavefronts of a store hit different banks).
template <class T> struct KsASlab {
    static constexpr int ROWS = T::WM, QUADS = T::BN / 4; // rows per slab, 16-byte pieces per row
    static_assert(ROWS * T::BN * 4 <= T::LDS_ELEMS * 2, "a slab must fit into the stream stages");
    static_assert(T::BN % 64 == 0, "swizzle");
};
template <class T>
__device__ __forceinline__ void ks_a_stage_slab(const f32x16_t (&acc)[T::FM][T::FN], float *st, int p) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (wave / T::WAVES_N != p) return;
    const int wn0 = (wave % T::WAVES_N) * T::WN;
#pragma unroll
    for (int fm = 0; fm < T::FM; ++fm)
#pragma unroll
        for (int fn = 0; fn < T::FN; ++fn)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = fm * 32 + 8 * (r / 4) + 4 * (lane >> 5) + (r & 3);
                const int col = (wn0 + fn * 32 + (lane & 31)) ^ (((row >> 2) & 1) << 5);
                st[row * T::BN + col] = acc[fm][fn][r];
            }
}
// elements (row, 4 * quad .. 4 * quad + 3) of the staged slab
template <class T> __device__ __forceinline__ float4 ks_a_slab_quad(const float *st, int row, int quad) {
    return *(const float4 *)(st + row * T::BN + ((quad * 4) ^ (((row >> 2) & 1) << 5)));
}

template <class T> __device__ __forceinline__ void ks_a_clear(f32x16_t (&acc)[T::FM][T::FN]) {
#pragma unroll
    for (int fm = 0; fm < T::FM; ++fm)
#pragma unroll
        for (int fn = 0; fn < T::FN; ++fn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[fm][fn][r] = 0.f;
}
