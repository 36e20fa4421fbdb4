// bf16 MFMA tile engine for gfx950 (64-wide wavefronts, v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//
// A workgroup computes a BM x BN tile of  C[m][n] = sum_k A[m][k] * B[n][k].  Both operands are staged
// through LDS in "row = m (or n), k contiguous" form, rows padded by 8 elements so that the 16-byte
// fragment reads of 32 consecutive rows fall on distinct banks.  Operands that live in memory with k
// as the slow index (k-major) are transposed on the way: each thread loads an 8(k) x 8(column) block
// with 16-byte loads and writes its 8 columns as 16-byte LDS rows.
//
// Software pipeline: two LDS buffers; the global loads of k-tile t+1 are issued before the MFMAs of
// k-tile t and written to the other buffer afterwards, one barrier per k-tile.
#pragma once
#include "ks_common.h"

template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_> struct KsTile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
    static constexpr int NT = WAVES_M * WAVES_N * 64;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N; // per-wave tile
    static constexpr int FM = WM / 32, FN = WN / 32;           // 32x32 blocks per wave
    static constexpr int LDK = BK + 8;                         // padded LDS row, in bf16 elements
    static constexpr int LDS_ELEMS = 2 * (BM + BN) * LDK;      // two buffers
    static_assert(WM % 32 == 0 && WN % 32 == 0 && BK % 16 == 0, "tile shape");
};

// ---------------------------------------------------------------------------------------------
// Operand with k contiguous: element (row, k) at base[src_row(row) * ld + k]; src_row goes through an
// optional gather index.  Rows >= row_limit and k >= k_limit read as zero (k_limit % 8 == 0).
// ---------------------------------------------------------------------------------------------
template <int ROWS, int BK, int NT> struct KsRowLoader {
    static constexpr int CPR = BK / 8;            // 16-byte chunks per row
    static constexpr int CH = ROWS * CPR / NT;    // chunks per thread
    static_assert(ROWS * CPR % NT == 0 && CH >= 1, "loader shape");
    uint4 regs[CH];
    const uint16_t *ptr[CH]; // row start + chunk offset, or nullptr
    int k_limit;

    __device__ __forceinline__ void init(const uint16_t *base, int64_t ld, const int32_t *gidx, int row0,
                                         int row_limit, int k_limit_) {
        k_limit = k_limit_;
#pragma unroll
        for (int e = 0; e < CH; ++e) {
            int q = e * NT + threadIdx.x;
            int row = q / CPR, kc = q % CPR;
            int gr = row0 + row;
            if (gr < row_limit) {
                int64_t src = gidx ? (int64_t)gidx[gr] : (int64_t)gr;
                ptr[e] = base + src * ld + kc * 8;
            } else {
                ptr[e] = nullptr;
            }
        }
    }
    __device__ __forceinline__ void load(int k0) {
#pragma unroll
        for (int e = 0; e < CH; ++e) {
            int kc = (e * NT + threadIdx.x) % CPR;
            if (ptr[e] && k0 + kc * 8 < k_limit) regs[e] = *(const uint4 *)(ptr[e] + k0);
            else regs[e] = make_uint4(0, 0, 0, 0);
        }
    }
    __device__ __forceinline__ void store(uint16_t *lds) const { // lds: [ROWS][BK + 8]
#pragma unroll
        for (int e = 0; e < CH; ++e) {
            int q = e * NT + threadIdx.x;
            int row = q / CPR, kc = q % CPR;
            *(uint4 *)(lds + row * (BK + 8) + kc * 8) = regs[e];
        }
    }
};

// ---------------------------------------------------------------------------------------------
// Operand stored k-major: element (k, col) at base[src_row(k) * ld + col]; src_row goes through an
// optional gather index on k.  k >= k_limit and col >= col_limit read as zero (col_limit % 8 == 0).
// The tile lands in LDS as [COLS][BK + 8], i.e. transposed.
// ---------------------------------------------------------------------------------------------
template <int COLS, int BK, int NT> struct KsColLoader {
    static constexpr int CB = COLS / 8;                  // column blocks
    static constexpr int TOTAL = (BK / 8) * CB;          // 8x8 sub-blocks in the tile
    static constexpr int SB = (TOTAL + NT - 1) / NT;     // sub-blocks per thread (threads beyond TOTAL idle)
    static_assert(TOTAL % NT == 0 || TOTAL < NT, "loader shape");
    uint4 regs[SB][8];
    const uint16_t *base;
    const int32_t *gidx;
    int64_t ld;
    int col0, col_limit, k_limit;

    __device__ __forceinline__ void init(const uint16_t *base_, int64_t ld_, const int32_t *gidx_, int col0_,
                                         int col_limit_, int k_limit_) {
        base = base_; ld = ld_; gidx = gidx_; col0 = col0_; col_limit = col_limit_; k_limit = k_limit_;
    }
    __device__ __forceinline__ void load(int k0) {
#pragma unroll
        for (int e = 0; e < SB; ++e) {
            int q = e * NT + threadIdx.x;
            if (TOTAL < NT && q >= TOTAL) continue;
            int cb = q % CB, kb = q / CB;
            int col = col0 + cb * 8;
            bool col_ok = col < col_limit;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                int kg = k0 + kb * 8 + kk;
                if (col_ok && kg < k_limit) {
                    int64_t src = gidx ? (int64_t)gidx[kg] : (int64_t)kg;
                    regs[e][kk] = *(const uint4 *)(base + src * ld + col);
                } else {
                    regs[e][kk] = make_uint4(0, 0, 0, 0);
                }
            }
        }
    }
    static __device__ __forceinline__ uint32_t dword(const uint4 &v, int i) {
        return i == 0 ? v.x : (i == 1 ? v.y : (i == 2 ? v.z : v.w));
    }
    __device__ __forceinline__ void store(uint16_t *lds) const { // lds: [COLS][BK + 8]
#pragma unroll
        for (int e = 0; e < SB; ++e) {
            int q = e * NT + threadIdx.x;
            if (TOTAL < NT && q >= TOTAL) continue;
            int cb = q % CB, kb = q / CB;
#pragma unroll
            for (int n = 0; n < 8; ++n) {
                uint32_t o[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    // column n of rows k = 2j (goes to the low 16 bits) and k = 2j + 1 (high 16 bits)
                    uint32_t a = dword(regs[e][2 * j], n >> 1), b = dword(regs[e][2 * j + 1], n >> 1);
                    o[j] = (n & 1) ? ((a >> 16) | (b & 0xFFFF0000u)) : ((a & 0xFFFFu) | (b << 16));
                }
                *(uint4 *)(lds + (cb * 8 + n) * (BK + 8) + kb * 8) = make_uint4(o[0], o[1], o[2], o[3]);
            }
        }
    }
};

// ---------------------------------------------------------------------------------------------
// MFMAs of one k-tile from LDS
// ---------------------------------------------------------------------------------------------
template <class T>
__device__ __forceinline__ void ks_tile_mma(const uint16_t *ldsA, const uint16_t *ldsB, int wm0, int wn0,
                                            f32x16_t (&acc)[T::FM][T::FN]) {
    const int lane = threadIdx.x & 63;
    const int r = lane & 31, kh = (lane >> 5) * 8;
#pragma unroll
    for (int kk = 0; kk < T::BK / 16; ++kk) {
        bf16x8_t a[T::FM], b[T::FN];
#pragma unroll
        for (int fm = 0; fm < T::FM; ++fm)
            a[fm] = *(const bf16x8_t *)(ldsA + (wm0 + fm * 32 + r) * T::LDK + kk * 16 + kh);
#pragma unroll
        for (int fn = 0; fn < T::FN; ++fn)
            b[fn] = *(const bf16x8_t *)(ldsB + (wn0 + fn * 32 + r) * T::LDK + kk * 16 + kh);
#pragma unroll
        for (int fm = 0; fm < T::FM; ++fm)
#pragma unroll
            for (int fn = 0; fn < T::FN; ++fn)
                acc[fm][fn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[fm], b[fn], acc[fm][fn], 0, 0, 0);
    }
}

// Main loop over k-tiles [kt_begin, kt_end) (k0 = kt * BK).  acc is accumulated into (not cleared).
template <class T, class AL, class BL>
__device__ __forceinline__ void ks_gemm_mainloop(AL &al, BL &bl, int kt_begin, int kt_end, uint16_t *lds,
                                                 f32x16_t (&acc)[T::FM][T::FN]) {
    constexpr int BUF = (T::BM + T::BN) * T::LDK;
    const int wave = threadIdx.x >> 6;
    const int wm0 = (wave / T::WAVES_N) * T::WM, wn0 = (wave % T::WAVES_N) * T::WN;
    if (kt_begin >= kt_end) return;
    al.load(kt_begin * T::BK);
    bl.load(kt_begin * T::BK);
    al.store(lds);
    bl.store(lds + T::BM * T::LDK);
    __syncthreads();
    for (int kt = kt_begin; kt < kt_end; ++kt) {
        uint16_t *cur = lds + ((kt - kt_begin) & 1) * BUF;
        uint16_t *nxt = lds + (((kt - kt_begin) & 1) ^ 1) * BUF;
        const bool more = kt + 1 < kt_end;
        if (more) {
            al.load((kt + 1) * T::BK);
            bl.load((kt + 1) * T::BK);
        }
        ks_tile_mma<T>(cur, cur + T::BM * T::LDK, wm0, wn0, acc);
        if (more) {
            al.store(nxt);
            bl.store(nxt + T::BM * T::LDK);
        }
        __syncthreads();
    }
}

// Visit every accumulator element of this wave: f(m, n, value) with m, n relative to the tile origin.
// Register r of a 32x32 block holds row 8*(r/4) + 4*(lane/32) + r%4, column lane%32.
template <class T, class F>
__device__ __forceinline__ void ks_tile_foreach(const f32x16_t (&acc)[T::FM][T::FN], F f) {
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

template <class T> __device__ __forceinline__ void ks_tile_clear(f32x16_t (&acc)[T::FM][T::FN]) {
#pragma unroll
    for (int fm = 0; fm < T::FM; ++fm)
#pragma unroll
        for (int fn = 0; fn < T::FN; ++fn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[fm][fn][r] = 0.f;
}

// Launch-order -> tile-order remap for the 8 XCDs of the chip: consecutive workgroup ids go round-robin
// to the XCDs, each with its own L2, so XCD x is given a contiguous range of logical tile ids and tiles
// that share an operand panel meet in one L2.  Bijection on [0, n).
__device__ __forceinline__ int ks_xcd_remap(int id, int n) {
    const int q = n >> 3, rem = n & 7;
    const int x = id & 7, slot = id >> 3;
    return x * q + (x < rem ? x : rem) + slot;
}
