// Shared device/host helpers of the KNN-softmax HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/knnsoftmax.h"

#define KS_WAVE 64

// ----- host helpers ---------------------------------------------------------------------------
static inline size_t ks_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline int64_t ks_ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// bump allocator over the caller's workspace; every block 256-byte aligned
struct KsArena {
    char *base;
    size_t off;
    explicit KsArena(void *p) : base((char *)p), off(0) {}
    template <typename T> T *take(size_t n) {
        T *r = (T *)(base ? base + off : nullptr);
        off += ks_align_up(n * sizeof(T), 256);
        return r;
    }
};

#define KS_LAUNCH_CHECK()                                  \
    do {                                                   \
        if (hipGetLastError() != hipSuccess) return KS_HIP_ERROR; \
    } while (0)

// ----- device helpers -------------------------------------------------------------------------
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void ks_flag(int32_t *dev_status, int bit) {
    if (dev_status) atomicOr(dev_status, bit);
}

// fp32 -> bf16 bits, round to nearest even (finite inputs; NaN stays NaN)
__device__ __forceinline__ uint32_t ks_f2bf(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}
// two fp32 -> packed bf16 pair (lo in bits 0-15), round to nearest even: one v_cvt_pk_bf16_f32 on gfx950
__device__ __forceinline__ uint32_t ks_pack_bf2(float lo, float hi) {
    typedef __bf16 ks_bf16x2 __attribute__((ext_vector_type(2)));
    typedef float ks_f32x2 __attribute__((ext_vector_type(2)));
    ks_f32x2 v = {lo, hi};
    ks_bf16x2 b = __builtin_convertvector(v, ks_bf16x2);
    return *(uint32_t *)&b;
}
__device__ __forceinline__ float ks_bf2f(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ float ks_wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float ks_wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ int ks_wave_sum_i(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
// inclusive scan inside a wave
__device__ __forceinline__ int ks_wave_iscan(int v) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int t = __shfl_up(v, o, 64);
        if (lane >= o) v += t;
    }
    return v;
}
// exclusive scan over a block of NT threads (NT multiple of 64, <= 1024); returns the exclusive prefix
// of v, and the block total through *total.  `sh` needs NT/64 + 1 ints of LDS.  Contains barriers.
template <int NT> __device__ __forceinline__ int ks_block_escan(int v, int *sh, int *total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int inc = ks_wave_iscan(v);
    if (lane == 63) sh[w] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int i = 0; i < NT / 64; ++i) { int t = sh[i]; sh[i] = run; run += t; }
        sh[NT / 64] = run;
    }
    __syncthreads();
    int r = inc - v + sh[w];
    *total = sh[NT / 64];
    __syncthreads();
    return r;
}
