// Measurement aids: what this chip actually reaches on the two rooflines the kernels are priced against.
//   ks_peak_mfma   a loop of independent v_mfma_f32_32x32x16_bf16 on registers only (no memory, no LDS): the rate
//                  the matrix pipes sustain at the clock the chip settles at under that load;
//   ks_peak_copy   a streaming copy of a large buffer (16-byte loads and stores): the HBM rate a
//                  kernel with nothing else to do reaches.
// Both only launch kernels on the caller's stream; the caller times them (events) and divides.
#include "ks_common.h"

#define PK_NT 256
#define PK_NACC 16 /* independent accumulators per wavefront: no MFMA waits for the one before */

__global__ void __launch_bounds__(PK_NT) pk_mfma_kernel(float *out, int iters) {
    bf16x8_t a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)((threadIdx.x & 63) * 0.001f);
        b[e] = (__bf16)(e * 0.01f);
    }
    f32x16_t acc[PK_NACC];
#pragma unroll
    for (int i = 0; i < PK_NACC; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < PK_NACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < PK_NACC; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[(size_t)blockIdx.x * PK_NT + threadIdx.x] = s; // keeps the loop alive
}

// every workgroup copies one contiguous share of the buffer, eight independent 16-byte pieces per thread and round
// (of the layouts tried -- grid-stride or contiguous shares, four or eight pieces, nontemporal or plain accesses --
// this one came out fastest on the chip)
__global__ void __launch_bounds__(PK_NT) pk_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16) {
    constexpr int U = 8;
    const size_t per_block = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t begin = (size_t)blockIdx.x * per_block;
    const size_t end = begin + per_block < n16 ? begin + per_block : n16;
    size_t i = begin + threadIdx.x;
    for (; i + (U - 1) * PK_NT < end; i += U * PK_NT) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = src[i + u * PK_NT];
#pragma unroll
        for (int u = 0; u < U; ++u) dst[i + u * PK_NT] = v[u];
    }
    for (; i < end; i += PK_NT) dst[i] = src[i];
}

// flops = workgroups * 4 wavefronts * iters * PK_NACC * 32768.  `out` needs workgroups * 256 floats.
extern "C" int ks_peak_mfma(float *out, int workgroups, int iters, double *flops, void *stream) {
    if (!out || workgroups < 1 || iters < 1) return KS_INVALID_ARG;
    hipLaunchKernelGGL(pk_mfma_kernel, dim3(workgroups), dim3(PK_NT), 0, (hipStream_t)stream, out, iters);
    if (flops) *flops = (double)workgroups * (PK_NT / 64) * (double)iters * PK_NACC * 32768.0;
    KS_LAUNCH_CHECK();
    return KS_OK;
}

// copies `bytes` (a multiple of 16) from src to dst; traffic = 2 * bytes
extern "C" int ks_peak_copy(const void *src, void *dst, size_t bytes, int workgroups, void *stream) {
    if (!src || !dst || bytes < 16 || bytes % 16 != 0 || workgroups < 1) return KS_INVALID_ARG;
    if (((uintptr_t)src | (uintptr_t)dst) & 15) return KS_INVALID_ARG;
    hipLaunchKernelGGL(pk_copy_kernel, dim3(workgroups), dim3(PK_NT), 0, (hipStream_t)stream, (const uint4 *)src, (uint4 *)dst,
                       bytes / 16);
    KS_LAUNCH_CHECK();
    return KS_OK;
}
