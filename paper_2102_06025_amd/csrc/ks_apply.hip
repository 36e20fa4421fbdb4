// Local weight update of the model-parallel fc layer (paper Section 3.1 step 6): fp32 master rows are
// updated from the gradient rows addressed to them and the bf16 compute copy is refreshed.
//
// Atomic-free and deterministic.  Two paths:
//   - idx strictly ascending (the active list of one step): one wavefront per row, a single streaming pass.
//   - idx with repeats: (class id, position) keys are sorted (bitonic, in the workspace), so that the rows
//     addressed to one class are adjacent and in ascending position; the wavefront at the head of each
//     segment sums its segment in that order and applies it.
#include "ks_common.h"

#define AP_NT 256

__device__ __forceinline__ int ap_count(const int32_t *n, int n_max, int32_t *dev_status) {
    int v = n ? *n : n_max;
    if (v < 0 || v > n_max) {
        if (threadIdx.x == 0 && blockIdx.x == 0) ks_flag(dev_status, KS_DEV_BAD_COUNT);
        v = v < 0 ? 0 : n_max;
    }
    return v;
}

__device__ __forceinline__ void ap_update4(float *__restrict__ wm, uint16_t *__restrict__ wb, float alpha, float4 g) {
    float4 w = *(const float4 *)wm;
    w.x = fmaf(alpha, g.x, w.x);
    w.y = fmaf(alpha, g.y, w.y);
    w.z = fmaf(alpha, g.z, w.z);
    w.w = fmaf(alpha, g.w, w.w);
    *(float4 *)wm = w;
    if (wb) *(uint2 *)wb = make_uint2(ks_pack_bf2(w.x, w.y), ks_pack_bf2(w.z, w.w));
}

// strictly ascending idx: one wavefront per position
__global__ void __launch_bounds__(AP_NT)
apply_sorted_kernel(float *__restrict__ Wm, uint16_t *__restrict__ Wb, const int32_t *__restrict__ idx,
                    const int32_t *__restrict__ n_p, int n_max, const float *__restrict__ dW, float alpha, int64_t C,
                    int D, int32_t *dev_status) {
    const int n = ap_count(n_p, n_max, dev_status);
    const int p = blockIdx.x * (AP_NT / 64) + (threadIdx.x >> 6);
    if (p >= n) return;
    const int32_t c = idx[p];
    const bool lane0 = (threadIdx.x & 63) == 0;
    if (c < 0 || c >= C) {
        if (lane0) ks_flag(dev_status, KS_DEV_BAD_INDEX);
        return;
    }
    if (p > 0 && idx[p - 1] >= c) {
        // the promise is broken: two wavefronts could race on one row, so this position is skipped
        if (lane0) ks_flag(dev_status, KS_DEV_IDX_NOT_SORTED);
        return;
    }
    float *wm = Wm + (int64_t)c * D;
    uint16_t *wb = Wb ? Wb + (int64_t)c * D : nullptr;
    const float *dw = dW + (int64_t)p * D;
    for (int d = (threadIdx.x & 63) * 4; d < D; d += 256)
        ap_update4(wm + d, wb ? wb + d : nullptr, alpha, *(const float4 *)(dw + d));
}

// ---- general path ------------------------------------------------------------------------------
// key = class id in the high word, position in the low word; invalid / padding entries sort last
__global__ void __launch_bounds__(AP_NT)
apply_keys_kernel(const int32_t *__restrict__ idx, const int32_t *__restrict__ n_p, int n_max, int n_pow2, int64_t C,
                  uint64_t *keys, int32_t *dev_status) {
    const int n = ap_count(n_p, n_max, dev_status);
    int p = blockIdx.x * AP_NT + threadIdx.x;
    if (p >= n_pow2) return;
    uint64_t key = ~0ull;
    if (p < n) {
        int32_t c = idx[p];
        if (c < 0 || c >= C) ks_flag(dev_status, KS_DEV_BAD_INDEX);
        else key = ((uint64_t)(uint32_t)c << 32) | (uint32_t)p;
    }
    keys[p] = key;
}

// one compare-exchange step of the bitonic network (ascending sort)
__global__ void __launch_bounds__(AP_NT) apply_bitonic_kernel(uint64_t *keys, int n_pow2, int k, int j) {
    int t = blockIdx.x * AP_NT + threadIdx.x;
    if (t >= n_pow2) return;
    int partner = t ^ j;
    if (partner <= t) return;
    uint64_t a = keys[t], b = keys[partner];
    bool up = (t & k) == 0;
    if ((a > b) == up) {
        keys[t] = b;
        keys[partner] = a;
    }
}

// whole network on one workgroup's chunk in LDS, for the steps with j < chunk (k from k_begin to k_end)
#define AP_CHUNK 2048
__global__ void __launch_bounds__(AP_NT) apply_bitonic_lds_kernel(uint64_t *keys, int n_pow2, int k_begin, int k_end) {
    __shared__ uint64_t sh[AP_CHUNK];
    const int base = blockIdx.x * AP_CHUNK;
    for (int e = threadIdx.x; e < AP_CHUNK; e += AP_NT) sh[e] = (base + e < n_pow2) ? keys[base + e] : ~0ull;
    __syncthreads();
    for (int k = k_begin; k <= k_end; k <<= 1) {
        int j0 = (k >> 1) < AP_CHUNK ? (k >> 1) : (AP_CHUNK >> 1);
        for (int j = j0; j > 0; j >>= 1) {
            for (int e = threadIdx.x; e < AP_CHUNK; e += AP_NT) {
                int partner = e ^ j;
                if (partner > e) {
                    uint64_t a = sh[e], b = sh[partner];
                    bool up = ((base + e) & k) == 0;
                    if ((a > b) == up) { sh[e] = b; sh[partner] = a; }
                }
            }
            __syncthreads();
        }
    }
    for (int e = threadIdx.x; e < AP_CHUNK; e += AP_NT)
        if (base + e < n_pow2) keys[base + e] = sh[e];
}

// one wavefront per sorted position; the head of a segment sums and applies it (D <= 1024 * 4 per pass)
__global__ void __launch_bounds__(AP_NT)
apply_segments_kernel(float *__restrict__ Wm, uint16_t *__restrict__ Wb, const uint64_t *__restrict__ keys, int n_pow2,
                      const float *__restrict__ dW, float alpha, int D) {
    const int q = blockIdx.x * (AP_NT / 64) + (threadIdx.x >> 6);
    if (q >= n_pow2) return;
    const uint64_t key = keys[q];
    if (key == ~0ull) return;
    const uint32_t c = (uint32_t)(key >> 32);
    if (q > 0 && (uint32_t)(keys[q - 1] >> 32) == c) return; // not the head of its segment
    const int lane = threadIdx.x & 63;
    // D is processed in slabs of 1024 columns (4 per lane, 4 passes of 64 lanes x 4 floats)
    for (int d0 = 0; d0 < D; d0 += 1024) {
        float4 sum[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) sum[it] = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int r = q; r < n_pow2; ++r) {
            uint64_t kr = keys[r];
            if ((uint32_t)(kr >> 32) != c || kr == ~0ull) break;
            const float *row = dW + (int64_t)(uint32_t)kr * D + d0;
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                int d = lane * 4 + it * 256;
                if (d0 + d < D) {
                    float4 v = *(const float4 *)(row + d);
                    sum[it].x += v.x; sum[it].y += v.y; sum[it].z += v.z; sum[it].w += v.w;
                }
            }
        }
        float *wm = Wm + (int64_t)c * D + d0;
        uint16_t *wb = Wb ? Wb + (int64_t)c * D + d0 : nullptr;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            int d = lane * 4 + it * 256;
            if (d0 + d < D) ap_update4(wm + d, wb ? wb + d : nullptr, alpha, sum[it]);
        }
    }
}

static int ap_pow2(int n) {
    int p = 1;
    while (p < n) p <<= 1;
    return p;
}

extern "C" size_t apply_weight_grad_workspace(int64_t C, int D, int n_max, int idx_sorted_unique) {
    (void)C; (void)D;
    if (n_max < 1) return 0;
    if (idx_sorted_unique) return 256; // nothing needed; a non-zero size keeps callers' allocation code uniform
    return ks_align_up((size_t)ap_pow2(n_max) * sizeof(uint64_t), 256);
}

extern "C" int apply_weight_grad(float *W_master, uint16_t *W_bf16, const int32_t *idx, const int32_t *n, int n_max,
                                 const float *dW, float alpha, int64_t C, int D, int idx_sorted_unique, void *ws,
                                 size_t ws_bytes, int32_t *dev_status, void *stream) {
    if (!W_master || !idx || !dW) return KS_INVALID_ARG;
    if (n_max < 1 || C < 1 || C >= (int64_t)1 << 31 || D < 4 || D % 4 != 0) return KS_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (idx_sorted_unique) {
        hipLaunchKernelGGL(apply_sorted_kernel, dim3((unsigned)ks_ceil_div(n_max, AP_NT / 64)), dim3(AP_NT), 0, st, W_master,
                           W_bf16, idx, n, n_max, dW, alpha, C, D, dev_status);
        KS_LAUNCH_CHECK();
        return KS_OK;
    }
    if (!ws) return KS_INVALID_ARG;
    if (ws_bytes < apply_weight_grad_workspace(C, D, n_max, 0)) return KS_WORKSPACE_TOO_SMALL;
    const int np2 = ap_pow2(n_max);
    uint64_t *keys = (uint64_t *)ws;
    const unsigned gb = (unsigned)ks_ceil_div(np2, AP_NT);
    hipLaunchKernelGGL(apply_keys_kernel, dim3(gb), dim3(AP_NT), 0, st, idx, n, n_max, np2, C, keys, dev_status);
    // steps with j < AP_CHUNK run in LDS, the others as one launch per step
    const unsigned cb = (unsigned)ks_ceil_div(np2, AP_CHUNK);
    hipLaunchKernelGGL(apply_bitonic_lds_kernel, dim3(cb), dim3(AP_NT), 0, st, keys, np2, 2, np2 < AP_CHUNK ? np2 : AP_CHUNK);
    for (int k = AP_CHUNK * 2; k <= np2; k <<= 1) {
        for (int j = k >> 1; j >= AP_CHUNK; j >>= 1)
            hipLaunchKernelGGL(apply_bitonic_kernel, dim3(gb), dim3(AP_NT), 0, st, keys, np2, k, j);
        hipLaunchKernelGGL(apply_bitonic_lds_kernel, dim3(cb), dim3(AP_NT), 0, st, keys, np2, k, k);
    }
    hipLaunchKernelGGL(apply_segments_kernel, dim3((unsigned)ks_ceil_div(np2, AP_NT / 64)), dim3(AP_NT), 0, st, W_master,
                       W_bf16, keys, np2, dW, alpha, D);
    KS_LAUNCH_CHECK();
    return KS_OK;
}
