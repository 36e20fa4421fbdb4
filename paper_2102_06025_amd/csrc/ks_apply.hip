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


// ------------------------------------------------------------------------------------------------
// Normalisation inside the layer (paper Section 3.2.3, GPU pipeline step 2: W and X are normalised on the GPU): the layer keeps
// W un-normalised in fp32, its matrix kernels read the normalised 16-bit copy W_hat = W / |W| (row-wise), and
// gradients with respect to normalised rows are brought back through
//     dv = (g - v_hat <v_hat, g>) / |v|.
// All of it is row-local HBM-bound work: one wavefront per row, the row's two or three reductions in fp64.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ double ap_wave_sum_d(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const int lo = __shfl_xor(__double2loint(v), o, 64), hi = __shfl_xor(__double2hiint(v), o, 64);
        v += __hiloint2double(hi, lo);
    }
    return v;
}
template <typename IN> struct ApElem4;
template <> struct ApElem4<float> {
    static __device__ __forceinline__ float4 load(const float *p) { return *(const float4 *)p; }
};
template <> struct ApElem4<uint16_t> {
    static __device__ __forceinline__ float4 load(const uint16_t *p) {
        const uint2 v = *(const uint2 *)p;
        return make_float4(ks_bf2f(v.x & 0xFFFFu), ks_bf2f(v.x >> 16), ks_bf2f(v.y & 0xFFFFu), ks_bf2f(v.y >> 16));
    }
};
__device__ __forceinline__ double ap_dot4(float4 a, float4 b, double acc) {
    acc = __builtin_fma((double)a.x, (double)b.x, acc);
    acc = __builtin_fma((double)a.y, (double)b.y, acc);
    acc = __builtin_fma((double)a.z, (double)b.z, acc);
    return __builtin_fma((double)a.w, (double)b.w, acc);
}

// V_hat_bf16[i,:] = bf16(fp32(V[i,:] / |V[i,:]|)), inv_norm[i] = 1 / |V[i,:]| (0 for a zero row)
template <typename IN>
__global__ void __launch_bounds__(AP_NT)
normalize_rows_kernel(const IN *__restrict__ V, int64_t n, int D, uint16_t *__restrict__ Vh, float *__restrict__ inv_norm) {
    const int64_t i = (int64_t)blockIdx.x * (AP_NT / 64) + (threadIdx.x >> 6);
    if (i >= n) return;
    const int lane = threadIdx.x & 63;
    const IN *v = V + i * D;
    double ss = 0.0;
    for (int d = lane * 4; d < D; d += 256) {
        const float4 x = ApElem4<IN>::load(v + d);
        ss = ap_dot4(x, x, ss);
    }
    ss = ap_wave_sum_d(ss);
    const double inv = ss > 0.0 ? 1.0 / sqrt(ss) : 0.0;
    if (lane == 0 && inv_norm) inv_norm[i] = (float)inv;
    if (!Vh) return;
    for (int d = lane * 4; d < D; d += 256) {
        const float4 x = ApElem4<IN>::load(v + d);
        const float h0 = (float)((double)x.x * inv), h1 = (float)((double)x.y * inv), h2 = (float)((double)x.z * inv),
                    h3 = (float)((double)x.w * inv);
        *(uint2 *)(Vh + i * D + d) = make_uint2(ks_pack_bf2(h0, h1), ks_pack_bf2(h2, h3));
    }
}

// dV[i,:] = (G[i,:] - v_hat <v_hat, G[i,:]>) / |v|   (dV may be G)
template <typename IN>
__global__ void __launch_bounds__(AP_NT)
norm_backward_rows_kernel(const IN *__restrict__ V, const float *__restrict__ G, int64_t n, int D, float *__restrict__ dV) {
    const int64_t i = (int64_t)blockIdx.x * (AP_NT / 64) + (threadIdx.x >> 6);
    if (i >= n) return;
    const int lane = threadIdx.x & 63;
    const IN *v = V + i * D;
    const float *g = G + i * D;
    double ss = 0.0, dot = 0.0;
    for (int d = lane * 4; d < D; d += 256) {
        const float4 x = ApElem4<IN>::load(v + d);
        ss = ap_dot4(x, x, ss);
        dot = ap_dot4(x, *(const float4 *)(g + d), dot);
    }
    ss = ap_wave_sum_d(ss);
    dot = ap_wave_sum_d(dot);
    const double inv = ss > 0.0 ? 1.0 / sqrt(ss) : 0.0;
    const double c = dot * inv * inv; // <v_hat, g> / |v|
    for (int d = lane * 4; d < D; d += 256) {
        const float4 x = ApElem4<IN>::load(v + d);
        const float4 gg = *(const float4 *)(g + d);
        float4 o;
        o.x = (float)(((double)gg.x - (double)x.x * c) * inv);
        o.y = (float)(((double)gg.y - (double)x.y * c) * inv);
        o.z = (float)(((double)gg.z - (double)x.z * c) * inv);
        o.w = (float)(((double)gg.w - (double)x.w * c) * inv);
        *(float4 *)(dV + i * D + d) = o;
    }
}

// one wavefront: master row w of class c updated from the gradient g with respect to its normalised copy
__device__ __forceinline__ void ap_update_row_normalized(float *__restrict__ w, uint16_t *__restrict__ wh,
                                                         float *__restrict__ inv_out, const float *__restrict__ g,
                                                         double alpha, int D) {
    const int lane = threadIdx.x & 63;
    double ss = 0.0, dot = 0.0;
    for (int d = lane * 4; d < D; d += 256) {
        const float4 x = *(const float4 *)(w + d);
        ss = ap_dot4(x, x, ss);
        dot = ap_dot4(x, *(const float4 *)(g + d), dot);
    }
    ss = ap_wave_sum_d(ss);
    dot = ap_wave_sum_d(dot);
    const double inv = ss > 0.0 ? 1.0 / sqrt(ss) : 0.0;
    const double c = dot * inv * inv;
    double s2 = 0.0;
    for (int d = lane * 4; d < D; d += 256) { // second pass over the row (it is in cache)
        float4 x = *(const float4 *)(w + d);
        const float4 gg = *(const float4 *)(g + d);
        if (ss > 0.0) {
            x.x = (float)((double)x.x + alpha * (((double)gg.x - (double)x.x * c) * inv));
            x.y = (float)((double)x.y + alpha * (((double)gg.y - (double)x.y * c) * inv));
            x.z = (float)((double)x.z + alpha * (((double)gg.z - (double)x.z * c) * inv));
            x.w = (float)((double)x.w + alpha * (((double)gg.w - (double)x.w * c) * inv));
            *(float4 *)(w + d) = x;
        }
        s2 = ap_dot4(x, x, s2);
    }
    s2 = ap_wave_sum_d(s2);
    const double inv2 = s2 > 0.0 ? 1.0 / sqrt(s2) : 0.0;
    if (lane == 0 && inv_out) *inv_out = (float)inv2;
    if (!wh) return;
    __builtin_amdgcn_s_waitcnt(0x0070); // vmcnt(0): this wavefront's stores of the row are done before it is read back
    for (int d = lane * 4; d < D; d += 256) {
        const float4 x = *(const float4 *)(w + d);
        const float h0 = (float)((double)x.x * inv2), h1 = (float)((double)x.y * inv2), h2 = (float)((double)x.z * inv2),
                    h3 = (float)((double)x.w * inv2);
        *(uint2 *)(wh + d) = make_uint2(ks_pack_bf2(h0, h1), ks_pack_bf2(h2, h3));
    }
}

// strictly ascending idx: one wavefront per position
__global__ void __launch_bounds__(AP_NT)
apply_norm_sorted_kernel(float *__restrict__ Wm, uint16_t *__restrict__ Wh, float *__restrict__ inv_norm,
                         const int32_t *__restrict__ idx, const int32_t *__restrict__ n_p, int n_max,
                         const float *__restrict__ dW, float alpha, int64_t C, int D, int32_t *dev_status) {
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
        if (lane0) ks_flag(dev_status, KS_DEV_IDX_NOT_SORTED);
        return;
    }
    ap_update_row_normalized(Wm + (int64_t)c * D, Wh ? Wh + (int64_t)c * D : nullptr, inv_norm ? inv_norm + c : nullptr,
                             dW + (int64_t)p * D, (double)alpha, D);
}

// repeated idx: the head of a segment of the sorted keys sums its rows (ascending position) into its row of
// `gsum`, then updates the class from that sum
__global__ void __launch_bounds__(AP_NT)
apply_norm_segments_kernel(float *__restrict__ Wm, uint16_t *__restrict__ Wh, float *__restrict__ inv_norm,
                           const uint64_t *__restrict__ keys, int n_pow2, const float *__restrict__ dW, float alpha, int D,
                           float *__restrict__ gsum) {
    const int q = blockIdx.x * (AP_NT / 64) + (threadIdx.x >> 6);
    if (q >= n_pow2) return;
    const uint64_t key = keys[q];
    if (key == ~0ull) return;
    const uint32_t c = (uint32_t)(key >> 32);
    if (q > 0 && (uint32_t)(keys[q - 1] >> 32) == c) return; // not the head of its segment
    const int lane = threadIdx.x & 63;
    float *gs = gsum + (int64_t)q * D;
    for (int d = lane * 4; d < D; d += 256) {
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0; // fp64 sum, rounded to fp32 once
        for (int r = q; r < n_pow2; ++r) {
            const uint64_t kr = keys[r];
            if ((uint32_t)(kr >> 32) != c || kr == ~0ull) break;
            const float4 v = *(const float4 *)(dW + (int64_t)(uint32_t)kr * D + d);
            s0 += v.x; s1 += v.y; s2 += v.z; s3 += v.w;
        }
        *(float4 *)(gs + d) = make_float4((float)s0, (float)s1, (float)s2, (float)s3);
    }
    __builtin_amdgcn_s_waitcnt(0x0070); // vmcnt(0): the sum is in memory before the wavefront reads it back
    ap_update_row_normalized(Wm + (int64_t)c * D, Wh ? Wh + (int64_t)c * D : nullptr, inv_norm ? inv_norm + c : nullptr, gs,
                             (double)alpha, D);
}

static void ap_sort_keys(const int32_t *idx, const int32_t *n, int n_max, int np2, int64_t C, uint64_t *keys,
                         int32_t *dev_status, hipStream_t st);
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
    ap_sort_keys(idx, n, n_max, np2, C, keys, dev_status, st); // steps with j < AP_CHUNK run in LDS, the others one launch each
    hipLaunchKernelGGL(apply_segments_kernel, dim3((unsigned)ks_ceil_div(np2, AP_NT / 64)), dim3(AP_NT), 0, st, W_master,
                       W_bf16, keys, np2, dW, alpha, D);
    KS_LAUNCH_CHECK();
    return KS_OK;
}

// sort of the (class, position) keys shared by the two update entry points
static void ap_sort_keys(const int32_t *idx, const int32_t *n, int n_max, int np2, int64_t C, uint64_t *keys,
                         int32_t *dev_status, hipStream_t st) {
    const unsigned gb = (unsigned)ks_ceil_div(np2, AP_NT);
    hipLaunchKernelGGL(apply_keys_kernel, dim3(gb), dim3(AP_NT), 0, st, idx, n, n_max, np2, C, keys, dev_status);
    const unsigned cb = (unsigned)ks_ceil_div(np2, AP_CHUNK);
    hipLaunchKernelGGL(apply_bitonic_lds_kernel, dim3(cb), dim3(AP_NT), 0, st, keys, np2, 2, np2 < AP_CHUNK ? np2 : AP_CHUNK);
    for (int k = AP_CHUNK * 2; k <= np2; k <<= 1) {
        for (int j = k >> 1; j >= AP_CHUNK; j >>= 1)
            hipLaunchKernelGGL(apply_bitonic_kernel, dim3(gb), dim3(AP_NT), 0, st, keys, np2, k, j);
        hipLaunchKernelGGL(apply_bitonic_lds_kernel, dim3(cb), dim3(AP_NT), 0, st, keys, np2, k, k);
    }
}

extern "C" int knn_normalize_rows(const void *V, int dtype, int64_t n, int D, uint16_t *V_hat_bf16, float *inv_norm,
                                  void *stream) {
    if (!V || (!V_hat_bf16 && !inv_norm)) return KS_INVALID_ARG;
    if (n < 1 || D < 4 || D % 4 != 0) return KS_INVALID_ARG;
    if (dtype != KS_DTYPE_BF16 && dtype != KS_DTYPE_FP32) return KS_INVALID_ARG;
    const dim3 grid((unsigned)ks_ceil_div(n, AP_NT / 64));
    if (dtype == KS_DTYPE_FP32)
        hipLaunchKernelGGL(normalize_rows_kernel<float>, grid, dim3(AP_NT), 0, (hipStream_t)stream, (const float *)V, n, D,
                           V_hat_bf16, inv_norm);
    else
        hipLaunchKernelGGL(normalize_rows_kernel<uint16_t>, grid, dim3(AP_NT), 0, (hipStream_t)stream, (const uint16_t *)V, n,
                           D, V_hat_bf16, inv_norm);
    KS_LAUNCH_CHECK();
    return KS_OK;
}

extern "C" int knn_norm_backward_rows(const void *V, int dtype, const float *G, int64_t n, int D, float *dV, void *stream) {
    if (!V || !G || !dV) return KS_INVALID_ARG;
    if (n < 1 || D < 4 || D % 4 != 0) return KS_INVALID_ARG;
    if (dtype != KS_DTYPE_BF16 && dtype != KS_DTYPE_FP32) return KS_INVALID_ARG;
    const dim3 grid((unsigned)ks_ceil_div(n, AP_NT / 64));
    if (dtype == KS_DTYPE_FP32)
        hipLaunchKernelGGL(norm_backward_rows_kernel<float>, grid, dim3(AP_NT), 0, (hipStream_t)stream, (const float *)V, G, n,
                           D, dV);
    else
        hipLaunchKernelGGL(norm_backward_rows_kernel<uint16_t>, grid, dim3(AP_NT), 0, (hipStream_t)stream,
                           (const uint16_t *)V, G, n, D, dV);
    KS_LAUNCH_CHECK();
    return KS_OK;
}

extern "C" size_t apply_weight_grad_normalized_workspace(int64_t C, int D, int n_max, int idx_sorted_unique) {
    (void)C;
    if (n_max < 1 || D < 4) return 0;
    if (idx_sorted_unique) return 256;
    const size_t np2 = (size_t)ap_pow2(n_max);
    return ks_align_up(np2 * sizeof(uint64_t), 256) + ks_align_up(np2 * (size_t)D * sizeof(float), 256);
}

extern "C" int apply_weight_grad_normalized(float *W_master, uint16_t *W_hat_bf16, float *inv_norm, const int32_t *idx,
                                            const int32_t *n, int n_max, const float *dW_hat, float alpha, int64_t C, int D,
                                            int idx_sorted_unique, void *ws, size_t ws_bytes, int32_t *dev_status,
                                            void *stream) {
    if (!W_master || !idx || !dW_hat) return KS_INVALID_ARG;
    if (n_max < 1 || C < 1 || C >= (int64_t)1 << 31 || D < 4 || D % 4 != 0) return KS_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (idx_sorted_unique) {
        hipLaunchKernelGGL(apply_norm_sorted_kernel, dim3((unsigned)ks_ceil_div(n_max, AP_NT / 64)), dim3(AP_NT), 0, st,
                           W_master, W_hat_bf16, inv_norm, idx, n, n_max, dW_hat, alpha, C, D, dev_status);
        KS_LAUNCH_CHECK();
        return KS_OK;
    }
    if (!ws) return KS_INVALID_ARG;
    if (ws_bytes < apply_weight_grad_normalized_workspace(C, D, n_max, 0)) return KS_WORKSPACE_TOO_SMALL;
    const int np2 = ap_pow2(n_max);
    uint64_t *keys = (uint64_t *)ws;
    float *gsum = (float *)((char *)ws + ks_align_up((size_t)np2 * sizeof(uint64_t), 256));
    ap_sort_keys(idx, n, n_max, np2, C, keys, dev_status, st);
    hipLaunchKernelGGL(apply_norm_segments_kernel, dim3((unsigned)ks_ceil_div(np2, AP_NT / 64)), dim3(AP_NT), 0, st, W_master,
                       W_hat_bf16, inv_norm, keys, np2, dW_hat, alpha, D, gsum);
    KS_LAUNCH_CHECK();
    return KS_OK;
}
