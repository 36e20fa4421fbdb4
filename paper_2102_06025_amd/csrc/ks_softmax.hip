// KNN-softmax forward + backward on the active classes (paper Section 3.2; Section 3.1 steps 3-5).
//
// Pipeline on one stream (A = number of active classes, known only on the device):
//   select            -> active_idx, n_active, target_pos                         (ks_select.hip)
//   logits GEMM       Z[B, A]  = scale * X . W[active]^T     rows of W fetched through the index list
//   row statistics    lse_i, loss_i                           one workgroup per sample
//   loss mean         fixed-order tree sum
//   logit gradient    dZ[B, A] = g (exp(Z - lse) - onehot)    bf16
//   dX GEMM           split over the active dimension, partial tiles summed in a fixed order
//   dW GEMM           dW_active[A, D] = scale * dZ^T . X
// Launch sizes are taken from the cap M; workgroups beyond the active count exit at once.
#include "ks_gemm.h"
#include "ks_gemm_async.h"
#include "ks_gemm_soe.h"
#include "ks_select.h"

#ifndef KS_DX_IL
#define KS_DX_IL 0
#endif
#ifndef KS_DW_IL
#define KS_DW_IL 1
#endif
#ifndef KS_IL_SPREAD
#define KS_IL_SPREAD 2
#endif
typedef KsTile<128, 128, 64, 2, 2> TileG;      // generic path (any D % 32 == 0)
typedef KsATile<256, 256, 2, 4, 2> TileSm;     // fast path (D % 64 == 0): tile = 256 classes x 256 samples
typedef KsATile<128, 128, 2, 2, 2> TileDx;
#define DX_IDX_CACHE 4096 /* gather indices of one workgroup's share of the active dimension, staged in LDS */
// dW tiles: 256 columns of D, and 256, 192 or 128 active rows -- chosen inside the kernel from the number of active
// rows, which only the device knows (see dw_tile_rows)
typedef KsATile<256, 256, 2, 4, 2> TileDw;
typedef KsATile<192, 256, 2, 4, 2> TileDw192;
typedef KsATile<128, 256, 2, 4, 2> TileDw128;
#define KS_BP_ALIGN 256
#define SM_LIDX_CAP 1536 // gather-list entries a sweep keeps in LDS (longer slabs read the list from memory)
#define SM_SOE_GRID 256 /* workgroups of the stationary-operand softmax passes (one per compute unit) */

#define SM_NT 256
#define KS_MP_ALIGN 256

static inline int64_t sm_mp(int64_t M) { return (int64_t)ks_align_up((size_t)M, KS_MP_ALIGN); }

__device__ __forceinline__ int sm_clamp_n(const int32_t *n_active, int M) {
    int n = *n_active;
    return n < 0 ? 0 : (n > M ? M : n);
}

// ------------------------------------------------------------------------------------------------
// Z = scale * X . W[active]^T      (M index = sample i, N index = active position a, K index = d)
// ------------------------------------------------------------------------------------------------
template <class T>
__global__ void __launch_bounds__(T::NT)
logits_kernel(const uint16_t *__restrict__ X, const uint16_t *__restrict__ W, const int32_t *__restrict__ active_idx,
              const int32_t *__restrict__ n_active_p, int B, int D, int M, float scale, float *__restrict__ Z,
              int64_t ldz) {
    __shared__ __attribute__((aligned(16))) uint16_t lds[T::LDS_ELEMS];
    const int n_active = sm_clamp_n(n_active_p, M);
    const int tiles_m = (B + T::BM - 1) / T::BM;
    const int n_tiles = tiles_m * ((n_active + T::BN - 1) / T::BN);
    if ((int)blockIdx.x >= n_tiles) return;
    const int t = ks_xcd_remap(blockIdx.x, n_tiles);
    const int tm = t % tiles_m, tn = t / tiles_m;

    KsRowLoader<T::BM, T::BK, T::NT> al;
    KsRowLoader<T::BN, T::BK, T::NT> bl;
    al.init(X, D, nullptr, tm * T::BM, B, D);
    bl.init(W, D, active_idx, tn * T::BN, n_active, D);
    f32x16_t acc[T::FM][T::FN];
    ks_tile_clear<T>(acc);
    ks_gemm_mainloop<T>(al, bl, 0, (D + T::BK - 1) / T::BK, lds, acc);
    ks_tile_foreach<T>(acc, [&](int m, int n, float v) {
        int i = tm * T::BM + m, a = tn * T::BN + n;
        if (i < B && a < n_active) Z[(int64_t)i * ldz + a] = scale * v;
    });
}

// ------------------------------------------------------------------------------------------------
// per-sample log-sum-exp and loss; one workgroup per sample
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(SM_NT)
row_stats_kernel(const float *__restrict__ Z, int64_t ldz, const int32_t *__restrict__ n_active_p, int M,
                 const int32_t *__restrict__ target_pos, float *__restrict__ lse_out, float *__restrict__ loss_i) {
    __shared__ float sm[SM_NT / 64], sl[SM_NT / 64];
    const int i = blockIdx.x;
    const int n = sm_clamp_n(n_active_p, M);
    const float *z = Z + (int64_t)i * ldz;
    float m = -INFINITY, l = 0.f;
    const int n4 = n & ~3;
    for (int a = threadIdx.x * 4; a < n4; a += SM_NT * 4) {
        float4 v = *(const float4 *)(z + a);
        float mx = fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w));
        if (mx > m) { l *= __expf(m - mx); m = mx; }
        l += __expf(v.x - m) + __expf(v.y - m) + __expf(v.z - m) + __expf(v.w - m);
    }
    if (threadIdx.x < n - n4) {
        float v = z[n4 + threadIdx.x];
        if (v > m) { l *= __expf(m - v); m = v; }
        l += __expf(v - m);
    }
    // combine (m, l) pairs: wave, then block, in a fixed order
    float wm = ks_wave_max(m);
    float wl = ks_wave_sum(m == -INFINITY ? 0.f : l * __expf(m - wm));
    if ((threadIdx.x & 63) == 0) { sm[threadIdx.x >> 6] = wm; sl[threadIdx.x >> 6] = wl; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float bm = sm[0];
        for (int w = 1; w < SM_NT / 64; ++w) bm = fmaxf(bm, sm[w]);
        float bl = 0.f;
        for (int w = 0; w < SM_NT / 64; ++w) bl += (sm[w] == -INFINITY) ? 0.f : sl[w] * __expf(sm[w] - bm);
        float lse = bm + __logf(bl);
        int tp = target_pos[i];
        float zt = (tp >= 0 && tp < n) ? z[tp] : 0.f;
        lse_out[i] = lse;
        loss_i[i] = lse - zt;
    }
}

// (The mean of the per-sample losses is formed later in the stream, by one block of dx_reduce_kernel: folding
// it into the kernel above would need a device-scope fence per workgroup, which costs far more on this chip,
// whose eight L2 caches are only coherent through memory, and a launch of its own costs about 5 us.)

// ------------------------------------------------------------------------------------------------
// dZ = g (exp(Z - lse) - onehot) as bf16; columns in [n_active, round_up(n_active, 256)) are zeroed
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(SM_NT)
dz_kernel(const float *__restrict__ Z, int64_t ldz, const int32_t *__restrict__ n_active_p, int M,
          const int32_t *__restrict__ target_pos, const float *__restrict__ lse, float g, uint16_t *__restrict__ dZ) {
    const int n = sm_clamp_n(n_active_p, M);
    const int n_pad = (n + KS_MP_ALIGN - 1) / KS_MP_ALIGN * KS_MP_ALIGN; // <= ldz
    const int a0 = (blockIdx.x * SM_NT + threadIdx.x) * 8;
    if (a0 >= n_pad) return;
    const int i = blockIdx.y;
    const float ls = lse[i];
    const int tp = target_pos[i];
    const float *z = Z + (int64_t)i * ldz + a0;
    float v[8];
    if (a0 + 8 <= n) {
        float4 p = *(const float4 *)z, q = *(const float4 *)(z + 4);
        v[0] = p.x; v[1] = p.y; v[2] = p.z; v[3] = p.w; v[4] = q.x; v[5] = q.y; v[6] = q.z; v[7] = q.w;
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (a0 + e < n) ? z[e] : 0.f;
    }
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
        float d0 = (a0 + e < n) ? g * (__expf(v[e] - ls) - (a0 + e == tp ? 1.f : 0.f)) : 0.f;
        float d1 = (a0 + e + 1 < n) ? g * (__expf(v[e + 1] - ls) - (a0 + e + 1 == tp ? 1.f : 0.f)) : 0.f;
        o[e / 2] = ks_pack_bf2(d0, d1);
    }
    *(uint4 *)(dZ + (int64_t)i * ldz + a0) = make_uint4(o[0], o[1], o[2], o[3]);
}

// ------------------------------------------------------------------------------------------------
// dX partials: P[s][i][d] = sum over the s-th share of a of dZ[i][a] * W[active[a]][d]
// ------------------------------------------------------------------------------------------------
template <class T>
__global__ void __launch_bounds__(T::NT)
dx_partial_kernel(const uint16_t *__restrict__ dZ, int64_t ldz, const uint16_t *__restrict__ W,
                  const int32_t *__restrict__ active_idx, const int32_t *__restrict__ n_active_p, int B, int D, int M,
                  float *__restrict__ part) {
    __shared__ __attribute__((aligned(16))) uint16_t lds[T::LDS_ELEMS];
    const int n_active = sm_clamp_n(n_active_p, M);
    const int tiles_m = (B + T::BM - 1) / T::BM;
    const int tm = blockIdx.x % tiles_m, tn = blockIdx.x / tiles_m;
    const int s = blockIdx.y, S = gridDim.y;
    const int nk = (n_active + T::BK - 1) / T::BK;
    const int per = (nk + S - 1) / S;
    const int kt0 = s * per, kt1 = (kt0 + per < nk) ? kt0 + per : nk;

    KsRowLoader<T::BM, T::BK, T::NT> al;
    KsColLoader<T::BN, T::BK, T::NT> bl;
    al.init(dZ, ldz, nullptr, tm * T::BM, B, (n_active + 7) & ~7);
    bl.init(W, D, active_idx, tn * T::BN, D, n_active);
    f32x16_t acc[T::FM][T::FN];
    ks_tile_clear<T>(acc);
    ks_gemm_mainloop<T>(al, bl, kt0, kt1, lds, acc);
    float *out = part + (int64_t)s * B * D;
    ks_tile_foreach<T>(acc, [&](int m, int n, float v) {
        int i = tm * T::BM + m, d = tn * T::BN + n;
        if (i < B && d < D) out[(int64_t)i * D + d] = v;
    });
}

__global__ void __launch_bounds__(SM_NT)
dx_reduce_kernel(const float *__restrict__ part, int S, int64_t BD, float scale, const float *__restrict__ row_factor,
                 int D, float *__restrict__ dX, const float *__restrict__ loss_i, int B, float *loss_mean) {
    // the last block also folds the per-sample losses (complete since an earlier launch) into the batch
    // mean: thread t takes samples t, t + SM_NT, ..., then a tree -- a fixed order, and no launch of its own
    if (loss_mean && blockIdx.x == gridDim.x - 1) {
        __shared__ float sh[SM_NT];
        float s = 0.f;
        for (int i = threadIdx.x; i < B; i += SM_NT) s += loss_i[i];
        sh[threadIdx.x] = s;
        __syncthreads();
        for (int o = SM_NT / 2; o > 0; o >>= 1) {
            if (threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
            __syncthreads();
        }
        if (threadIdx.x == 0) *loss_mean = sh[0] / (float)B;
    }
    int64_t e = ((int64_t)blockIdx.x * SM_NT + threadIdx.x) * 4;
    if (e >= BD) return; // BD % 4 == 0, D % 4 == 0
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s = 0; s < S; ++s) {
        float4 v = *(const float4 *)(part + (int64_t)s * BD + e);
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    if (row_factor) scale *= row_factor[e / D]; // per-sample factor (the one-sweep softmax leaves 1 / sum there)
    *(float4 *)(dX + e) = make_float4(scale * acc.x, scale * acc.y, scale * acc.z, scale * acc.w);
}

// ------------------------------------------------------------------------------------------------
// dW_active[a][d] = scale * sum_i dZ[i][a] * X[i][d]     (both operands k-major: k = i)
// ------------------------------------------------------------------------------------------------
template <class T>
__global__ void __launch_bounds__(T::NT)
dw_kernel(const uint16_t *__restrict__ dZ, int64_t ldz, const uint16_t *__restrict__ X,
          const int32_t *__restrict__ n_active_p, int B, int D, int M, float scale, float *__restrict__ dW) {
    __shared__ __attribute__((aligned(16))) uint16_t lds[T::LDS_ELEMS];
    const int n_active = sm_clamp_n(n_active_p, M);
    const int tiles_n = (D + T::BN - 1) / T::BN;
    const int n_tiles = tiles_n * ((n_active + T::BM - 1) / T::BM);
    if ((int)blockIdx.x >= n_tiles) return;
    const int t = ks_xcd_remap(blockIdx.x, n_tiles);
    const int tn = t % tiles_n, tm = t / tiles_n;

    KsColLoader<T::BM, T::BK, T::NT> al;
    KsColLoader<T::BN, T::BK, T::NT> bl;
    al.init(dZ, ldz, nullptr, tm * T::BM, (int)ldz, B);
    bl.init(X, D, nullptr, tn * T::BN, D, B);
    f32x16_t acc[T::FM][T::FN];
    ks_tile_clear<T>(acc);
    ks_gemm_mainloop<T>(al, bl, 0, (B + T::BK - 1) / T::BK, lds, acc);
    ks_tile_foreach<T>(acc, [&](int m, int n, float v) {
        int a = tm * T::BM + m, d = tn * T::BN + n;
        if (a < n_active && d < D) dW[(int64_t)a * D + d] = scale * v;
    });
}

// ================================================================================================
// Fast path (D % 64 == 0).  All contractions run on the asynchronous engine and the logits are recomputed
// instead of stored (see below).  The logit gradient is stored once, transposed (dZT[a][i]); it is the
// k-contiguous operand of the dW contraction and a k-major operand of the dX contraction.  Weight rows (gathered through the index list) and X enter as
// k-major operands where k is their row index, so no transposed copies of them are made.
// ================================================================================================

// 8x8 transpose of 16-bit elements held as 8 rows of uint4 (row k, elements n=0..7) -> out[n] = 8 k's
__device__ __forceinline__ void sm_transpose8x8(const uint4 (&in)[8], uint4 (&out)[8]) {
#pragma unroll
    for (int n = 0; n < 8; ++n) {
        uint32_t o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint4 &ra = in[2 * j], &rb = in[2 * j + 1];
            uint32_t a = (n >> 1) == 0 ? ra.x : ((n >> 1) == 1 ? ra.y : ((n >> 1) == 2 ? ra.z : ra.w));
            uint32_t b = (n >> 1) == 0 ? rb.x : ((n >> 1) == 1 ? rb.y : ((n >> 1) == 2 ? rb.z : rb.w));
            o[j] = (n & 1) ? ((a >> 16) | (b & 0xFFFF0000u)) : ((a & 0xFFFFu) | (b << 16));
        }
        out[n] = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

#define TR_TILE 128
#define TR_LD (TR_TILE + 8)

// The logits are never stored on the fast path.  Two passes over the same tile product
//     Zt[a][i] = scale * <W[active[a]], X[i]>            (classes = MFMA rows, samples = MFMA columns)
// First pass: per-sample running max / sum of exponentials of each class tile, and the target logit.
// Second pass (after the per-sample log-sum-exp is known): the same product again, turned into the logit
// gradient in registers and stored transposed, dZT[a][i].  In this orientation a lane owns one sample
// column of the accumulator tile, so the per-sample reductions are lane-local.

// accumulator element (fm, r) of a lane: class row inside the wave's part of the tile
__device__ __forceinline__ int sm_tile_row(int fm, int r, int lane) { return fm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

template <class T>
__device__ __forceinline__ void sm_logits_tile(const uint16_t *X, const uint16_t *W, const int32_t *active_idx, int n_active,
                                               int B, int D, int tc, int ts, uint16_t *lds, f32x16_t (&acc)[T::FM][T::FN]) {
    KsARows<T::BM, T::NW> ar;
    KsARows<T::BN, T::NW> br;
    ar.init(W, D, active_idx, tc * T::BM, n_active);
    br.init(X, D, nullptr, ts * T::BN, B);
    ks_a_clear<T>(acc);
    ks_a_mainloop<T>(ar, br, 0, D / 64, lds, acc);
}

template <class T>
__global__ void __launch_bounds__(T::NT)
sm_stats_kernel(const uint16_t *__restrict__ X, const uint16_t *__restrict__ W, const int32_t *__restrict__ active_idx,
                const int32_t *__restrict__ n_active_p, const int32_t *__restrict__ target_pos, int B, int Bp, int D, int M,
                float scale, float *__restrict__ pm, float *__restrict__ pl, float *__restrict__ zt) {
    __shared__ __attribute__((aligned(16))) uint16_t lds[T::LDS_ELEMS];
    const int n_active = sm_clamp_n(n_active_p, M);
    const int tiles_s = (B + T::BN - 1) / T::BN;
    const int n_tiles = tiles_s * ((n_active + T::BM - 1) / T::BM);
    if ((int)blockIdx.x >= n_tiles) return;
    const int t = ks_xcd_remap(blockIdx.x, n_tiles);
    const int ts = t % tiles_s, tc = t / tiles_s;
    f32x16_t acc[T::FM][T::FN];
    sm_logits_tile<T>(X, W, active_idx, n_active, B, D, tc, ts, lds, acc); // ends with a barrier: LDS is free

    // per (wave row, sample) partial statistics go through LDS: [WAVES_M][BN] pairs
    float *s_m = (float *)lds, *s_l = s_m + T::WAVES_M * T::BN;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / T::WAVES_N, wn = wave % T::WAVES_N;
    const int c0 = tc * T::BM + wm * T::WM;
#pragma unroll
    for (int fn = 0; fn < T::FN; ++fn) {
        const int col = wn * T::WN + fn * 32 + (lane & 31);
        const int i = ts * T::BN + col;
        const int tp = (i < B) ? target_pos[i] : -1;
        float m = -INFINITY;
#pragma unroll
        for (int fm = 0; fm < T::FM; ++fm)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int c = c0 + sm_tile_row(fm, r, lane);
                const float z = scale * acc[fm][fn][r];
                if (c < n_active) m = fmaxf(m, z);
                if (c == tp) zt[i] = z;
            }
        float l = 0.f;
#pragma unroll
        for (int fm = 0; fm < T::FM; ++fm)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int c = c0 + sm_tile_row(fm, r, lane);
                if (c < n_active) l += __expf(scale * acc[fm][fn][r] - m);
            }
        // the two half-waves hold disjoint class rows of the same 32 samples
        const float mo = __shfl_xor(m, 32, 64), lo = __shfl_xor(l, 32, 64);
        const float mm = fmaxf(m, mo);
        const float ll = (m == -INFINITY ? 0.f : l * __expf(m - mm)) + (mo == -INFINITY ? 0.f : lo * __expf(mo - mm));
        if (lane < 32) {
            s_m[wm * T::BN + col] = mm;
            s_l[wm * T::BN + col] = ll;
        }
    }
    __syncthreads();
    for (int col = threadIdx.x; col < T::BN; col += T::NT) {
        const int i = ts * T::BN + col;
        if (i >= B) continue;
        float mm = s_m[col], ll = s_l[col];
#pragma unroll
        for (int w = 1; w < T::WAVES_M; ++w) { // fixed order
            const float m2 = s_m[w * T::BN + col], l2 = s_l[w * T::BN + col];
            const float mx = fmaxf(mm, m2);
            ll = (mm == -INFINITY ? 0.f : ll * __expf(mm - mx)) + (m2 == -INFINITY ? 0.f : l2 * __expf(m2 - mx));
            mm = mx;
        }
        pm[(int64_t)tc * Bp + i] = mm;
        pl[(int64_t)tc * Bp + i] = ll;
    }
}

// one wavefront per sample: merge the per-tile (max, sum) pairs in tile order -> lse_i, loss_i
__global__ void __launch_bounds__(SM_NT)
sm_combine_kernel(const float *__restrict__ pm, const float *__restrict__ pl, const float *__restrict__ zt,
                  const int32_t *__restrict__ n_active_p, int M, int tile_rows, int B, int Bp, float *__restrict__ lse_out,
                  float *__restrict__ loss_i) {
    const int i = blockIdx.x * (SM_NT / 64) + (threadIdx.x >> 6);
    if (i >= B) return;
    const int lane = threadIdx.x & 63;
    const int n = sm_clamp_n(n_active_p, M);
    const int nt = (n + tile_rows - 1) / tile_rows;
    float m = -INFINITY, l = 0.f;
    for (int t = lane; t < nt; t += 64) {
        const float tm = pm[(int64_t)t * Bp + i], tl = pl[(int64_t)t * Bp + i];
        if (tm > m) { l *= __expf(m - tm); m = tm; }
        if (tm != -INFINITY) l += tl * __expf(tm - m);
    }
    const float wm = ks_wave_max(m);
    const float wl = ks_wave_sum(m == -INFINITY ? 0.f : l * __expf(m - wm));
    if (lane == 0) {
        const float lse = wm + __logf(wl);
        lse_out[i] = lse;
        loss_i[i] = lse - zt[i];
    }
}

// second pass: logit gradient, stored transposed.  dZT[a][i] = g (exp(Zt[a][i] - lse_i) - [a == target_pos[i]]),
// zero for a >= n_active (up to the end of the class tile) and for i >= B (up to Bp).
template <class T>
__global__ void __launch_bounds__(T::NT)
sm_grad_kernel(const uint16_t *__restrict__ X, const uint16_t *__restrict__ W, const int32_t *__restrict__ active_idx,
               const int32_t *__restrict__ n_active_p, const int32_t *__restrict__ target_pos, const float *__restrict__ lse,
               int B, int Bp, int D, int M, float scale, float g, uint16_t *__restrict__ dZT) {
    constexpr int STAGE_LD = T::BN + 8;
    constexpr int STAGE_ELEMS = T::BM * STAGE_LD;
    constexpr int LDS_N = STAGE_ELEMS > T::LDS_ELEMS ? STAGE_ELEMS : T::LDS_ELEMS;
    __shared__ __attribute__((aligned(16))) uint16_t lds[LDS_N];
    const int n_active = sm_clamp_n(n_active_p, M);
    const int tiles_s = (B + T::BN - 1) / T::BN;
    const int n_tiles = tiles_s * ((n_active + T::BM - 1) / T::BM);
    if ((int)blockIdx.x >= n_tiles) return;
    const int t = ks_xcd_remap(blockIdx.x, n_tiles);
    const int ts = t % tiles_s, tc = t / tiles_s;
    f32x16_t acc[T::FM][T::FN];
    sm_logits_tile<T>(X, W, active_idx, n_active, B, D, tc, ts, lds, acc); // ends with a barrier: LDS is free

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / T::WAVES_N, wn = wave % T::WAVES_N;
    const int r0 = wm * T::WM;         // first class row of this wave inside the tile
    const int c0 = tc * T::BM + r0;
    const bool odd = lane & 1;
#pragma unroll
    for (int fn = 0; fn < T::FN; ++fn) {
        const int col = wn * T::WN + fn * 32 + (lane & 31); // sample column inside the tile
        const int i = ts * T::BN + col;
        const bool i_ok = i < B;
        const float ls = i_ok ? lse[i] : 0.f;
        const int tp = i_ok ? target_pos[i] : -1;
#pragma unroll
        for (int fm = 0; fm < T::FM; ++fm)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                float d[2];
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int c = c0 + sm_tile_row(fm, r + e, lane);
                    d[e] = (i_ok && c < n_active) ? g * (__expf(scale * acc[fm][fn][r + e] - ls) - (c == tp ? 1.f : 0.f)) : 0.f;
                }
                // neighbouring lanes (samples 2j, 2j+1) trade so that each holds two adjacent samples of one class
                // row: the even lane ends up with row r, the odd lane with row r+1
                const float send = odd ? d[0] : d[1];
                const float recv =
                    __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(send), 0xB1, 0xF, 0xF, true));
                const uint32_t packed = odd ? ks_pack_bf2(recv, d[1]) : ks_pack_bf2(d[0], recv);
                const int row = r0 + sm_tile_row(fm, r + (odd ? 1 : 0), lane);
                *(uint32_t *)(lds + row * STAGE_LD + (col & ~1)) = packed;
            }
    }
    __syncthreads();
    // coalesced store of the staged tile: 16 bytes per lane along the sample index
    constexpr int CHUNKS = T::BM * (T::BN / 8);
    for (int q = threadIdx.x; q < CHUNKS; q += T::NT) {
        const int row = q / (T::BN / 8), ch = q % (T::BN / 8);
        *(uint4 *)(dZT + (int64_t)(tc * T::BM + row) * Bp + ts * T::BN + ch * 8) = *(const uint4 *)(lds + row * STAGE_LD + ch * 8);
    }
}

// ================================================================================================
// Stationary-operand versions of the two softmax passes (D = 128, 256 or 512): a workgroup keeps the MFMA
// fragments of 256 samples in registers and streams its share ("slab") of the active classes past them.
// The active classes are cut into G / tiles_s equal slabs (multiples of 32 rows), so the chip is loaded
// evenly whatever the active count; per-sample softmax statistics are carried in registers along the slab.
// ================================================================================================
#define SOE_STAGES 3
#define KS_FUSED_MAX_SCALE 40.f // exp(-2 * scale) must stay a normal fp32 / bf16 number

// rows per slab for n64 = round_up(n_active, 64) rows and `slabs` slabs
__host__ __device__ __forceinline__ int sm_slab_rows(int n64, int slabs) {
    int h = (n64 + slabs - 1) / slabs;
    h = (h + 31) & ~31;
    return h < 32 ? 32 : h;
}

template <int KT>
__global__ void __launch_bounds__(512)
sm_stats_soe_kernel(const uint16_t *__restrict__ X, const uint16_t *__restrict__ W, const int32_t *__restrict__ active_idx,
                    const int32_t *__restrict__ n_active_p, const int32_t *__restrict__ target_pos, int B, int Bp, int D, int M,
                    int tiles_s, float scale, float *__restrict__ pm, float *__restrict__ pl, float *__restrict__ zt) {
    typedef KsSoe<KT, 96, SOE_STAGES, 2> CFG;
    __shared__ __attribute__((aligned(16))) uint16_t lds[CFG::LDS_ELEMS];
    __shared__ int32_t s_lidx[SM_LIDX_CAP];
    const int n = sm_clamp_n(n_active_p, M);
    const int n64 = (n + 63) & ~63;
    const int slabs = gridDim.x / tiles_s;
    const int h = sm_slab_rows(n64, slabs);
    const int id = ks_xcd_remap(blockIdx.x, gridDim.x);
    const int ts = id % tiles_s, slab = id / tiles_s;
    const int s0 = slab * h, s1 = (s0 + h < n64) ? s0 + h : n64;
    if (slab >= slabs || s0 >= s1) return;
    const int lane = threadIdx.x & 63;
    const int lim = n < s1 ? n : s1; // rows of this slab that are real classes
    const int i = ts * CFG::RES + ks_soe_col();
    const int tp = (i < B) ? target_pos[i] : -1;
    float m = -INFINITY, l = 0.f;
    // scale > 0 (checked by the host): statistics are carried on the raw products, m = max of acc,
    // l = sum exp(scale * (acc - m)) = sum exp2(fma(acc, k1, -k1 * m)); one fused multiply-add per element
    const float k1 = scale * 1.4426950408889634f;
    auto epi = [&](int c0, int rows_here, f32x16_t (&acc)[CFG::FM]) {
        (void)rows_here;
        // the target logit of a sample whose label sits in this chunk (rare: a scan over this lane's rows)
        if (tp >= c0 && tp < c0 + CFG::CH && tp < lim) {
#pragma unroll
            for (int fm = 0; fm < CFG::FM; ++fm)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (c0 + ks_soe_row(fm, r, lane) == tp) zt[i] = scale * acc[fm][r];
        }
        if (c0 + CFG::CH <= lim) { // every row of the chunk is a real class: no masks
            float cmax = acc[0][0];
#pragma unroll
            for (int fm = 0; fm < CFG::FM; ++fm)
#pragma unroll
                for (int r = 0; r < 16; ++r) cmax = fmaxf(cmax, acc[fm][r]);
            const float mn = fmaxf(m, cmax);
            const float off = -k1 * mn;
            float q0 = 0.f, q1 = 0.f, q2 = 0.f, q3 = 0.f; // four chains: the exponentials do not wait on one sum
#pragma unroll
            for (int fm = 0; fm < CFG::FM; ++fm)
#pragma unroll
                for (int r = 0; r < 16; r += 4) {
                    q0 += __builtin_amdgcn_exp2f(fmaf(acc[fm][r], k1, off));
                    q1 += __builtin_amdgcn_exp2f(fmaf(acc[fm][r + 1], k1, off));
                    q2 += __builtin_amdgcn_exp2f(fmaf(acc[fm][r + 2], k1, off));
                    q3 += __builtin_amdgcn_exp2f(fmaf(acc[fm][r + 3], k1, off));
                }
            l = l * __builtin_amdgcn_exp2f(k1 * (m - mn)) + ((q0 + q1) + (q2 + q3)); // m = -inf, l = 0 at the start
            m = mn;
        } else {
            float cmax = -INFINITY;
#pragma unroll
            for (int fm = 0; fm < CFG::FM; ++fm)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (c0 + ks_soe_row(fm, r, lane) < lim) cmax = fmaxf(cmax, acc[fm][r]);
            if (cmax == -INFINITY) return; // no real class among this lane's rows of the chunk
            const float mn = fmaxf(m, cmax);
            const float off = -k1 * mn;
            float sum = 0.f;
#pragma unroll
            for (int fm = 0; fm < CFG::FM; ++fm)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (c0 + ks_soe_row(fm, r, lane) < lim) sum += __builtin_amdgcn_exp2f(fmaf(acc[fm][r], k1, off));
            l = l * __builtin_amdgcn_exp2f(k1 * (m - mn)) + sum;
            m = mn;
        }
    };
    ks_soe_sweep<CFG>(X, D, ts * CFG::RES, B, W, D, active_idx, s0, s1, n, lds, epi, s_lidx, SM_LIDX_CAP);
    {
        // the two half-waves hold disjoint class rows of the same 32 samples
        const float mz = scale * m; // back to logit units
        const float mo = __shfl_xor(mz, 32, 64), lo = __shfl_xor(l, 32, 64);
        const float mm = fmaxf(mz, mo);
        const float ll = (mz == -INFINITY ? 0.f : l * __expf(mz - mm)) + (mo == -INFINITY ? 0.f : lo * __expf(mo - mm));
        if (lane < 32 && i < B) {
            pm[(int64_t)slab * Bp + i] = mm;
            pl[(int64_t)slab * Bp + i] = ll;
        }
    }
}

template <int KT>
__global__ void __launch_bounds__(512)
sm_grad_soe_kernel(const uint16_t *__restrict__ X, const uint16_t *__restrict__ W, const int32_t *__restrict__ active_idx,
                   const int32_t *__restrict__ n_active_p, const int32_t *__restrict__ target_pos,
                   const float *__restrict__ lse, int B, int Bp, int D, int M, int tiles_s, float scale, float g,
                   uint16_t *__restrict__ dZT) {
    typedef KsSoe<KT, 96, SOE_STAGES, 2> CFG;
    constexpr int STAGE_LD = CFG::RES + 8;
    __shared__ __attribute__((aligned(16))) uint16_t lds[CFG::LDS_ELEMS];
    __shared__ int32_t s_lidx[SM_LIDX_CAP];
    __shared__ __attribute__((aligned(16))) uint16_t stage[CFG::CH * STAGE_LD];
    const int n = sm_clamp_n(n_active_p, M);
    const int n64 = (n + 63) & ~63;
    const int slabs = gridDim.x / tiles_s;
    const int h = sm_slab_rows(n64, slabs);
    const int id = ks_xcd_remap(blockIdx.x, gridDim.x);
    const int ts = id % tiles_s, slab = id / tiles_s;
    const int s0 = slab * h, s1 = (s0 + h < n64) ? s0 + h : n64;
    if (slab >= slabs || s0 >= s1) return;
    const int i0 = ts * CFG::RES + ks_soe_col();
    const float ls = i0 < B ? lse[i0] : 0.f;
    const int tp = i0 < B ? target_pos[i0] : -1;
    // scale > 0 and g > 0 (checked by the host): g * exp(scale * acc - lse) = exp2(fma(acc, k1, k2)) with
    // k2 = log2(g) - lse * log2(e): one fused multiply-add and one exponential per element
    const float k1 = scale * 1.4426950408889634f;
    const float k2 = __log2f(g) - ls * 1.4426950408889634f;
    const bool samples_ok = (ts + 1) * CFG::RES <= B;
    auto epi = [&](int c0, int rows_here, f32x16_t (&acc)[CFG::FM]) {
        const bool plain = samples_ok && c0 + CFG::CH <= n; // no row or column of this chunk needs masking
        // Everything derived from the thread index is derived afresh here, from a copy the compiler cannot see
        // through: otherwise it hoists the dozens of LDS addresses below out of the sweep, runs out of
        // registers and spills them -- and every reload of a spilled value is a vector-memory load whose wait
        // also waits for the stream loads in flight.
        int tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
        const int lane = tid & 63;
        const bool odd = lane & 1;
        const int col = (tid >> 6) * 32 + (tid & 31);
        const bool ok = ts * CFG::RES + col < B;
        // does any sample of this wavefront have its label inside the chunk?
        const bool mine = tp >= c0 && tp < c0 + CFG::CH;
        const bool any_target = __builtin_amdgcn_ballot_w64(mine) != 0;
#pragma unroll
        for (int fm = 0; fm < CFG::FM; ++fm)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                float d[2];
#pragma unroll
                for (int e = 0; e < 2; ++e) d[e] = __builtin_amdgcn_exp2f(fmaf(acc[fm][r + e], k1, k2));
                if (any_target) {
#pragma unroll
                    for (int e = 0; e < 2; ++e)
                        if (c0 + ks_soe_row(fm, r + e, lane) == tp) d[e] -= g;
                }
                if (!plain) {
#pragma unroll
                    for (int e = 0; e < 2; ++e)
                        if (!ok || c0 + ks_soe_row(fm, r + e, lane) >= n) d[e] = 0.f;
                }
                // neighbouring lanes (samples 2j, 2j+1) trade so that each holds two adjacent samples of one
                // class row: the even lane ends up with row r, the odd lane with row r+1
                const float send = odd ? d[0] : d[1];
                const float recv = __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(send), 0xB1, 0xF, 0xF, true));
                const uint32_t packed = odd ? ks_pack_bf2(recv, d[1]) : ks_pack_bf2(d[0], recv);
                const int row = ks_soe_row(fm, r + (odd ? 1 : 0), lane);
                *(uint32_t *)(stage + row * STAGE_LD + (col & ~1)) = packed;
            }
        __builtin_amdgcn_s_waitcnt(0xC07F); // LDS writes done (lgkmcnt 0); loads in flight are left alone
        ks_barrier_nofence();
        const int chunks = rows_here * (CFG::RES / 8);
        for (int q = tid; q < chunks; q += CFG::NT) {
            const int row = q / (CFG::RES / 8), ch = q % (CFG::RES / 8);
            *(uint4 *)(dZT + (int64_t)(c0 + row) * Bp + ts * CFG::RES + ch * 8) = *(const uint4 *)(stage + row * STAGE_LD + ch * 8);
        }
    };
    ks_soe_sweep<CFG>(X, D, ts * CFG::RES, B, W, D, active_idx, s0, s1, n, lds, epi, s_lidx, SM_LIDX_CAP);
}


// ------------------------------------------------------------------------------------------------
// One-sweep variant for rows of norm <= 1 (the paper normalises W and X, section 3.2): every logit
// lies in [-scale, scale], so the softmax can be evaluated against the fixed reference `scale` and no
// statistics pass is needed.  The sweep writes E[a][i] = exp(z_ia - scale) (bf16, transposed, zero in the
// padding) and per-slab sums of the stored (rounded) E; sm_combine_fused_kernel then forms sum_i = sum_a E_ia,
// the loss, and turns column i into (P_ia - [a = target_i]) * sum_i by replacing the target entry.  The
// factor g / sum_i that is still missing is applied where it is cheap: on the rows of dX after the
// contraction over classes, and on the rows of X (X2 = X / sum_i, bf16) before the contraction over samples.
// The reference only shifts the exponent range: results are the same function of the inputs as long as no
// exponential overflows and not all of a sample's vanish, which the combine kernel checks.
// ------------------------------------------------------------------------------------------------
// The sweep runs on the eight-wavefront engine (ks_gemm_soe.h): wavefront w owns samples [32 w, 32 w + 32) of the
// tile and two wavefronts share a SIMD, so the exponentials, the LDS writes and the copy-out of one overlap with
// the MFMAs of the other (measured on the headline shape: 34 us against 40 us with four wavefronts of 64 samples).
template <int KT>
__global__ void __launch_bounds__(512)
sm_fused_soe_kernel(const uint16_t *__restrict__ X, const uint16_t *__restrict__ W, const int32_t *__restrict__ active_idx,
                     const int32_t *__restrict__ n_active_p, const int32_t *__restrict__ target_pos, int B, int Bp, int D, int M,
                     int tiles_s, float scale, float *__restrict__ pl, float *__restrict__ pl_others, uint16_t *__restrict__ dZT) {
    typedef KsSoe<KT, 96, SOE_STAGES, 2> CFG;
    constexpr int STAGE_LD = CFG::RES + 8;
    constexpr int NT = CFG::NT;
    __shared__ __attribute__((aligned(16))) uint16_t lds[CFG::LDS_ELEMS];
    __shared__ int32_t s_lidx[SM_LIDX_CAP];
    __shared__ __attribute__((aligned(16))) uint16_t stage[CFG::CH * STAGE_LD];
    const int n = sm_clamp_n(n_active_p, M);
    const int n64 = (n + 63) & ~63;
    const int slabs = gridDim.x / tiles_s;
    const int h = sm_slab_rows(n64, slabs);
    const int id = ks_xcd_remap(blockIdx.x, gridDim.x);
    const int ts = id % tiles_s, slab = id / tiles_s;
    const int s0 = slab * h, s1 = (s0 + h < n64) ? s0 + h : n64;
    if (slab >= slabs || s0 >= s1) return;
    const int lim = n < s1 ? n : s1; // rows of this slab that are real classes
    __shared__ float s_sum[8 * NT];  // thread t: running sums of its eight samples over its rows, at [c * NT + t]
#pragma unroll
    for (int c = 0; c < 8; ++c) s_sum[c * NT + threadIdx.x] = 0.f;
    const float k1 = scale * 1.4426950408889634f; // exp(scale * acc - scale) = exp2(fma(acc, k1, -k1))
    const bool samples_ok = (ts + 1) * CFG::RES <= B;
    // For the loss: this lane's sum of the UNROUNDED exponentials of its sample over its rows, the sample's own class
    // left out (the combine step adds that one from an fp32 dot product).  The sums of the stored, rounded values
    // (`pl`) are what the gradient columns must add up to; for the loss of a confident sample they would carry the
    // bf16 rounding of its strongest competitor, 2^-9 relative.
    float others = 0.f;
    int my_tp = -1; // position of this lane's sample's class in the active list
    {
        const int i = ts * CFG::RES + ks_soe_col();
        if (i < B) my_tp = target_pos[i];
    }
    auto epi = [&](int c0, int rows_here, f32x16_t (&acc)[CFG::FM]) {
        const bool plain = samples_ok && c0 + CFG::CH <= lim; // no row or column of this chunk needs masking
        const int tl = my_tp - c0;                             // the own class's row in this chunk, if in [0, CH)
        const bool own_here = __any(tl >= 0 && tl < CFG::CH);  // uniform: some sample of this wavefront has its class here
        float csum = 0.f;
        // thread-index arithmetic is redone here behind a copy the compiler cannot see through, so that it does not
        // hoist the LDS addresses out of the sweep and spill them
        int tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
        const int lane = tid & 63;
        const bool odd = lane & 1;
        const int col = (tid >> 6) * 32 + (tid & 31);
        const bool ok = ts * CFG::RES + col < B;
        const int tq = tl - 4 * (lane >> 5); // the own class's accumulator element: fm * 32 + 8 * (r >> 2) + (r & 3) == tq
        // the element loop, compiled three times: plain chunks with and without the test for the own class, and chunks
        // with rows or samples to mask (no branch inside the loop)
        auto elements = [&](auto own, auto is_plain) __attribute__((always_inline)) {
            constexpr bool OWN = decltype(own)::value, PLAIN = decltype(is_plain)::value;
#pragma unroll
            for (int fm = 0; fm < CFG::FM; ++fm)
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    float d[2];
#pragma unroll
                    for (int e = 0; e < 2; ++e) d[e] = __builtin_amdgcn_exp2f(fmaf(acc[fm][r + e], k1, -k1));
                    if (!PLAIN) {
#pragma unroll
                        for (int e = 0; e < 2; ++e)
                            if (!ok || c0 + ks_soe_row(fm, r + e, lane) >= lim) d[e] = 0.f;
                    }
                    if (OWN) {
                        csum += (fm * 32 + 8 * (r >> 2) + (r & 3)) == tq ? 0.f : d[0];
                        csum += (fm * 32 + 8 * ((r + 1) >> 2) + ((r + 1) & 3)) == tq ? 0.f : d[1];
                    } else {
                        csum += d[0] + d[1];
                    }
                    // neighbouring lanes (samples 2j, 2j+1) trade so that each holds two adjacent samples of one class
                    // row: the even lane ends up with row r, the odd lane with row r+1
                    const float send = odd ? d[0] : d[1];
                    const float recv = __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(send), 0xB1, 0xF, 0xF, true));
                    const uint32_t packed = odd ? ks_pack_bf2(recv, d[1]) : ks_pack_bf2(d[0], recv);
                    const int row = ks_soe_row(fm, r + (odd ? 1 : 0), lane);
                    *(uint32_t *)(stage + row * STAGE_LD + (col & ~1)) = packed;
                }
        };
        if (plain) {
            if (own_here) elements(std::true_type(), std::true_type());
            else elements(std::false_type(), std::true_type());
        } else {
            elements(std::true_type(), std::false_type()); // (rare: the test for the own class is harmless where it is not needed)
        }
        others += csum;
        __builtin_amdgcn_s_waitcnt(0xC07F); // LDS writes done (lgkmcnt 0); loads in flight are left alone
    };
    // second half, one stage into the next chunk: copy the chunk out in 16-byte pieces; thread t always takes the
    // same eight samples (piece t % 32 of a row) of rows t / 32, t / 32 + 16, ..., and carries their sums
    auto post = [&](int c0, int rows_here) {
        int tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
        constexpr int PPR = CFG::RES / 8, RPP = NT / PPR; // pieces per row, rows per pass
        const int ch = tid % PPR;
        float l[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) l[c] = s_sum[c * NT + tid];
        for (int r0 = tid / PPR; r0 < rows_here; r0 += 3 * RPP) {
            uint4 v[3];
#pragma unroll
            for (int u = 0; u < 3; ++u) {
                const int row = r0 + u * RPP;
                v[u] = (row < rows_here) ? *(const uint4 *)(stage + row * STAGE_LD + ch * 8) : make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int u = 0; u < 3; ++u) {
                const int row = r0 + u * RPP;
                if (row < rows_here) *(uint4 *)(dZT + (int64_t)(c0 + row) * Bp + ts * CFG::RES + ch * 8) = v[u];
                const uint32_t w4[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    l[2 * c] += ks_bf2f(w4[c] & 0xFFFFu);
                    l[2 * c + 1] += ks_bf2f(w4[c] >> 16);
                }
            }
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) s_sum[c * NT + tid] = l[c];
    };
    ks_soe_sweep<CFG>(X, D, ts * CFG::RES, B, W, D, active_idx, s0, s1, n, lds, epi, s_lidx, SM_LIDX_CAP, post);
    __syncthreads();
    // the sixteen row groups of a sample meet through LDS (the stream stages are free now): red[group][sample]
    float *red = (float *)lds;
    static_assert(CFG::LDS_ELEMS * 2 >= (NT / (CFG::RES / 8)) * CFG::RES * 4, "reduction buffer");
    {
        const int grp = threadIdx.x / (CFG::RES / 8), ch = threadIdx.x % (CFG::RES / 8);
#pragma unroll
        for (int c = 0; c < 8; ++c) red[grp * CFG::RES + ch * 8 + c] = s_sum[c * NT + threadIdx.x];
    }
    __syncthreads();
    if (threadIdx.x < CFG::RES) {
        const int i = ts * CFG::RES + threadIdx.x;
        float sum = 0.f;
#pragma unroll
        for (int grp = 0; grp < NT / (CFG::RES / 8); ++grp) sum += red[grp * CFG::RES + threadIdx.x];
        if (i < B) pl[(int64_t)slab * Bp + i] = sum;
    }
    others += __shfl_xor(others, 32, 64); // the two lanes of a sample hold different rows
    if ((threadIdx.x & 63) < 32) {
        const int i = ts * CFG::RES + ks_soe_col();
        if (i < B) pl_others[(int64_t)slab * Bp + i] = others;
    }
}

// Combine step of the one-sweep variant.  A block owns 32 samples, eight threads per sample: sum of the slab
// sums (every eighth slab each, then the eight partial sums in order); the target logit as an fp32 dot
// product of the two bf16 rows (an eighth of the row each); with it the target's exponential E_t, which
// replaces the stored rounded one in the sum, so that the stored column (with the target entry set to
// E_t - sum = -(sum of the others)) sums to zero and P_t - 1 carries no cancellation; the loss; the
// reciprocal sum for dX; the scaled row of X2.
#define SM_CF_NT 256
#ifndef SM_CF_SPB
#define SM_CF_SPB 8 /* samples per workgroup of the combine kernel */
#endif
// The softmax split over the nodes of the model-parallel layer (Section 3.1 steps 3-5) runs the same kernels in two
// calls with an exchange of the per-sample statistics in between:
#define SM_WHOLE 0  /* one GPU owns all classes: statistics and gradient in one go */
#define SM_EXPORT 1 /* first call: this node's statistics go out, nothing is normalised yet */
#define SM_IMPORT 2 /* second call: the statistics combined over all nodes come in */
struct SmSplitIO {
    float *row_max, *row_sum, *tz_out;    // SM_EXPORT
    const float *gmax, *gsum, *gtz;       // SM_IMPORT
};
__global__ void __launch_bounds__(SM_CF_NT)
sm_combine_fused_kernel(const float *__restrict__ pl, const float *__restrict__ pl_others, const int32_t *__restrict__ n_active_p,
                        const int32_t *__restrict__ active_idx, const int32_t *__restrict__ target_pos,
                        const uint16_t *__restrict__ X, const uint16_t *__restrict__ W, int M, int slabs, int B, int Bp, int D,
                        float scale, float *__restrict__ inv_sum, float *__restrict__ loss_i, uint16_t *__restrict__ dZT,
                        uint16_t *__restrict__ X2, int32_t *dev_status, int mode, SmSplitIO io) {
    // SM_CF_SPB samples per workgroup, SM_CF_PARTS threads per sample (each takes a share of the slab sums and of
    // the dot product): the kernel is a chain of dependent round trips, so it is spread over many compute units
    constexpr int SPB = SM_CF_SPB, PARTS = SM_CF_NT / SPB;
    __shared__ float sh[SM_CF_NT], sh_dot[SM_CF_NT], sh_oth[SM_CF_NT];
    __shared__ float s_inv[SPB];
    const int n = sm_clamp_n(n_active_p, M);
    const int n64 = (n + 63) & ~63;
    const int h = sm_slab_rows(n64, slabs);
    const int nt = (n64 + h - 1) / h; // slabs that hold rows
    const int j = threadIdx.x % SPB, gq = threadIdx.x / SPB;
    const int i = blockIdx.x * SPB + j;
    int tp = 0;
    bool owned = n > 0; // split over nodes: does this node hold the sample's class?  (one GPU: always)
    {
        float part = 0.f, dot = 0.f, oth = 0.f;
        if (i < B && n > 0) {
            // all loads of a batch are issued before the first use: these are dependent only through the
            // running sums, and one round trip to another L2 costs as much as everything else here
            tp = target_pos[i];
            if (mode != SM_WHOLE) owned = tp >= 0 && tp < n;
            tp = tp < 0 ? 0 : (tp >= n ? n - 1 : tp); // stays in bounds whatever the selection flagged
            const int cls = active_idx[tp];
            for (int t0 = gq; mode != SM_IMPORT && t0 < nt; t0 += 4 * PARTS) {
                float v[4], u[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    v[q] = (t0 + PARTS * q < nt) ? pl[(int64_t)(t0 + PARTS * q) * Bp + i] : 0.f;
                    u[q] = (t0 + PARTS * q < nt) ? pl_others[(int64_t)(t0 + PARTS * q) * Bp + i] : 0.f;
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    part += v[q];
                    oth += u[q];
                }
            }
            // this thread's share of the dot product: D / PARTS elements, in 8-byte pieces (D is 128, 256 or 512)
            const int per = D / PARTS;
            const uint16_t *xr = X + (int64_t)i * D + gq * per;
            const uint16_t *wr = W + (int64_t)cls * D + gq * per;
            constexpr int MAXP = 512 / PARTS / 4;
            uint2 xv[MAXP], wv[MAXP];
#pragma unroll
            for (int q = 0; q < MAXP; ++q) {
                if (q * 4 < per) {
                    xv[q] = *(const uint2 *)(xr + q * 4);
                    wv[q] = *(const uint2 *)(wr + q * 4);
                }
            }
#pragma unroll
            for (int q = 0; q < MAXP; ++q) {
                if (q * 4 < per) {
                    dot = fmaf(ks_bf2f(xv[q].x & 0xFFFFu), ks_bf2f(wv[q].x & 0xFFFFu), dot);
                    dot = fmaf(ks_bf2f(xv[q].x >> 16), ks_bf2f(wv[q].x >> 16), dot);
                    dot = fmaf(ks_bf2f(xv[q].y & 0xFFFFu), ks_bf2f(wv[q].y & 0xFFFFu), dot);
                    dot = fmaf(ks_bf2f(xv[q].y >> 16), ks_bf2f(wv[q].y >> 16), dot);
                }
            }
        }
        sh[threadIdx.x] = part;
        sh_dot[threadIdx.x] = dot;
        sh_oth[threadIdx.x] = oth;
    }
    __syncthreads();
    if (threadIdx.x < SPB) {
        float inv = 0.f;
        if (i < B) {
            float sum = 0.f, dot = 0.f, oth = 0.f;
            for (int q = 0; q < PARTS; ++q) { // a fixed order
                sum += sh[q * SPB + j];
                dot += sh_dot[q * SPB + j];
                oth += sh_oth[q * SPB + j];
            }
            const float z_t = scale * dot;
            const float e_t = __expf(z_t - scale);
            uint16_t *cell = dZT + (int64_t)tp * Bp + i;
            if (mode == SM_IMPORT) {
                // the sum over the classes of all nodes, brought to this kernel's reference `scale`
                const float S = io.gsum[i] * __expf(io.gmax[i] - scale);
                if (!(S > 0.f) || !(S < INFINITY)) ks_flag(dev_status, KS_DEV_RANGE);
                loss_i[i] = (io.gmax[i] + __logf(io.gsum[i])) - io.gtz[i];
                inv = 1.f / S;
                inv_sum[i] = inv;
                if (owned) *cell = (uint16_t)ks_f2bf(e_t - S); // (P_t - 1) * S
            } else {
                float others = sum;
                if (owned) {
                    others = sum - ks_bf2f(*cell); // sum of the exponentials of the other classes
                    sum = others + e_t;
                }
                if (mode == SM_EXPORT) {
                    io.row_max[i] = scale;
                    io.row_sum[i] = sum;
                    io.tz_out[i] = owned ? z_t : 0.f;
                } else {
                    if (!(sum > 0.f) || !(sum < INFINITY)) ks_flag(dev_status, KS_DEV_RANGE);
                    // loss = log(1 + (unrounded exponentials of the other classes) / E_t): no difference of nearly
                    // equal numbers, and no bf16 rounding in it (a class list without the sample's class: plain form)
                    const float ratio = oth / e_t;
                    loss_i[i] = (owned && ratio < 1e30f) ? log1pf(ratio) : (scale + __logf(sum)) - z_t;
                    inv = 1.f / sum;
                    inv_sum[i] = inv;
                    *cell = (uint16_t)ks_f2bf(-others); // the column now holds (P - onehot) * sum
                }
            }
        }
        s_inv[j] = inv;
    }
    __syncthreads();
    if (mode == SM_EXPORT) return; // nothing is normalised before the nodes have exchanged their sums
    const int rows = (B - blockIdx.x * SPB < SPB) ? B - blockIdx.x * SPB : SPB;
    const int per_row = D / 8; // 16-byte pieces per row
    const int total = rows * per_row;
    const uint16_t *xb = X + (int64_t)blockIdx.x * SPB * D; // the block's rows are contiguous
    uint16_t *ob = X2 + (int64_t)blockIdx.x * SPB * D;
    for (int q0 = threadIdx.x; q0 < total; q0 += 4 * SM_CF_NT) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (q0 + u * SM_CF_NT < total) v[u] = *(const uint4 *)(xb + (int64_t)(q0 + u * SM_CF_NT) * 8);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int q = q0 + u * SM_CF_NT;
            if (q < total) {
                const float f = s_inv[q / per_row];
                uint4 o;
                o.x = ks_pack_bf2(ks_bf2f(v[u].x & 0xFFFFu) * f, ks_bf2f(v[u].x >> 16) * f);
                o.y = ks_pack_bf2(ks_bf2f(v[u].y & 0xFFFFu) * f, ks_bf2f(v[u].y >> 16) * f);
                o.z = ks_pack_bf2(ks_bf2f(v[u].z & 0xFFFFu) * f, ks_bf2f(v[u].z >> 16) * f);
                o.w = ks_pack_bf2(ks_bf2f(v[u].w & 0xFFFFu) * f, ks_bf2f(v[u].w >> 16) * f);
                *(uint4 *)(ob + (int64_t)q * 8) = o;
            }
        }
    }
}

// one wavefront per sample: merge the per-slab (max, sum) pairs in slab order -> lse_i, loss_i
__global__ void __launch_bounds__(SM_NT)
sm_combine_soe_kernel(const float *__restrict__ pm, const float *__restrict__ pl, const float *__restrict__ zt,
                      const int32_t *__restrict__ n_active_p, int M, int slabs, int B, int Bp, float *__restrict__ lse_out,
                      float *__restrict__ loss_i) {
    const int i = blockIdx.x * (SM_NT / 64) + (threadIdx.x >> 6);
    if (i >= B) return;
    const int lane = threadIdx.x & 63;
    const int n = sm_clamp_n(n_active_p, M);
    const int n64 = (n + 63) & ~63;
    const int h = sm_slab_rows(n64, slabs);
    const int nt = (n64 + h - 1) / h;
    float m = -INFINITY, l = 0.f;
    for (int t = lane; t < nt; t += 64) {
        const float tm = pm[(int64_t)t * Bp + i], tl = pl[(int64_t)t * Bp + i];
        if (tm > m) { l *= __expf(m - tm); m = tm; }
        if (tm != -INFINITY) l += tl * __expf(tm - m);
    }
    const float wm = ks_wave_max(m);
    const float wl = ks_wave_sum(m == -INFINITY ? 0.f : l * __expf(m - wm));
    if (lane == 0) {
        const float lse = wm + __logf(wl);
        lse_out[i] = lse;
        loss_i[i] = lse - zt[i];
    }
}

// dX partials on the asynchronous engine: P[s][i][d] = sum_{a in share s} dZT[a][i] * W[active[a]][d].
// Both operands are k-major (k = a): dZT as stored, the weight rows fetched through the index list.
template <class T>
__global__ void __launch_bounds__(T::NT)
dx_partial_async_kernel(const uint16_t *__restrict__ dZT, int Bp, int64_t Mp, const uint16_t *__restrict__ W,
                        const int32_t *__restrict__ active_idx, const int32_t *__restrict__ n_active_p, int B, int D, int M,
                        int S, float *__restrict__ part, KsSelNext next) {
    __shared__ __attribute__((aligned(16))) uint16_t lds[T::LDS_ELEMS];
    __shared__ int32_t s_idx[DX_IDX_CACHE];
    const int n_active = sm_clamp_n(n_active_p, M);
    const int tiles_m = (B + T::BM - 1) / T::BM, tiles_n = (D + T::BN - 1) / T::BN;
    const int n_tiles = tiles_m * tiles_n;
    if ((int)blockIdx.x >= n_tiles * S) { // blocks behind the tiles: the next batch's candidates are staged (if asked for)
        ks_sel_next_fetch<T::NT>(next, (int)blockIdx.x - n_tiles * S);
        return;
    }
    const int L = ks_xcd_remap(blockIdx.x, n_tiles * S);
    const int s = L / n_tiles, t = L % n_tiles;
    const int tm = t % tiles_m, tn = t / tiles_m;
    const int nk = (n_active + 63) / 64;
    const int per = (nk + S - 1) / S;
    const int kt0 = s * per, kt1 = (kt0 + per < nk) ? kt0 + per : nk;
    f32x16_t acc[T::FM][T::FN];
    ks_a_clear<T>(acc);
    if (kt0 < kt1) {
        // gather list of this share, staged in LDS (the host sizes S so that a share fits), clamped at the end:
        // rows at or beyond n_active meet zeros of dZT
        for (int e = threadIdx.x; e < (kt1 - kt0) * 64 && e < DX_IDX_CACHE; e += T::NT) {
            int k = kt0 * 64 + e;
            if (k >= n_active) k = n_active - 1;
            s_idx[e] = active_idx[k];
        }
        __syncthreads();
        KsAKmaj<T::BM, T::NW> ar;
        KsAKmaj<T::BN, T::NW> br;
        ar.init(dZT, Bp, nullptr, tm * T::BM, Bp, (int)Mp, kt0 * 64);
        br.init(W, D, s_idx, tn * T::BN, D, kt1 * 64, kt0 * 64);
#if KS_DX_IL
        ks_a_mainloop_il<T, true, true, KS_IL_SPREAD>(ar, br, kt0, kt1, lds, acc);
#else
        ks_a_mainloop<T, true, true>(ar, br, kt0, kt1, lds, acc);
#endif
    }
    // row-wise through LDS (the main loop has ended with a barrier): 16-byte pieces of whole rows, a quarter of the
    // store instructions of an element-wise hand-out
    float *out = part + (int64_t)s * B * D;
    typedef KsASlab<T> SL;
    float *st = (float *)lds;
    for (int p = 0; p < T::WAVES_M; ++p) {
        ks_a_stage_slab<T>(acc, st, p);
        __syncthreads();
        constexpr int PER = SL::ROWS * SL::QUADS / T::NT;
        static_assert(SL::ROWS * SL::QUADS % T::NT == 0, "slab shape");
#pragma unroll 4
        for (int q0 = 0; q0 < PER; ++q0) {
            const int q = q0 * T::NT + threadIdx.x;
            const int row = q / SL::QUADS, quad = q % SL::QUADS;
            const int i = tm * T::BM + p * SL::ROWS + row, d = tn * T::BN + quad * 4;
            if (i < B && d < D) *(float4 *)(out + (int64_t)i * D + d) = ks_a_slab_quad<T>(st, row, quad); // D % 4 == 0
        }
        __syncthreads();
    }
}

// dW_active[a][d] = scale * sum_i dZT[a][i] * X[i][d] on the asynchronous engine (X k-major, k = i).
// The grid is sized for M rows, so with fewer active rows part of the chip would idle; the last
// DW_REDUCE_BLOCKS blocks of the grid therefore do a job that is due anyway and does not depend on this
// kernel: the sum of the dX partial products of the kernel before (with the per-sample factor, if any) and
// the batch mean of the losses.  They land on the compute units the tiles leave free.
#define DW_REDUCE_BLOCKS 128
struct DxReduceJob {
    const float *part; // [S][B * D] partial sums
    int S;
    int64_t BD;
    float scale;
    const float *row_factor; // [B] or nullptr
    float *dX;
    const float *loss_i;
    float *loss_mean;
};
// The weight update of Section 3.1 step 6 done where the gradient is produced: the tile that has just computed a
// block of dW_active adds alpha times it to the fp32 rows of the active classes and refreshes their 16-bit copy,
// so the gradient never travels to memory and back (same arithmetic as the stand-alone update: one fused
// multiply-add per element on the stored fp32 value of the gradient).  Wm == nullptr: no update.
struct DwUpdate {
    float *Wm;
    uint16_t *Wb;
    const int32_t *idx;
    float alpha;
};
// Height of the dW tiles for n_active rows on a chip of n_cu compute units (one tile per compute unit at a time).
// With few active rows 256-row tiles leave compute units idle (17,425 rows x 512 columns are 138 tiles); lower tiles
// cost more per flop (the X panel is loaded per tile whatever its height) but fill the chip: estimated time =
// rounds x relative cost per tile (measured: 1, 0.81, 0.57), the smallest wins, ties to the taller tile.
__device__ __forceinline__ int dw_tile_rows(int n_active, int tiles_n, int n_cu) {
    const int heights[3] = {256, 192, 128}, cost[3] = {100, 81, 57};
    int best = 256, best_t = 0x7fffffff;
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        const int tiles = tiles_n * ((n_active + heights[k] - 1) / heights[k]);
        const int t = ((tiles + n_cu - 1) / n_cu) * cost[k];
        if (t < best_t) { best_t = t; best = heights[k]; }
    }
    return best;
}

template <class T>
__device__ __forceinline__ void dw_tile(int bid, uint16_t *lds, const uint16_t *__restrict__ dZT, const uint16_t *__restrict__ X, int B,
                                        int Bp, int n_active, int D, int64_t Mp, float scale, float *__restrict__ dW,
                                        const DwUpdate &up);

__global__ void __launch_bounds__(TileDw::NT)
dw_async_kernel(const uint16_t *__restrict__ dZT, const uint16_t *__restrict__ X, int B, int Bp,
                const int32_t *__restrict__ n_active_p, int D, int M, int64_t Mp, float scale, float *__restrict__ dW,
                int tiles_max, int n_cu, DxReduceJob job, DwUpdate up, KsSelNext next) {
    typedef TileDw T;
    static_assert(TileDw192::NT == T::NT && TileDw128::NT == T::NT && TileDw192::LDS_ELEMS <= T::LDS_ELEMS &&
                      TileDw128::LDS_ELEMS <= T::LDS_ELEMS, "one launch shape for all tile heights");
    constexpr int LDS_ELEMS = T::LDS_ELEMS > 2 * sel1_lds_words(T::NT) ? T::LDS_ELEMS : 2 * sel1_lds_words(T::NT);
    __shared__ __attribute__((aligned(16))) uint16_t lds[LDS_ELEMS];
    // The first next.nsel workgroups select the NEXT batch's active classes (Algorithm 1 needs only its labels): with a
    // few hundred tiles this launch leaves compute units idle, and being first they start at once.
    const int bid = (int)blockIdx.x - next.nsel;
    if (bid < 0) {
        ks_sel_next_select<T::NT>(next, (uint32_t *)lds, (int)blockIdx.x);
        return;
    }
    if (bid >= tiles_max) { // reduction blocks
        const int rb = bid - tiles_max, nrb = (int)gridDim.x - next.nsel - tiles_max;
        for (int64_t e = ((int64_t)rb * T::NT + threadIdx.x) * 4; e < job.BD; e += (int64_t)nrb * T::NT * 4) {
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int sp = 0; sp < job.S; ++sp) {
                const float4 v = *(const float4 *)(job.part + (int64_t)sp * job.BD + e);
                acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
            }
            const float f = job.row_factor ? job.scale * job.row_factor[e / D] : job.scale;
            *(float4 *)(job.dX + e) = make_float4(f * acc.x, f * acc.y, f * acc.z, f * acc.w);
        }
        if (rb == nrb - 1) { // thread t takes samples t, t + NT, ..., then a tree: a fixed order
            float *sh = (float *)lds;
            float sum = 0.f;
            for (int i = threadIdx.x; i < B; i += T::NT) sum += job.loss_i[i];
            sh[threadIdx.x] = sum;
            __syncthreads();
            for (int o = T::NT / 2; o > 0; o >>= 1) {
                if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
                __syncthreads();
            }
            if (threadIdx.x == 0) *job.loss_mean = sh[0] / (float)B;
        }
        return;
    }
    const int n_active = sm_clamp_n(n_active_p, M);
    const int rows = dw_tile_rows(n_active, (D + T::BN - 1) / T::BN, n_cu);
    if (rows == 256) dw_tile<TileDw>(bid, lds, dZT, X, B, Bp, n_active, D, Mp, scale, dW, up);
    else if (rows == 192) dw_tile<TileDw192>(bid, lds, dZT, X, B, Bp, n_active, D, Mp, scale, dW, up);
    else dw_tile<TileDw128>(bid, lds, dZT, X, B, Bp, n_active, D, Mp, scale, dW, up);
}

template <class T>
__device__ __forceinline__ void dw_tile(int bid, uint16_t *lds, const uint16_t *__restrict__ dZT, const uint16_t *__restrict__ X, int B,
                                        int Bp, int n_active, int D, int64_t Mp, float scale, float *__restrict__ dW,
                                        const DwUpdate &up) {
    const int tiles_n = (D + T::BN - 1) / T::BN;
    const int n_tiles = tiles_n * ((n_active + T::BM - 1) / T::BM);
    if (bid >= n_tiles) return;
    const int t = ks_xcd_remap(bid, n_tiles);
    const int tn = t % tiles_n, tm = t / tiles_n;
    KsARows<T::BM, T::NW> ar;
    KsAKmaj<T::BN, T::NW> br;
    ar.init(dZT, Bp, nullptr, tm * T::BM, (int)Mp);
    br.init(X, D, nullptr, tn * T::BN, D, B, 0);
    f32x16_t acc[T::FM][T::FN];
    ks_a_clear<T>(acc);
#if KS_DW_IL
    ks_a_mainloop_il<T, false, true, KS_IL_SPREAD>(ar, br, 0, Bp / 64, lds, acc);
#else
    ks_a_mainloop<T, false, true>(ar, br, 0, Bp / 64, lds, acc);
#endif
    // epilogue, row-wise through LDS: gradient rows out (if wanted) and, if asked for, the update of the master
    // rows and of their 16-bit copy.  Four rows per thread are in flight at a time.
    typedef KsASlab<T> SL;
    float *st = (float *)lds;
    const int d_base = tn * T::BN;
    for (int p = 0; p < T::WAVES_M; ++p) {
        ks_a_stage_slab<T>(acc, st, p);
        __syncthreads();
        constexpr int PER = SL::ROWS * SL::QUADS / T::NT; // pieces per thread
        static_assert(SL::ROWS * SL::QUADS % T::NT == 0 && PER % 4 == 0, "slab shape");
        for (int q0 = 0; q0 < PER; q0 += 4) {
            float4 g[4], w[4];
            int64_t at[4];
            int a_[4], d_[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int q = (q0 + u) * T::NT + threadIdx.x;
                const int row = q / SL::QUADS, quad = q % SL::QUADS;
                a_[u] = tm * T::BM + p * SL::ROWS + row;
                d_[u] = d_base + quad * 4;
                const float4 v = ks_a_slab_quad<T>(st, row, quad);
                g[u] = make_float4(scale * v.x, scale * v.y, scale * v.z, scale * v.w);
                at[u] = -1;
                if (a_[u] < n_active && d_[u] < D) at[u] = up.Wm ? (int64_t)up.idx[a_[u]] * D + d_[u] : 0; // D % 4 == 0
            }
            if (up.Wm) {
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    w[u] = at[u] >= 0 ? *(const float4 *)(up.Wm + at[u]) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (at[u] < 0) continue;
                if (dW) *(float4 *)(dW + (int64_t)a_[u] * D + d_[u]) = g[u];
                if (up.Wm) {
                    w[u].x = fmaf(up.alpha, g[u].x, w[u].x);
                    w[u].y = fmaf(up.alpha, g[u].y, w[u].y);
                    w[u].z = fmaf(up.alpha, g[u].z, w[u].z);
                    w[u].w = fmaf(up.alpha, g[u].w, w[u].w);
                    *(float4 *)(up.Wm + at[u]) = w[u];
                    if (up.Wb) *(uint2 *)(up.Wb + at[u]) = make_uint2(ks_pack_bf2(w[u].x, w[u].y), ks_pack_bf2(w[u].z, w[u].w));
                }
            }
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------------
// stand-alone row gather (Algorithm 1's W_active as a dense matrix); one wavefront per row
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(SM_NT)
gather_rows_kernel(const uint16_t *__restrict__ W, const int32_t *__restrict__ active_idx,
                   const int32_t *__restrict__ n_active_p, int M, int64_t C, int D, uint16_t *__restrict__ out,
                   int32_t *dev_status) {
    const int n = sm_clamp_n(n_active_p, M);
    const int a = blockIdx.x * (SM_NT / 64) + (threadIdx.x >> 6);
    if (a >= n) return;
    const int32_t c = active_idx[a];
    if (c < 0 || c >= C) {
        if ((threadIdx.x & 63) == 0) ks_flag(dev_status, KS_DEV_BAD_INDEX);
        return;
    }
    const uint4 *src = (const uint4 *)(W + (int64_t)c * D);
    uint4 *dst = (uint4 *)(out + (int64_t)a * D);
    for (int q = threadIdx.x & 63; q < D / 8; q += 64) dst[q] = src[q];
}

// identity active list for the full-softmax entry point
__global__ void __launch_bounds__(SM_NT)
full_prepare_kernel(const int32_t *__restrict__ labels, int64_t C, int B, int32_t *active_idx, int32_t *n_active,
                    int32_t *target_pos, int32_t *dev_status) {
    int64_t t = (int64_t)blockIdx.x * SM_NT + threadIdx.x;
    if (t == 0) *n_active = (int32_t)C;
    if (t < C) active_idx[t] = (int32_t)t;
    if (t < B) {
        int32_t y = labels[t];
        if (y < 0 || y >= C) { ks_flag(dev_status, KS_DEV_BAD_LABEL); y = 0; }
        target_pos[t] = y;
    }
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
// two-sweep softmax, split over nodes: what goes out after the statistics sweep, what comes in before the
// gradient sweep.  (lse_i, 1) is a valid (max, sum) pair: sum_a exp(z_ia - lse_i) = 1.
__global__ void __launch_bounds__(SM_NT)
sm_export_kernel(const float *__restrict__ lse, const float *__restrict__ zt, const int32_t *__restrict__ target_pos,
                 const int32_t *__restrict__ n_active_p, int M, int B, SmSplitIO io) {
    const int i = blockIdx.x * SM_NT + threadIdx.x;
    if (i >= B) return;
    const int n = sm_clamp_n(n_active_p, M);
    const int tp = target_pos[i];
    io.row_max[i] = n > 0 ? lse[i] : -INFINITY;
    io.row_sum[i] = n > 0 ? 1.f : 0.f;
    io.tz_out[i] = (tp >= 0 && tp < n) ? zt[i] : 0.f;
}
__global__ void __launch_bounds__(SM_NT)
sm_import_kernel(SmSplitIO io, int B, float *__restrict__ lse, float *__restrict__ loss_i) {
    const int i = blockIdx.x * SM_NT + threadIdx.x;
    if (i >= B) return;
    const float l = io.gmax[i] + __logf(io.gsum[i]);
    lse[i] = l;
    loss_i[i] = l - io.gtz[i];
}
// caller-supplied selection: ids outside [0, C) and positions outside the list are flagged and made harmless
__global__ void __launch_bounds__(SM_NT)
sm_sanitize_kernel(const int32_t *__restrict__ active_idx, const int32_t *__restrict__ n_active_p,
                   const int32_t *__restrict__ target_pos, int64_t C, int M, int B, int32_t *__restrict__ act_safe,
                   int32_t *__restrict__ n_safe, int32_t *__restrict__ tp_safe, int32_t *dev_status) {
    const int t = blockIdx.x * SM_NT + threadIdx.x;
    // (all three loads are issued before the count is looked at: the kernel is one round trip to memory long)
    const int32_t a_in = t < M ? active_idx[t] : -1;
    const int32_t tp_in = t < B ? target_pos[t] : -1;
    int n = *n_active_p;
    if (n < 0 || n > M) {
        if (t == 0) ks_flag(dev_status, KS_DEV_BAD_COUNT);
        n = n < 0 ? 0 : M;
    }
    if (t == 0) *n_safe = n;
    if (t < M) {
        int32_t a = -1;
        if (t < n) {
            a = a_in;
            if (a < 0 || a >= C) {
                ks_flag(dev_status, KS_DEV_BAD_INDEX);
                a = 0;
            }
        }
        act_safe[t] = a;
    }
    if (t < B) {
        int32_t tp = tp_in;
        if (tp >= n) {
            ks_flag(dev_status, KS_DEV_BAD_LABEL);
            tp = -1;
        }
        tp_safe[t] = tp < 0 ? -1 : tp;
    }
}

// compute units of the current device (asked once)
static int ks_n_cu() {
    static int n = 0;
    if (n == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            n = v;
        else
            n = 256;
    }
    return n;
}

struct SmWs {
    void *select;
    float *Z;
    uint16_t *dZ;
    float *lse;
    float *part;
    uint16_t *dZT; // fast path: the logit gradient is kept transposed only
    float *pm, *pl, *zt; // fast path: per class-tile softmax statistics, target logits
    float *inv;          // one-sweep softmax: 1 / sum_a exp(z_ia - scale) per sample
    uint16_t *X2;        // one-sweep softmax: rows of X scaled by that
    int S;
    int64_t Mp;
    int Bp;
    bool fast;
};

static int sm_splits(int B, int D, int64_t M, bool fast) {
    int tiles = fast ? (int)(ks_ceil_div(B, TileDx::BM) * ks_ceil_div(D, TileDx::BN))
                     : (int)(ks_ceil_div(B, TileG::BM) * ks_ceil_div(D, TileG::BN));
    // two workgroups per compute unit
    int S = (int)ks_ceil_div(512, tiles);
    if (S < 1) S = 1;
    if (S > 32) S = 32;
    if (fast) { // a share of the active dimension must fit the dX kernel's LDS index cache
        const int64_t nk = ks_ceil_div(M, 64);
        const int need = (int)ks_ceil_div(nk, DX_IDX_CACHE / 64);
        if (S < need) S = need;
    }
    return S;
}

static SmWs sm_carve(void *ws, int64_t C, int D, int B, int K, int64_t M, bool with_select, size_t *total) {
    KsArena ar(ws);
    SmWs w;
    w.fast = (D % 64 == 0);
    w.Mp = sm_mp(M);
    w.Bp = (int)ks_align_up((size_t)B, KS_BP_ALIGN);
    w.S = sm_splits(B, D, M, w.fast);
    w.select = with_select ? (void *)ar.take<char>(ks_select_ws_bytes(C, B, K)) : nullptr;
    w.lse = ar.take<float>((size_t)B);
    w.part = ar.take<float>((size_t)w.S * B * D);
    w.Z = nullptr;
    w.dZ = w.dZT = nullptr;
    w.pm = w.pl = w.zt = w.inv = nullptr;
    w.X2 = nullptr;
    if (w.fast) {
        w.dZT = ar.take<uint16_t>((size_t)w.Mp * w.Bp);
        size_t nt = (size_t)(w.Mp / TileSm::BM);
        if (nt < (size_t)SM_SOE_GRID) nt = SM_SOE_GRID; // per-slab statistics of the stationary-operand kernels
        w.pm = ar.take<float>(nt * w.Bp);
        w.pl = ar.take<float>(nt * w.Bp);
        w.zt = ar.take<float>((size_t)w.Bp);
        w.inv = ar.take<float>((size_t)w.Bp);
        w.X2 = ar.take<uint16_t>((size_t)w.Bp * D);
    } else {
        w.Z = ar.take<float>((size_t)B * w.Mp);
        w.dZ = ar.take<uint16_t>((size_t)B * w.Mp);
    }
    if (total) *total = ar.off;
    return w;
}

// everything after the selection; active_idx / n_active / target_pos are device-resident inputs here
static int sm_run(const uint16_t *W, const uint16_t *X, int D, int B, int64_t M, float scale, float grad_scale,
                  const int32_t *active_idx, const int32_t *n_active, const int32_t *target_pos,
                  float *loss_per_sample, float *loss_mean, float *dX, float *dW_active, const SmWs &w,
                  uint32_t flags, int32_t *dev_status, hipStream_t st, hipEvent_t *ev = nullptr, int mode = SM_WHOLE,
                  SmSplitIO io = SmSplitIO(), DwUpdate up = DwUpdate(), const KsSelNext *next_p = nullptr) {
    auto mark = [&](int k) { if (ev) (void)hipEventRecord(ev[k], st); };
    KsSelNext next = KsSelNext();
    if (next_p) next = *next_p; // (the caller has checked that this path takes it: w.fast, and the dX and dW launches are made)
    if (mode != SM_WHOLE && !w.fast) return KS_UNSUPPORTED;
    if (mode == SM_EXPORT) loss_per_sample = w.inv; // not known before the exchange: the kernels' loss output is scratch
    const int Mi = (int)M;
    const float g = grad_scale / (float)B;
    bool fused = false;
    if (w.fast) {
        const int tiles_s = (int)ks_ceil_div(B, 256);
        const bool soe = (D == 128 || D == 256 || D == 512) && tiles_s <= SM_SOE_GRID && scale > 0.f && g > 0.f;
        // unit rows: |logit| <= scale, and exp(-2 scale) must stay a normal number
        fused = soe && (flags & KS_FLAG_UNIT_ROWS) && scale <= KS_FUSED_MAX_SCALE;
        if (fused) {
            const int grid = SM_SOE_GRID / tiles_s * tiles_s, slabs = grid / tiles_s;
#define SM_FUSED_LAUNCH(KT)                                                                                               \
    hipLaunchKernelGGL(sm_fused_soe_kernel<KT>, dim3(grid), dim3(512), 0, st, X, W, active_idx, n_active, target_pos, B,   \
                       w.Bp, D, Mi, tiles_s, scale, w.pl, w.pm, w.dZT)
            if (mode != SM_IMPORT) { // the first call of a split has left the exponentials in the workspace
                if (D == 512) SM_FUSED_LAUNCH(8);
                else if (D == 256) SM_FUSED_LAUNCH(4);
                else SM_FUSED_LAUNCH(2);
            }
#undef SM_FUSED_LAUNCH
            mark(2);
            hipLaunchKernelGGL(sm_combine_fused_kernel, dim3((unsigned)ks_ceil_div(B, SM_CF_SPB)), dim3(SM_CF_NT), 0, st, w.pl,
                               w.pm, n_active, active_idx, target_pos, X, W, Mi, slabs, B, w.Bp, D, scale, w.inv, loss_per_sample,
                               w.dZT, w.X2, dev_status, mode, io);
            mark(3);
            if (mode == SM_EXPORT) {
                KS_LAUNCH_CHECK();
                return KS_OK;
            }
        } else if (soe) {
            const int grid = SM_SOE_GRID / tiles_s * tiles_s, slabs = grid / tiles_s;
#define SM_SOE_LAUNCH(KT)                                                                                                 \
    do {                                                                                                                  \
        if (mode != SM_IMPORT) {                                                                                          \
            hipLaunchKernelGGL(sm_stats_soe_kernel<KT>, dim3(grid), dim3(512), 0, st, X, W, active_idx, n_active,         \
                               target_pos, B, w.Bp, D, Mi, tiles_s, scale, w.pm, w.pl, w.zt);                              \
            mark(2);                                                                                                      \
            hipLaunchKernelGGL(sm_combine_soe_kernel, dim3((unsigned)ks_ceil_div(B, SM_NT / 64)), dim3(SM_NT), 0, st,     \
                               w.pm, w.pl, w.zt, n_active, Mi, slabs, B, w.Bp, w.lse, loss_per_sample);                    \
            mark(3);                                                                                                      \
        }                                                                                                                 \
        if (mode != SM_EXPORT)                                                                                            \
            hipLaunchKernelGGL(sm_grad_soe_kernel<KT>, dim3(grid), dim3(512), 0, st, X, W, active_idx, n_active,          \
                               target_pos, w.lse, B, w.Bp, D, Mi, tiles_s, scale, g, w.dZT);                               \
    } while (0)
            if (mode == SM_IMPORT)
                hipLaunchKernelGGL(sm_import_kernel, dim3((unsigned)ks_ceil_div(B, SM_NT)), dim3(SM_NT), 0, st, io, B, w.lse,
                                   loss_per_sample);
            if (D == 512) SM_SOE_LAUNCH(8);
            else if (D == 256) SM_SOE_LAUNCH(4);
            else SM_SOE_LAUNCH(2);
#undef SM_SOE_LAUNCH
        } else {
            typedef TileSm T;
            const int tiles = (int)(ks_ceil_div(B, T::BN) * ks_ceil_div(M, T::BM));
            if (mode != SM_IMPORT) {
                hipLaunchKernelGGL(sm_stats_kernel<T>, dim3(tiles), dim3(T::NT), 0, st, X, W, active_idx, n_active, target_pos,
                                   B, w.Bp, D, Mi, scale, w.pm, w.pl, w.zt);
                mark(2);
                hipLaunchKernelGGL(sm_combine_kernel, dim3((unsigned)ks_ceil_div(B, SM_NT / 64)), dim3(SM_NT), 0, st, w.pm,
                                   w.pl, w.zt, n_active, Mi, T::BM, B, w.Bp, w.lse, loss_per_sample);
                mark(3);
            } else {
                hipLaunchKernelGGL(sm_import_kernel, dim3((unsigned)ks_ceil_div(B, SM_NT)), dim3(SM_NT), 0, st, io, B, w.lse,
                                   loss_per_sample);
            }
            if (mode != SM_EXPORT)
                hipLaunchKernelGGL(sm_grad_kernel<T>, dim3(tiles), dim3(T::NT), 0, st, X, W, active_idx, n_active, target_pos,
                                   w.lse, B, w.Bp, D, Mi, scale, g, w.dZT);
        }
        if (mode == SM_EXPORT) { // two-sweep paths: the statistics sweep is done, (lse, 1) and the target logit go out
            hipLaunchKernelGGL(sm_export_kernel, dim3((unsigned)ks_ceil_div(B, SM_NT)), dim3(SM_NT), 0, st, w.lse, w.zt,
                               target_pos, n_active, Mi, B, io);
            KS_LAUNCH_CHECK();
            return KS_OK;
        }
        mark(4);
        {
            typedef TileDx T;
            const int tiles = (int)(ks_ceil_div(B, T::BM) * ks_ceil_div(D, T::BN));
            if (next.nsel) next.nfetch = (int)ks_ceil_div((int64_t)next.B * (next.K + 1), (int64_t)T::NT);
            hipLaunchKernelGGL(dx_partial_async_kernel<T>, dim3(tiles * w.S + next.nfetch), dim3(T::NT), 0, st, w.dZT, w.Bp,
                               w.Mp, W, active_idx, n_active, B, D, Mi, w.S, w.part, next);
        }
        mark(5);
        mark(6); // the reduction of the partial products rides along with the next launch
        {
            typedef TileDw T;
            const int tiles = (int)(ks_ceil_div(M, TileDw128::BM) * ks_ceil_div(D, T::BN)); // the most any tile height needs
            DxReduceJob job;
            job.part = w.part;
            job.S = w.S;
            job.BD = (int64_t)B * D;
            job.scale = fused ? scale * g : scale;
            job.row_factor = fused ? w.inv : nullptr;
            job.dX = dX;
            job.loss_i = loss_per_sample;
            job.loss_mean = loss_mean;
            hipLaunchKernelGGL(dw_async_kernel, dim3(next.nsel + tiles + DW_REDUCE_BLOCKS), dim3(T::NT), 0, st, w.dZT,
                               fused ? w.X2 : X, B, w.Bp, n_active, D, Mi, w.Mp, fused ? scale * g : scale, dW_active, tiles,
                               ks_n_cu(), job, up, next);
        }
        mark(7);
        KS_LAUNCH_CHECK();
        return KS_OK;
    }
    typedef TileG T;
    const int tiles_b = (int)ks_ceil_div(B, T::BM);
    const int tiles_a_n = (int)ks_ceil_div(M, T::BN), tiles_a_m = (int)ks_ceil_div(M, T::BM);
    const int tiles_d = (int)ks_ceil_div(D, T::BN);

    hipLaunchKernelGGL(logits_kernel<T>, dim3(tiles_b * tiles_a_n), dim3(T::NT), 0, st, X, W, active_idx, n_active, B, D,
                       Mi, scale, w.Z, w.Mp);
    mark(2);
    hipLaunchKernelGGL(row_stats_kernel, dim3(B), dim3(SM_NT), 0, st, w.Z, w.Mp, n_active, Mi, target_pos, w.lse,
                       loss_per_sample);
    mark(3);
    hipLaunchKernelGGL(dz_kernel, dim3((unsigned)ks_ceil_div(w.Mp, SM_NT * 8), B), dim3(SM_NT), 0, st, w.Z, w.Mp, n_active,
                       Mi, target_pos, w.lse, g, w.dZ);
    mark(4);
    hipLaunchKernelGGL(dx_partial_kernel<T>, dim3(tiles_b * tiles_d, w.S), dim3(T::NT), 0, st, w.dZ, w.Mp, W, active_idx,
                       n_active, B, D, Mi, w.part);
    mark(5);
    hipLaunchKernelGGL(dx_reduce_kernel, dim3((unsigned)ks_ceil_div((int64_t)B * D / 4, SM_NT)), dim3(SM_NT), 0, st, w.part,
                       w.S, (int64_t)B * D, scale, (const float *)nullptr, D, dX, loss_per_sample, B, loss_mean);
    mark(6);
    hipLaunchKernelGGL(dw_kernel<T>, dim3(tiles_a_m * tiles_d), dim3(T::NT), 0, st, w.dZ, w.Mp, X, n_active, B, D, Mi,
                       scale, dW_active);
    mark(7);
    KS_LAUNCH_CHECK();
    return KS_OK;
}

static int sm_check_dims(int64_t C, int D, int B) {
    if (C < 1 || C >= (int64_t)1 << 31 || D < 32 || D % 32 != 0 || B < 1) return KS_INVALID_ARG;
    return KS_OK;
}

extern "C" size_t knn_softmax_workspace(int64_t C, int D, int B, int K, int M) {
    if (sm_check_dims(C, D, B) != KS_OK || K < 0 || M < 1) return 0;
    size_t total = 0;
    sm_carve(nullptr, C, D, B, K, M, true, &total);
    return total;
}

static int sm_fwd_bwd(const uint16_t *W_bf16, const uint16_t *X_bf16, const int32_t *labels, const int32_t *graph,
                      int64_t C, int D, int B, int K, int M, float scale, float grad_scale, uint32_t flags,
                      int32_t *active_idx, int32_t *n_active, int32_t *target_pos, float *loss_per_sample,
                      float *loss_mean, float *dX, float *dW_active, void *ws, size_t ws_bytes, int32_t *dev_status,
                      void *stream, hipEvent_t *ev, float *W_master = nullptr, uint16_t *W_bf16_out = nullptr,
                      float alpha = 0.f) {
    if (!W_bf16 || !X_bf16 || !labels || !active_idx || !n_active || !target_pos || !loss_per_sample || !loss_mean ||
        !dX || !ws)
        return KS_INVALID_ARG;
    const bool fast = D % 64 == 0; // the update runs inside the dW kernel of these paths; the others keep dW_active
    if (!dW_active && !(W_master && fast)) return KS_INVALID_ARG;
    if (sm_check_dims(C, D, B) != KS_OK || K < 0 || M < 1) return KS_INVALID_ARG;
    if (K > 0 && !graph) return KS_INVALID_ARG;
    if (B > M || (int64_t)K + 1 > M) return KS_INVALID_ARG;
    size_t need = 0;
    SmWs w = sm_carve(ws, C, D, B, K, M, true, &need);
    if (ws_bytes < need) return KS_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)stream;
    if (ev) (void)hipEventRecord(ev[0], st);
    int rc = ks_select_launch(labels, graph, C, B, K, M, active_idx, n_active, target_pos, w.select, dev_status, st);
    if (rc != KS_OK) return rc;
    if (ev) (void)hipEventRecord(ev[1], st);
    DwUpdate up = DwUpdate();
    if (W_master && fast) {
        up.Wm = W_master;
        up.Wb = W_bf16_out;
        up.idx = active_idx;
        up.alpha = alpha;
    }
    rc = sm_run(W_bf16, X_bf16, D, B, M, scale, grad_scale, active_idx, n_active, target_pos, loss_per_sample, loss_mean,
                dX, dW_active, w, flags, dev_status, st, ev, SM_WHOLE, SmSplitIO(), up);
    if (rc != KS_OK || !W_master || fast) return rc;
    // other shapes: the stand-alone update on the stored gradient (active_idx is strictly ascending)
    return apply_weight_grad(W_master, W_bf16_out, active_idx, n_active, M, dW_active, alpha, C, D, 1, ws, ws_bytes,
                             dev_status, stream);
}

extern "C" int knn_softmax_fwd_bwd(const uint16_t *W_bf16, const uint16_t *X_bf16, const int32_t *labels,
                                   const int32_t *graph, int64_t C, int D, int B, int K, int M, float scale,
                                   float grad_scale, uint32_t flags, int32_t *active_idx, int32_t *n_active,
                                   int32_t *target_pos, float *loss_per_sample, float *loss_mean, float *dX,
                                   float *dW_active, void *ws, size_t ws_bytes, int32_t *dev_status, void *stream) {
    return sm_fwd_bwd(W_bf16, X_bf16, labels, graph, C, D, B, K, M, scale, grad_scale, flags, active_idx, n_active,
                      target_pos, loss_per_sample, loss_mean, dX, dW_active, ws, ws_bytes, dev_status, stream, nullptr);
}

extern "C" int knn_softmax_fwd_bwd_update(float *W_master, uint16_t *W_bf16, const uint16_t *X_bf16, const int32_t *labels,
                                          const int32_t *graph, int64_t C, int D, int B, int K, int M, float scale,
                                          float grad_scale, float alpha, uint32_t flags, int32_t *active_idx,
                                          int32_t *n_active, int32_t *target_pos, float *loss_per_sample, float *loss_mean,
                                          float *dX, float *dW_active, void *ws, size_t ws_bytes, int32_t *dev_status,
                                          void *stream) {
    if (!W_master) return KS_INVALID_ARG;
    return sm_fwd_bwd(W_bf16, X_bf16, labels, graph, C, D, B, K, M, scale, grad_scale, flags, active_idx, n_active,
                      target_pos, loss_per_sample, loss_mean, dX, dW_active, ws, ws_bytes, dev_status, stream, nullptr,
                      W_master, W_bf16, alpha);
}

extern "C" int knn_softmax_fwd_bwd_profiled(float *W_master, uint16_t *W_bf16, const uint16_t *X_bf16,
                                            const int32_t *labels, const int32_t *graph, int64_t C, int D, int B, int K,
                                            int M, float scale, float grad_scale, float alpha, uint32_t flags,
                                            int32_t *active_idx, int32_t *n_active, int32_t *target_pos,
                                            float *loss_per_sample, float *loss_mean, float *dX, float *dW_active, void *ws,
                                            size_t ws_bytes, int32_t *dev_status, void *stream, void **events,
                                            int n_events) {
    if (!events || n_events < KS_N_PHASE_EVENTS) return KS_INVALID_ARG;
    for (int k = 0; k < KS_N_PHASE_EVENTS; ++k)
        if (!events[k]) return KS_INVALID_ARG;
    return sm_fwd_bwd(W_bf16, X_bf16, labels, graph, C, D, B, K, M, scale, grad_scale, flags, active_idx, n_active,
                      target_pos, loss_per_sample, loss_mean, dX, dW_active, ws, ws_bytes, dev_status, stream,
                      (hipEvent_t *)events, W_master, W_bf16, alpha);
}

// The two calls of the softmax split over nodes.  Workspace: the softmax buffers (which carry the first call's
// exponentials, or nothing on the two-sweep paths, to the second call), then the sanitised copy of the selection.
struct SmSplitWs {
    SmWs w;
    int32_t *act, *n, *tp;
};
static SmSplitWs sm_split_carve(void *ws, int64_t C, int D, int B, int64_t M, size_t *total) {
    size_t used = 0;
    SmSplitWs s;
    s.w = sm_carve(ws, C, D, B, 0, M, false, &used);
    KsArena ar(ws ? (void *)((char *)ws + used) : nullptr);
    s.act = ar.take<int32_t>((size_t)M);
    s.tp = ar.take<int32_t>((size_t)B);
    s.n = ar.take<int32_t>(1);
    if (total) *total = used + ar.off;
    return s;
}
static int sm_split_check(int64_t C, int D, int B, int M, float scale, uint32_t flags) {
    if (sm_check_dims(C, D, B) != KS_OK || M < 1 || !(scale > 0.f)) return KS_INVALID_ARG;
    if (flags & ~(uint32_t)KS_FLAG_UNIT_ROWS) return KS_INVALID_ARG;
    if (D % 64 != 0) return KS_UNSUPPORTED;
    return KS_OK;
}

extern "C" size_t knn_softmax_split_workspace(int64_t C, int D, int B, int M) {
    if (sm_split_check(C, D, B, M, 1.f, 0) != KS_OK) return 0;
    size_t total = 0;
    sm_split_carve(nullptr, C, D, B, M, &total);
    return total;
}

extern "C" int knn_softmax_fwd_stats(const uint16_t *W_bf16, const uint16_t *X_bf16, const int32_t *active_idx,
                                     const int32_t *n_active, const int32_t *target_pos, int64_t C, int D, int B, int M,
                                     float scale, uint32_t flags, float *row_max, float *row_sumexp, float *target_logit,
                                     void *ws, size_t ws_bytes, int32_t *dev_status, void *stream) {
    if (!W_bf16 || !X_bf16 || !active_idx || !n_active || !target_pos || !row_max || !row_sumexp || !target_logit || !ws)
        return KS_INVALID_ARG;
    const bool trusted = (flags & KS_FLAG_TRUSTED_LIST) != 0;
    flags &= ~(uint32_t)KS_FLAG_TRUSTED_LIST;
    int rc = sm_split_check(C, D, B, M, scale, flags);
    if (rc != KS_OK) return rc;
    size_t need = 0;
    SmSplitWs s = sm_split_carve(ws, C, D, B, M, &need);
    if (ws_bytes < need) return KS_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)stream;
    const int nmax = M > B ? M : B;
    if (!trusted) {
        hipLaunchKernelGGL(sm_sanitize_kernel, dim3((unsigned)ks_ceil_div(nmax, SM_NT)), dim3(SM_NT), 0, st, active_idx,
                           n_active, target_pos, C, M, B, s.act, s.n, s.tp, dev_status);
        active_idx = s.act;
        n_active = s.n;
        target_pos = s.tp;
    }
    SmSplitIO io = SmSplitIO();
    io.row_max = row_max;
    io.row_sum = row_sumexp;
    io.tz_out = target_logit;
    return sm_run(W_bf16, X_bf16, D, B, M, scale, 1.f, active_idx, n_active, target_pos, nullptr, nullptr, nullptr, nullptr, s.w,
                  flags, dev_status, st, nullptr, SM_EXPORT, io);
}

// the next batch's selection on the node's compressed graph that rides along with the second call of a split (nullptr: none)
struct SmNextCsr {
    const int32_t *labels, *counts;
    const int64_t *offsets;
    const int32_t *flat;
    int64_t flat_len, Cg, c0;
    int K_max;
    uint32_t sel_flags;
    uint64_t pad_seed;
    int32_t *active_idx, *n_active, *n_found, *target_pos;
};
static int sm_bwd_from_stats(const uint16_t *W_bf16, const uint16_t *X_bf16, const int32_t *active_idx, const int32_t *n_active,
                             const int32_t *target_pos, const float *global_max, const float *global_sumexp,
                             const float *global_target_logit, int64_t C, int D, int B, int M, float scale, float grad_scale,
                             uint32_t flags, float *loss_per_sample, float *loss_mean, float *dX, float *dW_active,
                             const SmNextCsr *nx, void *ws, size_t ws_bytes, int32_t *dev_status, void *stream) {
    if (!W_bf16 || !X_bf16 || !active_idx || !n_active || !target_pos || !global_max || !global_sumexp ||
        !global_target_logit || !loss_per_sample || !loss_mean || !dX || !dW_active || !ws)
        return KS_INVALID_ARG;
    const bool trusted = (flags & KS_FLAG_TRUSTED_LIST) != 0;
    flags &= ~(uint32_t)KS_FLAG_TRUSTED_LIST;
    int rc = sm_split_check(C, D, B, M, scale, flags);
    if (rc != KS_OK) return rc;
    if (!(grad_scale > 0.f)) return KS_INVALID_ARG;
    if (nx) { // the conditions of knn_select_active_csr
        if (!nx->labels || !nx->counts || !nx->offsets || !nx->active_idx || !nx->n_active || !nx->target_pos) return KS_INVALID_ARG;
        if (nx->Cg < 1 || nx->Cg >= (int64_t)1 << 31 || nx->c0 < 0 || nx->c0 + C > nx->Cg) return KS_INVALID_ARG;
        if (nx->K_max < 0 || nx->flat_len < 0 || (nx->flat_len > 0 && !nx->flat)) return KS_INVALID_ARG;
        if (B > M || (int64_t)nx->K_max + 1 > M) return KS_INVALID_ARG;
        if (nx->sel_flags & ~(uint32_t)KS_FLAG_PAD_RANDOM) return KS_INVALID_ARG;
        if (trusted && (nx->active_idx == active_idx || nx->n_active == n_active || nx->target_pos == target_pos))
            return KS_INVALID_ARG; // a trusted list is read in place: the next one needs buffers of its own
    }
    size_t need = 0;
    SmSplitWs s = sm_split_carve(ws, C, D, B, M, &need);
    if (nx) need = ks_align_up(need, 256);
    void *sel_ws = (char *)ws + need;
    if (nx) need += ks_select_ws_bytes(C, B, nx->K_max);
    if (ws_bytes < need) return KS_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)stream;
    const int nmax = M > B ? M : B;
    if (!trusted) {
        hipLaunchKernelGGL(sm_sanitize_kernel, dim3((unsigned)ks_ceil_div(nmax, SM_NT)), dim3(SM_NT), 0, st, active_idx,
                           n_active, target_pos, C, M, B, s.act, s.n, s.tp, dev_status);
        active_idx = s.act;
        n_active = s.n;
        target_pos = s.tp;
    }
    SmSplitIO io = SmSplitIO();
    io.gmax = global_max;
    io.gsum = global_sumexp;
    io.gtz = global_target_logit;
    KsSelNext next = KsSelNext();
    const bool ride = nx && C <= (int64_t)SEL1_MAX_WORDS * 32;
    if (ride) {
        next.nsel = SEL1_GRID;
        next.csr_source = 1;
        next.csr = SelCsr{nx->labels, nx->counts, nx->offsets, nx->flat, nx->Cg, nx->c0, C, nx->flat_len, nx->K_max};
        next.pad = sel_pad_make((nx->sel_flags & KS_FLAG_PAD_RANDOM) != 0, C, nx->pad_seed);
        next.C = C;
        next.B = B;
        next.K = nx->K_max;
        next.M = M;
        next.cand = (int32_t *)sel_ws;
        next.active_idx = nx->active_idx;
        next.n_active = nx->n_active;
        next.n_found = nx->n_found;
        next.target_pos = nx->target_pos;
        next.dev_status = dev_status;
    }
    rc = sm_run(W_bf16, X_bf16, D, B, M, scale, grad_scale, active_idx, n_active, target_pos, loss_per_sample, loss_mean, dX,
                dW_active, s.w, flags, dev_status, st, nullptr, SM_IMPORT, io, DwUpdate(), ride ? &next : nullptr);
    if (rc == KS_OK && nx && !ride)
        rc = knn_select_active_csr(nx->labels, nx->counts, nx->offsets, nx->flat, nx->flat_len, nx->Cg, nx->c0, C, B, nx->K_max, M,
                                   nx->sel_flags, nx->pad_seed, nx->active_idx, nx->n_active, nx->n_found, nx->target_pos, sel_ws,
                                   ks_select_ws_bytes(C, B, nx->K_max), dev_status, stream);
    return rc;
}
extern "C" int knn_softmax_bwd_from_stats(const uint16_t *W_bf16, const uint16_t *X_bf16, const int32_t *active_idx,
                                          const int32_t *n_active, const int32_t *target_pos, const float *global_max,
                                          const float *global_sumexp, const float *global_target_logit, int64_t C, int D,
                                          int B, int M, float scale, float grad_scale, uint32_t flags,
                                          float *loss_per_sample, float *loss_mean, float *dX, float *dW_active, void *ws,
                                          size_t ws_bytes, int32_t *dev_status, void *stream) {
    return sm_bwd_from_stats(W_bf16, X_bf16, active_idx, n_active, target_pos, global_max, global_sumexp, global_target_logit,
                             C, D, B, M, scale, grad_scale, flags, loss_per_sample, loss_mean, dX, dW_active, nullptr, ws,
                             ws_bytes, dev_status, stream);
}
extern "C" size_t knn_softmax_split_next_workspace(int64_t C, int D, int B, int K_max, int M) {
    if (sm_split_check(C, D, B, M, 1.f, 0) != KS_OK || K_max < 0) return 0;
    size_t total = 0;
    sm_split_carve(nullptr, C, D, B, M, &total);
    return ks_align_up(total, 256) + ks_select_ws_bytes(C, B, K_max);
}
extern "C" int knn_softmax_bwd_from_stats_next(const uint16_t *W_bf16, const uint16_t *X_bf16, const int32_t *active_idx,
                                               const int32_t *n_active, const int32_t *target_pos, const float *global_max,
                                               const float *global_sumexp, const float *global_target_logit, int64_t C, int D,
                                               int B, int M, float scale, float grad_scale, uint32_t flags,
                                               float *loss_per_sample, float *loss_mean, float *dX, float *dW_active,
                                               const int32_t *labels_next, const int32_t *counts, const int64_t *offsets,
                                               const int32_t *flat, int64_t flat_len, int64_t Cg, int64_t c0, int K_max,
                                               uint32_t select_flags, uint64_t pad_seed, int32_t *active_idx_next,
                                               int32_t *n_active_next, int32_t *n_found_next, int32_t *target_pos_next,
                                               void *ws, size_t ws_bytes, int32_t *dev_status, void *stream) {
    SmNextCsr nx{labels_next, counts, offsets, flat, flat_len, Cg, c0, K_max, select_flags, pad_seed, active_idx_next,
                 n_active_next, n_found_next, target_pos_next};
    return sm_bwd_from_stats(W_bf16, X_bf16, active_idx, n_active, target_pos, global_max, global_sumexp, global_target_logit,
                             C, D, B, M, scale, grad_scale, flags, loss_per_sample, loss_mean, dX, dW_active, &nx, ws, ws_bytes,
                             dev_status, stream);
}

// The step on a selection computed earlier (possibly on another stream): sanitised copy of the list, then everything
// after the selection.  The softmax buffers come first in the workspace, the copy of the list after them.
static int sm_selected_check(int64_t C, int D, int B, int M) {
    if (sm_check_dims(C, D, B) != KS_OK || M < 1 || B > M) return KS_INVALID_ARG;
    return KS_OK;
}
extern "C" size_t knn_softmax_selected_workspace(int64_t C, int D, int B, int M) {
    if (sm_selected_check(C, D, B, M) != KS_OK) return 0;
    size_t total = 0;
    sm_split_carve(nullptr, C, D, B, M, &total);
    return total;
}
// the next batch's selection that rides along with a step on a given selection (nullptr: none)
struct SmNextArgs {
    const int32_t *labels, *graph;
    int K;
    int32_t *active_idx, *n_active, *target_pos;
};
static int sm_selected(float *W_master, uint16_t *W_bf16, const uint16_t *X_bf16, const int32_t *active_idx,
                       const int32_t *n_active, const int32_t *target_pos, int64_t C, int D, int B, int M, float scale,
                       float grad_scale, float alpha, uint32_t flags, float *loss_per_sample, float *loss_mean, float *dX,
                       float *dW_active, const SmNextArgs *nx, void *ws, size_t ws_bytes, int32_t *dev_status, void *stream) {
    if (!W_bf16 || !X_bf16 || !active_idx || !n_active || !target_pos || !loss_per_sample || !loss_mean || !dX || !ws)
        return KS_INVALID_ARG;
    if (sm_selected_check(C, D, B, M) != KS_OK) return KS_INVALID_ARG;
    if (flags & ~(uint32_t)(KS_FLAG_UNIT_ROWS | KS_FLAG_TRUSTED_LIST)) return KS_INVALID_ARG;
    const bool fast = D % 64 == 0;
    const bool trusted = (flags & KS_FLAG_TRUSTED_LIST) != 0;
    if (!dW_active && !(W_master && fast)) return KS_INVALID_ARG;
    // a trusted list is read where it lies, until the end of the call: the next batch's list needs buffers of its own
    if (nx && trusted && (nx->active_idx == active_idx || nx->n_active == n_active || nx->target_pos == target_pos))
        return KS_INVALID_ARG;
    if (nx) {
        if (!nx->labels || !nx->active_idx || !nx->n_active || !nx->target_pos || nx->K < 0 || (nx->K > 0 && !nx->graph))
            return KS_INVALID_ARG;
        if ((int64_t)nx->K + 1 > M) return KS_INVALID_ARG;
    }
    size_t need = 0;
    SmSplitWs s = sm_split_carve(ws, C, D, B, M, &need);
    if (nx) need = ks_align_up(need, 256);
    void *sel_ws = (char *)ws + need; // the selection's staging area follows the step's buffers
    if (nx) need += ks_select_ws_bytes(C, B, nx->K);
    if (ws_bytes < need) return KS_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)stream;
    const int nmax = M > B ? M : B;
    const int32_t *act = active_idx, *n_act = n_active, *tp = target_pos;
    if (!trusted) { // the validated copy (which also lets the next batch's list be written where this one came in)
        hipLaunchKernelGGL(sm_sanitize_kernel, dim3((unsigned)ks_ceil_div(nmax, SM_NT)), dim3(SM_NT), 0, st, active_idx,
                           n_active, target_pos, C, M, B, s.act, s.n, s.tp, dev_status);
        act = s.act;
        n_act = s.n;
        tp = s.tp;
    }
    DwUpdate up = DwUpdate();
    if (W_master && fast) {
        up.Wm = W_master;
        up.Wb = W_bf16;
        up.idx = act;
        up.alpha = alpha;
    }
    // The selection rides along with the dX and dW launches where those exist (D a multiple of 64) and the class bitmap
    // fits in LDS; otherwise it follows the step as launches of its own.  Either way it starts after the sanitised copy
    // of this step's list has been made, so its outputs may be the buffers this step's list came in.
    KsSelNext next = KsSelNext();
    const bool ride = nx && fast && C <= (int64_t)SEL1_MAX_WORDS * 32;
    if (ride) {
        next.nsel = SEL1_GRID;
        next.dense = SelDense{nx->labels, nx->graph, C, nx->K};
        next.pad = sel_pad_make(0, C, 0);
        next.C = C;
        next.B = B;
        next.K = nx->K;
        next.M = M;
        next.cand = (int32_t *)sel_ws;
        next.active_idx = nx->active_idx;
        next.n_active = nx->n_active;
        next.target_pos = nx->target_pos;
        next.dev_status = dev_status;
    }
    int rc = sm_run(W_bf16, X_bf16, D, B, M, scale, grad_scale, act, n_act, tp, loss_per_sample, loss_mean, dX, dW_active,
                    s.w, flags & KS_FLAG_UNIT_ROWS, dev_status, st, nullptr, SM_WHOLE, SmSplitIO(), up, ride ? &next : nullptr);
    if (rc == KS_OK && W_master && !fast)
        rc = apply_weight_grad(W_master, W_bf16, act, n_act, M, dW_active, alpha, C, D, 1, ws, ws_bytes, dev_status, stream);
    if (rc == KS_OK && nx && !ride)
        rc = ks_select_launch(nx->labels, nx->graph, C, B, nx->K, M, nx->active_idx, nx->n_active, nx->target_pos, sel_ws,
                              dev_status, st);
    return rc;
}
extern "C" int knn_softmax_fwd_bwd_update_selected(float *W_master, uint16_t *W_bf16, const uint16_t *X_bf16,
                                                   const int32_t *active_idx, const int32_t *n_active,
                                                   const int32_t *target_pos, int64_t C, int D, int B, int M, float scale,
                                                   float grad_scale, float alpha, uint32_t flags, float *loss_per_sample,
                                                   float *loss_mean, float *dX, float *dW_active, void *ws, size_t ws_bytes,
                                                   int32_t *dev_status, void *stream) {
    return sm_selected(W_master, W_bf16, X_bf16, active_idx, n_active, target_pos, C, D, B, M, scale, grad_scale, alpha, flags,
                       loss_per_sample, loss_mean, dX, dW_active, nullptr, ws, ws_bytes, dev_status, stream);
}
extern "C" size_t knn_softmax_selected_next_workspace(int64_t C, int D, int B, int K, int M) {
    if (sm_selected_check(C, D, B, M) != KS_OK || K < 0) return 0;
    size_t total = 0;
    sm_split_carve(nullptr, C, D, B, M, &total);
    return ks_align_up(total, 256) + ks_select_ws_bytes(C, B, K);
}
extern "C" int knn_softmax_fwd_bwd_update_selected_next(float *W_master, uint16_t *W_bf16, const uint16_t *X_bf16,
                                                        const int32_t *active_idx, const int32_t *n_active,
                                                        const int32_t *target_pos, int64_t C, int D, int B, int M,
                                                        float scale, float grad_scale, float alpha, uint32_t flags,
                                                        float *loss_per_sample, float *loss_mean, float *dX,
                                                        float *dW_active, const int32_t *labels_next, const int32_t *graph,
                                                        int K, int32_t *active_idx_next, int32_t *n_active_next,
                                                        int32_t *target_pos_next, void *ws, size_t ws_bytes,
                                                        int32_t *dev_status, void *stream) {
    SmNextArgs nx{labels_next, graph, K, active_idx_next, n_active_next, target_pos_next};
    return sm_selected(W_master, W_bf16, X_bf16, active_idx, n_active, target_pos, C, D, B, M, scale, grad_scale, alpha, flags,
                       loss_per_sample, loss_mean, dX, dW_active, &nx, ws, ws_bytes, dev_status, stream);
}

extern "C" size_t full_softmax_workspace(int64_t C, int D, int B) {
    if (sm_check_dims(C, D, B) != KS_OK) return 0;
    size_t total = 0;
    sm_carve(nullptr, C, D, B, 0, C, false, &total);
    total += ks_align_up((size_t)C * 4, 256) + ks_align_up((size_t)B * 4, 256) + 256;
    return total;
}

extern "C" int full_softmax_fwd_bwd(const uint16_t *W_bf16, const uint16_t *X_bf16, const int32_t *labels, int64_t C,
                                    int D, int B, float scale, float grad_scale, uint32_t flags, float *loss_per_sample,
                                    float *loss_mean, float *dX, float *dW, void *ws, size_t ws_bytes,
                                    int32_t *dev_status, void *stream) {
    if (!W_bf16 || !X_bf16 || !labels || !loss_per_sample || !loss_mean || !dX || !dW || !ws) return KS_INVALID_ARG;
    if (sm_check_dims(C, D, B) != KS_OK) return KS_INVALID_ARG;
    if (ws_bytes < full_softmax_workspace(C, D, B)) return KS_WORKSPACE_TOO_SMALL;
    size_t used = 0;
    SmWs w = sm_carve(ws, C, D, B, 0, C, false, &used);
    KsArena ar((char *)ws + used);
    int32_t *active_idx = ar.take<int32_t>((size_t)C);
    int32_t *target_pos = ar.take<int32_t>((size_t)B);
    int32_t *n_active = ar.take<int32_t>(1);
    hipStream_t st = (hipStream_t)stream;
    int64_t n = C > B ? C : B;
    hipLaunchKernelGGL(full_prepare_kernel, dim3((unsigned)ks_ceil_div(n, SM_NT)), dim3(SM_NT), 0, st, labels, C, B,
                       active_idx, n_active, target_pos, dev_status);
    return sm_run(W_bf16, X_bf16, D, B, C, scale, grad_scale, active_idx, n_active, target_pos, loss_per_sample,
                  loss_mean, dX, dW, w, flags, dev_status, st);
}

extern "C" int knn_gather_rows(const uint16_t *W_bf16, const int32_t *active_idx, const int32_t *n_active, int M,
                               int64_t C, int D, uint16_t *out, int32_t *dev_status, void *stream) {
    if (!W_bf16 || !active_idx || !n_active || !out) return KS_INVALID_ARG;
    if (M < 1 || C < 1 || D < 8 || D % 8 != 0) return KS_INVALID_ARG;
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)ks_ceil_div(M, SM_NT / 64)), dim3(SM_NT), 0, (hipStream_t)stream,
                       W_bf16, active_idx, n_active, M, C, D, out, dev_status);
    KS_LAUNCH_CHECK();
    return KS_OK;
}

extern "C" const char *ks_version(void) { return "knnsoftmax 0.1 (gfx950)"; }
