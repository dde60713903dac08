// Weight-streaming matrix-vector kernels for the single-token decode path
// (at most 8 activation rows).  Y[m][n] (+)= sum_k x[m][k] * W[n][k], W row-major
// [N][K] in fp32 or bf16, activations and accumulation in fp32.  Every weight
// is read from HBM exactly once per call; the activations (a few KB) are
// staged in LDS, optionally transformed on the way in:
//   PRO_NORM    x = X * rsqrt(mean(X^2) + eps) * gain   (RMSNorm fused in)
//   PRO_SWIGLU  x = silu(X[k]) * X[K + k]               (SwiGLU fused in)
// and the result is either stored or added to Y (residual stream).
#pragma once
#include "common.cuh"

enum { PRO_NONE = 0, PRO_NORM = 1, PRO_SWIGLU = 2 };
enum { EPI_STORE = 0, EPI_RESID = 1 };

// Block = 256 threads working on R consecutive rows of W.  The K axis is cut
// in 16-byte (8 bf16) slots dealt round-robin to the threads, so one block
// iteration reads 4 KiB contiguous from each of its rows.
template <typename WT, int MT, int R, int PRO, int EPI>
__global__ __launch_bounds__(256) void gemv_kernel(const WT* __restrict__ W, int N, int K,
                                                   const float* __restrict__ X, int ldx,
                                                   const WT* __restrict__ gain, float eps,
                                                   float* __restrict__ Y, int ldy, int M, int KC) {
    extern __shared__ float smem[];
    float* xs = smem;                 // [MT][KC]
    float* red = smem + MT * KC;      // [4][MT*R] then 4 scratch floats
    float* red4 = red + 4 * MT * R;
    const int tid = threadIdx.x;
    const int n0 = blockIdx.x * R;

    float rs[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) rs[m] = 1.0f;
    if (PRO == PRO_NORM) {
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            float ss = 0.0f;
            if (m < M)
                for (int k = tid * 4; k < K; k += 1024) {
                    const float4 v = *reinterpret_cast<const float4*>(X + (size_t)m * ldx + k);
                    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
                }
            ss = block256_sum(ss, red4);
            rs[m] = 1.0f / sqrtf(ss / (float)K + eps);
        }
    }

    float acc[MT][R];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int r = 0; r < R; ++r) acc[m][r] = 0.0f;

    const WT* wrow[R];
#pragma unroll
    for (int r = 0; r < R; ++r) wrow[r] = W + (size_t)min(n0 + r, N - 1) * K;

    for (int k0 = 0; k0 < K; k0 += KC) {
        const int kc = min(KC, K - k0);
        __syncthreads();
        for (int idx = tid * 4; idx < MT * kc; idx += 1024) {
            const int m = idx / kc, k = idx - m * kc;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (m < M) {
                const float* xp = X + (size_t)m * ldx + k0 + k;
                v = *reinterpret_cast<const float4*>(xp);
                if (PRO == PRO_NORM) {
                    const WT* gp = gain + k0 + k;
                    v.x *= rs[m] * ld1(gp);     v.y *= rs[m] * ld1(gp + 1);
                    v.z *= rs[m] * ld1(gp + 2); v.w *= rs[m] * ld1(gp + 3);
                } else if (PRO == PRO_SWIGLU) {
                    const float4 u = *reinterpret_cast<const float4*>(xp + K);
                    v.x = v.x / (1.0f + expf(-v.x)) * u.x; v.y = v.y / (1.0f + expf(-v.y)) * u.y;
                    v.z = v.z / (1.0f + expf(-v.z)) * u.z; v.w = v.w / (1.0f + expf(-v.w)) * u.w;
                }
            }
            *reinterpret_cast<float4*>(xs + m * KC + k) = v;
        }
        __syncthreads();
        const int slots = kc >> 3;
        for (int s = tid; s < slots; s += 256) {
            float w[R][8];
#pragma unroll
            for (int r = 0; r < R; ++r) load8(wrow[r] + k0 + s * 8, w[r]);
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                const float4 xa = *reinterpret_cast<const float4*>(xs + m * KC + s * 8);
                const float4 xb = *reinterpret_cast<const float4*>(xs + m * KC + s * 8 + 4);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    acc[m][r] += xa.x * w[r][0] + xa.y * w[r][1] + xa.z * w[r][2] + xa.w * w[r][3]
                               + xb.x * w[r][4] + xb.y * w[r][5] + xb.z * w[r][6] + xb.w * w[r][7];
                }
            }
        }
    }

    const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float v = wave_sum(acc[m][r]);
            if (lane == 0) red[wave * (MT * R) + m * R + r] = v;
        }
    __syncthreads();
    if (tid < MT * R) {
        const int m = tid / R, r = tid - m * R;
        const int n = n0 + r;
        if (m < M && n < N) {
            const float v = red[tid] + red[MT * R + tid] + red[2 * MT * R + tid] + red[3 * MT * R + tid];
            float* yp = Y + (size_t)m * ldy + n;
            *yp = (EPI == EPI_RESID) ? (*yp + v) : v;
        }
    }
}

template <typename WT, int MT, int R>
static void gemv_launch_mr(hipStream_t st, int pro, int epi, const WT* W, int N, int K, const float* X,
                           int ldx, const WT* gain, float eps, float* Y, int ldy, int M) {
    // LDS budget for the staged activations: 32 KB (48 KB when 8 rows are live)
    int KC = (MT == 8 ? 1536 : 8192 / MT);
    if (KC > K) KC = K;
    const size_t smem = (size_t)(MT * KC + 4 * MT * R + 8) * sizeof(float);
    const dim3 grid((N + R - 1) / R), block(256);
#define RSD_GEMV_CASE(P, E)                                                                          \
    if (pro == P && epi == E) {                                                                      \
        hipLaunchKernelGGL((gemv_kernel<WT, MT, R, P, E>), grid, block, smem, st, W, N, K, X, ldx,   \
                           gain, eps, Y, ldy, M, KC);                                                \
        return;                                                                                      \
    }
    RSD_GEMV_CASE(PRO_NONE, EPI_STORE)
    RSD_GEMV_CASE(PRO_NONE, EPI_RESID)
    RSD_GEMV_CASE(PRO_NORM, EPI_STORE)
    RSD_GEMV_CASE(PRO_SWIGLU, EPI_RESID)
#undef RSD_GEMV_CASE
}

// M <= 8.  Rows per block: 4 when N is small (more blocks), 8 for long outputs.
template <typename WT>
static void gemv_launch(hipStream_t st, int pro, int epi, const WT* W, int N, int K, const float* X, int ldx,
                        const WT* gain, float eps, float* Y, int ldy, int M) {
    const bool wide = N >= 16384;
    if (M <= 1) {
        if (wide) gemv_launch_mr<WT, 1, 8>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
        else      gemv_launch_mr<WT, 1, 4>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
    } else if (M <= 2) {
        if (wide) gemv_launch_mr<WT, 2, 8>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
        else      gemv_launch_mr<WT, 2, 4>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
    } else if (M <= 4) {
        gemv_launch_mr<WT, 4, 4>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
    } else {
        gemv_launch_mr<WT, 8, 4>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
    }
}
