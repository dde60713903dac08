// Weight-streaming matrix-vector kernels for the single-token decode path
// (at most 8 activation rows).  Y[m][n] (+)= sum_k x[m][k] * W[n][k], W row-major
// [N][K] in fp32 or bf16, activations and accumulation in fp32.  Every weight
// is read from HBM exactly once per call; the activations (a few KB) are
// staged in LDS, optionally transformed on the way in:
//   PRO_NORM    x = X * rsqrt(mean(X^2) + eps) * gain   (RMSNorm fused in)
//   PRO_SWIGLU  x = silu(X[k]) * X[K + k]               (SwiGLU fused in)
//   PRO_ATTN    x = merged attention output of the splits (single row only)
// and the result is either stored or added to Y (residual stream).
#pragma once
#include <algorithm>
#include <atomic>
#include <hip/hip_ext.h>
#include "common.h"

enum { PRO_NONE = 0, PRO_NORM = 1, PRO_SWIGLU = 2, PRO_ATTN = 3 };

// Timing hook: when set, the next single-row launch carries these two events in its own dispatch packet
// (start and end of the kernel itself, no dispatch gap in between) and clears the hook.
struct GemvTiming { hipEvent_t start = nullptr, stop = nullptr; };
static thread_local GemvTiming gemv_timing;

// Partial attention results of one row, one per (head, split): unnormalised sums [H][S][128] and
// (running maximum, sum of weights) pairs [H][S][2].  PRO_ATTN merges them while staging x.
struct AttnParts { const float* acc; const float* ml; int S; };
enum { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2 };

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

// Raw 8-element weight loads (kept packed in registers until they are used).  bf16 weights are marked
// non-temporal: every byte is read once per launch and should not displace anything in the caches
// (7B gate/up at one row: 48.9 -> 45.0 us; the whole 7B iteration 3.26 -> 2.99 ms).
#ifndef RSD_GEMV_NT
#define RSD_GEMV_NT 1
#endif
template <typename WT> struct Raw8;
template <> struct Raw8<bf16_t> {
    uint4 v;
    __device__ __forceinline__ void load(const bf16_t* p) {
#if RSD_GEMV_NT
        typedef uint32_t nt_u32x4 __attribute__((ext_vector_type(4)));
        const nt_u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const nt_u32x4*>(p));
        v = make_uint4(t.x, t.y, t.z, t.w);
#else
        v = *reinterpret_cast<const uint4*>(p);
#endif
    }
    __device__ __forceinline__ void unpack(float o[8]) const { unpack8(v, o); }
};
template <> struct Raw8<float> {
    float4 a, b;
    __device__ __forceinline__ void load(const float* p) {
        a = *reinterpret_cast<const float4*>(p); b = *reinterpret_cast<const float4*>(p + 4);
    }
    __device__ __forceinline__ void unpack(float o[8]) const {
        o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
    }
};

// Variant for activations that fit LDS whole (MT * K floats).  The block stages
// (and transforms) x once.  Each WAVE then owns row groups (R rows, or R gate/up
// row pairs) and walks them with its 64 lanes spread along K, 1 KiB per row and
// step; sums are finished with wave shuffles, so the main loop has no block
// barrier.  Weight loads run one step ahead of the arithmetic (also across the
// boundary between row groups, and the very first ones are issued before the
// prologue), which keeps 8..16 loads of 16 bytes per lane in flight.
//   EPI_SWIGLU: W holds [gate ; up] (2N rows); row n of gate and row N + n of up
//   are read together and silu(gate.x) * (up.x) is stored: N outputs.
template <typename WT, int MT, int R, int U, int PRO, int EPI>
__global__ __launch_bounds__(256) void gemv_full_kernel(const WT* __restrict__ W, int N, int K,
                                                        const float* __restrict__ X, int ldx,
                                                        const WT* __restrict__ gain, float eps,
                                                        float* __restrict__ Y, int ldy, int M) {
    constexpr int NA = (EPI == EPI_SWIGLU) ? 2 : 1;     // accumulator sets (gate and up)
    constexpr int NR = NA * R;                          // weight rows streamed together
    extern __shared__ float smem[];
    float* xs = smem;                                   // [MT][K]
    __shared__ float red4[4];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int slots = K >> 3, iters = (slots + 64 * U - 1) / (64 * U);    // a step covers U KiB of every row
    const int n_groups = (N + R - 1) / R;
    const int rg0 = blockIdx.x * 4 + wave, rg_stride = gridDim.x * 4;
    const int my_groups = rg0 < n_groups ? (n_groups - rg0 + rg_stride - 1) / rg_stride : 0;
    const int total = my_groups * iters;

    auto fetch = [&](int g, int i, Raw8<WT> dst[U][NR]) {
        const int n0 = (rg0 + g * rg_stride) * R;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int s = (i * U + u) * 64 + lane;
            if (s < slots) {
#pragma unroll
                for (int a = 0; a < NA; ++a)
#pragma unroll
                    for (int r = 0; r < R; ++r)
                        dst[u][a * R + r].load(W + ((size_t)a * N + min(n0 + r, N - 1)) * K + s * 8);
            }
        }
    };
    Raw8<WT> cur[U][NR], nxt[U][NR];
    if (total > 0) fetch(0, 0, cur);

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
    for (int idx = tid * 4; idx < MT * K; idx += 1024) {
        const int m = idx / K, k = idx - m * K;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (m < M) {
            v = *reinterpret_cast<const float4*>(X + (size_t)m * ldx + k);
            if (PRO == PRO_NORM) {
                const WT* gp = gain + k;
                v.x *= rs[m] * ld1(gp);     v.y *= rs[m] * ld1(gp + 1);
                v.z *= rs[m] * ld1(gp + 2); v.w *= rs[m] * ld1(gp + 3);
            }
        }
        *reinterpret_cast<float4*>(xs + idx) = v;
    }
    __syncthreads();

    float acc[NA][MT][R];
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int r = 0; r < R; ++r) acc[a][m][r] = 0.0f;

    // one step of the walk: use the registers in `buf` for step (g, i), finish the row group if it ends here
    auto use = [&](int g, int i, const Raw8<WT> buf[U][NR]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int s = (i * U + u) * 64 + lane;
            if (s < slots) {
                float w[NR][8];
#pragma unroll
                for (int q = 0; q < NR; ++q) buf[u][q].unpack(w[q]);
#pragma unroll
                for (int m = 0; m < MT; ++m) {
                    const float4 xa = *reinterpret_cast<const float4*>(xs + (size_t)m * K + s * 8);
                    const float4 xb = *reinterpret_cast<const float4*>(xs + (size_t)m * K + s * 8 + 4);
#pragma unroll
                    for (int a = 0; a < NA; ++a)
#pragma unroll
                        for (int r = 0; r < R; ++r) {
                            const float* ww = w[a * R + r];
                            acc[a][m][r] += xa.x * ww[0] + xa.y * ww[1] + xa.z * ww[2] + xa.w * ww[3]
                                          + xb.x * ww[4] + xb.y * ww[5] + xb.z * ww[6] + xb.w * ww[7];
                        }
                }
            }
        }
        if (i == iters - 1) {
            const int n0 = (rg0 + g * rg_stride) * R;
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    float v = wave_sum(acc[0][m][r]);
                    float u = (EPI == EPI_SWIGLU) ? wave_sum(acc[NA - 1][m][r]) : 0.0f;
                    acc[0][m][r] = 0.0f;
                    acc[NA - 1][m][r] = 0.0f;
                    if (lane == 0 && m < M && n0 + r < N) {
                        float* yp = Y + (size_t)m * ldy + n0 + r;
                        if (EPI == EPI_SWIGLU) *yp = v / (1.0f + expf(-v)) * u;
                        else *yp = (EPI == EPI_RESID) ? (*yp + v) : v;
                    }
                }
        }
    };
    // the two register buffers take turns (a copy between them would have to wait for the load)
    int g = 0, i = 0;
    for (int t = 0; t < total; t += 2) {
        int g1 = g, i1 = i + 1;
        if (i1 == iters) { i1 = 0; g1 = g + 1; }
        if (t + 1 < total) fetch(g1, i1, nxt);
        use(g, i, cur);
        if (t + 1 >= total) break;
        int g2 = g1, i2 = i1 + 1;
        if (i2 == iters) { i2 = 0; g2 = g1 + 1; }
        if (t + 2 < total) fetch(g2, i2, cur);
        use(g1, i1, nxt);
        g = g2; i = i2;
    }
}

constexpr size_t kGemvFullLds = 120 * 1024;      // most LDS the whole-activation variant may take

// Whole-activation variant with R rows (or gate/up pairs) per wave and U KiB per row and step.
template <typename WT, int MT, int R, int U>
static bool gemv_launch_full(hipStream_t st, int pro, int epi, const WT* W, int N, int K, const float* X,
                             int ldx, const WT* gain, float eps, float* Y, int ldy, int M) {
    const size_t full = (size_t)MT * K * sizeof(float);
    if (full > kGemvFullLds || pro == PRO_SWIGLU) return false;
    // blocks resident at once: limited by LDS (160 KB per compute unit), at most 6 per unit
    const int per_cu = (int)std::max<size_t>(1, std::min<size_t>(6, (160 * 1024) / (full + 64)));
    const int n_groups = (N + R - 1) / R;
    const dim3 grid(std::min((n_groups + 3) / 4, 256 * per_cu)), block(256);
#define RSD_GEMVF_CASE(P, E)                                                                                 \
    if (pro == P && epi == E) {                                                                              \
        static std::atomic<bool> raised{false};   /* per kernel instance: dynamic LDS above 64 KB must be allowed */ \
        if (!raised.load(std::memory_order_relaxed) && full > 64 * 1024) {                                                                   \
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemv_full_kernel<WT, MT, R, U, P, E>),   \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)kGemvFullLds);        \
            raised.store(true, std::memory_order_relaxed);                                                                                 \
        }                                                                                                    \
        hipLaunchKernelGGL((gemv_full_kernel<WT, MT, R, U, P, E>), grid, block, full, st, W, N, K, X, ldx,   \
                           gain, eps, Y, ldy, M);                                                            \
        return true;                                                                                         \
    }
    RSD_GEMVF_CASE(PRO_NONE, EPI_STORE)
    RSD_GEMVF_CASE(PRO_NONE, EPI_RESID)
    RSD_GEMVF_CASE(PRO_NORM, EPI_STORE)
    RSD_GEMVF_CASE(PRO_NORM, EPI_SWIGLU)
#undef RSD_GEMVF_CASE
    return false;
}

// Single activation row.  A block owns a contiguous span of rows of W (for EPI_SWIGLU the
// gate rows and the matching up rows); the span is cut into 1 KiB chunks (64 lanes x 16
// bytes of one row) and every wave streams an equal, contiguous run of chunks, so all
// waves of the launch do the same amount of work whatever N and K are.  The loop body
// has no conditional loads (chunks past the end re-read the last one and count as zero),
// which lets the compiler keep two stages of U loads in flight.  A wave finishes a row
// (or its part of one) with a lane sum into its own LDS slot; the slots are added in wave
// order at the end, so the result does not depend on timing.
template <typename WT, int NW, int U, int PRO, int EPI>
__global__ __launch_bounds__(NW * 64) void gemv_flat_kernel(const WT* __restrict__ W, int N, int K,
                                                            const float* __restrict__ X,
                                                            const WT* __restrict__ gain, float eps,
                                                            float* __restrict__ Y, uint32_t cpr_magic,
                                                            AttnParts parts) {
    constexpr int NA = (EPI == EPI_SWIGLU) ? 2 : 1;
    extern __shared__ float smem[];
    const int CPR = (K + 511) >> 9;         // chunks per row
    float* xs = smem;                       // [CPR][512], swizzled, zero beyond K
    float* red = smem + (CPR << 9);         // [NW][NA][V]
    __shared__ float red_ss[NW];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int G = gridDim.x, b = blockIdx.x;
    const int r0 = (int)((long long)b * N / G), r1 = (int)((long long)(b + 1) * N / G);
    const int V = r1 - r0;
    if (V == 0) return;
    const int C = V * CPR;
    const int c0 = (int)((long long)wave * C / NW), c1 = (int)((long long)(wave + 1) * C / NW);
    const int n_my = c1 - c0;
    const int c_last = max(c1 - 1, 0);
    const int n_stages = (n_my + U - 1) / U;
    const int k_lane = lane * 8;

    auto fetch = [&](Raw8<WT> buf[U][NA], int stage) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = min(c0 + stage * U + u, c_last);
            const int v = CPR == 1 ? c : (int)__umulhi((uint32_t)c, cpr_magic);     // c / CPR
            const int s = c - v * CPR;
            const int k = min((s << 9) + k_lane, K - 8);
#pragma unroll
            for (int a = 0; a < NA; ++a) buf[u][a].load(W + ((size_t)a * N + r0 + v) * K + k);
        }
    };
    Raw8<WT> b0[U][NA], b1[U][NA];
    fetch(b0, 0);
    fetch(b1, 1);

    float ss = 0.0f;
    for (int k = tid * 4; k < (CPR << 9); k += NW * 256) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (PRO == PRO_ATTN) {
            if (k < K) {        // head k / 128, elements k % 128 .. + 3
                const int h = k >> 7, e = k & 127, S = parts.S;
                const float* ml = parts.ml + (size_t)h * S * 2;
                const float* pa = parts.acc + (size_t)h * S * 128 + e;
                float mn = -INFINITY;
                for (int sp = 0; sp < S; ++sp) mn = fmaxf(mn, ml[sp * 2]);
                float ll = 0.0f;
                for (int sp = 0; sp < S; ++sp) {
                    const float m = ml[sp * 2];
                    const float cc = (m == -INFINITY) ? 0.0f : __expf(m - mn);
                    const float4 a = *reinterpret_cast<const float4*>(pa + (size_t)sp * 128);
                    v.x += a.x * cc; v.y += a.y * cc; v.z += a.z * cc; v.w += a.w * cc;
                    ll += ml[sp * 2 + 1] * cc;
                }
                v.x /= ll; v.y /= ll; v.z /= ll; v.w /= ll;
            }
        } else if (k < K) {
            v = *reinterpret_cast<const float4*>(X + k);
            if (PRO == PRO_NORM) {
                ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
                const WT* gp = gain + k;
                v.x *= ld1(gp); v.y *= ld1(gp + 1); v.z *= ld1(gp + 2); v.w *= ld1(gp + 3);
            }
        }
        // within each 512-float chunk the two halves of every lane's 8 values are stored 1 KiB
        // apart, so that both 16-byte LDS reads of a wave are contiguous across its lanes
        const int c = k >> 9, o = k & 511;
        *reinterpret_cast<float4*>(xs + (c << 9) + ((o >> 2) & 1) * 256 + (o >> 3) * 4) = v;
    }
    for (int i = tid; i < NW * NA * V; i += NW * 64) red[i] = 0.0f;
    if (PRO == PRO_NORM) {
        ss = wave_sum(ss);
        if (lane == 0) red_ss[wave] = ss;
    }
    __syncthreads();
    float rs = 1.0f;
    if (PRO == PRO_NORM) {
        float t = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) t += red_ss[w];
        rs = 1.0f / sqrtf(t / (float)K + eps);
    }

    float acc[NA];
#pragma unroll
    for (int a = 0; a < NA; ++a) acc[a] = 0.0f;
    auto use = [&](const Raw8<WT> buf[U][NA], int stage) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = stage * U + u;
            const int c = min(c0 + i, c_last);
            const int v = CPR == 1 ? c : (int)__umulhi((uint32_t)c, cpr_magic);     // c / CPR
            const int s = c - v * CPR;
            const float4 xa = *reinterpret_cast<const float4*>(xs + (s << 9) + lane * 4);
            const float4 xb = *reinterpret_cast<const float4*>(xs + (s << 9) + 256 + lane * 4);
            const float keep = i < n_my ? 1.0f : 0.0f;
#pragma unroll
            for (int a = 0; a < NA; ++a) {
                float w[8];
                buf[u][a].unpack(w);
                acc[a] += keep * (xa.x * w[0] + xa.y * w[1] + xa.z * w[2] + xa.w * w[3]
                                + xb.x * w[4] + xb.y * w[5] + xb.z * w[6] + xb.w * w[7]);
            }
            if (i < n_my && (s == CPR - 1 || i == n_my - 1)) {
#pragma unroll
                for (int a = 0; a < NA; ++a) {
                    const float t = wave_sum_dpp(acc[a]);
                    if (lane == 0) red[(wave * NA + a) * V + v] = t;
                    acc[a] = 0.0f;
                }
            }
        }
    };
    int s = 0;
    for (; s + 3 < n_stages; s += 2) {          // both refills are real stages
        use(b0, s);     fetch(b0, s + 2);
        use(b1, s + 1); fetch(b1, s + 3);
    }
    if (s < n_stages) {                          // at most three stages left
        use(b0, s);
        if (s + 2 < n_stages) fetch(b0, s + 2);
        if (s + 1 < n_stages) use(b1, s + 1);
        if (s + 2 < n_stages) use(b0, s + 2);
    }
    __syncthreads();
    for (int t = tid; t < V; t += NW * 64) {
        float g = 0.0f, up = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            g += red[w * NA * V + t];
            if (EPI == EPI_SWIGLU) up += red[(w * NA + NA - 1) * V + t];
        }
        g *= rs;
        float* yp = Y + r0 + t;
        if (EPI == EPI_SWIGLU) *yp = g / (1.0f + expf(-g)) * (up * rs);
        else *yp = (EPI == EPI_RESID) ? (*yp + g) : g;
    }
}

// Launch of the single-row kernel: blocks_per_cu blocks of NW waves per compute unit (fewer when
// LDS or the matrix is too small for that: a wave should still get min_chunks chunks).
template <typename WT, int NW, int U>
static bool gemv_launch_flat(hipStream_t st, int pro, int epi, const WT* W, int N, int K, const float* X,
                             const WT* gain, float eps, float* Y, int blocks_per_cu, int min_chunks,
                             AttnParts parts = AttnParts{nullptr, nullptr, 0}) {
    if (pro == PRO_SWIGLU || (K & 7) || K < 8) return false;
    if (pro == PRO_ATTN && (K & 127)) return false;
    const int NA = epi == EPI_SWIGLU ? 2 : 1;
    const int CPR = (K + 511) / 512;
    const size_t xs_bytes = (size_t)CPR * 512 * sizeof(float);
    int per_cu = blocks_per_cu;
    while (per_cu > 1 && per_cu * (xs_bytes + 4096) > 160 * 1024) --per_cu;
    int G = 256 * per_cu;
    {   // small matrices: fewer blocks, so that a wave still has min_chunks chunks
        const long long chunks = (long long)N * CPR;
        const int want = (int)std::max<long long>(1, chunks / ((long long)NW * min_chunks));
        if (want < G) G = want;
    }
    // bound the per-wave row slots to 16 KB
    while ((size_t)NW * NA * ((N + G - 1) / G) * sizeof(float) > 16 * 1024) G += 256 * per_cu;
    const int max_v = (N + G - 1) / G;
    if ((uint64_t)max_v * CPR * CPR >= (1ull << 31)) return false;      // range of the division by multiplication
    const uint32_t magic = CPR == 1 ? 0u : (uint32_t)(((1ull << 32) + CPR - 1) / CPR);    // ceil(2^32 / CPR)
    const size_t lds = xs_bytes + (size_t)NW * NA * max_v * sizeof(float);
    if (lds > kGemvFullLds) return false;
#define RSD_GEMVFLAT_CASE(P, E)                                                                              \
    if (pro == P && epi == E) {                                                                              \
        static std::atomic<bool> raised{false};                                                              \
        if (!raised.load(std::memory_order_relaxed) && lds > 64 * 1024) {                                                                    \
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemv_flat_kernel<WT, NW, U, P, E>),      \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)kGemvFullLds);        \
            raised.store(true, std::memory_order_relaxed);                                                                                 \
        }                                                                                                    \
        if (gemv_timing.start) {                                                                             \
            hipExtLaunchKernelGGL((gemv_flat_kernel<WT, NW, U, P, E>), dim3(G), dim3(NW * 64), lds, st,      \
                                  gemv_timing.start, gemv_timing.stop, 0, W, N, K, X, gain, eps, Y, magic,   \
                                  parts);                                                                    \
            gemv_timing = GemvTiming{};                                                                      \
        } else {                                                                                             \
            hipLaunchKernelGGL((gemv_flat_kernel<WT, NW, U, P, E>), dim3(G), dim3(NW * 64), lds, st, W, N,   \
                               K, X, gain, eps, Y, magic, parts);                                            \
        }                                                                                                    \
        return true;                                                                                         \
    }
    RSD_GEMVFLAT_CASE(PRO_NONE, EPI_STORE)
    RSD_GEMVFLAT_CASE(PRO_NONE, EPI_RESID)
    RSD_GEMVFLAT_CASE(PRO_NORM, EPI_STORE)
    RSD_GEMVFLAT_CASE(PRO_NORM, EPI_SWIGLU)
    RSD_GEMVFLAT_CASE(PRO_ATTN, EPI_RESID)
#undef RSD_GEMVFLAT_CASE
    return false;
}

// Fallback for activations too large for LDS: K is walked in chunks, one block per R rows.
template <typename WT, int MT, int R>
static void gemv_launch_chunked(hipStream_t st, int pro, int epi, const WT* W, int N, int K, const float* X,
                                int ldx, const WT* gain, float eps, float* Y, int ldy, int M) {
    int KC = (MT == 8 ? 1536 : 8192 / MT);   // LDS budget for the staged activations: 32 KB (48 KB for 8 rows)
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

// True when gemv_launch can fuse SwiGLU into the gate/up kernel for this shape (then the
// down projection reads the activated values with PRO_NONE).
static bool gemv_can_fuse_swiglu(int M, int K) {
    const int MT = M <= 1 ? 1 : M <= 2 ? 2 : M <= 4 ? 4 : 8;
    return (size_t)MT * K * sizeof(float) <= kGemvFullLds;
}

template <typename WT, int MT>
static void gemv_launch_mt(hipStream_t st, int pro, int epi, const WT* W, int N, int K, const float* X, int ldx,
                           const WT* gain, float eps, float* Y, int ldy, int M) {
    // rows per wave: as many as still leave every compute unit a couple of blocks; then enough
    // KiB per row and step to keep about 8 loads per lane in flight
    const int pairs = epi == EPI_SWIGLU ? 2 : 1;
    const int steps = (K / 8 + 63) / 64;          // KiB per row
    bool done = false;
    if (MT == 1) {
        // single row: equal chunk runs per wave.  Long rows (activations above 40 KB) take one block of
        // 16 waves per compute unit, so that the activations are staged once per unit; matrices of
        // 100 MB and more are cut into more blocks than are resident, which evens out the tail.
        const size_t w_bytes = (size_t)pairs * N * K * sizeof(WT);
        if ((size_t)K * sizeof(float) > 40 * 1024)
            done = gemv_launch_flat<WT, 16, 4>(st, pro, epi, W, N, K, X, gain, eps, Y, 1, 4);
        else
            done = gemv_launch_flat<WT, 8, 4>(st, pro, epi, W, N, K, X, gain, eps, Y, w_bytes >= (100u << 20) ? 3 : 2, 4);
    }
    if (!done && MT == 1) {
        int R = 8 / pairs;
        while (R > 1 && (N / R) < 2048) R >>= 1;
        int U = std::max(1, 8 / (R * pairs));
        while (U > 1 && U > steps) U >>= 1;
        if (pairs == 2) {
            if (R >= 4) done = gemv_launch_full<WT, MT, 4, 1>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
            else if (R == 2) done = gemv_launch_full<WT, MT, 2, 2>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
            else done = gemv_launch_full<WT, MT, 1, 4>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
        } else if (R == 8) done = gemv_launch_full<WT, MT, 8, 1>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
        else if (R == 4) done = U >= 2 ? gemv_launch_full<WT, MT, 4, 2>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M)
                                       : gemv_launch_full<WT, MT, 4, 1>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
        else if (R == 2) done = U >= 4 ? gemv_launch_full<WT, MT, 2, 4>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M)
                                       : gemv_launch_full<WT, MT, 2, 2>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
        else done = U >= 8 ? gemv_launch_full<WT, MT, 1, 8>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M)
                           : gemv_launch_full<WT, MT, 1, 4>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
    } else if (!done) {
        if (pairs == 2) done = gemv_launch_full<WT, MT, 2, 1>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
        else done = gemv_launch_full<WT, MT, 4, 1>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
    }
    if (!done) gemv_launch_chunked<WT, MT, 4>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
}

// Output projection of a single row straight from the attention partials: Y += W . merge(parts).
// Returns false if the shape does not fit (the caller then merges with a kernel of its own).
template <typename WT>
static bool gemv_launch_attn(hipStream_t st, const WT* W, int N, int K, AttnParts parts, float* Y) {
    if ((size_t)K * sizeof(float) > 40 * 1024) return false;
    // every block merges the whole row: one block per compute unit keeps that repeated work small
    if (K > 2048)
        return gemv_launch_flat<WT, 16, 4>(st, PRO_ATTN, EPI_RESID, W, N, K, (const float*)nullptr, (const WT*)nullptr, 0.f,
                                           Y, 1, 4, parts);
    return gemv_launch_flat<WT, 8, 4>(st, PRO_ATTN, EPI_RESID, W, N, K, (const float*)nullptr, (const WT*)nullptr, 0.f, Y,
                                      1, 4, parts);
}

// M <= 8
template <typename WT>
static void gemv_launch(hipStream_t st, int pro, int epi, const WT* W, int N, int K, const float* X, int ldx,
                        const WT* gain, float eps, float* Y, int ldy, int M) {
    if (M <= 1) gemv_launch_mt<WT, 1>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
    else if (M <= 2) gemv_launch_mt<WT, 2>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
    else if (M <= 4) gemv_launch_mt<WT, 4>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
    else gemv_launch_mt<WT, 8>(st, pro, epi, W, N, K, X, ldx, gain, eps, Y, ldy, M);
}
