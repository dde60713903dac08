// Tiled GEMMs for more than 8 activation rows (chunked prefill, large decode
// batches): Y[m][n] (+)= sum_k X[m][k] * W[n][k]; X fp32 [M][ldx], W row-major
// [N][K], Y fp32 [M][ldy].  Both operands are contiguous along K ("NT" form).
//   * fp32 weights: plain VALU tile kernel (the tiny configuration only).
//   * bf16 weights: MFMA kernel.  An fp32 activation x is staged into LDS as two
//     bf16 numbers, hi = bf16(x) and lo = bf16(x - hi), and every weight tile is
//     multiplied with both (W.hi + W.lo, fp32 accumulation): the activations keep
//     16 mantissa bits, which the bit-for-bit agreement of the bf16 KV-cache
//     entries with an exact evaluation needs; one bf16 pass would leave 8.
// Requirements checked by the caller: K % 32 == 0; N, M arbitrary.
#pragma once
#include "common.cuh"
#include "gemv.cuh"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

// ---------------------------------------------------------------- fp32 tiles
// 64x64 output tile, 16x16 threads, 4x4 outputs per thread, BK = 16.
template <int EPI>
__global__ __launch_bounds__(256) void sgemm_nt_kernel(const float* __restrict__ W, int N, int K,
                                                       const float* __restrict__ X, int ldx,
                                                       float* __restrict__ Y, int ldy, int M) {
    __shared__ float As[16][64 + 4];
    __shared__ float Bs[16][64 + 4];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        // 64 rows x 16 k = 1024 elements per operand: 4 per thread
        {
            const int row = tid >> 2, kq = (tid & 3) * 4;
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
            if (m0 + row < M) a = *reinterpret_cast<const float4*>(X + (size_t)(m0 + row) * ldx + k0 + kq);
            if (n0 + row < N) b = *reinterpret_cast<const float4*>(W + (size_t)(n0 + row) * K + k0 + kq);
            As[kq + 0][row] = a.x; As[kq + 1][row] = a.y; As[kq + 2][row] = a.z; As[kq + 3][row] = a.w;
            Bs[kq + 0][row] = b.x; Bs[kq + 1][row] = b.y; Bs[kq + 2][row] = b.z; Bs[kq + 3][row] = b.w;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n < N) {
                float* yp = Y + (size_t)m * ldy + n;
                *yp = (EPI == EPI_RESID) ? (*yp + acc[i][j]) : acc[i][j];
            }
        }
    }
}

// ---------------------------------------------------------------- bf16 MFMA
// Block tile BM x BN (64 or 128 each), K step 32, 256 threads = 2 x 2 waves.
// v_mfma_f32_32x32x16_bf16: per lane 8 consecutive-k bf16 of row (lane % 32) at
// k offset 8 * (lane / 32) for each operand; the 16 results of a lane sit at
// rows 8 * (v / 4) + 4 * (lane / 32) + v % 4, column lane % 32.
// blockIdx.z cuts K into gridDim.z slices (few-row GEMMs stream the weights and
// need more blocks than output tiles); with slices the tile is stored to
// part[z][M][N] and splitk_reduce_kernel adds the slices in a fixed order.
template <int BM, int BN, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const bf16_t* __restrict__ W, int N, int K,
                                                        const float* __restrict__ X, int ldx,
                                                        float* __restrict__ Y, int ldy, int M,
                                                        float* __restrict__ part) {
    constexpr int BK = 32, LDS_STRIDE = BK + 8;             // 80-byte rows: 16-byte aligned, conflict-free
    constexpr int WM = BM / 2, WN = BN / 2;                  // tile of one wave
    constexpr int TI = WM / 32, TJ = WN / 32;                // 32x32 MFMA tiles per wave
    __shared__ __attribute__((aligned(16))) uint16_t As[BM * LDS_STRIDE];    // hi parts
    __shared__ __attribute__((aligned(16))) uint16_t Al[BM * LDS_STRIDE];    // lo parts
    __shared__ __attribute__((aligned(16))) uint16_t Bs[BN * LDS_STRIDE];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int ksl = ((K / BK + gridDim.z - 1) / gridDim.z) * BK;             // K slice of this block
    const int k_begin = blockIdx.z * ksl, k_end = min(K, k_begin + ksl);

    f32x16_t acc[TI][TJ];
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    constexpr int A_F4 = BM * BK / 4 / 256;   // float4 loads of X per thread (2 or 4)
    constexpr int B_U4 = BN * BK / 8 / 256;   // uint4 loads of W per thread (1 or 2)
    for (int k0 = k_begin; k0 < k_end; k0 += BK) {
        float4 av[A_F4];
        uint4 bv[B_U4];
#pragma unroll
        for (int i = 0; i < A_F4; ++i) {
            const int idx = tid + i * 256, row = idx >> 3, c4 = idx & 7;
            av[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (m0 + row < M) av[i] = *reinterpret_cast<const float4*>(X + (size_t)(m0 + row) * ldx + k0 + c4 * 4);
        }
#pragma unroll
        for (int i = 0; i < B_U4; ++i) {
            const int idx = tid + i * 256, row = idx >> 2, c8 = idx & 3;
            bv[i] = make_uint4(0u, 0u, 0u, 0u);
            if (n0 + row < N) bv[i] = *reinterpret_cast<const uint4*>(W + (size_t)(n0 + row) * K + k0 + c8 * 8);
        }
        __syncthreads();          // previous tile fully consumed
#pragma unroll
        for (int i = 0; i < A_F4; ++i) {
            const int idx = tid + i * 256, row = idx >> 3, c4 = idx & 7;
            const float x[4] = {av[i].x, av[i].y, av[i].z, av[i].w};
            uint16_t hi[4], lo[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                hi[e] = f2bf(x[e]);
                lo[e] = f2bf(x[e] - bf2f(hi[e]));
            }
            uint2 p, q;
            p.x = (uint32_t)hi[0] | ((uint32_t)hi[1] << 16); p.y = (uint32_t)hi[2] | ((uint32_t)hi[3] << 16);
            q.x = (uint32_t)lo[0] | ((uint32_t)lo[1] << 16); q.y = (uint32_t)lo[2] | ((uint32_t)lo[3] << 16);
            *reinterpret_cast<uint2*>(&As[row * LDS_STRIDE + c4 * 4]) = p;
            *reinterpret_cast<uint2*>(&Al[row * LDS_STRIDE + c4 * 4]) = q;
        }
#pragma unroll
        for (int i = 0; i < B_U4; ++i) {
            const int idx = tid + i * 256, row = idx >> 2, c8 = idx & 3;
            *reinterpret_cast<uint4*>(&Bs[row * LDS_STRIDE + c8 * 8]) = bv[i];
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            bf16x8_t a[TI], al[TI], b[TJ];
#pragma unroll
            for (int i = 0; i < TI; ++i) {
                const int off = (wm * WM + i * 32 + (lane & 31)) * LDS_STRIDE + kk + (lane >> 5) * 8;
                a[i] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(&As[off]));
                al[i] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(&Al[off]));
            }
#pragma unroll
            for (int j = 0; j < TJ; ++j) {
                const uint4 r = *reinterpret_cast<const uint4*>(
                    &Bs[(wn * WN + j * 32 + (lane & 31)) * LDS_STRIDE + kk + (lane >> 5) * 8]);
                b[j] = __builtin_bit_cast(bf16x8_t, r);
            }
#pragma unroll
            for (int i = 0; i < TI; ++i)
#pragma unroll
                for (int j = 0; j < TJ; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i], b[j], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
                }
        }
    }
    const bool sliced = gridDim.z > 1;
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
            const int n = n0 + wn * WN + j * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * WM + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (m < M && n < N) {
                    if (sliced) {
                        part[((size_t)blockIdx.z * M + m) * N + n] = acc[i][j][v];
                    } else {
                        float* yp = Y + (size_t)m * ldy + n;
                        *yp = (EPI == EPI_RESID) ? (*yp + acc[i][j][v]) : acc[i][j][v];
                    }
                }
            }
        }
}

// ---------------------------------------------------------------- bf16 MFMA, few rows
// 9..64 activation rows (batched single-token decoding, short chunks): the time
// is the one pass over W.  Each wave owns 32 rows of W and streams them from HBM
// straight into MFMA operand registers (64 contiguous bytes per lane and 64-wide
// K block, two blocks ahead of the arithmetic); only the activations go through
// LDS (hi + lo bf16, double buffered), shared by the 4 waves of a block.
// Within a K block of 64 the lane of k-group g (lane / 32) holds elements
// g*32 + j*8 .. +8 for MFMA step j, for both operands: the same permutation of k
// on both sides leaves the products unchanged.
template <int MT, int EPI>     // MT: 32-row tiles of activations (1 or 2)
__global__ __launch_bounds__(256) void gemm_skinny_kernel(const bf16_t* __restrict__ W, int N, int K,
                                                          const float* __restrict__ X, int ldx,
                                                          float* __restrict__ Y, int ldy, int M,
                                                          float* __restrict__ part) {
    constexpr int BK = 64, STR = BK + 8;                 // LDS row stride in bf16 (144 bytes)
    constexpr int ROWS = 32 * MT;
    __shared__ __attribute__((aligned(16))) uint16_t Ah[2][ROWS * STR];
    __shared__ __attribute__((aligned(16))) uint16_t Al[2][ROWS * STR];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nw = blockIdx.x * 128 + wave * 32;         // first W row of this wave
    const int n_lane = min(nw + (lane & 31), N - 1), kg = lane >> 5;
    const int nkb = K / BK;
    const int per = (nkb + gridDim.z - 1) / gridDim.z;
    const int kb0 = blockIdx.z * per, kb1 = min(nkb, kb0 + per);
    const bf16_t* wp = W + (size_t)n_lane * K + kg * 32;

    f32x16_t acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;

    uint4 w0[4], w1[4], w2[4];
    auto fetch_w = [&](int kb, uint4 w[4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) w[j] = *reinterpret_cast<const uint4*>(wp + (size_t)kb * BK + j * 8);
    };
    constexpr int XF4 = ROWS * BK / 4 / 256;             // float4 of X per thread and K block (2 or 4)
    float4 xv[XF4];
    auto fetch_x = [&](int kb) {
#pragma unroll
        for (int i = 0; i < XF4; ++i) {
            const int idx = tid + i * 256, row = idx >> 4, c4 = idx & 15;
            xv[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < M) xv[i] = *reinterpret_cast<const float4*>(X + (size_t)row * ldx + (size_t)kb * BK + c4 * 4);
        }
    };
    auto stage_x = [&](int buf) {
#pragma unroll
        for (int i = 0; i < XF4; ++i) {
            const int idx = tid + i * 256, row = idx >> 4, c4 = idx & 15;
            const float x[4] = {xv[i].x, xv[i].y, xv[i].z, xv[i].w};
            uint16_t hi[4], lo[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) { hi[e] = f2bf(x[e]); lo[e] = f2bf(x[e] - bf2f(hi[e])); }
            *reinterpret_cast<uint2*>(&Ah[buf][row * STR + c4 * 4]) =
                make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
            *reinterpret_cast<uint2*>(&Al[buf][row * STR + c4 * 4]) =
                make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16));
        }
    };
    if (kb0 < kb1) { fetch_w(kb0, w0); fetch_x(kb0); }
    if (kb0 + 1 < kb1) fetch_w(kb0 + 1, w1);
    if (kb0 < kb1) stage_x(0);
    __syncthreads();
    for (int kb = kb0; kb < kb1; ++kb) {
        const int buf = (kb - kb0) & 1;
        if (kb + 2 < kb1) fetch_w(kb + 2, w2);
        if (kb + 1 < kb1) fetch_x(kb + 1);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bf16x8_t b = __builtin_bit_cast(bf16x8_t, w0[j]);
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                const int off = (t * 32 + (lane & 31)) * STR + kg * 32 + j * 8;
                const bf16x8_t ah = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(&Ah[buf][off]));
                const bf16x8_t al = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(&Al[buf][off]));
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, b, acc[t], 0, 0, 0);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, b, acc[t], 0, 0, 0);
            }
        }
        if (kb + 1 < kb1) stage_x(buf ^ 1);               // the other buffer was last read one iteration ago
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 4; ++j) { w0[j] = w1[j]; w1[j] = w2[j]; }
    }
    const bool sliced = gridDim.z > 1;
    const int n = nw + (lane & 31);
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = t * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            if (m < M && n < N) {
                if (sliced) part[((size_t)blockIdx.z * M + m) * N + n] = acc[t][v];
                else {
                    float* yp = Y + (size_t)m * ldy + n;
                    *yp = (EPI == EPI_RESID) ? (*yp + acc[t][v]) : acc[t][v];
                }
            }
        }
}

// Y[m][n] (+)= sum_z part[z][m][n], slices added in ascending z
template <int EPI>
__global__ void splitk_reduce_kernel(const float* __restrict__ part, int KS, int M, int N, float* __restrict__ Y, int ldy) {
    const size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i >= (size_t)M * N) return;
    const size_t m = i / N, n = i - m * N;           // N is a multiple of 4
    float4 a = *reinterpret_cast<const float4*>(part + i);
    for (int z = 1; z < KS; ++z) {
        const float4 b = *reinterpret_cast<const float4*>(part + (size_t)z * M * N + i);
        a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    float4* yp = reinterpret_cast<float4*>(Y + m * ldy + n);
    if (EPI == EPI_RESID) { const float4 y = *yp; a.x += y.x; a.y += y.y; a.z += y.z; a.w += y.w; }
    *yp = a;
}

// ---------------------------------------------------------------- dispatch
static void gemm_launch(hipStream_t st, int epi, const float* W, int N, int K, const float* X, int ldx,
                        float* Y, int ldy, int M, float* part, size_t part_floats) {
    (void)part; (void)part_floats;
    if (M <= 8) { gemv_launch<float>(st, PRO_NONE, epi, W, N, K, X, ldx, nullptr, 0.f, Y, ldy, M); return; }
    const dim3 grid((N + 63) / 64, (M + 63) / 64), block(256);
    if (epi == EPI_RESID) hipLaunchKernelGGL((sgemm_nt_kernel<EPI_RESID>), grid, block, 0, st, W, N, K, X, ldx, Y, ldy, M);
    else                  hipLaunchKernelGGL((sgemm_nt_kernel<EPI_STORE>), grid, block, 0, st, W, N, K, X, ldx, Y, ldy, M);
}

template <int BM, int BN>
static void gemm_bf16_launch(hipStream_t st, int epi, const bf16_t* W, int N, int K, const float* X, int ldx,
                             float* Y, int ldy, int M, float* part, int KS) {
    const dim3 grid((N + BN - 1) / BN, (M + BM - 1) / BM, KS), block(256);
    if (epi == EPI_RESID) hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, EPI_RESID>), grid, block, 0, st, W, N, K, X, ldx, Y, ldy, M, part);
    else                  hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, EPI_STORE>), grid, block, 0, st, W, N, K, X, ldx, Y, ldy, M, part);
    if (KS > 1) {
        const unsigned nb = (unsigned)(((size_t)M * N / 4 + 255) / 256);
        if (epi == EPI_RESID) hipLaunchKernelGGL((splitk_reduce_kernel<EPI_RESID>), dim3(nb), block, 0, st, part, KS, M, N, Y, ldy);
        else                  hipLaunchKernelGGL((splitk_reduce_kernel<EPI_STORE>), dim3(nb), block, 0, st, part, KS, M, N, Y, ldy);
    }
}

static void gemm_launch(hipStream_t st, int epi, const bf16_t* W, int N, int K, const float* X, int ldx,
                        float* Y, int ldy, int M, float* part, size_t part_floats) {
    if (M <= 8) { gemv_launch<bf16_t>(st, PRO_NONE, epi, W, N, K, X, ldx, nullptr, 0.f, Y, ldy, M); return; }
    if (M <= 64 && K % 64 == 0) {
        // weight-streaming kernel: 128 rows of W per block, K slices until about 3 blocks per compute unit
        const int nb = (N + 127) / 128;
        int ks = 1;
        while (ks < 32 && nb * ks < 768 && K / (ks * 2) >= 256 && (size_t)(ks * 2) * M * N <= part_floats) ks *= 2;
        if (!part) ks = 1;
        const dim3 grid(nb, 1, ks), block(256);
#define RSD_SK_CASE(T, E) hipLaunchKernelGGL((gemm_skinny_kernel<T, E>), grid, block, 0, st, W, N, K, X, ldx, Y, ldy, M, part)
        if (M <= 32) { if (epi == EPI_RESID) RSD_SK_CASE(1, EPI_RESID); else RSD_SK_CASE(1, EPI_STORE); }
        else         { if (epi == EPI_RESID) RSD_SK_CASE(2, EPI_RESID); else RSD_SK_CASE(2, EPI_STORE); }
#undef RSD_SK_CASE
        if (ks > 1) {
            const unsigned rb = (unsigned)(((size_t)M * N / 4 + 255) / 256);
            if (epi == EPI_RESID) hipLaunchKernelGGL((splitk_reduce_kernel<EPI_RESID>), dim3(rb), block, 0, st, part, ks, M, N, Y, ldy);
            else                  hipLaunchKernelGGL((splitk_reduce_kernel<EPI_STORE>), dim3(rb), block, 0, st, part, ks, M, N, Y, ldy);
        }
        return;
    }
    // Tiles: 64 rows of activations when there are few; narrow weight tiles and K slices until
    // about two blocks per compute unit exist (these shapes are bound by streaming W once).
    const int bm = M <= 64 ? 64 : 128;
    const int tm = (M + bm - 1) / bm;
    int bn = 128;
    if (((N + 127) / 128) * tm < 512) bn = 64;
    const int tiles = ((N + bn - 1) / bn) * tm;
    int ks = 1;
    while (ks < 16 && tiles * ks < 512 && K / (ks * 2) >= 512 && (size_t)(ks * 2) * M * N <= part_floats) ks *= 2;
    if (!part) ks = 1;
    if (bm == 64) {
        if (bn == 64) gemm_bf16_launch<64, 64>(st, epi, W, N, K, X, ldx, Y, ldy, M, part, ks);
        else          gemm_bf16_launch<64, 128>(st, epi, W, N, K, X, ldx, Y, ldy, M, part, ks);
    } else {
        if (bn == 64) gemm_bf16_launch<128, 64>(st, epi, W, N, K, X, ldx, Y, ldy, M, part, ks);
        else          gemm_bf16_launch<128, 128>(st, epi, W, N, K, X, ldx, Y, ldy, M, part, ks);
    }
}
