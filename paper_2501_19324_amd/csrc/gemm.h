// Tiled GEMMs for two or more activation rows (chunked prefill, batched decode,
// verification passes): Y[m][n] (+)= sum_k X[m][k] * W[n][k]; X fp32 [M][ldx], W row-major
// [N][K], Y fp32 [M][ldy].  Both operands are contiguous along K ("NT" form).
//   * fp32 weights: plain VALU tile kernel (the tiny configuration only).
//   * bf16 weights: MFMA kernels.  An fp32 activation x enters as two bf16 numbers,
//     hi = bf16(x) and lo = bf16(x - hi) (split_rows_kernel, or the producing kernel
//     writes the halves itself), and every weight tile is multiplied with both
//     (W.hi + W.lo, fp32 accumulation): the activations keep 16 mantissa bits, which
//     the bit-for-bit agreement of the bf16 KV-cache entries with an exact evaluation
//     needs; one bf16 pass would leave 8.  2..64 rows: weight-streaming
//     gemm_rows_kernel (gemm_rows64_kernel for small matrices); more rows: 256 x 256
//     or 128 x 256 tiles, gemm_tile_kernel.
// Requirements checked by the caller: K % 64 == 0; N, M arbitrary.
#pragma once
#include <algorithm>
#include <atomic>
#include "common.h"
#include "gemv.h"

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

// ---------------------------------------------------------------- bf16 MFMA, 2..64 rows, pre-split activations
// The activations arrive as two bf16 matrices Xh + Xl = x (hi and lo halves, [MT*32][K]; rows beyond M
// may hold anything: a row of x only ever meets its own row of the result).  A block of eight waves owns
// 256 rows of W and one K slice.  Every wave reads its 32 rows of W in whole 128-byte lines (8 lanes per
// row), two K blocks of 64 ahead in registers, and passes them through a private LDS tile into the MFMA
// operand layout (a lane of an MFMA operand holds 16 bytes of ONE row, so loading operands directly would
// touch every line with four separate instructions).  The activation tile of a K block (hi and lo) is
// copied as it is into LDS, double buffered, and shared by the eight waves.  LDS tiles are [row][64 k]
// with the eight 16-byte chunks of a row permuted by (row / 2) % 8, which makes both the line-wise
// writes and the operand reads conflict-free without padding.  No load in the loop is conditional
// (addresses past the end are clamped and never used), so the loads stay in flight across iterations.
// Partial results go to part[z][m][n]; a finish kernel adds the slices and applies the epilogue.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));    // native vector: stays in registers across LDS stores

// 16 bytes of a weight matrix that is read exactly once per launch: marked non-temporal, so that the stream of
// weights does not push the activation tiles (re-read by every block) out of L2
#ifndef RSD_W_NT
#define RSD_W_NT 1
#endif
__device__ __forceinline__ u32x4_t load_w16(const bf16_t* p) {
#if RSD_W_NT
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
#else
    return *reinterpret_cast<const u32x4_t*>(p);
#endif
}

// Thread blocks are handed to the eight XCDs round-robin by their linear index, and every XCD has an L2 of
// its own.  Blocks of one K slice read the same slice of the activations, so a K-sliced launch is renumbered:
// XCD k takes the logical indices [start(k), start(k + 1)), i.e. consecutive row blocks of few K slices, and
// fetches only those slices of the activations instead of all of them (7B down projection at 64 rows: the
// launch fetched 181 MB for 136 MB of weights, the 4.85 MB of activation halves once per XCD; 34.2 -> 32.1 us
// renumbered).  Done only where the activations weigh at least a tenth of the weights when fetched eight times
// (32 M >= 0.2 N): launches with small activations lose a little instead (72B output projection at 16 rows:
// 24.8 -> 26.9 us).  Results do not depend on the numbering.
__device__ __forceinline__ int xcd_major(int id, int nb, int M, int N) {
    if (160 * M < N) return id;
    constexpr int X = 8;
    const int k = id % X, j = id / X, q = nb / X, r = nb % X;
    return k * q + min(k, r) + j;
}

template <int MT>
__global__ __launch_bounds__(512, 2) void gemm_rows_kernel(const bf16_t* __restrict__ W, int N, int K,
                                                           const uint16_t* __restrict__ Xh,
                                                           const uint16_t* __restrict__ Xl,
                                                           float* __restrict__ part, int M) {
    constexpr int BK = 64, NWV = 8;
    constexpr int ROWS = 32 * MT;
    __shared__ __attribute__((aligned(16))) uint16_t Ah[2][ROWS * BK];
    __shared__ __attribute__((aligned(16))) uint16_t Al[2][ROWS * BK];
    __shared__ __attribute__((aligned(16))) uint16_t Ws[NWV][32 * BK];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lin = xcd_major(blockIdx.x + gridDim.x * blockIdx.y, gridDim.x * gridDim.y, M, N);
    const int bx = lin % gridDim.x, by = lin / gridDim.x;     // row block, K slice
    const int nw = bx * (32 * NWV) + wave * 32;  // first W row of this wave
    const int kg = lane >> 5, l32 = lane & 31;
    const int nkb = K / BK;
    const int per = (nkb + gridDim.y - 1) / gridDim.y;
    const int kb0 = by * per, kb1 = min(nkb, kb0 + per);
    const int nk = kb1 - kb0;                            // K blocks of this slice (may be <= 0)
    const int kb_last = max(kb1 - 1, 0);
    // loads: lane -> row lane / 8 (+ 8 p), 16-byte chunk lane % 8 of the row's 128 bytes
    const int lrow = lane >> 3, lchunk = lane & 7;
    const bf16_t* wr0 = W + (size_t)min(nw + lrow, N - 1) * K + lchunk * 8;
    const bf16_t* wr1 = W + (size_t)min(nw + lrow + 8, N - 1) * K + lchunk * 8;
    const bf16_t* wr2 = W + (size_t)min(nw + lrow + 16, N - 1) * K + lchunk * 8;
    const bf16_t* wr3 = W + (size_t)min(nw + lrow + 24, N - 1) * K + lchunk * 8;
    uint16_t* ws = Ws[wave];
    // LDS offset (in bf16) of chunk c of row r
    auto sw = [](int r, int c) { return r * BK + ((c ^ ((r >> 1) & 7)) << 3); };
    const int ws_st0 = sw(lrow, lchunk), ws_st1 = sw(lrow + 8, lchunk), ws_st2 = sw(lrow + 16, lchunk), ws_st3 = sw(lrow + 24, lchunk);
    // activation tile: MT = 2: thread -> (row tid / 8, chunk tid % 8) of both halves; MT = 1: threads 0..255 the hi half, the rest lo
    const int xrow = (MT == 2) ? (tid >> 3) : ((tid & 255) >> 3);
    const int xsrc = min(xrow, M - 1);      // tile rows beyond M are never used: they repeat row M - 1 instead of fetching more of L2
    const uint16_t* xp0 = ((MT == 2 || tid < 256) ? Xh : Xl) + (size_t)xsrc * K + lchunk * 8;
    const uint16_t* xp1 = Xl + (size_t)xsrc * K + lchunk * 8;      // MT = 2 only
    const int x_st = sw(xrow, lchunk);

    f32x16_t acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;

    // register sets named member by member (arrays indexed in loops end up in scratch memory)
    struct WRegs { u32x4_t w0, w1, w2, w3; };
    WRegs wa, wb;
    u32x4_t x0, x1;
#define RSD_FETCH_W(kb, R)                                                                       \
    {                                                                                            \
        const size_t k0_ = (size_t)min((kb), kb_last) * BK;                                      \
        R.w0 = load_w16(wr0 + k0_);                                     \
        R.w1 = load_w16(wr1 + k0_);                                     \
        R.w2 = load_w16(wr2 + k0_);                                     \
        R.w3 = load_w16(wr3 + k0_);                                     \
    }
#define RSD_FETCH_X(kb)                                                                          \
    {                                                                                            \
        const size_t k0_ = (size_t)min((kb), kb_last) * BK;                                      \
        x0 = *reinterpret_cast<const u32x4_t*>(xp0 + k0_);                                       \
        if (MT == 2) x1 = *reinterpret_cast<const u32x4_t*>(xp1 + k0_);                          \
    }
#define RSD_STAGE_W(R)                                                                           \
    {                                                                                            \
        *reinterpret_cast<u32x4_t*>(ws + ws_st0) = R.w0;                                         \
        *reinterpret_cast<u32x4_t*>(ws + ws_st1) = R.w1;                                         \
        *reinterpret_cast<u32x4_t*>(ws + ws_st2) = R.w2;                                         \
        *reinterpret_cast<u32x4_t*>(ws + ws_st3) = R.w3;                                         \
    }
#define RSD_STAGE_X(buf)                                                                         \
    {                                                                                            \
        if (MT == 2) {                                                                           \
            *reinterpret_cast<u32x4_t*>(&Ah[(buf)][x_st]) = x0;                                  \
            *reinterpret_cast<u32x4_t*>(&Al[(buf)][x_st]) = x1;                                  \
        } else {                                                                                 \
            *reinterpret_cast<u32x4_t*>((tid < 256 ? &Ah[(buf)][0] : &Al[(buf)][0]) + x_st) = x0; \
        }                                                                                        \
    }
    // one K block: W tile of this wave in ws, activation tile in LDS buffer `buf`
#define RSD_COMPUTE(buf)                                                                         \
    {                                                                                            \
        _Pragma("unroll") for (int j_ = 0; j_ < 4; ++j_) {                                       \
            const bf16x8_t b_ = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(ws + sw(l32, kg * 4 + j_))); \
            _Pragma("unroll") for (int t_ = 0; t_ < MT; ++t_) {                                  \
                const int off_ = sw(t_ * 32 + l32, kg * 4 + j_);                                 \
                const bf16x8_t ah_ = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(&Ah[(buf)][off_])); \
                const bf16x8_t al_ = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(&Al[(buf)][off_])); \
                acc[t_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al_, b_, acc[t_], 0, 0, 0);    \
                acc[t_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah_, b_, acc[t_], 0, 0, 0);    \
            }                                                                                    \
        }                                                                                        \
    }
    // step i: the activation tile of block i + 1 moves into the LDS buffer that block i - 1 has left and
    // its registers at once take the request of block i + 2; block i is multiplied while W of block i + 2
    // is requested into the free set F; then W of block i + 1 (set S) replaces the wave's W tile
#define RSD_STEP(i_step, F, S)                                                                   \
    {                                                                                            \
        RSD_STAGE_X(((i_step) + 1) & 1)                                                          \
        RSD_FETCH_X(kb0 + (i_step) + 2)                                                          \
        RSD_FETCH_W(kb0 + (i_step) + 2, F)                                                       \
        RSD_COMPUTE((i_step) & 1)                                                                \
        RSD_STAGE_W(S)                                                                           \
        __syncthreads();                                                                         \
    }
    RSD_FETCH_W(kb0, wa)
    RSD_FETCH_X(kb0)
    RSD_FETCH_W(kb0 + 1, wb)
    RSD_STAGE_W(wa)
    RSD_STAGE_X(0)
    RSD_FETCH_X(kb0 + 1)
    __syncthreads();
    int i = 0;
    for (; i + 1 < nk; i += 2) {
        RSD_STEP(i, wa, wb)
        RSD_STEP(i + 1, wb, wa)
    }
    if (i < nk) RSD_STEP(i, wa, wb)
#undef RSD_STEP
#undef RSD_COMPUTE
#undef RSD_STAGE_W
#undef RSD_STAGE_X
#undef RSD_FETCH_W
#undef RSD_FETCH_X

    const int n = nw + l32;
    if (n < N) {
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = t * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (m < M) part[((size_t)by * ROWS + m) * N + n] = acc[t][v];      // rows beyond M are never read
            }
    }
}

// The same kernel with the work dealt evenly: the (256-row block of W) x (K block of 64) units of the product,
// numbered row block by row block, are cut into gridDim.x equal runs, one per thread block, whatever N and K
// are.  A run crosses at most a few row blocks; each stretch inside one row block is computed like a K slice
// above and written as a partial tile.  The partial tiles of row block rb come from the consecutive thread
// blocks first(rb) .. last(rb); thread block g writes its tile of rb into slice z = g - first(rb), so the slices
// of a row block are in ascending K order and the finish kernels add them in that fixed order.  D = 2 or 4 W
// register sets (K blocks requested ahead of their use).
struct SkGeom {
    int nkb;            // K blocks of 64
    int units;          // row blocks x K blocks
    int G;              // thread blocks the units are dealt to
    int zmax;           // most partial tiles any row block receives (slices of the partial buffer)
};
__host__ __device__ __forceinline__ long long sk_start(const SkGeom& g, int b) { return (long long)b * g.units / g.G; }
// first / last thread block whose run holds units of row block rb
__host__ __device__ __forceinline__ int sk_first(const SkGeom& g, int rb) {
    const long long x = (long long)rb * g.nkb;                       // largest b with start(b) <= x
    return (int)(((x + 1) * g.G + g.units - 1) / g.units) - 1;
}
__host__ __device__ __forceinline__ int sk_last(const SkGeom& g, int rb) {
    const long long y = (long long)(rb + 1) * g.nkb;                 // largest b with start(b) < y
    return (int)((y * g.G + g.units - 1) / g.units) - 1;
}

template <int MT, int D>
__global__ __launch_bounds__(512, D == 2 ? 2 : 1) void gemm_rows_sk_kernel(const bf16_t* __restrict__ W, int N, int K,
                                                                        const uint16_t* __restrict__ Xh,
                                                                        const uint16_t* __restrict__ Xl,
                                                                        float* __restrict__ part, SkGeom geo, int M) {
    constexpr int BK = 64, NWV = 8;
    constexpr int ROWS = 32 * MT;
    __shared__ __attribute__((aligned(16))) uint16_t Ah[2][ROWS * BK];
    __shared__ __attribute__((aligned(16))) uint16_t Al[2][ROWS * BK];
    __shared__ __attribute__((aligned(16))) uint16_t Ws[NWV][32 * BK];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kg = lane >> 5, l32 = lane & 31;
    const int lrow = lane >> 3, lchunk = lane & 7;
    uint16_t* ws = Ws[wave];
    auto sw = [](int r, int c) { return r * BK + ((c ^ ((r >> 1) & 7)) << 3); };
    const int ws_st0 = sw(lrow, lchunk), ws_st1 = sw(lrow + 8, lchunk), ws_st2 = sw(lrow + 16, lchunk), ws_st3 = sw(lrow + 24, lchunk);
    const int xrow = (MT == 2) ? (tid >> 3) : ((tid & 255) >> 3);
    const int xsrc = min(xrow, M - 1);      // tile rows beyond M are never used: they repeat row M - 1 instead of fetching more of L2
    const uint16_t* xp0 = ((MT == 2 || tid < 256) ? Xh : Xl) + (size_t)xsrc * K + lchunk * 8;
    const uint16_t* xp1 = Xl + (size_t)xsrc * K + lchunk * 8;      // MT = 2 only
    const int x_st = sw(xrow, lchunk);

    long long u = sk_start(geo, blockIdx.x);
    const long long u_end = sk_start(geo, blockIdx.x + 1);
    while (u < u_end) {
        const int rb = (int)(u / geo.nkb);
        const int kb0 = (int)(u - (long long)rb * geo.nkb);
        const int kb1 = (int)min((long long)geo.nkb, kb0 + (u_end - u));
        const int nk = kb1 - kb0, kb_last = kb1 - 1;
        u += nk;
        const int nw = rb * (32 * NWV) + wave * 32;      // first W row of this wave
        const bf16_t* wr0 = W + (size_t)min(nw + lrow, N - 1) * K + lchunk * 8;
        const bf16_t* wr1 = W + (size_t)min(nw + lrow + 8, N - 1) * K + lchunk * 8;
        const bf16_t* wr2 = W + (size_t)min(nw + lrow + 16, N - 1) * K + lchunk * 8;
        const bf16_t* wr3 = W + (size_t)min(nw + lrow + 24, N - 1) * K + lchunk * 8;

        f32x16_t acc[MT];
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;

        struct WRegs { u32x4_t w0, w1, w2, w3; };
        WRegs wa, wb, wc, wd;
        u32x4_t x0, x1;
#define SK_FETCH_W(kb, R)                                                                        \
    {                                                                                            \
        const size_t k0_ = (size_t)min((kb), kb_last) * BK;                                      \
        R.w0 = load_w16(wr0 + k0_);                                     \
        R.w1 = load_w16(wr1 + k0_);                                     \
        R.w2 = load_w16(wr2 + k0_);                                     \
        R.w3 = load_w16(wr3 + k0_);                                     \
    }
#define SK_FETCH_X(kb)                                                                           \
    {                                                                                            \
        const size_t k0_ = (size_t)min((kb), kb_last) * BK;                                      \
        x0 = *reinterpret_cast<const u32x4_t*>(xp0 + k0_);                                       \
        if (MT == 2) x1 = *reinterpret_cast<const u32x4_t*>(xp1 + k0_);                          \
    }
#define SK_STAGE_W(R)                                                                            \
    {                                                                                            \
        *reinterpret_cast<u32x4_t*>(ws + ws_st0) = R.w0;                                         \
        *reinterpret_cast<u32x4_t*>(ws + ws_st1) = R.w1;                                         \
        *reinterpret_cast<u32x4_t*>(ws + ws_st2) = R.w2;                                         \
        *reinterpret_cast<u32x4_t*>(ws + ws_st3) = R.w3;                                         \
    }
#define SK_STAGE_X(buf)                                                                          \
    {                                                                                            \
        if (MT == 2) {                                                                           \
            *reinterpret_cast<u32x4_t*>(&Ah[(buf)][x_st]) = x0;                                  \
            *reinterpret_cast<u32x4_t*>(&Al[(buf)][x_st]) = x1;                                  \
        } else {                                                                                 \
            *reinterpret_cast<u32x4_t*>((tid < 256 ? &Ah[(buf)][0] : &Al[(buf)][0]) + x_st) = x0; \
        }                                                                                        \
    }
#define SK_COMPUTE(buf)                                                                          \
    {                                                                                            \
        _Pragma("unroll") for (int j_ = 0; j_ < 4; ++j_) {                                       \
            const bf16x8_t b_ = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(ws + sw(l32, kg * 4 + j_))); \
            _Pragma("unroll") for (int t_ = 0; t_ < MT; ++t_) {                                  \
                const int off_ = sw(t_ * 32 + l32, kg * 4 + j_);                                 \
                const bf16x8_t ah_ = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(&Ah[(buf)][off_])); \
                const bf16x8_t al_ = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(&Al[(buf)][off_])); \
                acc[t_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al_, b_, acc[t_], 0, 0, 0);    \
                acc[t_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah_, b_, acc[t_], 0, 0, 0);    \
            }                                                                                    \
        }                                                                                        \
    }
        // step i: the activation tile of block i + 1 moves into the LDS buffer that block i - 1 has left and its
        // registers take the request of block i + 2; W of block i + D is requested into the set F that block i
        // came from; block i is multiplied; W of block i + 1 (set S) replaces the wave's W tile
#define SK_STEP(i_step, F, S)                                                                    \
    {                                                                                            \
        SK_STAGE_X(((i_step) + 1) & 1)                                                           \
        SK_FETCH_X(kb0 + (i_step) + 2)                                                           \
        SK_FETCH_W(kb0 + (i_step) + D, F)                                                        \
        SK_COMPUTE((i_step) & 1)                                                                 \
        SK_STAGE_W(S)                                                                            \
        __syncthreads();                                                                         \
    }
        SK_FETCH_W(kb0, wa)
        SK_FETCH_X(kb0)
        SK_FETCH_W(kb0 + 1, wb)
        if (D == 4) {
            SK_FETCH_W(kb0 + 2, wc)
            SK_FETCH_W(kb0 + 3, wd)
        }
        SK_STAGE_W(wa)
        SK_STAGE_X(0)
        SK_FETCH_X(kb0 + 1)
        __syncthreads();
        int i = 0;
        if (D == 2) {
            for (; i + 1 < nk; i += 2) {
                SK_STEP(i, wa, wb)
                SK_STEP(i + 1, wb, wa)
            }
            if (i < nk) SK_STEP(i, wa, wb)
        } else {
            for (; i + 3 < nk; i += 4) {
                SK_STEP(i, wa, wb)
                SK_STEP(i + 1, wb, wc)
                SK_STEP(i + 2, wc, wd)
                SK_STEP(i + 3, wd, wa)
            }
            if (i < nk) { SK_STEP(i, wa, wb) ++i; }
            if (i < nk) { SK_STEP(i, wb, wc) ++i; }
            if (i < nk) { SK_STEP(i, wc, wd) }
        }
#undef SK_STEP
#undef SK_COMPUTE
#undef SK_STAGE_W
#undef SK_STAGE_X
#undef SK_FETCH_W
#undef SK_FETCH_X
        const int z = (int)blockIdx.x - sk_first(geo, rb);
        const int n = nw + l32;
        if (n < N) {
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = t * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                    if (m < M) part[((size_t)z * ROWS + m) * N + n] = acc[t][v];
                }
        }
    }
}

// The same product for small weight matrices (attention projections, the draft's MLP): with 256 rows of W
// per block such a matrix gives few blocks, the K slices needed to fill the chip get short (two K blocks
// for the 7B output projection) and their partial results weigh as much as the weights.  Here a block of
// eight waves owns 64 rows of W and one K slice; the W tile and the activation tile of a K block are
// shared through LDS (double buffered; W requested four K blocks ahead), the waves divide the
// 64 x ROWS x 64 product of a K block among themselves by (W half, activation half, K part) and add their
// K parts in a fixed order through LDS at the end.  Same partial-result layout and finish kernels.
// Measured at 64 rows (kernel alone, against the 256-row kernel): 7B output projection 17.0 -> 11.7 us,
// 7B QKV 16.7 -> 14.1, 1.5B down 16.4 -> 13.6, 1.5B QKV 7.8 -> 4.8; large matrices (7B down) lose.
template <int MT>
__global__ __launch_bounds__(512, 2) void gemm_rows64_kernel(const bf16_t* __restrict__ W, int N, int K,
                                                             const uint16_t* __restrict__ Xh,
                                                             const uint16_t* __restrict__ Xl,
                                                             float* __restrict__ part, int M) {
    constexpr int BK = 64, ROWS = 32 * MT, KH = 4 / MT, JS = 4 / KH;   // K parts per K block; operand steps per wave
    constexpr int WS_E = 64 * BK, XS_E = ROWS * BK;
    __shared__ __attribute__((aligned(16))) uint16_t smem[2 * WS_E + 4 * XS_E];
    uint16_t* Ws = smem;                       // [2][64 * 64]
    uint16_t* Ah = smem + 2 * WS_E;            // [2][ROWS * 64]
    uint16_t* Al = Ah + 2 * XS_E;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wi = wave & 1;                                   // W rows wi * 32 ..
    const int xj = (MT == 2) ? ((wave >> 1) & 1) : 0;          // activation rows xj * 32 ..
    const int kh = (MT == 2) ? (wave >> 2) : (wave >> 1);      // K part
    const int kg = lane >> 5, l32 = lane & 31;
    const int lin = xcd_major(blockIdx.x + gridDim.x * blockIdx.y, gridDim.x * gridDim.y, M, N);
    const int bx = lin % gridDim.x, by = lin / gridDim.x;     // row block, K slice
    const int n0 = bx * 64;
    const int nkb = K / BK;
    const int per = (nkb + gridDim.y - 1) / gridDim.y;
    const int kb0 = by * per, kb1 = min(nkb, kb0 + per);
    const int nk = kb1 - kb0;
    const int kb_last = max(kb1 - 1, 0);
    auto sw = [](int r, int c) { return r * BK + ((c ^ ((r >> 1) & 7)) << 3); };
    // copies: thread -> 16-byte chunk tid % 8 of row tid / 8 of the W tile; the same of the activation halves
    const int lrow = tid >> 3, lchunk = tid & 7;
    const bf16_t* wr = W + (size_t)min(n0 + lrow, N - 1) * K + lchunk * 8;
    const int w_st = sw(lrow, lchunk);
    const int xrow = (MT == 2) ? lrow : ((tid & 255) >> 3);
    const int xsrc = min(xrow, M - 1);      // as above: rows beyond M repeat row M - 1
    const uint16_t* xp0 = ((MT == 2 || tid < 256) ? Xh : Xl) + (size_t)xsrc * K + lchunk * 8;
    const uint16_t* xp1 = Xl + (size_t)xsrc * K + lchunk * 8;      // MT = 2 only
    const int x_st = sw(xrow, lchunk);

    f32x16_t acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    u32x4_t w0, w1, w2, w3, x0, x1;       // W: four K blocks requested ahead; activations (L2-resident): one
#define R64_FETCH_W(kb, R) { R = load_w16(wr + (size_t)min((kb), kb_last) * BK); }
#define R64_FETCH_X(kb)                                                                          \
    {                                                                                            \
        const size_t k0_ = (size_t)min((kb), kb_last) * BK;                                      \
        x0 = *reinterpret_cast<const u32x4_t*>(xp0 + k0_);                                       \
        if (MT == 2) x1 = *reinterpret_cast<const u32x4_t*>(xp1 + k0_);                          \
    }
#define R64_STAGE(buf, R)                                                                        \
    {                                                                                            \
        *reinterpret_cast<u32x4_t*>(Ws + (buf) * WS_E + w_st) = R;                               \
        if (MT == 2) {                                                                           \
            *reinterpret_cast<u32x4_t*>(Ah + (buf) * XS_E + x_st) = x0;                          \
            *reinterpret_cast<u32x4_t*>(Al + (buf) * XS_E + x_st) = x1;                          \
        } else {                                                                                 \
            *reinterpret_cast<u32x4_t*>((tid < 256 ? Ah : Al) + (buf) * XS_E + x_st) = x0;       \
        }                                                                                        \
    }
#define R64_COMPUTE(buf)                                                                         \
    {                                                                                            \
        _Pragma("unroll") for (int s_ = 0; s_ < JS; ++s_) {                                      \
            const int c_ = kg * 4 + kh * JS + s_;                                                \
            const bf16x8_t b_ = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(Ws + (buf) * WS_E + sw(wi * 32 + l32, c_))); \
            const int off_ = sw(xj * 32 + l32, c_);                                              \
            const bf16x8_t ah_ = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(Ah + (buf) * XS_E + off_)); \
            const bf16x8_t al_ = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(Al + (buf) * XS_E + off_)); \
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al_, b_, acc, 0, 0, 0);                \
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah_, b_, acc, 0, 0, 0);                \
        }                                                                                        \
    }
    // step i: block i + 1 (W in set S, activations in x0/x1) moves into the LDS buffer block i - 1 has
    // left; S at once takes the request of W block i + 5 and x0/x1 that of activation block i + 2; block i
    // is multiplied
#define R64_STEP(i_step, S)                                                                      \
    {                                                                                            \
        R64_STAGE(((i_step) + 1) & 1, S)                                                         \
        R64_FETCH_W(kb0 + (i_step) + 5, S)                                                       \
        R64_FETCH_X(kb0 + (i_step) + 2)                                                          \
        R64_COMPUTE((i_step) & 1)                                                                \
        __syncthreads();                                                                         \
    }
    R64_FETCH_W(kb0, w0)
    R64_FETCH_X(kb0)
    R64_FETCH_W(kb0 + 1, w1)
    R64_FETCH_W(kb0 + 2, w2)
    R64_FETCH_W(kb0 + 3, w3)
    R64_STAGE(0, w0)
    R64_FETCH_W(kb0 + 4, w0)
    R64_FETCH_X(kb0 + 1)
    __syncthreads();
    int i = 0;
    for (; i + 3 < nk; i += 4) {
        R64_STEP(i, w1)
        R64_STEP(i + 1, w2)
        R64_STEP(i + 2, w3)
        R64_STEP(i + 3, w0)
    }
    if (i < nk) { R64_STEP(i, w1) ++i; }
    if (i < nk) { R64_STEP(i, w2) ++i; }
    if (i < nk) { R64_STEP(i, w3) }
#undef R64_STEP
#undef R64_COMPUTE
#undef R64_STAGE
#undef R64_FETCH_W
#undef R64_FETCH_X

    // add the K parts in ascending order through LDS (the tiles are dead: every wave is past the last barrier)
    float* red = reinterpret_cast<float*>(smem);
    const int pair = wi + 2 * xj;                       // waves with equal (wi, xj) hold parts of one 32 x 32 result
    if (kh > 0) {
#pragma unroll
        for (int v = 0; v < 16; ++v) red[(((kh - 1) * (2 * MT) + pair) * 16 + v) * 64 + lane] = acc[v];
    }
    __syncthreads();
    if (kh == 0) {
#pragma unroll
        for (int p = 0; p < KH - 1; ++p)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] += red[((p * (2 * MT) + pair) * 16 + v) * 64 + lane];
        const int n = n0 + wi * 32 + l32;
        if (n < N) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = xj * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
                if (m < M) part[((size_t)by * ROWS + m) * N + n] = acc[v];
            }
        }
    }
}

// fp32 rows -> hi + lo bf16 rows, optionally through RMSNorm (gain != nullptr).  One block per row.
template <typename WT>
__global__ __launch_bounds__(256) void split_rows_kernel(const float* __restrict__ X, int ldx, int K,
                                                         const WT* __restrict__ gain, float eps,
                                                         uint16_t* __restrict__ Xh, uint16_t* __restrict__ Xl) {
    __shared__ float red[4];
    const float* xr = X + (size_t)blockIdx.x * ldx;
    float rs = 1.0f;
    if (gain) {
        float ss = 0.0f;
        for (int k = threadIdx.x * 4; k < K; k += 1024) {
            const float4 v = *reinterpret_cast<const float4*>(xr + k);
            ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
        }
        ss = block256_sum(ss, red);
        rs = 1.0f / sqrtf(ss / (float)K + eps);
    }
    for (int k = threadIdx.x * 4; k < K; k += 1024) {
        float4 v = *reinterpret_cast<const float4*>(xr + k);
        if (gain) {
            v.x *= rs * ld1(gain + k);     v.y *= rs * ld1(gain + k + 1);
            v.z *= rs * ld1(gain + k + 2); v.w *= rs * ld1(gain + k + 3);
        }
        const float x[4] = {v.x, v.y, v.z, v.w};
        uint16_t hi[4], lo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) { hi[e] = f2bf(x[e]); lo[e] = f2bf(x[e] - bf2f(hi[e])); }
        *reinterpret_cast<uint2*>(Xh + (size_t)blockIdx.x * K + k) =
            make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
        *reinterpret_cast<uint2*>(Xl + (size_t)blockIdx.x * K + k) =
            make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16));
    }
}

// sum over z (ascending) of the float4 at p + z * stride; eight loads are requested at a time, the last
// batch with clamped addresses (one round trip for the remainder instead of one per slice)
__device__ __forceinline__ float4 sum_slices(const float* __restrict__ p, size_t stride, int KS) {
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
    int z = 0;
    for (; z + 8 <= KS; z += 8) {
        float4 b[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) b[i] = *reinterpret_cast<const float4*>(p + (size_t)(z + i) * stride);
#pragma unroll
        for (int i = 0; i < 8; ++i) { a.x += b[i].x; a.y += b[i].y; a.z += b[i].z; a.w += b[i].w; }
    }
    if (z < KS) {
        float4 b[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) b[i] = *reinterpret_cast<const float4*>(p + (size_t)min(z + i, KS - 1) * stride);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (z + i < KS) { a.x += b[i].x; a.y += b[i].y; a.z += b[i].z; a.w += b[i].w; }
    }
    return a;
}

// Adds the K slices of gemm_rows_kernel (ascending z) and finishes:
//   EPI_STORE   Y[m][n]  = sum
//   EPI_RESID   Y[m][n] += sum
//   EPI_SWIGLU  N = 2F columns [gate ; up]: act = silu(gate) * up, written as hi + lo bf16 rows [m][F]
// geo.G > 0: the slices come from gemm_rows_sk_kernel, and a column of row block rb = n / 256 has
// sk_last(rb) - sk_first(rb) + 1 of them (KS is ignored).
template <int EPI>
__global__ void rows_finish_kernel(const float* __restrict__ part, int KS, int ROWS, int M, int N,
                                   float* __restrict__ Y, int ldy, uint16_t* __restrict__ Oh, uint16_t* __restrict__ Ol,
                                   SkGeom geo) {
    const int NO = (EPI == EPI_SWIGLU) ? N / 2 : N;
    const size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i >= (size_t)M * NO) return;
    const size_t m = i / NO, n = i - m * NO;           // NO is a multiple of 4
    auto sum = [&](size_t col) {
        int ks = KS;
        if (geo.G > 0) { const int rb = (int)(col >> 8); ks = sk_last(geo, rb) - sk_first(geo, rb) + 1; }
        return sum_slices(part + m * N + col, (size_t)ROWS * N, ks);
    };
    float4 a = sum(n);
    if (EPI == EPI_SWIGLU) {
        const float4 u = sum(NO + n);
        const float x[4] = {a.x / (1.0f + expf(-a.x)) * u.x, a.y / (1.0f + expf(-a.y)) * u.y,
                            a.z / (1.0f + expf(-a.z)) * u.z, a.w / (1.0f + expf(-a.w)) * u.w};
        uint16_t hi[4], lo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) { hi[e] = f2bf(x[e]); lo[e] = f2bf(x[e] - bf2f(hi[e])); }
        *reinterpret_cast<uint2*>(Oh + m * NO + n) =
            make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
        *reinterpret_cast<uint2*>(Ol + m * NO + n) =
            make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16));
    } else {
        float4* yp = reinterpret_cast<float4*>(Y + m * ldy + n);
        if (EPI == EPI_RESID) { const float4 y = *yp; a.x += y.x; a.y += y.y; a.z += y.z; a.w += y.w; }
        *yp = a;
    }
}

// EPI_RESID finish for a whole row per block, with the RMSNorm of the NEXT projection folded in: adds the K
// slices (ascending z) and the residual, stores the new residual stream H, and writes
// RMSNorm(H row) * gain as hi + lo bf16 halves.  N <= 8192, N % 4 == 0.
template <typename WT>
__global__ __launch_bounds__(1024) void rows_finish_norm_kernel(const float* __restrict__ part, int KS, int ROWS, int N,
                                                                float* __restrict__ H, int ldh,
                                                                const WT* __restrict__ gain, float eps,
                                                                uint16_t* __restrict__ Xh, uint16_t* __restrict__ Xl,
                                                                SkGeom geo) {
    __shared__ float red[16];
    const int m = blockIdx.x, tid = threadIdx.x;
    float4 v[2];
    float ss = 0.0f;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int n = tid * 4 + i * 4096;
        v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (n < N) {
            int ks = KS;
            if (geo.G > 0) { const int rb = n >> 8; ks = sk_last(geo, rb) - sk_first(geo, rb) + 1; }
            float4 a = sum_slices(part + (size_t)m * N + n, (size_t)ROWS * N, ks);
            float4* hp = reinterpret_cast<float4*>(H + (size_t)m * ldh + n);
            const float4 y = *hp;
            a.x += y.x; a.y += y.y; a.z += y.z; a.w += y.w;
            *hp = a;
            v[i] = a;
            ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
        }
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    float tot = 0.0f;
#pragma unroll
    for (int w = 0; w < 16; ++w) tot += red[w];
    const float rs = 1.0f / sqrtf(tot / (float)N + eps);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int n = tid * 4 + i * 4096;
        if (n < N) {
            const float x[4] = {v[i].x * (rs * ld1(gain + n)), v[i].y * (rs * ld1(gain + n + 1)),
                                v[i].z * (rs * ld1(gain + n + 2)), v[i].w * (rs * ld1(gain + n + 3))};
            uint16_t hi[4], lo[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) { hi[e] = f2bf(x[e]); lo[e] = f2bf(x[e] - bf2f(hi[e])); }
            *reinterpret_cast<uint2*>(Xh + (size_t)m * N + n) =
                make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
            *reinterpret_cast<uint2*>(Xl + (size_t)m * N + n) =
                make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16));
        }
    }
}

// K slices for gemm_rows_kernel.  Measured (K-slice sweeps over the 1.5B / 7B / 72B shapes at 16 and 64 rows):
// the kernel is fastest when the grid has at most one block per compute unit and covers most of them
// (7B down: 252 or 224 blocks 32 us, 280 blocks 45 us, 462 blocks 35 us); two co-resident blocks only
// pay when one per unit would leave the chip half empty (7B gate/up: 148 x 3 blocks 59 us, 148 x 1 86 us).
// So: the largest count with rows-of-blocks x slices <= 256 if that fills 200 units or more; otherwise the
// count that minimises (rounds of 512 resident blocks) x (K blocks per slice) plus the traffic of the
// partial results, in units of one K block over 256 rows of W.
static int gemm_rows64_slices(int N, int K, int rows, size_t part_floats);
static bool gemm_rows_small(int N, int K);
static int gemm_rows_slices(int N, int K, int rows, size_t part_floats) {
    if (gemm_rows_small(N, K)) return gemm_rows64_slices(N, K, rows, part_floats);
    const int nb = (N + 255) / 256, nkb = K / 64;
    {
        int ks = std::min(256 / nb, nkb / 2);
        while (ks > 1 && ((size_t)ks * rows * N > part_floats || (ks - 1) * ((nkb + ks - 1) / ks) >= nkb)) --ks;
        if (ks >= 1 && nb * ks >= 200 && (size_t)ks * rows * N <= part_floats) return ks;
    }
    int best = 1;
    double best_cost = 1e30;
    for (int ks = 1; ks <= 64 && ks <= nkb; ++ks) {
        if ((size_t)ks * rows * N > part_floats) break;
        const int per = (nkb + ks - 1) / ks;
        if ((ks - 1) * per >= nkb) continue;                 // would leave a slice empty
        const int rounds = (nb * ks + 511) / 512;
        const double cost = (double)rounds * per * 512 * 256 * 128 + (double)ks * rows * N * 8;
        if (cost < best_cost) { best_cost = cost; best = ks; }
    }
    return best;
}

// Small matrices (at most 17 M weights: the 7B QKV and output projections, the 1.5B down and attention
// projections) go to the 64-row kernel, with as many K slices as bring the grid to about 450 blocks (4..8, and
// at least two K blocks each).  The 7B QKV (16.5 M) is the largest of them: 16.5 us there against 18.0 us on
// 256-row blocks at 64 rows, and its 6 instead of 14 K slices make the attention kernel that adds them
// 2 us faster.
static bool gemm_rows_small(int N, int K) { return (size_t)N * K <= ((size_t)17 << 20); }
static int gemm_rows64_slices(int N, int K, int rows, size_t part_floats) {
    const int nb = (N + 63) / 64, nkb = K / 64;
    int ks = std::max(4, std::min(8, (448 + nb / 2) / nb));
    while (ks > 1 && (ks * 2 > nkb || (size_t)ks * rows * N > part_floats || (ks - 1) * ((nkb + ks - 1) / ks) >= nkb)) --ks;
    return ks;
}

// Geometry of the evenly dealt kernel for an [N][K] matrix on G thread blocks (G is lowered to the number of
// units when there are fewer).
static SkGeom sk_geometry(int N, int K, int G) {
    SkGeom g;
    const int nb = (N + 255) / 256;
    g.nkb = K / 64;
    g.units = nb * g.nkb;
    g.G = std::max(1, std::min(G, g.units));
    g.zmax = 1;
    for (int rb = 0; rb < nb; ++rb) g.zmax = std::max(g.zmax, sk_last(g, rb) - sk_first(g, rb) + 1);
    return g;
}
// Which few-row products take the evenly dealt kernel: those with 200 or more 256-row blocks, which uniform K
// slices cannot spread evenly over 256 compute units (measured at 16 rows: [59136][8192] 190 -> 183 us,
// [151936][8192] 526 -> 457 us, [151936][1536] 112 -> 106 us; with fewer row blocks uniform slices at two
// co-resident blocks per unit are as fast or faster: [37888][3584] 52 against 58 us).  One thread block per
// compute unit and two W register sets: 512 thread blocks or four sets were slower or equal.
constexpr int kSkBlocks = 256, kSkDepth = 2;
static bool gemm_rows_even(int N, int K) { (void)K; return (N + 255) / 256 >= 200; }
template <int D>
static void gemm_rows_sk_launch(hipStream_t st, const bf16_t* W, int N, int K, const uint16_t* Xh, const uint16_t* Xl,
                                int M, float* part, const SkGeom& g) {
    if (M <= 32) hipLaunchKernelGGL((gemm_rows_sk_kernel<1, D>), dim3(g.G), dim3(512), 0, st, W, N, K, Xh, Xl, part, g, M);
    else         hipLaunchKernelGGL((gemm_rows_sk_kernel<2, D>), dim3(g.G), dim3(512), 0, st, W, N, K, Xh, Xl, part, g, M);
}

static void gemm_rows_launch(hipStream_t st, const bf16_t* W, int N, int K, const uint16_t* Xh, const uint16_t* Xl,
                             int M, float* part, int ks) {
    if (gemm_rows_small(N, K)) {
        const dim3 grid((N + 63) / 64, ks), block(512);
        if (M <= 32) hipLaunchKernelGGL((gemm_rows64_kernel<1>), grid, block, 0, st, W, N, K, Xh, Xl, part, M);
        else         hipLaunchKernelGGL((gemm_rows64_kernel<2>), grid, block, 0, st, W, N, K, Xh, Xl, part, M);
        return;
    }
    const dim3 grid((N + 255) / 256, ks), block(512);
    if (M <= 32) hipLaunchKernelGGL((gemm_rows_kernel<1>), grid, block, 0, st, W, N, K, Xh, Xl, part, M);
    else         hipLaunchKernelGGL((gemm_rows_kernel<2>), grid, block, 0, st, W, N, K, Xh, Xl, part, M);
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

// ---------------------------------------------------------------- bf16 MFMA, many rows, pre-split activations
// Y[m][n] (+)= sum_k (Xh + Xl)[m][k] * W[n][k] for more than 64 rows (prefill chunks, large decode batches).
// Block tile BM (128 or 256 rows of X) x 256 (rows of W), BM / 32 waves of 64 x 128 (2 x 4 MFMA tiles of
// 32x32x16, hi and lo pass on each: 32 MFMAs against 16 operand reads of 16 bytes per K block of 32).
// The copies from L2 into LDS, not the MFMAs, bound this kernel (they alone take 85 % of its time at
// BM = 128): per K block a tile pulls 64 B x (2 BM + 256) through L2, so the larger tile moves 25 %
// fewer bytes per flop and is used whenever it still gives every compute unit two blocks.  LDS holds two stages of
// [rows][32 k] tiles (Xh, Xl, W), chunks of 16 bytes permuted by (row / 4) % 4 so that both the
// line-wise writes and the operand reads are conflict-free without padding.  While one stage is
// multiplied the next one is already on its way from global memory in registers.  gridDim.z > 1 cuts K into
// slices whose partial tiles go to part[z][M][N] (finished by rows_finish_kernel).
template <int EPI, int BM>
__global__ __launch_bounds__(BM * 2, BM == 128 ? 2 : 1) void gemm_tile_kernel(const bf16_t* __restrict__ W, int N, int K,
                                                           const uint16_t* __restrict__ Xh,
                                                           const uint16_t* __restrict__ Xl, int M,
                                                           float* __restrict__ Y, int ldy,
                                                           float* __restrict__ part,
                                                           uint16_t* __restrict__ Oh, uint16_t* __restrict__ Ol,
                                                           unsigned long long* __restrict__ clk) {
    // clk != nullptr (a timing probe is armed): the block in the middle of the grid reports how many shader clock
    // ticks and how many ticks of the constant 100 MHz counter its K loop took: {shader ticks, reference ticks,
    // launches} are added to clk[0..2], which gives the clock the chip sustains while this kernel runs
    long long clk_c0 = 0, clk_w0 = 0;
    if (clk) { clk_c0 = clock64(); clk_w0 = wall_clock64(); }
    constexpr int BN = 256, BK = 32, CR = BM / 2;        // CR: rows covered by one round of copies (threads / 4)
    __shared__ __attribute__((aligned(16))) uint16_t Ah[2][BM * BK];
    __shared__ __attribute__((aligned(16))) uint16_t Al[2][BM * BK];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][BN * BK];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;                 // wave tile: rows wm*64.., columns wn*128..
    // (K-sliced launches only: without slices the plain order already keeps an activation tile's blocks together)
    int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
    if (gridDim.z > 1) {
        const int nxy = gridDim.x * gridDim.y;
        const int lin = xcd_major(bx + gridDim.x * by + nxy * bz, nxy * gridDim.z, M, N);
        bz = lin / nxy; by = (lin - bz * nxy) / gridDim.x; bx = lin - bz * nxy - by * gridDim.x;
    }
    const int m0 = by * BM, n0 = bx * BN;
    const int nkb = K / BK;
    const int per = (nkb + gridDim.z - 1) / gridDim.z;
    const int kb0 = bz * per, kb1 = min(nkb, kb0 + per);
    const int nk = kb1 - kb0;
    const int kb_last = max(kb1 - 1, 0);
    // LDS offset (in bf16) of 16-byte chunk c (0..3) of row r
    auto sw = [](int r, int c) { return r * BK + ((c ^ ((r >> 2) & 3)) << 3); };
    // global -> LDS copies: thread -> chunk tid % 4 of rows tid / 4 + CR i (two rounds cover the X tile;
    // the W tile takes four rounds at BM = 128, two at BM = 256)
    const int crow = tid >> 2, cch = tid & 3;
    const uint16_t* ah0 = Xh + (size_t)min(m0 + crow, M - 1) * K + cch * 8;
    const uint16_t* ah1 = Xh + (size_t)min(m0 + crow + CR, M - 1) * K + cch * 8;
    const uint16_t* al0 = Xl + (size_t)min(m0 + crow, M - 1) * K + cch * 8;
    const uint16_t* al1 = Xl + (size_t)min(m0 + crow + CR, M - 1) * K + cch * 8;
    // W row behind tile column r.  EPI_SWIGLU (W = [gate | up], N = 2F, never K-sliced): the tile's columns are 128
    // gate rows and the 128 up rows of the same units, arranged so that a wave's column groups j and j + 2 hold
    // gate and up of one unit: columns 128 w + 64 h + i (w = wave column, h = 0 gate / 1 up) <- row h F + 128 bx + 64 w + i
    auto wrow = [&](int r) {
        if (EPI == EPI_SWIGLU) return min(((r >> 6) & 1) * (N / 2) + bx * 128 + (r >> 7) * 64 + (r & 63), N - 1);
        return min(n0 + r, N - 1);
    };
    const bf16_t* b0 = W + (size_t)wrow(crow) * K + cch * 8;
    const bf16_t* b1 = W + (size_t)wrow(crow + CR) * K + cch * 8;
    const bf16_t* b2 = W + (size_t)wrow(crow + 128) * K + cch * 8;       // BM = 128 only
    const bf16_t* b3 = W + (size_t)wrow(crow + 192) * K + cch * 8;
    const int st0 = sw(crow, cch), st1 = sw(crow + CR, cch), st2 = sw(crow + 128, cch), st3 = sw(crow + 192, cch);

    f32x16_t acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // two register sets named member by member: a K block is requested two steps before it moves into LDS
    struct Regs { u32x4_t h0, h1, l0, l1, b0, b1, b2, b3; };
    Regs ra, rb;
#define RSD_FETCH(kb, R)                                                                         \
    {                                                                                            \
        const size_t k0_ = (size_t)min((kb), kb_last) * BK;                                      \
        R.h0 = *reinterpret_cast<const u32x4_t*>(ah0 + k0_);                                     \
        R.h1 = *reinterpret_cast<const u32x4_t*>(ah1 + k0_);                                     \
        R.l0 = *reinterpret_cast<const u32x4_t*>(al0 + k0_);                                     \
        R.l1 = *reinterpret_cast<const u32x4_t*>(al1 + k0_);                                     \
        R.b0 = *reinterpret_cast<const u32x4_t*>(b0 + k0_);                                      \
        R.b1 = *reinterpret_cast<const u32x4_t*>(b1 + k0_);                                      \
        if (BM == 128) {                                                                         \
            R.b2 = *reinterpret_cast<const u32x4_t*>(b2 + k0_);                                  \
            R.b3 = *reinterpret_cast<const u32x4_t*>(b3 + k0_);                                  \
        }                                                                                        \
    }
#define RSD_STAGE(buf, R)                                                                        \
    {                                                                                            \
        *reinterpret_cast<u32x4_t*>(&Ah[(buf)][st0]) = R.h0;                                     \
        *reinterpret_cast<u32x4_t*>(&Ah[(buf)][st1]) = R.h1;                                     \
        *reinterpret_cast<u32x4_t*>(&Al[(buf)][st0]) = R.l0;                                     \
        *reinterpret_cast<u32x4_t*>(&Al[(buf)][st1]) = R.l1;                                     \
        *reinterpret_cast<u32x4_t*>(&Bs[(buf)][st0]) = R.b0;                                     \
        *reinterpret_cast<u32x4_t*>(&Bs[(buf)][st1]) = R.b1;                                     \
        if (BM == 128) {                                                                         \
            *reinterpret_cast<u32x4_t*>(&Bs[(buf)][st2]) = R.b2;                                 \
            *reinterpret_cast<u32x4_t*>(&Bs[(buf)][st3]) = R.b3;                                 \
        }                                                                                        \
    }
    const int l32 = lane & 31, kg = lane >> 5;
#define RSD_COMPUTE(buf)                                                                         \
    {                                                                                            \
        _Pragma("unroll") for (int kk_ = 0; kk_ < 2; ++kk_) {                                    \
            bf16x8_t a_[2], l_[2], b_[4];                                                        \
            _Pragma("unroll") for (int i_ = 0; i_ < 2; ++i_) {                                   \
                const int off_ = sw(wm * 64 + i_ * 32 + l32, kk_ * 2 + kg);                      \
                a_[i_] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(&Ah[(buf)][off_])); \
                l_[i_] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(&Al[(buf)][off_])); \
            }                                                                                    \
            _Pragma("unroll") for (int j_ = 0; j_ < 4; ++j_)                                     \
                b_[j_] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(&Bs[(buf)][sw(wn * 128 + j_ * 32 + l32, kk_ * 2 + kg)])); \
            /* all lo passes, then all hi passes: two MFMAs on one accumulator are eight apart */ \
            _Pragma("unroll") for (int i_ = 0; i_ < 2; ++i_)                                     \
                _Pragma("unroll") for (int j_ = 0; j_ < 4; ++j_)                                 \
                    acc[i_][j_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(l_[i_], b_[j_], acc[i_][j_], 0, 0, 0); \
            _Pragma("unroll") for (int i_ = 0; i_ < 2; ++i_)                                     \
                _Pragma("unroll") for (int j_ = 0; j_ < 4; ++j_)                                 \
                    acc[i_][j_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_[i_], b_[j_], acc[i_][j_], 0, 0, 0); \
        }                                                                                        \
    }
    RSD_FETCH(kb0, ra)
    RSD_FETCH(kb0 + 1, rb)
    RSD_STAGE(0, ra)
    __syncthreads();
    // step i: block i + 2 is requested into the set F that block i came from, block i is multiplied,
    // block i + 1 (set S, requested a step ago) moves into the LDS buffer block i - 1 has left
#define RSD_STEP(i_step, F, S)                                                                   \
    {                                                                                            \
        RSD_FETCH(kb0 + (i_step) + 2, F)                                                         \
        RSD_COMPUTE((i_step) & 1)                                                                \
        RSD_STAGE(((i_step) + 1) & 1, S)                                                         \
        __syncthreads();                                                                         \
    }
    int i = 0;
    for (; i + 1 < nk; i += 2) {
        RSD_STEP(i, ra, rb)
        RSD_STEP(i + 1, rb, ra)
    }
    if (i < nk) RSD_STEP(i, ra, rb)
#undef RSD_STEP
#undef RSD_FETCH
#undef RSD_STAGE
#undef RSD_COMPUTE
    if (clk && tid == 0 && blockIdx.x == gridDim.x / 2 && blockIdx.y == gridDim.y / 2 && blockIdx.z == 0) {
        atomicAdd(&clk[0], (unsigned long long)(clock64() - clk_c0));
        atomicAdd(&clk[1], (unsigned long long)(wall_clock64() - clk_w0));
        atomicAdd(&clk[2], 1ull);
    }

    if (EPI == EPI_SWIGLU) {
        // silu(gate) * up of the units this wave holds, straight into the hi / lo halves the down projection reads
        const int F = N / 2;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int col = bx * 128 + wn * 64 + j * 32 + l32;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
                    if (m < M && col < F) {
                        const float g = acc[i][j][v], u = acc[i][j + 2][v];
                        const float x = g / (1.0f + expf(-g)) * u;
                        const uint16_t hi = f2bf(x);
                        Oh[(size_t)m * F + col] = hi;
                        Ol[(size_t)m * F + col] = f2bf(x - bf2f(hi));
                    }
                }
            }
        return;
    }
    const bool sliced = gridDim.z > 1;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + wn * 128 + j * 32 + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
                if (m < M && n < N) {
                    if (sliced) {
                        part[((size_t)bz * M + m) * N + n] = acc[i][j][v];
                    } else {
                        float* yp = Y + (size_t)m * ldy + n;
                        *yp = (EPI == EPI_RESID) ? (*yp + acc[i][j][v]) : acc[i][j][v];
                    }
                }
            }
        }
}

// Block tile and K slices for gemm_tile_kernel.
// Many rows (chunked passes): gemm_tile_plan_chunked below.
// 65..256 rows (the decode iteration of a large batch: one row tile): the kernel is MFMA-bound there, two
// co-resident 128-row blocks run no faster than one (measured per K block of 32: 0.97 us for a 128-row block
// alone on its unit, 2.2 us each for two, 1.37 us for a 256-row block), so the grid is kept to one round of at
// most 256 blocks and filled with K slices: [3584][18944] at 256 rows 98 -> 72 us, [17920][1536] 53 -> 39 us,
// [37888][3584] (148 column tiles: no slices, no finish kernel) 178 + 18 -> 170 us.
static bool gemm_tile_decode_rows(int M) { return M <= 256; }
// Decode-size launches (one row tile of the batch): the 256-row tile wherever its N tiles x K slices (at least six
// K blocks each) give 128 blocks or more, else two 128-row tiles (small matrices: the 1.5B attention projections
// at 256 rows 22 -> 17 us).  A compute unit holds one block of the 256-row tile or two of the 128-row tile.
// Chunked passes (more than 256 rows): tile height and K slices by a small cost model in units of the measured
// time per K block (1.37 us for a 256-row block, one per compute unit; 2.2 us for two co-resident 128-row blocks,
// 0.97 us for one alone): rounds of resident blocks x K blocks per slice (+ 3 for filling and draining the
// pipeline), plus what the finish kernel pays to read the slices' partial sums back.
struct TilePlan { int bm, ks; };
static TilePlan gemm_tile_plan_chunked(int N, int K, int M, size_t part_floats) {
    const int tn = (N + 255) / 256, nkb = K / 32;
    TilePlan best{256, 1};
    double best_t = 1e30;
    for (int bm : {256, 128})
        for (int ks = 1; ks <= 32; ks *= 2) {
            if (ks > 1 && (nkb / ks < 8 || (size_t)ks * M * N > part_floats)) break;
            const long long blocks = (long long)tn * ((M + bm - 1) / bm) * ks;
            const double kb = (nkb + ks - 1) / ks + 3;
            double us;
            if (bm == 256) us = (double)((blocks + 255) / 256) * kb * 1.37;
            else {
                const long long rem = blocks % 512;
                us = (double)(blocks / 512) * kb * 2.2 + (rem == 0 ? 0.0 : rem <= 256 ? kb * 0.97 : kb * 2.2);
            }
            if (ks > 1) us += 4.0 + (double)ks * M * N * 8.0 / 5.0e6;
            if (us < best_t) { best_t = us; best = TilePlan{bm, ks}; }
        }
    return best;
}
static int gemm_tile_bm(int N, int K, int M, int ks) {
    if (gemm_tile_decode_rows(M)) {
        const int tn = (N + 255) / 256, nkb = K / 32;
        if (M <= 128) return 128;
        return tn * std::max(1, std::min(std::min(256 / tn, nkb / 6), 32)) >= 128 ? 256 : 128;
    }
    // (chunked: the height the plan chose for this slice count)
    TilePlan best{256, ks};
    double best_t = 1e30;
    const int tn = (N + 255) / 256, nkb = K / 32;
    for (int bm : {256, 128}) {
        const long long blocks = (long long)tn * ((M + bm - 1) / bm) * ks;
        const double kb = (nkb + ks - 1) / ks + 3;
        double us;
        if (bm == 256) us = (double)((blocks + 255) / 256) * kb * 1.37;
        else {
            const long long rem = blocks % 512;
            us = (double)(blocks / 512) * kb * 2.2 + (rem == 0 ? 0.0 : rem <= 256 ? kb * 0.97 : kb * 2.2);
        }
        if (us < best_t) { best_t = us; best.bm = bm; }
    }
    return best.bm;
}
static int gemm_tile_slices(int N, int K, int M, size_t part_floats) {
    if (gemm_tile_decode_rows(M)) {
        const int tn = (N + 255) / 256, nkb = K / 32;
        const int bm = gemm_tile_bm(N, K, M, 1);
        const int room = bm == 256 ? 256 / tn : 512 / (tn * ((M + 127) / 128));
        int ks = std::max(1, std::min(std::min(room, nkb / 6), 32));
        while (ks > 1 && ((size_t)ks * M * N > part_floats || (ks - 1) * ((nkb + ks - 1) / ks) >= nkb)) --ks;
        return ks;
    }
    return gemm_tile_plan_chunked(N, K, M, part_floats).ks;
}

// epi == EPI_SWIGLU (W = [gate | up], ks = 1): the activated values go to Oh / Ol [M][N / 2] as hi / lo halves
static void gemm_tile_launch(hipStream_t st, int epi, const bf16_t* W, int N, int K, const uint16_t* Xh,
                             const uint16_t* Xl, int M, float* Y, int ldy, float* part, int ks,
                             uint16_t* Oh = nullptr, uint16_t* Ol = nullptr, unsigned long long* clk = nullptr) {
    const int tn = (N + 255) / 256;
    if (gemm_tile_bm(N, K, M, ks) == 256) {
        const dim3 grid(tn, (M + 255) / 256, ks), block(512);
        if (epi == EPI_SWIGLU)     hipLaunchKernelGGL((gemm_tile_kernel<EPI_SWIGLU, 256>), grid, block, 0, st, W, N, K, Xh, Xl, M, Y, ldy, part, Oh, Ol, clk);
        else if (epi == EPI_RESID) hipLaunchKernelGGL((gemm_tile_kernel<EPI_RESID, 256>), grid, block, 0, st, W, N, K, Xh, Xl, M, Y, ldy, part, Oh, Ol, clk);
        else                       hipLaunchKernelGGL((gemm_tile_kernel<EPI_STORE, 256>), grid, block, 0, st, W, N, K, Xh, Xl, M, Y, ldy, part, Oh, Ol, clk);
        return;
    }
    const dim3 grid(tn, (M + 127) / 128, ks), block(256);
    if (epi == EPI_SWIGLU)     hipLaunchKernelGGL((gemm_tile_kernel<EPI_SWIGLU, 128>), grid, block, 0, st, W, N, K, Xh, Xl, M, Y, ldy, part, Oh, Ol, clk);
    else if (epi == EPI_RESID) hipLaunchKernelGGL((gemm_tile_kernel<EPI_RESID, 128>), grid, block, 0, st, W, N, K, Xh, Xl, M, Y, ldy, part, Oh, Ol, clk);
    else                       hipLaunchKernelGGL((gemm_tile_kernel<EPI_STORE, 128>), grid, block, 0, st, W, N, K, Xh, Xl, M, Y, ldy, part, Oh, Ol, clk);
}

