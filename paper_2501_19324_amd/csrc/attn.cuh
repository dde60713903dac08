// Grouped-query attention of one query token per row over a paged KV cache,
// plus the rotary-embedding / cache-write kernel that feeds it.
//
// KV pool of one model: [layer][page][K|V][kv_head][16 tokens][head_dim], so
// the keys (or values) of one page and KV head are 16*head_dim contiguous
// elements.  Token at position p of a sequence lives in logical page p / 16,
// slot p % 16; block_table[seq][logical page] gives the physical page.
#pragma once
#include "common.cuh"

#define RSD_PAGE 16

// One block per (row, kv head, split).  The G query heads of the group share
// every key/value load.  A "lane group" of HD/8 lanes covers one token (16
// bytes of bf16 per lane); each lane group runs its own online softmax over
// the tokens it sees, and the streams are merged at the end (lane groups by
// shuffles, waves through LDS, splits by attn_combine_kernel).
template <typename KT, int HD, int G>
__global__ __launch_bounds__(256) void attn_rows_kernel(const float* __restrict__ qkv, int ldq,
                                                        const KT* __restrict__ pool_layer,
                                                        const int* __restrict__ block_table, int max_pages,
                                                        RowMap rm, int H, int Hkv, int S, float scale,
                                                        float* __restrict__ out, int ldo,
                                                        float* __restrict__ part_acc,
                                                        float* __restrict__ part_ml) {
    constexpr int LPT = HD / 8;          // lanes per token
    constexpr int TPW = 64 / LPT;        // tokens per wave-wide load
    constexpr int ITERS = RSD_PAGE / TPW > 0 ? RSD_PAGE / TPW : 1;   // wave loads per page
    constexpr int PPW = TPW / RSD_PAGE > 0 ? TPW / RSD_PAGE : 1;     // pages per wave load (HD = 32: 1)
    static_assert(PPW == 1, "a wave load covers at most one page");
    const int r = blockIdx.x, hk = blockIdx.y, sp = blockIdx.z;
    int seq, pos;
    if (!row_lookup(rm, r, seq, pos)) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int part = lane % LPT, tsub = lane / LPT;

    float q[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        load8(qkv + (size_t)r * ldq + (hk * G + g) * HD + part * 8, q[g]);
#pragma unroll
        for (int e = 0; e < 8; ++e) q[g][e] *= scale;
    }
    float mx[G], l[G], acc[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        mx[g] = -INFINITY; l[g] = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = 0.0f;
    }

    const int n_keys = pos + 1;
    const int n_pages = (n_keys + RSD_PAGE - 1) / RSD_PAGE;
    const int pps = (n_pages + S - 1) / S;
    const int p_begin = sp * pps, p_end = min(n_pages, p_begin + pps);
    const int* bt = block_table + (size_t)seq * max_pages;
    const size_t page_elts = (size_t)2 * Hkv * RSD_PAGE * HD;

    for (int pg = p_begin + wave; pg < p_end; pg += 4) {
        const KT* kbase = pool_layer + (size_t)bt[pg] * page_elts + (size_t)hk * RSD_PAGE * HD;
        const KT* vbase = kbase + (size_t)Hkv * RSD_PAGE * HD;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int slot = it * TPW + tsub;
            const int t = pg * RSD_PAGE + slot;
            float kx[8], vx[8];
            load8(kbase + slot * HD + part * 8, kx);
            load8(vbase + slot * HD + part * 8, vx);
            float s[G];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float d = 0.0f;
#pragma unroll
                for (int e = 0; e < 8; ++e) d += q[g][e] * kx[e];
#pragma unroll
                for (int off = 1; off < LPT; off <<= 1) d += __shfl_xor(d, off, RSD_WAVE);
                s[g] = d;
            }
            if (t < n_keys) {
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const float mn = fmaxf(mx[g], s[g]);
                    const float corr = expf(mx[g] - mn);      // exp(-inf) = 0 on the first token
                    const float p = expf(s[g] - mn);
                    l[g] = l[g] * corr + p;
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[g][e] = acc[g][e] * corr + p * vx[e];
                    mx[g] = mn;
                }
            }
        }
    }

    // merge the lane groups of the wave
#pragma unroll
    for (int off = LPT; off < 64; off <<= 1) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float mo = __shfl_xor(mx[g], off, RSD_WAVE);
            const float lo = __shfl_xor(l[g], off, RSD_WAVE);
            const float mn = fmaxf(mx[g], mo);
            const float ca = (mx[g] == -INFINITY) ? 0.0f : expf(mx[g] - mn);
            const float cb = (mo == -INFINITY) ? 0.0f : expf(mo - mn);
            l[g] = l[g] * ca + lo * cb;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float ao = __shfl_xor(acc[g][e], off, RSD_WAVE);
                acc[g][e] = acc[g][e] * ca + ao * cb;
            }
            mx[g] = mn;
        }
    }
    // merge the four waves through LDS
    __shared__ float s_acc[4][G][HD];
    __shared__ float s_m[4][G], s_l[4][G];
    if (lane < LPT) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int e = 0; e < 8; ++e) s_acc[wave][g][part * 8 + e] = acc[g][e];
            if (lane == 0) { s_m[wave][g] = mx[g]; s_l[wave][g] = l[g]; }
        }
    }
    __syncthreads();
    const int H_ = H;
    for (int idx = tid; idx < G * HD; idx += 256) {
        const int g = idx / HD, e = idx - g * HD;
        float mn = fmaxf(fmaxf(s_m[0][g], s_m[1][g]), fmaxf(s_m[2][g], s_m[3][g]));
        float a = 0.0f, ll = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float c = (s_m[w][g] == -INFINITY) ? 0.0f : expf(s_m[w][g] - mn);
            a += s_acc[w][g][e] * c;
            ll += s_l[w][g] * c;
        }
        const int h = hk * G + g;
        if (S == 1) {
            out[(size_t)r * ldo + h * HD + e] = a / ll;
        } else {
            const size_t pi = ((size_t)r * H_ + h) * S + sp;
            part_acc[pi * HD + e] = a;
            if (e == 0) { part_ml[pi * 2] = mn; part_ml[pi * 2 + 1] = ll; }
        }
    }
}

// Merge the S partial results of every (row, head).
template <int HD>
__global__ void attn_combine_kernel(const float* __restrict__ part_acc, const float* __restrict__ part_ml,
                                    RowMap rm, int H, int S, float* __restrict__ out, int ldo) {
    const int r = blockIdx.x, h = blockIdx.y, e = threadIdx.x;
    int seq, pos;
    if (!row_lookup(rm, r, seq, pos)) return;
    const size_t base = ((size_t)r * H + h) * S;
    float mn = -INFINITY;
    for (int s = 0; s < S; ++s) mn = fmaxf(mn, part_ml[(base + s) * 2]);
    float a = 0.0f, ll = 0.0f;
    for (int s = 0; s < S; ++s) {
        const float m = part_ml[(base + s) * 2];
        const float c = (m == -INFINITY) ? 0.0f : expf(m - mn);
        a += part_acc[(base + s) * HD + e] * c;
        ll += part_ml[(base + s) * 2 + 1] * c;
    }
    out[(size_t)r * ldo + h * HD + e] = a / ll;
}

// Rotate q (in place, fp32) and k with the precomputed table rope[pos][i] =
// (cos, sin)(pos * theta^(-2i/HD)), pairing element i with i + HD/2; write the
// rotated k and v of the row's token into its cache slot.
template <typename KT, int HD>
__global__ __launch_bounds__(256) void rope_kv_kernel(float* __restrict__ qkv, int ldq,
                                                      KT* __restrict__ pool_layer,
                                                      const int* __restrict__ block_table, int max_pages,
                                                      RowMap rm, const float2* __restrict__ rope,
                                                      int H, int Hkv) {
    const int r = blockIdx.x;
    int seq, pos;
    if (!row_lookup(rm, r, seq, pos)) return;
    constexpr int HALF = HD / 2;
    float* row = qkv + (size_t)r * ldq;
    const float2* cs = rope + (size_t)pos * HALF;
    const int page = block_table[(size_t)seq * max_pages + pos / RSD_PAGE], slot = pos % RSD_PAGE;
    const size_t page_elts = (size_t)2 * Hkv * RSD_PAGE * HD;
    KT* kdst = pool_layer + (size_t)page * page_elts + (size_t)slot * HD;
    KT* vdst = kdst + (size_t)Hkv * RSD_PAGE * HD;
    const int nq = H * HALF, nk = Hkv * HALF, nv = Hkv * HD;
    for (int idx = threadIdx.x; idx < nq + nk + nv; idx += 256) {
        if (idx < nq + nk) {
            const int h = idx / HALF, i = idx - h * HALF;      // heads H.. are the key heads
            float* p = row + h * HD + i;
            const float a = p[0], b = p[HALF];
            const float2 c = cs[i];
            const float ra = a * c.x - b * c.y, rb = b * c.x + a * c.y;
            if (h < H) { p[0] = ra; p[HALF] = rb; }
            else {
                KT* d = kdst + (size_t)(h - H) * RSD_PAGE * HD + i;
                st1(d, ra); st1(d + HALF, rb);
            }
        } else {
            const int j = idx - nq - nk, hk = j / HD, e = j - hk * HD;
            st1(vdst + (size_t)hk * RSD_PAGE * HD + e, row[(H + Hkv) * HD + j]);
        }
    }
}
