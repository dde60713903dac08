// Grouped-query attention of one query token per row over a paged KV cache,
// plus the rotary-embedding / cache-write kernel that feeds it.
//
// KV pool of one model: [layer][page][K|V][kv_head][16 tokens][head_dim], so
// the keys (or values) of one page and KV head are 16*head_dim contiguous
// elements (in which order inside that block depends on the cache type, see
// KvTraits / KvTiled below).  Token at position p of a sequence lives in logical
// page p / 16, slot p % 16; block_table[seq][logical page] gives the physical page.
#pragma once
#include "common.h"

#define RSD_PAGE 16

// bf16 caches keep the values of a page transposed, [head_dim][16 tokens], so that
// the token axis (the contraction axis of P.V) is contiguous for the MFMA
// operands; fp32 caches (tiny configuration, VALU kernels only) keep [16][head_dim].
template <typename KT> struct KvTraits { static constexpr bool v_transposed = false; };
template <> struct KvTraits<bf16_t> { static constexpr bool v_transposed = true; };

// bf16 caches with head_dim 128 (the MFMA kernels) go one step further: inside the 4 KB key block and the
// 4 KB value block of a (page, KV head) the elements are stored in the order the MFMA operands are loaded,
// so that every operand load of a wave (lane l takes 16 bytes) reads 1 KB of consecutive memory:
//   keys:   chunk j (elements 32 j .. 32 j + 31) of the 16 tokens is 1 KB; lane l = 16 c + t holds
//           elements 32 j + 8 c .. + 7 of token t            -> offset ((4 j + c) * 16 + t) * 8 + i
//   values: head dims 32 m .. 32 m + 31 are 1 KB; lane l = 16 c + (d % 16) holds tokens 4 c .. 4 c + 3 of
//           dims 32 m + d % 16 and 32 m + 16 + d % 16        -> offset ((64 m + l) * 2 + (d / 16) % 2) * 4 + t % 4
template <typename KT, int HD> struct KvTiled { static constexpr bool value = false; };
template <> struct KvTiled<bf16_t, 128> { static constexpr bool value = true; };
__device__ __forceinline__ int kv_tiled_k(int t, int e) { return ((((e >> 5) * 4 + ((e >> 3) & 3)) * 16) + t) * 8 + (e & 7); }
__device__ __forceinline__ int kv_tiled_v(int t, int d) {
    return ((((d >> 5) * 64 + ((t >> 2) * 16 + (d & 15))) * 2 + ((d >> 4) & 1)) * 4) + (t & 3);
}
// offset of elements [e0, e0 + 8) (e0 a multiple of 8: they are contiguous in either layout) of token `slot` in a key block
template <typename KT, int HD>
__device__ __forceinline__ int k_off8(int slot, int e0) { return KvTiled<KT, HD>::value ? kv_tiled_k(slot, e0) : slot * HD + e0; }

// 8 consecutive head-dim elements [e0, e0+8) of token `slot` from one head's value page
template <typename KT, int HD>
__device__ __forceinline__ void load_v8(const KT* __restrict__ vhead, int slot, int e0, float o[8]) {
    if (KvTiled<KT, HD>::value) {
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = ld1(vhead + kv_tiled_v(slot, e0 + e));
    } else if (KvTraits<KT>::v_transposed) {
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = ld1(vhead + (e0 + e) * RSD_PAGE + slot);
    } else {
        load8(vhead + slot * HD + e0, o);
    }
}
template <typename KT, int HD>
__device__ __forceinline__ KT* v_addr(KT* vhead, int slot, int e) {
    if (KvTiled<KT, HD>::value) return vhead + kv_tiled_v(slot, e);
    return KvTraits<KT>::v_transposed ? vhead + e * RSD_PAGE + slot : vhead + slot * HD + e;
}

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
            load8(kbase + k_off8<KT, HD>(slot, part * 8), kx);
            load_v8<KT, HD>(vbase, slot, part * 8, vx);
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
                    const float corr = __expf(mx[g] - mn);      // exp(-inf) = 0 on the first token
                    const float p = __expf(s[g] - mn);
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
            const float ca = (mx[g] == -INFINITY) ? 0.0f : __expf(mx[g] - mn);
            const float cb = (mo == -INFINITY) ? 0.0f : __expf(mo - mn);
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
            const float c = (s_m[w][g] == -INFINITY) ? 0.0f : __expf(s_m[w][g] - mn);
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
                                    RowMap rm, int H, int S, float* __restrict__ out, int ldo,
                                    uint16_t* __restrict__ out_h = nullptr, uint16_t* __restrict__ out_l = nullptr) {
    const int r = blockIdx.x, h = blockIdx.y, e = threadIdx.x;
    int seq, pos;
    if (!row_lookup(rm, r, seq, pos)) return;
    const size_t base = ((size_t)r * H + h) * S;
    float mn = -INFINITY;
    for (int s = 0; s < S; ++s) mn = fmaxf(mn, part_ml[(base + s) * 2]);
    float a = 0.0f, ll = 0.0f;
    for (int s = 0; s < S; ++s) {
        const float m = part_ml[(base + s) * 2];
        const float c = (m == -INFINITY) ? 0.0f : __expf(m - mn);
        a += part_acc[(base + s) * HD + e] * c;
        ll += part_ml[(base + s) * 2 + 1] * c;
    }
    const float y = a / ll;
    if (out_h) {                // as hi + lo bf16 halves, for the MFMA projection that follows
        const uint16_t hi = f2bf(y);
        out_h[(size_t)r * ldo + h * HD + e] = hi;
        out_l[(size_t)r * ldo + h * HD + e] = f2bf(y - bf2f(hi));
    } else {
        out[(size_t)r * ldo + h * HD + e] = y;
    }
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
    KT* kpage = pool_layer + (size_t)page * page_elts;
    KT* vpage = pool_layer + (size_t)page * page_elts + (size_t)Hkv * RSD_PAGE * HD;
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
                KT* khead = kpage + (size_t)(h - H) * RSD_PAGE * HD;
                st1(khead + k_off8<KT, HD>(slot, i & ~7) + (i & 7), ra);
                st1(khead + k_off8<KT, HD>(slot, (i + HALF) & ~7) + (i & 7), rb);
            }
        } else {
            const int j = idx - nq - nk, hk = j / HD, e = j - hk * HD;
            st1(v_addr<KT, HD>(vpage + (size_t)hk * RSD_PAGE * HD, slot, e), row[(H + Hkv) * HD + j]);
        }
    }
}

// ---------------------------------------------------------------------------
// Single-token decode: rotary embedding, cache write and attention in one
// launch.  grid = (sequences, kv heads, S).  Every block rotates the group's
// queries itself; the cached positions 0..pos-1 are cut into S page ranges, one
// per block, and the new token (position pos) is added by the block of the
// last range straight from registers, after rounding its key and value to the
// cache's storage type, and written to the cache by that block.  With S > 1
// each block leaves a partial (max, sum, accumulator) for attn_combine_kernel.
// (Merging inside this kernel would need device-scope fences between blocks,
// which on this multi-die part write back and invalidate L2 and cost far more
// than a second launch.)
template <typename KT> __device__ __forceinline__ float round_store(float v);
template <> __device__ __forceinline__ float round_store<float>(float v) { return v; }
template <> __device__ __forceinline__ float round_store<bf16_t>(float v) { return bf2f(f2bf(v)); }

__device__ __forceinline__ void store8(float* p, const float v[8]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void store8(bf16_t* p, const float v[8]) {
    uint4 r;
    r.x = (uint32_t)f2bf(v[0]) | ((uint32_t)f2bf(v[1]) << 16);
    r.y = (uint32_t)f2bf(v[2]) | ((uint32_t)f2bf(v[3]) << 16);
    r.z = (uint32_t)f2bf(v[4]) | ((uint32_t)f2bf(v[5]) << 16);
    r.w = (uint32_t)f2bf(v[6]) | ((uint32_t)f2bf(v[7]) << 16);
    *reinterpret_cast<uint4*>(p) = r;
}

// rotate the 8 elements [e0, e0+8) of one head vector `src` (fp32, HD long)
template <int HD>
__device__ __forceinline__ void rope8(const float* __restrict__ src, const float2* __restrict__ cs, int e0, float o[8]) {
    constexpr int HALF = HD / 2;
    float own[8], oth[8];
    load8(src + e0, own);
    const bool first = e0 < HALF;
    load8(src + (first ? e0 + HALF : e0 - HALF), oth);
    const int i0 = first ? e0 : e0 - HALF;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float2 c = cs[i0 + e];
        o[e] = first ? (own[e] * c.x - oth[e] * c.y) : (own[e] * c.x + oth[e] * c.y);
    }
}

template <typename KT, int HD, int G>
__global__ __launch_bounds__(256) void attn_decode_kernel(const float* __restrict__ qkv, int ldq,
                                                          KT* __restrict__ pool_layer,
                                                          const int* __restrict__ block_table, int max_pages,
                                                          const int* __restrict__ kv_len,
                                                          const int* __restrict__ active,
                                                          const float2* __restrict__ rope, int H, int Hkv, int S,
                                                          float scale, float* __restrict__ out, int ldo,
                                                          float* __restrict__ part_acc, float* __restrict__ part_ml,
                                                          const int* __restrict__ row_seq) {
    constexpr int LPT = HD / 8, TPW = 64 / LPT;
    constexpr int ITERS = RSD_PAGE / TPW > 0 ? RSD_PAGE / TPW : 1;
    const int r = blockIdx.x, hk = blockIdx.y, sp = blockIdx.z;
    const int seq = row_seq ? row_seq[r] : r;       // packed rows: the sequence this row stands for (< 0: none)
    if (seq < 0 || !active[seq]) return;
    const int pos = kv_len[seq];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int part = lane % LPT, tsub = lane / LPT;
    const float* row = qkv + (size_t)r * ldq;
    const float2* cs = rope + (size_t)pos * (HD / 2);

    float q[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        rope8<HD>(row + (hk * G + g) * HD, cs, part * 8, q[g]);
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
    auto absorb = [&](const float kx[8], const float vx[8], bool valid) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float d = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) d += q[g][e] * kx[e];
#pragma unroll
            for (int off = 1; off < LPT; off <<= 1) d += __shfl_xor(d, off, RSD_WAVE);
            if (valid) {
                const float mn = fmaxf(mx[g], d);
                const float corr = __expf(mx[g] - mn);
                const float p = __expf(d - mn);
                l[g] = l[g] * corr + p;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[g][e] = acc[g][e] * corr + p * vx[e];
                mx[g] = mn;
            }
        }
    };

    const int n_pages = (pos + RSD_PAGE - 1) / RSD_PAGE;      // pages holding cached positions 0..pos-1
    const int pps = (n_pages + S - 1) / S;
    const int p_begin = sp * pps, p_end = min(n_pages, p_begin + pps);
    const int* bt = block_table + (size_t)seq * max_pages;
    const size_t page_elts = (size_t)2 * Hkv * RSD_PAGE * HD;
    const size_t head_off = (size_t)hk * RSD_PAGE * HD, v_off = (size_t)Hkv * RSD_PAGE * HD;

    for (int pg = p_begin + wave; pg < p_end; pg += 4) {
        const KT* kbase = pool_layer + (size_t)bt[pg] * page_elts + head_off;
        float kx[ITERS][8], vx[ITERS][8];
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int slot = it * TPW + tsub;
            load8(kbase + k_off8<KT, HD>(slot, part * 8), kx[it]);
            load_v8<KT, HD>(kbase + v_off, slot, part * 8, vx[it]);
        }
#pragma unroll
        for (int it = 0; it < ITERS; ++it) absorb(kx[it], vx[it], pg * RSD_PAGE + it * TPW + tsub < pos);
    }
    if (sp == S - 1 && wave == 0) {
        // the new token: rotate its key, round key and value as the cache stores them, write, attend
        float kn[8], vn[8];
        rope8<HD>(row + (H + hk) * HD, cs, part * 8, kn);
        load8(row + (H + Hkv + hk) * HD + part * 8, vn);
#pragma unroll
        for (int e = 0; e < 8; ++e) { kn[e] = round_store<KT>(kn[e]); vn[e] = round_store<KT>(vn[e]); }
        if (tsub == 0) {
            KT* khead = pool_layer + (size_t)bt[pos / RSD_PAGE] * page_elts + head_off;
            store8(khead + k_off8<KT, HD>(pos % RSD_PAGE, part * 8), kn);
#pragma unroll
            for (int e = 0; e < 8; ++e) st1(v_addr<KT, HD>(khead + v_off, pos % RSD_PAGE, part * 8 + e), vn[e]);
        }
        absorb(kn, vn, tsub == 0);
    }

#pragma unroll
    for (int off = LPT; off < 64; off <<= 1) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float mo = __shfl_xor(mx[g], off, RSD_WAVE);
            const float lo = __shfl_xor(l[g], off, RSD_WAVE);
            const float mn = fmaxf(mx[g], mo);
            const float ca = (mx[g] == -INFINITY) ? 0.0f : __expf(mx[g] - mn);
            const float cb = (mo == -INFINITY) ? 0.0f : __expf(mo - mn);
            l[g] = l[g] * ca + lo * cb;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float ao = __shfl_xor(acc[g][e], off, RSD_WAVE);
                acc[g][e] = acc[g][e] * ca + ao * cb;
            }
            mx[g] = mn;
        }
    }
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
    for (int idx = tid; idx < G * HD; idx += 256) {
        const int g = idx / HD, e = idx - g * HD;
        const float mn = fmaxf(fmaxf(s_m[0][g], s_m[1][g]), fmaxf(s_m[2][g], s_m[3][g]));
        float a = 0.0f, ll = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float c = (s_m[w][g] == -INFINITY) ? 0.0f : __expf(s_m[w][g] - mn);
            a += s_acc[w][g][e] * c;
            ll += s_l[w][g] * c;
        }
        const int h = hk * G + g;
        if (S == 1) {
            out[(size_t)r * ldo + h * HD + e] = a / ll;
        } else {
            const size_t pi = ((size_t)r * H + h) * S + sp;
            part_acc[pi * HD + e] = a;
            if (e == 0) { part_ml[pi * 2] = mn; part_ml[pi * 2 + 1] = ll; }
        }
    }
}

// ---------------------------------------------------------------------------
// MFMA single-token decode attention for bf16 caches, head_dim 128.
//
// One block per (sequence, kv head, split); each of its NW waves takes pages
// round-robin.  Per page (16 tokens) and wave:
//   S^T[token][head] = K . Q^T      v_mfma_f32_16x16x32_bf16, 4 steps over head_dim;
//                                   K straight from HBM (64 contiguous bytes per lane),
//                                   Q^T of the group's G heads padded to 16 columns
//   online softmax per head (column), in the accumulator layout
//   O[head][col]   += P . V         v_mfma_f32_16x16x16bf16_1k, 8 column blocks; the
//                                   softmax output already sits in the A-operand layout,
//                                   V^T pages give 8 contiguous bytes per lane
// The fp32 operands (rotated, scaled q and the probabilities) enter as hi + lo
// bf16 pairs, two MFMAs each, so they keep 16 significant bits; K and V are
// bf16 in the cache and enter exactly.  The new token is added from registers
// by wave 0 of the last split, which also writes it to the cache.  With S > 1
// the partials are merged by attn_combine_kernel.
typedef __attribute__((ext_vector_type(8))) __bf16 abf16x8_t;
typedef __attribute__((ext_vector_type(4))) short as16x4_t;
typedef __attribute__((ext_vector_type(4))) float af32x4_t;

__device__ __forceinline__ void split_hi_lo8(const float x[8], abf16x8_t& hi, abf16x8_t& lo) {
    uint32_t h[4], l[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const uint16_t h0 = f2bf(x[2 * e]), h1 = f2bf(x[2 * e + 1]);
        const uint16_t l0 = f2bf(x[2 * e] - bf2f(h0)), l1 = f2bf(x[2 * e + 1] - bf2f(h1));
        h[e] = (uint32_t)h0 | ((uint32_t)h1 << 16);
        l[e] = (uint32_t)l0 | ((uint32_t)l1 << 16);
    }
    hi = __builtin_bit_cast(abf16x8_t, make_uint4(h[0], h[1], h[2], h[3]));
    lo = __builtin_bit_cast(abf16x8_t, make_uint4(l[0], l[1], l[2], l[3]));
}

// Where the projected q, k, v of the rows come from when the projection's K slices have not been added up yet:
// part[z][row][col], z < ks, slices `stride` floats apart (the layout the few-row and the tile GEMM leave).
struct QkvParts { const float* part; int ks; size_t stride; };

// PARTS: the kernel adds the K slices of the QKV projection itself (ascending, like the finish kernels) while
// its first pages are in flight, which saves the launch of a finish kernel per layer; `qkv` is then unused.
// 16 bytes of a cache page in the decode kernel: every page is read once per launch, so the loads are marked
// non-temporal and leave the caches to what is used again (batch 256 at 4096 tokens: 392 -> 367 us per 7B
// layer, 200 -> 180 us per 1.5B layer; the 7B iteration at batch 64: 5.27 -> 4.94 ms)
#ifndef RSD_KV_NT
#define RSD_KV_NT 1
#endif
__device__ __forceinline__ uint4 load_kv16(const bf16_t* p) {
#if RSD_KV_NT
    typedef uint32_t nt_u32x4 __attribute__((ext_vector_type(4)));
    const nt_u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const nt_u32x4*>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
#else
    return *reinterpret_cast<const uint4*>(p);
#endif
}
template <int G, int NW, bool PARTS>
__global__ __launch_bounds__(NW * 64, NW == 4 ? 2 : 1) void attn_decode_mfma_kernel(const float* __restrict__ qkv, int ldq,
                                                                   bf16_t* __restrict__ pool_layer,
                                                                   const int* __restrict__ block_table, int max_pages,
                                                                   const int* __restrict__ kv_len,
                                                                   const int* __restrict__ active,
                                                                   const float2* __restrict__ rope, int H, int Hkv,
                                                                   int S, float scale, float* __restrict__ out, int ldo,
                                                                   float* __restrict__ part_acc, float* __restrict__ part_ml,
                                                                   uint16_t* __restrict__ out_h, uint16_t* __restrict__ out_l,
                                                                   const int* __restrict__ row_seq, QkvParts qp) {
    constexpr int HD = 128;
    const int r = blockIdx.x, hk = blockIdx.y, sp = blockIdx.z;
    const int seq_raw = row_seq ? row_seq[r] : r;   // packed rows: the sequence this row stands for (< 0: none)
    const int seq = max(seq_raw, 0);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Pages are dealt round-robin: the i-th page of (split sp, wave w) is sp + S * (w + NW * i), whatever
    // the position turns out to be.  So the table entries (lane i holds the i-th; entries beyond the
    // sequence are never used) are requested together with the position, not after it.
    const int is_active = seq_raw >= 0 && active[seq];
    const int pos = kv_len[seq];
    const int pg0 = sp + S * wave, pg_step = S * NW;
    int bt_mine = -1;
    if (pg0 + pg_step * lane < max_pages) bt_mine = block_table[(size_t)seq * max_pages + pg0 + pg_step * lane];
    if (!is_active) return;
    const int l16 = lane & 15, c = lane >> 4;
    const float* row = qkv + (size_t)r * ldq;
    const float2* cs = rope + (size_t)pos * (HD / 2);

    const int n_pages = (pos + RSD_PAGE - 1) / RSD_PAGE;      // pages holding cached positions 0..pos-1
    const int* bt = block_table + (size_t)seq * max_pages;
    const size_t page_elts = (size_t)2 * Hkv * RSD_PAGE * HD;
    const size_t head_off = (size_t)hk * RSD_PAGE * HD, v_off = (size_t)Hkv * RSD_PAGE * HD;

    // operands of one page (tiled page layout, see KvTiled): K chunk j of token l16 = K[l16][j*32 + c*8 ..+8] is
    // the lane's 16 bytes of the j-th KB of the key block; the lane's 16 bytes of the m-th KB of the value
    // block hold V^T[(2m)*16 + l16][c*4 ..+4] (.x, .y) and V^T[(2m+1)*16 + l16][c*4 ..+4] (.z, .w)
    uint4 kc[4], kn[4];
    uint4 vc[4], vn[4];
    auto fetch_phys = [&](int phys, uint4 k[4], uint4 v[4]) {
        const bf16_t* kb = pool_layer + (size_t)phys * page_elts + head_off;
#pragma unroll
        for (int j = 0; j < 4; ++j) k[j] = load_kv16(kb + (j * 64 + lane) * 8);
#pragma unroll
        for (int m = 0; m < 4; ++m) v[m] = load_kv16(kb + v_off + (m * 64 + lane) * 8);
    };
    // i-th page of this wave (i < 64: a wave never holds more than 64 pages)
    auto fetch = [&](int i, uint4 k[4], uint4 v[4]) { fetch_phys(__shfl(bt_mine, i, RSD_WAVE), k, v); };
    uint4 k2[4];
    uint4 v2[4];                 // two pages in flight ahead of the one being used
    int pg = pg0, it = 0;
    if (pg < n_pages) fetch(0, kc, vc);
    if (pg + pg_step < n_pages) fetch(1, kn, vn);

    // q of the group's heads, k and v of this KV head for the row: straight from qkv, or summed into LDS
    __shared__ float s_row[PARTS ? (G + 2) * HD : 1];
    const float *src_q, *src_k, *src_v;
    if constexpr (PARTS) {
        for (int i = tid; i < (G + 2) * HD; i += NW * 64) {
            const int col = i < G * HD ? hk * G * HD + i : (i < (G + 1) * HD ? (H + hk) * HD + (i - G * HD) : (H + Hkv + hk) * HD + (i - (G + 1) * HD));
            const float* p = qp.part + (size_t)r * ldq + col;
            float a = 0.0f;
            int z = 0;
            for (; z + 4 <= qp.ks; z += 4) {
                const float b0 = p[(size_t)z * qp.stride], b1 = p[(size_t)(z + 1) * qp.stride];
                const float b2 = p[(size_t)(z + 2) * qp.stride], b3 = p[(size_t)(z + 3) * qp.stride];
                a += b0; a += b1; a += b2; a += b3;
            }
            for (; z < qp.ks; ++z) a += p[(size_t)z * qp.stride];
            s_row[i] = a;
        }
        __syncthreads();
        src_q = s_row; src_k = s_row + G * HD; src_v = s_row + (G + 1) * HD;
    } else {
        src_q = row + hk * G * HD; src_k = row + (H + hk) * HD; src_v = row + (H + Hkv + hk) * HD;
    }
    // rotated, scaled queries of the group, computed once per block and kept in LDS as hi + lo bf16
    // (rows >= G stay zero); the waves read their MFMA operands from there for every page
    __shared__ __attribute__((aligned(16))) uint16_t s_qh[16][HD + 8];
    __shared__ __attribute__((aligned(16))) uint16_t s_ql[16][HD + 8];
    for (int idx = tid; idx < 16 * (HD / 2); idx += NW * 64) {
        const int g = idx / (HD / 2), e = idx - g * (HD / 2);
        float ra = 0.0f, rb = 0.0f;
        if (g < G) {
            const float* qe = src_q + g * HD + e;
            const float a = qe[0], b = qe[HD / 2];
            const float2 t = cs[e];
            ra = (a * t.x - b * t.y) * scale;
            rb = (b * t.x + a * t.y) * scale;
        }
        const uint16_t ha = f2bf(ra), hb = f2bf(rb);
        s_qh[g][e] = ha; s_qh[g][e + HD / 2] = hb;
        s_ql[g][e] = f2bf(ra - bf2f(ha)); s_ql[g][e + HD / 2] = f2bf(rb - bf2f(hb));
    }
    __syncthreads();

    // the new token as a pseudo page whose only valid token is row 0 (wave 0 of the last split):
    // rotate its key, round key and value to bf16 as the cache stores them, write them to the cache.
    // Done before the page loop so that its loads overlap the first page fetches.
    const bool owns_new = (sp == S - 1 && wave == 0);
    uint4 k1[4];
    uint4 v1[4];
    if (owns_new) {
        bf16_t* kb = pool_layer + (size_t)bt[pos / RSD_PAGE] * page_elts + head_off;
        const int slot = pos % RSD_PAGE;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float kv[8];
            rope8<HD>(src_k, cs, j * 32 + c * 8, kv);
            uint4 pk;
            pk.x = (uint32_t)f2bf(kv[0]) | ((uint32_t)f2bf(kv[1]) << 16);
            pk.y = (uint32_t)f2bf(kv[2]) | ((uint32_t)f2bf(kv[3]) << 16);
            pk.z = (uint32_t)f2bf(kv[4]) | ((uint32_t)f2bf(kv[5]) << 16);
            pk.w = (uint32_t)f2bf(kv[6]) | ((uint32_t)f2bf(kv[7]) << 16);
            if (l16 == 0) *reinterpret_cast<uint4*>(kb + kv_tiled_k(slot, j * 32 + c * 8)) = pk;
            k1[j] = (l16 == 0) ? pk : make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const uint16_t va = f2bf(src_v[(2 * m) * 16 + l16]);
            const uint16_t vb = f2bf(src_v[(2 * m + 1) * 16 + l16]);
            if (c == 0) {
                kb[v_off + kv_tiled_v(slot, (2 * m) * 16 + l16)].v = va;
                kb[v_off + kv_tiled_v(slot, (2 * m + 1) * 16 + l16)].v = vb;
            }
            v1[m] = make_uint4(c == 0 ? (uint32_t)va : 0u, 0u, c == 0 ? (uint32_t)vb : 0u, 0u);
        }
    }

    // Scores come out transposed, S^T[token c*4+i][head l16], which is at once the layout of P^T as the
    // B operand of O^T = V^T P^T.  So every lane works for ONE head (l16): its running maximum, sum and
    // rescaling factor are its own, and sums over tokens run over i and over the four 16-lane rows.
    float m_run = -INFINITY, l_run = 0.0f;
    af32x4_t o[8];                                          // o[nb][i] = O[head l16][nb*16 + c*4 + i]
#pragma unroll
    for (int nb = 0; nb < 8; ++nb) o[nb] = af32x4_t{0.f, 0.f, 0.f, 0.f};

    // one page: tokens c*4+i of it are valid iff (vmask >> i) & 1
    auto process = [&](const uint4 k[4], const uint4 v[4], int vmask) {
        af32x4_t s = {0.f, 0.f, 0.f, 0.f}, s2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const abf16x8_t ka = __builtin_bit_cast(abf16x8_t, k[j]);
            const abf16x8_t qlo = __builtin_bit_cast(abf16x8_t, *reinterpret_cast<const uint4*>(&s_ql[l16][j * 32 + c * 8]));
            const abf16x8_t qhi = __builtin_bit_cast(abf16x8_t, *reinterpret_cast<const uint4*>(&s_qh[l16][j * 32 + c * 8]));
            s2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qlo, s2, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qhi, s, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) s[i] += s2[i];
        float mloc = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4; ++i) if ((vmask >> i) & 1) mloc = fmaxf(mloc, s[i]);
        mloc = rows4_max(mloc);
        const float m_new = fmaxf(m_run, mloc);
        const float corr = (m_run == -INFINITY) ? 0.0f : __expf(m_run - m_new);
        float p[4], lsum = 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            p[i] = (((vmask >> i) & 1) && m_new > -INFINITY) ? __expf(s[i] - m_new) : 0.0f;
            lsum += p[i];
        }
        lsum = rows4_sum(lsum);
        l_run = l_run * corr + lsum;
        m_run = m_new;
        uint16_t ph[4], pl[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { ph[i] = f2bf(p[i]); pl[i] = f2bf(p[i] - bf2f(ph[i])); }
        const as16x4_t pa = __builtin_bit_cast(as16x4_t, make_uint2((uint32_t)ph[0] | ((uint32_t)ph[1] << 16), (uint32_t)ph[2] | ((uint32_t)ph[3] << 16)));
        const as16x4_t pb = __builtin_bit_cast(as16x4_t, make_uint2((uint32_t)pl[0] | ((uint32_t)pl[1] << 16), (uint32_t)pl[2] | ((uint32_t)pl[3] << 16)));
        // slots past the sequence hold whatever the pool held: zero them (0 * NaN would poison the sum)
        const uint32_t mk0 = ((vmask & 1) ? 0xFFFFu : 0u) | ((vmask & 2) ? 0xFFFF0000u : 0u);
        const uint32_t mk1 = ((vmask & 4) ? 0xFFFFu : 0u) | ((vmask & 8) ? 0xFFFF0000u : 0u);
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) {
#pragma unroll
            for (int i = 0; i < 4; ++i) o[nb][i] *= corr;
            const uint32_t vx = (nb & 1) ? v[nb >> 1].z : v[nb >> 1].x, vy = (nb & 1) ? v[nb >> 1].w : v[nb >> 1].y;
            const as16x4_t vb = __builtin_bit_cast(as16x4_t, make_uint2(vx & mk0, vy & mk1));
            o[nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vb, pb, o[nb], 0, 0, 0);
            o[nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vb, pa, o[nb], 0, 0, 0);
        }
    };

    if (owns_new) process(k1, v1, c == 0 ? 1 : 0);          // order of accumulation is free
    // Three register buffers take fixed turns (no copies between them: a copy would have to wait for
    // the load it copies): while page i is used, pages i+1 and i+2 are in flight.
    auto page_mask = [&](int page) {
        int vm = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) vm |= (page * RSD_PAGE + c * 4 + i < pos) ? (1 << i) : 0;
        return vm;
    };
    while (pg < n_pages) {
        if (pg + 2 * pg_step < n_pages) fetch(it + 2, k2, v2);
        process(kc, vc, page_mask(pg));
        pg += pg_step; ++it;
        if (pg >= n_pages) break;
        if (pg + 2 * pg_step < n_pages) fetch(it + 2, kc, vc);
        process(kn, vn, page_mask(pg));
        pg += pg_step; ++it;
        if (pg >= n_pages) break;
        if (pg + 2 * pg_step < n_pages) fetch(it + 2, kn, vn);
        process(k2, v2, page_mask(pg));
        pg += pg_step; ++it;
    }

    // ---- merge the waves of the block through LDS
    __shared__ __attribute__((aligned(16))) float s_o[NW][G][HD];
    __shared__ float s_m[NW][16], s_l[NW][16];
    if (c == 0) { s_m[wave][l16] = m_run; s_l[wave][l16] = l_run; }
    if (l16 < G) {
#pragma unroll
        for (int nb = 0; nb < 8; ++nb)
            *reinterpret_cast<float4*>(&s_o[wave][l16][nb * 16 + c * 4]) = make_float4(o[nb][0], o[nb][1], o[nb][2], o[nb][3]);
    }
    __syncthreads();
    for (int idx = tid; idx < G * HD; idx += NW * 64) {
        const int g = idx / HD, e = idx - g * HD;
        float mn = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) mn = fmaxf(mn, s_m[w][g]);
        float a = 0.0f, ll = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float cc = (s_m[w][g] == -INFINITY) ? 0.0f : __expf(s_m[w][g] - mn);
            a += s_o[w][g][e] * cc;
            ll += s_l[w][g] * cc;
        }
        const int h = hk * G + g;
        if (S == 1) {
            const float y = a / ll;
            if (out_h) {            // as hi + lo bf16 halves, for the MFMA projection that follows
                const uint16_t hi = f2bf(y);
                out_h[(size_t)r * ldo + h * HD + e] = hi;
                out_l[(size_t)r * ldo + h * HD + e] = f2bf(y - bf2f(hi));
            } else {
                out[(size_t)r * ldo + h * HD + e] = y;
            }
        } else {
            const size_t pi = ((size_t)r * H + h) * S + sp;
            part_acc[pi * HD + e] = a;
            if (e == 0) { part_ml[pi * 2] = mn; part_ml[pi * 2 + 1] = ll; }
        }
    }
}

// ---------------------------------------------------------------------------
// MFMA chunked-prefill attention for bf16 caches, head_dim 128.
//
// Runs after rope_kv_kernel has rotated q in place and written the chunk's
// keys/values to the cache.  One wave per work item = up to 4 consecutive rows
// (query tokens) of one sequence and one kv head: two 16-column tiles, a
// column being (row, head of the group); the wave walks every page up to the
// last row's position once and feeds both tiles from the same K / V^T
// registers.  Column (row, g) sees tokens <= position(row).  Same operand
// layouts and hi + lo splitting as attn_decode_mfma_kernel.
// gridDim.z = S > 1 (few rows over a long context): split sp walks its share of
// the pages and leaves a partial (max, sum, accumulator) per (row, head) for
// attn_combine_kernel, in the layout of the decode kernels.
template <int G>
__global__ __launch_bounds__(256, 2) void attn_prefill_mfma_kernel(const float* __restrict__ qkv, int ldq,
                                                                const bf16_t* __restrict__ pool_layer,
                                                                const int* __restrict__ block_table, int max_pages,
                                                                const int* __restrict__ row_seq,
                                                                const int* __restrict__ row_pos,
                                                                const int* __restrict__ item_row0,
                                                                const int* __restrict__ item_n, int n_items,
                                                                int H, int Hkv, float scale,
                                                                float* __restrict__ out, int ldo,
                                                                float* __restrict__ part_acc,
                                                                float* __restrict__ part_ml) {
    constexpr int HD = 128, NT = 2;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int item = blockIdx.x * 4 + wave, hk = blockIdx.y, sp = blockIdx.z, S = gridDim.z;
    if (item >= n_items) return;
    const int r0 = item_row0[item], n = item_n[item];
    const int seq = row_seq[r0], p0 = row_pos[r0];
    const int l16 = lane & 15, c = lane >> 4;
    const int* bt = block_table + (size_t)seq * max_pages;
    const size_t page_elts = (size_t)2 * Hkv * RSD_PAGE * HD;
    const size_t head_off = (size_t)hk * RSD_PAGE * HD, v_off = (size_t)Hkv * RSD_PAGE * HD;
    const int p_last = p0 + n - 1, n_pages = p_last / RSD_PAGE + 1;
    const int per = (n_pages + S - 1) / S;
    const int pg_lo = min(n_pages, sp * per), pg_hi = min(n_pages, pg_lo + per);     // this split's pages
    int bt_mine = ((pg_lo & ~63) + lane < n_pages) ? bt[(pg_lo & ~63) + lane] : -1;  // refreshed every 64 pages

    // column l16 of tile t: row r0 + 2t + l16 / 8, head l16 % 8
    const int g_col = l16 & 7;
    // Q^T operands of this wave's tiles live in LDS as hi + lo bf16: [wave][tile][hi|lo][16 columns][HD + 8]
    extern __shared__ __attribute__((aligned(16))) uint16_t s_qop[];
    constexpr int QSTR = HD + 8;
    uint16_t* qbase = s_qop + (size_t)wave * NT * 2 * 16 * QSTR;
    int pos_col[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int ri = 2 * t + (l16 >> 3);
        const bool live = ri < n && g_col < G;
        pos_col[t] = live ? p0 + ri : -1;                   // -1: the column sees no token
        uint16_t* qh_row = qbase + ((size_t)(t * 2 + 0) * 16 + l16) * QSTR;
        uint16_t* ql_row = qbase + ((size_t)(t * 2 + 1) * 16 + l16) * QSTR;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float qv[8];
            if (live) {
                load8(qkv + (size_t)(r0 + ri) * ldq + (hk * G + g_col) * HD + j * 32 + c * 8, qv);
#pragma unroll
                for (int e = 0; e < 8; ++e) qv[e] *= scale;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) qv[e] = 0.0f;
            }
            abf16x8_t h8, l8;
            split_hi_lo8(qv, h8, l8);
            *reinterpret_cast<uint4*>(qh_row + j * 32 + c * 8) = __builtin_bit_cast(uint4, h8);
            *reinterpret_cast<uint4*>(ql_row + j * 32 + c * 8) = __builtin_bit_cast(uint4, l8);
        }
    }
    // (each wave reads back only what it wrote itself: no block barrier needed)
    float m_run[NT], l_run[NT];
    af32x4_t o[NT][8];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        m_run[t] = -INFINITY; l_run[t] = 0.0f;
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) o[t][nb] = af32x4_t{0.f, 0.f, 0.f, 0.f};
    }

    uint4 kc[4], kn[4];
    uint4 vc[4], vn[4];
    auto fetch = [&](int pg, uint4 k[4], uint4 v[4]) {
        const int phys = __shfl(bt_mine, pg & 63, RSD_WAVE);
        const bf16_t* kb = pool_layer + (size_t)phys * page_elts + head_off;
#pragma unroll
        for (int j = 0; j < 4; ++j) k[j] = *reinterpret_cast<const uint4*>(kb + (j * 64 + lane) * 8);
#pragma unroll
        for (int m = 0; m < 4; ++m) v[m] = *reinterpret_cast<const uint4*>(kb + v_off + (m * 64 + lane) * 8);
    };
    auto do_page = [&](int pg, const uint4 k[4], const uint4 v[4]) {
        // slots past the last row's position hold whatever the pool held: zero those values
        int smask = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) smask |= (pg * RSD_PAGE + c * 4 + i <= p_last) ? (1 << i) : 0;
        const uint32_t mk0 = ((smask & 1) ? 0xFFFFu : 0u) | ((smask & 2) ? 0xFFFF0000u : 0u);
        const uint32_t mk1 = ((smask & 4) ? 0xFFFFu : 0u) | ((smask & 8) ? 0xFFFF0000u : 0u);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            af32x4_t s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const abf16x8_t ka = __builtin_bit_cast(abf16x8_t, k[j]);
                const abf16x8_t qhi = __builtin_bit_cast(abf16x8_t, *reinterpret_cast<const uint4*>(
                    qbase + ((size_t)(t * 2 + 0) * 16 + l16) * QSTR + j * 32 + c * 8));
                const abf16x8_t qlo = __builtin_bit_cast(abf16x8_t, *reinterpret_cast<const uint4*>(
                    qbase + ((size_t)(t * 2 + 1) * 16 + l16) * QSTR + j * 32 + c * 8));
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qlo, s, 0, 0, 0);
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qhi, s, 0, 0, 0);
            }
            int vmask = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) vmask |= (pg * RSD_PAGE + c * 4 + i <= pos_col[t]) ? (1 << i) : 0;
            float mloc = -INFINITY;
#pragma unroll
            for (int i = 0; i < 4; ++i) if ((vmask >> i) & 1) mloc = fmaxf(mloc, s[i]);
            mloc = fmaxf(mloc, __shfl_xor(mloc, 16, RSD_WAVE));
            mloc = fmaxf(mloc, __shfl_xor(mloc, 32, RSD_WAVE));
            const float m_new = fmaxf(m_run[t], mloc);
            const float corr = (m_run[t] == -INFINITY) ? 0.0f : __expf(m_run[t] - m_new);
            float p[4], lsum = 0.0f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                p[i] = (((vmask >> i) & 1) && m_new > -INFINITY) ? __expf(s[i] - m_new) : 0.0f;
                lsum += p[i];
            }
            lsum += __shfl_xor(lsum, 16, RSD_WAVE);
            lsum += __shfl_xor(lsum, 32, RSD_WAVE);
            l_run[t] = l_run[t] * corr + lsum;
            m_run[t] = m_new;
            uint16_t ph[4], pl[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { ph[i] = f2bf(p[i]); pl[i] = f2bf(p[i] - bf2f(ph[i])); }
            const as16x4_t pa = __builtin_bit_cast(as16x4_t, make_uint2((uint32_t)ph[0] | ((uint32_t)ph[1] << 16), (uint32_t)ph[2] | ((uint32_t)ph[3] << 16)));
            const as16x4_t pb = __builtin_bit_cast(as16x4_t, make_uint2((uint32_t)pl[0] | ((uint32_t)pl[1] << 16), (uint32_t)pl[2] | ((uint32_t)pl[3] << 16)));
            float cr[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) cr[i] = __shfl(corr, c * 4 + i, RSD_WAVE);
#pragma unroll
            for (int nb = 0; nb < 8; ++nb) {
#pragma unroll
                for (int i = 0; i < 4; ++i) o[t][nb][i] *= cr[i];
                const uint32_t vx = (nb & 1) ? v[nb >> 1].z : v[nb >> 1].x, vy = (nb & 1) ? v[nb >> 1].w : v[nb >> 1].y;
                const as16x4_t vb = __builtin_bit_cast(as16x4_t, make_uint2(vx & mk0, vy & mk1));
                o[t][nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pb, vb, o[t][nb], 0, 0, 0);
                o[t][nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa, vb, o[t][nb], 0, 0, 0);
            }
        }
    };
    auto prefetch = [&](int pg, uint4 k[4], uint4 v[4]) {     // pg < n_pages
        if ((pg & 63) == 0) bt_mine = (pg + lane < n_pages) ? bt[pg + lane] : -1;
        fetch(pg, k, v);
    };
    // two register buffers take turns (no copies between them: a copy would wait for the load)
    if (pg_lo < pg_hi) fetch(pg_lo, kc, vc);
    for (int pg = pg_lo; pg < pg_hi; pg += 2) {
        if (pg + 1 < pg_hi) prefetch(pg + 1, kn, vn);
        do_page(pg, kc, vc);
        if (pg + 1 >= pg_hi) break;
        if (pg + 2 < pg_hi) prefetch(pg + 2, kc, vc);
        do_page(pg + 1, kn, vn);
    }
    // accumulator row c*4+i of tile t is column (row r0 + 2t + (c*4+i)/8, head (c*4+i)%8)
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int col = c * 4 + i;
            const float den = __shfl(l_run[t], col, RSD_WAVE);
            const float mx = __shfl(m_run[t], col, RSD_WAVE);
            const int ri = 2 * t + (col >> 3), g = col & 7;
            if (ri < n && g < G) {
                if (S == 1) {
                    float* dst = out + (size_t)(r0 + ri) * ldo + (hk * G + g) * HD + l16;
                    const float inv = 1.0f / den;
#pragma unroll
                    for (int nb = 0; nb < 8; ++nb) dst[nb * 16] = o[t][nb][i] * inv;
                } else {
                    const size_t pi = ((size_t)(r0 + ri) * H + hk * G + g) * S + sp;
                    float* dst = part_acc + pi * HD + l16;
#pragma unroll
                    for (int nb = 0; nb < 8; ++nb) dst[nb * 16] = o[t][nb][i];
                    if (l16 == 0) { part_ml[pi * 2] = mx; part_ml[pi * 2 + 1] = den; }
                }
            }
        }
    }
}
