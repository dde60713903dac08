// Next-token choice from a row of fp32 logits: arg max (lowest id on ties), or
// temperature / nucleus (top-p) sampling by inverse CDF from a supplied uniform.
//
// Nucleus definition implemented here: with e_t = exp(x_t - max x), x = logit /
// temperature, the nucleus S is {t : e_t >= tau} for the largest tau whose set
// still holds at least top_p of the total mass (all ties at tau included); the
// draw walks S in ascending token id and returns the first token whose running
// mass exceeds u * mass(S).
//
// No sort: tau is found by a three-level radix select over the bit patterns of
// the non-negative floats e_t (10 + 11 + 10 bits), each level a histogram of
// masses in LDS.  Masses are summed as 64-bit fixed point (e * 2^40), so every
// sum is exact, order-independent and reproducible from run to run.
#pragma once
#include "common.cuh"

typedef unsigned long long u64_t;

__device__ __forceinline__ u64_t shfl_up_u64(u64_t v, int d) {
    const unsigned lo = __shfl_up((unsigned)v, d, RSD_WAVE), hi = __shfl_up((unsigned)(v >> 32), d, RSD_WAVE);
    return ((u64_t)hi << 32) | lo;
}
__device__ __forceinline__ u64_t shfl_xor_u64(u64_t v, int d) {
    const unsigned lo = __shfl_xor((unsigned)v, d, RSD_WAVE), hi = __shfl_xor((unsigned)(v >> 32), d, RSD_WAVE);
    return ((u64_t)hi << 32) | lo;
}
__device__ __forceinline__ u64_t wave_sum_u64(u64_t v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += shfl_xor_u64(v, off);
    return v;
}
__device__ __forceinline__ u64_t wave_incl_scan_u64(u64_t v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const u64_t o = shfl_up_u64(v, d);
        if (lane >= d) v += o;
    }
    return v;
}

// inclusive scan over the 1024 threads of the block; wtot is 16 u64 of LDS
__device__ __forceinline__ u64_t block1024_incl_scan_u64(u64_t v, u64_t* wtot) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const u64_t incl = wave_incl_scan_u64(v, lane);
    __syncthreads();
    if (lane == 63) wtot[wave] = incl;
    __syncthreads();
    u64_t base = 0;
    for (int w = 0; w < wave; ++w) base += wtot[w];
    return incl + base;
}

struct SampleArgs {
    const float* logits; int ld; int V;
    const float* u; const int* u_index; int u_stride;   // uniform of row r: u[r * u_stride + (u_index ? u_index[r] : 0)]
    float temperature, top_p;
    int sep_id; float sep_bias;                          // logit[sep_id] += sep_bias before anything else
    const int* active;                                   // nullable: rows with active[r] == 0 are skipped
    int* out;
};

__global__ __launch_bounds__(1024) void sample_kernel(SampleArgs a) {
    const int row = blockIdx.x;
    if (a.active && !a.active[row]) return;
    const float* lg = a.logits + (size_t)row * a.ld;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int V = a.V;
    __shared__ u64_t hist[2048];
    __shared__ u64_t wtot[16];
    __shared__ float fred[16];
    __shared__ int ired[16];
    __shared__ u64_t sh_above;
    __shared__ int sh_bin, sh_span, sh_last;
    __shared__ u64_t sh_base;

    // ------------------------------------------------------------ arg max
    if (a.temperature == 0.0f) {
        float bv = -INFINITY; int bi = 0x7FFFFFFF;
        for (int i = tid; i < V; i += 1024) {
            const float v = lg[i] + (i == a.sep_id ? a.sep_bias : 0.0f);
            if (v > bv) { bv = v; bi = i; }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float ov = __shfl_xor(bv, off, RSD_WAVE);
            const int oi = __shfl_xor(bi, off, RSD_WAVE);
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        }
        if (lane == 0) { fred[wave] = bv; ired[wave] = bi; }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < 16; ++w)
                if (fred[w] > bv || (fred[w] == bv && ired[w] < bi)) { bv = fred[w]; bi = ired[w]; }
            a.out[row] = bi;
        }
        return;
    }

    // ------------------------------------------------------------ nucleus
    const float T = a.temperature;
    auto xval = [&](int i) -> float { return (lg[i] + (i == a.sep_id ? a.sep_bias : 0.0f)) / T; };
    float mx = -INFINITY;
    for (int i = tid; i < V; i += 1024) mx = fmaxf(mx, xval(i));
    mx = wave_max(mx);
    if (lane == 0) fred[wave] = mx;
    __syncthreads();
    mx = fred[0];
    for (int w = 1; w < 16; ++w) mx = fmaxf(mx, fred[w]);
    auto eval = [&](int i) -> float { return expf(xval(i) - mx); };
    auto fixq = [](float e) -> u64_t { return (u64_t)(e * 1099511627776.0f); };   // e * 2^40, e in [0, 1]

    // level 1 histogram doubles as the total
    for (int i = tid; i < 2048; i += 1024) hist[i] = 0;
    __syncthreads();
    for (int i = tid; i < V; i += 1024) {
        const float e = eval(i);
        atomicAdd(&hist[__float_as_uint(e) >> 21], fixq(e));
    }
    __syncthreads();
    u64_t above = 0;        // mass strictly above the bin being refined
    u64_t thr = 0;
    uint32_t prefix = 0;    // key bits fixed so far
    for (int level = 0; level < 3; ++level) {
        // thread t owns bins 2047-2t and 2046-2t: a prefix scan over t is a suffix sum over bins
        const u64_t h_hi = hist[2047 - 2 * tid], h_lo = hist[2046 - 2 * tid];
        const u64_t incl = block1024_incl_scan_u64(h_hi + h_lo, wtot);
        if (level == 0) {
            __syncthreads();
            if (tid == 1023) sh_base = incl;       // total mass
            __syncthreads();
            const double t = (double)a.top_p * (double)sh_base;
            thr = (u64_t)ceil(t);
            if (thr < 1) thr = 1;
            if (thr > sh_base) thr = sh_base;
        }
        const u64_t A = above + (incl - h_hi - h_lo);
        const u64_t s_hi = A + h_hi, s_lo = s_hi + h_lo;
        __syncthreads();
        if (A < thr && s_hi >= thr) { sh_bin = 2047 - 2 * tid; sh_above = A; }
        else if (s_hi < thr && s_lo >= thr) { sh_bin = 2046 - 2 * tid; sh_above = s_hi; }
        __syncthreads();
        above = sh_above;
        const uint32_t bin = (uint32_t)sh_bin;
        if (level == 0) prefix = bin << 21;
        else if (level == 1) prefix |= bin << 10;
        else prefix |= bin;
        if (level == 2) break;
        __syncthreads();
        for (int i = tid; i < 2048; i += 1024) hist[i] = 0;
        __syncthreads();
        const uint32_t mask = (level == 0) ? 0xFFE00000u : 0xFFFFFC00u;
        for (int i = tid; i < V; i += 1024) {
            const float e = eval(i);
            const uint32_t key = __float_as_uint(e);
            if ((key & mask) == prefix)
                atomicAdd(&hist[level == 0 ? ((key >> 10) & 0x7FFu) : (key & 0x3FFu)], fixq(e));
        }
        __syncthreads();
    }
    // prefix is now the bit pattern of tau; mass(S) = above + hist[last bin]
    const uint32_t tau = prefix;
    const u64_t zs = above + hist[tau & 0x3FFu];
    const float uu = a.u[(size_t)row * a.u_stride + (a.u_index ? a.u_index[row] : 0)];
    const u64_t target = (u64_t)floor((double)uu * (double)zs);   // running > u * Z  <=>  running > floor(u * Z)

    // masses of 256 contiguous id spans, in id order
    const int span = (V + 255) / 256;
    __syncthreads();
    u64_t* span_sum = hist;          // reuse: 256 entries
    int last_member = -1;
    for (int sp = wave * 16; sp < wave * 16 + 16; ++sp) {
        const int s0 = sp * span, s1 = min(V, s0 + span);
        u64_t acc = 0;
        for (int i = s0 + lane; i < s1; i += 64) {
            const float e = eval(i);
            if (__float_as_uint(e) >= tau) { acc += fixq(e); last_member = max(last_member, i); }
        }
        acc = wave_sum_u64(acc);
        if (lane == 0) span_sum[sp] = acc;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) last_member = max(last_member, __shfl_xor(last_member, off, RSD_WAVE));
    if (lane == 0) ired[wave] = last_member;
    __syncthreads();
    if (tid == 0) {
        int lm = -1;
        for (int w = 0; w < 16; ++w) lm = max(lm, ired[w]);
        sh_last = lm;
        sh_span = -1;
    }
    const u64_t sv = (tid < 256) ? span_sum[tid] : 0;
    const u64_t sincl = block1024_incl_scan_u64(sv, wtot);
    __syncthreads();
    if (tid < 256 && sincl > target && sincl - sv <= target) { sh_span = tid; sh_base = sincl - sv; }
    __syncthreads();
    if (sh_span < 0) { if (tid == 0) a.out[row] = sh_last; return; }
    if (wave == 0) {
        const int s0 = sh_span * span, s1 = min(V, s0 + span);
        u64_t base = sh_base;
        for (int j = s0; j < s1; j += 64) {
            const int i = j + lane;
            u64_t q = 0;
            if (i < s1) { const float e = eval(i); if (__float_as_uint(e) >= tau) q = fixq(e); }
            const u64_t run = base + wave_incl_scan_u64(q, lane);
            const u64_t hit = __ballot(run > target);
            if (hit) {
                if (lane == 0) a.out[row] = j + (__ffsll((long long)hit) - 1);
                return;
            }
            base = __shfl(((unsigned)(run >> 32)), 63, RSD_WAVE);
            base = (base << 32) | __shfl((unsigned)run, 63, RSD_WAVE);
        }
        if (lane == 0) a.out[row] = sh_last;
    }
}
