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
// masses.  Masses are summed as 64-bit fixed point (e * 2^40), so every sum is
// exact, order-independent and reproducible from run to run.
//
// A row is spread over SMP_NB blocks (one vocabulary span each) so that a
// batch of one still uses many compute units; the phases are separate
// launches:  A  per-block max (or arg max) ->  B  level-1 histogram ->
// C  level 2 ->  D  level 3 ->  E  per-block nucleus mass ->  F  locate the
// draw, append the token to its sequence, clear the histograms.
#pragma once
#include "common.h"
#include "misc.h"

typedef unsigned long long u64_t;

constexpr int SMP_NB = 64;      // blocks per row
constexpr int SMP_T = 256;      // threads per block
constexpr int SMP_BINS = 2048;  // histogram size of every level (level 1 and 3 use 1024)

__device__ __forceinline__ u64_t shfl_up_u64(u64_t v, int d) {
    const unsigned lo = __shfl_up((unsigned)v, d, RSD_WAVE), hi = __shfl_up((unsigned)(v >> 32), d, RSD_WAVE);
    return ((u64_t)hi << 32) | lo;
}
__device__ __forceinline__ u64_t shfl_xor_u64(u64_t v, int d) {
    const unsigned lo = __shfl_xor((unsigned)v, d, RSD_WAVE), hi = __shfl_xor((unsigned)(v >> 32), d, RSD_WAVE);
    return ((u64_t)hi << 32) | lo;
}
__device__ __forceinline__ u64_t shfl_u64(u64_t v, int src) {
    const unsigned lo = __shfl((unsigned)v, src, RSD_WAVE), hi = __shfl((unsigned)(v >> 32), src, RSD_WAVE);
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
// inclusive scan over the 256 threads of a block; wtot is 4 u64 of LDS
__device__ __forceinline__ u64_t block256_incl_scan_u64(u64_t v, u64_t* wtot) {
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
    int* out;                                            // nullable when the result is appended
    // workspace, per row: pmax[SMP_NB], pidx[SMP_NB], hist[3][SMP_BINS], psum[SMP_NB], sel[8]
    float* pmax; int* pidx; u64_t* hist; u64_t* psum; u64_t* sel;
    // nullable: packed rows.  Row r then stands for sequence row_seq[r] (< 0: unused row); u, u_index, active and
    // the appended state are indexed by the sequence, logits, out and the workspace by the row
    const int* row_seq;
};
// the sequence of a row, or -1 when the row is unused or its sequence is not active
__device__ __forceinline__ int smp_seq(const SampleArgs& a, int row) {
    const int s = a.row_seq ? a.row_seq[row] : row;
    if (s < 0 || (a.active && !a.active[s])) return -1;
    return s;
}

// what phase F does with the chosen token besides (or instead of) storing it
struct AppendArgs {
    int enabled;                 // 0: off; 1: a token of a reasoning step; 2: a proposal of speculative regeneration
    SeqState st; int B, max_ctx, model;
    const int* forced; int sep_id, eos_id, step_cap, max_steps;
    int prop_stride;             // proposals recorded per step (mode 2): step_cap * proposals per round
};

__device__ __forceinline__ float smp_x(const SampleArgs& a, const float* lg, int i) {
    return (lg[i] + (i == a.sep_id ? a.sep_bias : 0.0f)) / a.temperature;
}
__device__ __forceinline__ u64_t smp_fix(float e) { return (u64_t)(e * 1099511627776.0f); }   // e * 2^40, e in [0, 1]

__device__ __forceinline__ float smp_row_max(const SampleArgs& a, int row, float* fred) {
    float m = -INFINITY;
    if (threadIdx.x < SMP_NB) m = a.pmax[(size_t)row * SMP_NB + threadIdx.x];
    m = wave_max(m);
    if ((threadIdx.x & 63) == 0) fred[threadIdx.x >> 6] = m;
    __syncthreads();
    return fmaxf(fmaxf(fred[0], fred[1]), fmaxf(fred[2], fred[3]));
}

// The bin (searching from the top) in which the running mass first reaches thr.
// hist has n_bins = 256 * P entries; `above` is the mass above this histogram on
// entry and the mass strictly above the chosen bin on exit.  Whole block calls.
template <int P>
__device__ __forceinline__ int smp_find_bin(const u64_t* hist, u64_t thr, u64_t& above, u64_t* wtot, int* s_bin,
                                            u64_t* s_above) {
    const int tid = threadIdx.x, top = 256 * P - 1 - tid * P;   // thread t owns bins top, top-1, ..., top-P+1
    u64_t h[P], loc = 0;
#pragma unroll
    for (int j = 0; j < P; ++j) { h[j] = hist[top - j]; loc += h[j]; }
    const u64_t incl = block256_incl_scan_u64(loc, wtot);
    u64_t run = above + (incl - loc);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < P; ++j) {
        if (run < thr && run + h[j] >= thr) { *s_bin = top - j; *s_above = run; }
        run += h[j];
    }
    __syncthreads();
    above = *s_above;
    return *s_bin;
}

// ---- phase A: per-block max of x (sampling) or arg max of the biased logits (greedy)
__global__ __launch_bounds__(SMP_T) void sample_max_kernel(SampleArgs a) {
    const int row = blockIdx.y, j = blockIdx.x, tid = threadIdx.x;
    const int seq = smp_seq(a, row);
    if (seq < 0) return;
    const float* lg = a.logits + (size_t)row * a.ld;
    const int span = (a.V + SMP_NB - 1) / SMP_NB, s0 = j * span, s1 = min(a.V, s0 + span);
    __shared__ float fred[4];
    __shared__ int ired[4];
    float bv = -INFINITY; int bi = 0x7FFFFFFF;
    const bool greedy = a.temperature == 0.0f;
    for (int i = s0 + tid; i < s1; i += SMP_T) {
        const float v = greedy ? lg[i] + (i == a.sep_id ? a.sep_bias : 0.0f) : smp_x(a, lg, i);
        if (v > bv) { bv = v; bi = i; }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(bv, off, RSD_WAVE);
        const int oi = __shfl_xor(bi, off, RSD_WAVE);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    if ((tid & 63) == 0) { fred[tid >> 6] = bv; ired[tid >> 6] = bi; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w)
            if (fred[w] > bv || (fred[w] == bv && ired[w] < bi)) { bv = fred[w]; bi = ired[w]; }
        a.pmax[(size_t)row * SMP_NB + j] = bv;
        a.pidx[(size_t)row * SMP_NB + j] = bi;
    }
}

// ---- phases B, C, D: one histogram level each (LEVEL = 0, 1, 2)
template <int LEVEL>
__global__ __launch_bounds__(SMP_T) void sample_hist_kernel(SampleArgs a) {
    const int row = blockIdx.y, j = blockIdx.x, tid = threadIdx.x;
    const int seq = smp_seq(a, row);
    if (seq < 0) return;
    const float* lg = a.logits + (size_t)row * a.ld;
    const int span = (a.V + SMP_NB - 1) / SMP_NB, s0 = j * span, s1 = min(a.V, s0 + span);
    __shared__ u64_t lh[SMP_BINS];
    __shared__ u64_t wtot[4];
    __shared__ float fred[4];
    __shared__ int s_bin;
    __shared__ u64_t s_above;
    u64_t* hist = a.hist + (size_t)row * 3 * SMP_BINS;
    u64_t* sel = a.sel + (size_t)row * 8;
    const float mx = smp_row_max(a, row, fred);
    uint32_t prefix = 0, mask = 0;
    if (LEVEL >= 1) {
        // every block repeats the (deterministic) search of the previous level
        u64_t above = (LEVEL == 1) ? 0 : sel[1];
        u64_t thr;
        if (LEVEL == 1) {
            u64_t loc = 0;
            for (int b = tid; b < 1024; b += SMP_T) loc += hist[b];
            const u64_t tot = block256_incl_scan_u64(loc, wtot);
            __syncthreads();
            if (tid == SMP_T - 1) s_above = tot;
            __syncthreads();
            const u64_t z = s_above;
            thr = (u64_t)ceil((double)a.top_p * (double)z);
            if (thr < 1) thr = 1;
            if (thr > z) thr = z;
            __syncthreads();
            const int bin = smp_find_bin<4>(hist, thr, above, wtot, &s_bin, &s_above);
            prefix = (uint32_t)bin << 21; mask = 0xFFE00000u;
            if (j == 0 && tid == 0) { sel[0] = thr; sel[1] = above; sel[2] = prefix; }
        } else {
            thr = sel[0];
            const int bin = smp_find_bin<8>(hist + SMP_BINS, thr, above, wtot, &s_bin, &s_above);
            prefix = (uint32_t)sel[2] | ((uint32_t)bin << 10); mask = 0xFFFFFC00u;
            if (j == 0 && tid == 0) { sel[3] = above; sel[4] = prefix; }
        }
    }
    for (int b = tid; b < SMP_BINS; b += SMP_T) lh[b] = 0;
    __syncthreads();
    for (int i = s0 + tid; i < s1; i += SMP_T) {
        const float e = expf(smp_x(a, lg, i) - mx);
        const uint32_t key = __float_as_uint(e);
        if (LEVEL == 0) atomicAdd(&lh[key >> 21], smp_fix(e));
        else if ((key & mask) == prefix) atomicAdd(&lh[LEVEL == 1 ? ((key >> 10) & 0x7FFu) : (key & 0x3FFu)], smp_fix(e));
    }
    __syncthreads();
    u64_t* gh = hist + LEVEL * SMP_BINS;
    for (int b = tid; b < SMP_BINS; b += SMP_T)
        if (lh[b]) atomicAdd(&gh[b], lh[b]);
}

// ---- phase E: tau and the draw target; per-block mass of the nucleus
__global__ __launch_bounds__(SMP_T) void sample_mass_kernel(SampleArgs a) {
    const int row = blockIdx.y, j = blockIdx.x, tid = threadIdx.x;
    const int seq = smp_seq(a, row);
    if (seq < 0) return;
    const float* lg = a.logits + (size_t)row * a.ld;
    const int span = (a.V + SMP_NB - 1) / SMP_NB, s0 = j * span, s1 = min(a.V, s0 + span);
    __shared__ u64_t wtot[4];
    __shared__ float fred[4];
    __shared__ int s_bin;
    __shared__ u64_t s_above;
    u64_t* hist = a.hist + (size_t)row * 3 * SMP_BINS;
    u64_t* sel = a.sel + (size_t)row * 8;
    const float mx = smp_row_max(a, row, fred);
    u64_t above = sel[3];
    const int bin = smp_find_bin<4>(hist + 2 * SMP_BINS, sel[0], above, wtot, &s_bin, &s_above);
    const uint32_t tau = (uint32_t)sel[4] | (uint32_t)bin;
    if (j == 0 && tid == 0) {
        const u64_t zs = above + hist[2 * SMP_BINS + bin];        // ties at tau are all inside
        const float uu = a.u[(size_t)seq * a.u_stride + (a.u_index ? a.u_index[seq] : 0)];
        sel[5] = tau;
        sel[6] = (u64_t)floor((double)uu * (double)zs);           // running > u * Z  <=>  running > floor(u * Z)
    }
    u64_t acc = 0;
    for (int i = s0 + tid; i < s1; i += SMP_T) {
        const float e = expf(smp_x(a, lg, i) - mx);
        if (__float_as_uint(e) >= tau) acc += smp_fix(e);
    }
    acc = wave_sum_u64(acc);
    __syncthreads();
    if ((tid & 63) == 0) wtot[tid >> 6] = acc;
    __syncthreads();
    if (tid == 0) a.psum[(size_t)row * SMP_NB + j] = wtot[0] + wtot[1] + wtot[2] + wtot[3];
}

// ---- phase F: one block per row: pick the token, append it, clear the histograms
__global__ __launch_bounds__(SMP_T) void sample_finish_kernel(SampleArgs a, AppendArgs ap) {
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seq = smp_seq(a, row);
    if (seq < 0) return;
    __shared__ u64_t wtot[4];
    __shared__ float fred[4];
    __shared__ int s_tok, s_blk;
    __shared__ u64_t s_base;
    int token;
    if (a.temperature == 0.0f) {
        float bv = -INFINITY; int bi = 0x7FFFFFFF;
        if (tid < SMP_NB) { bv = a.pmax[(size_t)row * SMP_NB + tid]; bi = a.pidx[(size_t)row * SMP_NB + tid]; }
        if (wave == 0) {
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const float ov = __shfl_xor(bv, off, RSD_WAVE);
                const int oi = __shfl_xor(bi, off, RSD_WAVE);
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            if (lane == 0) s_tok = bi;
        }
        __syncthreads();
        token = s_tok;
    } else {
        const float* lg = a.logits + (size_t)row * a.ld;
        u64_t* hist = a.hist + (size_t)row * 3 * SMP_BINS;
        const u64_t* sel = a.sel + (size_t)row * 8;
        const float mx = smp_row_max(a, row, fred);
        const uint32_t tau = (uint32_t)sel[5];
        const u64_t target = sel[6];
        const u64_t pv = (tid < SMP_NB) ? a.psum[(size_t)row * SMP_NB + tid] : 0;
        const u64_t pincl = block256_incl_scan_u64(pv, wtot);
        if (tid == 0) { s_blk = -1; s_tok = -1; }
        __syncthreads();
        if (tid < SMP_NB && pincl > target && pincl - pv <= target) { s_blk = tid; s_base = pincl - pv; }
        __syncthreads();
        const int span = (a.V + SMP_NB - 1) / SMP_NB;
        // if rounding of u * Z left no crossing, the draw is the last member: walk the last non-empty span
        int blk = s_blk;
        u64_t base = s_base;
        if (blk < 0) {
            if (tid == 0) {
                u64_t run = 0; int last = 0;
                for (int b = 0; b < SMP_NB; ++b) { const u64_t v = a.psum[(size_t)row * SMP_NB + b]; if (v) { last = b; s_base = run; } run += v; }
                s_blk = last;
            }
            __syncthreads();
            blk = s_blk; base = s_base;
        }
        const int s0 = blk * span, s1 = min(a.V, s0 + span);
        int last_member = -1;
        for (int c0 = s0; c0 < s1; c0 += SMP_T) {          // uniform trip count for the whole block
            const int i = c0 + tid;
            u64_t q = 0;
            if (i < s1) {
                const float e = expf(smp_x(a, lg, i) - mx);
                if (__float_as_uint(e) >= tau) { q = smp_fix(e); last_member = i; }
            }
            const u64_t incl = block256_incl_scan_u64(q, wtot);
            const u64_t run = base + incl;
            if (q && run > target && run - q <= target) s_tok = i;     // at most one thread
            __syncthreads();
            if (s_tok >= 0) break;
            __syncthreads();
            if (tid == SMP_T - 1) s_base = run;
            __syncthreads();
            base = s_base;
        }
        if (s_tok < 0) {
            // no crossing (u * Z rounded up to the full mass): the last member of the nucleus
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) last_member = max(last_member, __shfl_xor(last_member, off, RSD_WAVE));
            __shared__ int lred[4];
            if (lane == 0) lred[wave] = last_member;
            __syncthreads();
            if (tid == 0) s_tok = max(max(lred[0], lred[1]), max(lred[2], lred[3]));
            __syncthreads();
        }
        token = s_tok;
        for (int b = tid; b < 3 * SMP_BINS; b += SMP_T) hist[b] = 0;
    }
    if (tid != 0) return;
    if (a.out) a.out[row] = token;
    if (!ap.enabled) return;
    // append the token and decide whether the step of this sequence goes on
    const SeqState& st = ap.st;
    const int b = seq;
    const int pos = st.ctx_len[b];
    if (ap.enabled == 2) {
        // a proposal: written behind the committed tokens and recorded as the n-th proposal of the
        // step (a place of the step can be proposed for in several rounds); the step's own length
        // and records wait for the target's decision
        const size_t rec = ((size_t)b * ap.max_steps + st.cur_step[0]) * ap.prop_stride + st.sd_nprop[b] + (pos - st.sd_base[b]);
        st.sampled[2][rec] = token;
        int tok = token;
        if (ap.forced) { const int f = ap.forced[rec]; if (f >= 0) tok = f; }
        st.tokens[(size_t)b * ap.max_ctx + pos] = tok;
        st.ctx_len[b] = pos + 1;
        st.kv_len[ap.model * ap.B + b] = pos;
        if (tok == ap.sep_id || tok == ap.eos_id || pos + 1 >= st.sd_lim[b]) {
            st.active[b] = 0;
            atomicSub(st.n_active, 1);
        }
        return;
    }
    const size_t rec = ((size_t)b * ap.max_steps + st.cur_step[0]) * ap.step_cap + st.step_len[b];
    st.sampled[ap.model][rec] = token;
    int tok = token;
    if (ap.forced) { const int f = ap.forced[rec]; if (f >= 0) tok = f; }
    st.tokens[(size_t)b * ap.max_ctx + pos] = tok;
    st.ctx_len[b] = pos + 1;
    st.kv_len[ap.model * ap.B + b] = pos;          // every token before the new one has been fed
    const int sl = st.step_len[b] + 1;
    st.step_len[b] = sl;
    if (tok == ap.sep_id || tok == ap.eos_id || sl >= ap.step_cap || pos + 1 >= ap.max_ctx) {
        st.active[b] = 0;
        atomicSub(st.n_active, 1);
    }
}

static void sample_launch(hipStream_t st, const SampleArgs& a, const AppendArgs& ap, int rows) {
    const dim3 grid(SMP_NB, rows), block(SMP_T);
    hipLaunchKernelGGL(sample_max_kernel, grid, block, 0, st, a);
    if (a.temperature != 0.0f) {
        hipLaunchKernelGGL((sample_hist_kernel<0>), grid, block, 0, st, a);
        hipLaunchKernelGGL((sample_hist_kernel<1>), grid, block, 0, st, a);
        hipLaunchKernelGGL((sample_hist_kernel<2>), grid, block, 0, st, a);
        hipLaunchKernelGGL(sample_mass_kernel, grid, block, 0, st, a);
    }
    hipLaunchKernelGGL(sample_finish_kernel, dim3(rows), block, 0, st, a, ap);
}
