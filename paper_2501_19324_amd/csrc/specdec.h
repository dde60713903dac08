// Verification of speculative-decoding proposals under temperature / nucleus sampling
// (Section 5, "Combine RSD with SD"; the rule is the cited speculative-decoding algorithm):
// proposal x drawn from the draft's distribution q is kept iff u * q(x) < p(x) with p the
// target's distribution at the same place; the first refused proposal is replaced by a draw
// from the normalised positive part of p - q; after a fully kept run one more token is drawn
// from the target's next distribution.
//
// p and q are the distributions the sampler draws from (sample.h): e_t = exp(x_t - max x),
// x = (logit + separator bias) / temperature, restricted to the nucleus {e_t >= tau} and
// divided by the nucleus mass Z.  The sampler's phases A-E run first on every row and leave
// max x (per-block maxima), tau and the per-block masses in its workspace; masses are 2^40
// fixed point and are summed exactly.  Here probabilities are formed in fp64 from those
// integers, and the positive part of p - q is summed as 2^50 fixed point, so that every sum is
// exact and order-independent and the draw is reproducible.
#pragma once
#include "sample.h"

struct SdRowSet {                 // rows the sampler has prepared (phases A-E)
    const float* logits; int ld;
    const float* pmax;            // [rows][SMP_NB]
    const u64_t* psum;            // [rows][SMP_NB]
    const u64_t* sel;             // [rows][8]; [5] = tau
};

struct SdVerifyArgs {
    SdRowSet p, q;
    int V, k;                     // q row of proposal i of sequence s: s * k + i
    float temperature; int sep_id; float sep_bias;
    const int* live;              // nullable: sequences with live[s] == 0 are skipped
    const int* n_prop_base;       // proposals of s: n_prop_end[s] - n_prop_base[s] (engine: ctx_len - sd_base)
    const int* n_prop_end;
    const int* p_row0;            // first p row of s (it owns proposals + 1 consecutive rows)
    const int* tok; int tok_stride; const int* tok_off;       // proposal i of s: tok[s * tok_stride + tok_off[s] + i]
    const float* u_acc; int u_stride; const int* u_off;       // its acceptance uniform: u_acc[s * u_stride + u_off[s] + i]
    const float* u_new;                                        // uniform of a token the target draws at that place (same indexing)
    int* kept_own;                // [nseq] leading proposals kept
    int* acc_own;                 // [nseq][k] 1 kept / 0 refused, for every proposal (also those behind a refusal)
    int* choice;                  // [p rows]; on entry the sampler's own draw from every p row; on exit row0 + i holds
                                  // proposal i for i < kept, the replacement at i == kept < proposals
    u64_t* rpart;                 // [nseq][SMP_NB] workspace
};

__device__ __forceinline__ float sd_x(const SdVerifyArgs& a, const float* lg, int i) {
    return (lg[i] + (i == a.sep_id ? a.sep_bias : 0.0f)) / a.temperature;
}

// max x, tau and nucleus mass of one prepared row; all 64 lanes of a wave call it
__device__ __forceinline__ void sd_row_stats(const SdRowSet& R, int row, int lane, float& mx, uint32_t& tau, u64_t& Z) {
    mx = wave_max(R.pmax[(size_t)row * SMP_NB + lane]);
    Z = wave_sum_u64(R.psum[(size_t)row * SMP_NB + lane]);
    tau = (uint32_t)R.sel[(size_t)row * 8 + 5];
}

// probability of token t under a prepared row (0 outside the nucleus)
__device__ __forceinline__ double sd_prob(const SdVerifyArgs& a, const SdRowSet& R, int row, int t, float mx, uint32_t tau, u64_t Z) {
    const float e = expf(sd_x(a, R.logits + (size_t)row * R.ld, t) - mx);
    return __float_as_uint(e) >= tau ? (double)smp_fix(e) / (double)Z : 0.0;
}

// ---- one wave per sequence: the acceptance test of every proposal, the number of leading ones kept
__global__ __launch_bounds__(64) void sd_accept_kernel(SdVerifyArgs a) {
    const int s = blockIdx.x, lane = threadIdx.x;
    if (a.live && !a.live[s]) return;
    const int np = a.n_prop_end[s] - a.n_prop_base[s];
    int kept = np;
    for (int i = 0; i < np; ++i) {
        float mp, mq; uint32_t tp, tq; u64_t zp, zq;
        const int rp = a.p_row0[s] + i, rq = s * a.k + i;
        sd_row_stats(a.p, rp, lane, mp, tp, zp);
        sd_row_stats(a.q, rq, lane, mq, tq, zq);
        const int x = a.tok[(size_t)s * a.tok_stride + a.tok_off[s] + i];
        const double pp = sd_prob(a, a.p, rp, x, mp, tp, zp), qq = sd_prob(a, a.q, rq, x, mq, tq, zq);
        const double u = (double)a.u_acc[(size_t)s * a.u_stride + a.u_off[s] + i];
        const int ok = u * qq < pp;
        if (lane == 0) a.acc_own[s * a.k + i] = ok;
        if (!ok && kept == np) kept = i;
    }
    if (lane == 0) a.kept_own[s] = kept;
}

__device__ __forceinline__ u64_t sd_fix50(double r) { return (u64_t)(r * 1125899906842624.0); }   // r * 2^50, r in [0, 1]

// ---- positive part of p - q at the first refused place: per-block mass
__global__ __launch_bounds__(SMP_T) void sd_residual_mass_kernel(SdVerifyArgs a, const int* __restrict__ where) {
    const int s = blockIdx.y, j = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
    if (a.live && !a.live[s]) return;
    const int np = a.n_prop_end[s] - a.n_prop_base[s], at = where[s];
    if (at >= np) return;
    __shared__ u64_t wtot[4];
    float mp, mq; uint32_t tp, tq; u64_t zp, zq;
    const int rp = a.p_row0[s] + at, rq = s * a.k + at;
    sd_row_stats(a.p, rp, lane, mp, tp, zp);
    sd_row_stats(a.q, rq, lane, mq, tq, zq);
    const int span = (a.V + SMP_NB - 1) / SMP_NB, s0 = j * span, s1 = min(a.V, s0 + span);
    u64_t acc = 0;
    for (int t = s0 + tid; t < s1; t += SMP_T) {
        const double r = sd_prob(a, a.p, rp, t, mp, tp, zp) - sd_prob(a, a.q, rq, t, mq, tq, zq);
        if (r > 0.0) acc += sd_fix50(r);
    }
    acc = wave_sum_u64(acc);
    if (lane == 0) wtot[tid >> 6] = acc;
    __syncthreads();
    if (tid == 0) a.rpart[(size_t)s * SMP_NB + j] = wtot[0] + wtot[1] + wtot[2] + wtot[3];
}

// ---- one block per sequence: the replacement draw (ascending token id, first running mass above
// u * total), and the choices of the kept places
__global__ __launch_bounds__(SMP_T) void sd_residual_draw_kernel(SdVerifyArgs a, const int* __restrict__ where) {
    const int s = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
    if (a.live && !a.live[s]) return;
    const int np = a.n_prop_end[s] - a.n_prop_base[s], at = where[s], r0 = a.p_row0[s];
    for (int i = tid; i < min(at, np); i += SMP_T) a.choice[r0 + i] = a.tok[(size_t)s * a.tok_stride + a.tok_off[s] + i];
    if (at >= np) return;                                  // fully kept: choice[r0 + np] already holds the target's next draw
    __shared__ u64_t wtot[4];
    __shared__ int s_tok, s_blk;
    __shared__ u64_t s_base;
    const u64_t pv = (tid < SMP_NB) ? a.rpart[(size_t)s * SMP_NB + tid] : 0;
    const u64_t pincl = block256_incl_scan_u64(pv, wtot);
    if (tid == 0) { s_blk = -1; s_tok = -1; s_base = 0; }
    __syncthreads();
    if (tid == SMP_NB - 1) s_base = pincl;                 // total mass, read below before it is reused
    __syncthreads();
    const u64_t total = s_base;
    if (total == 0) return;                                // rounding left no positive part: keep the target's own draw from p
    const double u = (double)a.u_new[(size_t)s * a.u_stride + a.u_off[s] + at];
    const u64_t target = (u64_t)floor(u * (double)total);
    __syncthreads();
    if (tid < SMP_NB && pincl > target && pincl - pv <= target) { s_blk = tid; s_base = pincl - pv; }
    __syncthreads();
    int blk = s_blk;
    u64_t base = s_base;
    if (blk < 0) {                                         // u * total rounded up to the total: the last block with mass
        if (tid == 0) {
            u64_t run = 0; int last = 0;
            for (int b = 0; b < SMP_NB; ++b) { const u64_t v = a.rpart[(size_t)s * SMP_NB + b]; if (v) { last = b; s_base = run; } run += v; }
            s_blk = last;
        }
        __syncthreads();
        blk = s_blk; base = s_base;
    }
    float mp, mq; uint32_t tp, tq; u64_t zp, zq;
    const int rp = r0 + at, rq = s * a.k + at;
    sd_row_stats(a.p, rp, lane, mp, tp, zp);
    sd_row_stats(a.q, rq, lane, mq, tq, zq);
    const int span = (a.V + SMP_NB - 1) / SMP_NB, s0 = blk * span, s1 = min(a.V, s0 + span);
    int last_member = -1;
    for (int c0 = s0; c0 < s1; c0 += SMP_T) {              // uniform trip count for the whole block
        const int t = c0 + tid;
        u64_t m = 0;
        if (t < s1) {
            const double r = sd_prob(a, a.p, rp, t, mp, tp, zp) - sd_prob(a, a.q, rq, t, mq, tq, zq);
            if (r > 0.0) { m = sd_fix50(r); if (m) last_member = t; }
        }
        const u64_t incl = block256_incl_scan_u64(m, wtot);
        const u64_t run = base + incl;
        if (m && run > target && run - m <= target) s_tok = t;       // at most one thread
        __syncthreads();
        if (s_tok >= 0) break;
        __syncthreads();
        if (tid == SMP_T - 1) s_base = run;
        __syncthreads();
        base = s_base;
    }
    if (s_tok < 0) {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) last_member = max(last_member, __shfl_xor(last_member, off, RSD_WAVE));
        __shared__ int lred[4];
        if (lane == 0) lred[tid >> 6] = last_member;
        __syncthreads();
        if (tid == 0) s_tok = max(max(lred[0], lred[1]), max(lred[2], lred[3]));
        __syncthreads();
    }
    if (tid == 0 && s_tok >= 0) a.choice[rp] = s_tok;
}

// ---- engine side: where the round's first refusal is applied, and the record of the own decisions.
// Without a teacher that is the number of leading proposals kept.  Under a teacher (forced[] holds the
// tokens to commit) a proposal counts as kept iff the forced token at its place equals it.
__global__ void sd_where_kernel(SeqState st, int B, int k, const int* __restrict__ forced, const int* __restrict__ kept_own,
                                const int* __restrict__ acc_own, int max_ctx, int max_steps, int step_cap, int prop_stride,
                                int* __restrict__ where, int* __restrict__ acc_rec) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B || !st.sd_live[b]) return;
    const int base = st.sd_base[b], np = st.ctx_len[b] - base;
    const size_t step = (size_t)b * max_steps + st.cur_step[0];
    for (int i = 0; i < np; ++i) acc_rec[step * prop_stride + st.sd_nprop[b] + i] = acc_own[b * k + i];
    int w = kept_own[b];
    if (forced) {
        w = np;
        for (int i = 0; i < np; ++i) {
            const int f = forced[step * step_cap + st.step_len[b] + i];
            const bool keep = f >= 0 ? f == st.tokens[(size_t)b * max_ctx + base + i] : acc_own[b * k + i] != 0;
            if (!keep) { w = i; break; }
        }
    }
    where[b] = w;
}
