// Element-wise and bookkeeping kernels: embedding gather, RMSNorm, SwiGLU, row
// gather, reward head, per-token step bookkeeping, acceptance criterion with
// rollback.
#pragma once
#include "common.h"

template <typename WT>
__global__ void embed_kernel(const WT* __restrict__ E, int d, const int* __restrict__ tokens, int max_ctx,
                             RowMap rm, float* __restrict__ h) {
    const int r = blockIdx.x;
    int seq, pos;
    if (!row_lookup(rm, r, seq, pos)) return;
    const int tok = tokens[(size_t)seq * max_ctx + pos];
    const WT* src = E + (size_t)tok * d;
    float* dst = h + (size_t)r * d;
    for (int k = threadIdx.x * 8; k < d; k += blockDim.x * 8) {
        float v[8];
        load8(src + k, v);
        *reinterpret_cast<float4*>(dst + k) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(dst + k + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
}

// y = gain * x / sqrt(mean(x^2) + eps), one 256-thread block per row
template <typename WT>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ x, int d,
                                                      const WT* __restrict__ gain, float eps,
                                                      float* __restrict__ y) {
    __shared__ float red[4];
    const float* xr = x + (size_t)blockIdx.x * d;
    float* yr = y + (size_t)blockIdx.x * d;
    float ss = 0.0f;
    for (int k = threadIdx.x * 4; k < d; k += 1024) {
        const float4 v = *reinterpret_cast<const float4*>(xr + k);
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    ss = block256_sum(ss, red);
    const float rs = 1.0f / sqrtf(ss / (float)d + eps);
    for (int k = threadIdx.x * 4; k < d; k += 1024) {
        float4 v = *reinterpret_cast<const float4*>(xr + k);
        v.x *= rs * ld1(gain + k);     v.y *= rs * ld1(gain + k + 1);
        v.z *= rs * ld1(gain + k + 2); v.w *= rs * ld1(gain + k + 3);
        *reinterpret_cast<float4*>(yr + k) = v;
    }
}

// act[r][f] = silu(gu[r][f]) * gu[r][F + f]
__global__ void swiglu_kernel(const float* __restrict__ gu, int F, float* __restrict__ act, size_t total) {
    const size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i >= total) return;
    const size_t r = i / F, f = i - r * F;
    const float4 g = *reinterpret_cast<const float4*>(gu + r * 2 * F + f);
    const float4 u = *reinterpret_cast<const float4*>(gu + r * 2 * F + F + f);
    float4 o;
    o.x = g.x / (1.0f + expf(-g.x)) * u.x; o.y = g.y / (1.0f + expf(-g.y)) * u.y;
    o.z = g.z / (1.0f + expf(-g.z)) * u.z; o.w = g.w / (1.0f + expf(-g.w)) * u.w;
    *reinterpret_cast<float4*>(act + i) = o;
}

// dst[i][:] = src[src_row[b]][:] for src_row[b] >= 0, where b = i, or b = row_seq[i] (< 0: skipped) when given
__global__ void gather_rows_kernel(const float* __restrict__ src, const int* __restrict__ src_row, int d,
                                   float* __restrict__ dst, const int* __restrict__ row_seq) {
    const int i = blockIdx.x, b = row_seq ? row_seq[i] : i;
    if (b < 0) return;
    const int r = src_row[b];
    if (r < 0) return;
    for (int k = threadIdx.x * 4; k < d; k += blockDim.x * 4)
        *reinterpret_cast<float4*>(dst + (size_t)i * d + k) = *reinterpret_cast<const float4*>(src + (size_t)r * d + k);
}

// Diagnostic: do the page tables on the device cover what a pass over these rows will touch?  A row in use at
// (seq, pos) reads the pages 0 .. pos / RSD_PAGE of its sequence and writes into the last of them, so the
// sequence must own that many pages and every entry up to there must name a page of the pool.  The first
// violation found is recorded in err[0..3] = (code, row, seq, pos); the kernel itself reads nothing it has not
// bounds-checked first.  Codes: 1 sequence index outside the batch, 2 position outside [0, max_ctx), 3 position
// beyond the pages the sequence owns (or more pages than a table row holds), 4 table entry outside the pool.
__global__ void check_rows_kernel(RowMap rm, int M, int B, const int* __restrict__ block_table, int max_pages,
                                  const int* __restrict__ n_pages, int pool_pages, int max_ctx, int* __restrict__ err) {
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= M) return;
    int seq, pos, bad = 0;
    if (rm.row_seq) {                    // (row_lookup indexes kv_len / active by the sequence: check it first)
        seq = rm.row_seq[r];
        if (!rm.row_pos && seq < 0) return;
        if (seq < 0 || seq >= B) { bad = 1; pos = -1; }
    }
    if (!bad) {
        if (!row_lookup(rm, r, seq, pos)) return;
        if (pos < 0 || pos >= max_ctx) bad = 2;
        else {
            const int np = n_pages[seq], last = pos / RSD_PAGE;
            if (np > max_pages || last >= np) bad = 3;
            else
                for (int i = 0; i <= last; ++i) {
                    const int pg = block_table[(size_t)seq * max_pages + i];
                    if (pg < 0 || pg >= pool_pages) { bad = 4; break; }
                }
        }
    }
    if (bad && atomicCAS(&err[0], 0, bad) == 0) { err[1] = r; err[2] = seq; err[3] = pos; }
}

// Reward head on hidden rows: out[out_index] = logistic(w_r . RMSNorm(h[row]) + b_r).
// rows == nullptr: row i -> out[i].  rows[i] < 0: skipped.
template <typename WT>
__global__ __launch_bounds__(256) void reward_head_kernel(const float* __restrict__ h, int d,
                                                          const int* __restrict__ rows,
                                                          const WT* __restrict__ gain, float eps,
                                                          const WT* __restrict__ w_r, const WT* __restrict__ b_r,
                                                          float* __restrict__ out) {
    __shared__ float red[4];
    const int i = blockIdx.x;
    const int r = rows ? rows[i] : i;
    if (r < 0) return;
    const float* xr = h + (size_t)r * d;
    float ss = 0.0f, dot = 0.0f;
    for (int k = threadIdx.x; k < d; k += 256) {
        const float v = xr[k];
        ss += v * v;
        dot += v * ld1(gain + k) * ld1(w_r + k);
    }
    ss = block256_sum(ss, red);
    dot = block256_sum(dot, red);
    if (threadIdx.x == 0) {
        const float z = dot / sqrtf(ss / (float)d + eps) + ld1(b_r);
        out[i] = 1.0f / (1.0f + expf(-z));
    }
}

// Device-side sequence state, one int per sequence unless noted.
struct SeqState {
    int* tokens;        // [B][max_ctx]
    int* ctx_len;       // tokens in the sequence, in-flight step included
    int* kv_len;        // [3][B]
    int* active;        // still generating in the current stage
    int* step_len;      // tokens of the current step so far
    int* finished;      // RSD_RUNNING or reason
    int* ctx_pre;       // ctx_len when the current step began
    int* accepted;      // decision applied in the current step
    int* own_accept;    // decision the criterion took
    float* reward;
    int* n_active;      // [1] sequences still active after the last bookkeeping pass
    int* cur_step;      // [1] index of the reasoning step in progress
    int* sampled[3];    // [B][max_steps][step_cap] each: tokens chosen by the draft / target samplers; [2]: the draft's proposals
    // speculative regeneration of rejected steps (Section 5, "Combine RSD with SD")
    int* sd_live;       // the step of this sequence is still being regenerated
    int* sd_base;       // ctx_len when the round began
    int* sd_lim;        // proposals of the round stay below this position
    int* sd_nprop;      // proposals made / kept and rounds run in the current step
    int* sd_nkept;
    int* sd_nround;
};

// Acceptance criterion A_omega (Algorithm 2) on the rewards of the draft steps,
// then the rollback of rejected sequences to their pre-step context.
__global__ void gate_kernel(SeqState st, int B, float delta, int omega_kind, float omega_a,
                            const float* __restrict__ u_gate, int max_steps, int step,
                            const int* __restrict__ forced_accept, const int* __restrict__ in_step,
                            int merge) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    if (!in_step[b]) { st.accepted[b] = 0; st.own_accept[b] = 0; st.active[b] = 0; return; }
    const float r = st.reward[b];
    float w;
    switch (omega_kind) {
        case 1: w = omega_a; break;
        case 2: w = fminf(1.0f, fmaxf(0.0f, r)); break;
        case 3: w = fmaxf(0.0f, r / (1.0f + r)); break;
        case 4: w = 1.0f / (1.0f + expf(-omega_a * (r - delta))); break;
        default: w = (r >= delta) ? 1.0f : 0.0f; break;
    }
    int acc;
    if (w == 0.0f || w == 1.0f) acc = (w == 1.0f);
    else acc = (w >= u_gate[(size_t)b * max_steps + step]);
    st.own_accept[b] = acc;
    if (forced_accept) { const int f = forced_accept[(size_t)b * max_steps + step]; if (f >= 0) acc = f; }
    st.accepted[b] = acc;
    if (!acc) {
        const int pre = st.ctx_pre[b];
        st.ctx_len[b] = pre;
        st.kv_len[0 * B + b] = pre;     // draft: keys of the rejected step are dropped
        if (merge == 0) st.kv_len[2 * B + b] = pre;     // a separate reward model likewise
        // a target that scored the step (reward head on its trunk, merge == 2) has read it too: back to
        // the token before the step, which its regeneration feeds first
        if (merge == 2) st.kv_len[1 * B + b] = pre - 1;
    }
    st.active[b] = !acc;                // the target stage runs on the rejected sequences
}

// Verification of one round of speculative regeneration, greedy decoding (Section 5, "Combine RSD
// with SD"; Section 3: SD runs greedily).  Sequence b proposed tokens[base .. ctx_len) and the target
// chose choice[row0[b] + i] for position base + i, i = 0 .. number of proposals.  The step grows by
// the target's choices up to and including the first one that differs from the proposal at its place
// (or the one after the last proposal), or that ends the step.  Both models keep keys/values for the
// committed tokens they were fed only, never for the newest one.
__global__ void sd_verify_kernel(SeqState st, int B, const int* __restrict__ row0, const int* __restrict__ choice,
                                 const int* __restrict__ forced, int max_ctx, int max_steps, int step_cap,
                                 int sep_id, int eos_id) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B || !st.sd_live[b]) return;
    const int base = st.sd_base[b], np = st.ctx_len[b] - base, r0 = row0[b];
    int sl = st.step_len[b], live = 1, kept = 0, m = 0;
    for (int i = 0; i <= np && live; ++i) {
        const size_t rec = ((size_t)b * max_steps + st.cur_step[0]) * step_cap + sl;
        int t = choice[r0 + i];
        st.sampled[1][rec] = t;
        if (forced) { const int f = forced[rec]; if (f >= 0) t = f; }
        const int pos = base + i;
        const bool same = i < np && st.tokens[(size_t)b * max_ctx + pos] == t;
        st.tokens[(size_t)b * max_ctx + pos] = t;
        ++sl;
        m = i + 1;
        kept += same;
        if (t == sep_id || t == eos_id || sl >= step_cap || pos + 1 >= max_ctx) live = 0;
        if (!same) break;
    }
    st.step_len[b] = sl;
    st.ctx_len[b] = base + m;
    st.kv_len[1 * B + b] = base + m - 1;
    st.kv_len[0 * B + b] = min(st.kv_len[0 * B + b], base + m - 1);
    st.sd_nprop[b] += np;
    st.sd_nkept[b] += kept;
    st.sd_nround[b] += 1;
    st.sd_live[b] = live;
    st.active[b] = 0;
}

__global__ void fill_int_kernel(int* p, int v, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}
