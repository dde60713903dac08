// Host side of the RSD library: context, KV page bookkeeping, the per-model
// forward passes built from the kernels in this directory, and the loop of
// Algorithm 1 (Section 2.1) with the acceptance criterion of Algorithm 2.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <type_traits>
#include <vector>

#include "rsd.h"
#include "pages.h"
#include "common.h"
#include "gemv.h"
#include "gemm.h"
#include "attn.h"
#include "misc.h"
#include "sample.h"
#include "specdec.h"

namespace {

constexpr int kMaxRows = 8192;   // rows of one chunked-prefill pass (bounds the workspaces)
constexpr int kPoll = 16;        // decode iterations between looks at the active counter
constexpr int kPfSplitRows = 128;   // chunked-prefill passes of at most this many rows may split the context
constexpr int kPfSplits = 16;       // ... into at most this many parts

struct LayerOff { size_t attn_norm, wqkv, wo, ffn_norm, wgu, wdown; };

struct Model : PageTable {       // page bookkeeping: pages.h
    rsd_model_shape s{};
    const char* blob = nullptr;
    int hd = 0, q_dim = 0, kv_dim = 0, n_qkv = 0, G = 0, esz = 0;
    size_t off_embed = 0, off_final_norm = 0, off_head = 0, off_br = 0, n_elts = 0;
    std::vector<LayerOff> layers;
    // paged KV
    char* pool = nullptr;
    size_t page_elts = 0;        // elements of one page of one layer (K and V, all KV heads)
    int splits = 1;
    int* bt_dev = nullptr;       // device copy of the block table (bt_host is pinned)
    float2* rope = nullptr;      // [max_ctx][hd/2]
};

struct Piece { int b, start, end; };

}  // namespace

struct rsd_ctx {
    Model m[3];
    rsd_params p{};
    int B = 0;
    hipStream_t st = nullptr;
    std::string err;
    // device state block and its pinned mirror (ints; reward stored as float bits)
    int* sb_dev = nullptr;
    int* sb = nullptr;
    size_t sb_ints = 0;
    SeqState ds{};               // device pointers into sb_dev and friends
    int* in_step_dev = nullptr;
    // mirror accessors
    int* ctx_len() { return sb; }
    int* kv_len(int model) { return sb + (1 + model) * B; }
    int* active() { return sb + 4 * B; }
    int* step_len() { return sb + 5 * B; }
    int* finished() { return sb + 6 * B; }
    int* ctx_pre() { return sb + 7 * B; }
    int* accepted() { return sb + 8 * B; }
    int* own_accept() { return sb + 9 * B; }
    float* reward() { return reinterpret_cast<float*>(sb + 10 * B); }
    int* in_step() { return sb + 11 * B; }
    int* n_active() { return sb + 12 * B; }
    int* cur_step() { return sb + 12 * B + 1; }
    int* sd_live() { return sb + 12 * B + 4; }
    int* sd_base() { return sb + 13 * B + 4; }
    int* sd_lim() { return sb + 14 * B + 4; }
    int* sd_nprop() { return sb + 15 * B + 4; }
    int* sd_nkept() { return sb + 16 * B + 4; }
    int* sd_nround() { return sb + 17 * B + 4; }
    std::vector<int> prompt_len;
    // process Best-of-N: sequences, the lane holding each sequence's committed state, page-sharing counters,
    // and the staging of page copies ([src, dst] pairs per model; pinned + device)
    int n_seq = 0;
    std::vector<int> canon;
    long long bon_shared = 0, bon_copied = 0, bon_alloc = 0;
    int *bon_copy_h = nullptr, *bon_copy_dev = nullptr, *bon_src_h = nullptr, *bon_src_dev = nullptr;
    int steps_done = 0;
    bool have_prompts = false;
    // borrowed
    const float *u_draft = nullptr, *u_target = nullptr, *u_gate = nullptr;
    const int *forced_draft = nullptr, *forced_target = nullptr, *forced_accept = nullptr, *forced_prop = nullptr;
    // speculative regeneration: hidden rows and logits the target's head is applied to, its choices,
    // and per round the rows to gather ([rows] then first row of every sequence [B]; pinned + device)
    float *sd_h = nullptr, *sd_logits = nullptr;
    int *sd_choice = nullptr, *sd_rows_dev = nullptr, *sd_rows_h = nullptr;
    // sampled speculation: the draft's logits of every proposal of the round ([B][sd_k][V]), sampler
    // workspaces for the target's rows and the draft's rows, uniforms of proposals / acceptance tests
    const float *u_prop = nullptr, *u_acc = nullptr;
    float* sd_qlogits = nullptr;
    struct SmpWs { float* pmax; int* pidx; u64_t *hist, *psum, *sel; } sd_ws[2] = {};
    int *sd_aux_dev = nullptr, *sd_aux_h = nullptr;      // per round: uniform index of every p row, of every q row, q row in use
    int *sd_kept_own = nullptr, *sd_where = nullptr, *sd_acc_own = nullptr, *sd_acc_rec = nullptr;
    u64_t* sd_rpart = nullptr;
    SdVerifyArgs sd_va{};                                 // arguments of the round in flight
    // workspaces (fp32 unless noted)
    int ws_rows = 0;
    float *h = nullptr, *xn = nullptr, *qkv = nullptr, *att = nullptr, *gu = nullptr, *act = nullptr;
    float *part_acc = nullptr, *part_ml = nullptr;
    float* part_k = nullptr;         // K-slice partial sums of few-row GEMMs
    uint16_t *xs_h = nullptr, *xs_l = nullptr;   // [rows][widest K]: hi / lo bf16 halves of the activations of the MFMA GEMMs
    size_t part_k_floats = 0;
    // sampler workspace (per row: block maxima, histograms of the three radix levels, block masses, selections)
    int smp_rows = 0;
    float* smp_pmax = nullptr; int* smp_pidx = nullptr;
    u64_t *smp_hist = nullptr, *smp_psum = nullptr, *smp_sel = nullptr;
    float *hl = nullptr, *xl = nullptr, *logits = nullptr, *tmp_reward = nullptr;
    int *chosen = nullptr, *steptok_dev = nullptr;
    int *row_seq_dev = nullptr, *row_pos_dev = nullptr, *last_row_dev = nullptr;
    int *row_seq_h = nullptr, *row_pos_h = nullptr, *last_row_h = nullptr, *steptok_h = nullptr;
    // decode iterations over packed rows: row r stands for sequence dec_seq[r] (-1: unused); 0 rows = one row per sequence
    int *dec_seq_dev = nullptr, *dec_seq_h = nullptr;
    int dec_rows = 0;
    // table check (rsd_check_rows; before every pass in a build with RSD_DEBUG): page counts and the error record
    int *chk_n_pages_dev = nullptr, *chk_err_dev = nullptr, *chk_h = nullptr;
    // halves the next MFMA GEMM reads instead of xs_h / xs_l (set by a producer that could not write there; used once)
    const uint16_t *xin_h = nullptr, *xin_l = nullptr;
    // chunked-prefill attention work items: first row and row count (<= 4 rows of one sequence)
    int *item_row0_dev = nullptr, *item_n_dev = nullptr, *item_row0_h = nullptr, *item_n_h = nullptr;
    int n_items = 0;
    int pf_rows = 0, pf_max_end = 0;     // rows of the chunked pass in flight and the longest context among its pieces
    int *poll_h = nullptr;
    double stage_ms[4] = {0, 0, 0, 0};
    // kernel timing probes
    struct Probe {
        int model = -1, phase = 0, op = -1, stride = 1, seen = 0, iters = 0;
        bool iter_on = false;                                // inside the decode loop whole iterations are probed
        size_t used = 0;
        long long bytes = 0, flops = 0;
        std::vector<hipEvent_t> ev;
    } probe[RSD_PROBE_SLOTS];
    unsigned long long* clk_dev = nullptr;                  // per probe slot: {shader ticks, 100 MHz ticks, launches} of probed tile GEMMs
    bool in_decode_loop = false;
    int cur_phase = RSD_PROBE_DECODE;                        // what run_layers is launching for
    // accounting of the decode loops of the draft and the target
    struct IterStats { long long iters = 0, seq_iters = 0, kv_read = 0, row_iters = 0; double ms = 0; hipEvent_t e0 = nullptr, e1 = nullptr; } it[2];
    // single-token decode iterations recorded as graphs, one per (model, uniforms, teacher tokens)
    struct DecodeGraph { int which; const float* u; const int* forced; int mode; int rows; hipGraph_t graph; hipGraphExec_t exec; };
    std::vector<DecodeGraph> graphs;
    hipStream_t cap_st = nullptr;          // recording stream (the caller's may be the null stream)
    bool graphs_ok = true;                 // cleared when recording fails: eager launches from then on
    bool decode_warm[3] = {false, false, false};
    long long n_eager_iters = 0, n_graph_replays = 0;
};

namespace {

int fail(rsd_ctx* c, int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c) c->err = buf;
    return code;
}

#define HIPCHK(c, call)                                                                         \
    do {                                                                                        \
        hipError_t e_ = (call);                                                                 \
        if (e_ != hipSuccess)                                                                   \
            return fail(c, RSD_EHIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
    } while (0)

template <typename T>
hipError_t dev_alloc(T** p, size_t n) { return hipMalloc(reinterpret_cast<void**>(p), std::max<size_t>(n, 1) * sizeof(T)); }
template <typename T>
hipError_t pin_alloc(T** p, size_t n) { return hipHostMalloc(reinterpret_cast<void**>(p), std::max<size_t>(n, 1) * sizeof(T), hipHostMallocDefault); }

int ceil_div(int a, int b) { return (a + b - 1) / b; }

// ------------------------------------------------------------------ model set-up
int setup_model(rsd_ctx* c, Model& m, const rsd_model_shape& s, const rsd_weights& w, int which, bool head_only = false) {
    m.s = s;
    if (s.n_layers < 1 || s.d_model < 64 || s.n_heads < 1 || s.n_kv_heads < 1 || s.vocab < 2 || s.d_ffn < 64)
        return fail(c, RSD_EINVAL, "model %d: non-positive dimension", which);
    if (s.d_model % s.n_heads) return fail(c, RSD_EINVAL, "model %d: d_model %% n_heads != 0", which);
    m.hd = s.d_model / s.n_heads;
    if (m.hd != 32 && m.hd != 128) return fail(c, RSD_EINVAL, "model %d: head_dim %d not in {32,128}", which, m.hd);
    if (s.n_heads % s.n_kv_heads) return fail(c, RSD_EINVAL, "model %d: n_heads %% n_kv_heads != 0", which);
    m.G = s.n_heads / s.n_kv_heads;
    if (!(m.G == 1 || m.G == 2 || m.G == 4 || m.G == 6 || m.G == 7 || m.G == 8))
        return fail(c, RSD_EINVAL, "model %d: query group of %d heads unsupported", which, m.G);
    if (s.d_model % 64 || s.d_ffn % 64) return fail(c, RSD_EINVAL, "model %d: d_model and d_ffn must be multiples of 64", which);
    if (s.dtype != RSD_F32 && s.dtype != RSD_BF16) return fail(c, RSD_EINVAL, "model %d: bad dtype", which);
    if (s.dtype == RSD_BF16 && m.hd != 128) return fail(c, RSD_EINVAL, "model %d: bf16 models need head_dim 128", which);
    if (s.head_kind != (which == RSD_PRM ? RSD_HEAD_REWARD : RSD_HEAD_LM))
        return fail(c, RSD_EINVAL, "model %d: wrong head kind", which);
    m.esz = s.dtype == RSD_F32 ? 4 : 2;
    m.q_dim = s.n_heads * m.hd;
    m.kv_dim = s.n_kv_heads * m.hd;
    m.n_qkv = m.q_dim + 2 * m.kv_dim;
    const size_t d = s.d_model, F = s.d_ffn;
    size_t off = 0;
    m.off_embed = off; off += (size_t)s.vocab * d;
    m.layers.resize(s.n_layers);
    for (int l = 0; l < s.n_layers; ++l) {
        LayerOff& o = m.layers[l];
        o.attn_norm = off; off += d;
        o.wqkv = off; off += (size_t)m.n_qkv * d;
        o.wo = off; off += d * (size_t)m.q_dim;
        o.ffn_norm = off; off += d;
        o.wgu = off; off += 2 * F * d;
        o.wdown = off; off += d * F;
    }
    m.off_final_norm = off; off += d;
    m.off_head = off;
    if (s.head_kind == RSD_HEAD_LM) off += (size_t)s.vocab * d;
    else { off += d; m.off_br = off; off += 8; }
    if (head_only) {     // merged reward model: the blob holds w_r and b_r only
        m.layers.clear();
        m.off_head = 0; m.off_br = d; off = d + 8;
    }
    m.n_elts = off;
    if (!w.blob || w.nbytes < off * m.esz)
        return fail(c, RSD_EINVAL, "model %d: weight blob holds %llu bytes, %llu needed", which,
                    (unsigned long long)w.nbytes, (unsigned long long)(off * m.esz));
    if (reinterpret_cast<uintptr_t>(w.blob) % 16) return fail(c, RSD_EINVAL, "model %d: blob not 16-byte aligned", which);
    m.blob = static_cast<const char*>(w.blob);
    return RSD_OK;
}

template <typename WT> const WT* wptr(const Model& m, size_t off) { return reinterpret_cast<const WT*>(m.blob) + off; }

int setup_kv(rsd_ctx* c, Model& m, int which) {
    const int B = c->B;
    m.max_pages = ceil_div(c->p.max_ctx, RSD_PAGE);
    m.page_elts = (size_t)2 * m.s.n_kv_heads * RSD_PAGE * m.hd;
    const size_t page_bytes = m.page_elts * m.esz * m.s.n_layers;
    size_t pages = (size_t)B * m.max_pages;
    if (c->p.kv_pool_bytes[which]) pages = std::min<size_t>(pages, c->p.kv_pool_bytes[which] / page_bytes);
    if (pages < 1) return fail(c, RSD_EINVAL, "model %d: KV pool smaller than one page", which);
    HIPCHK(c, hipMalloc(reinterpret_cast<void**>(&m.pool), pages * page_bytes));
    int* storage = nullptr;
    HIPCHK(c, pin_alloc(&storage, (size_t)B * m.max_pages));
    HIPCHK(c, dev_alloc(&m.bt_dev, (size_t)B * m.max_pages));
    m.init_pages(B, m.max_pages, (int)pages, storage);
    // rotary table in fp64 on the host, rounded once to fp32
    const int half = m.hd / 2;
    std::vector<float2> tab((size_t)c->p.max_ctx * half);
    for (int i = 0; i < half; ++i) {
        const double inv = std::pow((double)m.s.rope_theta, -2.0 * i / m.hd);
        for (int pos = 0; pos < c->p.max_ctx; ++pos) {
            const double a = pos * inv;
            tab[(size_t)pos * half + i] = make_float2((float)std::cos(a), (float)std::sin(a));
        }
    }
    HIPCHK(c, dev_alloc(&m.rope, tab.size()));
    HIPCHK(c, hipMemcpy(m.rope, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice));
    // splits of the decode attention: enough blocks to occupy the chip, at least 4 pages each
    int s = 256 / std::max(1, B * m.s.n_kv_heads);
    s = std::min(s, std::min(32, ceil_div(m.max_pages, 4)));
    m.splits = std::max(1, s);
    if (m.s.dtype == RSD_BF16) {
        // MFMA kernel, 8 waves per block.  One split (nothing to merge) whenever the batch alone gives
        // enough blocks, or the context is short and merging would cost a launch (a single sequence
        // merges inside its output projection); otherwise enough splits for about 128 blocks, none
        // below 16 pages.  A wave keeps at most 64 page-table entries.
        const int pairs = B * m.s.n_kv_heads;
        if (pairs >= 64 || (B > 1 && m.max_pages <= 128)) m.splits = 1;
        else m.splits = std::max(1, std::min(64, std::min(ceil_div(128, pairs), ceil_div(m.max_pages, 16))));
        while (ceil_div(m.max_pages, m.splits * 8) > 64) ++m.splits;
    }
    return RSD_OK;
}

bool ensure_pages(Model& m, int b, int need) { return m.ensure(b, need); }
void trim_pages(Model& m, int b, int keep) { m.trim(b, keep); }
void share_page(Model& m, int b, int pg) { m.share(b, pg); }
int upload_tables(rsd_ctx* c, Model& m) {
    if (!m.bt_dirty) return RSD_OK;
    HIPCHK(c, hipMemcpyAsync(m.bt_dev, m.bt_host, (size_t)c->B * m.max_pages * sizeof(int), hipMemcpyHostToDevice, c->st));
    m.bt_dirty = false;
    return RSD_OK;
}

int push_state(rsd_ctx* c) {
    *c->cur_step() = c->steps_done;
    HIPCHK(c, hipMemcpyAsync(c->sb_dev, c->sb, c->sb_ints * sizeof(int), hipMemcpyHostToDevice, c->st));
    return RSD_OK;
}
int pull_state(rsd_ctx* c) {
    HIPCHK(c, hipMemcpyAsync(c->sb, c->sb_dev, c->sb_ints * sizeof(int), hipMemcpyDeviceToHost, c->st));
    HIPCHK(c, hipStreamSynchronize(c->st));
    return RSD_OK;
}

// Runs the table check for M rows of a pass through model `which` and waits for its verdict: RSD_ESTATE (with
// the first offending row in the message) when a kernel of that pass would index outside what its row owns.
int check_rows(rsd_ctx* c, int which, const RowMap& rm, int M) {
    Model& m = c->m[which];
    if (M <= 0 || !m.bt_dev) return RSD_OK;
    int rc = upload_tables(c, m);
    if (rc) return rc;
    std::copy(m.n_pages.begin(), m.n_pages.begin() + c->B, c->chk_h + 4);
    c->chk_h[0] = c->chk_h[1] = c->chk_h[2] = c->chk_h[3] = 0;
    HIPCHK(c, hipMemcpyAsync(c->chk_err_dev, c->chk_h, 4 * sizeof(int), hipMemcpyHostToDevice, c->st));
    HIPCHK(c, hipMemcpyAsync(c->chk_n_pages_dev, c->chk_h + 4, c->B * sizeof(int), hipMemcpyHostToDevice, c->st));
    hipLaunchKernelGGL(check_rows_kernel, dim3(ceil_div(M, 256)), dim3(256), 0, c->st, rm, M, c->B, m.bt_dev, m.max_pages,
                       c->chk_n_pages_dev, m.pool_pages, c->p.max_ctx, c->chk_err_dev);
    HIPCHK(c, hipMemcpyAsync(c->chk_h, c->chk_err_dev, 4 * sizeof(int), hipMemcpyDeviceToHost, c->st));
    HIPCHK(c, hipStreamSynchronize(c->st));
    if (c->chk_h[0]) {
        static const char* what[] = {"", "sequence index outside the batch", "position outside the context limit",
                                     "position beyond the pages its sequence owns", "block-table entry outside the pool"};
        return fail(c, RSD_ESTATE, "table check, model %d: row %d (sequence %d, position %d): %s", which, c->chk_h[1],
                    c->chk_h[2], c->chk_h[3], what[std::min(std::max(c->chk_h[0], 0), 4)]);
    }
    return RSD_OK;
}
#ifdef RSD_DEBUG
constexpr bool kDebugChecks = true;
#else
constexpr bool kDebugChecks = false;
#endif

// ------------------------------------------------------------------ forward passes
template <typename KT, int HD>
void launch_attn_g(rsd_ctx* c, const Model& m, int l, int M, const RowMap& rm, int S) {
    const KT* pool_l = reinterpret_cast<const KT*>(m.pool) + (size_t)l * m.pool_pages * m.page_elts;
    const float scale = 1.0f / std::sqrt((float)HD);
    const dim3 grid(M, m.s.n_kv_heads, S), block(256);
#define RSD_ATTN_CASE(GG)                                                                                   \
    case GG:                                                                                                \
        hipLaunchKernelGGL((attn_rows_kernel<KT, HD, GG>), grid, block, 0, c->st, c->qkv, m.n_qkv, pool_l,  \
                           m.bt_dev, m.max_pages, rm, m.s.n_heads, m.s.n_kv_heads, S, scale, c->att,        \
                           m.q_dim, c->part_acc, c->part_ml);                                               \
        break;
    switch (m.G) {
        RSD_ATTN_CASE(1) RSD_ATTN_CASE(2) RSD_ATTN_CASE(4) RSD_ATTN_CASE(6) RSD_ATTN_CASE(7) RSD_ATTN_CASE(8)
    }
#undef RSD_ATTN_CASE
    if (S > 1)
        hipLaunchKernelGGL((attn_combine_kernel<HD>), dim3(M, m.s.n_heads), dim3(HD), 0, c->st, c->part_acc,
                           c->part_ml, rm, m.s.n_heads, S, c->att, m.q_dim);
}

// Brackets one launch with a pair of events when a probe is armed for it.
struct ProbeScope {
    rsd_ctx* c;
    rsd_ctx::Probe* p = nullptr;
    bool direct = false;
    long long bytes, flops;
    // direct: the launch inside the scope is a single-row projection, which can carry the events in its
    // own dispatch packet (kernel start to kernel end); otherwise the events are recorded around it
    ProbeScope(rsd_ctx* c_, const Model& m, int op, long long bytes_, long long flops_, bool direct_ = false)
        : c(c_), direct(direct_), bytes(bytes_), flops(flops_) {
        const int which = (int)(&m - &c->m[0]);
        for (auto& q : c->probe) {
            if (q.model != which || q.op != op || q.phase != c->cur_phase) continue;
            if (q.used + 2 > q.ev.size()) continue;
            if (c->in_decode_loop) { if (!q.iter_on) continue; }
            else if (q.seen++ % q.stride) continue;
            p = &q;
            break;
        }
        if (!p) return;
        if (direct) gemv_timing = GemvTiming{p->ev[p->used], p->ev[p->used + 1]};
        else (void)hipEventRecord(p->ev[p->used], c->st);
    }
    // where a probed many-row GEMM adds its clock readings (nullptr: no probe armed for this launch)
    unsigned long long* clk() const { return p ? c->clk_dev + 3 * (p - c->probe) : nullptr; }
    ~ProbeScope() {
        if (!p) return;
        if (direct) {
            const bool taken = gemv_timing.start == nullptr;    // the launcher clears the hook when it uses it
            gemv_timing = GemvTiming{};
            if (!taken) return;                                  // another kernel served this shape: no sample
        } else {
            (void)hipEventRecord(p->ev[p->used + 1], c->st);
        }
        p->used += 2;
        p->bytes += bytes;
        p->flops += flops;
    }
};

RowMap decode_map(rsd_ctx* c, int which) {
    return RowMap{c->dec_rows ? c->dec_seq_dev : nullptr, nullptr, c->ds.kv_len + (size_t)which * c->B, c->ds.active};
}
const int* decode_seq(rsd_ctx* c) { return c->dec_rows ? c->dec_seq_dev : nullptr; }

template <typename KT, int HD>
void launch_attn_decode(rsd_ctx* c, const Model& m, int l, int M, int which) {
    KT* pool_l = reinterpret_cast<KT*>(m.pool) + (size_t)l * m.pool_pages * m.page_elts;
    const float scale = 1.0f / std::sqrt((float)HD);
    const int S = m.splits;
    const dim3 grid(M, m.s.n_kv_heads, S), block(256);
#define RSD_ATTN_CASE(GG)                                                                                     \
    case GG:                                                                                                  \
        hipLaunchKernelGGL((attn_decode_kernel<KT, HD, GG>), grid, block, 0, c->st, c->qkv, m.n_qkv, pool_l,  \
                           m.bt_dev, m.max_pages, c->ds.kv_len + (size_t)which * c->B, c->ds.active, m.rope,  \
                           m.s.n_heads, m.s.n_kv_heads, S, scale, c->att, m.q_dim, c->part_acc, c->part_ml,   \
                           decode_seq(c));                                                                    \
        break;
    switch (m.G) {
        RSD_ATTN_CASE(1) RSD_ATTN_CASE(2) RSD_ATTN_CASE(4) RSD_ATTN_CASE(6) RSD_ATTN_CASE(7) RSD_ATTN_CASE(8)
    }
#undef RSD_ATTN_CASE
    if (S > 1)
        hipLaunchKernelGGL((attn_combine_kernel<HD>), dim3(M, m.s.n_heads), dim3(HD), 0, c->st, c->part_acc,
                           c->part_ml, decode_map(c, which), m.s.n_heads, S, c->att, m.q_dim);
}

// bf16 caches with head_dim 128: the MFMA kernel, 8 waves per block
// merge_here = false leaves the partial results of the splits to the caller (S > 1 only)
// qp.ks > 0: q, k, v are still the K slices of the QKV projection (the kernel adds them up itself)
void launch_attn_decode_mfma(rsd_ctx* c, const Model& m, int l, int M, int which, bool merge_here = true,
                             bool halves = false, QkvParts qp = QkvParts{nullptr, 0, 0}) {
    bf16_t* pool_l = reinterpret_cast<bf16_t*>(m.pool) + (size_t)l * m.pool_pages * m.page_elts;
    const float scale = 1.0f / std::sqrt(128.0f);
    const int S = m.splits;
    const dim3 grid(M, m.s.n_kv_heads, S);
#define RSD_ATTN_ARGS                                                                                              \
    grid, dim3(512), 0, c->st, c->qkv, m.n_qkv, pool_l, m.bt_dev, m.max_pages, c->ds.kv_len + (size_t)which * c->B, \
        c->ds.active, m.rope, m.s.n_heads, m.s.n_kv_heads, S, scale, c->att, m.q_dim, c->part_acc, c->part_ml,     \
        halves ? c->xs_h : nullptr, halves ? c->xs_l : nullptr, decode_seq(c), qp
#define RSD_ATTN_CASE(GG)                                                                                          \
    case GG:                                                                                                       \
        if (qp.ks > 0) hipLaunchKernelGGL((attn_decode_mfma_kernel<GG, 8, true>), RSD_ATTN_ARGS);                  \
        else hipLaunchKernelGGL((attn_decode_mfma_kernel<GG, 8, false>), RSD_ATTN_ARGS);                           \
        break;
    switch (m.G) {
        RSD_ATTN_CASE(1) RSD_ATTN_CASE(2) RSD_ATTN_CASE(4) RSD_ATTN_CASE(6) RSD_ATTN_CASE(7) RSD_ATTN_CASE(8)
    }
#undef RSD_ATTN_CASE
#undef RSD_ATTN_ARGS
    if (S > 1 && merge_here)
        hipLaunchKernelGGL((attn_combine_kernel<128>), dim3(M, m.s.n_heads), dim3(128), 0, c->st, c->part_acc,
                           c->part_ml, decode_map(c, which), m.s.n_heads, S, c->att, m.q_dim,
                           halves ? c->xs_h : nullptr, halves ? c->xs_l : nullptr);
}

// chunked prefill over a bf16 cache: rows of the pass are described by the context's item arrays
void launch_attn_prefill_mfma(rsd_ctx* c, const Model& m, int l, const RowMap& rm) {
    const bf16_t* pool_l = reinterpret_cast<const bf16_t*>(m.pool) + (size_t)l * m.pool_pages * m.page_elts;
    const float scale = 1.0f / std::sqrt(128.0f);
    // few rows over long contexts (a verification pass, the scoring of one step, a short catch-up): the
    // work items alone leave most of the chip idle, so every item's pages are dealt to several splits
    int S = 1;
    const int waves = c->n_items * m.s.n_kv_heads, pages = ceil_div(c->pf_max_end, RSD_PAGE);
    if (waves < 512 && pages > 8 && c->pf_rows <= kPfSplitRows)
        S = std::max(1, std::min(kPfSplits, std::min(ceil_div(pages, 4), 1024 / waves)));
    const dim3 grid(ceil_div(c->n_items, 4), m.s.n_kv_heads, S), block(256);
    constexpr size_t qlds = (size_t)4 * 2 * 2 * 16 * (128 + 8) * sizeof(uint16_t);     // Q operands of 4 waves
#define RSD_ATTN_CASE(GG)                                                                                     \
    case GG: {                                                                                                \
        /* set once per process; the call is idempotent, so a race between contexts costs a repeat at most */ \
        static std::atomic<bool> raised{false};                                                               \
        if (!raised.load(std::memory_order_relaxed)) {                                                        \
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(attn_prefill_mfma_kernel<GG>),            \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)qlds);                 \
            raised.store(true, std::memory_order_relaxed);                                                    \
        }                                                                                                     \
        hipLaunchKernelGGL((attn_prefill_mfma_kernel<GG>), grid, block, qlds, c->st, c->qkv, m.n_qkv, pool_l, \
                           m.bt_dev, m.max_pages, rm.row_seq, rm.row_pos, c->item_row0_dev, c->item_n_dev,    \
                           c->n_items, m.s.n_heads, m.s.n_kv_heads, scale, c->att, m.q_dim, c->part_acc,      \
                           c->part_ml);                                                                       \
    } break;
    switch (m.G) {
        RSD_ATTN_CASE(1) RSD_ATTN_CASE(2) RSD_ATTN_CASE(4) RSD_ATTN_CASE(6) RSD_ATTN_CASE(7) RSD_ATTN_CASE(8)
    }
#undef RSD_ATTN_CASE
    if (S > 1)
        hipLaunchKernelGGL((attn_combine_kernel<128>), dim3(c->pf_rows, m.s.n_heads), dim3(128), 0, c->st, c->part_acc,
                           c->part_ml, rm, m.s.n_heads, S, c->att, m.q_dim, (uint16_t*)nullptr, (uint16_t*)nullptr);
}

// Two or more rows over bf16 weights: MFMA kernels on activations split into hi + lo bf16 halves, which
// live in c->xs_h / c->xs_l between the launches (2..64 rows: weight-streaming kernel; more: tile kernel).
// (Measured on the 7B shape: a pass over 2 / 4 / 8 rows takes 6.5 / 6.3 / 5.7 ms this way and
// 6.8 / 8.5 / 16.1 ms through the multi-row vector kernel, which fp32 weights still use.)
template <typename WT>
bool rows_path(const Model& m, int M) {
    return std::is_same<WT, bf16_t>::value && M >= 2 && m.s.d_model % 64 == 0 && m.q_dim % 64 == 0 && m.s.d_ffn % 64 == 0;
}
// x (fp32 rows, optionally through RMSNorm with `gain`) -> the hi / lo halves
void rows_split(rsd_ctx* c, const float* X, int ldx, int M, int K, const bf16_t* gain, float eps) {
    hipLaunchKernelGGL((split_rows_kernel<bf16_t>), dim3(M), dim3(256), 0, c->st, X, ldx, K, gain, eps, c->xs_h, c->xs_l);
}
template <int EPI>
void rows_finish(rsd_ctx* c, int ks, int rows, int M, int N, float* Y, int ldy, const SkGeom& geo) {
    const int NO = EPI == EPI_SWIGLU ? N / 2 : N;
    const dim3 grid((unsigned)(((size_t)M * NO / 4 + 255) / 256)), block(256);
    hipLaunchKernelGGL((rows_finish_kernel<EPI>), grid, block, 0, c->st, c->part_k, ks, rows, M, N, Y, ldy, c->xs_h, c->xs_l, geo);
}
// Y (+)= halves . W^T with epilogue `epi`; EPI_SWIGLU (N = 2F) writes the activated values back as halves.
// next_gain != nullptr (EPI_RESID): RMSNorm(Y row) * next_gain is left in the halves for the projection that
// follows (inside the finish kernel where there is one and N <= 8192).
// (m, op) name the projection for the timing probes: the matrix kernel alone is bracketed.
// defer != nullptr (EPI_STORE): when the product is left as uniform K slices, they are not added up here but
// described in *defer for a consumer that adds them itself (ks = 0: Y holds the result as usual).
void rows_gemm(rsd_ctx* c, const Model& m, int op, int epi, const bf16_t* W, int N, int K, int M, float* Y, int ldy,
               const bf16_t* next_gain = nullptr, float eps = 0.f, QkvParts* defer = nullptr) {
    if (defer) *defer = QkvParts{nullptr, 0, 0};
    const uint16_t* Xh = c->xin_h ? c->xin_h : c->xs_h;
    const uint16_t* Xl = c->xin_l ? c->xin_l : c->xs_l;
    c->xin_h = c->xin_l = nullptr;
    const bool few = M <= 64 && N % 4 == 0;
    SkGeom geo{};                                            // G = 0: uniform K slices
    const int rows = few ? (M <= 32 ? 32 : 64) : M;          // rows of one slice of partial results
    // algorithmic traffic: the weights once, fp32 activations in and out (SwiGLU leaves N / 2 columns)
    const long long pb = (long long)N * K * 2 + 4LL * M * (K + (epi == EPI_SWIGLU ? N / 2 : N) + (epi == EPI_RESID ? N : 0));
    const long long pf = 2LL * M * N * K;
    int ks;
    if (few && gemm_rows_even(N, K)) {
        geo = sk_geometry(N, K, kSkBlocks);
        if ((size_t)geo.zmax * rows * N > c->part_k_floats) geo = SkGeom{};
    }
    if (few && geo.G > 0) {
        ks = geo.zmax;
        ProbeScope ps(c, m, op, pb, pf);
        gemm_rows_sk_launch<kSkDepth>(c->st, W, N, K, Xh, Xl, M, c->part_k, geo);
    } else if (few) {
        ks = gemm_rows_slices(N, K, rows, c->part_k_floats);
        ProbeScope ps(c, m, op, pb, pf);
        gemm_rows_launch(c->st, W, N, K, Xh, Xl, M, c->part_k, ks);
    } else {
        ks = N % 4 ? 1 : gemm_tile_slices(N, K, M, c->part_k_floats);
        if (ks == 1) {      // the tile kernel finishes by itself
            if (epi == EPI_SWIGLU) {
                // the kernel activates in its epilogue; the halves cannot go to xs_h / xs_l, which other blocks still
                // read as this product's input, so they go to the (otherwise unused) gate/up workspace and the down
                // projection that follows is pointed there
                uint16_t* oh = reinterpret_cast<uint16_t*>(c->gu);
                uint16_t* ol = oh + (size_t)M * (N / 2);
                ProbeScope ps(c, m, op, pb, pf);
                gemm_tile_launch(c->st, EPI_SWIGLU, W, N, K, Xh, Xl, M, nullptr, 0, nullptr, 1, oh, ol, ps.clk());
                c->xin_h = oh; c->xin_l = ol;
            } else {
                {
                    ProbeScope ps(c, m, op, pb, pf);
                    gemm_tile_launch(c->st, epi, W, N, K, Xh, Xl, M, Y, ldy, nullptr, 1, nullptr, nullptr, ps.clk());
                }
                if (next_gain) rows_split(c, Y, ldy, M, N, next_gain, eps);
            }
            return;
        }
        ProbeScope ps(c, m, op, pb, pf);
        gemm_tile_launch(c->st, EPI_STORE, W, N, K, Xh, Xl, M, nullptr, 0, c->part_k, ks, nullptr, nullptr, ps.clk());
    }
    if (defer && geo.G == 0 && ldy == N) {
        *defer = QkvParts{c->part_k, ks, (size_t)rows * N};
        return;
    }
    if (next_gain && N <= 8192) {
        hipLaunchKernelGGL((rows_finish_norm_kernel<bf16_t>), dim3(M), dim3(1024), 0, c->st, c->part_k, ks, rows, N, Y, ldy,
                           next_gain, eps, c->xs_h, c->xs_l, geo);
        return;
    }
    if (epi == EPI_SWIGLU) rows_finish<EPI_SWIGLU>(c, ks, rows, M, N, Y, ldy, geo);
    else if (epi == EPI_RESID) rows_finish<EPI_RESID>(c, ks, rows, M, N, Y, ldy, geo);
    else rows_finish<EPI_STORE>(c, ks, rows, M, N, Y, ldy, geo);
    if (next_gain) rows_split(c, Y, ldy, M, N, next_gain, eps);
}
void rows_split(rsd_ctx*, const float*, int, int, int, const float*, float) {}    // fp32 weights never take this path
void rows_gemm(rsd_ctx*, const Model&, int, int, const float*, int, int, int, float*, int, const float* = nullptr, float = 0.f,
               QkvParts* = nullptr) {}

template <typename WT>
void run_layers(rsd_ctx* c, Model& m, int M, const RowMap& rm, bool decode) {
    hipStream_t st = c->st;
    const int d = m.s.d_model, F = m.s.d_ffn;
    const float eps = m.s.rms_eps;
    c->xin_h = c->xin_l = nullptr;          // (a redirection is only ever meant for the projection right after its producer)
    hipLaunchKernelGGL((embed_kernel<WT>), dim3(M), dim3(256), 0, st, wptr<WT>(m, m.off_embed), d, c->ds.tokens,
                       c->p.max_ctx, rm, c->h);
    const int S = decode ? m.splits : 1;
    c->cur_phase = decode ? RSD_PROBE_DECODE : RSD_PROBE_PREFILL;
    const bool rows = rows_path<WT>(m, M);
    const bool fused = M <= 8 && !rows;   // few rows: norm / SwiGLU / residual folded into the weight-streaming kernels
    const bool rows_fuse_norm = rows;                        // the residual GEMMs leave RMSNorm(h) for the next projection
    // batched decode: the attention kernel (or its merge kernel) writes the output as hi / lo halves itself
    const bool att_halves = rows && decode && m.s.dtype == RSD_BF16 && m.hd == 128;
    // single-row decode over a bf16 cache: the output projection merges the attention splits itself
    const bool parts_to_o = decode && M == 1 && S > 1 && m.s.dtype == RSD_BF16 && m.hd == 128 &&
                            (size_t)m.q_dim * sizeof(float) <= 40 * 1024;
    for (int l = 0; l < m.s.n_layers; ++l) {
        const LayerOff& o = m.layers[l];
        const long long esz = sizeof(WT);
        QkvParts qkv_parts{nullptr, 0, 0};
        if (fused) {
            ProbeScope ps(c, m, 0, (long long)m.n_qkv * d * esz + 4LL * M * (d + m.n_qkv), 2LL * M * m.n_qkv * d, M == 1);
            gemv_launch<WT>(st, PRO_NORM, EPI_STORE, wptr<WT>(m, o.wqkv), m.n_qkv, d, c->h, d,
                            wptr<WT>(m, o.attn_norm), eps, c->qkv, m.n_qkv, M);
        } else if (rows) {
            // (after the first layer the halves of RMSNorm(h) come from the previous layer's last finish)
            if (l == 0 || !rows_fuse_norm) rows_split(c, c->h, d, M, d, wptr<WT>(m, o.attn_norm), eps);
            // (the batched decode attention over a bf16 cache adds the projection's K slices itself)
            rows_gemm(c, m, 0, EPI_STORE, wptr<WT>(m, o.wqkv), m.n_qkv, d, M, c->qkv, m.n_qkv, nullptr, 0.f,
                      att_halves ? &qkv_parts : nullptr);
        } else if constexpr (std::is_same<WT, float>::value) {
            hipLaunchKernelGGL((rmsnorm_kernel<WT>), dim3(M), dim3(256), 0, st, c->h, d, wptr<WT>(m, o.attn_norm), eps, c->xn);
            gemm_launch(st, EPI_STORE, wptr<WT>(m, o.wqkv), m.n_qkv, d, c->xn, d, c->qkv, m.n_qkv, M, c->part_k, c->part_k_floats);
        }
        WT* pool_l = reinterpret_cast<WT*>(m.pool) + (size_t)l * m.pool_pages * m.page_elts;
        if (decode) {
            const int which = (int)(&m - &c->m[0]);
            if (m.s.dtype == RSD_BF16) launch_attn_decode_mfma(c, m, l, M, which, !parts_to_o, att_halves, qkv_parts);
            else if (m.hd == 128) launch_attn_decode<WT, 128>(c, m, l, M, which);
            else launch_attn_decode<WT, 32>(c, m, l, M, which);
        } else if (m.hd == 128) {
            hipLaunchKernelGGL((rope_kv_kernel<WT, 128>), dim3(M), dim3(256), 0, st, c->qkv, m.n_qkv, pool_l, m.bt_dev,
                               m.max_pages, rm, m.rope, m.s.n_heads, m.s.n_kv_heads);
            if (m.s.dtype == RSD_BF16) launch_attn_prefill_mfma(c, m, l, rm);
            else launch_attn_g<WT, 128>(c, m, l, M, rm, S);
        } else {
            hipLaunchKernelGGL((rope_kv_kernel<WT, 32>), dim3(M), dim3(256), 0, st, c->qkv, m.n_qkv, pool_l, m.bt_dev,
                               m.max_pages, rm, m.rope, m.s.n_heads, m.s.n_kv_heads);
            launch_attn_g<WT, 32>(c, m, l, M, rm, S);
        }
        if (fused) {
            {
                ProbeScope ps(c, m, 1, (long long)d * m.q_dim * esz + 4LL * M * (m.q_dim + 2 * d), 2LL * M * d * m.q_dim, M == 1);
                if (parts_to_o)
                    gemv_launch_attn<WT>(st, wptr<WT>(m, o.wo), d, m.q_dim, AttnParts{c->part_acc, c->part_ml, S}, c->h);
                else
                    gemv_launch<WT>(st, PRO_NONE, EPI_RESID, wptr<WT>(m, o.wo), d, m.q_dim, c->att, m.q_dim,
                                    (const WT*)nullptr, 0.f, c->h, d, M);
            }
            if (gemv_can_fuse_swiglu(M, d) && gemv_can_fuse_swiglu(M, F)) {
                {
                    ProbeScope ps(c, m, 2, 2LL * F * d * esz + 4LL * M * (d + F), 4LL * M * F * d, M == 1);
                    gemv_launch<WT>(st, PRO_NORM, EPI_SWIGLU, wptr<WT>(m, o.wgu), F, d, c->h, d,
                                    wptr<WT>(m, o.ffn_norm), eps, c->act, F, M);
                }
                {
                    ProbeScope ps(c, m, 3, (long long)d * F * esz + 4LL * M * (F + 2 * d), 2LL * M * d * F, M == 1);
                    gemv_launch<WT>(st, PRO_NONE, EPI_RESID, wptr<WT>(m, o.wdown), d, F, c->act, F,
                                    (const WT*)nullptr, 0.f, c->h, d, M);
                }
            } else {
                {
                    ProbeScope ps(c, m, 2, 2LL * F * d * esz + 4LL * M * (d + 2 * F), 4LL * M * F * d);
                    gemv_launch<WT>(st, PRO_NORM, EPI_STORE, wptr<WT>(m, o.wgu), 2 * F, d, c->h, d,
                                    wptr<WT>(m, o.ffn_norm), eps, c->gu, 2 * F, M);
                }
                {
                    ProbeScope ps(c, m, 3, (long long)d * F * esz + 4LL * M * (2 * F + 2 * d), 2LL * M * d * F);
                    gemv_launch<WT>(st, PRO_SWIGLU, EPI_RESID, wptr<WT>(m, o.wdown), d, F, c->gu, 2 * F,
                                    (const WT*)nullptr, 0.f, c->h, d, M);
                }
            }
        } else if (rows) {
            if (!att_halves) rows_split(c, c->att, m.q_dim, M, m.q_dim, (const WT*)nullptr, 0.f);
            if (rows_fuse_norm) {
                rows_gemm(c, m, 1, EPI_RESID, wptr<WT>(m, o.wo), d, m.q_dim, M, c->h, d, wptr<WT>(m, o.ffn_norm), eps);
            } else {
                rows_gemm(c, m, 1, EPI_RESID, wptr<WT>(m, o.wo), d, m.q_dim, M, c->h, d);
                rows_split(c, c->h, d, M, d, wptr<WT>(m, o.ffn_norm), eps);
            }
            rows_gemm(c, m, 2, EPI_SWIGLU, wptr<WT>(m, o.wgu), 2 * F, d, M, nullptr, 0);     // activated values stay as halves
            if (rows_fuse_norm && l + 1 < m.s.n_layers)
                rows_gemm(c, m, 3, EPI_RESID, wptr<WT>(m, o.wdown), d, F, M, c->h, d, wptr<WT>(m, m.layers[l + 1].attn_norm), eps);
            else
                rows_gemm(c, m, 3, EPI_RESID, wptr<WT>(m, o.wdown), d, F, M, c->h, d);
        } else if constexpr (std::is_same<WT, float>::value) {
            gemm_launch(st, EPI_RESID, wptr<WT>(m, o.wo), d, m.q_dim, c->att, m.q_dim, c->h, d, M, c->part_k, c->part_k_floats);
            hipLaunchKernelGGL((rmsnorm_kernel<WT>), dim3(M), dim3(256), 0, st, c->h, d, wptr<WT>(m, o.ffn_norm), eps, c->xn);
            gemm_launch(st, EPI_STORE, wptr<WT>(m, o.wgu), 2 * F, d, c->xn, d, c->gu, 2 * F, M, c->part_k, c->part_k_floats);
            const size_t total = (size_t)M * F;
            hipLaunchKernelGGL(swiglu_kernel, dim3((unsigned)((total / 4 + 255) / 256)), dim3(256), 0, st, c->gu, F, c->act, total);
            gemm_launch(st, EPI_RESID, wptr<WT>(m, o.wdown), d, F, c->act, F, c->h, d, M, c->part_k, c->part_k_floats);
        }
    }
}

// Vocabulary logits of M hidden rows X[M][d] -> Y[M][ldy]
template <typename WT>
void lm_head(rsd_ctx* c, Model& m, const float* X, int M, float* Y, int ldy) {
    const int d = m.s.d_model, V = m.s.vocab;
    if (M <= 8 && !rows_path<WT>(m, M)) {
        ProbeScope ps(c, m, 4, (long long)V * d * sizeof(WT) + 4LL * M * (d + V), 2LL * M * V * d, M == 1);
        gemv_launch<WT>(c->st, PRO_NORM, EPI_STORE, wptr<WT>(m, m.off_head), V, d, X, d, wptr<WT>(m, m.off_final_norm),
                        m.s.rms_eps, Y, ldy, M);
    } else if (rows_path<WT>(m, M)) {
        rows_split(c, X, d, M, d, wptr<WT>(m, m.off_final_norm), m.s.rms_eps);
        rows_gemm(c, m, 4, EPI_STORE, wptr<WT>(m, m.off_head), V, d, M, Y, ldy);
    } else if constexpr (std::is_same<WT, float>::value) {
        for (int r0 = 0; r0 < M; r0 += kMaxRows) {
            const int mm = std::min(kMaxRows, M - r0);
            hipLaunchKernelGGL((rmsnorm_kernel<WT>), dim3(mm), dim3(256), 0, c->st, X + (size_t)r0 * d, d,
                               wptr<WT>(m, m.off_final_norm), m.s.rms_eps, c->xn);
            gemm_launch(c->st, EPI_STORE, wptr<WT>(m, m.off_head), V, d, c->xn, d, Y + (size_t)r0 * ldy, ldy, mm, c->part_k, c->part_k_floats);
        }
    }
}

// `trunk` supplies the final RMSNorm (the reward model itself, or the policy model it is merged with)
template <typename WT>
void reward_rows(rsd_ctx* c, Model& m, const float* H, int n, const int* rows, float* out, const Model* trunk = nullptr) {
    const Model& t = trunk ? *trunk : m;
    hipLaunchKernelGGL((reward_head_kernel<WT>), dim3(n), dim3(256), 0, c->st, H, m.s.d_model, rows,
                       wptr<WT>(t, t.off_final_norm), t.s.rms_eps, wptr<WT>(m, m.off_head), wptr<WT>(m, m.off_br), out);
}

// Sample one token per row; with `ap` the chosen token is also appended to its sequence.
// row_seq (packed rows): u, u_index, active and the appended state are indexed by the sequence of a row
void sample_rows(rsd_ctx* c, const float* logits, int ld, int V, const float* u, const int* u_index, int u_stride,
                 float temperature, float top_p, int sep_id, float sep_bias, const int* active, int n, int* out,
                 const AppendArgs& ap, const int* row_seq = nullptr) {
    for (int r0 = 0; r0 < n; r0 += c->smp_rows) {
        const int rows = std::min(c->smp_rows, n - r0);
        const int s0 = row_seq ? 0 : r0;         // per-sequence arrays keep their base under a row map
        SampleArgs a{logits + (size_t)r0 * ld, ld, V, u ? u + (size_t)s0 * u_stride : nullptr,
                     u_index ? u_index + s0 : nullptr, u_stride, temperature, top_p, sep_id, sep_bias,
                     active ? active + s0 : nullptr, out ? out + r0 : nullptr,
                     c->smp_pmax, c->smp_pidx, c->smp_hist, c->smp_psum, c->smp_sel, row_seq ? row_seq + r0 : nullptr};
        sample_launch(c->st, a, ap, rows);
    }
}

AppendArgs append_args(rsd_ctx* c, int which, const int* forced, int mode = 1) {
    AppendArgs ap{};
    ap.enabled = mode; ap.st = c->ds; ap.B = c->B; ap.max_ctx = c->p.max_ctx; ap.model = which; ap.forced = forced;
    ap.sep_id = c->p.sep_id; ap.eos_id = c->p.eos_id; ap.step_cap = c->p.step_cap;
    ap.max_steps = c->p.max_steps;
    ap.prop_stride = c->p.step_cap * c->p.sd_k;
    return ap;
}

// One single-token iteration of an LM model over all sequences: forward, head, sample, append.
// logits[b][:] -> q[b * k + (ctx_len[b] - sd_base[b])][:] for the active sequences: the distribution a
// sampled proposal is about to be drawn from, kept for its acceptance test
__global__ void sd_stash_kernel(const float* __restrict__ logits, int V, SeqState st, int k, float* __restrict__ q) {
    const int b = blockIdx.y;
    if (!st.active[b]) return;
    const int slot = st.ctx_len[b] - st.sd_base[b];
    if (slot < 0 || slot >= k) return;
    const float* src = logits + (size_t)b * V;
    float* dst = q + ((size_t)b * k + slot) * V;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < V; i += gridDim.x * blockDim.x) dst[i] = src[i];
}
void propose_stash(rsd_ctx* c, int mode) {
    if (mode != 2 || c->p.temperature == 0.f) return;
    const int V = c->m[RSD_DRAFT].s.vocab;
    hipLaunchKernelGGL(sd_stash_kernel, dim3(std::min(64, ceil_div(V, 256)), c->B), dim3(256), 0, c->st, c->logits, V, c->ds,
                       c->p.sd_k, c->sd_qlogits);
}

// mode 1: the token belongs to a reasoning step; mode 2: it is a proposal of speculative regeneration.
template <typename WT>
void decode_iter(rsd_ctx* c, int which, const float* u, const int* forced, int mode = 1) {
    Model& m = c->m[which];
    const int M = c->dec_rows ? c->dec_rows : c->B;
    run_layers<WT>(c, m, M, decode_map(c, which), true);
    lm_head<WT>(c, m, c->h, M, c->logits, m.s.vocab);
    propose_stash(c, mode);
    sample_rows(c, c->logits, m.s.vocab, m.s.vocab, u, c->ds.ctx_len, c->p.max_ctx, c->p.temperature, c->p.top_p,
                c->p.sep_id, c->p.sep_logit_bias, c->ds.active, M, nullptr, append_args(c, which, forced, mode), decode_seq(c));
}

// The graph of one decode iteration of model `which`, recorded on first use.  Everything an
// iteration reads that changes between replays (positions, activity flags, step index, block
// tables, tokens) lives in device memory, so one recording serves every later iteration with the
// same model, uniforms, teacher arrays and row count.  nullptr: recording is not possible (eager from then on).
template <typename WT>
hipGraphExec_t decode_graph(rsd_ctx* c, int which, const float* u, const int* forced, int mode = 1) {
    for (const auto& g : c->graphs)
        if (g.which == which && g.u == u && g.forced == forced && g.mode == mode && g.rows == c->dec_rows) return g.exec;
    auto give_up = [&]() { (void)hipGetLastError(); c->graphs_ok = false; return (hipGraphExec_t) nullptr; };
    if (!c->cap_st && hipStreamCreateWithFlags(&c->cap_st, hipStreamNonBlocking) != hipSuccess) return give_up();
    if (hipStreamBeginCapture(c->cap_st, hipStreamCaptureModeThreadLocal) != hipSuccess) return give_up();
    hipStream_t user = c->st;
    c->st = c->cap_st;
    decode_iter<WT>(c, which, u, forced, mode);
    c->st = user;
    hipGraph_t graph = nullptr;
    if (hipStreamEndCapture(c->cap_st, &graph) != hipSuccess || !graph) return give_up();
    hipGraphExec_t exec = nullptr;
    if (hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0) != hipSuccess || !exec) {
        (void)hipGraphDestroy(graph);
        return give_up();
    }
    c->graphs.push_back(rsd_ctx::DecodeGraph{which, u, forced, mode, c->dec_rows, graph, exec});
    return exec;
}

// Chunked prefill of `pieces` (per sequence consecutive, ascending) through model `which`.
// after_pass(first_row_of_piece[], pieces_in_pass, M) runs after the layers of every pass.
template <typename WT, typename AfterPass>
int prefill(rsd_ctx* c, int which, std::vector<Piece> pieces, AfterPass after_pass) {
    Model& m = c->m[which];
    // the kernels index the block table without checks: every position a pass touches must lie on a page its
    // row owns, and the device must hold the table the host has
    for (const Piece& pc : pieces)
        if (pc.b < 0 || pc.b >= c->B || pc.start < 0 || pc.end > c->p.max_ctx || pc.end < pc.start ||
            ceil_div(pc.end, RSD_PAGE) > m.n_pages[pc.b])
            return fail(c, RSD_ESTATE, "internal: row %d feeds positions [%d, %d) of model %d but owns %d pages", pc.b, pc.start,
                        pc.end, which, pc.b >= 0 && pc.b < c->B ? m.n_pages[pc.b] : -1);
    if (m.bt_dirty) return fail(c, RSD_ESTATE, "internal: block table of model %d not uploaded before a pass", which);
    size_t i = 0;
    std::vector<Piece> pass;
    std::vector<int> first_row;
    while (i < pieces.size()) {
        pass.clear();
        first_row.clear();
        int M = 0, n_items = 0;
        HIPCHK(c, hipStreamSynchronize(c->st));      // staging buffers of the previous pass are free again
        std::fill(c->last_row_h, c->last_row_h + c->B, -1);
        while (i < pieces.size() && M < kMaxRows) {
            Piece pc = pieces[i];
            const int room = kMaxRows - M;
            Piece take = pc;
            if (pc.end - pc.start > room) take.end = pc.start + room;
            first_row.push_back(M);
            pass.push_back(take);
            for (int r = 0; r < take.end - take.start; r += 4) {
                c->item_row0_h[n_items] = M + r;
                c->item_n_h[n_items++] = std::min(4, take.end - take.start - r);
            }
            for (int p = take.start; p < take.end; ++p, ++M) { c->row_seq_h[M] = take.b; c->row_pos_h[M] = p; }
            // "last row" of a sequence: the final position of its final piece
            const bool final_piece = take.end == pc.end && (i + 1 == pieces.size() || pieces[i + 1].b != pc.b);
            if (final_piece) c->last_row_h[take.b] = M - 1;
            if (take.end < pc.end) { pieces[i].start = take.end; break; }
            ++i;
        }
        HIPCHK(c, hipMemcpyAsync(c->row_seq_dev, c->row_seq_h, M * sizeof(int), hipMemcpyHostToDevice, c->st));
        HIPCHK(c, hipMemcpyAsync(c->row_pos_dev, c->row_pos_h, M * sizeof(int), hipMemcpyHostToDevice, c->st));
        HIPCHK(c, hipMemcpyAsync(c->last_row_dev, c->last_row_h, c->B * sizeof(int), hipMemcpyHostToDevice, c->st));
        HIPCHK(c, hipMemcpyAsync(c->item_row0_dev, c->item_row0_h, n_items * sizeof(int), hipMemcpyHostToDevice, c->st));
        HIPCHK(c, hipMemcpyAsync(c->item_n_dev, c->item_n_h, n_items * sizeof(int), hipMemcpyHostToDevice, c->st));
        c->n_items = n_items;
        c->pf_rows = M;
        c->pf_max_end = 0;
        for (const Piece& pc : pass) c->pf_max_end = std::max(c->pf_max_end, pc.end);
        RowMap rm{c->row_seq_dev, c->row_pos_dev, nullptr, nullptr};
        if (kDebugChecks) {
            const int rc = check_rows(c, which, rm, M);
            if (rc != RSD_OK) return rc;
        }
        run_layers<WT>(c, m, M, rm, false);
        const int rc = after_pass(pass, first_row, M);
        if (rc != RSD_OK) return rc;
    }
    HIPCHK(c, hipGetLastError());
    return RSD_OK;
}

// One stage of token generation (a reasoning step) with an LM model on the
// currently active sequences.  The first iteration feeds whatever the model
// has not seen yet (one token, or a catch-up chunk), the rest one token each.
// mode 2 / max_iters: the draft's proposals of one round of speculative regeneration (at most
// max_iters tokens per sequence, each sequence bounded by its own sd_lim).
template <typename WT>
int gen_stage(rsd_ctx* c, int which, const float* u, const int* forced, int mode = 1, int max_iters = 0) {
    const int B = c->B;
    const int cap = mode == 2 ? max_iters : c->p.step_cap;
    Model& m = c->m[which];
    std::vector<Piece> pieces;
    bool all_single = true;
    int n_act = 0;
    for (int b = 0; b < B; ++b)
        if (c->active()[b]) {
            ++n_act;
            const int s = c->kv_len(which)[b], e = c->ctx_len()[b];
            if (e - s != 1) all_single = false;
            pieces.push_back(Piece{b, s, e});
        }
    if (!n_act) return RSD_OK;
    // (the decode loop appends without host checks: the pages for everything it can write must be reserved)
    for (const Piece& pc : pieces) {
        const int room = mode == 2 ? c->sd_lim()[pc.b] : std::min(pc.end + cap, c->p.max_ctx);
        if (ceil_div(room, RSD_PAGE) > m.n_pages[pc.b])
            return fail(c, RSD_ESTATE, "internal: row %d may grow to %d tokens in model %d but owns %d pages", pc.b, room, which,
                        m.n_pages[pc.b]);
    }
    // A stage that only some sequences take part in (the target's, after the reward model has accepted the
    // others' steps) runs its iterations over packed rows: every launch then costs what the rows in use cost, not
    // what the batch costs.  The row count is rounded up to the next size at which the matrix kernels change
    // (few counts, so few recorded graphs); unused rows are marked -1.  Sequences that finish their step early
    // keep their row until the stage ends.
    struct PackScope {
        rsd_ctx* c;
        ~PackScope() { c->dec_rows = 0; }
    } pack_scope{c};
    c->dec_rows = mode == 1 ? packed_rows(n_act, B) : 0;
    if (c->dec_rows) {
        std::vector<int> seqs;
        for (const Piece& pc : pieces) seqs.push_back(pc.b);
        fill_packed_rows(seqs, c->dec_rows, c->dec_seq_h);
        HIPCHK(c, hipMemcpyAsync(c->dec_seq_dev, c->dec_seq_h, c->dec_rows * sizeof(int), hipMemcpyHostToDevice, c->st));
    }
    const int M = c->dec_rows ? c->dec_rows : B;
    int iters = 0;
    // decode-loop accounting (steps of the reasoning loop only): contexts before the stage
    const bool count = mode == 1 && which < 2;
    std::vector<int> ctx0;
    if (count) ctx0.assign(c->ctx_len(), c->ctx_len() + B);
    const std::vector<int> was_active(c->active(), c->active() + B);
    if (!all_single) {
        int rc = prefill<WT>(c, which, pieces, [&](const std::vector<Piece>&, const std::vector<int>&, int) {
            hipLaunchKernelGGL(gather_rows_kernel, dim3(M), dim3(256), 0, c->st, c->h, c->last_row_dev, m.s.d_model, c->hl,
                               decode_seq(c));
            return RSD_OK;
        });
        if (rc != RSD_OK) return rc;
        lm_head<WT>(c, m, c->hl, M, c->logits, m.s.vocab);
        propose_stash(c, mode);
        sample_rows(c, c->logits, m.s.vocab, m.s.vocab, u, c->ds.ctx_len, c->p.max_ctx, c->p.temperature, c->p.top_p,
                    c->p.sep_id, c->p.sep_logit_bias, c->ds.active, M, nullptr, append_args(c, which, forced, mode),
                    decode_seq(c));
        iters = 1;
    }
    const int first = iters;
    if (count) HIPCHK(c, hipEventRecord(c->it[which].e0, c->st));
    c->in_decode_loop = true;
    while (iters < cap) {
        // an iteration whose launches are timed runs eagerly (events cannot bracket a node of a graph),
        // and so does the first one of a model (it raises the kernels' LDS limits)
        bool timed = false;
        for (auto& q : c->probe) {
            q.iter_on = q.model == which && q.phase == RSD_PROBE_DECODE && q.used + 2 <= q.ev.size() &&
                        (q.iters++ % q.stride) == 0;
            timed |= q.iter_on;
        }
        if (kDebugChecks) {      // the positions live on the device: every iteration is checked, none is replayed
            const int rc = check_rows(c, which, decode_map(c, which), M);
            if (rc != RSD_OK) { c->in_decode_loop = false; return rc; }
        }
        hipGraphExec_t exec = nullptr;
        if (!kDebugChecks && c->p.use_graphs && c->graphs_ok && !timed && c->decode_warm[which])
            exec = decode_graph<WT>(c, which, u, forced, mode);
        if (exec) {
            const hipError_t e = hipGraphLaunch(exec, c->st);
            if (e != hipSuccess) { c->in_decode_loop = false; return fail(c, RSD_EHIP, "hipGraphLaunch: %s", hipGetErrorString(e)); }
            ++c->n_graph_replays;
        } else {
            decode_iter<WT>(c, which, u, forced, mode);
            ++c->n_eager_iters;
            c->decode_warm[which] = true;
        }
        ++iters;
        if (iters % kPoll == 0 || iters == cap) {
            HIPCHK(c, hipMemcpyAsync(c->poll_h, c->ds.n_active, sizeof(int), hipMemcpyDeviceToHost, c->st));
            HIPCHK(c, hipStreamSynchronize(c->st));
            if (*c->poll_h <= 0) break;
        }
    }
    c->in_decode_loop = false;
    for (auto& q : c->probe) q.iter_on = false;
    if (count) {
        rsd_ctx::IterStats& is = c->it[which];
        HIPCHK(c, hipEventRecord(is.e1, c->st));
        int rc = pull_state(c);
        if (rc) return rc;
        if (iters > first) {
            float ms = 0.f;
            HIPCHK(c, hipEventElapsedTime(&ms, is.e0, is.e1));
            is.ms += ms;
            is.iters += iters - first;
            is.row_iters += (long long)(iters - first) * M;
            for (int b = 0; b < B; ++b) {
                if (!was_active[b]) continue;
                // tokens this sequence sampled inside the loop; its j-th one attends to ctx0 + first + j keys
                const long long n = std::max(0, c->ctx_len()[b] - ctx0[b] - first);
                is.seq_iters += n;
                is.kv_read += n * (ctx0[b] + first) + n * (n - 1) / 2;
            }
        }
    }
    HIPCHK(c, hipGetLastError());
    return RSD_OK;
}

// Token rows as handed to the caller: the committed tokens, then -1 (what lies behind them in the device buffer
// - rolled-back steps, losing candidates, memory never written - is nobody's business)
void blank_tails(int32_t* tokens, int rows, int max_ctx, const int* ctx_len_of_row) {
    for (int r = 0; r < rows; ++r) {
        const int n = std::min(std::max(ctx_len_of_row[r], 0), max_ctx);
        std::fill(tokens + (size_t)r * max_ctx + n, tokens + (size_t)(r + 1) * max_ctx, -1);
    }
}

int gen_stage_any(rsd_ctx* c, int which, const float* u, const int* forced, int mode = 1, int max_iters = 0) {
    return c->m[which].s.dtype == RSD_F32 ? gen_stage<float>(c, which, u, forced, mode, max_iters)
                                          : gen_stage<bf16_t>(c, which, u, forced, mode, max_iters);
}

// tokens[b][ctx_pre[b] + j] -> dst[b][j], j < step_cap
__global__ void extract_step_kernel(const int* tokens, const int* ctx_pre, const int* ctx_len, int max_ctx, int cap, int* dst) {
    const int b = blockIdx.x;
    for (int j = threadIdx.x; j < cap; j += blockDim.x) {
        const int p = ctx_pre[b] + j;
        dst[b * cap + j] = (p < ctx_len[b]) ? tokens[(size_t)b * max_ctx + p] : -1;
    }
}

int fetch_step_tokens(rsd_ctx* c) {
    hipLaunchKernelGGL(extract_step_kernel, dim3(c->B), dim3(64), 0, c->st, c->ds.tokens, c->ds.ctx_pre, c->ds.ctx_len,
                       c->p.max_ctx, c->p.step_cap, c->steptok_dev);
    HIPCHK(c, hipMemcpyAsync(c->steptok_h, c->steptok_dev, (size_t)c->B * c->p.step_cap * sizeof(int), hipMemcpyDeviceToHost, c->st));
    return RSD_OK;
}

// Sampled verification, shared by the engine and the stand-alone entry point: the sampler's phases on
// the target's rows (their own draws land in `choice`) and on the draft's rows in use, then the
// acceptance test of every proposal.  sd_sampled_replace then draws the replacement at where[s].
int sd_sampled_verify(rsd_ctx* c, const float* p_logits, int p_rows, const float* q_logits, const int* p_uidx,
                      const int* q_uidx, const int* q_active, const float* u_new, int* choice, int nseq, const int* live,
                      const int* n_prop_base, const int* n_prop_end, const int* p_row0, const int* tok, int tok_stride,
                      const int* tok_off, const float* u_acc, int u_stride, const int* u_off, int* kept_own) {
    const rsd_params& P = c->p;
    const int V = c->m[RSD_TARGET].s.vocab, k = P.sd_k;
    AppendArgs off{};
    auto& wp = c->sd_ws[0];
    auto& wq = c->sd_ws[1];
    SampleArgs ap{p_logits, V, V, u_new, p_uidx, 0, P.temperature, P.top_p, P.sep_id, P.sep_logit_bias, nullptr, choice,
                  wp.pmax, wp.pidx, wp.hist, wp.psum, wp.sel};
    sample_launch(c->st, ap, off, p_rows);
    SampleArgs aq{q_logits, V, V, u_new, q_uidx, 0, P.temperature, P.top_p, P.sep_id, P.sep_logit_bias, q_active, nullptr,
                  wq.pmax, wq.pidx, wq.hist, wq.psum, wq.sel};
    sample_launch(c->st, aq, off, nseq * k);
    SdVerifyArgs& va = c->sd_va;
    va = SdVerifyArgs{};
    va.p = SdRowSet{p_logits, V, wp.pmax, wp.psum, wp.sel};
    va.q = SdRowSet{q_logits, V, wq.pmax, wq.psum, wq.sel};
    va.V = V; va.k = k; va.temperature = P.temperature; va.sep_id = P.sep_id; va.sep_bias = P.sep_logit_bias;
    va.live = live; va.n_prop_base = n_prop_base; va.n_prop_end = n_prop_end; va.p_row0 = p_row0;
    va.tok = tok; va.tok_stride = tok_stride; va.tok_off = tok_off;
    va.u_acc = u_acc; va.u_stride = u_stride; va.u_off = u_off; va.u_new = u_new;
    va.kept_own = kept_own; va.acc_own = c->sd_acc_own; va.choice = choice; va.rpart = c->sd_rpart;
    hipLaunchKernelGGL(sd_accept_kernel, dim3(nseq), dim3(64), 0, c->st, va);
    HIPCHK(c, hipGetLastError());
    return RSD_OK;
}
void sd_sampled_replace(rsd_ctx* c, int nseq, const int* where) {
    hipLaunchKernelGGL(sd_residual_mass_kernel, dim3(SMP_NB, nseq), dim3(SMP_T), 0, c->st, c->sd_va, where);
    hipLaunchKernelGGL(sd_residual_draw_kernel, dim3(nseq), dim3(SMP_T), 0, c->st, c->sd_va, where);
}

// Target step of the rejected sequences by token-level speculative decoding with the draft
// (Section 5, "Combine RSD with SD"), greedy.  On entry the host mirror is current and active[] marks
// the rejected sequences.  Each round: the host fixes every live sequence's proposal budget, the
// draft decodes up to sd_k proposals, the target reads its unseen tokens and the proposals in one
// chunked pass, its head and arg max run on the last proposals + 1 rows of every sequence, and
// sd_verify_kernel commits.  The host reads the state back twice per round (it builds the row maps).
template <typename WT>
int sd_stage(rsd_ctx* c) {
    const int B = c->B, k = c->p.sd_k;
    const rsd_params& P = c->p;
    Model& mt = c->m[RSD_TARGET];
    const int d = mt.s.d_model, V = mt.s.vocab;
    for (int b = 0; b < B; ++b) {
        c->sd_live()[b] = c->active()[b];
        c->sd_nprop()[b] = c->sd_nkept()[b] = c->sd_nround()[b] = 0;
    }
    int rc;
    for (;;) {
        int n_live = 0, n_prop = 0, max_g = 0;
        for (int b = 0; b < B; ++b) {
            c->active()[b] = 0;
            if (!c->sd_live()[b]) continue;
            ++n_live;
            const int n = c->ctx_len()[b], used = n - c->ctx_pre()[b];
            const int g = std::max(0, std::min(k, std::min(P.step_cap - used - 1, P.max_ctx - n - 1)));
            c->sd_base()[b] = n;
            c->sd_lim()[b] = n + g;
            // both models feed the newest committed token again (its keys may be missing or stale)
            c->kv_len(RSD_DRAFT)[b] = std::min(c->kv_len(RSD_DRAFT)[b], n - 1);
            c->kv_len(RSD_TARGET)[b] = std::min(c->kv_len(RSD_TARGET)[b], n - 1);
            if (g > 0) { c->active()[b] = 1; ++n_prop; max_g = std::max(max_g, g); }
        }
        if (!n_live) break;
        *c->n_active() = n_prop;
        if ((rc = push_state(c))) return rc;
        if (n_prop) {
            if ((rc = gen_stage_any(c, RSD_DRAFT, c->u_prop, c->forced_prop, 2, max_g))) return rc;
            if ((rc = pull_state(c))) return rc;
        }
        // ---- the target's pass: catch-up first when everything together exceeds one pass
        std::vector<Piece> pieces;
        long long rows_all = 0;
        for (int b = 0; b < B; ++b)
            if (c->sd_live()[b]) rows_all += c->ctx_len()[b] - c->kv_len(RSD_TARGET)[b];
        if (rows_all > kMaxRows) {
            for (int b = 0; b < B; ++b)
                if (c->sd_live()[b] && c->kv_len(RSD_TARGET)[b] < c->sd_base()[b] - 1)
                    pieces.push_back(Piece{b, c->kv_len(RSD_TARGET)[b], c->sd_base()[b] - 1});
            rc = prefill<WT>(c, RSD_TARGET, pieces, [](const std::vector<Piece>&, const std::vector<int>&, int) { return RSD_OK; });
            if (rc) return rc;
            for (const Piece& pc : pieces) c->kv_len(RSD_TARGET)[pc.b] = pc.end;
            pieces.clear();
        }
        int n_rows = 0;
        for (int b = 0; b < B; ++b)
            if (c->sd_live()[b]) pieces.push_back(Piece{b, c->kv_len(RSD_TARGET)[b], c->ctx_len()[b]});
        auto after = [&](const std::vector<Piece>& pass, const std::vector<int>& first_row, int) {
            // one pass holds every piece whole here: the rows of the last proposals + 1 positions
            int* rows = c->sd_rows_h;
            int* row0 = c->sd_rows_h + (size_t)B * (k + 1);
            std::fill(row0, row0 + B, 0);
            for (size_t i = 0; i < pass.size(); ++i) {
                const Piece& pc = pass[i];
                const int cnt = pc.end - c->sd_base()[pc.b] + 1;
                row0[pc.b] = n_rows;
                for (int j = 0; j < cnt; ++j) rows[n_rows++] = first_row[i] + (pc.end - pc.start) - cnt + j;
            }
            HIPCHK(c, hipMemcpyAsync(c->sd_rows_dev, c->sd_rows_h, ((size_t)B * (k + 2)) * sizeof(int), hipMemcpyHostToDevice, c->st));
            hipLaunchKernelGGL(gather_rows_kernel, dim3(n_rows), dim3(256), 0, c->st, c->h, c->sd_rows_dev, d, c->sd_h,
                               (const int*)nullptr);
            return RSD_OK;
        };
        if ((rc = prefill<WT>(c, RSD_TARGET, pieces, after))) return rc;
        lm_head<WT>(c, mt, c->sd_h, n_rows, c->sd_logits, V);
        AppendArgs off{};
        if (P.temperature == 0.f) {
            sample_rows(c, c->sd_logits, V, V, nullptr, nullptr, 0, 0.0f, 1.0f, P.sep_id, P.sep_logit_bias, nullptr, n_rows,
                        c->sd_choice, off);
        } else {
            // uniform of every target row (the token the target would draw at that place) and the draft rows in use
            const int rows = B * (k + 1), qrows = B * k;
            int *pu = c->sd_aux_h, *qu = pu + rows, *qa = qu + qrows;
            std::fill(qa, qa + qrows, 0);
            const int* row0 = c->sd_rows_h + (size_t)B * (k + 1);
            for (int b = 0; b < B; ++b) {
                if (!c->sd_live()[b]) continue;
                const int base = c->sd_base()[b], np = c->ctx_len()[b] - base;
                for (int i = 0; i <= np; ++i) pu[row0[b] + i] = b * P.max_ctx + base + i;
                for (int i = 0; i < np; ++i) { qu[b * k + i] = b * P.max_ctx + base + i; qa[b * k + i] = 1; }
            }
            HIPCHK(c, hipMemcpyAsync(c->sd_aux_dev, c->sd_aux_h, (size_t)(rows + 2 * qrows) * sizeof(int), hipMemcpyHostToDevice, c->st));
            int rc2 = sd_sampled_verify(c, c->sd_logits, n_rows, c->sd_qlogits, c->sd_aux_dev, c->sd_aux_dev + rows,
                                        c->sd_aux_dev + rows + qrows, c->u_target, c->sd_choice, B, c->ds.sd_live, c->ds.sd_base,
                                        c->ds.ctx_len, c->sd_rows_dev + (size_t)B * (k + 1), c->ds.tokens, P.max_ctx, c->ds.sd_base,
                                        c->u_acc, P.max_ctx, c->ds.sd_base, c->sd_kept_own);
            if (rc2) return rc2;
            hipLaunchKernelGGL(sd_where_kernel, dim3(ceil_div(B, 64)), dim3(64), 0, c->st, c->ds, B, k, c->forced_target,
                               c->sd_kept_own, c->sd_acc_own, P.max_ctx, P.max_steps, P.step_cap, P.step_cap * k, c->sd_where,
                               c->sd_acc_rec);
            sd_sampled_replace(c, B, c->sd_where);
        }
        hipLaunchKernelGGL(sd_verify_kernel, dim3(ceil_div(B, 64)), dim3(64), 0, c->st, c->ds, B,
                           c->sd_rows_dev + (size_t)B * (k + 1), c->sd_choice, c->forced_target, P.max_ctx, P.max_steps,
                           P.step_cap, P.sep_id, P.eos_id);
        if ((rc = pull_state(c))) return rc;
    }
    HIPCHK(c, hipGetLastError());
    return RSD_OK;
}

// ---- process Best-of-N: candidates of a step fork from the sequence's committed lane
// tokens[lane][0 .. n[lane]) = tokens[src[lane]][...] for every lane with src[lane] >= 0 and != lane
__global__ void bon_fork_tokens_kernel(int* __restrict__ tokens, int max_ctx, const int* __restrict__ src,
                                       const int* __restrict__ n) {
    const int lane = blockIdx.x, from = src[lane];
    if (from < 0 || from == lane) return;
    const int cnt = n[lane];
    for (int i = threadIdx.x; i < cnt; i += blockDim.x)
        tokens[(size_t)lane * max_ctx + i] = tokens[(size_t)from * max_ctx + i];
}
// physical page pairs[2 i] -> pairs[2 i + 1] in every layer (blockIdx.y) of one model's pool
__global__ void bon_copy_pages_kernel(char* __restrict__ pool, size_t layer_bytes, size_t page_bytes,
                                      const int* __restrict__ pairs) {
    const int from = pairs[2 * blockIdx.x], to = pairs[2 * blockIdx.x + 1];
    const uint4* s = reinterpret_cast<const uint4*>(pool + blockIdx.y * layer_bytes + (size_t)from * page_bytes);
    uint4* d = reinterpret_cast<uint4*>(pool + blockIdx.y * layer_bytes + (size_t)to * page_bytes);
    for (size_t i = threadIdx.x; i < page_bytes / 16; i += blockDim.x) d[i] = s[i];
}

// Recorded decode iterations bake in the uniform and teacher arrays they were recorded with: drop those
// whose arrays the caller has replaced, so that the cache holds at most one graph per live combination.
int drop_stale_graphs(rsd_ctx* c) {
    if (c->graphs.empty()) return RSD_OK;
    auto live_u = [&](const float* u) { return u == c->u_draft || u == c->u_target || u == c->u_prop; };
    auto live_f = [&](const int* f) { return f == c->forced_draft || f == c->forced_target || f == c->forced_prop; };
    bool synced = false;
    for (size_t i = 0; i < c->graphs.size();) {
        const auto& g = c->graphs[i];
        if (live_u(g.u) && live_f(g.forced)) { ++i; continue; }
        if (!synced) { HIPCHK(c, hipStreamSynchronize(c->st)); synced = true; }
        (void)hipGraphExecDestroy(g.exec);
        (void)hipGraphDestroy(g.graph);
        c->graphs.erase(c->graphs.begin() + i);
    }
    return RSD_OK;
}

double now_ms() {
    return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

void reset_sequences(rsd_ctx* c) {
    for (int i = 0; i < 3; ++i)
        for (int b = 0; b < c->B; ++b) trim_pages(c->m[i], b, 0);
    std::fill(c->sb, c->sb + c->sb_ints, 0);
    c->steps_done = 0;
}

}  // namespace

// =========================================================================== C ABI
extern "C" {

const char* rsd_last_error(const rsd_ctx* c) { return c ? c->err.c_str() : "null context"; }

void rsd_destroy(rsd_ctx* c) {
    if (!c) return;
    (void)hipStreamSynchronize(c->st);
    for (auto& m : c->m) {
        (void)hipFree(m.pool); (void)hipFree(m.bt_dev); (void)hipFree(m.rope);
        if (m.bt_host) (void)hipHostFree(m.bt_host);
    }
    void* dev[] = {c->sb_dev, c->ds.tokens, c->ds.sampled[0], c->ds.sampled[1], c->ds.sampled[2], c->sd_h, c->sd_logits, c->sd_choice, c->sd_rows_dev, c->sd_qlogits, c->sd_aux_dev,
                   c->sd_kept_own, c->sd_where, c->sd_acc_own, c->sd_acc_rec, c->sd_rpart,
                   c->sd_ws[0].pmax, c->sd_ws[0].pidx, c->sd_ws[0].hist, c->sd_ws[0].psum, c->sd_ws[0].sel,
                   c->sd_ws[1].pmax, c->sd_ws[1].pidx, c->sd_ws[1].hist, c->sd_ws[1].psum, c->sd_ws[1].sel, c->h, c->xn, c->qkv, c->att, c->gu, c->act,
                   c->part_acc, c->part_ml, c->part_k, c->xs_h, c->xs_l, c->smp_pmax, c->smp_pidx, c->smp_hist, c->smp_psum, c->smp_sel, c->hl, c->xl, c->logits, c->tmp_reward, c->chosen, c->steptok_dev,
                   c->row_seq_dev, c->row_pos_dev, c->last_row_dev, c->item_row0_dev, c->item_n_dev, c->bon_copy_dev, c->bon_src_dev, c->dec_seq_dev, c->chk_n_pages_dev, c->chk_err_dev, c->clk_dev};
    for (void* p : dev) if (p) (void)hipFree(p);
    for (auto& q : c->probe)
        for (hipEvent_t e : q.ev) (void)hipEventDestroy(e);
    for (auto& is : c->it) {
        if (is.e0) (void)hipEventDestroy(is.e0);
        if (is.e1) (void)hipEventDestroy(is.e1);
    }
    for (auto& g : c->graphs) { (void)hipGraphExecDestroy(g.exec); (void)hipGraphDestroy(g.graph); }
    if (c->cap_st) (void)hipStreamDestroy(c->cap_st);
    void* pin[] = {c->sb, c->sd_rows_h, c->sd_aux_h, c->item_row0_h, c->item_n_h, c->row_seq_h, c->row_pos_h, c->last_row_h, c->steptok_h, c->poll_h,
                   c->bon_copy_h, c->bon_src_h, c->dec_seq_h, c->chk_h};
    for (void* p : pin) if (p) (void)hipHostFree(p);
    delete c;
}

int rsd_init(rsd_ctx** out, const rsd_model_shape shape[3], const rsd_weights w[3], const rsd_params* p, int32_t batch,
             void* hip_stream) {
    if (!out) return RSD_EINVAL;
    *out = nullptr;
    rsd_ctx* c = new rsd_ctx();
    *out = c;   // handed back even on failure so that the caller can read the error, then destroy
    if (!shape || !w || !p) return fail(c, RSD_EINVAL, "null argument");
    c->p = *p;
    c->B = batch;
    c->st = static_cast<hipStream_t>(hip_stream);
    if (batch < 1 || batch > 4096) return fail(c, RSD_EINVAL, "batch %d out of range", batch);
    if (p->page_tokens != RSD_PAGE) return fail(c, RSD_EINVAL, "page_tokens must be %d", RSD_PAGE);
    if (p->step_cap < 1 || p->max_steps < 1 || p->max_ctx < 2) return fail(c, RSD_EINVAL, "bad step_cap/max_steps/max_ctx");
    if (p->temperature < 0.f || p->top_p < 0.f || p->top_p > 1.f) return fail(c, RSD_EINVAL, "bad temperature/top_p");
    if (p->omega_kind < 0 || p->omega_kind > 4) return fail(c, RSD_EINVAL, "bad omega_kind");
    if (p->merge_prm < RSD_MERGE_NONE || p->merge_prm > RSD_MERGE_TARGET) return fail(c, RSD_EINVAL, "bad merge_prm");
    if (p->sd_k < 0 || p->sd_k > 15) return fail(c, RSD_EINVAL, "sd_k %d outside [0, 15]", p->sd_k);
    if (p->sd_k > 0 && (long long)batch * (p->sd_k + 1) > kMaxRows)
        return fail(c, RSD_EINVAL, "batch * (sd_k + 1) exceeds the %d rows of one verification pass", kMaxRows);
    const bool bon = p->bon_n > 0;
    if (p->bon_n < 0 || p->bon_n > 1024) return fail(c, RSD_EINVAL, "bon_n %d outside [0, 1024]", p->bon_n);
    if (bon && (batch % p->bon_n || p->merge_prm != RSD_MERGE_NONE || p->sd_k != 0))
        return fail(c, RSD_EINVAL, "Best-of-N: batch must be a multiple of bon_n, and merge_prm and sd_k must be 0");
    c->n_seq = bon ? batch / p->bon_n : batch;
    c->canon.resize(c->n_seq);
    for (int s2 = 0; s2 < c->n_seq; ++s2) c->canon[s2] = bon ? s2 * p->bon_n : s2;
    for (int i = 0; i < 3; ++i) {
        if (bon && i == RSD_TARGET) continue;           // no target model in Best-of-N
        int rc = setup_model(c, c->m[i], shape[i], w[i], i, i == RSD_PRM && p->merge_prm != RSD_MERGE_NONE);
        if (rc) return rc;
    }
    if (p->merge_prm != RSD_MERGE_NONE) {
        const rsd_model_shape& a = shape[p->merge_prm == RSD_MERGE_DRAFT ? RSD_DRAFT : RSD_TARGET];
        const rsd_model_shape& r = shape[RSD_PRM];
        if (a.n_layers != r.n_layers || a.d_model != r.d_model || a.n_heads != r.n_heads || a.n_kv_heads != r.n_kv_heads ||
            a.d_ffn != r.d_ffn || a.dtype != r.dtype)
            return fail(c, RSD_EINVAL, "merged reward model: its shape must repeat the policy model's");
    }
    if ((!bon && shape[0].vocab != shape[1].vocab) || shape[0].vocab != shape[2].vocab)
        return fail(c, RSD_EINVAL, "the models must share one vocabulary");
    if (p->sep_id < 0 || p->sep_id >= shape[0].vocab || p->eos_id >= shape[0].vocab)
        return fail(c, RSD_EINVAL, "sep_id/eos_id outside the vocabulary");
    for (int i = 0; i < 3; ++i) {
        if ((i == RSD_PRM && p->merge_prm != RSD_MERGE_NONE) || (bon && i == RSD_TARGET)) {      // no cache for this one
            c->m[i].n_pages.assign(batch, 0);
            continue;
        }
        int rc = setup_kv(c, c->m[i], i);
        if (rc) return rc;
    }
    const int B = batch;
    const size_t mc = p->max_ctx;
    c->sb_ints = (size_t)18 * B + 4;
    HIPCHK(c, dev_alloc(&c->sb_dev, c->sb_ints));
    HIPCHK(c, pin_alloc(&c->sb, c->sb_ints));
    std::fill(c->sb, c->sb + c->sb_ints, 0);
    HIPCHK(c, dev_alloc(&c->ds.tokens, B * mc));
    HIPCHK(c, dev_alloc(&c->ds.sampled[0], (size_t)B * p->max_steps * p->step_cap));
    HIPCHK(c, dev_alloc(&c->ds.sampled[1], (size_t)B * p->max_steps * p->step_cap));
    HIPCHK(c, dev_alloc(&c->ds.sampled[2], (size_t)B * p->max_steps * p->step_cap * p->sd_k));
    c->ds.ctx_len = c->sb_dev;
    c->ds.kv_len = c->sb_dev + B;
    c->ds.active = c->sb_dev + 4 * B;
    c->ds.step_len = c->sb_dev + 5 * B;
    c->ds.finished = c->sb_dev + 6 * B;
    c->ds.ctx_pre = c->sb_dev + 7 * B;
    c->ds.accepted = c->sb_dev + 8 * B;
    c->ds.own_accept = c->sb_dev + 9 * B;
    c->ds.reward = reinterpret_cast<float*>(c->sb_dev + 10 * B);
    c->in_step_dev = c->sb_dev + 11 * B;
    c->ds.n_active = c->sb_dev + 12 * B;
    c->ds.cur_step = c->sb_dev + 12 * B + 1;
    c->ds.sd_live = c->sb_dev + 12 * B + 4;
    c->ds.sd_base = c->sb_dev + 13 * B + 4;
    c->ds.sd_lim = c->sb_dev + 14 * B + 4;
    c->ds.sd_nprop = c->sb_dev + 15 * B + 4;
    c->ds.sd_nkept = c->sb_dev + 16 * B + 4;
    c->ds.sd_nround = c->sb_dev + 17 * B + 4;
    // workspaces sized for the widest model
    int d = 0, nq = 0, qd = 0, F = 0, V = 0, HS = 0;
    for (auto& m : c->m) {
        d = std::max(d, m.s.d_model); nq = std::max(nq, m.n_qkv); qd = std::max(qd, m.q_dim);
        F = std::max(F, m.s.d_ffn); V = std::max(V, m.s.vocab);
        HS = std::max(HS, m.s.n_heads * m.splits * m.hd);
    }
    const size_t R = std::max(kMaxRows, B);
    c->ws_rows = (int)R;
    HIPCHK(c, dev_alloc(&c->h, R * d));
    HIPCHK(c, dev_alloc(&c->xn, R * d));
    HIPCHK(c, dev_alloc(&c->qkv, R * nq));
    HIPCHK(c, dev_alloc(&c->att, R * qd));
    HIPCHK(c, dev_alloc(&c->gu, R * 2 * F));
    HIPCHK(c, dev_alloc(&c->act, R * F));
    size_t part = (size_t)B * HS;        // decode splits, or the splits of a small chunked pass
    for (auto& m : c->m) part = std::max(part, (size_t)kPfSplitRows * m.s.n_heads * kPfSplits * m.hd);
    HIPCHK(c, dev_alloc(&c->part_acc, part));
    HIPCHK(c, dev_alloc(&c->part_ml, part));
    c->part_k_floats = (size_t)48 << 20;
    HIPCHK(c, dev_alloc(&c->part_k, c->part_k_floats));
    HIPCHK(c, dev_alloc(&c->clk_dev, 3 * RSD_PROBE_SLOTS));
    HIPCHK(c, hipMemsetAsync(c->clk_dev, 0, 3 * RSD_PROBE_SLOTS * sizeof(unsigned long long), c->st));
    {
        const size_t kmax = (size_t)std::max(std::max(d, qd), F), xr = std::max<size_t>(R, 64);
        HIPCHK(c, dev_alloc(&c->xs_h, xr * kmax));
        HIPCHK(c, dev_alloc(&c->xs_l, xr * kmax));
        HIPCHK(c, hipMemsetAsync(c->xs_h, 0, xr * kmax * sizeof(uint16_t), c->st));
        HIPCHK(c, hipMemsetAsync(c->xs_l, 0, xr * kmax * sizeof(uint16_t), c->st));
    }
    c->smp_rows = std::max(B, 64);
    HIPCHK(c, dev_alloc(&c->smp_pmax, (size_t)c->smp_rows * SMP_NB));
    HIPCHK(c, dev_alloc(&c->smp_pidx, (size_t)c->smp_rows * SMP_NB));
    HIPCHK(c, dev_alloc(&c->smp_hist, (size_t)c->smp_rows * 3 * SMP_BINS));
    HIPCHK(c, dev_alloc(&c->smp_psum, (size_t)c->smp_rows * SMP_NB));
    HIPCHK(c, dev_alloc(&c->smp_sel, (size_t)c->smp_rows * 8));
    HIPCHK(c, hipMemsetAsync(c->smp_hist, 0, (size_t)c->smp_rows * 3 * SMP_BINS * sizeof(u64_t), c->st));
    HIPCHK(c, hipMemsetAsync(c->smp_sel, 0, (size_t)c->smp_rows * 8 * sizeof(u64_t), c->st));
    HIPCHK(c, dev_alloc(&c->hl, (size_t)B * d));
    HIPCHK(c, dev_alloc(&c->xl, (size_t)B * d));
    HIPCHK(c, dev_alloc(&c->logits, (size_t)B * V));
    HIPCHK(c, dev_alloc(&c->tmp_reward, R));
    if (p->sd_k > 0) {
        const size_t rows = (size_t)B * (p->sd_k + 1);
        HIPCHK(c, dev_alloc(&c->sd_h, rows * d));
        HIPCHK(c, dev_alloc(&c->sd_logits, rows * V));
        HIPCHK(c, dev_alloc(&c->sd_choice, rows));
        HIPCHK(c, dev_alloc(&c->sd_rows_dev, rows + B));
        HIPCHK(c, pin_alloc(&c->sd_rows_h, rows + B));
        std::fill(c->sd_rows_h, c->sd_rows_h + rows + B, 0);
        HIPCHK(c, dev_alloc(&c->sd_acc_rec, (size_t)B * p->max_steps * p->step_cap * p->sd_k));
        if (p->temperature > 0.f) {
            const size_t qrows = (size_t)B * p->sd_k;
            HIPCHK(c, dev_alloc(&c->sd_qlogits, qrows * V));
            for (int i = 0; i < 2; ++i) {
                const size_t n = i == 0 ? rows : qrows;
                auto& ws = c->sd_ws[i];
                HIPCHK(c, dev_alloc(&ws.pmax, n * SMP_NB));
                HIPCHK(c, dev_alloc(&ws.pidx, n * SMP_NB));
                HIPCHK(c, dev_alloc(&ws.hist, n * 3 * SMP_BINS));
                HIPCHK(c, dev_alloc(&ws.psum, n * SMP_NB));
                HIPCHK(c, dev_alloc(&ws.sel, n * 8));
                HIPCHK(c, hipMemsetAsync(ws.hist, 0, n * 3 * SMP_BINS * sizeof(u64_t), c->st));
                HIPCHK(c, hipMemsetAsync(ws.sel, 0, n * 8 * sizeof(u64_t), c->st));
            }
            HIPCHK(c, dev_alloc(&c->sd_aux_dev, rows + 2 * qrows));
            HIPCHK(c, pin_alloc(&c->sd_aux_h, rows + 2 * qrows));
            std::fill(c->sd_aux_h, c->sd_aux_h + rows + 2 * qrows, 0);
            HIPCHK(c, dev_alloc(&c->sd_kept_own, (size_t)B));
            HIPCHK(c, dev_alloc(&c->sd_where, (size_t)B));
            HIPCHK(c, dev_alloc(&c->sd_acc_own, qrows));
            HIPCHK(c, dev_alloc(&c->sd_rpart, (size_t)B * SMP_NB));
        }
    }
    HIPCHK(c, dev_alloc(&c->chosen, (size_t)B));
    HIPCHK(c, dev_alloc(&c->steptok_dev, (size_t)B * p->step_cap));
    HIPCHK(c, dev_alloc(&c->row_seq_dev, R));
    HIPCHK(c, dev_alloc(&c->row_pos_dev, R));
    HIPCHK(c, dev_alloc(&c->last_row_dev, (size_t)B));
    HIPCHK(c, dev_alloc(&c->dec_seq_dev, (size_t)B));
    HIPCHK(c, dev_alloc(&c->chk_n_pages_dev, (size_t)B));
    HIPCHK(c, dev_alloc(&c->chk_err_dev, (size_t)4));
    HIPCHK(c, dev_alloc(&c->item_row0_dev, R));
    HIPCHK(c, dev_alloc(&c->item_n_dev, R));
    HIPCHK(c, pin_alloc(&c->item_row0_h, R));
    HIPCHK(c, pin_alloc(&c->item_n_h, R));
    HIPCHK(c, pin_alloc(&c->row_seq_h, R));
    HIPCHK(c, pin_alloc(&c->row_pos_h, R));
    HIPCHK(c, pin_alloc(&c->last_row_h, (size_t)B));
    HIPCHK(c, pin_alloc(&c->dec_seq_h, (size_t)B));
    HIPCHK(c, pin_alloc(&c->chk_h, (size_t)B + 4));
    HIPCHK(c, pin_alloc(&c->steptok_h, (size_t)B * p->step_cap));
    HIPCHK(c, pin_alloc(&c->poll_h, 4));
    if (bon) {
        HIPCHK(c, pin_alloc(&c->bon_copy_h, (size_t)4 * B));        // [model 0: B pairs][model 2: B pairs]
        HIPCHK(c, dev_alloc(&c->bon_copy_dev, (size_t)4 * B));
        HIPCHK(c, pin_alloc(&c->bon_src_h, (size_t)2 * B));         // source lane and token count of every lane
        HIPCHK(c, dev_alloc(&c->bon_src_dev, (size_t)2 * B));
    }
    for (auto& is : c->it) {
        HIPCHK(c, hipEventCreate(&is.e0));
        HIPCHK(c, hipEventCreate(&is.e1));
    }
    HIPCHK(c, hipMemsetAsync(c->h, 0, R * d * sizeof(float), c->st));
    HIPCHK(c, hipMemsetAsync(c->hl, 0, (size_t)B * d * sizeof(float), c->st));
    HIPCHK(c, hipMemsetAsync(c->att, 0, R * qd * sizeof(float), c->st));
    HIPCHK(c, hipMemsetAsync(c->gu, 0, R * 2 * F * sizeof(float), c->st));
    HIPCHK(c, hipMemsetAsync(c->logits, 0, (size_t)B * V * sizeof(float), c->st));
    HIPCHK(c, hipStreamSynchronize(c->st));
    c->prompt_len.assign(B, 0);
    return RSD_OK;
}

int rsd_set_prompts(rsd_ctx* c, const int32_t* tokens_dev, const int32_t* prompt_len_host) {
    if (!c || !tokens_dev || !prompt_len_host) return fail(c, RSD_EINVAL, "null argument");
    const int B = c->B;
    const int N = c->p.bon_n > 0 ? c->p.bon_n : 1;      // Best-of-N: one prompt per sequence, placed in its first lane
    for (int b = 0; b < c->n_seq; ++b)
        if (prompt_len_host[b] < 1 || prompt_len_host[b] > c->p.max_ctx)
            return fail(c, RSD_EINVAL, "prompt_len[%d] = %d outside [1, max_ctx]", b, prompt_len_host[b]);
    HIPCHK(c, hipStreamSynchronize(c->st));
    reset_sequences(c);
    const size_t row = (size_t)c->p.max_ctx * sizeof(int);
    HIPCHK(c, hipMemcpy2DAsync(c->ds.tokens, row * N, tokens_dev, row, row, c->n_seq, hipMemcpyDeviceToDevice, c->st));
    for (int s2 = 0; s2 < c->n_seq; ++s2) c->canon[s2] = s2 * N;
    const size_t ns = (size_t)B * c->p.max_steps * c->p.step_cap;
    for (int s = 0; s < 2; ++s)
        hipLaunchKernelGGL(fill_int_kernel, dim3((unsigned)((ns + 255) / 256)), dim3(256), 0, c->st, c->ds.sampled[s], -1, ns);
    if (const size_t np = ns * c->p.sd_k) {
        hipLaunchKernelGGL(fill_int_kernel, dim3((unsigned)((np + 255) / 256)), dim3(256), 0, c->st, c->ds.sampled[2], -1, np);
        hipLaunchKernelGGL(fill_int_kernel, dim3((unsigned)((np + 255) / 256)), dim3(256), 0, c->st, c->sd_acc_rec, -1, np);
    }
    for (int b = 0; b < B; ++b) {
        const int pl = prompt_len_host[b / N];
        c->prompt_len[b] = pl;
        c->ctx_len()[b] = pl;
        c->finished()[b] = pl >= c->p.max_ctx ? RSD_FIN_MAX_CTX : RSD_RUNNING;
    }
    int rc = push_state(c);
    if (rc) return rc;
    HIPCHK(c, hipStreamSynchronize(c->st));
    c->have_prompts = true;
    return RSD_OK;
}

int rsd_set_uniforms(rsd_ctx* c, const float* u_draft_dev, const float* u_target_dev, const float* u_gate_dev) {
    if (!c) return RSD_EINVAL;
    c->u_draft = u_draft_dev; c->u_target = u_target_dev; c->u_gate = u_gate_dev;
    return drop_stale_graphs(c);
}

int rsd_set_criterion(rsd_ctx* c, float delta, int32_t omega_kind, float omega_a) {
    if (!c) return RSD_EINVAL;
    if (omega_kind < 0 || omega_kind > 4) return fail(c, RSD_EINVAL, "bad omega_kind");
    c->p.delta = delta; c->p.omega_kind = omega_kind; c->p.omega_a = omega_a;
    return RSD_OK;
}

int rsd_set_teacher(rsd_ctx* c, const int32_t* forced_draft_dev, const int32_t* forced_target_dev,
                    const int32_t* forced_accept_dev) {
    if (!c) return RSD_EINVAL;
    c->forced_draft = forced_draft_dev; c->forced_target = forced_target_dev; c->forced_accept = forced_accept_dev;
    return drop_stale_graphs(c);
}

int rsd_step(rsd_ctx* c, rsd_step_out* out) {
    if (!c) return RSD_EINVAL;
    if (!c->have_prompts) return fail(c, RSD_ESTATE, "no prompts set");
    if (c->p.bon_n > 0) return fail(c, RSD_ESTATE, "this context runs Best-of-N: use rsd_bon_step");
    const int B = c->B;
    const rsd_params& P = c->p;
    const int merge = P.merge_prm;
    if (P.temperature > 0.f && (!c->u_draft || !c->u_target)) return fail(c, RSD_ESTATE, "sampling needs uniforms");
    if (P.omega_kind != RSD_OMEGA_BINARY && !c->u_gate) return fail(c, RSD_ESTATE, "this omega needs u_gate");
    if (P.sd_k > 0 && P.temperature > 0.f && (!c->u_prop || !c->u_acc))
        return fail(c, RSD_ESTATE, "sampled speculative regeneration needs the proposal and acceptance uniforms");
    int n_in = 0;
    for (int b = 0; b < B; ++b) n_in += c->finished()[b] == RSD_RUNNING;
    if (!n_in) return fail(c, RSD_ESTATE, "every sequence has finished");

    // ---- set-up: mark the sequences taking part, reserve pages for draft and reward model
    std::vector<int> kv_save(c->kv_len(0), c->kv_len(0) + 3 * B);
    auto trim_all = [&]() {
        for (int i = 0; i < 3; ++i)
            for (int b = 0; b < B; ++b) trim_pages(c->m[i], b, ceil_div(c->kv_len(i)[b], RSD_PAGE));
    };
    for (int b = 0; b < B; ++b) {
        const int in = c->finished()[b] == RSD_RUNNING;
        c->in_step()[b] = in;
        c->active()[b] = in;
        c->step_len()[b] = 0;
        c->ctx_pre()[b] = c->ctx_len()[b];
        c->accepted()[b] = 0;
        c->own_accept()[b] = 0;
        c->reward()[b] = 0.f;
        c->sd_live()[b] = c->sd_nprop()[b] = c->sd_nkept()[b] = c->sd_nround()[b] = 0;
    }
    *c->n_active() = n_in;
    for (int b = 0; b < B; ++b)
        if (c->in_step()[b]) {
            const int need = ceil_div(std::min(c->ctx_pre()[b] + P.step_cap, P.max_ctx), RSD_PAGE);
            // the model that scores the step needs room for it too: the reward model, or the target it is merged with
            const int scorer = merge == RSD_MERGE_NONE ? RSD_PRM : merge == RSD_MERGE_TARGET ? RSD_TARGET : RSD_DRAFT;
            if (!ensure_pages(c->m[RSD_DRAFT], b, need) || !ensure_pages(c->m[scorer], b, need)) {
                trim_all();
                return fail(c, RSD_ENOMEM, "KV pool exhausted reserving the draft step of sequence %d", b);
            }
        }
    int rc;
    if ((rc = push_state(c))) return rc;
    if ((rc = upload_tables(c, c->m[RSD_DRAFT]))) return rc;
    if ((rc = upload_tables(c, c->m[RSD_PRM]))) return rc;
    if (merge == RSD_MERGE_TARGET && (rc = upload_tables(c, c->m[RSD_TARGET]))) return rc;

    // ---- draft step  (Algorithm 1: "Generate draft step")
    double t0 = now_ms();
    if ((rc = gen_stage_any(c, RSD_DRAFT, c->u_draft, c->forced_draft))) return rc;
    if ((rc = fetch_step_tokens(c))) return rc;
    if ((rc = pull_state(c))) return rc;
    double t1 = now_ms();
    c->stage_ms[0] += t1 - t0;
    if (out) {
        for (int b = 0; b < B; ++b) {
            const int n = c->in_step()[b] ? c->ctx_len()[b] - c->ctx_pre()[b] : 0;
            if (out->draft_len) out->draft_len[b] = n;
            if (out->draft_tokens)
                std::memcpy(out->draft_tokens + (size_t)b * P.step_cap, c->steptok_h + (size_t)b * P.step_cap, P.step_cap * sizeof(int));
        }
    }
    std::vector<int> last_tok(B, -1);
    for (int b = 0; b < B; ++b)
        if (c->in_step()[b]) last_tok[b] = c->steptok_h[(size_t)b * P.step_cap + (c->ctx_len()[b] - c->ctx_pre()[b] - 1)];

    // ---- reward of the draft step  ("Compute reward")
    {
        // Without merge the reward model reads what it has not seen, [kv_p, ctx).  Merged with the draft:
        // the draft reads the one token it has not been fed, [ctx - 1, ctx), and its kv_len stays ctx - 1
        // (the next step feeds that token again and rewrites the same cache entry).  Merged with the
        // target: the target reads [kv_t, ctx) and then stands at ctx - 1 for the same reason.
        const int scorer = merge == RSD_MERGE_NONE ? RSD_PRM : merge == RSD_MERGE_TARGET ? RSD_TARGET : RSD_DRAFT;
        std::vector<Piece> pieces;
        for (int b = 0; b < B; ++b)
            if (c->in_step()[b]) {
                pieces.push_back(Piece{b, c->kv_len(scorer)[b], c->ctx_len()[b]});
                if (merge == RSD_MERGE_NONE) c->kv_len(RSD_PRM)[b] = c->ctx_len()[b];
                else if (merge == RSD_MERGE_TARGET) c->kv_len(RSD_TARGET)[b] = c->ctx_len()[b] - 1;
            }
        if ((rc = push_state(c))) return rc;
        Model& pm = c->m[RSD_PRM];
        const Model* trunk = merge == RSD_MERGE_NONE ? nullptr : &c->m[scorer];
        auto after = [&](const std::vector<Piece>&, const std::vector<int>&, int) {
            if (pm.s.dtype == RSD_F32) reward_rows<float>(c, pm, c->h, B, c->last_row_dev, c->ds.reward, trunk);
            else reward_rows<bf16_t>(c, pm, c->h, B, c->last_row_dev, c->ds.reward, trunk);
            return RSD_OK;
        };
        rc = pm.s.dtype == RSD_F32 ? prefill<float>(c, scorer, pieces, after) : prefill<bf16_t>(c, scorer, pieces, after);
        if (rc) return rc;
    }
    HIPCHK(c, hipStreamSynchronize(c->st));
    double t2 = now_ms();
    c->stage_ms[1] += t2 - t1;

    // ---- acceptance criterion and rollback  (Algorithm 2)
    hipLaunchKernelGGL(gate_kernel, dim3(ceil_div(B, 64)), dim3(64), 0, c->st, c->ds, B, P.delta, P.omega_kind, P.omega_a,
                       c->u_gate, P.max_steps, c->steps_done, c->forced_accept, c->in_step_dev, merge);
    if ((rc = pull_state(c))) return rc;
    double t3 = now_ms();
    c->stage_ms[2] += t3 - t2;
    if (out) {
        for (int b = 0; b < B; ++b) {
            if (out->reward) out->reward[b] = c->reward()[b];
            if (out->accepted) out->accepted[b] = c->accepted()[b];
            if (out->own_accept) out->own_accept[b] = c->own_accept()[b];
        }
    }

    // ---- target step for the rejected sequences  ("Generate a target step")
    int n_rej = 0;
    for (int b = 0; b < B; ++b) n_rej += c->in_step()[b] && !c->accepted()[b];
    if (n_rej) {
        bool ok = true;
        for (int b = 0; b < B && ok; ++b)
            if (c->in_step()[b] && !c->accepted()[b]) {
                const int need = ceil_div(std::min(c->ctx_pre()[b] + P.step_cap, P.max_ctx), RSD_PAGE);
                ok = ensure_pages(c->m[RSD_TARGET], b, need);
            }
        if (!ok) {
            // undo the whole step: every sequence back to its pre-step context
            for (int b = 0; b < B; ++b) {
                if (c->in_step()[b]) c->ctx_len()[b] = c->ctx_pre()[b];
                c->active()[b] = 0;
            }
            std::copy(kv_save.begin(), kv_save.end(), c->kv_len(0));
            trim_all();
            if ((rc = push_state(c))) return rc;
            HIPCHK(c, hipStreamSynchronize(c->st));
            return fail(c, RSD_ENOMEM, "KV pool exhausted reserving the target step");
        }
        for (int b = 0; b < B; ++b) c->step_len()[b] = 0;
        *c->n_active() = n_rej;
        if ((rc = push_state(c))) return rc;
        if ((rc = upload_tables(c, c->m[RSD_TARGET]))) return rc;
        if (P.sd_k > 0) rc = c->m[RSD_TARGET].s.dtype == RSD_F32 ? sd_stage<float>(c) : sd_stage<bf16_t>(c);
        else rc = gen_stage_any(c, RSD_TARGET, c->u_target, c->forced_target);
        if (rc) return rc;
        if ((rc = fetch_step_tokens(c))) return rc;
        if ((rc = pull_state(c))) return rc;
        for (int b = 0; b < B; ++b)
            if (c->in_step()[b] && !c->accepted()[b])
                last_tok[b] = c->steptok_h[(size_t)b * P.step_cap + (c->ctx_len()[b] - c->ctx_pre()[b] - 1)];
    }
    double t4 = now_ms();
    c->stage_ms[3] += t4 - t3;

    // ---- termination test and record
    c->steps_done += 1;
    for (int b = 0; b < B && out; ++b) {
        if (out->sd_rounds) out->sd_rounds[b] = c->sd_nround()[b];
        if (out->sd_proposed) out->sd_proposed[b] = c->sd_nprop()[b];
        if (out->sd_kept) out->sd_kept[b] = c->sd_nkept()[b];
    }
    for (int b = 0; b < B; ++b) {
        if (!c->in_step()[b]) {
            if (out && out->final_len) out->final_len[b] = 0;
            if (out && out->finished) out->finished[b] = c->finished()[b];
            if (out && out->final_tokens) std::fill(out->final_tokens + (size_t)b * P.step_cap, out->final_tokens + (size_t)(b + 1) * P.step_cap, -1);
            continue;
        }
        const int n = c->ctx_len()[b] - c->ctx_pre()[b];
        if (P.eos_id >= 0 && last_tok[b] == P.eos_id) c->finished()[b] = RSD_FIN_EOS;
        else if (c->ctx_len()[b] >= P.max_ctx) c->finished()[b] = RSD_FIN_MAX_CTX;
        else if (c->steps_done >= P.max_steps) c->finished()[b] = RSD_FIN_MAX_STEPS;
        if (out) {
            if (out->final_len) out->final_len[b] = n;
            if (out->finished) out->finished[b] = c->finished()[b];
            if (out->final_tokens) {
                // accepted: the draft step is the committed one and steptok still holds it
                std::memcpy(out->final_tokens + (size_t)b * P.step_cap, c->steptok_h + (size_t)b * P.step_cap, P.step_cap * sizeof(int));
            }
        }
    }
    trim_all();
    return RSD_OK;
}

int rsd_generate(rsd_ctx* c, int32_t max_steps, rsd_gen_out* out) {
    if (!c) return RSD_EINVAL;
    if (!c->have_prompts) return fail(c, RSD_ESTATE, "no prompts set");
    const int B = c->B;
    const int limit = max_steps > 0 ? std::min(max_steps, c->p.max_steps) : c->p.max_steps;
    std::vector<int> dl(B), fl(B), acc(B), sr(B), sp(B), sk(B);
    rsd_step_out so{};
    so.draft_len = dl.data(); so.final_len = fl.data(); so.accepted = acc.data();
    so.sd_rounds = sr.data(); so.sd_proposed = sp.data(); so.sd_kept = sk.data();
    rsd_gen_out g{};
    if (out) { g.tokens = out->tokens; g.ctx_len = out->ctx_len; g.finished = out->finished; }
    while (c->steps_done < limit) {
        bool any = false;
        for (int b = 0; b < B; ++b) any |= c->finished()[b] == RSD_RUNNING;
        if (!any) break;
        std::vector<int> was(B);
        for (int b = 0; b < B; ++b) was[b] = c->finished()[b] == RSD_RUNNING;
        int rc = rsd_step(c, &so);
        if (rc) { if (out) *out = g; return rc; }
        g.steps_run += 1;
        for (int b = 0; b < B; ++b)
            if (was[b]) {
                g.n_draft += dl[b];
                if (acc[b]) g.n_accept += 1; else { g.n_reject += 1; g.n_target += fl[b]; }
                g.n_sd_rounds += sr[b]; g.n_sd_proposed += sp[b]; g.n_sd_kept += sk[b];
            }
    }
    for (int b = 0; b < B; ++b) g.n_committed += c->ctx_len()[b] - c->prompt_len[b];
    if (g.ctx_len) std::memcpy(g.ctx_len, c->ctx_len(), B * sizeof(int));
    if (g.finished) std::memcpy(g.finished, c->finished(), B * sizeof(int));
    if (g.tokens) {
        HIPCHK(c, hipMemcpyAsync(g.tokens, c->ds.tokens, (size_t)B * c->p.max_ctx * sizeof(int), hipMemcpyDeviceToHost, c->st));
        HIPCHK(c, hipStreamSynchronize(c->st));
        blank_tails(g.tokens, B, c->p.max_ctx, c->ctx_len());
    }
    if (out) *out = g;
    return RSD_OK;
}

int rsd_bon_step(rsd_ctx* c, rsd_bon_out* out) {
    if (!c) return RSD_EINVAL;
    if (c->p.bon_n <= 0) return fail(c, RSD_ESTATE, "this context was not created for Best-of-N (bon_n = 0)");
    if (!c->have_prompts) return fail(c, RSD_ESTATE, "no prompts set");
    const int B = c->B, N = c->p.bon_n, S = c->n_seq;
    const rsd_params& P = c->p;
    if (P.temperature > 0.f && !c->u_draft) return fail(c, RSD_ESTATE, "sampling needs uniforms");
    int n_in = 0;
    for (int s = 0; s < S; ++s) n_in += c->finished()[c->canon[s]] == RSD_RUNNING;
    if (!n_in) return fail(c, RSD_ESTATE, "every sequence has finished");
    Model &md = c->m[RSD_DRAFT], &mp = c->m[RSD_PRM];
    const bool f32 = md.s.dtype == RSD_F32;
    int rc;
    double t0 = now_ms();

    // ---- the committed lane of every running sequence catches up: the base model holds all tokens but the
    // newest, the reward model all of them (only the prompt of the first step is ever missing)
    auto undo = [&]() {      // pool exhausted: candidates give their pages back, committed lanes keep what they hold tokens for
        for (int s = 0; s < S; ++s)
            for (int n = 0; n < N; ++n) {
                const int L = s * N + n;
                const bool keep = L == c->canon[s];
                trim_pages(md, L, keep ? ceil_div(c->kv_len(RSD_DRAFT)[L], RSD_PAGE) : 0);
                trim_pages(mp, L, keep ? ceil_div(c->kv_len(RSD_PRM)[L], RSD_PAGE) : 0);
            }
    };
    {
        std::vector<Piece> pd, pp;
        for (int s = 0; s < S; ++s) {
            const int L = c->canon[s];
            if (c->finished()[L] != RSD_RUNNING) continue;
            const int ctx = c->ctx_len()[L];
            if (!ensure_pages(md, L, ceil_div(ctx - 1, RSD_PAGE)) || !ensure_pages(mp, L, ceil_div(ctx, RSD_PAGE))) {
                undo();
                return fail(c, RSD_ENOMEM, "KV pool exhausted reading the context of sequence %d", s);
            }
            if (c->kv_len(RSD_DRAFT)[L] < ctx - 1) pd.push_back(Piece{L, c->kv_len(RSD_DRAFT)[L], ctx - 1});
            if (c->kv_len(RSD_PRM)[L] < ctx) pp.push_back(Piece{L, c->kv_len(RSD_PRM)[L], ctx});
        }
        auto nothing = [](const std::vector<Piece>&, const std::vector<int>&, int) { return RSD_OK; };
        if (!pd.empty() || !pp.empty()) {
            if ((rc = upload_tables(c, md))) return rc;
            if ((rc = upload_tables(c, mp))) return rc;
        }
        if (!pd.empty()) {
            rc = f32 ? prefill<float>(c, RSD_DRAFT, pd, nothing) : prefill<bf16_t>(c, RSD_DRAFT, pd, nothing);
            if (rc) return rc;
            for (const Piece& pc : pd) c->kv_len(RSD_DRAFT)[pc.b] = pc.end;
        }
        if (!pp.empty()) {
            rc = f32 ? prefill<float>(c, RSD_PRM, pp, nothing) : prefill<bf16_t>(c, RSD_PRM, pp, nothing);
            if (rc) return rc;
            for (const Piece& pc : pp) c->kv_len(RSD_PRM)[pc.b] = pc.end;
        }
    }

    // ---- fork: every candidate lane names the committed pages that are full, gets a copy of the page the
    // step's first entries go into (if the committed context ends inside one), and reserves pages of its own
    // for the step
    int n_copy[2] = {0, 0};
    for (int s = 0; s < S; ++s) {
        const int L0 = c->canon[s];
        const bool run = c->finished()[L0] == RSD_RUNNING;
        for (int n = 0; n < N; ++n) {
            const int L = s * N + n;
            c->bon_src_h[L] = -1;
            c->bon_src_h[B + L] = 0;
            c->in_step()[L] = run;
            if (!run) { c->active()[L] = 0; continue; }
            const int ctx = c->ctx_len()[L0];
            const int need = ceil_div(std::min(ctx + P.step_cap, P.max_ctx), RSD_PAGE);
            bool ok = true;
            if (L != L0) {
                Model* ms[2] = {&md, &mp};
                const int held[2] = {ctx - 1, ctx};           // tokens the base / the reward model hold entries for
                for (int k = 0; k < 2 && ok; ++k) {
                    Model& m = *ms[k];
                    trim_pages(m, L, 0);
                    const int full = held[k] / RSD_PAGE;
                    const int* src = m.bt_host + (size_t)L0 * m.max_pages;
                    for (int i = 0; i < full; ++i) share_page(m, L, src[i]);
                    c->bon_shared += full;
                    if (held[k] % RSD_PAGE) {
                        ok = ensure_pages(m, L, full + 1);
                        if (ok) {
                            int* pr = c->bon_copy_h + (size_t)k * 2 * B + 2 * n_copy[k]++;
                            pr[0] = src[full];
                            pr[1] = m.bt_host[(size_t)L * m.max_pages + full];
                            ++c->bon_copied;
                            ++c->bon_alloc;
                        }
                    }
                }
                c->bon_src_h[L] = L0;
                c->bon_src_h[B + L] = ctx;
            }
            const int had_d = md.n_pages[L], had_p = mp.n_pages[L];
            ok = ok && ensure_pages(md, L, need) && ensure_pages(mp, L, need);
            if (!ok) {
                undo();
                return fail(c, RSD_ENOMEM, "KV pool exhausted reserving candidate %d of sequence %d", n, s);
            }
            c->bon_alloc += (md.n_pages[L] - had_d) + (mp.n_pages[L] - had_p);
        }
    }
    for (int s = 0; s < S; ++s) {
        const int L0 = c->canon[s];
        if (c->finished()[L0] != RSD_RUNNING) continue;
        const int ctx = c->ctx_len()[L0];
        for (int n = 0; n < N; ++n) {
            const int L = s * N + n;
            c->ctx_len()[L] = ctx;
            c->ctx_pre()[L] = ctx;
            c->kv_len(RSD_DRAFT)[L] = ctx - 1;
            c->kv_len(RSD_PRM)[L] = ctx;
            c->active()[L] = 1;
            c->step_len()[L] = 0;
            c->finished()[L] = RSD_RUNNING;
            c->reward()[L] = 0.f;
        }
    }
    *c->n_active() = n_in * N;
    if ((rc = push_state(c))) return rc;
    if ((rc = upload_tables(c, md))) return rc;
    if ((rc = upload_tables(c, mp))) return rc;
    HIPCHK(c, hipMemcpyAsync(c->bon_src_dev, c->bon_src_h, (size_t)2 * B * sizeof(int), hipMemcpyHostToDevice, c->st));
    hipLaunchKernelGGL(bon_fork_tokens_kernel, dim3(B), dim3(256), 0, c->st, c->ds.tokens, P.max_ctx, c->bon_src_dev,
                       c->bon_src_dev + B);
    if (n_copy[0] + n_copy[1]) {
        HIPCHK(c, hipMemcpyAsync(c->bon_copy_dev, c->bon_copy_h, (size_t)4 * B * sizeof(int), hipMemcpyHostToDevice, c->st));
        Model* ms[2] = {&md, &mp};
        for (int k = 0; k < 2; ++k)
            if (n_copy[k]) {
                Model& m = *ms[k];
                const size_t page_bytes = m.page_elts * m.esz;
                hipLaunchKernelGGL(bon_copy_pages_kernel, dim3(n_copy[k], m.s.n_layers), dim3(256), 0, c->st, m.pool,
                                   (size_t)m.pool_pages * page_bytes, page_bytes, c->bon_copy_dev + (size_t)k * 2 * B);
            }
    }
    double t1 = now_ms();
    c->stage_ms[2] += t1 - t0;

    // ---- every candidate's step with the base model
    if ((rc = gen_stage_any(c, RSD_DRAFT, c->u_draft, c->forced_draft))) return rc;
    if ((rc = fetch_step_tokens(c))) return rc;
    if ((rc = pull_state(c))) return rc;
    double t2 = now_ms();
    c->stage_ms[0] += t2 - t1;

    // ---- every candidate's reward
    {
        std::vector<Piece> pieces;
        for (int L = 0; L < B; ++L)
            if (c->in_step()[L]) {
                pieces.push_back(Piece{L, c->kv_len(RSD_PRM)[L], c->ctx_len()[L]});
                c->kv_len(RSD_PRM)[L] = c->ctx_len()[L];
            }
        if ((rc = push_state(c))) return rc;
        auto after = [&](const std::vector<Piece>&, const std::vector<int>&, int) {
            if (f32) reward_rows<float>(c, mp, c->h, B, c->last_row_dev, c->ds.reward);
            else reward_rows<bf16_t>(c, mp, c->h, B, c->last_row_dev, c->ds.reward);
            return RSD_OK;
        };
        rc = f32 ? prefill<float>(c, RSD_PRM, pieces, after) : prefill<bf16_t>(c, RSD_PRM, pieces, after);
        if (rc) return rc;
    }
    if ((rc = pull_state(c))) return rc;
    double t3 = now_ms();
    c->stage_ms[1] += t3 - t2;

    // ---- the choice, the release of the other candidates, the termination test
    std::vector<int> forced_choice;
    if (c->forced_accept) {
        forced_choice.resize(S);
        HIPCHK(c, hipMemcpy2DAsync(forced_choice.data(), sizeof(int), c->forced_accept + c->steps_done, (size_t)P.max_steps * sizeof(int),
                                   sizeof(int), S, hipMemcpyDeviceToHost, c->st));
        HIPCHK(c, hipStreamSynchronize(c->st));
    }
    c->steps_done += 1;
    for (int s = 0; s < S; ++s) {
        const int L0 = c->canon[s];
        const bool run = c->in_step()[L0] != 0;
        if (out) {
            for (int n = 0; n < N; ++n) {
                const int L = s * N + n;
                const int len = run ? c->ctx_len()[L] - c->ctx_pre()[L] : 0;
                if (out->cand_len) out->cand_len[L] = len;
                if (out->cand_reward) out->cand_reward[L] = run ? c->reward()[L] : 0.f;
                if (out->cand_tokens) {
                    int* dst = out->cand_tokens + (size_t)L * P.step_cap;
                    if (run) std::memcpy(dst, c->steptok_h + (size_t)L * P.step_cap, P.step_cap * sizeof(int));
                    else std::fill(dst, dst + P.step_cap, -1);
                }
            }
        }
        if (!run) {
            if (out) {
                if (out->chosen) out->chosen[s] = -1;
                if (out->own_choice) out->own_choice[s] = -1;
                if (out->finished) out->finished[s] = c->finished()[L0];
                if (out->ctx_len) out->ctx_len[s] = c->ctx_len()[L0];
                if (out->kv_len) { out->kv_len[s] = c->kv_len(RSD_DRAFT)[L0]; out->kv_len[S + s] = c->kv_len(RSD_PRM)[L0]; }
                if (out->n_pages) { out->n_pages[s] = md.n_pages[L0]; out->n_pages[S + s] = mp.n_pages[L0]; }
            }
            continue;
        }
        int best = 0;
        for (int n = 1; n < N; ++n)
            if (c->reward()[s * N + n] > c->reward()[s * N + best]) best = n;      // the first of equal maxima stays
        int pick = best;
        if (!forced_choice.empty() && forced_choice[s] >= 0 && forced_choice[s] < N) pick = forced_choice[s];
        const int Lw = s * N + pick;
        c->canon[s] = Lw;
        for (int n = 0; n < N; ++n) {
            const int L = s * N + n;
            if (L == Lw) continue;
            trim_pages(md, L, 0);
            trim_pages(mp, L, 0);
        }
        trim_pages(md, Lw, ceil_div(c->kv_len(RSD_DRAFT)[Lw], RSD_PAGE));
        trim_pages(mp, Lw, ceil_div(c->kv_len(RSD_PRM)[Lw], RSD_PAGE));
        const int len = c->ctx_len()[Lw] - c->ctx_pre()[Lw];
        const int last_tok = c->steptok_h[(size_t)Lw * P.step_cap + len - 1];
        int fin = RSD_RUNNING;
        if (P.eos_id >= 0 && last_tok == P.eos_id) fin = RSD_FIN_EOS;
        else if (c->ctx_len()[Lw] >= P.max_ctx) fin = RSD_FIN_MAX_CTX;
        else if (c->steps_done >= P.max_steps) fin = RSD_FIN_MAX_STEPS;
        for (int n = 0; n < N; ++n) c->finished()[s * N + n] = fin;
        if (out) {
            if (out->chosen) out->chosen[s] = pick;
            if (out->own_choice) out->own_choice[s] = best;
            if (out->finished) out->finished[s] = fin;
            if (out->ctx_len) out->ctx_len[s] = c->ctx_len()[Lw];
            if (out->kv_len) { out->kv_len[s] = c->kv_len(RSD_DRAFT)[Lw]; out->kv_len[S + s] = c->kv_len(RSD_PRM)[Lw]; }
            if (out->n_pages) { out->n_pages[s] = md.n_pages[Lw]; out->n_pages[S + s] = mp.n_pages[Lw]; }
        }
    }
    c->stage_ms[2] += now_ms() - t3;
    return RSD_OK;
}

int rsd_bon_generate(rsd_ctx* c, int32_t max_steps, rsd_gen_out* out) {
    if (!c) return RSD_EINVAL;
    if (c->p.bon_n <= 0) return fail(c, RSD_ESTATE, "this context was not created for Best-of-N (bon_n = 0)");
    if (!c->have_prompts) return fail(c, RSD_ESTATE, "no prompts set");
    const int S = c->n_seq, N = c->p.bon_n;
    const int limit = max_steps > 0 ? std::min(max_steps, c->p.max_steps) : c->p.max_steps;
    std::vector<int> cl((size_t)S * N);
    rsd_bon_out bo{};
    bo.cand_len = cl.data();
    rsd_gen_out g{};
    if (out) { g.tokens = out->tokens; g.ctx_len = out->ctx_len; g.finished = out->finished; }
    while (c->steps_done < limit) {
        bool any = false;
        for (int s = 0; s < S; ++s) any |= c->finished()[c->canon[s]] == RSD_RUNNING;
        if (!any) break;
        int rc = rsd_bon_step(c, &bo);
        if (rc) { if (out) *out = g; return rc; }
        g.steps_run += 1;
        for (int v : cl) g.n_draft += v;
    }
    for (int s = 0; s < S; ++s) {
        const int L = c->canon[s];
        g.n_committed += c->ctx_len()[L] - c->prompt_len[L];
        if (g.ctx_len) g.ctx_len[s] = c->ctx_len()[L];
        if (g.finished) g.finished[s] = c->finished()[L];
        if (g.tokens)
            HIPCHK(c, hipMemcpyAsync(g.tokens + (size_t)s * c->p.max_ctx, c->ds.tokens + (size_t)L * c->p.max_ctx,
                                     (size_t)c->p.max_ctx * sizeof(int), hipMemcpyDeviceToHost, c->st));
    }
    HIPCHK(c, hipStreamSynchronize(c->st));
    if (g.tokens) {
        std::vector<int> len(S);
        for (int s = 0; s < S; ++s) len[s] = c->ctx_len()[c->canon[s]];
        blank_tails(g.tokens, S, c->p.max_ctx, len.data());
    }
    if (out) *out = g;
    return RSD_OK;
}

int rsd_bon_stats(rsd_ctx* c, int64_t* pages_shared, int64_t* pages_copied, int64_t* pages_allocated) {
    if (!c) return RSD_EINVAL;
    if (pages_shared) *pages_shared = c->bon_shared;
    if (pages_copied) *pages_copied = c->bon_copied;
    if (pages_allocated) *pages_allocated = c->bon_alloc;
    return RSD_OK;
}

int rsd_export_state(rsd_ctx* c, int32_t* ctx_len, int32_t* kv_len, int32_t* n_pages, int32_t* tokens) {
    if (!c) return RSD_EINVAL;
    const int B = c->B;
    if (ctx_len) std::memcpy(ctx_len, c->ctx_len(), B * sizeof(int));
    if (kv_len) std::memcpy(kv_len, c->kv_len(0), 3 * B * sizeof(int));
    if (n_pages)
        for (int i = 0; i < 3; ++i)
            for (int b = 0; b < B; ++b) n_pages[i * B + b] = c->m[i].n_pages[b];
    if (tokens) {
        HIPCHK(c, hipMemcpyAsync(tokens, c->ds.tokens, (size_t)B * c->p.max_ctx * sizeof(int), hipMemcpyDeviceToHost, c->st));
        HIPCHK(c, hipStreamSynchronize(c->st));
        blank_tails(tokens, B, c->p.max_ctx, c->ctx_len());
    }
    return RSD_OK;
}

int rsd_export_pages(rsd_ctx* c, int32_t model, int32_t* block_table, int32_t* max_pages, int32_t* pool_pages,
                     int32_t* free_pages) {
    if (!c || model < 0 || model > 2) return fail(c, RSD_EINVAL, "bad model index");
    Model& m = c->m[model];
    if (block_table && m.bt_host) std::memcpy(block_table, m.bt_host, (size_t)c->B * m.max_pages * sizeof(int));
    if (max_pages) *max_pages = m.max_pages;
    if (pool_pages) *pool_pages = m.pool_pages;
    if (free_pages) *free_pages = (int)m.free_list.size();
    return RSD_OK;
}

int rsd_export_sampled(rsd_ctx* c, int32_t* sampled_draft, int32_t* sampled_target) {
    if (!c) return RSD_EINVAL;
    const size_t n = (size_t)c->B * c->p.max_steps * c->p.step_cap * sizeof(int);
    if (sampled_draft) HIPCHK(c, hipMemcpyAsync(sampled_draft, c->ds.sampled[0], n, hipMemcpyDeviceToHost, c->st));
    if (sampled_target) HIPCHK(c, hipMemcpyAsync(sampled_target, c->ds.sampled[1], n, hipMemcpyDeviceToHost, c->st));
    HIPCHK(c, hipStreamSynchronize(c->st));
    return RSD_OK;
}

int rsd_set_teacher_sd(rsd_ctx* c, const int32_t* forced_proposal_dev) {
    if (!c) return RSD_EINVAL;
    c->forced_prop = forced_proposal_dev;
    return drop_stale_graphs(c);
}

int rsd_export_proposed(rsd_ctx* c, int32_t* proposed, int32_t* kept_flags) {
    if (!c) return RSD_EINVAL;
    if (c->p.sd_k <= 0) return fail(c, RSD_ESTATE, "no speculative regeneration in this context");
    const size_t n = (size_t)c->B * c->p.max_steps * c->p.step_cap * c->p.sd_k * sizeof(int);
    if (proposed) HIPCHK(c, hipMemcpyAsync(proposed, c->ds.sampled[2], n, hipMemcpyDeviceToHost, c->st));
    if (kept_flags) HIPCHK(c, hipMemcpyAsync(kept_flags, c->sd_acc_rec, n, hipMemcpyDeviceToHost, c->st));
    HIPCHK(c, hipStreamSynchronize(c->st));
    return RSD_OK;
}

int rsd_set_uniforms_sd(rsd_ctx* c, const float* u_proposal_dev, const float* u_accept_dev) {
    if (!c) return RSD_EINVAL;
    c->u_prop = u_proposal_dev; c->u_acc = u_accept_dev;
    return drop_stale_graphs(c);
}

int rsd_sd_verify(rsd_ctx* c, const float* p_logits_dev, const float* q_logits_dev, const int32_t* proposals_dev,
                  const int32_t* n_proposals_host, const float* u_accept_dev, const float* u_new_dev, int32_t n,
                  int32_t* emitted_dev, int32_t* kept_dev) {
    if (!c || !p_logits_dev || !q_logits_dev || !proposals_dev || !n_proposals_host || !u_accept_dev || !u_new_dev ||
        !emitted_dev || !kept_dev)
        return fail(c, RSD_EINVAL, "null argument");
    const int k = c->p.sd_k;
    if (k <= 0 || c->p.temperature <= 0.f) return fail(c, RSD_ESTATE, "needs a context with sd_k > 0 and temperature > 0");
    if (n < 1 || n > c->B) return fail(c, RSD_EINVAL, "n outside [1, batch]");
    for (int s = 0; s < n; ++s)
        if (n_proposals_host[s] < 0 || n_proposals_host[s] > k) return fail(c, RSD_EINVAL, "n_proposals[%d] outside [0, sd_k]", s);
    HIPCHK(c, hipStreamSynchronize(c->st));
    // index arrays: zeros [n], proposals per sequence [n], first target row [n]; uniform index per row; draft rows in use
    int *zeros = c->sd_rows_h, *cnt = zeros + n, *row0 = cnt + n;
    const int rows = c->B * (k + 1), qrows = c->B * k;
    int *pu = c->sd_aux_h, *qu = pu + rows, *qa = qu + qrows;
    std::fill(qa, qa + qrows, 0);
    for (int s = 0; s < n; ++s) {
        zeros[s] = 0; cnt[s] = n_proposals_host[s]; row0[s] = s * (k + 1);
        for (int i = 0; i <= k; ++i) pu[s * (k + 1) + i] = s * (k + 1) + i;
        for (int i = 0; i < cnt[s]; ++i) { qu[s * k + i] = s * (k + 1) + i; qa[s * k + i] = 1; }
    }
    HIPCHK(c, hipMemcpyAsync(c->sd_rows_dev, c->sd_rows_h, (size_t)3 * n * sizeof(int), hipMemcpyHostToDevice, c->st));
    HIPCHK(c, hipMemcpyAsync(c->sd_aux_dev, c->sd_aux_h, (size_t)(rows + 2 * qrows) * sizeof(int), hipMemcpyHostToDevice, c->st));
    const int *zeros_d = c->sd_rows_dev, *cnt_d = zeros_d + n, *row0_d = cnt_d + n;
    int rc = sd_sampled_verify(c, p_logits_dev, n * (k + 1), q_logits_dev, c->sd_aux_dev, c->sd_aux_dev + rows,
                               c->sd_aux_dev + rows + qrows, u_new_dev, emitted_dev, n, nullptr, zeros_d, cnt_d, row0_d,
                               proposals_dev, k, zeros_d, u_accept_dev, k + 1, zeros_d, kept_dev);
    if (rc) return rc;
    sd_sampled_replace(c, n, kept_dev);
    HIPCHK(c, hipStreamSynchronize(c->st));
    HIPCHK(c, hipGetLastError());
    return RSD_OK;
}

int rsd_stage_ms(rsd_ctx* c, double ms[4], int32_t reset) {
    if (!c || !ms) return RSD_EINVAL;
    for (int i = 0; i < 4; ++i) { ms[i] = c->stage_ms[i]; if (reset) c->stage_ms[i] = 0; }
    return RSD_OK;
}

int rsd_decode_stats(rsd_ctx* c, int64_t* eager_iters, int64_t* graph_replays, int64_t* graphs_recorded) {
    if (!c) return RSD_EINVAL;
    if (eager_iters) *eager_iters = c->n_eager_iters;
    if (graph_replays) *graph_replays = c->n_graph_replays;
    if (graphs_recorded) *graphs_recorded = (int64_t)c->graphs.size();
    return RSD_OK;
}

int rsd_probe_start(rsd_ctx* c, int32_t slot, int32_t model, int32_t phase, int32_t op, int32_t max_samples,
                    int32_t stride) {
    if (!c) return RSD_EINVAL;
    if (slot < 0 || slot >= RSD_PROBE_SLOTS || model < 0 || model > 2 || op < 0 || op > 4 || max_samples < 0 ||
        max_samples > (1 << 20) || stride < 1 || (phase != RSD_PROBE_DECODE && phase != RSD_PROBE_PREFILL))
        return fail(c, RSD_EINVAL, "bad probe argument");
    HIPCHK(c, hipStreamSynchronize(c->st));
    rsd_ctx::Probe& q = c->probe[slot];
    while (q.ev.size() < 2 * (size_t)max_samples) {
        hipEvent_t e;
        HIPCHK(c, hipEventCreate(&e));
        q.ev.push_back(e);
    }
    q.model = model; q.phase = phase; q.op = op; q.stride = stride;
    q.seen = 0; q.iters = 0; q.used = 0; q.bytes = 0; q.flops = 0; q.iter_on = false;
    HIPCHK(c, hipMemsetAsync(c->clk_dev + 3 * slot, 0, 3 * sizeof(unsigned long long), c->st));   // ordered before the probed launches
    return RSD_OK;
}

int rsd_probe_clock(rsd_ctx* c, int32_t slot, int64_t* launches, int64_t* shader_ticks, int64_t* ref_ticks) {
    if (!c) return RSD_EINVAL;
    if (slot < 0 || slot >= RSD_PROBE_SLOTS) return fail(c, RSD_EINVAL, "bad probe slot");
    HIPCHK(c, hipStreamSynchronize(c->st));
    unsigned long long h[3] = {0, 0, 0};
    HIPCHK(c, hipMemcpyAsync(h, c->clk_dev + 3 * slot, sizeof(h), hipMemcpyDeviceToHost, c->st));
    HIPCHK(c, hipStreamSynchronize(c->st));
    if (shader_ticks) *shader_ticks = (int64_t)h[0];
    if (ref_ticks) *ref_ticks = (int64_t)h[1];
    if (launches) *launches = (int64_t)h[2];
    return RSD_OK;
}

int rsd_probe_read(rsd_ctx* c, int32_t slot, int64_t* n_samples, double* total_ms, int64_t* total_bytes,
                   int64_t* total_flops) {
    if (!c) return RSD_EINVAL;
    if (slot < 0 || slot >= RSD_PROBE_SLOTS) return fail(c, RSD_EINVAL, "bad probe slot");
    HIPCHK(c, hipStreamSynchronize(c->st));
    rsd_ctx::Probe& q = c->probe[slot];
    double tot = 0;
    for (size_t i = 0; i + 1 < q.used; i += 2) {
        float ms = 0.f;
        HIPCHK(c, hipEventElapsedTime(&ms, q.ev[i], q.ev[i + 1]));
        tot += ms;
    }
    if (n_samples) *n_samples = (int64_t)(q.used / 2);
    if (total_ms) *total_ms = tot;
    if (total_bytes) *total_bytes = q.bytes;
    if (total_flops) *total_flops = q.flops;
    q.model = -1;
    return RSD_OK;
}

int rsd_iter_stats(rsd_ctx* c, int32_t model, int64_t* iterations, double* gpu_ms, int64_t* seq_iterations,
                   int64_t* kv_tokens_read, int32_t reset) {
    if (!c) return RSD_EINVAL;
    if (model != RSD_DRAFT && model != RSD_TARGET) return fail(c, RSD_EINVAL, "decode loops exist for the draft and the target only");
    rsd_ctx::IterStats& is = c->it[model];
    if (iterations) *iterations = is.iters;
    if (gpu_ms) *gpu_ms = is.ms;
    if (seq_iterations) *seq_iterations = is.seq_iters;
    if (kv_tokens_read) *kv_tokens_read = is.kv_read;
    if (reset) { is.iters = is.seq_iters = is.kv_read = is.row_iters = 0; is.ms = 0; }
    return RSD_OK;
}

int rsd_iter_rows(rsd_ctx* c, int32_t model, int64_t* row_iterations) {
    if (!c || !row_iterations) return fail(c, RSD_EINVAL, "null argument");
    if (model != RSD_DRAFT && model != RSD_TARGET) return fail(c, RSD_EINVAL, "decode loops exist for the draft and the target only");
    *row_iterations = c->it[model].row_iters;
    return RSD_OK;
}

int rsd_debug_build(void) { return kDebugChecks ? 1 : 0; }

int rsd_check_rows(rsd_ctx* c, int32_t model, const int32_t* seq_host, const int32_t* pos_host, int32_t n) {
    if (!c || !seq_host || !pos_host) return fail(c, RSD_EINVAL, "null argument");
    if (model < 0 || model > 2 || n < 1 || n > kMaxRows) return fail(c, RSD_EINVAL, "bad model or row count");
    if (!c->m[model].bt_dev) return fail(c, RSD_EINVAL, "model %d has no cache", model);
    HIPCHK(c, hipStreamSynchronize(c->st));          // the staging arrays of the last pass are free
    std::copy(seq_host, seq_host + n, c->row_seq_h);
    std::copy(pos_host, pos_host + n, c->row_pos_h);
    HIPCHK(c, hipMemcpyAsync(c->row_seq_dev, c->row_seq_h, n * sizeof(int), hipMemcpyHostToDevice, c->st));
    HIPCHK(c, hipMemcpyAsync(c->row_pos_dev, c->row_pos_h, n * sizeof(int), hipMemcpyHostToDevice, c->st));
    return check_rows(c, model, RowMap{c->row_seq_dev, c->row_pos_dev, nullptr, nullptr}, n);
}

int rsd_probe_attention(rsd_ctx* c, int32_t model, const int32_t* ctx_len_host, int32_t reps, double* total_ms) {
    if (!c || !ctx_len_host || !total_ms) return fail(c, RSD_EINVAL, "null argument");
    if (model < 0 || model > 2 || reps < 1 || reps > (1 << 20)) return fail(c, RSD_EINVAL, "bad model or reps");
    if (model == RSD_PRM && c->p.merge_prm != RSD_MERGE_NONE) return fail(c, RSD_EINVAL, "the merged reward model has no cache");
    const int B = c->B;
    Model& m = c->m[model];
    for (int b = 0; b < B; ++b)
        if (ctx_len_host[b] < 1 || ctx_len_host[b] > c->p.max_ctx) return fail(c, RSD_EINVAL, "ctx_len[%d] outside [1, max_ctx]", b);
    HIPCHK(c, hipStreamSynchronize(c->st));
    reset_sequences(c);
    c->have_prompts = false;
    for (int b = 0; b < B; ++b) {
        if (!ensure_pages(m, b, ceil_div(ctx_len_host[b], RSD_PAGE))) {
            reset_sequences(c);
            return fail(c, RSD_ENOMEM, "KV pool too small for these contexts");
        }
        c->ctx_len()[b] = ctx_len_host[b];
        c->kv_len(model)[b] = ctx_len_host[b] - 1;       // the new token sits at the last position
        c->active()[b] = 1;
    }
    int rc;
    if ((rc = push_state(c))) return rc;
    if ((rc = upload_tables(c, m))) return rc;
    HIPCHK(c, hipMemsetAsync(m.pool, 0, (size_t)m.pool_pages * m.page_elts * m.esz * m.s.n_layers, c->st));
    HIPCHK(c, hipMemsetAsync(c->qkv, 0, (size_t)B * m.n_qkv * sizeof(float), c->st));
    hipEvent_t e0, e1;
    HIPCHK(c, hipEventCreate(&e0));
    HIPCHK(c, hipEventCreate(&e1));
    const bool halves = B >= 2 && m.s.dtype == RSD_BF16;
    // a single sequence leaves the merge of its context splits to the output projection, as run_layers does
    const bool merge_here = !(B == 1 && m.splits > 1 && (size_t)m.q_dim * sizeof(float) <= 40 * 1024);
    auto one = [&](int l) {
        if (m.s.dtype == RSD_BF16) launch_attn_decode_mfma(c, m, l, B, model, merge_here, halves);
        else if (m.hd == 128) launch_attn_decode<float, 128>(c, m, l, B, model);
        else launch_attn_decode<float, 32>(c, m, l, B, model);
    };
    for (int l = 0; l < std::min(2, m.s.n_layers); ++l) one(l);      // untimed: first-use costs
    HIPCHK(c, hipEventRecord(e0, c->st));
    for (int r = 0; r < reps; ++r) one(r % m.s.n_layers);
    HIPCHK(c, hipEventRecord(e1, c->st));
    HIPCHK(c, hipEventSynchronize(e1));
    float ms = 0.f;
    HIPCHK(c, hipEventElapsedTime(&ms, e0, e1));
    *total_ms = ms;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    HIPCHK(c, hipGetLastError());
    reset_sequences(c);
    return RSD_OK;
}

int rsd_sample(rsd_ctx* c, const float* logits_dev, const float* u_dev, int32_t n, int32_t vocab, float temperature,
               float top_p, int32_t* out_dev) {
    if (!c || !logits_dev || !out_dev || n < 1 || vocab < 1) return fail(c, RSD_EINVAL, "bad argument");
    if (temperature > 0.f && !u_dev) return fail(c, RSD_EINVAL, "sampling needs uniforms");
    if (temperature < 0.f || top_p < 0.f || top_p > 1.f) return fail(c, RSD_EINVAL, "bad temperature/top_p");
    sample_rows(c, logits_dev, vocab, vocab, u_dev, nullptr, 1, temperature, top_p, -1, 0.f, nullptr, n, out_dev, AppendArgs{});
    HIPCHK(c, hipGetLastError());
    HIPCHK(c, hipStreamSynchronize(c->st));
    return RSD_OK;
}

}  // extern "C"

#include "sample_static.h"

// --------------------------------------------------------------------------- rsd_forward
namespace {

template <typename WT>
int forward_impl(rsd_ctx* c, int which, const int32_t* tokens_host, const int32_t* lens, int T, int chunk, float* out) {
    const int B = c->B;
    Model& m = c->m[which];
    const bool lm = m.s.head_kind == RSD_HEAD_LM;
    const int V = m.s.vocab;
    HIPCHK(c, hipStreamSynchronize(c->st));
    reset_sequences(c);
    c->have_prompts = false;
    int maxlen = 0;
    for (int b = 0; b < B; ++b) {
        if (lens[b] < 0 || lens[b] > T) return fail(c, RSD_EINVAL, "lens[%d] out of range", b);
        maxlen = std::max(maxlen, lens[b]);
        if (!ensure_pages(m, b, ceil_div(lens[b], RSD_PAGE))) return fail(c, RSD_ENOMEM, "KV pool too small for rsd_forward");
        c->ctx_len()[b] = lens[b];
    }
    int rc;
    if ((rc = upload_tables(c, m))) return rc;
    HIPCHK(c, hipMemcpy2DAsync(c->ds.tokens, (size_t)c->p.max_ctx * sizeof(int), tokens_host, (size_t)T * sizeof(int),
                               (size_t)T * sizeof(int), B, hipMemcpyHostToDevice, c->st));
    if (chunk <= 1) {
        for (int t = 0; t < maxlen; ++t) {
            for (int b = 0; b < B; ++b) { c->active()[b] = t < lens[b]; c->kv_len(which)[b] = t; }
            if ((rc = push_state(c))) return rc;
            run_layers<WT>(c, m, B, decode_map(c, which), true);
            if (lm) lm_head<WT>(c, m, c->h, B, c->logits, V);
            else reward_rows<WT>(c, m, c->h, B, nullptr, c->tmp_reward);
            for (int b = 0; b < B; ++b)
                if (t < lens[b]) {
                    if (lm) HIPCHK(c, hipMemcpyAsync(out + ((size_t)b * T + t) * V, c->logits + (size_t)b * V, (size_t)V * sizeof(float), hipMemcpyDeviceToDevice, c->st));
                    else HIPCHK(c, hipMemcpyAsync(out + (size_t)b * T + t, c->tmp_reward + b, sizeof(float), hipMemcpyDeviceToDevice, c->st));
                }
            HIPCHK(c, hipStreamSynchronize(c->st));   // the mirror is rewritten next iteration
        }
    } else {
        for (int s0 = 0; s0 < maxlen; s0 += chunk) {
            std::vector<Piece> pieces;
            for (int b = 0; b < B; ++b)
                if (s0 < lens[b]) pieces.push_back(Piece{b, s0, std::min(lens[b], s0 + chunk)});
            auto after = [&](const std::vector<Piece>& pass, const std::vector<int>& first, int M) {
                if (!lm) reward_rows<WT>(c, m, c->h, M, nullptr, c->tmp_reward);
                for (size_t i = 0; i < pass.size(); ++i) {
                    const Piece& pc = pass[i];
                    const int n = pc.end - pc.start;
                    if (lm) lm_head<WT>(c, m, c->h + (size_t)first[i] * m.s.d_model, n, out + ((size_t)pc.b * T + pc.start) * V, V);
                    else HIPCHK(c, hipMemcpyAsync(out + (size_t)pc.b * T + pc.start, c->tmp_reward + first[i], n * sizeof(float), hipMemcpyDeviceToDevice, c->st));
                }
                return RSD_OK;
            };
            if ((rc = prefill<WT>(c, which, pieces, after))) return rc;
        }
    }
    HIPCHK(c, hipGetLastError());
    HIPCHK(c, hipStreamSynchronize(c->st));
    reset_sequences(c);
    return RSD_OK;
}

}  // namespace

extern "C" int rsd_forward(rsd_ctx* c, int32_t model, const int32_t* tokens_host, const int32_t* lens_host, int32_t T,
                           int32_t chunk, float* out_dev) {
    if (!c || model < 0 || model > 2 || !tokens_host || !lens_host || !out_dev) return fail(c, RSD_EINVAL, "bad argument");
    if (T < 1 || T > c->p.max_ctx) return fail(c, RSD_EINVAL, "T outside [1, max_ctx]");
    if (model == RSD_PRM && c->p.merge_prm != RSD_MERGE_NONE)
        return fail(c, RSD_EINVAL, "the merged reward model has no layers of its own to run");
    if (model == RSD_TARGET && c->p.bon_n > 0) return fail(c, RSD_EINVAL, "a Best-of-N context has no target model");
    return c->m[model].s.dtype == RSD_F32 ? forward_impl<float>(c, model, tokens_host, lens_host, T, chunk, out_dev)
                                           : forward_impl<bf16_t>(c, model, tokens_host, lens_host, T, chunk, out_dev);
}
