/*
 * rsd.h - C ABI of the Reward-Guided Speculative Decoding (RSD) hot path for
 * AMD MI355X (gfx950).
 *
 * One context runs the loop of the paper's Algorithm 1 (Section 2.1) for a
 * batch of independent sequences: per reasoning step the draft model m decodes
 * a candidate step, the process reward model r scores it with one scalar, the
 * acceptance criterion A_omega (Algorithm 2, Section 2.2; weighting functions
 * of Table 1) keeps it or the target model M regenerates the step from the
 * same context z_i = [x, y_1..i-1].  Inputs follow Algorithm 1's list: prompts
 * x, the three models, the criterion (delta, omega), the EOS token and the
 * length limits; the reasoning-step separator of Section 3 ("Default
 * Setting") and the sampling uniforms are explicit arguments.
 *
 * Conventions
 *  - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary
 *    host memory.  The library never frees or writes caller memory except the
 *    output buffers named below.  Weights, uniforms and teacher buffers are
 *    BORROWED: they must stay valid and unchanged while the context lives.
 *  - All GPU work is enqueued on the HIP stream given to rsd_init.  Calls
 *    return after their host-visible outputs are valid.
 *  - Every entry point returns RSD_OK (0) or a negative code; the text of the
 *    last failure is available from rsd_last_error.  Nothing aborts or throws.
 *  - A context is not thread-safe; distinct contexts may be used concurrently.
 */
#ifndef RSD_H
#define RSD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RSD_OK       0
#define RSD_EINVAL  (-1)  /* bad shape or argument */
#define RSD_ENOMEM  (-2)  /* KV page pool exhausted; sequence state is as before the call */
#define RSD_ESTATE  (-3)  /* call not valid in the current state (e.g. step after all finished) */
#define RSD_EHIP    (-4)  /* HIP runtime error */

enum { RSD_F32 = 0, RSD_BF16 = 1 };                 /* storage type of weights and KV cache */
enum { RSD_HEAD_LM = 0, RSD_HEAD_REWARD = 1 };
enum { RSD_DRAFT = 0, RSD_TARGET = 1, RSD_PRM = 2 };
/* weighting functions omega(r) of Table 1 */
enum { RSD_OMEGA_BINARY = 0,    /* 1(r >= delta): the paper's default                */
       RSD_OMEGA_CONSTANT = 1,  /* omega_a                                             */
       RSD_OMEGA_CLIP = 2,      /* min(1, max(0, r))                                   */
       RSD_OMEGA_RATIO = 3,     /* max(0, r / (1 + r))                                 */
       RSD_OMEGA_LOGISTIC = 4   /* 1 / (1 + exp(-omega_a (r - delta)))                 */ };
/* Model merge (Appendix "Model Merge"): the reward model may share every layer below the heads with a
 * policy model and keep only its own projection.  NONE: three separate models.  DRAFT / TARGET: the reward
 * is read off the final-norm hidden state of that model at the step's last token; shape[RSD_PRM] must
 * then repeat that model's dimensions and dtype (head_kind RSD_HEAD_REWARD), weights[RSD_PRM] holds only
 * w_r[d_model] followed by b_r (8 elements, the first is used), and no third KV cache exists
 * (kv_len[RSD_PRM] stays 0).  After a step: DRAFT as without merge; TARGET: kv_len[RSD_TARGET] = ctx - 1
 * for every sequence of the step (the target has read every committed token but the last). */
enum { RSD_MERGE_NONE = 0, RSD_MERGE_DRAFT = 1, RSD_MERGE_TARGET = 2 };
/* why a sequence stopped */
enum { RSD_RUNNING = 0, RSD_FIN_EOS = 1, RSD_FIN_MAX_CTX = 2, RSD_FIN_MAX_STEPS = 3 };

/* Decoder-only transformer: RMSNorm, rotary embedding (rotate-half pairing,
 * angle pos * theta^(-2i/hd)), grouped-query attention with head_dim =
 * d_model / n_heads (32 or 128; bf16 models: 128), SwiGLU MLP, untied head.
 * Constraints (rsd_init returns RSD_EINVAL otherwise): d_model and d_ffn
 * multiples of 64 and at least 64; n_heads % n_kv_heads == 0 with a group of
 * 1, 2, 4, 6, 7 or 8 query heads per KV head; vocab >= 2. */
typedef struct rsd_model_shape {
    int32_t n_layers, d_model, n_heads, n_kv_heads, d_ffn, vocab;
    float   rope_theta, rms_eps;
    int32_t dtype;       /* RSD_F32 | RSD_BF16 */
    int32_t head_kind;   /* RSD_HEAD_LM: lm_head[vocab][d] | RSD_HEAD_REWARD: w_r[d], b_r */
} rsd_model_shape;

/* One model's weights: a single dev blob, row-major [out][in] matrices of the
 * model's dtype in this order:
 *   embed[vocab][d];
 *   per layer: attn_norm[d], wq[H*hd][d], wk[Hkv*hd][d], wv[Hkv*hd][d],
 *              wo[d][H*hd], ffn_norm[d], w_gate[F][d], w_up[F][d], w_down[d][F];
 *   final_norm[d];
 *   lm_head[vocab][d]            (RSD_HEAD_LM)
 *   w_r[d], b_r[8] (b_r[0] used) (RSD_HEAD_REWARD; reward = logistic(w_r.y + b_r),
 *                                 the scalar projection on the last layer described
 *                                 in the appendix section "Model Merge")
 * The blob must be 16-byte aligned. */
typedef struct rsd_weights { const void *blob; uint64_t nbytes; } rsd_weights;

typedef struct rsd_params {
    float   delta;          /* threshold of the binary step / centre of the logistic */
    int32_t omega_kind;     /* RSD_OMEGA_* */
    float   omega_a;        /* constant p, or logistic slope alpha */
    int32_t sep_id;         /* token that ends a reasoning step (the step includes it) */
    int32_t eos_id;         /* -1: none */
    int32_t step_cap;       /* most tokens in one step */
    int32_t max_steps;      /* iterations of Algorithm 1's loop */
    int32_t max_ctx;        /* most tokens per sequence, prompt included */
    float   temperature;    /* 0: greedy (lowest id on ties) */
    float   top_p;          /* nucleus mass, used when temperature > 0 */
    float   sep_logit_bias; /* added to the separator's logit before sampling (synthetic workloads) */
    int32_t page_tokens;    /* tokens per KV page; must be 16 */
    uint64_t kv_pool_bytes[3]; /* KV page pool per model (draft, target, reward); 0: enough for batch * max_ctx */
    int32_t use_graphs;     /* 1: replay single-token decode iterations as HIP graphs */
    int32_t merge_prm;      /* RSD_MERGE_*: where the reward head sits */
    int32_t sd_k;           /* > 0: a rejected step is regenerated by token-level speculative decoding with
                               the draft and the target (Section 5, "Combine RSD with SD"), this many
                               proposals per round (the paper's SD runs use 7); 0: plain target decoding.
                               Greedy (the paper's SD setting, Section 3 "Default Setting") or
                               sampled (then rsd_set_uniforms_sd supplies two more uniform streams).
                               At most 15. */
    int32_t bon_n;          /* > 0: the context runs process Best-of-N instead of RSD (one of the paper's comparison
                               procedures, Section 3 "Baselines": per reasoning step the base model samples bon_n
                               candidate steps from the same context, the reward model scores each, the best is
                               committed).  `batch` then counts candidate lanes = sequences * bon_n (lane s * bon_n + n
                               is candidate n of sequence s); only the draft (the base model) and the reward model are
                               used (shape[RSD_TARGET] / w[RSD_TARGET] are ignored); merge_prm and sd_k must be 0.
                               See rsd_bon_step.  0: RSD. */
} rsd_params;

/* Per-step record, all HOST buffers supplied by the caller (any may be NULL).
 * Index b is the sequence. */
typedef struct rsd_step_out {
    int32_t *draft_len;     /* [B]            tokens in the draft step (0 if the sequence was finished) */
    int32_t *draft_tokens;  /* [B][step_cap]  the draft step as appended                                 */
    float   *reward;        /* [B]            r_i of the draft step                                      */
    int32_t *accepted;      /* [B]            decision applied                                           */
    int32_t *own_accept;    /* [B]            decision the criterion took (differs only under a teacher) */
    int32_t *final_len;     /* [B]            tokens in the committed step                               */
    int32_t *final_tokens;  /* [B][step_cap]                                                             */
    int32_t *finished;      /* [B]            RSD_RUNNING or a RSD_FIN_* reason, after this step         */
    /* speculative regeneration of a rejected step (sd_k > 0), zero otherwise */
    int32_t *sd_rounds;     /* [B]            propose-and-verify rounds of this step                     */
    int32_t *sd_proposed;   /* [B]            tokens the draft proposed in them                          */
    int32_t *sd_kept;       /* [B]            proposals the target kept                                  */
} rsd_step_out;

typedef struct rsd_gen_out {
    int32_t *tokens;        /* host [B][max_ctx] or NULL: the ctx_len[b] tokens of sequence b, then -1 */
    int32_t *ctx_len;       /* host [B] or NULL */
    int32_t *finished;      /* host [B] or NULL */
    int32_t  steps_run;
    int64_t  n_committed;   /* tokens committed over all sequences (what tokens/s counts) */
    int64_t  n_draft;       /* tokens the draft model sampled (rejected ones included)    */
    int64_t  n_target;      /* tokens the target model sampled                            */
    int64_t  n_accept;      /* accepted steps */
    int64_t  n_reject;      /* rejected steps */
    int64_t  n_sd_rounds;   /* sd_k > 0: propose-and-verify rounds, proposals made, proposals kept */
    int64_t  n_sd_proposed;
    int64_t  n_sd_kept;
} rsd_gen_out;

typedef struct rsd_ctx rsd_ctx;

/* Create a context for `batch` sequences.  shape[i]/w[i] with i = RSD_DRAFT,
 * RSD_TARGET, RSD_PRM; draft and target need RSD_HEAD_LM and one common
 * vocabulary, the reward model RSD_HEAD_REWARD.  Allocates the KV page pools,
 * block tables, rotary tables and workspaces (library-owned, freed by
 * rsd_destroy).  hip_stream is a hipStream_t (NULL: the default stream). */
int rsd_init(rsd_ctx **out, const rsd_model_shape shape[3], const rsd_weights w[3],
             const rsd_params *p, int32_t batch, void *hip_stream);

/* Load prompts x and reset every sequence to "no step taken": tokens is dev
 * [B][max_ctx] int32 (only the first prompt_len[b] entries of a row are read),
 * prompt_len is host [B], each in [1, max_ctx]. */
int rsd_set_prompts(rsd_ctx *c, const int32_t *tokens_dev, const int32_t *prompt_len_host);

/* Uniforms in [0,1), BORROWED dev arrays: u_draft/u_target [B][max_ctx], the
 * token placed at absolute position i of sequence b is drawn with u[b][i];
 * u_gate [B][max_steps] is the draw of Algorithm 2 for step i (only read when
 * omega(r) is strictly between 0 and 1).  May be NULL when never needed
 * (greedy decoding / binary omega). */
int rsd_set_uniforms(rsd_ctx *c, const float *u_draft_dev, const float *u_target_dev,
                     const float *u_gate_dev);

/* Change delta / omega without rebuilding the context (takes effect at the next step). */
int rsd_set_criterion(rsd_ctx *c, float delta, int32_t omega_kind, float omega_a);

/* One iteration of Algorithm 1's loop body for all unfinished sequences:
 * draft step, reward, criterion, target step for the rejected ones, EOS test.
 * On RSD_ENOMEM the sequences are left as before the call.
 *
 * With sd_k > 0 the target step is produced in rounds: with `used` tokens of the
 * step so far the draft proposes g = min(sd_k, step_cap - used - 1,
 * max_ctx - ctx_len - 1) tokens one by one (stopping after a separator or EOS),
 * the target reads what it has not seen plus the proposals in one chunked pass,
 * and the step grows by the leading proposals the target keeps plus one token of
 * its own at the first refused place (or after the last proposal), until a
 * committed token ends the step.  Greedy: a proposal is kept iff it equals the
 * target's arg max, which is also the token of its own.  Sampled: proposal x,
 * drawn from the draft's distribution q, is kept iff u_accept * q(x) < p(x) with p
 * the target's distribution at that place (both as the sampler draws from them:
 * temperature, nucleus, renormalised); the replacement is drawn from the
 * normalised positive part of p - q, the token after a fully kept run from p.  Afterwards neither
 * model holds keys/values for the newest token or for a dropped proposal. */
int rsd_step(rsd_ctx *c, rsd_step_out *out);

/* Algorithm 1's loop: rsd_step until every sequence has finished or max_steps
 * (<= params.max_steps, 0 = params.max_steps) steps have run since the prompts
 * were set. */
int rsd_generate(rsd_ctx *c, int32_t max_steps, rsd_gen_out *out);

/* ---- process Best-of-N (contexts created with bon_n > 0) ----
 * Candidate n of a sequence draws the token it places at absolute position i with u_draft[s * bon_n + n][i]
 * (rsd_set_uniforms: u_draft is [batch][max_ctx] over lanes; u_target / u_gate are unused); rsd_set_prompts
 * takes one prompt per SEQUENCE (tokens dev [sequences][max_ctx], prompt_len host [sequences]).  The
 * candidates of a step share the cache pages of the committed context (reference-counted; the one page a
 * candidate would write into while others still read it is copied first), each owns the pages of its own
 * step, and after the choice the pages of the other candidates return to the pool.
 *
 * Per-step record, HOST buffers (any may be NULL); N = bon_n, s = sequence. */
typedef struct rsd_bon_out {
    int32_t *cand_len;      /* [sequences][N]            tokens of every candidate step (0: sequence had finished) */
    int32_t *cand_tokens;   /* [sequences][N][step_cap]                                                           */
    float   *cand_reward;   /* [sequences][N]                                                                     */
    int32_t *chosen;        /* [sequences]               candidate committed                                      */
    int32_t *own_choice;    /* [sequences]               arg max of the rewards, lowest index among equals
                                                         (differs from chosen only under a teacher)               */
    int32_t *finished;      /* [sequences]               RSD_RUNNING or a RSD_FIN_* reason, after this step       */
    int32_t *ctx_len;       /* [sequences]               tokens of the sequence after the step                    */
    int32_t *kv_len;        /* [2][sequences]            leading tokens the base / the reward model hold keys and
                                                         values for (ctx_len - 1 and ctx_len after a step)        */
    int32_t *n_pages;       /* [2][sequences]            cache pages the sequence owns in each of the two caches  */
} rsd_bon_out;

/* One reasoning step of process Best-of-N for all unfinished sequences.  RSD_ENOMEM (a page pool ran out)
 * leaves every sequence as before the call.  Under rsd_set_teacher the forced_draft array is indexed by lane
 * ([batch][max_steps][step_cap]) and forced_accept ([sequences][max_steps]), when >= 0, is the candidate to
 * commit. */
int rsd_bon_step(rsd_ctx *c, rsd_bon_out *out);

/* rsd_bon_step until every sequence has finished or max_steps (<= params.max_steps, 0 = params.max_steps)
 * steps have run since the prompts were set.  out->tokens is [sequences][max_ctx], ctx_len / finished
 * [sequences]; n_draft counts every candidate token sampled, n_committed the committed ones. */
int rsd_bon_generate(rsd_ctx *c, int32_t max_steps, rsd_gen_out *out);

/* Page sharing since the context was created: page references handed to candidates by sharing a committed
 * page instead of allocating one, pages copied because a candidate had to write into a shared one, and pages
 * taken from the pools.  Host counters. */
int rsd_bon_stats(rsd_ctx *c, int64_t *pages_shared, int64_t *pages_copied, int64_t *pages_allocated);

/* Sequence state for bit-exact checks, HOST buffers (any may be NULL):
 * ctx_len [B]; kv_len [3][B] = leading tokens each model holds keys/values
 * for; n_pages [3][B] = KV pages owned; tokens [B][max_ctx] = the ctx_len[b]
 * tokens of row b, then -1. */
int rsd_export_state(rsd_ctx *c, int32_t *ctx_len, int32_t *kv_len, int32_t *n_pages,
                     int32_t *tokens);

/* Page bookkeeping of one model, HOST buffers: block_table [B][max_pages]
 * (physical page of each logical page, -1 beyond n_pages), *max_pages,
 * *pool_pages, *free_pages. */
int rsd_export_pages(rsd_ctx *c, int32_t model, int32_t *block_table, int32_t *max_pages,
                     int32_t *pool_pages, int32_t *free_pages);

/* Teacher forcing for parity tests, BORROWED dev arrays (NULL switches a part
 * off): forced_draft / forced_target [B][max_steps][step_cap]: when entry
 * [b][i][j] is >= 0, the j-th token that model appends in step i of sequence b
 * is the forced one (the model's own choice is still recorded, see
 * rsd_export_sampled); forced_accept [B][max_steps]: when >= 0, the decision
 * applied at that step. */
int rsd_set_teacher(rsd_ctx *c, const int32_t *forced_draft_dev, const int32_t *forced_target_dev,
                    const int32_t *forced_accept_dev);

/* The tokens each model's sampler chose: HOST [B][max_steps][step_cap] each,
 * -1 where the model sampled nothing. */
int rsd_export_sampled(rsd_ctx *c, int32_t *sampled_draft, int32_t *sampled_target);

/* Speculative regeneration (sd_k > 0), for parity tests.  Both arrays are
 * [B][max_steps][step_cap * sd_k]; entry [b][i][n] belongs to the n-th proposal
 * the draft makes while step i of sequence b is regenerated (a place of the step
 * can be proposed for in several rounds, so proposals are counted, in the order
 * they are made).  forced_proposal (BORROWED dev, NULL: off): when >= 0, the
 * proposal is replaced by it.  proposed (HOST): the draft's own choices, -1
 * beyond the proposals made.  With sd_k > 0 sampled_target of rsd_export_sampled
 * holds the target's choice at every committed place of a regenerated step, kept
 * proposals included. */
int rsd_set_teacher_sd(rsd_ctx *c, const int32_t *forced_proposal_dev);
/* kept_flags (HOST, same shape, may be NULL; sampled decoding only): 1 / 0 = the
 * acceptance test u * q(x) < p(x) kept / refused that proposal (taken for every
 * proposal of a round, also those behind its first refusal), -1 elsewhere. */
int rsd_export_proposed(rsd_ctx *c, int32_t *proposed, int32_t *kept_flags);

/* Uniforms of sampled speculative regeneration (temperature > 0 and sd_k > 0),
 * BORROWED dev arrays [B][max_ctx]: the proposal for absolute position i of
 * sequence b is drawn with u_proposal[b][i] and judged with u_accept[b][i]; a token
 * the target draws itself at position i (replacement of a refused proposal, or
 * the token after a fully kept run) uses u_target[b][i] of rsd_set_uniforms. */
int rsd_set_uniforms_sd(rsd_ctx *c, const float *u_proposal_dev, const float *u_accept_dev);

/* The verification rule alone, for parity tests (context with sd_k > 0 and
 * temperature > 0; its temperature, top_p and separator bias apply).  n <= batch
 * cases; case s has n_proposals[s] <= sd_k proposals (HOST array).  dev inputs:
 * p_logits [n][sd_k+1][vocab] (target), q_logits [n][sd_k][vocab] (draft),
 * proposals [n][sd_k], u_accept [n][sd_k+1] (last column unused), u_new
 * [n][sd_k+1] (uniform of a token the target draws at that place).  dev outputs:
 * emitted [n][sd_k+1]: the kept proposals, then the replacement of the first
 * refused one or, after a fully kept run, the draw from the next target row
 * (entries behind that one are unspecified); kept [n]. */
int rsd_sd_verify(rsd_ctx *c, const float *p_logits_dev, const float *q_logits_dev,
                  const int32_t *proposals_dev, const int32_t *n_proposals_host,
                  const float *u_accept_dev, const float *u_new_dev, int32_t n,
                  int32_t *emitted_dev, int32_t *kept_dev);

/* Teacher-forced evaluation of one model for parity tests.  tokens is host
 * [B][T], lens host [B] (<= T).  Sequence b is fed in pieces of `chunk` tokens
 * (chunk == 1 runs the single-token decode kernels, larger values the chunked
 * prefill kernels) through the model's own paged KV cache, starting empty.
 * out is dev fp32: [B][T][vocab] logits for RSD_HEAD_LM models, [B][T] rewards
 * for the reward model; entries at positions >= lens[b] are not written.
 * Resets the sequences: call rsd_set_prompts before stepping again. */
int rsd_forward(rsd_ctx *c, int32_t model, const int32_t *tokens_host, const int32_t *lens_host,
                int32_t T, int32_t chunk, float *out_dev);

/* The sampler alone: for each of n rows pick a token from logits[row][vocab]
 * (dev fp32) with uniform u[row] (dev), at the given temperature / top_p
 * (temperature 0: arg max).  out_dev is dev int32 [n]. */
int rsd_sample(rsd_ctx *c, const float *logits_dev, const float *u_dev, int32_t n, int32_t vocab,
               float temperature, float top_p, int32_t *out_dev);

/* Wall-clock milliseconds spent in the stages of rsd_step since the context was
 * created or the counters were last reset (host timers around synchronised
 * stages): ms[0] draft, ms[1] reward model, ms[2] criterion + rollback,
 * ms[3] target.  reset != 0 clears them after reading. */
int rsd_stage_ms(rsd_ctx *c, double ms[4], int32_t reset);

/* Launch statistics of the single-token decode loop (Algorithm 1's token-by-token generation of a
 * step): iterations launched kernel by kernel, iterations replayed from a recorded graph, and the
 * number of graphs recorded so far.  With use_graphs = 1 every iteration is a replay except a
 * model's first one and those the timing probe brackets; replays = 0 there means that recording
 * failed and the context fell back to kernel-by-kernel launches.  Host counters, no GPU work. */
int rsd_decode_stats(rsd_ctx *c, int64_t *eager_iters, int64_t *graph_replays, int64_t *graphs_recorded);

/* Kernel timing probes for roofline reports.  RSD_PROBE_SLOTS independent probes; while slot `slot` is armed,
 * every `stride`-th launch of one weight-streaming projection (op: 0 qkv, 1 attention output, 2 gate+up,
 * 3 down, 4 output head) of `model` is bracketed by a pair of HIP events on the context's stream, up to
 * max_samples pairs.  phase RSD_PROBE_DECODE: launches of the single-token decode iteration (Algorithm 1's
 * token-by-token generation of a step; inside the decode loop every stride-th *iteration* is launched kernel
 * by kernel with its launch timed, the others are replayed from the recorded graph); phase RSD_PROBE_PREFILL:
 * launches of chunked passes (reward scoring of a step, catch-up).  Only the matrix kernel itself is timed
 * (not the kernels that add K slices or apply the epilogue).  rsd_probe_read synchronises, returns the
 * number of timed launches, their summed duration, and over the same launches the summed algorithmic bytes
 * (weights once + activations in and out) and floating-point operations (2 * rows * N * K), and disarms. */
#define RSD_PROBE_SLOTS 4
enum { RSD_PROBE_DECODE = 0, RSD_PROBE_PREFILL = 1 };
int rsd_probe_start(rsd_ctx *c, int32_t slot, int32_t model, int32_t phase, int32_t op, int32_t max_samples,
                    int32_t stride);
int rsd_probe_read(rsd_ctx *c, int32_t slot, int64_t *n_samples, double *total_ms, int64_t *total_bytes,
                   int64_t *total_flops);

/* The clock the chip sustains under the probed many-row (chunked-pass) GEMMs.  While slot `slot` is armed with
 * phase RSD_PROBE_PREFILL, every probed launch of the tile GEMM has the thread block in the middle of its grid
 * read the shader clock counter and the constant 100 MHz reference counter around its K loop; the differences
 * are summed per slot (cleared by rsd_probe_start, kept across rsd_probe_read).  Returns the number of launches
 * that reported, the summed shader ticks and the summed reference ticks: shader_ticks / ref_ticks * 100 MHz is
 * the mean shader clock during those launches (the published MFMA peak assumes 2400 MHz).  Launches served by
 * the few-row kernels (<= 64 rows) report nothing.  Synchronises the stream; host pointers; any may be NULL. */
int rsd_probe_clock(rsd_ctx *c, int32_t slot, int64_t *launches, int64_t *shader_ticks, int64_t *ref_ticks);

/* Accounting of the single-token decode loop of one policy model (RSD_DRAFT or RSD_TARGET; the loop that
 * generates a reasoning step token by token, Algorithm 1) since the context was created or the counters
 * were last reset: iterations launched (each streams the model's weights once, whatever the number of
 * sequences), GPU time between HIP events recorded before the first and after the last iteration of every
 * loop (the polls of the active counter inside are included, chunked first passes are not), sequence-
 * iterations (one per token sampled in the loop), and the keys/values read: the sum over those
 * sequence-iterations of the context length attended to.  Iterations of speculative regeneration are not
 * counted.  reset != 0 clears the counters after reading.  Host outputs, any may be NULL. */
int rsd_iter_stats(rsd_ctx *c, int32_t model, int64_t *iterations, double *gpu_ms, int64_t *seq_iterations,
                   int64_t *kv_tokens_read, int32_t reset);

/* Rows launched by the iterations rsd_iter_stats counts: the sum over those iterations of the number of
 * activation rows every kernel of the iteration was launched over.  A stage in which only some sequences
 * take part (the target's stage of Algorithm 1 after the reward model accepted the other sequences' steps)
 * packs its sequences into fewer rows than the batch has (1..8 exactly, then 32, 64, multiples of 128), so
 * row_iterations / iterations lies between the mean number of active sequences and the batch size.
 * Cleared together with rsd_iter_stats' counters.  Host output. */
int rsd_iter_rows(rsd_ctx *c, int32_t model, int64_t *row_iterations);

/* Diagnostic for the paged caches (Section 3 serves the models from a paged KV cache; the kernels index the block
 * tables without checks): would a pass over n rows, row i standing for position pos_host[i] of sequence
 * seq_host[i] (HOST arrays), stay inside what the device-side tables of `model` give those sequences?  Checked
 * by a kernel that reads nothing it has not bounds-checked itself: the sequence index lies in the batch, the
 * position in [0, max_ctx), the sequence owns the pages 0 .. pos / 16, and each of those table entries names a
 * page of the pool.  Returns RSD_OK, or RSD_ESTATE with the first offending row in rsd_last_error.  Waits for the
 * stream.  n in 1 .. 8192.
 *
 * A library compiled with -DRSD_DEBUG (rsd_debug_build() returns 1; the package builds it as librsd_debug.so)
 * runs the same check before every chunked pass and before every single-token iteration of every entry point,
 * on the rows and the device-side positions that pass is about to use, waits for the verdict and returns
 * RSD_ESTATE instead of launching a pass that would leave its pages; it records no graphs.  Nothing traps. */
int rsd_check_rows(rsd_ctx *c, int32_t model, const int32_t *seq_host, const int32_t *pos_host, int32_t n);
int rsd_debug_build(void);

/* Timing of the decode attention kernel alone (grouped-query attention of one new token per sequence over
 * the paged cache, rotary embedding and cache write included), for roofline reports.  Sequence b gets a
 * context of ctx_len_host[b] tokens (1 .. max_ctx; HOST array [B]) in `model`'s cache, whose pool is
 * cleared; the kernel (and the kernel merging context splits, when the context is split) is launched
 * `reps` times in the launch configuration of the decode iteration, cycling through the layers so that
 * successive launches read different memory, between two HIP events.  *total_ms is the time between the
 * events.  Resets the sequences: call rsd_set_prompts before stepping again.  RSD_ENOMEM when the pool
 * cannot hold the contexts. */
int rsd_probe_attention(rsd_ctx *c, int32_t model, const int32_t *ctx_len_host, int32_t reps, double *total_ms);

/* rsd_sample for callers that cannot allocate device memory: code recording a HIP graph, tight serving
 * loops, harnesses that forbid hipMalloc.  Same choice rule and arguments as rsd_sample (dev logits [n][vocab]
 * fp32, dev uniforms [n], dev out [n]), but no context: the sampler's workspace (block maxima, radix
 * histograms, block masses; about 49 KiB per row) is a device array built into the library, which every GPU
 * the library runs on holds until the process ends (RSD_SAMPLE_STATIC_MAX_ROWS rows, 3.1 MiB).  The call
 * allocates and frees nothing and does not synchronise: the kernels are enqueued on hip_stream (a
 * hipStream_t, NULL: the default stream) and out_dev is valid once that stream has reached them.
 * n > RSD_SAMPLE_STATIC_MAX_ROWS, n < 1, vocab < 1, NULL logits/out, sampling without uniforms or a bad
 * temperature / top_p return RSD_EINVAL; a HIP failure returns RSD_EHIP (there is no context to hold an
 * error text).  All calls on one GPU share that GPU's array: calls that overlap on one GPU (two streams, two
 * threads) race; successive calls on one stream do not. */
#define RSD_SAMPLE_STATIC_MAX_ROWS 64
int rsd_sample_static(const float *logits_dev, const float *u_dev, int32_t n, int32_t vocab, float temperature,
                      float top_p, int32_t *out_dev, void *hip_stream);

const char *rsd_last_error(const rsd_ctx *c);
void rsd_destroy(rsd_ctx *c);

#ifdef __cplusplus
}
#endif
#endif /* RSD_H */
