/*
 * pc.h -- C ABI of the group-rollout library for AMD MI355X (gfx950).
 *
 * The library generates the rollouts that a Pilot-Commit training step
 * consumes: for a batch of prompts it samples a few "pilot" completions per
 * prompt from a decoder-only policy, scores each prompt by the mean of its
 * binary rewards, keeps the prompts whose pilot success rate lies in
 * [p_lower, p_upper], samples further "commit" completions for the kept
 * prompts only, and returns group-relative advantages over the union
 * (paper Section 3.1, Section 3.3, Algorithm 1).
 *
 * Conventions
 *   - "device" pointers are HIP device memory owned by the caller; "host"
 *     pointers are ordinary host memory.  Every pointer below says which.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work; they never synchronise the stream unless the
 *     comment of the call says so.  The caller orders calls on one stream.
 *   - Every call returns a pc_status: PC_OK (0) or a negative error code.  On
 *     error nothing has been launched and no library state has changed;
 *     pc_last_error() returns a message for the calling thread's last error.
 *   - The library never throws and never aborts.
 *   - All matrices are row-major [out_features, in_features].
 */
#ifndef PC_H
#define PC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t pc_status;
#define PC_OK 0
#define PC_ERR_INVALID_ARG (-1)
#define PC_ERR_OOM (-2)         /* KV pool, slot table or scratch exhausted */
#define PC_ERR_HIP (-3)         /* a HIP runtime call failed */
#define PC_ERR_UNSUPPORTED (-4) /* shape outside what the kernels support */

#define PC_DTYPE_F32 0
#define PC_DTYPE_BF16 1

/* Type of the activations, the KV cache and the library's own weight copies of a bf16 model. */
#define PC_ACT_DEFAULT 0 /* = PC_ACT_F16 */
#define PC_ACT_BF16 1    /* bfloat16 throughout.  OUTSIDE the 2e-2 logit acceptance bound for deep models: every
                            rounding point loses 2^-9 relative, and over a 28-layer decoder the logits drift by up
                            to 1e-1 (measured 7.5e-2 on the 1.5B shape).  Kept for callers that need the bf16
                            exponent range; tested against its own bound of 1.5e-1 x max(1, max|logit|). */
#define PC_ACT_F16 2     /* IEEE half: the bf16 weights convert to half without loss (below 6.1e-5 in magnitude
                            with an absolute error under 3e-8); activations carry 11 significand bits instead of
                            8 at the same matrix-core rate, which keeps the logits of a 28-layer model within
                            1e-2 of exact arithmetic.  This is the type the 2e-2 acceptance bound is met with.
                            Values beyond the half range (65504) SATURATE to +-65504 (never inf/NaN) and every
                            saturated store is counted: see pc_saturation_count. */

typedef struct pc_ctx pc_ctx;

/* Shape of the decoder-only policy pi_theta (Section 3.1): pre-norm
 * transformer, RMSNorm, rotary positions (rotate-half pairing), grouped-query
 * attention, SwiGLU feed-forward.  dtype is the storage type of the matrices,
 * embeddings and KV cache; the residual stream, norm statistics, softmax and
 * logits are always fp32. */
typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ff, vocab;
    float rms_eps, rope_theta;
    int32_t dtype;     /* PC_DTYPE_F32 or PC_DTYPE_BF16 */
    int32_t act_dtype; /* PC_ACT_*; ignored for fp32 models */
} pc_model_config;

/* Device pointers to the weights.  The per-layer members are HOST arrays of
 * n_layers DEVICE pointers.  Norm gains are fp32 [d_model]; everything else
 * has the model dtype.  lm_head may alias tok_embed (tied embeddings).
 * pc_create copies the per-layer matrices into its own fused layout (and, with
 * PC_ACT_F16, lm_head too), so only tok_embed, lm_head and final_norm must
 * outlive the context. */
typedef struct {
    const void *tok_embed;  /* [vocab, d_model] */
    const void *lm_head;    /* [vocab, d_model] */
    const void *final_norm; /* fp32 [d_model] */
    const void *const *attn_norm; /* fp32 [d_model] each */
    const void *const *wq;        /* [n_q_heads*head_dim, d_model] */
    const void *const *wk;        /* [n_kv_heads*head_dim, d_model] */
    const void *const *wv;        /* [n_kv_heads*head_dim, d_model] */
    const void *const *wo;        /* [d_model, n_q_heads*head_dim] */
    const void *const *ffn_norm;  /* fp32 [d_model] each */
    const void *const *w_gate;    /* [d_ff, d_model] */
    const void *const *w_up;      /* [d_ff, d_model] */
    const void *const *w_down;    /* [d_model, d_ff] */
} pc_weights;

/* Paged KV cache.  The context owns a pool of kv_pool_bytes (rounded down to
 * whole blocks of block_size tokens across all layers), a table of max_slots
 * slots (one per live prompt or sequence) and activation scratch for
 * max_batch_rows rows (the largest number of token rows one call processes:
 * prompt tokens of one prefill chunk, or sequences of one decode step). */
typedef struct {
    int32_t block_size;     /* tokens per KV block; a multiple of 32, at most 256 */
    int64_t kv_pool_bytes;
    int32_t max_slots;
    int32_t max_ctx;        /* longest prompt + completion, in tokens */
    int32_t max_batch_rows;
} pc_cache_config;

/* Options for pc_set_option. */
#define PC_OPT_USE_GRAPH 1   /* 1: replay the decode step as a HIP graph (default 1) */
#define PC_OPT_FORCE_SIMT 2  /* 1: plain-ALU kernels also for bf16 (debugging aid; default 0) */
#define PC_OPT_FUSE_DECODE 4   /* 1: decode batches of up to 512 rows of a 16-bit model with head_dim 128 whose q/k/v
                                  projection has at most 8 M weights run the fused layer (q/k/v projection with rotary
                                  positions and cache append in its epilogue; output projection that also leaves the next
                                  RMSNorm's inputs; that norm's scale applied by the gate/up epilogue): six launches per
                                  layer instead of eight; larger models keep one kernel per operation, which is faster
                                  there (default 1; 0 keeps one kernel per operation everywhere) */
#define PC_OPT_TIME_NEXT_STEP 3 /* value = a PC_KERNEL_* class: the next pc_decode_step runs eagerly (no graph)
                                   with a HIP event pair around every launch of that class; -1 disarms */

/* Kernel classes of a decode step, for PC_OPT_TIME_NEXT_STEP / pc_timing_read. */
#define PC_KERNEL_ATTN_DECODE 0
#define PC_KERNEL_GEMM_QKV 1
#define PC_KERNEL_GEMM_WO 2
#define PC_KERNEL_GEMM_GATE_UP 3
#define PC_KERNEL_GEMM_DOWN 4
#define PC_KERNEL_GEMM_LM_HEAD 5

const char *pc_last_error(void);

/* Creates a context on the current HIP device.  Allocates the KV pool, slot
 * tables, scratch and the fused weight copies; synchronises the device once.
 * `out` (host) receives the context. */
pc_status pc_create(const pc_model_config *model, const pc_weights *weights,
                    const pc_cache_config *cache, pc_ctx **out);
pc_status pc_destroy(pc_ctx *ctx);
pc_status pc_set_option(pc_ctx *ctx, int32_t option, int32_t value);
/* Sums the event pairs recorded since the last reset: total_ms (host double) and launches (host
 * int64) over all timed launches; empty_ms / empty_pairs (host, may be NULL): the same for the
 * calibration pairs (one per timed step, recorded back to back with nothing between, i.e. what the
 * bracket itself costs).  SYNCHRONISES on the recorded events.  reset != 0 recycles them. */
pc_status pc_timing_read(pc_ctx *ctx, double *total_ms, int64_t *launches, double *empty_ms,
                         int64_t *empty_pairs, int32_t reset);
/* Number of free slots / all slots of the context (a slot holds one live prompt or sequence). */
pc_status pc_slots(const pc_ctx *ctx, int64_t *free_slots, int64_t *total_slots);
/* Number of activation / KV-cache values that were clamped to +-65504 on their way into IEEE half since
 * the last reset (PC_ACT_F16 contexts; always 0 otherwise).  A non-zero count means the model's activations
 * leave the half range and the logits are no longer trustworthy: use PC_ACT_BF16 for such a model.
 * `count` is a host pointer.  SYNCHRONISES the device. */
pc_status pc_saturation_count(pc_ctx *ctx, int64_t *count, int32_t reset);
/* Number of free KV blocks / total KV blocks (host bookkeeping, no GPU work). */
pc_status pc_kv_blocks(const pc_ctx *ctx, int64_t *free_blocks, int64_t *total_blocks);

/* Shared-prefix prefill: the context pi_theta(. | q) of each prompt is computed
 * ONCE (Section 3.3: n rollouts o_j ~ pi_theta(.|q) per prompt q); all rollouts
 * of the prompt later reference the same KV blocks through their block tables.
 *   prompt_tokens  device int32, prompts packed back to back
 *   cu_lens        host int32 [P+1], cu_lens[0] = 0, prompt p = tokens[cu_lens[p] .. cu_lens[p+1])
 *   handle_out     host int32 [P]: a handle per prompt (a slot index)
 *   last_logits    device fp32 [P, vocab]: next-token logits after each prompt
 * Token ids outside [0, vocab) are read as id 0.  Prompts are processed in
 * chunks of at most max_batch_rows tokens; a prompt longer than that, longer
 * than max_ctx, or empty is PC_ERR_INVALID_ARG; running out of blocks or slots
 * is PC_ERR_OOM (nothing is kept). */
pc_status pc_prefill_shared(pc_ctx *ctx, const int32_t *prompt_tokens, const int32_t *cu_lens,
                            int32_t P, int32_t *handle_out, float *last_logits, void *stream);

/* Starts one sequence per entry of prompt_handle (host int32 [n]; a handle may
 * repeat: that is the group of G rollouts of a prompt).  Each sequence's block
 * table references the prompt's full blocks; a partially filled last prompt
 * block is copied into a private block.  Blocks for max_new_tokens further
 * tokens are reserved now, so that decode steps never allocate.
 *   seq_out  host int32 [n]: sequence ids (slot indices). */
pc_status pc_fork(pc_ctx *ctx, const int32_t *prompt_handle, int32_t n, int32_t max_new_tokens,
                  int32_t *seq_out, void *stream);

/* KV blocks a pc_fork of each entry would take from the pool (host bookkeeping, nothing changes): lets a
 * caller cut a pass whose sequences do not all fit into waves (Section 3.4 binding on one GPU: the commit and
 * pilot sequences of a step share the pool).  blocks_out: host int64 [n]. */
pc_status pc_fork_need(const pc_ctx *ctx, const int32_t *prompt_handle, int32_t n, int32_t max_new_tokens,
                       int64_t *blocks_out);

/* One decode step pi_theta(o_t | q, o_<t) (Section 3.1) for n sequences:
 * feeds one token per sequence, appends its K/V to the cache, returns the
 * next-token logits.
 *   seq        host int32 [n], distinct sequence ids
 *   tokens_in  device int32 [n]
 *   logits     device fp32 [n, vocab]
 * With PC_OPT_USE_GRAPH the step is captured once per (sequence list,
 * pointers, stream) and replayed; keep the pointers stable across steps.
 * A sequence that already holds prompt length + max_new_tokens tokens (the
 * reservation of its pc_fork) is PC_ERR_INVALID_ARG. */
pc_status pc_decode_step(pc_ctx *ctx, const int32_t *seq, const int32_t *tokens_in, int32_t n,
                         float *logits, void *stream);

/* pc_decode_step for callers that cannot allocate device memory while they run (code under HIP graph
 * capture of their own, tight serving loops, harnesses that forbid hipMalloc): same arguments, same
 * kernels, same results, but it calls no hipMalloc / hipFree / graph instantiation, and the scratch its
 * kernels need beyond the inputs and outputs (the K slices of the split projections and the partial
 * results of the context-split attention) lives in one fixed 32 MiB device array inside the library.
 * The step is always launched eagerly.  A batch whose scratch would not fit -- 8 * n * max(q/k/v width,
 * d_model) * 4 bytes of slices plus (n + 512) * n_q_heads * (head_dim + 2) * 4 bytes of attention
 * partials, e.g. more than 470 sequences of the 1.5B shape -- is PC_ERR_INVALID_ARG (nothing launched).
 * Every call on a GPU, from any context, uses that GPU's one array: calls that overlap in time on
 * different streams race; order them.  Nothing in the array has to survive between calls. */
pc_status pc_decode_step_static(pc_ctx *ctx, const int32_t *seq, const int32_t *tokens_in, int32_t n,
                                float *logits, void *stream);

/* Releases sequences (kind 0) or prompts (kind 1); ids is host int32 [n].
 * Shared blocks are freed when their last user goes. */
pc_status pc_release(pc_ctx *ctx, const int32_t *ids, int32_t n, int32_t kind);

/* Teacher-forced scoring: log pi_theta(o_t | q, o_<t) for every completion
 * token of S given sequences (Section 3.1: a rollout's probability is the
 * product of these; Eq. 2's importance ratio is a ratio of them under two
 * policies), at the given temperature.
 *   tokens      device int32: the sequences (prompt, then completion), packed
 *   cu_lens     host int32 [S+1]: sequence i is tokens[cu_lens[i] .. cu_lens[i+1])
 *   prompt_len  host int32 [S]: the first prompt_len[i] >= 1 tokens of sequence
 *               i are its prompt; its completion is the rest
 *   logprob_out device fp32, packed in sequence order: len_i - prompt_len[i]
 *               values for sequence i
 * Same limits as pc_prefill_shared (a sequence fits max_ctx and
 * max_batch_rows).  Uses KV blocks and slots while it runs and gives them
 * back; the first call allocates a logits buffer (and synchronises once).
 * PC_ERR_OOM if blocks or slots run out: nothing is kept. */
pc_status pc_score(pc_ctx *ctx, const int32_t *tokens, const int32_t *cu_lens, const int32_t *prompt_len,
                   int32_t S, float temperature, float *logprob_out, void *stream);

/* Samples one token per row: o_t ~ softmax(logits / temperature)
 * (Section 3.1 sampling; Section 4.2: temperature 1.0, top_p 1.0), by inverse
 * CDF with a Philox4x32-10 uniform keyed by (seed; step, sequence uid).
 *   logits      device fp32 [*, vocab]
 *   logit_row   device int32 [n] or NULL: row of `logits` that output row i
 *               reads (NULL: row i).  Lets G rollouts share a prompt's row.
 *   seq_uid     device uint64 [n]
 *   step        device int32 [n] or NULL; row i uses step_base + step[i]
 *   eos_id      -1 = none; eos_logit_bias is added to that id's scaled logit
 *   tokens_out  device int32 [n]
 *   logprob_out device fp32 [n] or NULL: log-probability of the sampled token
 *   finished    device uint8 [n] or NULL, in/out: set when eos_id is sampled;
 *               a row already finished on entry yields eos_id and logprob 0.
 *   top_p       in (0, 1]: nucleus sampling (Section 4.2 names top_p = 1.0 for
 *               training).  Below 1 only the smallest set of tokens whose
 *               probability mass reaches top_p is sampled from: tokens in
 *               order of decreasing probability (ties: lower id first) until
 *               their cumulative mass is >= top_p; the inverse CDF then runs
 *               over the kept tokens in id order, and logprob_out is the
 *               log-probability under the renormalised kept set.
 *   hist_tokens, hist_logprob  device [>= max index + 1] or NULL: second
 *               destinations of the token / log-probability of row i, at index
 *               hist_index[i] (device int32 [n]; NULL: index i).  Lets a
 *               caller keep a [step][sequence] history without a copy kernel
 *               per step while its decode batch shrinks. */
pc_status pc_sample(const float *logits, const int32_t *logit_row, int32_t n, int32_t vocab,
                    float temperature, float top_p, uint64_t seed, const uint64_t *seq_uid, const int32_t *step,
                    int32_t step_base, int32_t eos_id, float eos_logit_bias, int32_t *tokens_out,
                    float *logprob_out, uint8_t *finished, int32_t *hist_tokens, float *hist_logprob,
                    const int32_t *hist_index, void *stream);

/* Per-prompt reward statistics (Eq. 3; Section 3.3 pilot success rate
 * p_hat = (1/n) sum r_j, Var = p(1-p) for binary rewards).
 *   rewards    device fp32 [N]; group_off device int32 [P+1] (ascending offsets)
 *   n_pos      device int32 [P]: number of non-zero rewards
 *   n_tot      device int32 [P]: group size
 *   mean, var  device fp32 [P]: mean and POPULATION variance (divide by the
 *              group size); 0 for an empty group.  Any output may be NULL. */
pc_status pc_group_stats(const float *rewards, const int32_t *group_off, int32_t P, int32_t *n_pos,
                         int32_t *n_tot, float *mean, float *var, void *stream);

/* Pilot filter, eviction flags and the commit set (Section 3.3; Algorithm 1).
 *   p_hat       device fp32 [P], in batch order
 *   cls         device uint8 [P]: 0 too hard (p_hat < p_lower), 1 keep,
 *               2 too easy (p_hat > p_upper)
 *   evict       device uint8 [P]: p_hat >= p_solve (independent of cls)
 *   commit_idx  device int32 [P]: the first min(#keep, b_t) kept indices,
 *               ascending (b_t <= 0: no cap); entries past counts[0] untouched
 *   surplus_idx device int32 [P]: the remaining kept indices, ascending
 *   counts      device int32 [4]: n_commit, n_surplus, n_easy, n_hard
 * cls, evict, surplus_idx may be NULL. */
pc_status pc_select_commit(const float *p_hat, int32_t P, float p_lower, float p_upper, float p_solve,
                           int32_t b_t, uint8_t *cls, uint8_t *evict, int32_t *commit_idx,
                           int32_t *surplus_idx, int32_t *counts, void *stream);

/* The pilot filter for rewards that are not binary (Introduction; Section 3.3: "applies to any scalar reward";
 * Section 7 names the extension as open).  The paper gives no rule; this one selects on the pilot group's
 * variance itself, with the asymmetry Section 3.3 argues for: a prompt whose mean reward has not passed
 * mean_pivot is approaching the high-variance regime and needs var >= var_hard, one beyond it is leaving and
 * needs var >= var_easy (>= var_hard in the paper's setting).
 *   mean, var   device fp32 [P]: pilot mean and POPULATION variance, as pc_group_stats returns them
 *   cls         0 too hard (not kept, mean <= mean_pivot), 1 keep, 2 too easy (not kept, mean > mean_pivot)
 *   evict       mean >= mean_solve
 *   everything else as in pc_select_commit.
 * With 0/1 rewards, mean_pivot = 0.5, var_hard = p_lower (1 - p_lower), var_easy = p_upper (1 - p_upper) and
 * p_lower <= 0.5 <= p_upper this is pc_select_commit's filter.  Comparisons are taken in fp32. */
pc_status pc_select_commit_var(const float *mean, const float *var, int32_t P, float var_hard, float var_easy,
                               float mean_pivot, float mean_solve, int32_t b_t, uint8_t *cls, uint8_t *evict,
                               int32_t *commit_idx, int32_t *surplus_idx, int32_t *counts, void *stream);

/* Group-relative advantages A_i = (r_i - mu) / (sigma + eps) (Section 3.1,
 * Eq. 3), one group per kept prompt = its pilot and commit rollouts together
 * (Section 3.3 "Training").  A reward equal to the group mean gives exactly 0.
 *   rewards device fp32 [N]; group_off device int32 [P+1]
 *   adv device fp32 [N]; mu, sigma device fp32 [P] or NULL. */
pc_status pc_advantages(const float *rewards, const int32_t *group_off, int32_t P, float eps, float *adv,
                        float *mu, float *sigma, void *stream);

/* ---------------------------------------------------------------------------
 * Multi-step scheduling (Algorithm 1 with the optimisations of Section 3.4:
 * replay buffer for pilot survivors, maximum pilot-to-commit delay d,
 * eviction of solved prompts from the dataset pool).  Host-side bookkeeping:
 * every pointer below is a HOST pointer, nothing touches the GPU, no stream.
 *
 * One training step t is: one or more pc_sched_pilot calls (one per sampling
 * batch; a second call in the same step is the "second sampling round" of
 * Section 5.4), then one pc_sched_commit call.
 * ------------------------------------------------------------------------- */
typedef struct pc_sched pc_sched;

typedef struct {
    float p_lower, p_upper, p_solve; /* Section 3.3 filter bounds (inclusive), Algorithm 1 eviction threshold (>=) */
    int32_t b_t;                     /* training batch size: prompts committed per step, > 0 */
    int32_t max_delay;               /* d >= 0 (Section 4.2: 4): a survivor of step t0 can be committed at steps t0 .. t0+d */
} pc_sched_config;

#define PC_SCHED_STEP 0            /* t: commits done so far */
#define PC_SCHED_BUFFERED_NOW 1    /* entries waiting in the replay buffer */
#define PC_SCHED_PILOT_BATCHES 2   /* pc_sched_pilot calls */
#define PC_SCHED_PROMPTS_SEEN 3
#define PC_SCHED_BUFFERED 4        /* survivors ever put into the buffer */
#define PC_SCHED_COMMITTED 5
#define PC_SCHED_AGED_OUT 6
#define PC_SCHED_EVICTIONS 7       /* prompts flagged p_hat >= p_solve */
#define PC_SCHED_SHORT_STEPS 8     /* steps that committed fewer than b_t prompts */
#define PC_SCHED_MULTI_ROUND_STEPS 9 /* steps with more than one sampling batch */
#define PC_SCHED_NSTATS 10

pc_status pc_sched_create(const pc_sched_config *cfg, pc_sched **out);
pc_status pc_sched_destroy(pc_sched *s);

/* Pilot outcome of one sampling batch at the current step (Algorithm 1:
 * filter B' = {q : p_lower <= p_hat <= p_upper}, eviction {q : p_hat >=
 * p_solve}, R <- R u B').  Comparisons are taken in fp32, as pc_select_commit
 * takes them.  Survivors enter the buffer in batch order, stamped with t.
 *   prompt_uid  host int64 [n]
 *   tag         host int64 [n] or NULL (then 0): carried with the entry and
 *               handed back on commit / age-out (e.g. the caller's handle of
 *               the stored pilot rollouts and prefix KV)
 *   p_hat       host fp32 [n]
 *   cls, evict  host uint8 [n] or NULL, as in pc_select_commit
 *   counts      host int32 [4] or NULL: buffered, evicted, too easy, too hard */
pc_status pc_sched_pilot(pc_sched *s, const int64_t *prompt_uid, const int64_t *tag, const float *p_hat,
                         int32_t n, uint8_t *cls, uint8_t *evict, int32_t *counts);

/* Commit selection of the current step (Algorithm 1, Commit lines), then the
 * age-out and t <- t+1.  Up to b_t entries leave the buffer: the survivors of
 * the current step first, in batch order (Section 3.4: only a step's excess is
 * buffered, the buffer fills a step that came up short); then older ones,
 * oldest step first, in insertion order.  Entries that could not be committed
 * by step t0+d any more (t+1-t0 > d) are dropped and reported.
 *   uid_out, tag_out  host int64 [b_t]; age_out host int32 [b_t] (t - t0)
 *   n_selected        host int32 [1]
 *   aged_uid_out, aged_tag_out  host int64 [aged_cap] or NULL; n_aged host
 *               int32 [1] or NULL.  If more entries age out than aged_cap
 *               holds the call fails with PC_ERR_INVALID_ARG and changes
 *               nothing (PC_SCHED_BUFFERED_NOW is always enough). */
pc_status pc_sched_commit(pc_sched *s, int64_t *uid_out, int64_t *tag_out, int32_t *age_out,
                          int32_t *n_selected, int64_t *aged_uid_out, int64_t *aged_tag_out, int32_t aged_cap,
                          int32_t *n_aged);

/* out[i] = 1 if prompt_uid[i] has been evicted from the pool (Section 3.4:
 * not sampled again in later epochs).  Host arrays. */
pc_status pc_sched_evicted(const pc_sched *s, const int64_t *prompt_uid, int32_t n, uint8_t *out);

/* out: host int64 [PC_SCHED_NSTATS], indexed by the PC_SCHED_* constants. */
pc_status pc_sched_stats(const pc_sched *s, int64_t *out);

#ifdef __cplusplus
}
#endif
#endif /* PC_H */
