/*
 * rlhf.h -- C ABI of the fused generation + inference stage for one MI355X.
 *
 * The stage is the one the paper's Section 2.1 defines and Section 4 fuses: the Actor
 * generates a response for every prompt (prefill, then one token per decoding step until
 * the termination point), and the Reference, Critic and Reward models each run a forward
 * pass over prompt + response.  Section 4.1's observation is that the dependency between
 * the two stages holds per sample, so a finished sample can be scored while long-tailed
 * samples are still decoding; this library runs the two as streams on one GPU.
 *
 * Conventions
 *   - Every call returns 0 (RLHF_OK) or a negative rlhf_status; rlhf_last_error() then
 *     gives a message owned by the context.  Nothing throws or aborts across this ABI.
 *   - "device" pointers are HIP device memory on the current device; "host" pointers are
 *     ordinary host memory.  Weight tensors are caller-owned and BORROWED: they must stay
 *     alive and unchanged until rlhf_destroy().  Host arrays passed to rlhf_submit() are
 *     copied before it returns.  Result and snapshot buffers are caller-allocated host
 *     arrays filled before the call returns.
 *   - The library owns the paged KV pool, page tables, workspaces and (unless given) its
 *     two HIP streams.  It allocates device memory only in rlhf_create(), in
 *     rlhf_load_weights() when half_weight_copies is set, and for temporaries inside
 *     rlhf_compute_gae().
 *   - One context may be used from one host thread at a time.
 */
#ifndef RLHF_H
#define RLHF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rlhf_ctx rlhf_ctx;

enum rlhf_status {
    RLHF_OK = 0,
    RLHF_EINVAL = -1,  /* bad argument, shape the kernels do not support, id out of range */
    RLHF_ENOMEM = -2,  /* KV pool cannot hold a sample's reservation; allocation failed    */
    RLHF_ESTATE = -3,  /* call out of order (e.g. scoring a sample still generating)       */
    RLHF_EDEVICE = -4, /* a HIP call failed                                                */
    RLHF_ENONFINITE = -5 /* a result of the stage is not finite (rlhf_get_results)         */
};

/* The four models of Section 2.1 ("RLHF models"). */
enum rlhf_role { RLHF_ACTOR = 0, RLHF_REF = 1, RLHF_CRITIC = 2, RLHF_REWARD = 3 };
#define RLHF_ROLE_BIT(r) (1u << (r))

enum rlhf_dtype { RLHF_FP32 = 0, RLHF_BF16 = 1 };

/* Decoder shape shared by the four roles: pre-norm blocks, RMSNorm, rotary embedding on
 * pairs (k, k + head_dim/2), grouped KV heads, SwiGLU MLP, no biases.  dtype is the
 * storage type of the matrices.  The residual stream, norms, softmax and all accumulation
 * are float32 in either case.  With BF16 matrices, the activations fed to the matrix units
 * and the KV cache are IEEE half (2 bytes as well): the bf16 weights convert to half inside
 * the kernels (exactly, for magnitudes of at least 2^-14; smaller ones land on half's subnormal
 * grid, an absolute error below 2^-24), and the 8 times finer rounding of half is what keeps
 * the rounding noise of log-probs, values and rewards near the stated tolerances at 32 layers.
 * There is no scaling: activations beyond half's range (65504) overflow, and a stage whose
 * results are not finite reports RLHF_ENONFINITE.
 * Requirements: head_dim in {64, 128}; d_model, ffn multiples of 8; n_q_heads a multiple
 * of n_kv_heads. */
typedef struct rlhf_model_cfg {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    int32_t dtype;                 /* rlhf_dtype */
    float rms_eps, rope_base;
} rlhf_model_cfg;

/* Engine limits.  kv_pool_bytes is the budget "C" of Section 4.2's memory constraint; a
 * sample reserves ceil((prompt + max_new) / page_tokens) pages on admission ("M"), unless
 * optimistic_admission is set. */
typedef struct rlhf_engine_cfg {
    int32_t page_tokens;           /* tokens per KV page; must be 16                          */
    int64_t kv_pool_bytes;         /* device bytes for the paged KV pool                      */
    int32_t max_samples;           /* upper bound on samples per rlhf_submit()                */
    int32_t max_ctx;               /* upper bound on prompt + max_new of any sample           */
    int32_t max_active;            /* decode batch limit (rows of the decode workspace)       */
    int32_t max_batch_tokens;      /* rows of one prefill / scoring pass; >= max_ctx          */
    int32_t eos_id;                /* termination token                                       */
    int32_t stop_on_eos;           /* 1: a sample also ends when it emits eos_id (costs one
                                      device->host copy per step); 0: length-driven only     */
    int32_t corun_decode_cus;      /* > 0: while scoring work is in flight inside rlhf_run_stage,
                                      decode steps are issued on a stream whose CU mask holds
                                      this many compute units (bits from the low end) and
                                      scoring on a stream with the remaining ones, so that the
                                      bandwidth-bound and the matrix-bound work do not queue
                                      behind one another; whichever side is alone uses the whole
                                      chip.  0 = no partition.  Needs a multiple of 32          */
    int32_t optimistic_admission;  /* 0: a sample is admitted when its reservation at the cap fits
                                      (never preempted).  1: admission on present need: the head
                                      of the queue is admitted while the pages for the rows it
                                      (re)builds plus one token fit in what is free and, unless
                                      nothing is running, one more free page is left per running
                                      sample; when a step's decode needs more pages than are
                                      free, the most recently admitted unfinished samples are
                                      preempted (rlhf_migrate to the head of the queue, in
                                      admission order) until it fits                            */
    void* decode_stream;           /* hipStream_t to use, or NULL: the library creates one    */
    void* score_stream;            /* hipStream_t to use, or NULL                             */
    int32_t half_weight_copies;    /* 1 (bf16 models): rlhf_load_weights also makes an IEEE-half
                                      copy of every matrix (library-owned device memory, as many
                                      bytes again as the bf16 weights; RLHF_ENOMEM if they do not
                                      fit beside the KV pool), which the prefill / scoring passes
                                      read instead: both GEMM operands then go from memory straight
                                      into LDS with no conversion in the loop.  Results are
                                      bit-identical either way (the on-the-fly conversion yields
                                      the same half values).  0: no copies                       */
} rlhf_engine_cfg;

/* One role's tensors (device pointers, element type per rlhf_model_cfg.dtype except the
 * norm gains, which are float32).  Row-major, last index contiguous:
 *   embed      [vocab, d_model]
 *   wqkv       [n_layers, (n_q_heads + 2 n_kv_heads) * head_dim, d_model]  Q rows, K rows, V rows
 *   wo         [n_layers, d_model, n_q_heads * head_dim]
 *   w_gate_up  [n_layers, 2 * ffn, d_model]                                gate rows, up rows
 *   w_down     [n_layers, d_model, ffn]
 *   g_attn, g_mlp [n_layers, d_model] float32;  g_final [d_model] float32
 *   head       ACTOR/REF: LM head [vocab, d_model]; CRITIC/REWARD: one row [1, d_model]
 * y = W x for every matrix (rows are outputs). */
typedef struct rlhf_weights {
    const void* embed;
    const void* wqkv;
    const void* wo;
    const void* w_gate_up;
    const void* w_down;
    const float* g_attn;
    const float* g_mlp;
    const float* g_final;
    const void* head;
} rlhf_weights;

typedef struct rlhf_step_info {
    int32_t step;                  /* index of the step just run (0-based)                    */
    int32_t n_admitted;            /* samples admitted and prefilled at the top of the step   */
    int32_t n_prefill_tokens;
    int32_t n_decoded;             /* rows of the decode batch                                */
    int32_t n_active;              /* active-array length after the step (before retire)      */
    int32_t n_preempted;           /* samples preempted before the decode (optimistic admission) */
} rlhf_step_info;

typedef struct rlhf_stage_opts {
    int32_t fused;                 /* 1: score retired samples on the score stream while
                                      decoding goes on (Section 4); 0: generate everything,
                                      then score (the serial plan of Figure 4, top); 2: the
                                      library chooses: the serial plan when a decode step of this
                                      model is bound by kernel launches rather than by streaming
                                      its weights (small models, where a second stream has nothing
                                      idle to fill), else the fused one; rlhf_stage_stats.fused_used
                                      tells which                                               */
    int32_t R_t;                   /* Section 4.2 trigger: scoring is enabled once the number
                                      of samples still in generation is below R_t.  R_t >
                                      n_samples enables it from the first retirement          */
    int32_t score_chunk_tokens;    /* a scoring batch holds at most this many prompt+response
                                      tokens (and at least one sample): it closes when the next
                                      retired sample would not fit, or when generation ends.
                                      A multiple of 256 close to max_batch_tokens keeps the
                                      passes' 256-row GEMM tiles full                         */
    uint32_t role_mask;            /* roles to score: bits REF, CRITIC, REWARD, and ACTOR to
                                      re-score the Actor's log-probs by a full forward        */
    int32_t* trace_active;         /* optional host arrays, trace_cap entries: per step the   */
    int32_t* trace_decoded;        /*   active count after retire, the decode rows, and the   */
    float* trace_step_ms;          /*   decode-stream time of the step (adds two events/step) */
    int64_t* trace_step_bytes;     /*   algorithmic bytes of the step's decode (weights + KV) */
    int32_t* trace_prefill_tokens; /*   prompt tokens prefilled at the top of the step        */
    int32_t trace_cap;
} rlhf_stage_opts;

typedef struct rlhf_stage_stats {
    int32_t n_steps, n_batches;
    int64_t generated_tokens;      /* sum of output lengths                                   */
    int64_t scored_tokens;         /* sum of prompt+response lengths (counted once)           */
    int64_t prefill_tokens;
    double wall_ms;                /* host wall clock of the whole stage, device drained      */
    double decode_stream_ms;       /* first to last work on the decode stream                 */
    double score_stream_ms;        /* first to last work on the score stream (0 if none)      */
    int64_t decode_weight_bytes;   /* algorithmic bytes: weights read by all decode steps     */
    int64_t decode_kv_bytes;       /*   KV read + written by all decode steps                 */
    int32_t fused_used;            /* the plan that ran: 1 fused, 0 serial                    */
} rlhf_stage_stats;

/* Stage outputs, in sample-id order.  Any pointer may be NULL to skip it. */
typedef struct rlhf_results {
    int32_t* gen_len;              /* [n]                                                     */
    int64_t* resp_offsets;         /* [n+1] prefix sums of gen_len                            */
    int32_t* tokens;               /* packed by resp_offsets: y_1 .. y_L of each sample       */
    float* lp_actor;               /* packed: Actor log-prob of y_j, captured while decoding  */
    float* lp_actor_rescored;      /* packed: the same by a scoring forward (role ACTOR)      */
    float* lp_ref;                 /* packed: Reference log-prob of y_j                       */
    float* values;                 /* packed: Critic value at the state before y_j            */
    float* reward;                 /* [n] Reward model score at the last token                */
    int64_t packed_capacity;       /* entries available in each packed array                  */
} rlhf_results;

/* Integer state for bit-exact checks of the bookkeeping. */
typedef struct rlhf_snapshot {
    int32_t step, n_samples, n_waiting, n_active, n_retired, n_batches, n_free;
    int32_t reserved_pages, pool_pages, max_pages;   /* max_pages = row stride of page_table */
    int32_t* active;               /* [cap_samples] sample ids in slot order                  */
    int32_t* ctx;                  /* [cap_samples] tokens whose K/V are cached               */
    int32_t* gen_len;              /* [cap_samples]                                           */
    int32_t* n_pages;              /* [cap_samples]                                           */
    int32_t* page_table;           /* [cap_samples * cap_max_pages]                           */
    int32_t* free_list;            /* [cap_pool_pages] stack, top last                        */
    int32_t* retired;              /* [cap_samples] retire order                              */
    int32_t* batch_offsets;        /* [cap_samples + 1] batches tile `retired` in order       */
    int32_t* batch_step;           /* [cap_samples] step after which each batch closed        */
    int32_t cap_samples, cap_max_pages, cap_pool_pages;
} rlhf_snapshot;

/* Create a context: validates shapes, allocates the KV pool, page tables, workspaces and
 * streams.  On failure *out is NULL and the message is available from rlhf_last_error(NULL). */
int rlhf_create(const rlhf_model_cfg* model, const rlhf_engine_cfg* engine, rlhf_ctx** out);
void rlhf_destroy(rlhf_ctx* ctx);
const char* rlhf_last_error(const rlhf_ctx* ctx);

/* Bind one role's weights (borrowed device pointers).  ACTOR is needed to generate; a role
 * must be bound before it is scored. */
int rlhf_load_weights(rlhf_ctx* ctx, int role, const rlhf_weights* w);

/* Queue n samples (ids 0..n-1 in this order) and reset the stage state: empty KV pool,
 * empty active set, no results.  Host arrays:
 *   prompt_tokens packed by prompt_offsets[n+1]; every prompt has >= 1 token
 *   max_new[n]      cap on output length (>= 1); drives the KV reservation
 *   forced_len[n]   or NULL: the sample ends at exactly this output length and its last token
 *                   is replaced by eos_id (the synthetic workloads' termination rule);
 *                   NULL: ends at max_new (or at eos_id when stop_on_eos)
 *   forced_tokens   or NULL: teacher forcing, packed by forced_offsets[n+1] (one entry per
 *                   output index up to the sample's length); -1 leaves the position greedy
 * RLHF_ENOMEM if one sample's reservation alone exceeds the pool. */
int rlhf_submit(rlhf_ctx* ctx, int32_t n, const int32_t* prompt_tokens,
                const int64_t* prompt_offsets, const int32_t* max_new,
                const int32_t* forced_len, const int32_t* forced_tokens,
                const int64_t* forced_offsets);

/* One step of the generation stage (Section 2.1): admit waiting samples while their KV
 * reservation fits, prefill them (first output token), grow page tables, then ONE decoding
 * step over the active set: greedy token (lowest id on ties) and its Actor log-prob per
 * sample.  Work is enqueued on the decode stream; the call does not wait for it unless
 * stop_on_eos.  RLHF_ESTATE if nothing is waiting or active. */
int rlhf_generate_step(rlhf_ctx* ctx, rlhf_step_info* out);

/* Termination test after a step: samples that reached their length (or emitted eos_id)
 * leave the active set in slot order, their pages return to the pool, the survivors are
 * compacted keeping their order, and the leavers join the retired FIFO.  retired_ids (host,
 * capacity >= active count, may be NULL) receives them. */
int rlhf_retire(rlhf_ctx* ctx, int32_t* retired_ids, int32_t* n_retired);

/* Migration of unfinished samples by re-prefill (Section 4.2, "Migration mechanism", the
 * second choice: the KV cache is discarded, only the sample's tokens travel, and the receiver
 * reruns the prefill phase to regenerate the cache).  On one GPU sender and receiver are the
 * same instance: each listed sample gives its pages back to the pool (in reverse page-table
 * order, samples in the order listed), releases its reservation, leaves the active set
 * (survivors keep their order) and re-enters the waiting queue, at its head in the order
 * listed, or at its tail when to_back != 0.  When rlhf_generate_step admits it again, one
 * packed prefill over its prompt and all generated tokens but the newest rebuilds the cache;
 * nothing is emitted, recorded log-probs stay, and the sample takes part in that step's decode.
 * Also usable as preemption: the pages go to whoever is admitted next.
 * ids: host array of n distinct ids of active samples that have not reached their end;
 * otherwise RLHF_EINVAL and nothing changes.  Host bookkeeping only, no device work. */
int rlhf_migrate(rlhf_ctx* ctx, const int32_t* ids, int32_t n, int32_t to_back);

/* Inference stage for n retired samples as one packed batch (Section 2.1): for each role in
 * role_mask one causal forward over prompt + response; REF/ACTOR give the log-prob of every
 * response token, CRITIC a value per response token, REWARD one scalar at the last token.
 * Enqueued on the score stream (on_score_stream != 0), which first waits for the decode
 * stream's work issued so far, or on the decode stream.  Results stay on the device until
 * rlhf_get_results(). */
int rlhf_score(rlhf_ctx* ctx, int32_t n, const int32_t* sample_ids, uint32_t role_mask,
               int32_t on_score_stream);

/* The whole stage: loop {generate_step, retire, form scoring batches, score} until every
 * sample is generated and scored; returns with both streams drained.  fused = 0 is the
 * serial baseline with the same kernels and the same batch rule. */
int rlhf_run_stage(rlhf_ctx* ctx, const rlhf_stage_opts* opts, rlhf_stage_stats* out);

/* Drain both streams, then copy the stage outputs to the caller's host arrays. */
int rlhf_get_results(rlhf_ctx* ctx, rlhf_results* out);

/* Generalized Advantage Estimation over the finished stage's results, computed the way
 * Section 6 ("System optimizations", inference stage) describes: the recursion
 * A_t = delta_t + gamma*lam*A_{t+1} is unrolled along the output length, so that all samples'
 * advantages are ONE matrix multiply A = D U^T, with D the zero-padded [n, L] matrix of
 * delta_t = r_t + gamma*V_{t+1} - V_t (V after the last token = 0) and U[t][s] = (gamma*lam)^(s-t)
 * for s >= t.  The per-token reward is r_t = -kl_coef*(lp_actor_t - lp_ref_t), plus the Reward
 * model's score at the last token.  Needs REF, CRITIC and REWARD to have been scored for every
 * sample.  advantages / returns (= A + V) are host arrays packed like rlhf_results (either may
 * be NULL).  Float32 throughout; allocates and frees its temporaries; waits for both streams. */
int rlhf_compute_gae(rlhf_ctx* ctx, float gamma, float lam, float kl_coef, float* advantages,
                     float* returns, int64_t packed_capacity);

/* Copy the integer bookkeeping state (host-side, no device work). */
int rlhf_debug_snapshot(rlhf_ctx* ctx, rlhf_snapshot* out);

/* Wait for all work enqueued so far on both streams. */
int rlhf_sync(rlhf_ctx* ctx);

/* Measurement hook (for benchmarks, not part of the method): between begin and end, every
 * sample_every-th launch of each kernel class is bracketed by two HIP events on the stream it
 * runs on.  Classes: 0 = projections of the decode step (weight-streaming, HBM-bound regime of
 * Section 4.2), 1 = projections of prefill / scoring passes (Section 2.1 inference forward),
 * 2 = paged decode attention, 3 = packed causal attention.  Bytes and flops are algorithmic:
 * operands read once, results written once, 2 flops per multiply-add.  The event pairs are
 * folded into the sums whenever rlhf_run_stage returns, so any number of stages may run between
 * begin and end and each is sampled alike.  An event bracket measures from the end of the work
 * queued before the launch on that stream to the end of the launch: with a second stream busy it
 * includes the time the kernel shares the chip with the other stream's kernels.
 * rlhf_profile_end drains both streams and fills out[4]. */
typedef struct rlhf_kernel_profile {
    int64_t launches;              /* launches of the class between begin and end             */
    int64_t sampled;               /* of which were timed                                     */
    double sampled_ms;             /* summed event time of the timed launches                 */
    double sampled_bytes;          /* algorithmic bytes of the timed launches                 */
    double sampled_flops;
    double total_bytes;            /* algorithmic bytes of all launches                       */
    double total_flops;
    int64_t dropped;               /* launches due for timing that found every event pair of the
                                      running stage in use (65536 per stage): raise sample_every */
    double bracket_overhead_ms;    /* what an event bracket costs beyond the kernels inside it
                                      (launch and signalling latency), measured by
                                      rlhf_profile_begin on the decode stream: twice the median
                                      bracket of one empty kernel minus that of two             */
} rlhf_kernel_profile;
int rlhf_profile_begin(rlhf_ctx* ctx, int32_t sample_every);
int rlhf_profile_end(rlhf_ctx* ctx, rlhf_kernel_profile* out /* [4] */);

#ifdef __cplusplus
}
#endif
#endif /* RLHF_H */
