/*
 * rollout.h -- C ABI of the MI355X rollout library (librollout.so).
 *
 * The library implements the data-parallel hot path of a PPO-RLHF step as the
 * NeMo-Aligner paper states it: response generation for a batch of prompts,
 * one token per forward pass per sequence over a KV cache held next to the
 * weights (Section 3.2), then log-probabilities of every rollout under the
 * actor and under the frozen reference policy -- the same network with other
 * weights (Section 3.1) -- and the per-token KL penalty term between the two
 * (Section 2.2 step 3; coefficient 0.003 in Section 3.3).
 *
 * Conventions for every call
 *  - Return value 0 (RL_OK) on success, a negative RL_E* code otherwise.  No
 *    call throws or aborts; rollout_last_error() returns thread-local text for
 *    the last failure on the calling thread.
 *  - "dev" pointers are device (HBM) addresses on the current HIP device,
 *    "host" pointers are ordinary host memory.  The caller owns ALL device
 *    memory: weights, KV pool, workspace, inputs and outputs.  The library only
 *    borrows those pointers (they must outlive the context) and owns nothing
 *    but a small host-side state object.  It never allocates device memory.
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All
 *    GPU work of a call is queued on it; calls return without waiting and the
 *    caller synchronises.  Calls on one context must not overlap.
 *  - Model: Llama-style decoder (pre-norm RMSNorm, rotary embedding with
 *    half-split pairing (j, j + head_dim/2), grouped-query attention, SwiGLU
 *    FFN, untied embedding / LM head, no biases).  Weight matrices are row-major
 *    [out_features, in_features] and are applied as y = x * W^T.
 *  - Token ids are int32; log-probs and KL are fp32 whatever the weight dtype.
 */
#ifndef ROLLOUT_H
#define ROLLOUT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    RL_OK = 0,
    RL_EINVAL = -1,        /* bad argument or unsupported configuration */
    RL_ENOMEM_PAGES = -2,  /* KV page pool exhausted */
    RL_ESTATE = -3,        /* call not valid in the context's current state */
    RL_EHIP = -4,          /* a HIP runtime call failed */
    RL_ENOSPACE = -5       /* workspace / pool buffer smaller than required */
};

enum { RL_FP32 = 0, RL_BF16 = 1 };   /* dtype of the weight tensors */

typedef struct rl_ctx rl_ctx; /* opaque */

typedef struct rl_model_cfg {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float rope_base;          /* theta_j = rope_base^(-2j/head_dim) */
    float rms_eps;
    int32_t dtype;            /* RL_FP32: fp32 weights, activations and KV cache.  RL_BF16: bf16 weights;
                                 activations between kernels and the KV cache are fp16 (11-bit significand; pairs
                                 of fp16 values, about 22 bits, in the first layer: see
                                 rollout_set_precise_layers), accumulation and the residual stream fp32 */
    int32_t max_batch;        /* most sequences alive at once */
    int32_t max_seq;          /* longest sequence, prompt + generated tokens */
    int32_t page_tokens;      /* tokens per KV page (16) */
    int32_t max_chunk_tokens; /* most tokens one prefill / scoring pass holds at once; >= max_seq */
    int64_t n_pages;          /* pages in the KV pool (shared by all layers: page p of every layer
                                 belongs to the same sequence) */
} rl_model_cfg;

/* One weight set.  Every pointer is dev unless location says otherwise.  The six
 * per-layer members are HOST arrays of n_layers dev pointers. */
typedef struct rl_weights {
    const void* tok_embed;          /* [vocab, d_model] */
    const void* final_norm;         /* [d_model] */
    const void* lm_head;            /* [vocab, d_model] */
    const void* const* attn_norm;   /* [d_model] */
    const void* const* wqkv;        /* [(n_q_heads + 2 n_kv_heads) head_dim, d_model]: q heads, k heads, v heads */
    const void* const* wo;          /* [d_model, n_q_heads head_dim] */
    const void* const* ffn_norm;    /* [d_model] */
    const void* const* w_gate_up;   /* [2 d_ffn, d_model]: gate rows then up rows */
    const void* const* w_down;      /* [d_model, d_ffn] */
    int32_t location;               /* 0 = device resident.
                                       1 = every tensor pointer above (globals and the entries of the per-layer
                                       arrays) is HOST memory -- pinned (hipHostMalloc) if the transfers are to
                                       overlap with compute.  score_logprobs_kl and score_values stream such a set
                                       layer by layer through `staging`; rollout_set_policy uploads it whole into
                                       `staging`; rollout_init and score_kl_exact want location 0. */
    void* staging;                  /* location 1 only, dev, 256-byte aligned.  For the scoring calls:
                                       rollout_weight_staging_bytes(cfg) bytes, scratch for the duration of the call.
                                       For rollout_set_policy: rollout_weight_resident_bytes(cfg) bytes, owned by the
                                       context while this policy is in use.  Ignored for location 0. */
    size_t staging_bytes;
    void* fp16_copy;                /* optional (NULL = none), device-resident bf16 sets on the tuned path only: a dev
                                       buffer of rollout_weight_shadow_bytes(cfg) bytes, 256-byte aligned, in which the
                                       library keeps an fp16 copy of the bf16 matrices; the GEMMs that can, read the
                                       copy and skip the conversion (same results bit for bit; 3-10 % faster).
                                       POLICY given to rollout_init / rollout_set_policy: owned by the context until it
                                       is destroyed or given another policy; rebuilt by those calls and by
                                       rollout_refresh_policy.
                                       REFERENCE given to score_logprobs_kl / score_kl_exact: filled the first time
                                       the set is seen and reused while the same set (its first layer's QKV matrix)
                                       comes back with the same buffer; the set is taken to be frozen (Section 3.1) --
                                       after changing its values in place call rollout_forget_fp16_copies.  The
                                       context remembers one such set.  Ignored elsewhere. */
    size_t fp16_copy_bytes;
} rl_weights;

typedef struct rl_sample_cfg {
    uint64_t seed;
    float temperature;   /* 0 = greedy arg-max (lowest id on ties); > 0 = inverse-CDF sampling of
                            softmax(z / temperature) in vocabulary order */
    int32_t eos_id;      /* -1 = never stop */
    int64_t seq_id_base; /* sequence b draws uniform U(seed, seq_id_base + b, n) for its n-th token */
} rl_sample_cfg;

/* Bytes the caller must provide as `workspace` / `kv_pool` for this configuration
 * (0 if cfg is NULL or invalid). */
size_t rollout_workspace_bytes(const rl_model_cfg* cfg);
size_t rollout_kv_pool_bytes(const rl_model_cfg* cfg);
/* Bytes of the optional fp16 copy of a device-resident bf16 policy (rl_weights.fp16_copy of the policy): the
 * per-layer matrices and the LM head, i.e. about the size of the policy; 0 for fp32 configurations. */
size_t rollout_weight_shadow_bytes(const rl_model_cfg* cfg);
/* Bytes of a device-resident copy of a whole weight set: rl_weights.staging of a host-resident POLICY given to
 * rollout_set_policy, which uploads the set into it. */
size_t rollout_weight_resident_bytes(const rl_model_cfg* cfg);
/* Bytes of rl_weights.staging for a host-resident weight set (location 1): two layers of weights, one
 * [vocab, d_model] table and the fp32 residual stream of max_batch sequences of max_seq tokens. */
size_t rollout_weight_staging_bytes(const rl_model_cfg* cfg);

/* Create a context that generates with `policy` (Section 3.2: the engine keeps
 * weights, KV cache and activations resident).  workspace and kv_pool are dev
 * buffers of at least the sizes above, 256-byte aligned; their contents are
 * scratch owned by the context until rollout_destroy.  Blocks until the
 * context's tables are initialised.  Errors: RL_EINVAL (NULL, n_q_heads %
 * n_kv_heads != 0, head_dim not 64/128, d_model or d_ffn not a multiple of 64,
 * page_tokens != 16, max_chunk_tokens < max_seq, ...), RL_ENOSPACE, RL_EHIP. */
int rollout_init(const rl_model_cfg* cfg, const rl_weights* policy,
                 void* workspace, size_t workspace_bytes,
                 void* kv_pool, size_t kv_pool_bytes, rl_ctx** out);

/* Start B new sequences (dropping any earlier ones): cache tokens [0, P_b - 1)
 * of every prompt in the paged KV cache and remember the prompt's last token as
 * the next decode input, so that every generated token -- the first included --
 * comes out of one forward pass in rollout_decode_step (Section 3.2).
 * prompt_ids: dev int32 [B, Pmax] row-major, entries at or beyond prompt_len[b]
 * ignored.  prompt_len: host int32 [B], 1 <= P_b <= Pmax.  Errors: RL_EINVAL
 * (B > max_batch, P_b out of range), RL_ENOMEM_PAGES.  Token ids outside
 * [0, vocab) are reported by the next rollout_check. */
int rollout_prefill(rl_ctx* ctx, const int32_t* prompt_ids, const int32_t* prompt_len,
                    int32_t B, int32_t Pmax, void* stream);

/* One forward pass for every live sequence: feed tok_in[b] (dev int32 [B]) or,
 * if tok_in is NULL, the token remembered from the previous step / prefill;
 * append its K/V to the cache; sample the next token into tok_out[b] (dev int32
 * [B], may be NULL) and its temperature-1 log-probability into logp_out[b] (dev
 * fp32 [B], may be NULL).  A sequence that has emitted eos_id keeps emitting
 * eos_id with log-prob 0 and no longer grows its cache.  Errors: RL_ESTATE (no prefill yet), RL_EINVAL
 * (sequence would exceed max_seq), RL_ENOMEM_PAGES. */
int rollout_decode_step(rl_ctx* ctx, const rl_sample_cfg* sample, const int32_t* tok_in,
                        int32_t* tok_out, float* logp_out, void* stream);

/* rollout_prefill followed by G decode steps.  out_ids: dev int32 [B, G];
 * out_len: dev int32 [B] or NULL, tokens generated up to and including the first
 * eos_id (G if none); out_logp: dev fp32 [B, G] or NULL. */
int rollout_generate(rl_ctx* ctx, const rl_sample_cfg* sample,
                     const int32_t* prompt_ids, const int32_t* prompt_len,
                     int32_t B, int32_t Pmax, int32_t G,
                     int32_t* out_ids, int32_t* out_len, float* out_logp, void* stream);

/* Queue mode of rollout_generate (Section 3.2: response lengths vary widely, so generation work is handed
 * out dynamically rather than in fixed batches).  Q prompts, any number; at most max_batch are live at a
 * time.  Prompt q generates until it emits eos_id or has produced gen_limit[q] tokens; its cache pages
 * then go back to the pool and its slot takes the next prompt in line, which is prefilled while the other
 * slots wait.  The host looks at the finished flags every 8 decode steps; a finished sequence is parked
 * meanwhile (no cache growth, no attention).  Row q's tokens and log-probs are exactly those
 * rollout_generate would give it in any batch: it draws U(seed, seq_id_base + q, n) for its n-th token and
 * no kernel mixes rows.
 * prompt_ids: dev int32 [Q, Pmax]; prompt_len, gen_limit: host int32 [Q], 1 <= gen_limit[q] <= Gmax and
 * prompt_len[q] - 1 + gen_limit[q] <= max_seq.  out_ids: dev int32 [Q, Gmax]; out_len: dev int32 [Q]
 * (tokens generated, the eos included); out_logp: dev fp32 [Q, Gmax] or NULL.  Entries past out_len[q]
 * hold eos_id (-1 when there is none) and log-prob 0.  Waits for `stream` between bursts; no sequence
 * stays live afterwards.  Errors: RL_EINVAL, RL_ENOMEM_PAGES (the pool cannot hold max_batch live
 * sequences of these lengths). */
int rollout_generate_queue(rl_ctx* ctx, const rl_sample_cfg* sample,
                           const int32_t* prompt_ids, const int32_t* prompt_len, const int32_t* gen_limit,
                           int32_t Q, int32_t Pmax, int32_t Gmax,
                           int32_t* out_ids, int32_t* out_len, float* out_logp, void* stream);

/* Teacher-forced scoring (the "log-probs calculation" stage, Section 3.1 and the
 * stage tables of Section 3.3).  For every sequence b of length L_b and every
 * t in [1, L_b):  logp[b,t] = log softmax(z_{t-1})[ids[b,t]]  under `policy`
 * and under `reference`;  kl[b,t] = logp_policy - logp_ref on response
 * positions t in [prompt_len[b], L_b), and kl_penalty = kl_coef * kl.  Every
 * other entry of the [B, Lmax] outputs is written as 0.  No [tokens, vocab]
 * array is ever written to memory.
 * ids: dev int32 [B, Lmax]; seq_len, prompt_len: host int32 [B], 1 <= L_b <=
 * min(Lmax, max_seq), 0 <= prompt_len[b] <= L_b.  Outputs: dev fp32 [B, Lmax],
 * any may be NULL.  reference may be NULL (policy pass only; logp_ref, kl and
 * kl_penalty must then be NULL).  Does not touch the KV cache of live sequences.
 * policy may be NULL: the set the context currently generates with (the one given to rollout_init or the last
 * rollout_set_policy, also when that was uploaded from host memory).
 * Either weight set may be host-resident (location 1: "reference weights streamed layer by layer"): its
 * layers are copied into the set's staging buffer on a stream of the library's own, two layers deep,
 * while the previous layer runs on `stream` for all tokens; results are identical to the resident case.
 * Errors: RL_EINVAL, RL_ENOSPACE (staging buffer too small). */
int score_logprobs_kl(rl_ctx* ctx, const rl_weights* policy, const rl_weights* reference,
                      const int32_t* ids, const int32_t* seq_len, const int32_t* prompt_len,
                      int32_t B, int32_t Lmax, float kl_coef,
                      float* logp_policy, float* logp_ref, float* kl, float* kl_penalty,
                      void* stream);

/* Exact per-token KL between the two policies' next-token distributions, in one pass (the sampled term of
 * score_logprobs_kl estimates this quantity from the one token that was drawn):
 *   kl_full[b,t] = sum_v pi_policy(v | ids[b,<t]) * (log pi_policy(v | .) - log pi_ref(v | .))
 * on response positions t in [max(prompt_len[b], 1), L_b); 0 elsewhere.  Both bodies run on each chunk of
 * tokens; then ONE kernel forms both models' logits tile by tile and keeps, per row and column group, five
 * running numbers (max and sum-exp of each model, and the policy-weighted sum of logit differences).
 * Neither model's [tokens, vocab] logits or probabilities are written to memory.
 * Arguments as for score_logprobs_kl; both weight sets device-resident (location 0); kl_full: dev fp32
 * [B, Lmax].  Errors: RL_EINVAL, RL_ENOSPACE. */
int score_kl_exact(rl_ctx* ctx, const rl_weights* policy, const rl_weights* reference,
                   const int32_t* ids, const int32_t* seq_len, const int32_t* prompt_len,
                   int32_t B, int32_t Lmax, float* kl_full, void* stream);

/* Critic values / reward-model scores (Section 2.2 step 2 and Section 3.1: the reward model and the critic
 * are decoders of the actor's kind with a scalar head, served for inference on the rollouts).  The same
 * teacher-forced pass as score_logprobs_kl with a [d_model] -> 1 head in place of the LM head:
 * values[b,t] = value_head . RMSNorm(x_t; final_norm) for t in [0, L_b), the state after reading token t;
 * 0 beyond.  A sequence-level reward is values[b, L_b - 1].
 * model: body weights of this context's shape (lm_head is not read and may be NULL; location 0 or 1);
 * value_head: dev, [d_model] in the weight dtype; ids: dev int32 [B, Lmax]; seq_len: host int32 [B];
 * values: dev fp32 [B, Lmax].  Errors: RL_EINVAL, RL_ENOSPACE. */
int score_values(rl_ctx* ctx, const rl_weights* model, const void* value_head,
                 const int32_t* ids, const int32_t* seq_len, int32_t B, int32_t Lmax,
                 float* values, void* stream);

/* Per-token PPO reward (Section 2.2 step 3: the reward-model score of the rollout regularised by the KL
 * penalty; coefficient 0.003 in Section 3.3): rewards[b,t] = -kl_coef * kl[b,t] on response positions
 * t in [prompt_len[b], L_b), plus seq_reward[b] on the last token t = L_b - 1; 0 elsewhere.
 * kl, rewards: dev fp32 [B, Lmax] (kl as written by score_logprobs_kl); seq_reward: dev fp32 [B];
 * seq_len, prompt_len: host int32 [B].  Errors: RL_EINVAL. */
int ppo_rewards(rl_ctx* ctx, const float* kl, const float* seq_reward,
                const int32_t* seq_len, const int32_t* prompt_len, int32_t B, int32_t Lmax,
                float kl_coef, float* rewards, void* stream);

/* ppo_rewards for callers that cannot allocate device memory or have the runtime copy for them: code that is
 * being recorded into a HIP graph, tight serving loops, harnesses that forbid allocation.  Same arguments and
 * results as ppo_rewards without the context: the lengths travel as kernel arguments into a fixed 32 KB array
 * inside the library (one per GPU, held until the process ends) instead of the context's workspace.  The call
 * allocates nothing, copies nothing and does not wait.  At most 4096 sequences per call (RL_EINVAL beyond).  All
 * calls on one GPU share that array: calls whose GPU work may overlap (different streams) race on it; calls on one
 * stream are ordered and safe.  Errors: RL_EINVAL, RL_EHIP. */
int ppo_rewards_noalloc(const float* kl, const float* seq_reward,
                        const int32_t* seq_len, const int32_t* prompt_len, int32_t B, int32_t Lmax,
                        float kl_coef, float* rewards, void* stream);

/* Wait for `stream` and report device-side findings since the last check:
 * RL_EINVAL if a token id outside [0, vocab) was seen (it was clamped), RL_EHIP
 * if the stream is in error. */
int rollout_check(rl_ctx* ctx, void* stream);

/* Generate with another weight set from now on (Section 3.1 / 3.2: the actor's weights change every PPO
 * step and the generation engine has to pick them up; weight sets that are not in use are kept in host memory
 * and swapped in).  Same shapes and dtype as the context's.  Drops all live sequences -- their caches belong to the
 * old weights -- and the captured decode step.
 *  - location 0 (device-resident set): the library uses weights in place, so this only swaps pointers (values
 *    updated IN PLACE at the same addresses need no call at all, unless the policy has an fp16 copy: then
 *    rollout_refresh_policy).  The caller must have waited for work that uses the old set.  Blocks until the fp16
 *    copy, if any, is rebuilt.
 *  - location 1 (host-resident set, pinned for the copies to be asynchronous): every tensor is copied into
 *    policy->staging (rollout_weight_resident_bytes) on a stream of the library's own and the call returns at once;
 *    work already queued with the old policy keeps running while the upload proceeds (the old set's memory is not
 *    touched, so with two device buffers the next set loads while the current one generates), and every later call
 *    that reads the policy makes its stream wait for the upload.  The host tensors must stay valid until then.
 * Errors: RL_EINVAL, RL_ENOSPACE, RL_EHIP. */
int rollout_set_policy(rl_ctx* ctx, const rl_weights* policy);

/* The policy's values were updated IN PLACE: rebuild the fp16 copy (if the policy came with a buffer for one; the
 * conversion is queued on `stream`) and drop all live sequences.  Without a copy this only drops the sequences.
 * Errors: RL_EINVAL. */
int rollout_refresh_policy(rl_ctx* ctx, void* stream);

/* Forget all sequences and return every page to the pool. */
int rollout_reset(rl_ctx* ctx);
void rollout_destroy(rl_ctx* ctx);
const char* rollout_last_error(void);

/* ---- implementation switches and measurement hooks (not part of the method) ----
 * The switches that change which kernels run (rollout_set_impl, rollout_set_precise_layers,
 * rollout_set_fused_sampling, rollout_set_fused_qkv_consumer) discard the captured decode step: call them only when the work queued on the context
 * has finished (e.g. after rollout_check), never while a rollout_generate is still running on its stream. */

/* impl 0 = plain reference kernels for every step (any dtype);
 * impl 1 = tuned gfx950 kernels where they exist (bf16 MFMA GEMMs, MFMA
 * attention, fused LM-head log-sum-exp).  Default 1 for bf16, 0 for fp32.
 * impl 2 = impl 1, except that the large-M GEMMs take their 256 x 256-tile kernel for every shape it
 * supports instead of only where the grid fills the chip (lets small test shapes reach that kernel).
 * Drops all live sequences (their caches were written by the other kernels). */
int rollout_set_impl(rl_ctx* ctx, int32_t impl);

/* Tuned bf16 path only: the first n layers (0 <= n <= 2, default 1) carry their activations -- GEMM inputs,
 * q, k, v, softmax probabilities, attention output, FFN activation, and their share of the KV cache -- as PAIRS
 * of fp16 values (hi + lo, about 22 significant bits) instead of single fp16 values; their GEMMs and attention
 * take twice / three times the MFMA work.  Rounding in the first layer alone accounts for about nine tenths
 * of the path's log-prob error variance against an unrounded evaluation, so n = 1 buys a three times smaller
 * error for about 3 % more MFMA work at 32 layers.  n = 0 is the plain fp16 path.  Drops all live sequences.
 * Errors: RL_EINVAL (n out of range, or n > 0 on a context that runs the plain kernels). */
int rollout_set_precise_layers(rl_ctx* ctx, int32_t n);

/* Tuned bf16 path only.  on != 0 (default): the LM head of a decode step writes, per row and 32 vocabulary
 * columns, the maximum, its column and two sums of exponentials (Section 3.2's generation step never needs the
 * logits themselves), and the sampler draws from those, recomputing the 32 logits of the one block the draw lands
 * in.  on = 0: the LM head writes fp32 logits [batch, vocab] and the sampler reads them all.  Same rule for the
 * token either way (arg-max with the lowest id on ties; inverse CDF in vocabulary order for the shared uniform);
 * the sums are formed in a different order, so log-probs agree to rounding and a sampled token can differ where the
 * uniform falls within rounding of a CDF step.  The caller must have waited for work on the context.  Takes effect
 * with the next decode step; live sequences are kept.  Errors: RL_EINVAL. */
int rollout_set_fused_sampling(rl_ctx* ctx, int32_t on);

/* Tuned bf16 path only.  on != 0 (default): in a decode step (Section 3.2's generation stage) the attention kernel of
 * a plain layer is itself the consumer of the QKV projection's split-K partial sums: each workgroup adds up the
 * partial rows of its own query heads and of its kv head's new key and value (in split order), applies the rotary
 * embedding, appends key and value to the cache page and attends with them.  on = 0: a separate kernel does that
 * first and attention reads its results.  The arithmetic is the same either way; fp16-pair layers
 * (rollout_set_precise_layers) and models with more than 6 query heads per kv head at head_dim 128 always use the
 * separate kernel.  The caller must have waited for work on the context.
 * Takes effect with the next decode step; live sequences are kept.  Errors: RL_EINVAL. */
int rollout_set_fused_qkv_consumer(rl_ctx* ctx, int32_t on);

/* Forget the fp16 copy the context keeps of a reference set (rl_weights.fp16_copy): the next scoring call that
 * brings one rebuilds it.  For callers that overwrite a reference set's values in place. */
int rollout_forget_fp16_copies(rl_ctx* ctx);

/* Measurement switch (process-wide): decode-step GEMMs of more than `rows` rows run on the 128 x 128 tile kernel
 * instead of the LDS-ring weight streamer (default: a negative value = ring kernel for every batch). */
int rollout_set_decode_tile_rows(int32_t rows);
/* Measurement switch, process-wide: on = 0 makes the large-M GEMMs convert the bf16 weights even where an fp16 copy
 * (rl_weights.fp16_copy) exists; on != 0 (default) lets them read the copy.  Results are the same bit for bit. */
int rollout_set_large_gemm_copy(int32_t on);

/* Kernel classes for timing. */
enum {
    RL_K_GEMM_DECODE = 0,   /* weight-streaming GEMMs of a decode step */
    RL_K_ATTN_DECODE = 1,   /* paged GQA decode attention */
    RL_K_GEMM_PREFILL = 2,  /* large-M GEMMs of prefill / scoring */
    RL_K_ATTN_PREFILL = 3,  /* causal prefill attention */
    RL_K_LMHEAD_SCORE = 4,  /* fused LM head + log-sum-exp + gather */
    RL_K_COUNT = 5
};
/* on = 0: off.  on = n >= 1: every n-th launch of that class is bracketed by HIP
 * events on the launch stream (up to an internal cap of 8192 timed launches
 * between reads; later launches go untimed). */
int rollout_profile_enable(rl_ctx* ctx, int32_t kernel_class, int32_t on);
/* Waits for the recorded events; returns summed milliseconds and launch count,
 * then clears the records.  total_ms / launches: host. */
int rollout_profile_read(rl_ctx* ctx, int32_t kernel_class, double* total_ms, int64_t* launches);
/* What such a bracket reads with nothing inside it: the mean elapsed time of `pairs` (1 .. 4096) back-to-back event
 * pairs recorded on `stream` behind one small kernel, in milliseconds.  A timed launch reads its kernel's duration
 * plus about this much; callers that compare with a tracer's kernel durations subtract it.  Synchronises `stream`.
 * overhead_ms: host. */
int rollout_profile_event_overhead(rl_ctx* ctx, int32_t pairs, double* overhead_ms, void* stream);
/* Instrument for reading the MFMA roofline: the rate (TFLOP/s) at which the matrix cores of this GPU sustain
 * back-to-back fp16 16x16x32 MFMAs (the shape the large-M GEMMs run) on operands held in registers -- no memory
 * traffic, one workgroup of four waves per compute unit, about 0.2 s -- on random operands (random_operands != 0) or
 * on zeros.  Power management makes the two differ by a third; a GEMM on real data cannot run faster than the first
 * figure.  Uses the context's workspace
 * between calls (live sequences are not touched); synchronises `stream`.  tflops: host.
 * Errors: RL_EINVAL, RL_ENOSPACE, RL_EHIP. */
int rollout_probe_mfma_rate(rl_ctx* ctx, int32_t random_operands, double* tflops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ROLLOUT_H */
