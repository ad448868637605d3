/*
 * rlgen -- generation hot path of asynchronous online-DPO RLHF on one MI355X (gfx950).
 *
 * The method (paper, Section 3 and Appendix D, Algorithm 1, procedure Generate) spends most of
 * its run time drawing K completions per prompt from the current policy pi_theta at a sampling
 * temperature (0.7 in Appendix A.1-A.3) and needs, for every drawn token, log pi(y_t | x, y_<t):
 * the per-token terms of log pi_theta(y|x) in the Online DPO objective (Section 2.1) and of
 * pi_old in the importance ratio of Appendix B, Eq. 1.  This library is that computation for a
 * GPT-NeoX-shaped (Pythia) or Llama-shaped decoder, written as hand-made HIP kernels.
 *
 * Conventions
 *  - Plain C ABI.  Every pointer is a DEVICE pointer unless its comment says HOST.
 *  - The caller owns all memory, including the workspace.  The library allocates no device
 *    memory (host side it allocates its context, small pinned staging buffers, two internal streams
 *    and a few events); rlgen_destroy frees only that host-side state.
 *  - rlgen_generate / rlgen_score enqueue work on the stream given to the call and return; outputs
 *    are valid once the caller has synchronised that stream.  HOST arrays are read before return.
 *  - One context serves one call at a time (calls on one context must not overlap).
 *  - Every function returns RLGEN_OK (0) or a negative RLGEN_ERR_* code.  A call rejected by host
 *    validation launches nothing and writes nothing.  Conditions only the device can see (a token
 *    id outside [0, vocab), a uniform outside [0, 1)) clamp the value, never read out of bounds,
 *    and set a sticky flag reported by rlgen_status.
 *  - Arithmetic: weights are bf16 values (held in fp16, which represents them exactly in its normal
 *    range); GEMM and attention inputs are fp16; the KV cache is bf16; accumulation, the residual
 *    stream, normalisation statistics, softmax and log-sum-exp are fp32 (fp64 for the CDF scan).
 *    cfg.precise = 1 widens every 16-bit activation and cache entry to a pair of bf16 numbers.
 */
#ifndef RLGEN_H
#define RLGEN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RLGEN_OK                  0
#define RLGEN_ERR_NULL           -1   /* a required pointer is null                         */
#define RLGEN_ERR_BAD_CFG        -2   /* inconsistent or unsupported model configuration    */
#define RLGEN_ERR_BAD_ARG        -3   /* a per-call argument is out of its domain           */
#define RLGEN_ERR_CAPACITY       -4   /* the call exceeds max_seqs / max_kv_tokens / max_seq_len / max_batch_tokens */
#define RLGEN_ERR_WORKSPACE      -5   /* workspace too small or misaligned                  */
#define RLGEN_ERR_UNIMPLEMENTED  -6
#define RLGEN_ERR_DEVICE         -7   /* a HIP call failed, or a device-detected input fault */

#define RLGEN_ARCH_NEOX   0  /* LayerNorm+bias, parallel residual, GELU (erf), biased linears   */
#define RLGEN_ARCH_LLAMA  1  /* RMSNorm, sequential residual, SwiGLU, no biases, grouped KV heads */

#define RLGEN_DTYPE_F32   0  /* tensors supplied as fp32; rounded to bf16 (nearest even) on load */
#define RLGEN_DTYPE_BF16  1  /* tensors supplied as bf16                                          */

/* Threads: calls on one context must not overlap; different contexts may be used from different
 * threads.  The library reads no environment variables. */
typedef struct rlgen_ctx rlgen_ctx; /* opaque */

typedef struct {
  int32_t arch;            /* RLGEN_ARCH_*                                                     */
  int32_t n_layers;
  int32_t d_model;         /* = n_q_heads * head_dim; multiple of 32                            */
  int32_t n_q_heads;
  int32_t n_kv_heads;      /* divides n_q_heads; = n_q_heads for NeoX                            */
  int32_t head_dim;        /* multiple of 16, at most 256                                        */
  int32_t d_ffn;           /* multiple of 32                                                     */
  int32_t vocab;
  int32_t rotary_dim;      /* even, <= head_dim: first rotary_dim dims of each head are rotated  */
  float   rope_theta;      /* 10000 for the Pythia shapes, 500000 for the Llama-3.1 shape        */
  float   norm_eps;
  int32_t weight_dtype;    /* RLGEN_DTYPE_*: element type of every tensor in rlgen_weights       */
  int32_t max_seqs;        /* capacity: sequences alive in one call (prompts * k)                */
  int32_t max_seq_len;     /* capacity: longest prompt_len + max_new, or scored sequence         */
  int64_t max_kv_tokens;   /* capacity: sum over sequences of (prompt_len + max_new) rounded up
                              to a multiple of 32                                                */
  int32_t max_batch_tokens;/* rows processed at once by prefill / score; >= max_seq_len;
                              0 selects a default (32768, or max_seqs * max_seq_len if smaller)      */
  int32_t share_prompt_kv; /* 0: every sequence owns a contiguous cache holding prompt and new tokens.
                              1: rlgen_generate stores a prompt's keys/values once and its k samples
                              read them together (the k samples of a prompt condition on the same
                              prefix: Section 2.1, Section 4.2); results are the same up to rounding
                              order.  Then k * (n_q_heads / n_kv_heads) <= 16 is required and the
                              max_kv_tokens need is sum over prompts of round32(prompt_len) +
                              prompts * k * round32(max_new).  rlgen_score is unaffected.        */
  int32_t precise;         /* 0: the formats of the Conventions above (fp16 matrix-product inputs, bf16 cache).
                              1: every 16-bit activation and every cached key and value is held as the sum of
                              two bf16 numbers (16 significant bits, fp32's exponent range), the queries stay
                              fp32, the weights stay the caller's bf16 values, and each matrix product runs once
                              per half on the bf16 matrix instructions.  For checking a policy against an fp32
                              reference where the 16-bit formats themselves exceed the tolerance (random
                              Llama-shaped weights amplify every rounding: Appendix A.2's model shape); it
                              doubles the cache, the activation buffers and the matrix work.  Requires
                              rotary_dim % 4 == 0 and head_dim <= 128.                              */
} rlgen_model_cfg;

/* Per-layer tensors, row-major, linear layers stored [out, in] and applied as y = W x + b.
 * Pointers marked (NeoX) are null for Llama and vice versa. */
typedef struct {
  const void *norm1_g, *norm1_b;  /* [d]; _b (NeoX)                                     */
  const void *norm2_g, *norm2_b;  /* [d]; _b (NeoX)                                     */
  const void *wq, *wk, *wv;       /* [Hq*h, d], [Hkv*h, d], [Hkv*h, d]                  */
  const void *bq, *bk, *bv;       /* (NeoX)                                             */
  const void *wo, *bo;            /* [d, Hq*h]; bo (NeoX)                               */
  const void *w_up, *b_up;        /* [F, d]; b_up (NeoX)                                */
  const void *w_gate;             /* [F, d] (Llama)                                     */
  const void *w_down, *b_down;    /* [d, F]; b_down (NeoX)                              */
} rlgen_layer_weights;

typedef struct {
  const void *embed_in;                      /* [V, d]                                    */
  const void *final_norm_g, *final_norm_b;   /* [d]; _b (NeoX)                            */
  const void *lm_head;                       /* [V, d], no bias, not tied to embed_in     */
  const rlgen_layer_weights *layers;         /* HOST array of n_layers entries            */
} rlgen_weights;

/* Bytes of workspace rlgen_create needs for this configuration (its private 16-bit copy of the
 * weights, the KV cache, activations and sampler partials), or 0 if cfg is null or invalid. */
size_t rlgen_workspace_bytes(const rlgen_model_cfg *cfg);

/* Builds a context for one policy (Algorithm 1: procedure Generate starts by loading the current
 * parameters theta_i into the generation model).
 * cfg, weights: HOST structs holding DEVICE tensor pointers.  workspace: DEVICE, 256-byte aligned,
 * at least rlgen_workspace_bytes(cfg); it must stay alive, and must not be written by the caller,
 * until rlgen_destroy.  The weight tensors are converted/copied on `hip_stream` (a hipStream_t, or
 * null for the default stream); once that stream has been synchronised the library no longer reads
 * them.  *out receives the context.  Errors: NULL, BAD_CFG, WORKSPACE, DEVICE.
 * Creation also times the tile shapes of every linear layer at this configuration's row counts (on
 * `hip_stream` and two internal streams, a few hundred launches, 1-3 s at the 2.8B shape) and
 * synchronises with them, so it must not be called under stream capture.  Timing chooses tile shapes
 * only: how a linear layer's sum over its inner dimension is cut and ordered is a fixed function of
 * the configuration, so two contexts of one configuration return the same bits whatever they picked. */
int rlgen_create(const rlgen_model_cfg *cfg, const rlgen_weights *weights, void *workspace,
                 size_t workspace_bytes, void *hip_stream, rlgen_ctx **out);

/* Replaces the policy's weights in place with a new theta_i of the same shape (Algorithm 1,
 * procedure Generate, first step; Appendix A.2 notes that this hand-off blocks the learner). */
int rlgen_update_weights(rlgen_ctx *ctx, const rlgen_weights *weights, void *hip_stream);

/* y ~ pi_theta(. | x): k completions of exactly max_new tokens per prompt by inverse-CDF sampling
 * from softmax(z / temperature), plus the log-probability of each emitted token under that same
 * distribution (Section 2.1; Algorithm 1, procedure Generate; temperature: Appendix A.1).
 *
 *  prompts        [B, prompt_stride] int32, right-padded; cells at or beyond prompt_lens[b] are never read
 *  prompt_lens    HOST [B] int32, each >= 1
 *  uniforms       [B, k, max_new] fp32 in [0, 1): the random numbers of the draw.  Token t of sample
 *                 (b, j) is the first vocabulary index whose cumulative probability, accumulated in
 *                 ascending index order, exceeds uniforms[b, j, t] (if rounding leaves none, the last
 *                 index with positive probability)
 *  forced         nullable [B, k, max_new] int32: an entry >= 0 replaces the drawn token (used by
 *                 parity tests to keep two implementations on one trajectory); its log-prob is reported
 *  tokens         out [B, k, max_new] int32
 *  token_logprobs out [B, k, max_new] fp32 = log softmax(z / temperature)[token]
 *
 * The k samples of one prompt share one prompt pass.  Errors: NULL, BAD_ARG (B, k, max_new < 1,
 * prompt_len < 1, prompt_stride < max prompt_len, temperature not finite or < 0, or with
 * share_prompt_kv k * (n_q_heads / n_kv_heads) > 16), CAPACITY, DEVICE.
 *
 * temperature == 0 decodes greedily (the evaluation protocol of Section 5.2): every token is the
 * first index of the largest logit, uniforms are not read (but must be non-null), and
 * token_logprobs = log softmax(z)[token].
 * With an EOS token set (rlgen_set_eos) a completion ends at its first EOS: the entries after it
 * hold the EOS id at log-prob 0 (forced entries after it are ignored); rlgen_set_eos says what then
 * happens to the ended sequence's place in the batch. */
int rlgen_generate(rlgen_ctx *ctx, const int32_t *prompts, const int32_t *prompt_lens, int32_t B,
                   int32_t prompt_stride, int32_t k, int32_t max_new, float temperature,
                   const float *uniforms, const int32_t *forced, int32_t *tokens,
                   float *token_logprobs, void *hip_stream);

/* Teacher-forced log-probabilities, the terms of log pi(y | x) in the DPO objective (Section 2.1)
 * and of the ratio in Appendix B, Eq. 1:
 *   out[n, t] = log softmax(z_{t-1} / temperature)[seqs[n, t]]   for max(1, score_from[n]) <= t < seq_lens[n]
 *   out[n, t] = 0                                                 elsewhere in [0, stride)
 *  seqs [N, stride] int32 right-padded; seq_lens HOST [N]; score_from HOST [N] or null (= 1).
 * Errors: NULL, BAD_ARG, CAPACITY, DEVICE. */
int rlgen_score(rlgen_ctx *ctx, const int32_t *seqs, const int32_t *seq_lens,
                const int32_t *score_from, int32_t N, int32_t stride, float temperature,
                float *token_logprobs, void *hip_stream);

/* Raw (temperature 1) logits at the last position of each sequence, [N, vocab] fp32.  The product
 * path never writes logits to memory; this entry point exists so that tests can bound them. */
int rlgen_debug_logits(rlgen_ctx *ctx, const int32_t *seqs, const int32_t *seq_lens, int32_t N,
                       int32_t stride, float *logits, void *hip_stream);

/* The final-norm + LM-head + sampling stage alone (the last line of procedure Generate applied to
 * given residual rows): hidden [R, d] fp32, uniforms [R], forced nullable [R] -> tokens [R],
 * token_logprobs [R].  R <= max_batch_tokens. */
int rlgen_debug_sample(rlgen_ctx *ctx, const float *hidden, int32_t R, float temperature,
                       const float *uniforms, const int32_t *forced, int32_t *tokens,
                       float *token_logprobs, void *hip_stream);

/* rlgen_debug_sample for callers that cannot allocate or hand over scratch memory at the time of the call: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same results;
 * the stage's intermediate buffers (the normalised rows, the per-row per-64-column softmax partials) live in a static
 * device array of the library (about 4.3 MB per GPU, held until the process ends) instead of the context's workspace,
 * so the call does not touch the workspace's activation buffers.  It allocates nothing, on the host or the device.
 * Limits: R <= 64 rows, d_model <= 8192, vocab <= 262144; beyond them RLGEN_ERR_CAPACITY.  The device the context was
 * created on must be current.  All calls on one GPU, from any context, share the one array: calls that overlap in time
 * on that GPU (different streams or contexts) race; calls on one stream are ordered.  Nothing in the array needs to
 * start at zero: every element a call reads it has written itself.
 * Errors: NULL, BAD_ARG, CAPACITY, DEVICE. */
int rlgen_sample_static(rlgen_ctx *ctx, const float *hidden, int32_t R, float temperature,
                        const float *uniforms, const int32_t *forced, int32_t *tokens,
                        float *token_logprobs, void *hip_stream);

/* Consumers of the log-probs (Section 2.1, DPO objective).  seq_logprob[n] = sum of
 * token_logprobs[n, t] over from[n] <= t < lens[n] (from, lens: DEVICE [N] int32). */
int rlgen_sequence_logprob(const float *token_logprobs, const int32_t *from, const int32_t *lens,
                           int32_t N, int32_t stride, float *seq_logprob, void *hip_stream);
/* loss[p] = -log sigmoid(beta * ((pol_pos[p] - ref_pos[p]) - (pol_neg[p] - ref_neg[p]))), all [P] fp32. */
int rlgen_dpo_loss(const float *pol_pos, const float *ref_pos, const float *pol_neg,
                   const float *ref_neg, int32_t P, float beta, float *loss, void *hip_stream);

/* Proximal RLOO, the off-policy baseline the paper compares Online DPO with (Appendix B, Eq. 1): for each of
 * a prompt's k >= 2 completions, objective = min(r A, clip(r, 1 - epsilon, 1 + epsilon) A) with
 * r = exp(pol_logprob - old_logprob) (pi_theta over the generating policy pi_old, both sequence log-probs as
 * rlgen_sequence_logprob returns them) and A = the completion's reward minus the mean reward of the prompt's
 * other k - 1 completions (at k = 2, the other completion's reward, as the appendix writes it).
 * pol_logprob, old_logprob, rewards, objective: DEVICE [B, k] fp32.
 * Errors: NULL, BAD_ARG (B < 1, k < 2, epsilon negative or not finite), DEVICE. */
int rlgen_proximal_rloo(const float *pol_logprob, const float *old_logprob, const float *rewards, int32_t B,
                        int32_t k, float epsilon, float *objective, void *hip_stream);

/* Which two of a prompt's k completions are trained on (Section 2.1: the two samples ranked by reward;
 * Section 4.2: of K = 4 samples the highest and the lowest rewarded).  rewards [B, k] fp32 (the caller's
 * reward model; no NaN), idx_pos / idx_neg [B] int32 out, all DEVICE: idx_pos[b] = first index of the
 * maximum, idx_neg[b] = last index of the minimum (so they differ whenever k >= 2).
 * Errors: NULL, BAD_ARG (B or k < 1), DEVICE. */
int rlgen_select_pairs(const float *rewards, int32_t B, int32_t k, int32_t *idx_pos, int32_t *idx_neg,
                       void *hip_stream);

/* Per-phase device times of the last rlgen_generate / rlgen_score on this context, in ms (any
 * pointer may be null).  Synchronises the events it reads.  decode_attn_ms / decode_attn_launches
 * cover the decode-attention kernel alone and are filled only while profiling is on:
 * rlgen_set_profiling(ctx, n) with n >= 1 brackets every n-th decode-attention launch (rotating
 * over the layers from step to step) with events on the call's stream; decode_attn_ms is the sum
 * over the decode_attn_launches bracketed launches.  Each bracketed launch costs about 10 us. */
int rlgen_get_timings(rlgen_ctx *ctx, float *prefill_ms, float *decode_ms, float *decode_attn_ms,
                      int32_t *decode_attn_launches);
int rlgen_set_profiling(rlgen_ctx *ctx, int32_t on);

/* The token id that ends a completion in later rlgen_generate calls on this context (the paper's
 * completions end in an EOS token or are penalised for lacking one: hyper-parameter tables of
 * Appendix A.1 and A.2); -1 (the default) = none.  With an EOS id set and one cache per sequence
 * (share_prompt_kv = 0), rlgen_generate drops ended sequences from the batch: every 8 decode steps
 * it WAITS for the stream, reads which sequences have ended, fills the rest of their outputs and
 * continues with the others (and returns early once none is left), so the call is no longer purely
 * asynchronous.  With share_prompt_kv = 1 ended sequences stay in the batch and only stop reading
 * their cache.  The outputs are the same either way.
 * Errors: NULL, BAD_ARG (id outside [-1, vocab)). */
int rlgen_set_eos(rlgen_ctx *ctx, int32_t eos_token);

/* The sequences a learner scores come in groups: a prompt x and its k completions (the pair y+, y-
 * of the DPO objective, Section 2.1; K = 4 in Section 4.2).  After rlgen_set_score_groups(ctx, k),
 * k > 1, rlgen_score requires N to be a multiple of k, score_from non-null and equal within every
 * group of k consecutive sequences (1 <= score_from <= seq_len), and takes the caller's word that
 * the group's sequences agree in their first score_from tokens: that shared part then goes through
 * the model once per group instead of once per sequence.  Outputs are the same as without grouping
 * up to rounding order.  The agreement is checked on the device; a group that breaks it sets the
 * sticky status (rlgen_status returns DEVICE) and its log-probs are meaningless.  k = 1 (the
 * default) scores every sequence on its own.  A call falls back to scoring every sequence on its
 * own when a group does not fit one chunk of max_batch_tokens rows, or when rotary_dim is not a
 * multiple of 4.  Errors: NULL, BAD_ARG (k < 1). */
int rlgen_set_score_groups(rlgen_ctx *ctx, int32_t k);

/* rlgen_generate decodes a batch of 256 or more sequences as two halves on two internal streams
 * (forked from and joined to the call's stream), so that one half's cache-streaming attention runs
 * beside the other half's linear layers.  on = 0 turns that off for later calls on this context
 * (every kernel then runs alone on the call's stream, which is what a per-kernel measurement
 * needs); on != 0 turns it back on.  Results do not depend on it. */
int rlgen_set_decode_split(rlgen_ctx *ctx, int32_t on);

/* ended sequences leave the batch every `every` decode steps (default 8; 0: never, they stay in the batch and
 * only stop reading their cache).  Outputs do not depend on it.  Errors: NULL, BAD_ARG (every < 0). */
int rlgen_set_eos_compaction(rlgen_ctx *ctx, int32_t every);

/* min_seqs >= 2 replaces the 256-sequence threshold of the two-stream decode together with its criterion that a
 * step's cache traffic must outweigh the weights four times (tests use it to send small batches down that path);
 * 0 restores the default.  Results do not depend on it.  Errors: NULL, BAD_ARG. */
int rlgen_set_decode_split_min(rlgen_ctx *ctx, int32_t min_seqs);

/* The tile shape (`variant`, an index into the library's list of GEMM tilings) and the K split the context uses for
 * linear layer `which` (0 QKV, 1 attention output, 2 FFN up, 3 FFN down, 4 LM head) in `mode` (0: decode of the whole
 * batch, 1: prompt pass and scoring, 2: decode of half a batch).  variant -1 = chosen per call from the problem size.
 * rlgen_debug_set_gemm replaces the tile shape (testing and measurement); the K split cannot be set: it is a function
 * of the configuration.  Errors: NULL, BAD_ARG (mode, which or variant out of range, or a tile shape this layer's
 * epilogue does not support). */
int rlgen_debug_get_gemm(rlgen_ctx *ctx, int32_t mode, int32_t which, int32_t *variant, int32_t *splits);
int rlgen_debug_set_gemm(rlgen_ctx *ctx, int32_t mode, int32_t which, int32_t variant);

/* Synchronises `hip_stream` and returns RLGEN_ERR_DEVICE if a kernel has flagged a device-detected fault since the
 * context was created (sticky), else RLGEN_OK: a token id outside [0, vocab), a uniform outside [0, 1), a score group
 * whose members disagree on their shared part, or an activation beyond the largest finite fp16 value (65504), which
 * the library's fp16 matrix-product inputs cannot hold: such a value is clamped to +-65504, never turned into
 * infinity.  *faults (nullable, HOST) receives the bit set: 1 token id, 2 uniform, 4 score group, 8 fp16 range. */
int rlgen_status(rlgen_ctx *ctx, void *hip_stream);
int rlgen_status_bits(rlgen_ctx *ctx, void *hip_stream, uint32_t *faults);

const char *rlgen_strerror(int code);
void rlgen_destroy(rlgen_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* RLGEN_H */
