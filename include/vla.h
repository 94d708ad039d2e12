/*
 * vla.h — C ABI of the MI355X (gfx950) library for batched Vision-Language-Action policy
 * inference: the GPU work of an Inference Worker in the paper's "Inference-as-a-Service" rollout
 * path (Section 3.2): a batch of observations goes in, discretised action tokens, their per-token
 * behaviour log-probabilities (Section 3.2, Eq. 2: mu_t; Appendix "Token-level Policy
 * Optimization") and the de-tokenised continuous actions come out.
 *
 * Model: decoder-only transformer (pre-norm RMSNorm, rotary embedding on half-split pairs,
 * causal multi-head attention, SwiGLU feed-forward, no biases) over the prefix
 * [visual patch embeddings ; instruction token embeddings], followed by autoregressive decoding
 * of K action tokens.  The output head is the LM head restricted to the rows of the action bins
 * (Appendix "Vocabulary Slimming"): bins are the last n_action_bins vocabulary ids, bin j is id
 * vocab - n_action_bins + j, and the distribution is normalised over the bins only.
 *
 * Conventions
 *   - "device" pointers are HIP device memory on the current device; "host" pointers are ordinary
 *     host memory that is read before the call returns.
 *   - The library never allocates device memory.  The caller owns the weight arena, the KV cache
 *     and the workspace (sizes from vla_query_sizes), binds them once, and keeps them alive and
 *     untouched until vla_destroy.
 *   - Every call that takes `hip_stream` (a hipStream_t, or NULL for the default stream) only
 *     enqueues work on it and returns; results are valid once the caller has synchronised that
 *     stream.  No call synchronises the device.  A context is used from one thread, with calls
 *     ordered on one stream.
 *   - Every function returns VLA_OK or a negative vla_status.  Arguments are validated before
 *     anything is enqueued, so a failing call leaves the context unchanged.  vla_last_error gives
 *     a human-readable description of the last failure on that context.
 *   - Storage dtype (config.dtype): VLA_F32 = IEEE float32 throughout; VLA_BF16 = weights, patch embeddings
 *     and the embedding table are bfloat16 at this boundary.  Inside, the matrix cores are fed in IEEE half
 *     precision: each bf16 weight is re-encoded exactly as f16(w * 2^8) at load time (exact for
 *     2^-25 <= |w| <= 255), activations and the KV cache are half precision (one or two terms, see
 *     vla_precision), accumulation, the residual stream, norm statistics, softmax, log-softmax and the head
 *     are float32.
 */
#ifndef VLA_H
#define VLA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct vla_ctx vla_ctx;

enum vla_dtype { VLA_F32 = 0, VLA_BF16 = 1 };

/* Arithmetic of the VLA_BF16 path (config.precision; ignored for VLA_F32).
 *   VLA_PREC_HIGH  in the first config.two_term_layers layers every activation that feeds a matrix core (the
 *                  normalised rows of both blocks, queries, keys, values, softmax weights, attention output, SwiGLU
 *                  output) and the cached keys / values are carried as two terms hi + lo (about 22 significant
 *                  bits; the cache of those layers takes 1.5x the bytes); the layers after them run with one
 *                  half-precision term.  Rounding errors made in the first layers are amplified by all the
 *                  layers that follow and dominate the logit error; with the default of 4 such layers the
 *                  stated tolerances (logits 2e-2, log-probs 1e-2) hold at 32 layers with a margin of 3.
 *   VLA_PREC_FAST  one half-precision term everywhere: about 5 % faster than the default above, logit error
 *                  about 5x larger (rms 7e-3 / max 3e-2 at 32 layers). */
enum vla_precision { VLA_PREC_HIGH = 0, VLA_PREC_FAST = 1 };

enum vla_status {
  VLA_OK = 0,
  VLA_E_NULL = -1,      /* a required pointer is NULL */
  VLA_E_CONFIG = -2,    /* unsupported or inconsistent vla_config */
  VLA_E_SHAPE = -3,     /* batch / offsets / tensor shapes do not fit the config */
  VLA_E_CAPACITY = -4,  /* max_batch, max_seq or max_prefill_tokens would be exceeded */
  VLA_E_STATE = -5,     /* call out of order (buffers not bound, weights not loaded, no prefill) */
  VLA_E_WEIGHTS = -6,   /* missing, duplicate or mis-shaped tensor in vla_load_weights */
  VLA_E_HIP = -7,       /* a HIP runtime call failed */
  VLA_E_DRAINING = -8   /* refused because a weight update is pending or open (see vla_drain_begin) */
};

/* Serving state of a context with respect to weight updates (vla_get_state). */
enum vla_serving_state { VLA_ACCEPTING = 0, VLA_DRAINING = 1, VLA_UPDATING = 2 };

/* Plain data, copied by vla_create.  Requirements: n_heads * head_dim == d_model; head_dim is 64
 * or 128 for VLA_BF16 (32, 64, 128 or 256 for VLA_F32); d_model a multiple of 128 and d_ffn of 64
 * for VLA_BF16 (d_model a multiple of 4 for VLA_F32); 0 < n_action_bins <= vocab, n_action_bins <= 1024; max_seq counts prefix plus decoded
 * positions of one sequence; max_prefill_tokens bounds the packed prefix tokens of one batch. */
typedef struct {
  int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab, n_action_bins;
  float rope_theta, rms_eps;
  int32_t dtype;              /* enum vla_dtype */
  int32_t max_batch, max_seq;
  int64_t max_prefill_tokens;
  int32_t value_max_steps;    /* rows of the value head's step-embedding table; 0 = no value head */
  int32_t precision;          /* enum vla_precision */
  int32_t two_term_layers;    /* VLA_PREC_HIGH: leading layers with two-term operands; 0 = default (4); values
                               * above n_layers mean all layers; negative values are rejected */
} vla_config;

/* One named tensor handed to vla_load_weights: device pointer, row-major, nn.Linear layout
 * [out_features, in_features] for matrices, dtype = the config's storage dtype. */
typedef struct {
  const char* name;
  const void* dev_ptr;
  int32_t dtype;
  int32_t ndim;
  int64_t shape[4];
} vla_tensor;

/* Context life cycle.  vla_create validates the config and allocates host-side state only. */
int vla_create(const vla_config* cfg, vla_ctx** out);
int vla_destroy(vla_ctx* ctx);
const char* vla_last_error(const vla_ctx* ctx);

/* Bytes the caller must provide (each buffer 256-byte aligned): the weight arena (repacked
 * weights, only the action rows of the head), the KV cache [layer][K|V][slot][head][position][head_dim]
 * in the storage dtype (the position extent is max_seq rounded up to an odd number, which keeps the
 * blocks of different heads on different memory channels), and the activation workspace. */
int vla_query_sizes(const vla_config* cfg, size_t* weight_arena_bytes, size_t* kv_bytes,
                    size_t* workspace_bytes);
int vla_bind_buffers(vla_ctx* ctx, void* weight_arena, void* kv, void* workspace);

/* Copies and repacks the named tensors into the arena (fused QKV, fused gate/up, MFMA fragment
 * order, only the action rows of `lm_head`).  Names: "embed" [V,d]; per layer l
 * "layers.<l>.attn_norm" [d], ".wq" ".wk" ".wv" ".wo" [d,d], ".ffn_norm" [d], ".w_gate" ".w_up"
 * [f,d], ".w_down" [d,f]; "final_norm" [d]; "lm_head" [V,d] or already slimmed [A,d].  All must
 * be present exactly once.  Sources may be freed once the stream has completed.  Calling it again
 * replaces the whole set in place as one step: the copies wait, on the device, for every compute
 * call enqueued before, later compute calls wait for the copies, the version counter goes up and the
 * batch in flight is dropped (its cached keys and values belong to the old weights).  Refused with
 * VLA_E_DRAINING while an update opened by vla_update_begin is not committed. */
int vla_load_weights(vla_ctx* ctx, const vla_tensor* tensors, int32_t n_tensors, void* hip_stream);

/* VLA_BF16 only: the re-encoding of a weight matrix element as f16(w * 2^8) is exact for 2^-25 <= |w| <= 255 (and
 * w = 0); a smaller nonzero value is rounded with an absolute error below 2^-33.  The load kernels check every
 * matrix element; a value above 255 in magnitude, or not finite, is never accepted silently: once the load's
 * device work has completed, every compute call returns VLA_E_WEIGHTS until a
 * whole set is loaded again with vla_load_weights (a partial update does not clear the finding).  Compute calls
 * look at the result without waiting (a call enqueued while the load is still running goes ahead);
 * vla_check_weights waits for the last load / update on the host and returns VLA_OK or VLA_E_WEIGHTS. */
int vla_check_weights(vla_ctx* ctx);

/* Prefill: sequence slot b (0 <= b < B) gets the prefix
 *   [patch_emb rows cu_patch[b] .. cu_patch[b+1]) ; embed[instr_ids[cu_instr[b] .. cu_instr[b+1])]]
 * at positions 0 .. S_b-1; its keys/values are written to the cache and its length is set to S_b.
 *   patch_emb  device, [cu_patch[B], d_model], storage dtype
 *   cu_patch   host,   [B+1] non-decreasing, cu_patch[0] == 0
 *   instr_ids  device, [cu_instr[B]] int32 in [0, vocab)   (may be NULL if cu_instr[B] == 0)
 *   cu_instr   host,   [B+1] non-decreasing, cu_instr[0] == 0
 *   logits_out device, [B, n_action_bins] float32 or NULL: action-bin logits at the last prefix
 *              position of each sequence.
 * Every sequence needs S_b >= 1 and S_b <= max_seq; sum S_b <= max_prefill_tokens. */
int vla_prefill(vla_ctx* ctx, int32_t B, const void* patch_emb, const int32_t* cu_patch,
                const int32_t* instr_ids, const int32_t* cu_instr, float* logits_out,
                void* hip_stream);

/* One decode step for slots 0..B-1 (B = the batch of the last prefill): token_ids (device, [B],
 * absolute vocabulary ids) are embedded and appended at each sequence's current length; returns
 * the action-bin logits for the following token.  VLA_E_CAPACITY if a sequence is full. */
int vla_decode_step(vla_ctx* ctx, int32_t B, const int32_t* token_ids, float* logits_out,
                    void* hip_stream);

/* vla_decode_step for callers that cannot provide or allocate staging memory at call time (code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation): same arguments, same results bit for
 * bit, but the step's GEMM staging (the split-K partial sums of the 16-bit path, the GEMM output of the float32
 * path) lives in a 32 MiB array that is part of the library's device code instead of the bound workspace, and
 * the call allocates nothing.  The step needs 4 * B * max(3 d_model, 2 d_ffn) * 4 bytes (VLA_BF16) or
 * B * max(3 d_model, 2 d_ffn) * 4 bytes (VLA_F32); VLA_E_CAPACITY if that exceeds the array (e.g. the 7B shape
 * fits up to B = 95).  Every context on a GPU shares that GPU's one array: calls that overlap in time on one GPU
 * (two streams, two contexts, two threads) race; calls ordered on one stream do not.  Nothing in the array has
 * to survive between calls and nothing in it is read before this call has written it. */
int vla_decode_step_static(vla_ctx* ctx, int32_t B, const int32_t* token_ids, float* logits_out,
                           void* hip_stream);

/* Whole policy step, all on the device: prefill, then K = n_tokens action tokens chosen one by one
 * (K-1 decode steps), each with its log-probability under the distribution it was chosen from.
 *   temperature  0 => greedy (argmax of the logits, log-prob at temperature 1);
 *                >0 => argmax of logits/temperature + gumbel (Gumbel-max sampling); if gumbel is
 *                NULL the noise is taken as zero.  Exact ties go to the lowest bin.
 *   gumbel       device, [B, K, n_action_bins] float32 or NULL
 *   act_scale, act_offset  device, [action_dim] float32 or NULL (identity): token k belongs to
 *                action dimension k mod action_dim (timestep-major chunk);
 *                action = centre(bin) * scale + offset, centre(j) = -1 + (2j+1)/n_action_bins.
 *   tokens_out   device, [B, K] int32 bin indices in [0, n_action_bins)
 *   logp_out     device, [B, K] float32
 *   actions_out  device, [B, K] float32
 *   logits_out   device, [B, K, n_action_bins] float32 or NULL (for tests)
 * Needs S_b + K <= max_seq for every sequence. */
int vla_policy_step(vla_ctx* ctx, int32_t B, const void* patch_emb, const int32_t* cu_patch,
                    const int32_t* instr_ids, const int32_t* cu_instr, int32_t n_tokens,
                    float temperature, const float* gumbel, const float* act_scale,
                    const float* act_offset, int32_t action_dim, int32_t* tokens_out,
                    float* logp_out, float* actions_out, float* logits_out, void* hip_stream);

/* Value head on the rollout path (Appendix "Value Head Design": action-aware attention pooling).  Needs
 * config.value_max_steps > 0.  vla_load_value_head takes, in the storage dtype, "value.attn_w" [d],
 * "value.attn_b" [1], "value.step_emb" [value_max_steps, d], "value.w1" [d, d] (nn.Linear layout),
 * "value.b1" [d], "value.w2" [d], "value.b2" [1]; all must be present exactly once.
 * vla_policy_step_value is vla_policy_step plus the state value of each observation:
 *   hidden_k = final RMSNorm output at the position that emits action token k (k = 0..K-1);
 *   alpha = softmax_k(attn_w . hidden_k + attn_b);  z = sum_k alpha_k hidden_k;
 *   value = w2 . gelu(w1 (z + step_emb[step_t]) + b1) + b2   (exact erf GELU).
 *   step_t      device, [B] int32 episode step of each observation (clamped to the table)
 *   values_out  device, [B] float32
 * The hidden states are only read: nothing of the value head feeds back into the policy outputs. */
int vla_load_value_head(vla_ctx* ctx, const vla_tensor* tensors, int32_t n_tensors, void* hip_stream);
int vla_policy_step_value(vla_ctx* ctx, int32_t B, const void* patch_emb, const int32_t* cu_patch,
                          const int32_t* instr_ids, const int32_t* cu_instr, int32_t n_tokens,
                          float temperature, const float* gumbel, const float* act_scale,
                          const float* act_offset, int32_t action_dim, const int32_t* step_t,
                          int32_t* tokens_out, float* logp_out, float* actions_out, float* logits_out,
                          float* values_out, void* hip_stream);

/* In-place weight update with an early drain (Appendix "High-Performance NCCL-based Weight
 * Synchronization": the received tensors overwrite the inference weights in place, and a drain signal,
 * sent well before the new parameters are ready, makes the worker stop scheduling new batches, finish
 * what is running and only then switch to receiving).  On this boundary the received tensors are device
 * buffers (what a broadcast leaves on the inference GPU) and "overwrite" re-encodes them into the arena.
 *
 *   state      accepting --vla_drain_begin--> draining --vla_update_begin--> updating --vla_update_commit--> accepting
 *   accepting  every call allowed.
 *   draining   vla_prefill / vla_policy_step(_value) return VLA_E_DRAINING (no new batch); vla_decode_step
 *              and vla_select of the batch in flight still run, so it can be finished.
 *   updating   every compute call returns VLA_E_DRAINING; vla_update_tensors may be called any number of
 *              times, each with any subset of the tensor names of vla_load_weights / vla_load_value_head
 *              (same layouts, each name at most once per call), e.g. one call per received bucket.
 *
 * vla_drain_begin touches host state only and may be repeated.  vla_update_begin (allowed from accepting
 * too) makes `hip_stream` wait on the device for every compute call enqueued so far, so the overwrite can
 * be enqueued at once on a second stream without a host synchronisation, and drops the batch in flight.
 * vla_update_commit records the end of the update on `hip_stream`, adds one to the version and returns it;
 * every later compute call first makes its own stream wait for that point.  Hence no compute call ever
 * reads tensors of two versions, whichever streams are used.  Compute calls themselves are expected on
 * one stream at a time (they share the workspace). */
int vla_get_state(const vla_ctx* ctx, int32_t* state /* enum vla_serving_state */, int64_t* version);
int vla_drain_begin(vla_ctx* ctx);
int vla_update_begin(vla_ctx* ctx, void* hip_stream);
int vla_update_tensors(vla_ctx* ctx, const vla_tensor* tensors, int32_t n_tensors, void* hip_stream);
int vla_update_commit(vla_ctx* ctx, void* hip_stream, int64_t* version_out);

/* All K action rows in one forward pass.  Every sequence is run once over [prefix ; K-1 fed tokens]; row k of
 * the result (k = 0..K-1) is the position that emits action token k: the last prefix position, then the fed
 * positions.  1 <= K <= 64; S_b + K - 1 <= max_seq; the packed prefix tokens plus B*(K-1) <= max_prefill_tokens.
 * Both calls start a new batch (they overwrite the KV cache of slots 0..B-1) and take the prefix arguments of
 * vla_prefill.
 *
 * vla_policy_step_parallel — parallel decoding.  The token-level ratio of Appendix "Token-level Policy
 *   Optimization" conditions every action token on the observation alone; here the K-1 fed positions hold the
 *   fixed token `placeholder_id` (any vocabulary id) instead of sampled tokens, so the K distributions come from
 *   one pass and each token is selected on its own, with the rules and outputs of vla_policy_step ([B, K]
 *   tokens / log-probs / actions, optional logits [B, K, A]).  It equals vla_policy_step run with the placeholder
 *   fed back at every step; for K = 1 the two coincide.
 *
 * vla_score_tokens — learner-side evaluation of stored action tokens (the trainer's twin of the rollout step):
 *   tokens      device, [B, K] int32 bin indices (values outside [0, A) are clamped)
 *   placeholder_id  < 0: autoregressive conditioning, the stored tokens 0..K-2 are fed back, so
 *               logp[b,k] = log pi(a_k | o, a_<k) as vla_policy_step reports it; >= 0: the conditioning of
 *               vla_policy_step_parallel with that placeholder.
 *   logp_out    device, [B, K] float32: log_softmax(logits / temperature)[token] (temperature 0 means 1)
 *   mu_logp     device, [B, K] behaviour log-probabilities, or NULL.  With it:
 *   ratio_out   device, [B, K] or NULL: rho = exp(logp - mu)                     (token-level importance ratio)
 *   weight_out  device, [B, K] or NULL: omega(rho; sigma) * rho with omega = exp(-(log rho / sigma)^2 / 2),
 *               the GIPO coefficient of the advantage (Section 3.3); sigma > 0.
 *   logits_out  device, [B, K, A] or NULL. */
int vla_policy_step_parallel(vla_ctx* ctx, int32_t B, const void* patch_emb, const int32_t* cu_patch,
                             const int32_t* instr_ids, const int32_t* cu_instr, int32_t n_tokens,
                             int32_t placeholder_id, float temperature, const float* gumbel,
                             const float* act_scale, const float* act_offset, int32_t action_dim,
                             int32_t* tokens_out, float* logp_out, float* actions_out, float* logits_out,
                             void* hip_stream);
int vla_score_tokens(vla_ctx* ctx, int32_t B, const void* patch_emb, const int32_t* cu_patch,
                     const int32_t* instr_ids, const int32_t* cu_instr, int32_t n_tokens, const int32_t* tokens,
                     int32_t placeholder_id, float temperature, const float* mu_logp, float sigma,
                     float* logp_out, float* ratio_out, float* weight_out, float* logits_out, void* hip_stream);

/* Continuous batching: the same two steps on an arbitrary set of cache slots, so that newly admitted requests are
 * prefilled while the sequences already running keep decoding in shared steps.  Sequence i of a call lives in
 * cache slot slot_ids[i] (host array, n distinct values in [0, max_batch)); rows of patch_emb / offsets /
 * token_ids / logits_out are in call order, not slot order.  Sequences are independent, so a sequence's
 * results do not depend on which slot it occupies or on what runs beside it.
 *   vla_prefill_slots  arguments as vla_prefill; overwrites the given slots only (an occupied slot restarts).
 *   vla_decode_slots   arguments as vla_decode_step; VLA_E_STATE if a slot holds no sequence,
 *                      VLA_E_CAPACITY if one is full.
 *   vla_release_slots  marks slots free (host state only).
 * Mixing with the whole-batch calls: vla_prefill and the policy-step calls reset every slot and use slots
 * 0..B-1; after vla_prefill_slots / vla_release_slots, vla_decode_step is refused until the next whole-batch
 * prefill.  A weight update (vla_update_begin, vla_load_weights) frees every slot. */
int vla_prefill_slots(vla_ctx* ctx, int32_t n, const int32_t* slot_ids, const void* patch_emb,
                      const int32_t* cu_patch, const int32_t* instr_ids, const int32_t* cu_instr,
                      float* logits_out, void* hip_stream);
int vla_decode_slots(vla_ctx* ctx, int32_t n, const int32_t* slot_ids, const int32_t* token_ids,
                     float* logits_out, void* hip_stream);
int vla_release_slots(vla_ctx* ctx, int32_t n, const int32_t* slot_ids);

/* Request queue with the dynamic-window trigger of Section 3.2, Eq. 1 (host code; no GPU work):
 *     Trigger = (|Q| >= target_batch) or (t_now - t_first >= t_max),   t_first = arrival of the oldest request.
 * Times are seconds on any monotonic clock of the caller's choice, passed in explicitly.  A poll that
 * triggers hands out the oldest requests in arrival order: at most target_batch, and, if max_tokens > 0,
 * only while their packed prefix tokens (n_patches + n_instr summed) fit (always at least one); the rest
 * stay queued with their own arrival times, so the next poll may trigger again at once.  An empty queue
 * never triggers.  vla_batcher_push may be called from any thread, concurrently with polls; an arrival stamp
 * older than the previous push's is raised to it (the queue is first-in first-out).
 *   vla_batcher_create   VLA_E_CONFIG unless target_batch > 0, t_max >= 0 and finite, max_tokens >= 0.
 *   vla_batcher_push     VLA_E_SHAPE for an empty or negative prefix or a NaN stamp, VLA_E_CAPACITY if the
 *                        request alone exceeds max_tokens.  The struct is copied; `id` is opaque.
 *   vla_batcher_poll     out: host array of cap >= 1 entries (else VLA_E_CAPACITY); a triggered poll hands out at
 *                        most min(target_batch, cap) requests (cap = what the caller can take now, e.g. its
 *                        free cache slots); *n_out = number handed out (0: not triggered).
 *   vla_batcher_deadline *t = t_first + t_max, the time at which waiting alone will trigger (+inf if empty). */
typedef struct vla_batcher vla_batcher;
typedef struct {
  uint64_t id;
  int32_t n_patches, n_instr;
  double t_arrival;
} vla_request;
int vla_batcher_create(int32_t target_batch, double t_max, int64_t max_tokens, vla_batcher** out);
int vla_batcher_destroy(vla_batcher* b);
int vla_batcher_push(vla_batcher* b, const vla_request* r);
int vla_batcher_size(vla_batcher* b, int32_t* n);
int vla_batcher_deadline(vla_batcher* b, double* t);
int vla_batcher_poll(vla_batcher* b, double t_now, vla_request* out, int32_t cap, int32_t* n_out);

/* Selection alone, for callers that drive vla_prefill / vla_decode_step themselves:
 * logits [B, n_action_bins] (device) -> bin index, log-prob, action, for token index k of the
 * chunk (k selects the action dimension k mod action_dim and the row [b, k] of gumbel [B, K, A]).
 * next_ids_out (device, [B] int32 or NULL) receives the absolute vocabulary id to feed back. */
int vla_select(vla_ctx* ctx, int32_t B, const float* logits, float temperature, const float* gumbel,
               int32_t k, int32_t n_tokens, const float* act_scale, const float* act_offset,
               int32_t action_dim, int32_t* tokens_out, float* logp_out, float* actions_out,
               int32_t out_stride, int32_t* next_ids_out, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* VLA_H */
