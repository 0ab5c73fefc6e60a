/*
 * rl_rollout.h - C boundary of the batched multi-turn rollout engine (one GPU).
 *
 * The engine runs the GPU part of the "Generate - Parse - Invoke - Update" loop of the
 * paper's Section 2.3.2: Generate = rl_decode_step repeated, Update = rl_append_observation,
 * termination of a trajectory (Section 2.2, last paragraph; Section 2.3.2 Parse step: no tool
 * call found) = rl_release.  A trajectory is the interleaving of model-generated chunks X and
 * observation chunks O of Section 2.2; the engine keeps, per trajectory, the tokens, the
 * observation mask (1 = appended from outside, 0 = sampled by the policy; observation tokens
 * do not take part in the loss, Section 2.2 / "Loss Mask" in Section 2.3.2) and the log-prob
 * of every sampled token.
 *
 * General rules
 *  - All pointers in the signatures are HOST pointers; the library owns every device buffer.
 *  - The caller owns every buffer it passes in or receives results in.
 *  - Every function returns 0 (RL_OK) or a negative rl_status; a failing call changes no
 *    trajectory or allocator state (pages are reserved for the whole call before any write).
 *    rl_last_error() gives a thread-local message for the last failure.
 *  - Calls are synchronous: results are in the output buffers when the call returns.
 *  - One caller thread per rl_model; different models are independent.
 *  - Trajectory ids are arbitrary non-negative int32 chosen by the caller.
 */
#ifndef RL_ROLLOUT_H
#define RL_ROLLOUT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rl_model rl_model;

typedef enum {
  RL_OK = 0,
  RL_E_ARG = -1,          /* null pointer, negative count / id / temperature, bad config */
  RL_E_BAD_TRAJ = -2,     /* unknown trajectory id */
  RL_E_DUP_ID = -3,       /* the same id twice in one call, or a fork destination that exists */
  RL_E_BAD_TOKEN = -4,    /* token id outside [0, vocab) */
  RL_E_NOPAGES = -5,      /* KV page pool exhausted */
  RL_E_CTX_OVERFLOW = -6, /* a trajectory would exceed max_context */
  RL_E_EMPTY = -7,        /* decode on a trajectory without any token */
  RL_E_HIP = -8,          /* a HIP runtime call failed */
  RL_E_TOO_MANY = -9      /* more live trajectories than max_trajectories */
} rl_status;

/* Decoder shape, as stored in the weight blob's header. */
typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, intermediate, vocab;
  float rms_eps, rope_theta;
  int32_t qk_norm;        /* 1: per-head RMSNorm on q and k before RoPE */
  int32_t tie_embeddings; /* 1: lm-head shares the embedding matrix */
  int32_t weight_dtype;   /* 0: fp32 weights, fp32 arithmetic and cache; 1: bf16 weights,
                             bf16 activations / cache, fp32 accumulation and residual */
} rl_model_config;

typedef struct {
  int32_t page_tokens;      /* tokens per KV page; must be 16 */
  int32_t max_context;      /* longest trajectory, in tokens */
  int32_t max_trajectories; /* live trajectories at any time */
  int64_t kv_pool_pages;    /* pages in the pool (each holds page_tokens tokens of every layer);
                               0: sized automatically: max_trajectories x ceil(max_context / 16),
                               capped by 85 % of the device memory free at load time */
  int32_t max_batch_rows;   /* rows processed per internal pass of an append (0: default 8192) */
  int32_t flags;            /* RL_FLAG_* */
} rl_runtime_config;

#define RL_FLAG_GENERIC_KERNELS 1 /* bf16 models: use the shape-generic kernels even where the
                                     MFMA kernels apply (testing) */
#define RL_FLAG_SHARED_PREFIX_ATTENTION 2 /* decode attention reads the pages that the members of a
                                     forked group share (Section 2.3.2: several samples per prompt)
                                     once per group of 16 / (n_q / n_kv) members instead of once per
                                     member, and merges the result with each member's own pages */
#define RL_FLAG_FP8_KV_CACHE 4 /* keys (after QK-norm and RoPE) and values are cached as OCP FP8 E4M3
                                     codes: nearest code, ties to even, magnitudes above 448 stored
                                     as +-448; read back exactly and used in bf16 arithmetic.  Halves
                                     the bytes of the cache and of the decode attention.  A variant
                                     with its own numerical contract (the paper describes no cache);
                                     bf16 models with head_dim 128 on the MFMA kernels only, else
                                     rl_model_load fails with ARG */

/*
 * Load a model: parse the blob (64-byte header: "RLW1", u32 version 1, the rl_model_config
 * fields in declaration order, zero padding; then tensors back to back, row-major [out, in]:
 * embed[V,H]; per layer g_in[H] W_q W_k W_v g_q[d] g_k[d] W_o g_post[H] W_gate W_up W_down;
 * g_final[H]; lm_head[V,H] unless tied), copy and repack the weights into device memory,
 * build the RoPE table and allocate the KV page pool.  `weights` may be freed on return.
 * head_dim must be even and at most 128.
 * Errors: RL_E_ARG (bad header / size / config), RL_E_HIP (allocation).
 */
int rl_model_load(const rl_runtime_config* rt, const void* weights, size_t nbytes,
                  rl_model** out);
void rl_model_free(rl_model* m);
int rl_model_get_config(const rl_model* m, rl_model_config* out);
const char* rl_last_error(void);

/*
 * Update step (Section 2.3.2): append lens[i] tokens (observation tokens, or the prompt) to
 * trajectory traj_ids[i]; `tokens` is the concatenation in call order.  Unknown ids are
 * created.  Every appended token gets mask 1 and no log-prob.  The tokens' keys / values are
 * computed by chunked prefill into the paged cache.  Pages are taken lowest-free-index first,
 * trajectories in call order.  lens[i] = 0 is allowed.
 * Errors: ARG, DUP_ID, BAD_TOKEN, CTX_OVERFLOW, TOO_MANY, NOPAGES, HIP.
 */
int rl_append_observation(rl_model* m, const int32_t* traj_ids, int32_t n,
                          const int32_t* tokens, const int32_t* lens);

/*
 * Generate step (Section 2.3.2; a_t ~ pi_theta(. | s_t), Section 2.2): one new token for each
 * listed trajectory.  The token is drawn from softmax(logits / temperature) by integer
 * inverse CDF at the 32-bit uniform rl_uniform_u32(rng_seed, traj_id, index of the new token);
 * temperature 0 selects the arg-max (lowest index on ties).  token_ids_out[i] and
 * logprobs_out[i] (log-prob under the temperature-scaled distribution; temperature 0 reports
 * it at temperature 1) are in call order.  The token is appended with mask 0.
 * Errors: ARG, BAD_TRAJ, DUP_ID, EMPTY, CTX_OVERFLOW, NOPAGES, HIP.
 */
int rl_decode_step(rl_model* m, const int32_t* active_traj_ids, int32_t n, float temperature,
                   uint64_t rng_seed, int32_t* token_ids_out, float* logprobs_out);

/*
 * Generate step repeated (Section 2.3.2: the model generates a response token by token until the
 * Parse step looks at it): exactly n_steps calls of rl_decode_step(active_traj_ids, n, temperature,
 * rng_seed, ...) in a row, in one call.  token_ids_out and logprobs_out hold n_steps x n entries,
 * step-major (entry s * n + i belongs to step s, trajectory active_traj_ids[i]).  Results, state and
 * page indices are identical, bit for bit, to the single steps; what differs is the timing: a
 * sampled token feeds the next step on the device, and the host stages the following steps while the
 * GPU works instead of waiting for every step's ids, so the GPU does not idle between steps.  The
 * caller decides how many tokens to generate before it looks at them (a turn of known length, or a
 * window after which it checks for a tool call).  All or nothing over the whole call: context
 * overflow and page needs are checked for all n_steps tokens before anything changes.
 * n_steps = 0 is allowed.  Errors: as rl_decode_step.
 */
int rl_decode_steps(rl_model* m, const int32_t* active_traj_ids, int32_t n, int32_t n_steps,
                    float temperature, uint64_t rng_seed, int32_t* token_ids_out, float* logprobs_out);

/*
 * Update + Generate in one pass (continuous batching, Section 2.3.2: tool calls return at different
 * times, the batch must not wait): exactly rl_append_observation(app_*) followed by
 * rl_decode_step(active_traj_ids, ...), but the appended tokens' keys / values are computed in the
 * same forward pass as the decode rows, so the weights are streamed once for both.  A trajectory
 * may be in both lists (it decodes right after its observation).  If the appended rows and the
 * decode rows exceed one pass (max_batch_rows) the append is prefilled first.  Results equal the
 * two separate calls within floating-point tolerance (integer state identically).  Errors: those
 * of the two calls; when the append part succeeds and the decode part is rejected, the append has
 * taken effect (as it would have with two calls).
 */
int rl_decode_step_with_appends(rl_model* m, const int32_t* app_traj_ids, int32_t n_app,
                                const int32_t* app_tokens, const int32_t* app_lens,
                                const int32_t* active_traj_ids, int32_t n, float temperature,
                                uint64_t rng_seed, int32_t* token_ids_out, float* logprobs_out);

/* Trajectory ended: give its pages back (shared pages when their last holder lets go). */
int rl_release(rl_model* m, const int32_t* traj_ids, int32_t n);

/* ---- auxiliaries --------------------------------------------------------------------- */

/*
 * Group sampling (Section 2.3, the GRPO example: several trajectories continue one prompt):
 * create dst_ids[0..n) as copies of trajectory `src`.  Pages lying entirely before src's last
 * token are shared by reference count; the remaining page is copied into a fresh page per
 * destination.  Errors: ARG, BAD_TRAJ, DUP_ID, TOO_MANY, NOPAGES, HIP.
 */
int rl_fork(rl_model* m, int32_t src, const int32_t* dst_ids, int32_t n);

int rl_traj_info(rl_model* m, int32_t traj_id, int32_t* n_tokens, int32_t* n_pages);
/* Any output may be NULL; non-NULL ones must hold n_tokens (pages: n_pages) entries.
 * logprobs[t] is 0 where obs_mask[t] = 1. */
int rl_traj_read(rl_model* m, int32_t traj_id, int32_t* tokens, uint8_t* obs_mask,
                 float* logprobs, int32_t* pages);
int64_t rl_free_pages(const rl_model* m);

/*
 * Teacher-forced full-trajectory pass (the log-prob recomputation that consumes the loss
 * mask): for each listed trajectory with n tokens writes n floats, out[t] = log softmax(
 * z_{t-1} / temperature)[x_t] where x_t was sampled (mask 0), 0 where it was appended (mask 1)
 * and at t = 0; trajectories are concatenated in call order.  Temperature 0 means 1.
 */
int rl_recompute_logprobs(rl_model* m, const int32_t* traj_ids, int32_t n, float temperature,
                          float* out);

/*
 * Forward value of the token-level masked GRPO objective over trajectories held in the cache
 * (group sampling: Section 2.3, the multi-turn interaction example; tool results excluded from
 * the loss: Section 2.2, last paragraph, and the loss mask of Section 2.3.2).  The paper prints
 * no formula; this is the published GRPO objective restricted to the tokens the policy sampled:
 *   A_i   = (r_i - mean_g(r)) / (std_g(r) + eps_std)      g = group of group_size consecutive ids
 *   rho_t = exp(lp_new[t] - lp_old[t]),  k3_t = exp(d) - d - 1,  d = lp_ref[t] - lp_new[t]
 *   J_i   = mean over sampled tokens t of  min(rho_t A_i, clip(rho_t, 1 - clip_eps, 1 + clip_eps) A_i) - beta k3_t
 *   J     = mean over the n trajectories of J_i  (a trajectory without sampled tokens gives 0)
 * lp_new is recomputed by a teacher-forced pass of the current weights at `temperature` (as
 * rl_recompute_logprobs; the log-probs stay on the device).  All pointers are host memory.
 *   rewards        [n] finite floats, one per trajectory
 *   old_logprobs   one float per token of every listed trajectory, concatenated in call order
 *                  (the layout rl_recompute_logprobs writes); NULL = the log-probs recorded when
 *                  the tokens were sampled.  Values at appended tokens are ignored.
 *   ref_logprobs   same layout, or NULL: no KL term (beta ignored, *kl_out = 0)
 *   std_ddof       0: population standard deviation; 1: sample (needs group_size >= 2)
 *   objective_out  J (to be maximised);  kl_out (may be NULL): mean over trajectories of their
 *                  mean k3;  n_tokens_out (may be NULL): sampled tokens that took part;
 *                  advantages_out (may be NULL): [n] doubles A_i
 * Sums are float64 in a fixed order: results are reproducible run to run.  No state changes.
 * Errors: ARG (n <= 0, n not a multiple of group_size, negative or non-finite parameter,
 * non-finite reward, null pointer), BAD_TRAJ, DUP_ID, HIP.
 */
int rl_grpo_objective(rl_model* m, const int32_t* traj_ids, int32_t n, int32_t group_size,
                      const float* rewards, const float* old_logprobs, const float* ref_logprobs,
                      float temperature, double clip_eps, double beta, double eps_std,
                      int32_t std_ddof, double* objective_out, double* kl_out,
                      int64_t* n_tokens_out, double* advantages_out);

/* Parity aids.  rl_debug_logits: next-token logits [vocab] of one trajectory, no state change.
 * rl_decode_step_forced: a decode step that appends forced_token_ids[i] instead of sampling and
 * returns its log-prob. */
int rl_debug_logits(rl_model* m, int32_t traj_id, float* logits_out);
int rl_decode_step_forced(rl_model* m, const int32_t* traj_ids, int32_t n, float temperature,
                          const int32_t* forced_token_ids, float* logprobs_out);
/* rl_decode_step_with_appends with forced tokens (parity aid). */
int rl_decode_step_forced_with_appends(rl_model* m, const int32_t* app_traj_ids, int32_t n_app,
                                       const int32_t* app_tokens, const int32_t* app_lens,
                                       const int32_t* traj_ids, int32_t n, float temperature,
                                       const int32_t* forced_token_ids, float* logprobs_out);

/* The sampler in isolation, on the GPU: `rows` rows of `vocab` float32 logits (host), one
 * uniform per row.  Same arithmetic as inside rl_decode_step. */
int rl_sample_from_logits(const float* logits, int32_t rows, int32_t vocab, float temperature,
                          const uint32_t* u32, int32_t* ids_out, float* logprobs_out);
/*
 * rl_sample_from_logits for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Unlike every other call here the
 * pointers are DEVICE pointers (`rows` rows of `vocab` float32 logits, row stride `vocab`; one
 * uniform per row; outputs ids and log-probs); `stream` is a hipStream_t (NULL: the default stream).
 * The kernels are enqueued on `stream` and the call returns without waiting for them.  It calls no
 * hipMalloc / hipFree: the per-segment scratch of the sampler is a fixed array inside the library's
 * device image (384 KiB per GPU, held until the process ends) that holds rows x ceil(vocab / 4096)
 * <= 16384 segments; larger requests fail with RL_E_ARG and launch nothing.  All calls on one GPU
 * share that array: calls that overlap in time on one GPU (different streams or threads) race.
 * Nothing in the array has to be cleared between calls.  The address of the array is looked up
 * once per GPU, by rl_model_load or by the first call on that GPU; make that first call outside
 * graph capture.  Same arithmetic and results as rl_sample_from_logits.
 * Errors: ARG, HIP.
 */
int rl_sample_device_logits(const float* d_logits, int32_t rows, int32_t vocab, float temperature,
                            const uint32_t* d_u32, int32_t* d_ids_out, float* d_logprobs_out,
                            void* stream);
/* SplitMix64 output number ((traj_id << 32) | position) + 1 from state `seed`, top 32 bits. */
uint32_t rl_uniform_u32(uint64_t seed, int32_t traj_id, int32_t position);

/*
 * Kernel timing for benchmarks: when enabled, every `every`-th decode step brackets its
 * decode-attention launches with HIP events on the engine's stream.  rl_timing_read returns
 * the accumulated duration, the number of timed launches and the bytes of keys / values
 * those launches had to read: attn_kv_bytes sums context length x bytes per token per layer over
 * the rows; attn_kv_unique_bytes counts a page shared by several trajectories of the step once.
 */
int rl_timing_enable(rl_model* m, int32_t every);
int rl_timing_read(rl_model* m, double* attn_ms, int64_t* attn_launches, double* attn_kv_bytes,
                   double* attn_kv_unique_bytes, int reset);
/* Byte accounting of the decode steps (Generate step, Section 2.3.2) made while timing is enabled
 * (every step, not only the timed ones; steps that also carried appended rows are left out): keys +
 * values of one layer that the steps' attention had to read, summed over the steps.  kv_bytes
 * counts every trajectory's context; kv_unique_bytes counts a page that several trajectories of a
 * step share (a forked prompt) once per step.  Multiply by the layer count for a whole step. */
int rl_timing_read_decode_bytes(rl_model* m, double* kv_bytes, double* kv_unique_bytes,
                                int64_t* steps, int reset);
/* GPU time of the timed decode steps, first kernel to sampler (HIP events), and their count. */
int rl_timing_read_steps(rl_model* m, double* step_gpu_ms, int64_t* steps, int reset);

/* Benchmark calibration: rate (GB/s) at which a plain kernel streams `bytes` (>= 16 MiB) of a
 * freshly allocated device buffer, averaged over `iters` passes: the read ceiling of the GPU the
 * library runs on, to set beside the nominal HBM figure.  Allocates and frees its own buffer. */
int rl_measure_stream_read(size_t bytes, int32_t iters, double* gb_per_s);

#ifdef __cplusplus
}
#endif
#endif /* RL_ROLLOUT_H */
