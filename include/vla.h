/*
 * vla.h -- C-ABI of the MI355X (gfx950) library for the batched VLA policy rollout step and
 * the PPO/GRPO log-probability recompute.
 *
 * The operations follow the paper's statement of the problem:
 *   - generation: at every simulator step the policy infers an action (chunk) from the current
 *     observation, a_t ~ pi_theta(. | o_t), for all parallel environments (sections III-A,
 *     III-C); an atomic action is M tokens, one per action dimension, a chunk is C atomic
 *     actions (section III-B);
 *   - token-level log-probabilities pi(d_{t,i,j} | o_t, d_{t,i,:j-1}) (section IV-C.1);
 *   - the recompute of log pi_theta on stored (o_t, a_t) that the importance ratio
 *     rho = pi_theta / pi_theta_old of the PPO and GRPO objectives needs (appendix I-B, I-C);
 *   - a lightweight value head attached to the language model (section IV-C.2).
 * The decoder itself is a Llama-style pre-norm transformer (RMSNorm, rotary with half-split
 * pairing, multi-head causal attention without biases, SwiGLU); action tokens are the last
 * n_bins = 256 vocabulary ids and every distribution is over those 256 bins only.
 *
 * Conventions for every function below
 *   - Pointers marked DEVICE are device memory owned by the caller; pointers marked HOST are
 *     host memory.  The three hot calls never allocate or free device memory.
 *   - All device work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream).  No call synchronises; outputs are valid once the caller has
 *     synchronised the stream.  Calls that share a KV buffer or workspace must be ordered by
 *     the caller (same stream, or events).
 *   - Return value: VLA_OK (0) or a negative error code.  On error nothing has been enqueued
 *     (except for VLA_EHIP, which reports a failed launch) and vla_last_error() returns a
 *     thread-local, NUL-terminated HOST string describing it.  No exception crosses the ABI.
 *   - "dtype" below means the storage type selected by vla_config.dtype: float (VLA_DTYPE_F32)
 *     or bfloat16 (VLA_DTYPE_BF16).  Weight matrices, patch embeddings, slot embeddings and the
 *     KV cache use it; norm gains, the value head, noise and every output are fp32.
 *     Accumulation, the residual stream, norms, softmax and the action-bin head are fp32.
 *   - Weight matrices are row-major [out, in].
 */
#ifndef VLA_H
#define VLA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VLA_VERSION 1

#define VLA_OK          0
#define VLA_EINVAL     (-1)  /* null pointer, negative or zero size, bad enum              */
#define VLA_ESHAPE     (-2)  /* exceeds max_batch / max_seq, or unsupported dimensions      */
#define VLA_EWORKSPACE (-3)  /* workspace (or KV buffer) smaller than required              */
#define VLA_EDTYPE     (-4)  /* unknown dtype                                               */
#define VLA_EHIP       (-5)  /* a HIP call or kernel launch failed                          */

#define VLA_DTYPE_F32  0
#define VLA_DTYPE_BF16 1

#define VLA_MODE_AR             0  /* autoregressive: token j+1 conditioned on tokens 1..j   */
#define VLA_MODE_PARALLEL_CHUNK 1  /* all A slots in one forward, bidirectional among slots  */

#define VLA_ENTRY_PREFILL   0
#define VLA_ENTRY_DECODE    1
#define VLA_ENTRY_RECOMPUTE 2

#define VLA_N_BINS 256

typedef struct vla_config {
    int32_t n_layers, hidden, n_heads, ffn, vocab;
    int32_t n_bins;      /* must be 256; bin k is token id vocab - 256 + k                   */
    int32_t dtype;       /* VLA_DTYPE_*                                                      */
    float   rms_eps;     /* RMSNorm epsilon                                                  */
    float   rope_theta;  /* rotary base                                                      */
    int32_t max_batch;   /* capacity: sequences per call                                     */
    int32_t max_seq;     /* capacity: positions per sequence (prefix + action rows); also the
                            position stride of the KV buffer                                 */
    int32_t value_dim;   /* outputs of the value head: 1 = one scalar per observation (chunk-level
                            value), C = one value per atomic action of the chunk (action-level
                            value, section IV-C.2); 0 is read as 1                            */
} vla_config;

/* DEVICE pointers.  attn_norm, ffn_norm: fp32 [hidden].  wq, wk, wv, wo: dtype [hidden, hidden].
 * w_gate, w_up: dtype [ffn, hidden].  w_down: dtype [hidden, ffn]. */
typedef struct vla_layer_weights {
    const void *attn_norm, *wq, *wk, *wv, *wo, *ffn_norm, *w_gate, *w_up, *w_down;
} vla_layer_weights;

/* embed, lm_head: DEVICE dtype [vocab, hidden] (only the last 256 rows of lm_head are read).
 * final_norm: DEVICE fp32 [hidden].  value_w: DEVICE fp32 [value_dim, hidden] or NULL (no value head).
 * value_b: scalar bias added to every value output; value_bias: DEVICE fp32 [value_dim] added per
 * output, or NULL.  layers: HOST array of n_layers entries, copied by vla_create. */
typedef struct vla_weights {
    const void *embed, *lm_head, *final_norm, *value_w;
    float value_b;
    const vla_layer_weights *layers;
    const void *value_bias;
} vla_weights;

typedef struct vla_model vla_model;

int vla_version(void);

/* HOST string describing the calling thread's last error ("" if none). */
const char *vla_last_error(void);

/* Create a host-side model object.  It stores the configuration and the weight POINTERS only;
 * the weights stay owned by the caller and must outlive the model.  Checks the dimensions:
 * hidden = n_heads * head_dim with head_dim a multiple of 16 and at most 256; n_bins = 256
 * <= vocab; positive sizes.  Touches no device. */
int vla_create(const vla_config *cfg, const vla_weights *weights, vla_model **out);
int vla_destroy(vla_model *model);

/* Optional repacked copy of the decoder-layer projection weights for the multi-row (prefill, parallel chunk,
 * recompute) forwards of bf16 models.  The large GEMM loads its operands straight into LDS; with the weights
 * stored [K / 32][rows][32] instead of row-major [rows, K] every such load reads whole cache lines.
 * vla_prepack_bytes: size of the copy for this configuration, 0 if the configuration has no use for it
 *   (fp32 storage, head_dim other than 128, widths that are not tile aligned).
 * vla_prepack: enqueues the repack of all layers on `stream` into `buffer` (DEVICE, 256-byte aligned, at least
 *   vla_prepack_bytes bytes, caller owned) and makes the model use it from then on; the caller orders later
 *   calls after it (same stream, or events) and keeps the buffer alive and unchanged while the model uses it.
 *   buffer = NULL detaches.  The original weights stay in use for single-row (decode) forwards.  Results
 *   with and without the copy are bit-identical. */
size_t vla_prepack_bytes(const vla_config *cfg);
int vla_prepack(vla_model *model, void *buffer, size_t bytes, void *stream);

/* Bytes of the caller-allocated KV buffer for B sequences of up to max_pos positions
 * (max_pos <= cfg->max_seq; the buffer is always laid out with cfg->max_seq positions per
 * sequence, so the same B must be used by every call sharing it).  Layout is opaque.
 * Returns 0 on invalid arguments (see vla_last_error). */
size_t vla_kv_bytes(const vla_config *cfg, int B, int max_pos);

/* Bytes of workspace the given entry point needs for B sequences, prefix length S and A action
 * tokens (for VLA_ENTRY_RECOMPUTE, B is the number of stored rollouts N; the call processes
 * them in micro-batches, so the size stops growing beyond an internal micro-batch).  The
 * workspace holds no state between calls.  Returns 0 on invalid arguments. */
size_t vla_workspace_bytes(const vla_config *cfg, int entry, int B, int S, int A);

/* Prefill (sections III-A, III-C: the observation o_t enters the policy).  For each of B
 * environments, the prefix rows x_p = patch[p] (p < P), x_{P+t} = embed[ids[t]] run through all
 * decoder layers with causal attention; K and V of every prefix row are written to `kv`.
 *   kv        DEVICE, >= vla_kv_bytes(cfg, B, P+T)        ws  DEVICE workspace, ws_bytes long
 *   patch     DEVICE dtype [B, P, hidden] (P may be 0)     ids DEVICE int32 [B, T] in [0, vocab)
 *   h_last    DEVICE fp32 [B, hidden] out: final-norm output of the last prefix row
 *   value     DEVICE fp32 [B, value_dim] out or NULL: value_w . h_last + bias (section IV-C.2)
 * Requires P + T >= 1, B <= max_batch, P + T <= max_seq, and B * (P + T) rows within what one
 * pass can hold: the residual stream [rows, hidden] fp32 and the widest activation
 * [rows + 256 + pad, max(hidden, ffn)] in the storage dtype each below 2 GiB (32-bit byte
 * offsets in the kernels; 97,254 rows at the 7B shape in bf16).  Beyond that VLA_ESHAPE: split
 * the batch over several calls (each with its own kv). */
int vla_prefill(vla_model *model, void *kv, void *ws, size_t ws_bytes,
                const void *patch, const int32_t *ids, int B, int P, int T,
                float *h_last, float *value, void *stream);

/* Decode A action tokens per environment after vla_prefill on the same kv with the same B
 * (section III-C generation; token factorisation of section IV-C.1).
 *   mode VLA_MODE_AR: token 1 is read from h_last; for j = 1..A-1 token id vocab-256+bin_j is
 *     embedded at position S+j-1 and run through the decoder against the cache (its K, V are
 *     appended); token j+1 is read from that row.  The sampled bin feeds the next forward on
 *     the device.  The last token is not fed back.
 *   mode VLA_MODE_PARALLEL_CHUNK: one forward over A slot rows with inputs slot_embed[s] at
 *     positions S+s; slot rows attend to all S prefix rows and all A slot rows; slot s is read
 *     from its own row.  h_last is ignored.
 *   For every token: y = z / temperature over the 256 bins, bin = argmax_k (y_k + gumbel_k)
 *   (lowest k wins ties; gumbel NULL = greedy), logp = y_bin - logsumexp(y),
 *   entropy = -sum_k p_k log p_k (nats).
 *   h_last     DEVICE fp32 [B, hidden] from vla_prefill    S   prefix length P+T of that prefill
 *   slot_embed DEVICE dtype [A, hidden] (mode 1) or NULL   temperature > 0
 *   gumbel     DEVICE fp32 [B, A, 256] or NULL
 *   bins       DEVICE int32 [B, A] out                     logp, entropy DEVICE fp32 [B, A] out
 *   logits     DEVICE fp32 [B, A, 256] out or NULL: untempered z, for parity checks
 * Requires A >= 1 and S + A - 1 <= max_seq (mode 0), S + A <= max_seq (mode 1); mode 1 also
 * B * A rows within one pass (see vla_prefill). */
int vla_decode_actions(vla_model *model, void *kv, void *ws, size_t ws_bytes,
                       const float *h_last, int B, int S, int A, int mode,
                       const void *slot_embed, float temperature, const float *gumbel,
                       int32_t *bins, float *logp, float *entropy, float *logits, void *stream);

/* Log-probability recompute for the policy update (appendix I-B: rho needs log pi_theta of
 * the stored actions under the current weights).  Teacher-forced forward over N stored
 * rollouts without a persistent KV cache.
 *   mode VLA_MODE_AR: rows = prefix, then the stored tokens 1..A-1 (S + A - 1 rows, causal);
 *     token j is read from row S + j - 2 (1-based j).
 *   mode VLA_MODE_PARALLEL_CHUNK: rows = prefix, then the A slot inputs; prefix rows causal,
 *     slot rows see all rows.
 *   bins   DEVICE int32 [N, A], each in [0, 256): the stored actions
 *   logp   DEVICE fp32 [N, A] out: log-prob of the stored bin at the given temperature
 *   entropy DEVICE fp32 [N, A] out      value DEVICE fp32 [N, value_dim] out or NULL (last prefix row)
 *   logits DEVICE fp32 [N, A, 256] out or NULL
 * N may exceed max_batch: rollouts are processed in internal micro-batches of max_batch rollouts
 * (fewer if that many rows do not fit one pass, see vla_prefill) and the result does not depend
 * on the split. */
int vla_logprob_recompute(vla_model *model, void *ws, size_t ws_bytes,
                          const void *patch, const int32_t *ids, const int32_t *bins,
                          int N, int P, int T, int A, int mode, const void *slot_embed,
                          float temperature, float *logp, float *entropy, float *value,
                          float *logits, void *stream);

/* ---- profiling (auxiliary; process-wide, not thread safe) --------------------------------------
 * While enabled, every kernel launch of the three hot calls is bracketed by a pair of HIP events
 * recorded on the launch stream, tagged with a label and with the launch's algorithmic work (flops
 * for contractions, bytes for streaming kernels).  Events add a few microseconds per launch, so
 * timed throughput runs keep profiling off.
 *   vla_profile_enable(on)   turn recording on (1) or off (0); turning it on clears old records.
 *   vla_profile_report(buf, n) synchronises the recorded events and writes, into the HOST buffer
 *     buf of n bytes, one line per label: "label count total_ms total_work" (NUL terminated,
 *     truncated to n).  Returns the number of labels, or a negative error code. */
int vla_profile_enable(int on);
int vla_profile_report(char *buf, size_t n);

/* Triage aid (process-wide, not thread safe): a bit mask of steps that take the shape-generic kernel even where a
 * gfx950 fast path applies -- 1 large GEMM, 2 decode GEMM, 4 multi-row attention, 8 decode attention, 16 rotary / KV
 * write / RMSNorm; 0 (the default) selects every fast path.  Results stay within the parity tolerances either way;
 * the tests use it to run the generic kernels on shapes that would otherwise never reach them. */
int vla_debug_force_generic(int mask);

/* Calibration aid for hardware-counter runs: a plain copy kernel (`bytes` must be a multiple of 16;
 * dst, src DEVICE, 16-byte aligned) that reads and writes exactly `bytes` bytes, so that HBM
 * traffic counters collected around the hot kernels can be scaled by what they read for it. */
int vla_calibration_copy(void *dst, const void *src, size_t bytes, void *stream);

/* ---- consumers of the recomputed log-probabilities in the policy update ------------------------
 * All arrays DEVICE fp32 (flags and masks int32), row-major; launches on `stream`, no sync.  Sums are
 * taken in a fixed order (no atomics), so results are bit-reproducible.
 *
 * vla_gae -- generalized advantage estimation (appendix I-B):
 *   delta_t = r_t + gamma V(s_{t+1}) - V(s_t),  A_t = sum_k (gamma lambda)^k delta_{t+k}.
 *   rewards [n, T]; values [n, T+1] (column T bootstraps the last step); dones [n, T] or NULL: a
 *   non-zero done_t ends an episode at step t inside the row (partial reset), cutting both the
 *   bootstrap term and the sum.  Outputs adv [n, T] and returns = adv + V [n, T] (returns may be NULL).
 *
 * vla_grpo_advantage -- group-relative advantage (appendix I-C): for each group of G consecutive
 *   trajectories A_i = (R_i - mean) / std with the population standard deviation.  total_reward
 *   [n_groups * G]; adv out, same shape; keep [n_groups] out or NULL: 0 for groups whose returns are
 *   all equal (advantages 0; the success-rate filter of section IV-C.3 drops them), else 1.
 *
 * vla_policy_objective -- clipped surrogate of PPO / GRPO (appendix I-B, I-C, II-C.2):
 *   s = min(rho A, clip(rho, 1 - clip_low, 1 + clip_high) A), rho = exp(logp_new - logp_old).
 *   logp_new, logp_old [n_traj, T]; adv [n_traj, T] if adv_per_step else [n_traj]; mask [n_traj, T]
 *   (non-zero = valid step) or NULL.  per_trajectory = 0: objective = mean of s over all valid steps
 *   (PPO's E_t); 1: (1/n_traj) sum_i (1/T_i) sum_t s with T_i the valid steps of trajectory i (GRPO
 *   with the valid-action mask; a trajectory without valid steps contributes 0).
 *   ws: DEVICE scratch of vla_policy_objective_workspace_bytes(n_traj) bytes.
 *   Outputs: objective [1]; per_step [n_traj, T] or NULL (masked s); clip_frac [1] or NULL (share of
 *   valid steps where the clipped branch is the smaller one).
 *
 * vla_logp_aggregate -- log-probability granularity (section IV-C.1): out[i] = sum of the `inner`
 *   consecutive entries logp[i * inner ...], i < n_out: token -> action with inner = tokens per action,
 *   action -> chunk with inner = actions per chunk. */
int vla_gae(const float *rewards, const float *values, const int32_t *dones, int n, int T, float gamma,
            float lambda, float *adv, float *returns, void *stream);
int vla_grpo_advantage(const float *total_reward, int n_groups, int G, float *adv, int32_t *keep, void *stream);
size_t vla_policy_objective_workspace_bytes(int n_traj);
int vla_policy_objective(const float *logp_new, const float *logp_old, const float *adv, int adv_per_step,
                         const int32_t *mask, int n_traj, int T, float clip_low, float clip_high,
                         int per_trajectory, void *ws, size_t ws_bytes, float *objective, float *per_step,
                         float *clip_frac, void *stream);
int vla_logp_aggregate(const float *logp, size_t n_out, int inner, float *out, void *stream);

/* ---- backward pass of the log-probability recompute: LoRA gradients (section IV-B.2; appendix I-B, I-C) -------------
 * The policy update differentiates the clipped surrogate through rho = exp(logp_theta - logp_old) only, so what it
 * needs from the model is the gradient of  L = sum_{n,j} coef[n,j] * logp_theta[n,j]  with coef = dJ/dlogp (rho * A-hat
 * where the unclipped branch is active, 0 elsewhere; the per_step output of vla_policy_objective times the caller's
 * normalisation).  The trainable parameters are the LoRA factors of the seven projections of every decoder layer:
 * W_eff = W + scale * B A, A [rank, in], B [out, rank].  The model's weights are the EFFECTIVE ones (the caller keeps
 * them merged); with X a projection's input and dY the gradient at its output,
 *     dL/dB = scale * dY^T (X A^T)   [out, rank],      dL/dA = scale * (dY B)^T X   [rank, in].
 * Embeddings, norm gains, the action head and the value head are frozen.
 *
 * vla_lora_layer: DEVICE pointers, storage dtype, per projection a [rank, in] and b [out, rank]
 *   (in / out: hidden / hidden for q, k, v, o; hidden / ffn for gate, up; ffn / hidden for down).
 * vla_lora_layer_grads: DEVICE fp32 outputs of the same shapes, overwritten.
 * vla_logprob_backward: teacher-forced forward over the N stored rollouts exactly as vla_logprob_recompute (same
 *   arguments, same modes), then the backward.  lora, grads: HOST arrays of n_layers entries.  coef DEVICE fp32 [N, A].
 *   logp DEVICE fp32 [N, A] out or NULL: the forward's log-probabilities of the stored bins (the kernels of
 *   vla_logprob_recompute with every row taken through the last layer, so equal to its output up to the rounding
 *   differences of two evaluations).  Rollouts are processed in
 *   micro-batches of max_batch; gradients are summed over micro-batches in order, every sum in a fixed order, so the
 *   result is reproducible bit for bit.  Gradient operands of the GEMMs are rounded to the storage dtype.
 *   keep_activations = 0: the first pass is the forward of vla_logprob_recompute keeping the residual stream at every
 *   layer input, and every layer is run a second time for its backward; ws: DEVICE, at least
 *   vla_backward_workspace_bytes(cfg, N, P + T, A, rank) bytes (grows with max_batch; 11.7 GB at the 7B shape with
 *   max_batch 32).  keep_activations = 1: the first pass keeps what every layer's backward reads for one micro-batch
 *   and no layer is run twice; ws at least vla_backward_keep_workspace_bytes(...) bytes (78 GB there): for GPUs with
 *   memory to spare.  Same gradients up to rounding (the first pass then uses the unfused kernels). */
typedef struct { const void *a, *b; } vla_lora_factor;
typedef struct { vla_lora_factor q, k, v, o, gate, up, down; } vla_lora_layer;
typedef struct { float *da, *db; } vla_lora_grad;
typedef struct { vla_lora_grad q, k, v, o, gate, up, down; } vla_lora_layer_grads;
size_t vla_backward_workspace_bytes(const vla_config *cfg, int N, int S, int A, int rank);
size_t vla_backward_keep_workspace_bytes(const vla_config *cfg, int N, int S, int A, int rank);
int vla_logprob_backward(vla_model *model, void *ws, size_t ws_bytes, const void *patch, const int32_t *ids,
                         const int32_t *bins, const float *coef, int N, int P, int T, int A, int mode,
                         const void *slot_embed, float temperature, int rank, float scale, int keep_activations,
                         const vla_lora_layer *lora, const vla_lora_layer_grads *grads, float *logp, void *stream);

/* vla_policy_objective_noalloc -- vla_policy_objective for callers that cannot allocate device memory (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without the workspace,
 * same kernels, same results bit for bit.  The per-trajectory partial sums live in an array built into the library
 * (786,432 bytes of device memory per GPU, held until the process ends), so n_traj is limited to
 * vla_policy_objective_noalloc_max_traj() = 65,536; beyond that VLA_ESHAPE and nothing is enqueued.  The call
 * allocates and frees nothing, on the device or through any library; the first call on a GPU looks the array's
 * address up once (hipGetSymbolAddress).  Every call on one GPU shares that GPU's array: two calls that overlap in
 * time on the same GPU (different streams or threads) race and must be ordered by the caller.  Nothing of an
 * earlier call is read: every slot the second kernel reads is written by the first. */
int vla_policy_objective_noalloc_max_traj(void);
int vla_policy_objective_noalloc(const float *logp_new, const float *logp_old, const float *adv, int adv_per_step,
                                 const int32_t *mask, int n_traj, int T, float clip_low, float clip_high,
                                 int per_trajectory, float *objective, float *per_step, float *clip_frac,
                                 void *stream);

/* ---------------------------------------------------------------- GPU allocation modes (section IV-A)
 * Host-only arithmetic (no device work, all pointers HOST): the rollout-time model behind the
 * automatic placement.  One rollout epoch is m_chunks steps, each a Generation phase (t_gen for the
 * environments of one Generation GPU) followed by a Simulator phase (t_sim likewise).
 *
 * vla_pipeline_time -- k = 1, collocated mode: *out = m_chunks (t_gen + t_sim), the section's t_1.
 *   k = 2, hybrid mode with fine-grained pipelining: the environments are split in two sub-batches that
 *   take turns on the Generation and on the Simulator partition (times are then per sub-batch):
 *   *out = 2 m_chunks max(t_gen, t_sim) + min(t_gen, t_sim).  The section gives no formula for
 *   t_2, only that it is an estimate for pipelined execution; this is the makespan of the schedule it describes.  Other k: VLA_EINVAL.
 *
 * vla_profile_lookup -- profile[i] is a component's measured time at batch 2^i, i < n_prof (the
 *   section profiles batch sizes 2^0 ... n_S); other batches are interpolated linearly between the two
 *   neighbours.  batch < 1 or above 2^(n_prof-1): VLA_ESHAPE.
 *
 * vla_auto_placement -- min over k in {1, 2} and N_G + N_S = n_gpus of the rollout time.  k = 1 uses
 *   all n_gpus for both components with ceil(n_envs / n_gpus) environments each; k = 2 gives n_gen GPUs
 *   to Generation and n_sim = n_gpus - n_gen to the Simulator, each sub-batch holding
 *   ceil(n_envs / (2 n_gen)) resp. ceil(n_envs / (2 n_sim)) environments per GPU (splits that leave a
 *   GPU without an environment are skipped).  *best receives the fastest candidate (the first on ties,
 *   in the order k = 1, then n_gen = 1, 2, ...); if `all` is not NULL up to all_cap candidates are
 *   written in that order and *n_all (if not NULL) receives their total number. */
typedef struct {
    int32_t k;        /* pipeline stages: 1 collocated, 2 hybrid with pipelining */
    int32_t n_gen;    /* GPUs running Generation (all of them when k = 1)        */
    int32_t n_sim;    /* GPUs running the Simulator (all of them when k = 1)     */
    double time;      /* modelled time of one rollout epoch                       */
} vla_placement;
int vla_pipeline_time(double t_gen, double t_sim, int k, int m_chunks, double *out);
int vla_profile_lookup(const double *profile, int n_prof, double batch, double *out);
int vla_auto_placement(const double *t_gen, const double *t_sim, int n_prof, int n_envs, int n_gpus,
                       int m_chunks, vla_placement *best, vla_placement *all, int all_cap, int *n_all);

#ifdef __cplusplus
}
#endif
#endif /* VLA_H */
