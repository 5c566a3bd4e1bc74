/*
 * rlhf_rollout.h -- C ABI of the MI355X (gfx950) rollout + rescoring library.
 *
 * The library runs the two inference stages of one PPO iteration of RLHF on a GPT-NeoX /
 * Pythia-shaped policy:
 *   rollout_generate : left-padded query batch -> a fixed number of tokens sampled at a temperature,
 *                      truncated at the first EOS            (paper: Dataset Details, "left pad the
 *                      queries"; PPO hyperparameter table, "Sampling Temperature"; PPO Details,
 *                      "EOS trick", steps 1-2)
 *   score_sequences  : teacher-forced forward over the (B, query+response) batch -> per-token
 *                      log-probabilities and values           (paper: Preliminaries, Eq. (RL), KL term;
 *                      General Details, "Disable dropout"; Reward Model Details, "Minor numerical
 *                      differences ..." for the mask; PPO Details, "Value model initializes from the
 *                      reward model" / Preliminaries Step 2 for the scalar linear head)
 *
 * Conventions
 *   - Every function returns 0 on success or a negative rlhf_status; it never throws or aborts.
 *     rlhf_last_error() gives a thread-local message for the last failure on the calling thread.
 *   - "dev" pointers are HIP device pointers, "host" pointers ordinary host memory.  The caller owns
 *     every buffer: weights, workspaces and, in bf16 mode, the fp16 weight image the matrix products read
 *     (rlhf_weight_image_bytes / rlhf_create / rlhf_refresh_weights).  The handle itself allocates only the
 *     two small rotary cos/sin tables (2 x 8192 x rotary_dims/2 floats) in rlhf_create and frees them in
 *     rlhf_destroy; no other call allocates or frees device memory.
 *   - All work is enqueued on the hipStream_t passed as `stream` (NULL = the default stream).  The
 *     calls do not synchronise with the host: outputs are valid once the stream has run the call's
 *     work.  Sizes that depend on the mask (number of real tokens) stay on the device.
 *   - Results are deterministic functions of the inputs: no floating-point atomics are used.
 *   - Calls that share a workspace, or a handle (it owns a helper stream and events on which parts of
 *     the decode loop run next to the caller's stream, joined again before the call's work ends), must
 *     not overlap in time.
 */
#ifndef RLHF_ROLLOUT_H
#define RLHF_ROLLOUT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  RLHF_OK = 0,
  RLHF_EINVAL = -1,       /* null pointer, bad shape, temperature <= 0, max_new_tokens <= 0, ... */
  RLHF_ENOMEM = -2,       /* workspace smaller than rlhf_workspace_bytes reports */
  RLHF_EHIP = -3,         /* a HIP runtime call failed */
  RLHF_EUNSUPPORTED = -4  /* dtype / head_dim / size outside what the kernels are built for */
} rlhf_status;

enum { RLHF_DTYPE_FP32 = 0, RLHF_DTYPE_BF16 = 1 };

/* Model shape.  Architecture: pre-LayerNorm decoder with parallel residual
 * x <- x + Attn(LN1(x)) + MLP(LN2(x)), exact-erf GELU, rotary embedding on the first rotary_dims
 * of every head (pairs (i, i + rotary_dims/2), angle pos * rope_base^(-2i/rotary_dims)), softmax
 * scale 1/sqrt(head_dim), final LayerNorm before the untied, bias-free LM head and the value head.
 * d_model must equal n_heads * head_dim; rotary_dims must be even and <= head_dim. */
typedef struct {
  int32_t n_layers, d_model, n_heads, head_dim, rotary_dims, d_ff, vocab;
  int32_t dtype;          /* RLHF_DTYPE_FP32 (check mode) or RLHF_DTYPE_BF16: type of every weight */
  int32_t eos_id, pad_id; /* pad_id is written after EOS and never read as an input embedding */
  float ln_eps, rope_base;
} rlhf_model_config;

/* Weights: DEVICE pointers, read-only, caller-owned, must outlive the handle.  Matrices are
 * row-major [out_features, in_features] (y = x W^T + b).  The per-layer members are HOST arrays of
 * n_layers device pointers (the arrays themselves are only read inside rlhf_create). */
typedef struct {
  const void *embed_in;        /* [vocab, d_model] */
  const void *const *ln1_g, *const *ln1_b, *const *ln2_g, *const *ln2_b; /* [d_model] each */
  const void *const *w_qkv, *const *b_qkv; /* [3*d_model, d_model], rows: q of all heads | k | v; [3*d_model] */
  const void *const *w_o, *const *b_o;     /* [d_model, d_model]; [d_model] */
  const void *const *w_fc1, *const *b_fc1; /* [d_ff, d_model]; [d_ff] */
  const void *const *w_fc2, *const *b_fc2; /* [d_model, d_ff]; [d_model] */
  const void *lnf_g, *lnf_b;   /* [d_model] */
  const void *embed_out;       /* [vocab, d_model] */
  const void *value_w;         /* [d_model], or NULL: values are then not computed */
  float value_b;
} rlhf_weights;

typedef struct rlhf_handle rlhf_handle;

/* bf16 mode feeds the matrix cores fp16 operands: the five matrix families (W_qkv with its bias, W_o, W_fc1,
 * W_fc2, embed_out) are read from an fp16 image, converted from the caller's bf16 arrays (exact inside fp16's
 * normal range).  rlhf_weight_image_bytes gives the image's size (0 for an fp32 model; about the size of the
 * bf16 matrices themselves, e.g. 5.5 GB for the 2.8B shape): the caller allocates it, 256-byte aligned, passes
 * it to rlhf_create and keeps it alive and untouched until rlhf_destroy.  Everything else (LayerNorm gains and
 * biases, linear biases other than b_qkv, embed_in, the value head) is read from the caller's arrays directly. */
int rlhf_weight_image_bytes(const rlhf_model_config *cfg, size_t *out);

/* Creates a handle for one model on the current HIP device: allocates the rotary tables and fills the weight
 * image (synchronous).  weight_image: dev buffer of at least rlhf_weight_image_bytes() bytes (may be NULL for an
 * fp32 model); RLHF_EINVAL if it is NULL or misaligned, RLHF_ENOMEM if too small.  *out is NULL on failure. */
int rlhf_create(const rlhf_model_config *cfg, const rlhf_weights *w, void *weight_image,
                size_t weight_image_bytes, rlhf_handle **out);
void rlhf_destroy(rlhf_handle *h);

/* Re-converts the caller's (changed) bf16 matrices into the weight image: call it after an optimizer step
 * (rlhf_adamw_step with param_bf16 = the weight arrays) and before the next forward pass.  Enqueued on
 * `stream`, allocates nothing; a no-op for an fp32 model.  Until it has run, the matrix products still see the
 * previous matrices while LayerNorm parameters, biases and embed_in are already the new ones. */
int rlhf_refresh_weights(rlhf_handle *h, void *stream);

/* Bytes of device workspace that rollout_generate(B, Lq, max_new) and score_sequences(B, L_score)
 * need (the maximum of the two; pass 0 for a call you will not make). */
int rlhf_workspace_bytes(const rlhf_handle *h, int32_t B, int32_t Lq, int32_t max_new, int32_t L_score,
                         size_t *out);

/* Rollout.  queries: dev int32 [B, Lq], left-padded; pad_mask: dev uint8 [B, Lq], 1 = real token
 * (each row's real tokens are its last n_b slots).  Positions count real tokens only and padding
 * never enters attention.  Step t of row b samples argmax_v(logits_v / temperature + g) with
 * Gumbel noise g from a counter hash keyed (seed, seq_id_base + b, t, v); ties go to the lowest id.
 * Outputs (dev):
 *   out_tokens   int32 [B, Lq + max_new]: the query copied, then the response; pad_id after EOS
 *   out_logprobs float [B, max_new]: log softmax(logits/temperature)[token]; 0 after EOS
 *   out_lengths  int32 [B]: response tokens up to and including EOS (max_new if none; 0 for an
 *                all-pad row, whose outputs are all pad_id / 0)
 *   out_mask     uint8 [B, Lq + max_new] or NULL: pad_mask followed by 1 for every kept response
 *                token: with out_tokens, the input of score_sequences
 * One prefill pass and max_new-1 single-token passes are run. */
int rollout_generate(rlhf_handle *h, const int32_t *queries, const uint8_t *pad_mask, int32_t B, int32_t Lq,
                     uint64_t seed, uint64_t seq_id_base, float temperature, int32_t max_new_tokens,
                     int32_t *out_tokens, float *out_logprobs, int32_t *out_lengths, uint8_t *out_mask,
                     void *workspace, size_t workspace_bytes, void *stream);

/* Rescoring.  tokens: dev int32 [B, L]; mask: dev uint8 [B, L], 1 = real; the real tokens of a row
 * must form one contiguous run (left pads from the query, right pads after EOS).
 * Outputs (dev float [B, L]):
 *   out_logprobs[b,t] = log softmax(logits[b,t-1]/temperature)[tokens[b,t]] where t and t-1 are
 *                       real; 0 elsewhere (so 0 at pads and at the first real token)
 *   out_values[b,t]   = value_w . LN_f(x[b,t]) + value_b at real t (unshifted); 0 elsewhere.
 *                       May be NULL. */
int score_sequences(rlhf_handle *h, const int32_t *tokens, const uint8_t *mask, int32_t B, int32_t L,
                    float temperature, float *out_logprobs, float *out_values,
                    void *workspace, size_t workspace_bytes, void *stream);

/* Rescoring of the response only (paper: PPO Details -- the log-probabilities PPO, the KL penalty and the
 * advantages use are those of the response tokens, sliced from the forward pass at the columns from the query
 * length on; values and the reward-model score likewise start at the last query column).  Same inputs and
 * outputs as score_sequences, except that out_logprobs[b,t] is 0 for t < first_col and out_values[b,t] is 0 for
 * t < first_col - 1; the other entries equal score_sequences' up to the rounding order of the kernel variants
 * that the smaller row count selects.  What it saves: the LM head and the
 * final layer's attention output, out-projection and MLP run only on the rows from column first_col - 1 on
 * (every layer still computes K and V for every row).  first_col in [0, L]; 0 or 1 = score_sequences.  The
 * workspace size depends on first_col: rlhf_score_responses_workspace_bytes. */
int rlhf_score_responses_workspace_bytes(const rlhf_handle *h, int32_t B, int32_t L, int32_t first_col,
                                         size_t *out);
int score_responses(rlhf_handle *h, const int32_t *tokens, const uint8_t *mask, int32_t B, int32_t L,
                    int32_t first_col, float temperature, float *out_logprobs, float *out_values,
                    void *workspace, size_t workspace_bytes, void *stream);

/* ---- What PPO consumes after the rollout (stateless: no handle, no workspace). ------------------
 *
 * Reward assembly (paper: Preliminaries, Eq. (RL); Reward Model Details, "Extract reward from the EOS
 * token"; PPO Details, "EOS trick" step 3 and the figure "Reward and values of a completion").
 * For row b let first = index of the first pad_id among its N response tokens (N if none) and
 * last = first - 1.  Then for t <= last
 *   out_rewards[b,t] = -beta * (logprobs[b,t] - ref_logprobs[b,Lq+t])   (+ score_b at t = last)
 * where score_b = rm_values[b,Lq+last] if the token at last is eos_id, else missing_eos_score (the
 * paper's -1); rewards are 0 for t > last, and a row that starts with pad_id is all 0.
 * Inputs (dev): logprobs float [B,N] as written by rollout_generate; ref_logprobs, rm_values float
 * [B,Lq+N] as written by score_sequences (out_logprobs with the reference policy's weights,
 * out_values with the reward model's weights); tokens int32 [B,Lq+N].
 * Outputs (dev): out_rewards float [B,N]; out_scores float [B] (score_b); out_kl float [B]
 * (sum over t <= last of logprobs - ref_logprobs); out_kept int32 [B] (last + 1, the number of
 * response tokens PPO treats as real).  All four outputs are required. */
int rlhf_ppo_assemble_rewards(const float *logprobs, const float *ref_logprobs, const float *rm_values,
                              const int32_t *tokens, int32_t B, int32_t Lq, int32_t N, int32_t eos_id,
                              int32_t pad_id, float beta, float missing_eos_score, float *out_rewards,
                              float *out_scores, float *out_kl, int32_t *out_kept, void *stream);

/* Generalised advantage estimation (paper: PPO hyperparameter table, gamma = 1, lambda = 0.95; the
 * estimator itself is the standard one): over t < kept[b], delta_t = r_t + gamma V_{t+1} - V_t with
 * V = 0 at t+1 >= kept[b], A_t = delta_t + gamma lambda A_{t+1}, returns = A + V; 0 elsewhere.
 * rewards dev float [B,N]; values dev float, element (b,t) at values[b*values_row_stride + t] (so a
 * [B,Lq+N] array from score_sequences is passed as pointer + column offset, stride Lq+N);
 * kept dev int32 [B]; outputs dev float [B,N]. */
int rlhf_ppo_gae(const float *rewards, const float *values, int64_t values_row_stride, const int32_t *kept,
                 int32_t B, int32_t N, float gamma, float lambda, float *out_advantages, float *out_returns,
                 void *stream);

/* Whitening (paper: PPO Details, "(Optional) Reward whitening" and "Advantage whitening"):
 * (x - mean) / sqrt(var + 1e-8) with the biased variance over the positions t < kept[b] of the whole
 * batch (kept == NULL: every position); shift_mean == 0 adds the mean back, as the paper's
 * whiten(rewards, shift_mean=False) does.  Positions that are not kept get 0.  x, out: dev float
 * [B,N] (may be the same buffer). */
int rlhf_ppo_whiten(const float *x, const int32_t *kept, int32_t B, int32_t N, int32_t shift_mean, float *out,
                    void *stream);

/* The PPO objective on a rollout batch and its gradient with respect to the model's outputs (paper:
 * PPO hyperparameter table -- policy clipping coefficient 0.2, value clipping coefficient 0.2, value
 * function coefficient c1 = 0.1, value function loss clipping on; the formulas are the standard
 * ones of that lineage).  Over the kept positions t < kept[b], n of them in the batch:
 *   ratio = exp(new_logprobs - old_logprobs)
 *   pg    = mean max(-A ratio, -A clip(ratio, 1-cliprange, 1+cliprange))
 *   vf    = mean 0.5 max((V - R)^2, (clip(V, Vold - cliprange_value, Vold + cliprange_value) - R)^2)
 *   loss  = pg + vf_coef * vf
 * d_logprobs = d loss / d new_logprobs = -A ratio / n where the unclipped surrogate is the larger or
 * equal one, else 0; d_values = vf_coef (V - R) / n where the unclipped square is the larger or equal
 * one, else 0; both 0 at positions that are not kept.
 * stats dev float [8]: loss, pg, vf, approx_kl = mean 0.5 (new - old)^2, fraction of tokens with the
 * clipped surrogate strictly larger, same for the value term, mean ratio, n.  With n = 0 everything
 * is 0.  All arrays dev float [B,N] over the response positions (contiguous), kept dev int32 [B];
 * every pointer is required.  One launch on `stream`; sums in double in a fixed order. */
int rlhf_ppo_loss(const float *new_logprobs, const float *old_logprobs, const float *advantages,
                  const float *new_values, const float *old_values, const float *returns, const int32_t *kept,
                  int32_t B, int32_t N, float cliprange, float cliprange_value, float vf_coef, float *d_logprobs,
                  float *d_values, float *stats, void *stream);

/* One AdamW update of a flat parameter array (paper: PPO hyperparameter table, "AdamW (eps = 1e-5,
 * lr = 3e-6)"; the algorithm is the published one, Adam with decoupled weight decay), update number
 * `step` >= 1:
 *   g = grad * grad_scale;  p *= 1 - lr * weight_decay;
 *   m = beta1 m + (1 - beta1) g;  v = beta2 v + (1 - beta2) g^2;
 *   p -= lr / (1 - beta1^step) * m / (sqrt(v) / sqrt(1 - beta2^step) + eps)
 * param, exp_avg, exp_avg_sq: dev float [n], updated in place; grad: dev float [n]; param_bf16: dev
 * uint16 [n] or NULL, receives the updated parameters rounded to bf16 (nearest even) -- the storage format of
 * a bf16 model's weights; the forward passes see updated matrices after rlhf_refresh_weights.  fp32 arrays 16-byte aligned, the bf16 array 8-byte aligned; n == 0 is a no-op.  The caller
 * supplies `lr` already scheduled (the paper's linear schedule: lr * (1 - k / K) for update k of K).
 * Arithmetic in fp32; the hyperparameters are doubles, and 1 - beta, lr * weight_decay and the two bias
 * corrections are formed in double on the host before being rounded to fp32.  One launch on
 * `stream`; elementwise, so a model's tensors can be updated as one flat array or one by one. */
int rlhf_adamw_step(float *param, const float *grad, float *exp_avg, float *exp_avg_sq, uint16_t *param_bf16,
                    uint64_t n, int32_t step, double lr, double beta1, double beta2, double eps,
                    double weight_decay, double grad_scale, void *stream);

/* Backward pass through the output heads: from the gradients the loss head returns to the residual
 * stream after the last decoder layer and to the head parameters (paper: the PPO update trains the
 * policy and the value model by gradient descent on the loss of the PPO hyperparameter table; the
 * heads are those of `score_sequences`: Tech stack for the GPT-NeoX final LayerNorm and untied LM
 * head, Preliminaries Step 2 / PPO Details "Value model initializes from the reward model" for the
 * scalar head, the sampling temperature dividing the logits).  For packed rows t < T with
 *   h_t = LN_f(x_t),  z_t = W h_t,  lp_t = log softmax(z_t / temperature)[targets[t]],  v_t = w_v . h_t + b_v
 * and a loss L with dL/dlp_t = d_logprobs[t] (ignored where targets[t] < 0) and dL/dv_t = d_values[t],
 * every output is grad_scale times the gradient of L:
 *   d_x [T, d]            w.r.t. x (the residual stream: what the layers' backward pass continues from)
 *   d_lnf_g, d_lnf_b [d]  w.r.t. the final LayerNorm's gain and bias
 *   d_embed_out [V, d]    w.r.t. the LM head (overwritten, not accumulated)
 *   d_value_w [d], d_value_b [1]   w.r.t. the value head (required iff the model has one, with d_values)
 * x_final: dev float [T, d]; targets: dev int32 [T], the token id row t predicts, or -1; all outputs
 * dev float.  grad_scale (finite) exists because in bf16 mode dL/dz and h are fp16 matrix operands of
 * the two gradient products: pick it so that grad_scale * d_logprobs / temperature is well inside
 * fp16's range, and undo it in rlhf_adamw_step.  Sums over rows run in a fixed order (no
 * floating-point atomics).  Logits exist for 16,384 rows at a time inside the workspace, whose size
 * rlhf_head_backward_workspace_bytes reports; RLHF_ENOMEM if it is smaller.  Work is enqueued on `stream`. */
int rlhf_head_backward_workspace_bytes(const rlhf_handle *h, int32_t T, size_t *out);
int rlhf_head_backward(rlhf_handle *h, const float *x_final, const int32_t *targets, const float *d_logprobs,
                       const float *d_values, int32_t T, float temperature, float grad_scale, float *d_x,
                       float *d_lnf_g, float *d_lnf_b, float *d_embed_out, float *d_value_w, float *d_value_b,
                       void *workspace, size_t workspace_bytes, void *stream);

/* Backward pass through the MLP branch of decoder layer `layer` (paper: as for rlhf_head_backward; the
 * layer is the parallel-residual GPT-NeoX layer of Tech stack, x_out = x + attention(LN1(x)) + mlp(LN2(x)),
 * so this branch is a function of the layer input alone).  With m = LN2(x), u = m W1^T + b1, f = gelu(u)
 * (exact erf form), y = f W2^T + b2 and an upstream gradient d_out = dL/dx_out (any scale: the call is
 * linear in it), the outputs are the gradients of L through this branch:
 *   d_x [T, d]        the branch's term of dL/dx (the residual's identity term d_out is NOT included)
 *   d_ln2_g, d_ln2_b [d];  d_w_fc1 [d_ff, d], d_b_fc1 [d_ff];  d_w_fc2 [d, d_ff], d_b_fc2 [d]   (overwritten)
 * The branch's forward is recomputed from x_in (nothing but the layer inputs has to be kept by a training
 * forward pass).  x_in, d_out: dev float [T, d], packed rows in any order (the branch acts on rows
 * independently); all outputs dev float.  In bf16 mode d_out, f and dL/du are rounded to fp16 as operands of
 * the gradient products: scale d_out into fp16's range (see grad_scale of rlhf_head_backward).  Sums over
 * rows run in a fixed order.  Workspace size from rlhf_mlp_backward_workspace_bytes; RLHF_ENOMEM if smaller. */
int rlhf_mlp_backward_workspace_bytes(const rlhf_handle *h, int32_t T, size_t *out);
int rlhf_mlp_backward(rlhf_handle *h, int32_t layer, const float *x_in, const float *d_out, int32_t T, float *d_x,
                      float *d_ln2_g, float *d_ln2_b, float *d_w_fc1, float *d_b_fc1, float *d_w_fc2, float *d_b_fc2,
                      void *workspace, size_t workspace_bytes, void *stream);

/* Backward pass through packed causal softmax attention, the core of a layer's attention branch
 * (paper: as for rlhf_head_backward; Tech stack for the GPT-NeoX attention).  Stateless: no handle.
 * For every sequence b (packed rows cu_seqlens[b] .. cu_seqlens[b+1]-1) and head h, with Q, K, V the
 * rows' slices [h*head_dim, (h+1)*head_dim) after the rotary turn,
 *   S = Q K^T / sqrt(head_dim),  P = softmax over keys j <= i,  O = P V,
 * and d_out = dL/dO:  dV = P^T dO;  dP = dO V^T;  dS = P * (dP - rowsum(P * dP));
 *   dQ = dS K / sqrt(head_dim);  dK = dS^T Q / sqrt(head_dim).
 * q, k, v, d_out and the outputs dq, dk, dv: dev [T, n_heads*head_dim] row-major, float (dtype
 * RLHF_DTYPE_FP32) or fp16 (RLHF_DTYPE_BF16: the activation type of that mode), 16-byte aligned;
 * cu_seqlens: dev int32 [B+1], increasing from 0 to T; lse_scratch, delta_scratch: dev float [T*n_heads]
 * (left holding the rows' log-sum-exp and sum_j P_ij dP_ij).  max_len (host): at least the longest
 * sequence; longer sequences are cut off at max_len rows (wrong results there, nothing out of bounds).
 * head_dim <= 256 and a multiple of 4 (fp32) or 8 (fp16); arithmetic in fp32; sums in a fixed order.
 * Two launches on `stream`. */
int rlhf_attention_backward(const void *q, const void *k, const void *v, const void *d_out,
                            const int32_t *cu_seqlens, int32_t B, int32_t T, int32_t n_heads, int32_t head_dim,
                            int32_t dtype, int32_t max_len, float *lse_scratch, float *delta_scratch, void *dq,
                            void *dk, void *dv, void *stream);

/* rlhf_attention_backward for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving or training loops, harnesses that forbid hipMalloc): the same kernels and results, with the two
 * per-(row, head) scratch arrays taken from a fixed 8 MB array inside the library instead of from the caller.
 * Limit: T * n_heads <= 1,048,576 (e.g. 32,768 packed rows of 32 heads), otherwise RLHF_EUNSUPPORTED.  The call
 * allocates and frees nothing (its first call on a device looks up the array's address).  Every call on one
 * GPU uses the same array: calls that overlap in time on one GPU race; calls on one stream do not.  All other
 * arguments, errors and alignment rules are those of rlhf_attention_backward. */
int rlhf_attention_backward_noalloc(const void *q, const void *k, const void *v, const void *d_out,
                                    const int32_t *cu_seqlens, int32_t B, int32_t T, int32_t n_heads,
                                    int32_t head_dim, int32_t dtype, int32_t max_len, void *dq, void *dk, void *dv,
                                    void *stream);

/* Backward pass through the attention branch of decoder layer `layer` (paper: as for rlhf_mlp_backward; the
 * other branch of the parallel-residual layer).  With a = LN1(x), [q | k | v] = a Wqkv^T + bqkv, the rotary turn
 * of q and k by each row's position in its sequence, o = packed causal attention (rlhf_attention_backward's
 * forward), y = o Wo^T + bo and an upstream gradient d_out = dL/dx_out (any scale: the call is linear in it):
 *   d_x [T, d]        the branch's term of dL/dx (the residual's identity term d_out is NOT included)
 *   d_ln1_g, d_ln1_b [d];  d_w_qkv [3d, d], d_b_qkv [3d] (rows in the caller's order: q of all heads | k | v);
 *   d_w_o [d, d], d_b_o [d]                                                                    (overwritten)
 * The branch's forward is recomputed from x_in.  x_in, d_out: dev float [T, d], packed rows, sequence b in rows
 * cu_seqlens[b] .. cu_seqlens[b+1]-1 (dev int32 [B+1], from 0 to T), positions counted from each sequence's
 * first row; max_len (host) at least the longest sequence and at most 8192.  In bf16 mode d_out, q, k, v, o and
 * the attention gradients are fp16 (operands of the gradient products): scale d_out into fp16's range.  Sums
 * run in a fixed order.  Workspace size from rlhf_attention_branch_backward_workspace_bytes. */
int rlhf_attention_branch_backward_workspace_bytes(const rlhf_handle *h, int32_t T, size_t *out);
int rlhf_attention_branch_backward(rlhf_handle *h, int32_t layer, const float *x_in, const float *d_out,
                                   const int32_t *cu_seqlens, int32_t B, int32_t T, int32_t max_len, float *d_x,
                                   float *d_ln1_g, float *d_ln1_b, float *d_w_qkv, float *d_b_qkv, float *d_w_o,
                                   float *d_b_o, void *workspace, size_t workspace_bytes, void *stream);

/* ---- The whole backward pass of the policy (with its value head) for one PPO update. ------------------
 *
 * rlhf_forward_keep: the forward pass of score_sequences over tokens / mask (same conventions), keeping what
 * the backward pass needs: x_keep dev float [(n_layers + 1), B*L, d_model] receives the residual stream at the
 * input of every layer and after the last one, packed rows first (row cu[b] + i = token i of sequence b;
 * rows past the number of real tokens are undefined); cu_seqlens dev int32 [B+1] and packed_tokens dev int32
 * [B*L] receive the packing.  Workspace as for score_sequences(B, L).
 *
 * Gradients are returned through rlhf_grads, the mirror of rlhf_weights: DEVICE float arrays of the weights'
 * shapes, overwritten; the per-layer members are HOST arrays of n_layers device pointers; value_w / value_b
 * may be NULL iff the model has no value head.
 *
 * rlhf_policy_backward: from dL/dlogprob and dL/dvalue per packed row (see rlhf_head_backward for targets,
 * d_logprobs, d_values, temperature and grad_scale) through the heads, every layer's two branches (the
 * residual stream's gradient is the sum of the upstream gradient and the two branch terms, added in that
 * order) and the input embedding (rows of equal tokens summed in packed order).  T (host) is the number of
 * real tokens = cu_seqlens[B]; max_len (host) at least the longest sequence.  Everything is grad_scale times
 * the gradient; rlhf_adamw_step divides it out.  (paper: PPO Details / PPO hyperparameter table -- the update
 * is gradient descent on the loss of rlhf_ppo_loss; the model is Tech stack's GPT-NeoX with the scalar head.) */
typedef struct {
  float *embed_in;
  float *const *ln1_g, *const *ln1_b, *const *ln2_g, *const *ln2_b;
  float *const *w_qkv, *const *b_qkv, *const *w_o, *const *b_o;
  float *const *w_fc1, *const *b_fc1, *const *w_fc2, *const *b_fc2;
  float *lnf_g, *lnf_b, *embed_out, *value_w, *value_b;
} rlhf_grads;
int rlhf_forward_keep(rlhf_handle *h, const int32_t *tokens, const uint8_t *mask, int32_t B, int32_t L,
                      float *x_keep, int32_t *cu_seqlens, int32_t *packed_tokens, void *workspace,
                      size_t workspace_bytes, void *stream);
int rlhf_policy_backward_workspace_bytes(const rlhf_handle *h, int32_t T, size_t *out);
int rlhf_policy_backward(rlhf_handle *h, const float *x_keep, int64_t x_keep_layer_stride, const int32_t *cu_seqlens,
                         const int32_t *packed_tokens, int32_t B, int32_t T, int32_t max_len, const int32_t *targets,
                         const float *d_logprobs, const float *d_values, float temperature, float grad_scale,
                         const rlhf_grads *grads, void *workspace, size_t workspace_bytes, void *stream);

/* ---- One PPO update on a rollout batch: K update iterations over mini-batches (paper: PPO hyperparameter table --
 * "K (Number of PPO Update Iteration Per Epoch) 4", "N_mb Number of Mini-batches 1", AdamW (eps 1e-5, lr 3e-6),
 * linear scheduler, clipping coefficients 0.2, c1 0.1, value function loss clipping; PPO Details for the model with
 * its scalar head).  For iteration k < epochs and mini-batch j < n_minibatches (rows j*B/n_minibatches ... of the
 * batch, in row order): the forward pass of the CURRENT weights over tokens / mask (as score_sequences, at
 * `temperature`), keeping the layer inputs; rlhf_ppo_loss of the new log-probs of the N response tokens and the new
 * values at the positions that emitted them (columns Lq-1 .. Lq+N-2) against the rollout's old_logprobs / old_values,
 * advantages, returns and kept [B,N] / [B]; rlhf_policy_backward; rlhf_adamw_step on every tensor with step number
 * first_step + (optimizer steps taken so far in this call) and the given lr (constant within the call: the linear
 * schedule moves once per rollout batch); rlhf_refresh_weights.  The 8 loss statistics of every (k, j) go to
 * out_stats dev float [epochs * n_minibatches, 8].
 *
 * rlhf_train_state: DEVICE float arrays shaped like the weights, in four rlhf_grads-style sets (per-layer members
 * HOST arrays of n_layers device pointers): `grads` (scratch, overwritten), `exp_avg` / `exp_avg_sq` (the optimizer's
 * moments, updated in place) and `master` (bf16 model: the fp32 master weights, updated in place, from which the
 * caller's bf16 weight arrays -- the ones given to rlhf_create -- are rewritten; fp32 model: unused except value_b,
 * the weight arrays themselves are updated).  THE CALL WRITES THE CALLER'S WEIGHT ARRAYS.  value_b: a device float in
 * each set; master.value_b must hold the model's value bias on entry, and from the first call on the handle reads the
 * bias from there (it must outlive the handle) instead of rlhf_weights.value_b.
 * minibatch_tokens: HOST int32 [n_minibatches], the number of real tokens (mask == 1) of each mini-batch; max_len
 * (host): at least the longest row.  grad_scale: see rlhf_head_backward (64 x the kept response tokens of a
 * mini-batch is a good value in bf16 mode; 1 in fp32 mode).  Workspace size from rlhf_ppo_update_workspace_bytes
 * (B_minibatch = B / n_minibatches, L = Lq + N, T_max = the largest entry of minibatch_tokens): that is the minimum.
 * A bf16 model uses whatever the caller passes beyond it to keep FC1's output (before the GELU) of the forward pass
 * instead of recomputing it in the backward pass: T_max * d_ff * 2 bytes (rounded up to 256) per layer, for as many
 * of the first layers as fit; results are the same up to the rounding of the GELU's two forms.  Everything is
 * enqueued on `stream`; no host synchronisation. */
typedef struct {
  int32_t epochs, n_minibatches;            /* the paper: 4, 1 */
  float cliprange, cliprange_value, vf_coef; /* 0.2, 0.2, 0.1 */
  float temperature;                        /* 0.7: the sampling temperature */
  double lr, beta1, beta2, eps, weight_decay;
  int32_t first_step;                       /* >= 1 */
  float grad_scale;
} rlhf_ppo_update_config;
typedef struct {
  rlhf_grads grads, master, exp_avg, exp_avg_sq;
} rlhf_train_state;
int rlhf_ppo_update_workspace_bytes(const rlhf_handle *h, int32_t B_minibatch, int32_t L, int32_t N, int32_t T_max,
                                    size_t *out);
int rlhf_ppo_update(rlhf_handle *h, const rlhf_ppo_update_config *cfg, const rlhf_train_state *state,
                    const int32_t *tokens, const uint8_t *mask, int32_t B, int32_t Lq, int32_t N,
                    const float *old_logprobs, const float *advantages, const float *old_values, const float *returns,
                    const int32_t *kept, const int32_t *minibatch_tokens, int32_t max_len, float *out_stats,
                    void *workspace, size_t workspace_bytes, void *stream);

/* Debug / parity aid: raw (pre-temperature) fp32 logits of the same forward pass as
 * score_sequences at n (row, column) pairs.  rows_bt: HOST int32 [n, 2]; out_logits: dev float
 * [n, vocab].  Every pair must name a real position. */
int rlhf_debug_logits_rows(rlhf_handle *h, const int32_t *tokens, const uint8_t *mask, int32_t B, int32_t L,
                           const int32_t *rows_bt, int32_t n, float *out_logits,
                           void *workspace, size_t workspace_bytes, void *stream);

/* Per-kernel timing for benchmarks.  While enabled, every kernel launch of this handle is bracketed
 * by HIP events on the call's stream.  rlhf_profile_read synchronises the stream's events, then
 * fills up to `cap` entries: names[i] (static strings), total_ms[i], launches[i]; *n_out = number
 * of kernel classes seen.  Reading clears the record. */
int rlhf_profile_enable(rlhf_handle *h, int32_t on);
int rlhf_profile_read(rlhf_handle *h, int32_t cap, const char **names, double *total_ms, int64_t *launches,
                      int32_t *n_out);

/* Marks on the stream between the phases of the last rollout_generate: milliseconds spent in the
 * prefill pass and in the decode loop (synchronises on the call's last event). */
int rlhf_last_rollout_phases(rlhf_handle *h, double *prefill_ms, double *decode_ms);

const char *rlhf_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* RLHF_ROLLOUT_H */
