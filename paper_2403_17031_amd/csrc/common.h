// Shared device helpers and the launcher declarations of the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rlhf {

// ------------------------------------------------------------------------------------------------
// Element types.  bf16_t: the storage type of a bf16 model's weights (raw 16-bit patterns).
// half_t: the type of activations, K/V cache and matrix-core operands in bf16 mode.  Both matrix
// operand types run at the same MFMA rate and occupy the same bytes; fp16's 11-bit significand
// keeps the activation rounding error 8x below bf16's, which the parity bar of this library needs,
// and every bf16 weight converts to fp16 exactly inside fp16's normal range.  Accumulation, the
// residual stream, LayerNorm statistics, softmax and the sampler are always fp32.
// ------------------------------------------------------------------------------------------------
struct bf16_t {
  uint16_t bits;
};
typedef _Float16 half_t;

struct ModeF32 {  // fp32 check mode
  typedef float W;  // weights as stored by the caller
  typedef float A;  // activations and GEMM operands
};
struct ModeBF16 {  // bf16 weights, fp16 operands
  typedef bf16_t W;
  typedef half_t A;
};

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x.bits) << 16); }
__device__ __forceinline__ float to_f32(half_t x) { return (float)x; }

// round-to-nearest-even fp32 -> bf16 (inputs are finite in this library; NaN stays NaN-ish)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
template <typename T>
__device__ __forceinline__ T from_f32(float f);
template <>
__device__ __forceinline__ float from_f32<float>(float f) {
  return f;
}
template <>
__device__ __forceinline__ bf16_t from_f32<bf16_t>(float f) {
  bf16_t r;
  r.bits = f32_to_bf16_bits(f);
  return r;
}
template <>
__device__ __forceinline__ half_t from_f32<half_t>(float f) {  // round to nearest even, saturating
  return (half_t)fminf(fmaxf(f, -65504.0f), 65504.0f);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ------------------------------------------------------------------------------------------------
// Launchers (host).  dtype: 0 = ModeF32, 1 = ModeBF16.  All enqueue on `s` and return the
// launch status.  "n_rows_dev", where present, points to the device-resident row count; the grid
// is sized for the host-side upper bound and surplus blocks exit.
// ------------------------------------------------------------------------------------------------
enum Epilogue {
  EPI_BIAS = 0,         // out[T]   = acc + bias
  EPI_BIAS_GELU = 1,    // out[T]   = gelu_erf(acc + bias)
  EPI_BIAS_RESADD = 2,  // out[f32] += acc + bias      (residual stream update, in place)
  EPI_F32 = 3,          // out[f32] = acc              (logits)
  EPI_LSE = 4,          // nothing stored but per-row softmax statistics of acc/T (scoring LM head)
  EPI_QKV = 5           // acc + bias with the rotary turn applied, q stored as rows, K and V into the cache
};

// EPI_LSE: the product is a [rows, vocab] logits matrix that is never stored.  Each part p (the columns of
// one wave of a tile; gemm_lse_parts() of them per row)
// of packed row t leaves max_v z and sum_v exp(z - max) (z = logit / temperature) in pmax/psum
// [p * stride + t]; the part that holds the row's target token (the next token of the same
// sequence) also leaves its z in ztgt[t].  launch_lse_combine turns these into log-probabilities.
struct LseArgs {
  const int* tok;     // [rows] packed token ids
  const int* pos;     // [rows] packed positions (pos[t+1] == pos[t] + 1 <=> same sequence)
  const int* T_dev;   // number of packed rows
  float inv_temperature;
  float* pmax;
  float* psum;
  float* ztgt;
  int stride;         // rows_max
  int vocab;
  // Rows that are a selection of the packed rows (launch_select_rows): tgt[j] is row j's target token (-1: none)
  // and replaces the tok / pos test; dst[j] is the packed row it stands for.
  const int* tgt = nullptr;
  const int* dst = nullptr;
  const float* val_in = nullptr;  // with dst: per-row values to scatter, val_out[dst[j]] = val_in[j]
  float* val_out = nullptr;
};
// lp_packed[t + 1] = ztgt[t] - logsumexp over the nparts parts, for every t whose successor is in
// the same sequence (with a selection: lp_packed[dst[j] + 1] for every row j with a target).
hipError_t launch_lse_combine(const LseArgs& a, int rows_max, int nparts, float* lp_packed, hipStream_t s);
// The rows of a packed batch from padded column first_col - 1 on (what predicts the tokens at columns >=
// first_col): sel[j] = their packed row, sequence by sequence, j < *n_sel; tgt[j] = the token the row predicts
// (-1 for a sequence's last row).  Entries n_sel .. rows_max-1 are filled with row 0 / -1, so that a gather over
// rows_max entries stays in bounds.  off [B + 1] is scratch (the selection's offsets per sequence).  One block.
hipError_t launch_select_rows(int first_col, int B, const int* start, const int* len, const int* cu, const int* tok,
                              int rows_max, int* sel, int* tgt, int* n_sel, int* off, hipStream_t s);
// Per-row scalars of the selected rows: tgt_out[j] = tgt[sel[j]], a_out[j] = a[sel[j]], b_out[j] = b[sel[j]]
// for j < *n_sel; (-1, 0, 0) for the entries up to rows.  b / b_out may be null.
hipError_t launch_gather_row_scalars(const int* sel, const int* n_sel, int rows, const int* tgt, const float* a,
                                     const float* b, int* tgt_out, float* a_out, float* b_out, hipStream_t s);
// out row sel[j] = in row j for j < *n_sel (distinct rows of row_bytes, a multiple of 16).
hipError_t launch_scatter_rows(const void* in, const int* sel, const int* n_sel, int rows, size_t row_bytes, void* out,
                               hipStream_t s);
// out row r (out_stride bytes apart) = the first row_bytes of in row src[r] (in_stride bytes apart).
hipError_t launch_gather_rows_strided(const void* in, size_t in_stride, const int* src, int rows, size_t row_bytes,
                                      void* out, size_t out_stride, hipStream_t s);
// True when launch_gemm would take EPI_LSE for these arguments (large-M fp16 kernel only).
// EPI_QKV: the product is the [rows, 3*d] QKV matrix in sections q | k | v with the rotary pairs of a
// head in neighbouring columns.  The epilogue adds the bias, turns the pairs by the row's position,
// rounds to fp16 and stores q to q[row, d] and the K / V heads to the cache slot of (sequence, head,
// position): what the product followed by the stand-alone rotary kernel leaves, without the
// [rows, 3*d] intermediate.  Large-M fp16 kernel only.
struct QkvArgs {
  const int* pos;      // [rows] position of a packed row (+ pos_add); rows are indexed from the start of the
                       // packed batch: a launch over a row chunk (GemmArgs::M_sub) adds its offset
  const int* rowid;    // [rows] sequence of a packed row, or null (row = sequence)
  const int* kvoff;    // [sequences] first cache slot of a sequence (in units of H slots)
  const int* len;      // [sequences] real length; a head's slab holds len + kv_extra slots
  const float* cos_t;  // [positions][r/2]
  const float* sin_t;
  void* q;             // [rows, d] fp16
  void* kc;            // K cache, V cache (fp16)
  void* vc;
  long kv_extra;
  int pos_add, H, hd, r;
};
struct GemmArgs;
bool gemm_takes_qkv(int dtype, const GemmArgs& a, int H, int hd, int r);
bool gemm_takes_lse(int dtype, const GemmArgs& a);
bool gemm_takes_k_major(int dtype, const GemmArgs& a);
int gemm_lse_parts(int n_cols);

struct GemmArgs {
  const void* A;      // [M, K] activations, row-major, Mode::A
  const void* W;      // [N, K] weight, row-major, Mode::A (bf16 weights are converted at create)
  const void* bias;   // [N] Mode::W or nullptr
  void* out;          // [M, ldo] (Mode::A or float by epilogue)
  int M_max;          // host upper bound of M
  const int* M_dev;   // device row count or nullptr (then M = M_max)
  int M_sub = 0;      // with M_dev: M = min(M_max, *M_dev - M_sub)  (row chunk starting at M_sub)
  int N, K, ldo;
  int epilogue;
  void* splitk_ws = nullptr;   // fp32 scratch for split-K partial sums (decode-sized M), or null
  size_t splitk_ws_bytes = 0;
  int phase = 0;               // split-K only: 0 = GEMM + reduce, 1 = partial sums only, 2 = reduce only
  const struct LseArgs* lse = nullptr;  // EPI_LSE only
  const struct QkvArgs* qkv = nullptr;  // EPI_QKV only
  int lda = 0, ldw = 0;        // row strides of A and W in elements (0: K); fp16 kernels only
  const void* bias2 = nullptr; // second bias added like the first; large-M fp16 kernel only
  int max_split = 0;           // few-rows kernel: cap on the K split (0: as many as cover the chip)
  bool k_major = false;        // operands given K-major: A is [K, M_max], W is [K, N], row-major, lda / ldw their row
                               // strides (0: M_max / N); out = A^T W, fp32 (EPI_F32), large-M fp16 kernel only: ask
                               // gemm_takes_k_major first
  bool long_k = false;         // large-M kernel, fp32 output, no bias: K may be cut into slices whose fp32 slabs (in
                               // splitk_ws) are then summed in slice order -- for products with few output tiles and
                               // a very long K (weight gradients)
  bool small_footprint = false;  // few rows: stay on the staged tile kernel (24 KB of LDS, 4 blocks per CU), whose
                                 // blocks fit next to another kernel's on a CU; the weight-streaming kernel takes a
                                 // whole CU per block
};
// The few-rows (decode) kernel of gemm_skinny.hip: whether it takes these arguments, the K split it would use,
// and the launch itself (ks > 1: fp32 partial slabs into a.splitk_ws; ks == 1: epilogue in the kernel).
bool gemm_skinny_takes(int dtype, const GemmArgs& a);
int gemm_skinny_splitk(const GemmArgs& a);
void launch_gemm_skinny(const GemmArgs& a, int ks, hipStream_t s);
// True when launch_gemm would route these arguments to the kernel that honours bias2.
bool gemm_takes_bias2(int dtype, const GemmArgs& a);
// > 1 when launch_gemm would take the split-K path for these arguments.
int gemm_splitk_factor(int dtype, const GemmArgs& a);
hipError_t launch_gemm(int dtype, const GemmArgs& a, hipStream_t s);

// Row metadata of a packed batch -------------------------------------------------------------------
// mask [B, L] (1 = real) -> start[b], len[b]; then cu[b] = sum_{b'<b} len, kvoff[b] = sum_{b'<b}
// (len + kv_extra), total[0] = cu[B], total[1] = kvoff[B].
hipError_t launch_row_spans(const uint8_t* mask, int B, int L, int kv_extra, int* start, int* len, int* cu,
                            int* kvoff, int* total, hipStream_t s);
// Packed row t = cu[b] + i for i < len[b]: pos[t] = i, rowid[t] = b, tok[t] = tokens[b, start[b]+i],
// x[t, :] = embed[tok[t], :].
hipError_t launch_pack_embed(int dtype, const int32_t* tokens, int B, int L, const int* start, const int* len,
                             const int* cu, const void* embed, int d, int vocab, int* pos, int* rowid, int* tok,
                             float* x, hipStream_t s);
// Decode step: x[b, :] = embed[cur_tok[b], :] for b < B.
hipError_t launch_gather_rows(const void* in, const int* src, int src_add, int rows, size_t row_bytes, void* out,
                              hipStream_t s);
hipError_t launch_embed_rows(int dtype, const int32_t* tok, int B, const void* embed, int d, int vocab, float* x,
                             hipStream_t s);

// LayerNorm of fp32 rows; two affine outputs from one set of statistics (g2 may be null -> one).
hipError_t launch_layernorm(int dtype, const float* x, int rows_max, const int* rows_dev, int d, float eps,
                            const void* g1, const void* b1, void* out1, const void* g2, const void* b2,
                            void* out2, hipStream_t s);
// Two split-K products (fp32 partial slabs of `slab` floats each, row-major [rows, d]) whose reduction
// into the residual stream is still pending: x <- (x + (sum_z A_z + bias_a)) + (sum_z B_z + bias_b).
struct PendingResidual {
  const float* part_a = nullptr;
  const float* part_b = nullptr;
  const void* bias_a = nullptr;  // bf16 [d]
  const void* bias_b = nullptr;
  int ks_a = 0, ks_b = 0;
  size_t slab = 0;
};
bool layernorm_pending_supported(int dtype, int rows_max, int d);
// LayerNorm as above, after folding the pending products into x (written back in place).
hipError_t launch_layernorm_pending(float* x, int rows_max, const int* rows_dev, int d, float eps, const void* g1,
                                    const void* b1, void* out1, const void* g2, const void* b2, void* out2,
                                    const PendingResidual& pend, hipStream_t s);
// Final LayerNorm of selected rows: row r reads x[src[r]] (src may be null: identity), optionally
// also the value head val[r] = w_v . h + b_v.
hipError_t launch_final_ln(int dtype, const float* x, const int* src, int src_add, int rows_max,
                           const int* rows_dev, int d, float eps, const void* g, const void* b, void* out,
                           const void* value_w, float value_b, float* val, hipStream_t s);

// K/V layout: sequence b owns the slab of slots [kvoff[b]*H, kvoff[b+1]*H); inside it head h has
// len[b] + kv_extra consecutive rows of hd elements (kv_extra = room for generated tokens), so one
// (sequence, head) pair is one contiguous run and a sequence's heads are neighbours.
// Rotary on q,k (first r dims of each head) + K/V store.  qkv [rows, 3d] -> q [rows, d] and
// kc/vc at row pos[t] + pos_add of (sequence rowid[t], head h).  rowid may be null (row t is
// sequence t).  cos/sin tables are [max_pos][r/2].
hipError_t launch_rope_kv(int dtype, const void* qkv, int rows_max, const int* rows_dev, const int* pos,
                          int pos_add, const int* rowid, const int* kvoff, const int* len, int H, int hd, int r,
                          const float* cos_t, const float* sin_t, void* q, void* kc, void* vc,
                          long kv_extra, hipStream_t s);

// Same, one row per sequence, with the qkv row formed from the fp32 partial slabs of a split-K
// product (`slab` floats each, row-major [rows, 3*H*hd]) plus bias instead of being read.
bool rope_kv_splitk_supported(int dtype, int H, int hd, int r);
hipError_t launch_rope_kv_splitk(const float* part, int ksplit, size_t slab, const void* bias, int rows_max,
                                 const int* rows_dev, const int* pos, int pos_add, const int* rowid,
                                 const int* kvoff, const int* len, int H, int hd, int r, const float* cos_t,
                                 const float* sin_t, void* q, void* kc, void* vc, long kv_extra, hipStream_t s);

// Causal attention over packed sequences (prefill / scoring).  q [T, H*hd]; kc/vc [H][*][hd] with
// sequence b's keys at slots kvoff[b] .. kvoff[b]+len[b]; out [T, H*hd].
hipError_t launch_attn_prefill(int dtype, const void* q, const void* kc, const void* vc, long kv_extra,
                               int B, int Lmax, const int* len, const int* cu, const int* kvoff, int H, int hd,
                               void* out, int out_ld, hipStream_t s);
// Decode attention: one query row per sequence against ctx = len[b] + ctx_add cached keys.
hipError_t launch_attn_decode(int dtype, const void* q, const void* kc, const void* vc, long kv_extra,
                              int B, const int* len, int ctx_add, int ctx_max, const int* kvoff, int H, int hd,
                              void* out, hipStream_t s);

// Sampler: one step for every row from fp32 logits [B, V].
struct SampleArgs {
  const float* logits;
  int B, V, Lq, N, step;
  uint64_t seed, seq_base;
  float temperature;
  int eos_id, pad_id;
  const int* len;       // true query lengths (0 = all-pad row)
  int* finished;        // [B] state, initialised at step 0
  int32_t* cur_tok;     // [B] token fed to the next pass
  int32_t* out_tokens;  // [B, Lq+N]
  float* out_logprobs;  // [B, N]
  int32_t* out_lengths; // [B]
  uint8_t* out_mask;    // [B, Lq+N] or null
};
hipError_t launch_sampler(const SampleArgs& a, hipStream_t s);
hipError_t launch_copy_queries(const int32_t* queries, const uint8_t* pad_mask, int B, int Lq, int N, int pad_id,
                               int32_t* out_tokens, uint8_t* out_mask, hipStream_t s);

// Scoring: log softmax(logits[t]/T)[tok[t+1]] for packed rows t0 .. t0+rows of a logits chunk;
// result goes to lp_packed[t+1] when t+1 belongs to the same sequence.
hipError_t launch_lse_gather(const float* logits, int rows_max, int t0, const int* T_dev, int V,
                             float temperature, const int* tok, const int* pos, float* lp_packed,
                             hipStream_t s);
// Packed -> padded [B, L] outputs with zeros at masked slots; logprob of a row's first token is 0.
// val_bias_dev: optional device scalar added to every real position's value (a value-head bias that lives on the
// device because an optimizer updates it there).
// first_col: log-probs of columns before it and values of columns before first_col - 1 are written as 0.
hipError_t launch_unpack_scores(const float* lp_packed, const float* val_packed, int B, int L, const int* start,
                                const int* len, const int* cu, float* out_lp, float* out_val, hipStream_t s,
                                const float* val_bias_dev = nullptr, int first_col = 0);
// Gather helper for the debug entry point: idx[i] = cu[b_i] + (col_i - start[b_i]).
hipError_t launch_rows_to_packed(const int32_t* rows_bt, int n, const int* start, const int* cu, int* idx,
                                 hipStream_t s);

// PPO signals (reward assembly, advantage estimation, whitening); see ppo_signals.hip.
hipError_t launch_ppo_rewards(const float* lp, const float* ref_full, const float* rm_full, const int* tokens, int B,
                              int Lq, int N, int eos_id, int pad_id, float beta, float miss, float* rewards,
                              float* scores, float* kl, int* kept, hipStream_t s);
hipError_t launch_ppo_gae(const float* rewards, const float* values, long vstride, const int* kept, int B, int N,
                          float gamma, float lam, float* adv, float* ret, hipStream_t s);
hipError_t launch_ppo_whiten(const float* x, const int* kept, int B, int N, int shift_mean, float* out,
                             hipStream_t s);
hipError_t launch_ppo_loss(const float* lp, const float* lp0, const float* adv, const float* v, const float* v0,
                           const float* ret, const int* kept, int B, int N, float eps, float eps_v, float c1,
                           float* d_lp, float* d_v, float* stats, hipStream_t s);
// The PPO update's glue between the padded [B, L] outputs of a forward pass and the packed rows of the backward
// pass.  Slices: new_lp[b, j] = lp_full[b, Lq + j], new_v[b, j] = val_full[b, Lq - 1 + j] (j < N).
hipError_t launch_ppo_slice(const float* lp_full, const float* val_full, int B, int L, int Lq, int N, float* new_lp,
                            float* new_v, hipStream_t s);
// Packed row cu[b] + i holds token (b, c = start[b] + i); it predicts token (b, c + 1):
//   targets = that token if it is real, else -1;  gl = d_lp[b, c + 1 - Lq] if that is a response position, else 0;
//   gv = d_v[b, c - (Lq - 1)] if 0 <= c - (Lq - 1) < N, else 0.
hipError_t launch_ppo_pack_grads(const int32_t* tokens, int B, int L, int Lq, int N, const int* start, const int* len,
                                 const int* cu, const float* d_lp, const float* d_v, int32_t* targets, float* gl,
                                 float* gv, hipStream_t s);
// Optimizer step (optimizer.hip).
hipError_t launch_adamw(float* p, const float* g, float* m, float* v, uint16_t* p_bf16, size_t n, float decay,
                        float beta1, float omb1, float beta2, float omb2, float step_size, float inv_sqrt_bias2,
                        float eps, float grad_scale, hipStream_t s);

// bf16 -> fp16 conversion of a weight matrix (exact within fp16's normal range).
// ---- backward through the output heads (head_backward.hip); dtype 0: float operands, 1: fp16 ----
// dst[c][r] = src[r][c] (r < R, c < C); dst columns R .. R_pad-1 are zeroed.
hipError_t launch_transpose_pad(int dtype, const void* src, size_t ld_src, void* dst, size_t ld_dst, int R, int C,
                                int R_pad, hipStream_t s);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);  // bytes: a multiple of 4
// dz[r][v] = gl[r] * scale * inv_temp * (onehot(targets[r])[v] - softmax(logits[r] * inv_temp)[v]) for r < rows with
// a target; zero for rows without one, rows rows .. rows_pad-1 and columns V .. V_pad-1.
hipError_t launch_softmax_grad(int dtype, const float* logits, int V, int V_pad, const int* targets, const float* gl,
                               int rows, int rows_pad, float inv_temp, float scale, void* dz, hipStream_t s);
// dy = dhl + gv * scale * value_w; dx = LayerNorm input gradient of dy; d_g = sum_t dy * xhat, d_b = sum_t dy,
// d_wv = sum_t gv * scale * h, d_bv = scale * sum_t gv.  stats [T, 2] and part [splits, 3, d] are scratch.
// LayerNorm backward of a layer (no value-head term) in one pass: dx, d_g = sum_t dy * xhat, d_b = sum_t dy.
// bf16 parameters, d a multiple of 256 up to 4096; part: ln_backward_rows_scratch_floats(T, d) floats of scratch.
bool ln_backward_rows_supported(int dtype, int d);
size_t ln_backward_rows_scratch_floats(int T, int d);
// base (optional): dx = base + the LayerNorm input gradient (rows of d floats like dx).
hipError_t launch_ln_backward_rows(const float* x, const float* dy, const void* g, int T, int d, float eps, float* dx,
                                   float* part, float* d_g, float* d_b, hipStream_t s, const float* base = nullptr);
// sums[c] = sum_r a[r][c] of a float [R, C] matrix (C a multiple of 4) and out_f16 = its fp16 copy, in one pass;
// part: [splits][C] floats of scratch.
hipError_t launch_convert_colsum(const float* a, int R, int C, float* part, int splits, float* sums, void* out_f16,
                                 hipStream_t s);
hipError_t launch_head_ln_backward(int dtype, const float* x, const float* dhl, const float* gv, float scale,
                                   const void* value_w, const void* g, const void* b, int T, int d, float eps,
                                   float* dx, float* stats, float* part, int splits, float* d_g, float* d_b,
                                   float* d_wv, float* d_bv, hipStream_t s);

// Element-wise pieces of a layer's backward pass (dtype 0: float activations, 1: fp16).
hipError_t launch_gelu(int dtype, const void* u, void* f, size_t n, hipStream_t s);            // f = gelu(u)
// the same on fp16 rows with strides (elements; cols and strides multiples of 8, 16-byte aligned bases)
hipError_t launch_gelu_rows_f16(const void* u, size_t ld_u, void* f, size_t ld_f, int rows, int cols, hipStream_t s);
hipError_t launch_gelu_backward(int dtype, const void* u, void* df, size_t n, hipStream_t s);  // df *= gelu'(u)
// the same on an fp16 [R, C] matrix together with the column sums of the result (sums[c]; part: [splits][C] scratch)
bool gelu_backward_colsum_supported(int dtype, const void* u, const void* df, int C);
hipError_t launch_gelu_backward_colsum(const void* u, void* df, int R, int C, float* part, int splits, float* sums,
                                       hipStream_t s);
hipError_t launch_convert_from_f32(int dtype, const float* src, void* dst, size_t n, hipStream_t s);
// out[c] = sum_r a[r][c] over a contiguous [R, C] matrix (elem 0: float, 1: fp16); part: [splits][C] scratch.
hipError_t launch_colsum(int elem, const void* a, int R, int C, float* part, int splits, float* out, hipStream_t s);

// Backward of packed causal attention (attention_backward.hip): q, k, v, g = dO and the outputs dq, dk, dv are
// [T, H*hd] row-major in float (dtype 0) or fp16 (1); cu [B+1] packed-row offsets of the sequences;
// lse, delta: [T*H] floats of scratch.  hd a multiple of 4 (float) or 8 (fp16); sequences of at most max_len rows.
hipError_t launch_attention_backward(int dtype, const void* q, const void* k, const void* v, const void* g,
                                     const int* cu, int B, int Tn, int H, int hd, int max_len, float* lse,
                                     float* delta, void* dq, void* dk, void* dv, hipStream_t s, size_t ld_qkv = 0,
                                     size_t ld_g = 0, size_t ld_out = 0, void* o = nullptr, size_t ld_o = 0,
                                     bool kv_cache = false);
// (row strides in elements: ld_qkv of q, k, v; ld_g of g; ld_out of dq, dk, dv; 0 = H*hd.  o: optional forward
// output O = P V, [T, ld_o].  kv_cache: k and v are a layer's K / V cache as the forward pass of a packed batch
// leaves it -- sequence b's slab starts at slot cu[b] * H, head h of it holds the sequence's rows consecutively --
// and ld_qkv is q's stride alone; only where attention_backward_takes_cache says so.)
bool attention_backward_takes_cache(int dtype, int hd);

// Rotary turn, in place, of the q and k sections of a [T, 3*d] matrix (row stride ld) by each row's position in
// its sequence; backward != 0 applies the transpose (turn by the negative angle).  dtype 1 uses the reordered
// pair layout (2i, 2i+1) of the fp16 path, dtype 0 the pairs (i, i + r/2).
hipError_t launch_rope_inplace(int dtype, void* qkv, size_t ld, const int* cu, int B, int Tn, int H, int hd, int r,
                               const float* cos_t, const float* sin_t, int backward, hipStream_t s);
// Rows of a [3*d, C] fp32 matrix from the fp16 path's reordered W_qkv row order back to the caller's.
hipError_t launch_qkv_rows_to_caller_order(const float* in, float* out, int d, int hd, int r, int C, hipStream_t s);

// out[v][:] = sum over packed rows t with tok[t] == v of dx[t][:], in increasing t; out is [V, d], d <= 8192.
hipError_t launch_embed_backward(const int* tok, const float* dx, int T, int d, int V, float* out, hipStream_t s);
hipError_t launch_add3(const float* a, const float* b, const float* c, float* out, size_t n, hipStream_t s);  // (a+b)+c

hipError_t launch_bf16_to_f16(const void* src, void* dst, size_t n, hipStream_t s);
// Same for a [rows, cols] matrix written with row stride dst_ld (elements).
// fp16 copy of W_qkv and a bf16 copy of its bias with the rotary dims of every q and k head
// reordered pairwise ((i, i + r/2) -> (2i, 2i + 1)): the layout every fp16 rotary kernel assumes.
hipError_t launch_qkv_weights_f16(const void* w, const void* b, void* w16, void* b_out, int d, int hd, int r,
                                  hipStream_t s);
hipError_t launch_bf16_to_f16_2d(const void* src, void* dst, size_t rows, size_t cols, size_t dst_ld, hipStream_t s);

}  // namespace rlhf
