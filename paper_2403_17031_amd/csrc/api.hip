// C ABI and host-side orchestration: validates arguments, carves the caller's workspace and
// enqueues the kernels of rollout_generate / score_sequences on the caller's stream.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/rlhf_rollout.h"
#include "common.h"

using namespace rlhf;

namespace {

thread_local std::string g_err;

int fail(int code, const std::string& msg) {
  g_err = msg;
  return code;
}

#define HIP_OK(expr)                                                                              \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess)                                                                         \
      return fail(RLHF_EHIP, std::string(#expr) + ": " + hipGetErrorString(e_));                  \
  } while (0)

constexpr int kMaxPos = 8192;

// Scratch of the allocation-free attention backward: log-sum-exp and delta, one float per (row, head) each.
// Every GPU the library runs on holds its own 8 MB copy until the process ends.
constexpr size_t kStaticScratchFloats = (size_t)1 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) float g_static_scratch[2 * kStaticScratchFloats];
float* g_static_scratch_ptr[kMaxDevices] = {};  // device address of the array, per device (host code never uses its name)
std::mutex g_static_scratch_mu;
constexpr int kLogitChunk = 4096;  // rows of fp32 logits materialised at a time while scoring

struct Carver {  // bump allocator over the workspace; base == nullptr only measures
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base((char*)b) {}
  template <typename T>
  T* take(size_t n) {
    off = (off + 255) & ~(size_t)255;
    T* p = base ? (T*)(base + off) : nullptr;
    off += n * sizeof(T);
    return p;
  }
  void* take_bytes(size_t n) { return take<char>(n); }
};

struct Meta {
  int *start, *len, *cu, *kvoff, *total, *pos, *rowid, *tok;
};
struct Acts {
  float* x;
  void *a, *m, *qkv, *q, *att, *ffn;  // att and ffn are carved back to back: [rows, d + d_ff] when viewed as one
  void* splitk = nullptr;   // fp32 partial sums of the decode GEMMs (attention branch)
  void* splitk2 = nullptr;  // same for the MLP branch, which runs on a second stream
  size_t splitk_bytes = 0;
};

}  // namespace

struct rlhf_handle {
  rlhf_model_config cfg;
  rlhf_weights w;
  std::vector<const void*> ln1_g, ln1_b, ln2_g, ln2_b, w_qkv, b_qkv, w_o, b_o, w_fc1, b_fc1, w_fc2, b_fc2;
  // the caller's own arrays of the tensors that bf16 mode reads through the fp16 image (sources of a refresh)
  std::vector<const void*> src_w_qkv, src_b_qkv, src_w_o, src_w_fc1, src_w_fc2;
  float *rope_cos = nullptr, *rope_sin = nullptr;
  void* w16 = nullptr;                // bf16 mode: fp16 image of the matrices the GEMMs read (caller's buffer)
  const void* embed_out_mm = nullptr; // LM-head operand (the caller's in fp32 mode, the copy in bf16 mode)
  // bf16 mode: the fp16 copies of the out-projection [d, d] and FC2 [d, d_ff] of a layer sit side by
  // side as one [d, d + d_ff] matrix (w_o = its column 0, w_fc2 = its column d, both with this row
  // stride), so that prefill / scoring can run them as a single product over K = d + d_ff
  int ld_o2 = 0;
  size_t esz = 2;
  // once an update has run, the value head's bias lives on the device (the optimizer updates it there)
  const float* value_b_dev = nullptr;
  // profiling
  bool prof_on = false;
  std::vector<const char*> prof_names;
  std::vector<hipEvent_t> prof_ev;  // pairs
  std::vector<hipEvent_t> ev_pool;
  size_t ev_used = 0;
  hipEvent_t ph[3] = {nullptr, nullptr, nullptr};
  bool ph_valid = false;
  // decode runs the MLP branch of the parallel-residual layer on a second stream (default priority)
  hipStream_t side = nullptr;
  hipEvent_t fork_ev[8] = {}, join_ev[8] = {};
  unsigned ev_rr = 0;

  hipEvent_t get_event() {
    if (ev_used == ev_pool.size()) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) return nullptr;
      ev_pool.push_back(e);
    }
    return ev_pool[ev_used++];
  }
};

namespace {

struct ProfScope {
  rlhf_handle* h;
  hipStream_t s;
  ProfScope(rlhf_handle* h_, const char* name, hipStream_t s_) : h(h_), s(s_) {
    if (!h->prof_on) return;
    hipEvent_t e = h->get_event();
    if (!e) return;
    (void)hipEventRecord(e, s);
    h->prof_names.push_back(name);
    h->prof_ev.push_back(e);
  }
  ~ProfScope() {
    if (!h->prof_on) return;
    hipEvent_t e = h->get_event();
    if (!e) return;
    (void)hipEventRecord(e, s);
    h->prof_ev.push_back(e);
  }
};

#define LAUNCH(name, call)                                                                        \
  do {                                                                                            \
    hipError_t e_;                                                                                \
    {                                                                                             \
      ProfScope ps_(h, name, s);                                                                  \
      e_ = (call);                                                                                \
    }                                                                                             \
    if (e_ != hipSuccess) return fail(RLHF_EHIP, std::string(name) + ": " + hipGetErrorString(e_)); \
  } while (0)

Meta carve_meta(Carver& c, int B, size_t Tmax) {
  Meta m;
  m.start = c.take<int>(B);
  m.len = c.take<int>(B);
  m.cu = c.take<int>(B + 1);
  m.kvoff = c.take<int>(B + 1);
  m.total = c.take<int>(2);
  m.pos = c.take<int>(Tmax);
  m.rowid = c.take<int>(Tmax);
  m.tok = c.take<int>(Tmax);
  return m;
}

Acts carve_acts(Carver& c, const rlhf_model_config& cfg, size_t rows, size_t esz) {
  Acts a;
  const size_t d = cfg.d_model;
  a.x = c.take<float>(rows * d);
  a.a = c.take_bytes(rows * d * esz);
  a.m = c.take_bytes(rows * d * esz);
  a.qkv = c.take_bytes(rows * 3 * d * esz);
  a.q = c.take_bytes(rows * d * esz);
  a.att = c.take_bytes(rows * (d + (size_t)cfg.d_ff) * esz);
  a.ffn = (char*)a.att + rows * d * esz;
  return a;
}

struct RolloutWs {
  Meta meta;
  Acts acts;
  Acts last;  // [B, .] activations of the final prefill layer's last-position rows
  int *finished, *cur_tok;
  void* hl;
  float* logits;
  char* kv;
  size_t kv_slots;
};
RolloutWs carve_rollout(Carver& c, const rlhf_model_config& cfg, int B, int Lq, int N, size_t esz) {
  RolloutWs w;
  const size_t Tmax = (size_t)B * Lq;
  w.meta = carve_meta(c, B, Tmax);
  w.acts = carve_acts(c, cfg, Tmax, esz);
  w.finished = c.take<int>(B);
  w.cur_tok = c.take<int>(B);
  w.hl = c.take_bytes((size_t)B * cfg.d_model * esz);
  w.logits = c.take<float>((size_t)B * cfg.vocab);
  w.acts.splitk_bytes = (size_t)16 * B * std::max(3 * cfg.d_model, cfg.d_ff) * sizeof(float);
  w.acts.splitk = c.take_bytes(w.acts.splitk_bytes);
  w.acts.splitk2 = c.take_bytes(w.acts.splitk_bytes);
  w.last = carve_acts(c, cfg, (size_t)B, esz);
  w.last.splitk_bytes = w.acts.splitk_bytes;
  w.last.splitk = w.acts.splitk;  // decode has not started: its partial-sum scratch is free
  w.kv_slots = (size_t)B * (Lq + N - 1);
  w.kv = (char*)c.take_bytes((size_t)cfg.n_layers * 2 * w.kv_slots * cfg.d_model * esz);
  return w;
}

struct ScoreWs {
  Meta meta;
  Acts acts;
  char* kv;  // one layer: [2][H][Tmax][hd]
  float *val, *lp, *logits;
  float *pmax = nullptr, *psum = nullptr, *ztgt = nullptr;  // fused LM head: per-part softmax statistics
  int nparts = 0;
  bool fused_lm = false;
  int* idx;
  int32_t* rows_dev;
  size_t Tmax;
  int chunk;
  // Scoring from a first column on (score_responses): only the rows from column first_col - 1 on go through the
  // LM head (and, outside the training forward, through the final layer's attention output, out-projection and MLP).
  // sel_rows = 0: no selection, every row is computed and the outputs before first_col are just written as 0.
  int first_col = 0;
  int sel_rows = 0;            // host bound of the selected rows, B * (L - first_col + 1)
  int *sel = nullptr, *tgt = nullptr, *n_sel = nullptr, *sel_off = nullptr;
  Acts z;                      // [sel_rows, .] activations of the selected rows
  float* val_sel = nullptr;
  bool sel_layers = false;     // set by score_forward: the final layer ran on the selected rows, z.x holds its output
};
ScoreWs carve_score(Carver& c, const rlhf_model_config& cfg, int B, int L, size_t esz, int first_col = 0) {
  ScoreWs w;
  w.Tmax = (size_t)B * L;
  w.meta = carve_meta(c, B, w.Tmax);
  w.acts = carve_acts(c, cfg, w.Tmax, esz);
  w.kv = (char*)c.take_bytes(2 * w.Tmax * cfg.d_model * esz);
  w.val = c.take<float>(w.Tmax);
  w.lp = c.take<float>(w.Tmax);
  // the LM head either keeps the logits in registers and leaves per-part statistics (large batches),
  // or materialises them for a chunk of rows at a time
  GemmArgs lf;
  lf.A = nullptr; lf.W = nullptr; lf.bias = nullptr; lf.out = nullptr;
  lf.M_max = (int)w.Tmax; lf.M_dev = nullptr;
  lf.N = cfg.vocab; lf.K = cfg.d_model; lf.ldo = cfg.vocab; lf.epilogue = EPI_LSE;
  w.fused_lm = gemm_takes_lse(cfg.dtype, lf);
  w.first_col = std::max(first_col, 0);
  if (w.first_col > 1 && w.first_col <= L && w.fused_lm) {
    lf.M_max = B * (L - w.first_col + 1);
    if (gemm_takes_lse(cfg.dtype, lf)) w.sel_rows = lf.M_max;
  }
  const size_t lm_rows = w.sel_rows ? (size_t)w.sel_rows : w.Tmax;
  w.chunk = (int)std::min<size_t>(w.Tmax, kLogitChunk);
  w.logits = w.fused_lm ? nullptr : c.take<float>((size_t)w.chunk * cfg.vocab);
  w.nparts = gemm_lse_parts(cfg.vocab);
  if (w.fused_lm) {
    w.pmax = c.take<float>((size_t)w.nparts * lm_rows);
    w.psum = c.take<float>((size_t)w.nparts * lm_rows);
    w.ztgt = c.take<float>(lm_rows);
  }
  if (w.sel_rows) {
    w.sel = c.take<int>(w.sel_rows);
    w.tgt = c.take<int>(w.sel_rows);
    w.n_sel = c.take<int>(1);
    w.sel_off = c.take<int>(B + 1);
    w.z = carve_acts(c, cfg, (size_t)w.sel_rows, esz);
    w.val_sel = c.take<float>(w.sel_rows);
  }
  w.idx = c.take<int>(w.Tmax);
  w.rows_dev = c.take<int32_t>(2 * w.Tmax);
  return w;
}

// One pass through all decoder layers.  mode 0: packed causal attention over whole sequences
// (prefill, scoring); mode 1: one new row per sequence against the cache (decode).
struct PassArgs {
  int mode;
  int rows_max;
  const int* rows_dev;
  const int* pos;
  int pos_add;
  const int* rowid;
  const int* kvoff;
  const int* len;
  const int* cu;
  int B, Lmax;
  int ctx_add, ctx_max;
  int kv_extra;        // slots per head beyond len[b] in a sequence's K/V slab
  char* kv;            // layer l: K at kv + (2l)*kv_layer_bytes/2 ...
  size_t kv_slots;     // slots per head
  bool kv_per_layer;   // false: every layer reuses the same single-layer scratch
  // Prefill of a rollout only needs the last position of every sequence after the final layer
  // (the first sampled token comes from it): when `last` is set, the final layer computes K and V
  // for every row as usual, but attention, out-projection and MLP run on the B gathered last rows
  // only, into last->x ([B, d], row b = sequence b).
  const Acts* last = nullptr;
  // Training forward: when set, the residual stream at the input of layer l is copied to
  // keep + l * keep_stride (rows_max rows), and the stream after the last layer to slot n_layers.
  float* keep = nullptr;
  size_t keep_stride = 0;
  size_t keep_rows = 0;
  // Scoring from a first column on: when `sel` is set, the final layer computes K and V for every row as usual
  // and attention for every query, but the out-projection and the MLP run on the sel_rows selected rows only
  // (sel[j] = packed row, *n_sel of them), into selz->x.
  const int* sel = nullptr;
  const int* n_sel = nullptr;
  int sel_rows = 0;
  const Acts* selz = nullptr;
  // Training forward that also keeps every layer's QKV product: layer l's rotated q rows go to q_keep + l *
  // q_keep_stride bytes instead of the pass's own q buffer (its K / V are kept through kv_per_layer).
  char* q_keep = nullptr;
  size_t q_keep_stride = 0;
  // ... and, for the first u_keep_layers layers, FC1's output before the GELU (keep_rows rows of d_ff each, layer l at
  // u_keep + l * u_keep_stride bytes): those layers run FC1 with the plain bias epilogue and the GELU as a pass of its own.
  char* u_keep = nullptr;
  size_t u_keep_stride = 0;
  int u_keep_layers = 0;
};

int run_layers(rlhf_handle* h, const Acts& A, const PassArgs& p, hipStream_t s) {
  const rlhf_model_config& c = h->cfg;
  if (c.n_layers == 0) {  // nothing to run (and no layer 0 to take shapes from below)
    if (p.keep)
      HIP_OK(hipMemcpyAsync(p.keep, A.x, p.keep_rows * c.d_model * sizeof(float), hipMemcpyDeviceToDevice, s));
    return RLHF_OK;
  }
  const int d = c.d_model, dt = c.dtype;
  const size_t plane = p.kv_slots * (size_t)d * h->esz;  // bytes of one K (or V) plane of one layer

  GemmArgs base;
  base.M_max = p.rows_max;
  base.M_dev = p.rows_dev;
  if (p.mode == 1) {
    base.splitk_ws = A.splitk;
    base.splitk_ws_bytes = A.splitk_bytes;
  }
  auto gemm_args = [&](const void* in, const void* w, const void* bias, void* out, int N, int K, int epi) {
    GemmArgs g = base;
    g.A = in; g.W = w; g.bias = bias; g.out = out; g.N = N; g.K = K; g.ldo = N; g.epilogue = epi;
    return g;
  };

  // Decode with every product on the split-K path: the reductions of the partial sums are folded
  // into the kernels that consume them (QKV into the rotary kernel; out-projection and FC2 into the
  // next layer's LayerNorm), which takes four short kernels per layer off the critical path.
  // Decode products.  QKV and the out-projection sit on the critical path of a layer and run alone on the chip:
  // they take the weight-streaming kernel, K split 4 ways (more splits shorten them further but cost the next
  // LayerNorm / rotary kernel as much again in partial sums to add up).  FC1 and FC2 run in the shadow of the
  // attention kernel on a second stream: there the staged tile kernel's small blocks, which fit on a CU next to
  // attention blocks, do better than blocks that each take a whole CU (measured: decode 476 against 525-580 ms).
  const int cap_qkv = 4, cap_o = 4, cap_1 = 0, cap_2 = 0;
  const bool mlp_small = p.mode == 1;
  auto capped = [](GemmArgs g, int cap) {
    g.max_split = cap;
    return g;
  };
  int ks_qkv = 1, ks_o = 1, ks_2 = 1;
  if (p.mode == 1) {
    ks_qkv = gemm_splitk_factor(dt, capped(gemm_args(A.a, nullptr, nullptr, A.qkv, 3 * d, d, EPI_BIAS), cap_qkv));
    ks_o = gemm_splitk_factor(dt, capped(gemm_args(A.att, nullptr, nullptr, A.x, d, d, EPI_BIAS_RESADD), cap_o));
    GemmArgs t2 = capped(gemm_args(A.ffn, nullptr, nullptr, A.x, d, c.d_ff, EPI_BIAS_RESADD), cap_2);
    t2.small_footprint = mlp_small;
    ks_2 = gemm_splitk_factor(dt, t2);
  }
  const bool fold = p.mode == 1 && ks_qkv > 1 && ks_o > 1 && ks_2 > 1 &&
                    rope_kv_splitk_supported(dt, c.n_heads, c.head_dim, c.rotary_dims) &&
                    layernorm_pending_supported(dt, p.rows_max, d);
  // Decode: the MLP branch (weights streaming through the matrix cores) overlaps the attention
  // branch (K/V streaming from HBM).  Needs FC2 on the split-K path, so that only its final
  // reduction touches the residual stream; not used while per-kernel profiling is on.
  const bool fork_mlp = p.mode == 1 && !h->prof_on && ks_2 > 1;
  // Prefill / scoring: out-projection and FC2 both add into the residual stream, so they run as one
  // product over the concatenated K = d + d_ff when the large-M kernel takes that shape.
  auto gcat = [&](int l) {
    GemmArgs g = gemm_args(A.att, h->w_o[l], h->b_o[l], A.x, d, d + c.d_ff, EPI_BIAS_RESADD);
    g.bias2 = h->b_fc2[l];
    return g;
  };
  const bool cat = p.mode == 0 && h->ld_o2 != 0 && gemm_takes_bias2(dt, gcat(0));
  const size_t slab = (size_t)p.rows_max * d;
  bool pending = false;  // out-projection and FC2 partial sums of the previous layer not yet in x

  for (int l = 0; l < c.n_layers; ++l) {
    if (p.keep)
      HIP_OK(hipMemcpyAsync(p.keep + (size_t)l * p.keep_stride, A.x, p.keep_rows * d * sizeof(float),
                            hipMemcpyDeviceToDevice, s));
    char* kc = p.kv + (p.kv_per_layer ? (size_t)l * 2 * plane : 0);
    char* vc = kc + plane;
    void* const q_l = p.q_keep ? (void*)(p.q_keep + (size_t)l * p.q_keep_stride) : A.q;  // this layer's rotated q rows
    if (pending) {
      PendingResidual pr;
      pr.part_a = (const float*)A.splitk; pr.ks_a = ks_o; pr.bias_a = h->b_o[l - 1];
      pr.part_b = (const float*)A.splitk2; pr.ks_b = ks_2; pr.bias_b = h->b_fc2[l - 1];
      pr.slab = slab;
      LAUNCH("layernorm_decode", launch_layernorm_pending(A.x, p.rows_max, p.rows_dev, d, c.ln_eps, h->ln1_g[l], h->ln1_b[l],
                                                          A.a, h->ln2_g[l], h->ln2_b[l], A.m, pr, s));
      pending = false;
    } else {
      LAUNCH(p.mode ? "layernorm_decode" : "layernorm", launch_layernorm(dt, A.x, p.rows_max, p.rows_dev, d, c.ln_eps, h->ln1_g[l], h->ln1_b[l],
                                           A.a, h->ln2_g[l], h->ln2_b[l], A.m, s));
    }
    GemmArgs g = gemm_args(A.a, h->w_qkv[l], h->b_qkv[l], A.qkv, 3 * d, d, EPI_BIAS);
    if (p.mode == 1) g.max_split = cap_qkv;
    if (fold) {
      g.phase = 1;
      LAUNCH("gemm_decode_qkv", launch_gemm(dt, g, s));
      LAUNCH("rope_kv_decode", launch_rope_kv_splitk((const float*)A.splitk, ks_qkv, (size_t)p.rows_max * 3 * d, h->b_qkv[l],
                                                     p.rows_max, p.rows_dev, p.pos, p.pos_add, p.rowid, p.kvoff, p.len,
                                                     c.n_heads, c.head_dim, c.rotary_dims, h->rope_cos, h->rope_sin, q_l,
                                                     kc, vc, (long)p.kv_extra, s));
    } else if (p.mode == 0 && gemm_takes_qkv(dt, g, c.n_heads, c.head_dim, c.rotary_dims)) {
      // prefill / scoring: the rotary turn and the K/V store are the epilogue of the QKV product
      QkvArgs qa;
      qa.pos = p.pos; qa.rowid = p.rowid; qa.kvoff = p.kvoff; qa.len = p.len;
      qa.cos_t = h->rope_cos; qa.sin_t = h->rope_sin;
      qa.q = q_l; qa.kc = kc; qa.vc = vc; qa.kv_extra = (long)p.kv_extra;
      qa.pos_add = p.pos_add; qa.H = c.n_heads; qa.hd = c.head_dim; qa.r = c.rotary_dims;
      g.epilogue = EPI_QKV;
      g.qkv = &qa;
      LAUNCH("gemm", launch_gemm(dt, g, s));
    } else {
      LAUNCH(p.mode ? "gemm_decode_qkv" : "gemm", launch_gemm(dt, g, s));
      LAUNCH(p.mode ? "rope_kv_decode" : "rope_kv", launch_rope_kv(dt, A.qkv, p.rows_max, p.rows_dev, p.pos, p.pos_add, p.rowid, p.kvoff,
                                       p.len, c.n_heads, c.head_dim, c.rotary_dims, h->rope_cos, h->rope_sin, q_l, kc, vc,
                                       (long)p.kv_extra, s));
    }
    if (p.mode == 0 && p.last && l + 1 == c.n_layers) {
      const Acts& Z = *p.last;
      const size_t rb = (size_t)d * h->esz;
      LAUNCH("gather_last", launch_gather_rows(q_l, p.cu + 1, -1, p.B, rb, Z.q, s));
      LAUNCH("gather_last", launch_gather_rows(A.m, p.cu + 1, -1, p.B, rb, Z.m, s));
      LAUNCH("gather_last", launch_gather_rows(A.x, p.cu + 1, -1, p.B, (size_t)d * sizeof(float), Z.x, s));
      // the last query of a sequence attends over all of its rows: the single-row kernel with ctx = len
      LAUNCH("attn_decode", launch_attn_decode(dt, Z.q, kc, vc, (long)p.kv_extra, p.B, p.len, 0, p.ctx_max, p.kvoff,
                                               c.n_heads, c.head_dim, Z.att, s));
      GemmArgs z;
      z.M_max = p.B;
      z.M_dev = nullptr;
      z.splitk_ws = Z.splitk;
      z.splitk_ws_bytes = Z.splitk_bytes;
      auto few = [&](const void* in, const void* w, const void* bias, void* out, int N, int K, int epi) {
        GemmArgs g = z;
        g.A = in; g.W = w; g.bias = bias; g.out = out; g.N = N; g.K = K; g.ldo = N; g.epilogue = epi;
        return g;
      };
      GemmArgs zo = few(Z.att, h->w_o[l], h->b_o[l], Z.x, d, d, EPI_BIAS_RESADD);
      GemmArgs z1 = few(Z.m, h->w_fc1[l], h->b_fc1[l], Z.ffn, c.d_ff, d, EPI_BIAS_GELU);
      GemmArgs z2 = few(Z.ffn, h->w_fc2[l], h->b_fc2[l], Z.x, d, c.d_ff, EPI_BIAS_RESADD);
      zo.ldw = z2.ldw = h->ld_o2;
      LAUNCH("gemm_decode", launch_gemm(dt, zo, s));
      LAUNCH("gemm_decode", launch_gemm(dt, z1, s));
      LAUNCH("gemm_decode", launch_gemm(dt, z2, s));
      break;
    }
    if (p.mode == 0 && p.sel && l + 1 == c.n_layers) {
      const Acts& Z = *p.selz;
      const size_t esz = h->esz, ld_att = (size_t)(cat ? d + c.d_ff : d);
      LAUNCH("attn_prefill", launch_attn_prefill(dt, q_l, kc, vc, (long)p.kv_extra, p.B, p.Lmax, p.len, p.cu, p.kvoff,
                                                 c.n_heads, c.head_dim, A.att, (int)ld_att, s));
      LAUNCH("gather_sel", launch_gather_rows_strided(A.att, ld_att * esz, p.sel, p.sel_rows, (size_t)d * esz, Z.att,
                                                      ld_att * esz, s));
      LAUNCH("gather_sel", launch_gather_rows_strided(A.m, (size_t)d * esz, p.sel, p.sel_rows, (size_t)d * esz, Z.m,
                                                      (size_t)d * esz, s));
      LAUNCH("gather_sel", launch_gather_rows_strided(A.x, (size_t)d * 4, p.sel, p.sel_rows, (size_t)d * 4, Z.x,
                                                      (size_t)d * 4, s));
      GemmArgs zb;
      zb.M_max = p.sel_rows;
      zb.M_dev = p.n_sel;
      auto zg = [&](const void* in, const void* w, const void* bias, void* out, int N, int K, int epi) {
        GemmArgs g = zb;
        g.A = in; g.W = w; g.bias = bias; g.out = out; g.N = N; g.K = K; g.ldo = N; g.epilogue = epi;
        return g;
      };
      GemmArgs z1 = zg(Z.m, h->w_fc1[l], h->b_fc1[l], Z.ffn, c.d_ff, d, EPI_BIAS_GELU);
      if (cat) {
        z1.out = (char*)Z.att + (size_t)d * esz;
        z1.ldo = d + c.d_ff;
        GemmArgs zc = zg(Z.att, h->w_o[l], h->b_o[l], Z.x, d, d + c.d_ff, EPI_BIAS_RESADD);
        zc.bias2 = h->b_fc2[l];
        LAUNCH("gemm", launch_gemm(dt, z1, s));
        LAUNCH("gemm", launch_gemm(dt, zc, s));
      } else {
        GemmArgs zo = zg(Z.att, h->w_o[l], h->b_o[l], Z.x, d, d, EPI_BIAS_RESADD);
        GemmArgs z2 = zg(Z.ffn, h->w_fc2[l], h->b_fc2[l], Z.x, d, c.d_ff, EPI_BIAS_RESADD);
        zo.ldw = z2.ldw = h->ld_o2;
        LAUNCH("gemm", launch_gemm(dt, zo, s));
        LAUNCH("gemm", launch_gemm(dt, z1, s));
        LAUNCH("gemm", launch_gemm(dt, z2, s));
      }
      break;
    }
    GemmArgs go = gemm_args(A.att, h->w_o[l], h->b_o[l], A.x, d, d, EPI_BIAS_RESADD);
    GemmArgs g1 = gemm_args(A.m, h->w_fc1[l], h->b_fc1[l], A.ffn, c.d_ff, d, EPI_BIAS_GELU);
    GemmArgs g2 = gemm_args(A.ffn, h->w_fc2[l], h->b_fc2[l], A.x, d, c.d_ff, EPI_BIAS_RESADD);
    go.ldw = g2.ldw = h->ld_o2;
    if (p.mode == 1) {
      go.max_split = cap_o;
      g1.max_split = cap_1;
      g2.max_split = cap_2;
      g1.small_footprint = g2.small_footprint = mlp_small;
    }
    if (cat) {  // attention output and FFN hidden side by side: [rows, d + d_ff]
      g1.out = (char*)A.att + (size_t)d * h->esz;
      g1.ldo = d + c.d_ff;
    }
    if (p.mode == 1) {  // the MLP branch has partial-sum scratch of its own
      g1.splitk_ws = A.splitk2;
      g2.splitk_ws = A.splitk2;
    }
    hipEvent_t join = nullptr;
    if (fork_mlp) {
      hipEvent_t fork = h->fork_ev[h->ev_rr & 7];
      join = h->join_ev[h->ev_rr & 7];
      ++h->ev_rr;
      HIP_OK(hipEventRecord(fork, s));
      HIP_OK(hipStreamWaitEvent(h->side, fork, 0));
      GemmArgs m2 = g2;
      m2.phase = 1;
      hipError_t e1 = launch_gemm(dt, g1, h->side);
      if (e1 == hipSuccess) e1 = launch_gemm(dt, m2, h->side);
      if (e1 != hipSuccess) return fail(RLHF_EHIP, std::string("gemm_decode (side stream): ") + hipGetErrorString(e1));
      HIP_OK(hipEventRecord(join, h->side));
    }
    if (p.mode == 0)
      LAUNCH("attn_prefill", launch_attn_prefill(dt, q_l, kc, vc, (long)p.kv_extra, p.B, p.Lmax, p.len, p.cu, p.kvoff,
                                                 c.n_heads, c.head_dim, A.att, cat ? d + c.d_ff : d, s));
    else
      LAUNCH("attn_decode", launch_attn_decode(dt, q_l, kc, vc, (long)p.kv_extra, p.B, p.len, p.ctx_add, p.ctx_max,
                                               p.kvoff, c.n_heads, c.head_dim, A.att, s));
    // From here on the order of the additions into x is the serial one: x = (x + attn) + mlp.
    const bool keep_u = p.mode == 0 && p.u_keep && l < p.u_keep_layers && dt == 1;
    if (keep_u) {  // FC1 into the kept buffer, GELU from there into where FC2 reads its operand
      GemmArgs gu = g1;
      gu.epilogue = EPI_BIAS;
      gu.out = p.u_keep + (size_t)l * p.u_keep_stride;
      gu.ldo = c.d_ff;
      LAUNCH("gemm", launch_gemm(dt, gu, s));
      LAUNCH("gelu", launch_gelu_rows_f16(gu.out, (size_t)c.d_ff, g1.out, (size_t)g1.ldo, (int)p.keep_rows, c.d_ff, s));
    }
    if (cat) {
      // x += [att | ffn] [W_o | W_fc2]^T + b_o + b_fc2: one product, one pass over the residual stream
      if (!keep_u) LAUNCH("gemm", launch_gemm(dt, g1, s));
      LAUNCH("gemm", launch_gemm(dt, gcat(l), s));
      continue;
    }
    const bool defer = fold && l + 1 < c.n_layers;  // the next layer's LayerNorm adds both products
    if (fold) go.phase = 1;
    LAUNCH(p.mode ? "gemm_decode_out" : "gemm", launch_gemm(dt, go, s));
    if (fork_mlp) {
      HIP_OK(hipStreamWaitEvent(s, join, 0));
    } else {
      if (!keep_u) LAUNCH(p.mode ? "gemm_decode_fc1" : "gemm", launch_gemm(dt, g1, s));
      if (fold) g2.phase = 1;
      LAUNCH(p.mode ? "gemm_decode_fc2" : "gemm", launch_gemm(dt, g2, s));
    }
    if (defer) {
      pending = true;
    } else if (fold) {
      go.phase = 2;
      g2.phase = 2;
      LAUNCH("gemm_decode_out", launch_gemm(dt, go, s));
      LAUNCH("gemm_decode_fc2", launch_gemm(dt, g2, s));
    } else if (fork_mlp) {
      g2.phase = 2;
      LAUNCH("gemm_decode_fc2", launch_gemm(dt, g2, s));
    }
  }
  if (p.keep)
    HIP_OK(hipMemcpyAsync(p.keep + (size_t)c.n_layers * p.keep_stride, A.x, p.keep_rows * d * sizeof(float),
                          hipMemcpyDeviceToDevice, s));
  return RLHF_OK;
}

// Bytes of the fp16 weight image of a bf16-mode model: per layer W_qkv (rotary pairs made neighbours) with its
// reordered bias, W_fc1, and W_o | W_fc2 side by side; then the LM head.
size_t weight_image_bytes_of(const rlhf_model_config& c) {
  const size_t d = c.d_model, F = c.d_ff;
  const size_t per_layer_elems = 3 * d * d + 3 * d + d * F + d * d + d * F;
  return (per_layer_elems * (size_t)c.n_layers + (size_t)c.vocab * d) * 2;
}

// (Re)fills the image from the caller's bf16 arrays and points the handle's per-layer matrix pointers into it.
hipError_t convert_weight_image(rlhf_handle* h, hipStream_t s) {
  const rlhf_model_config& c = h->cfg;
  const size_t d = c.d_model, F = c.d_ff;
  char* p = (char*)h->w16;
  hipError_t e = hipSuccess;
  h->ld_o2 = (int)(d + F);
  for (int l = 0; l < c.n_layers && e == hipSuccess; ++l) {
    char* wq = p;
    char* bq = wq + 3 * d * d * 2;
    char* w1 = bq + 3 * d * 2;
    char* wo = w1 + d * F * 2;
    e = launch_qkv_weights_f16(h->src_w_qkv[l], h->src_b_qkv[l], wq, bq, (int)d, c.head_dim, c.rotary_dims, s);
    if (e == hipSuccess) e = launch_bf16_to_f16(h->src_w_fc1[l], w1, d * F, s);
    if (e == hipSuccess) e = launch_bf16_to_f16_2d(h->src_w_o[l], wo, d, d, d + F, s);
    if (e == hipSuccess) e = launch_bf16_to_f16_2d(h->src_w_fc2[l], wo + d * 2, d, F, d + F, s);
    h->w_qkv[l] = wq;
    h->b_qkv[l] = bq;
    h->w_fc1[l] = w1;
    h->w_o[l] = wo;
    h->w_fc2[l] = wo + d * 2;
    p = wo + (d * d + d * F) * 2;
  }
  if (e == hipSuccess) e = launch_bf16_to_f16(h->w.embed_out, p, (size_t)c.vocab * d, s);
  h->embed_out_mm = p;
  return e;
}

int check_common(const rlhf_handle* h, int B, int L) {
  if (!h) return fail(RLHF_EINVAL, "null handle");
  if (B <= 0 || L <= 0) return fail(RLHF_EINVAL, "batch and length must be positive");
  if ((size_t)B * (size_t)L > (size_t)1 << 30) return fail(RLHF_EUNSUPPORTED, "batch * length too large");
  if (L > kMaxPos) return fail(RLHF_EUNSUPPORTED, "sequence longer than the rotary table");
  return RLHF_OK;
}

}  // namespace

extern "C" {

const char* rlhf_last_error(void) { return g_err.c_str(); }

int rlhf_ppo_assemble_rewards(const float* logprobs, const float* ref_logprobs, const float* rm_values,
                              const int32_t* tokens, int32_t B, int32_t Lq, int32_t N, int32_t eos_id,
                              int32_t pad_id, float beta, float missing_eos_score, float* out_rewards,
                              float* out_scores, float* out_kl, int32_t* out_kept, void* stream) {
  if (!logprobs || !ref_logprobs || !rm_values || !tokens || !out_rewards || !out_kept || !out_scores || !out_kl)
    return fail(RLHF_EINVAL, "null pointer argument");
  if (B <= 0 || N <= 0 || Lq < 0) return fail(RLHF_EINVAL, "batch and response length must be positive");
  if ((size_t)B * ((size_t)Lq + N) > (size_t)1 << 30) return fail(RLHF_EUNSUPPORTED, "batch * length too large");
  HIP_OK(launch_ppo_rewards(logprobs, ref_logprobs, rm_values, tokens, B, Lq, N, eos_id, pad_id, beta,
                            missing_eos_score, out_rewards, out_scores, out_kl, out_kept, (hipStream_t)stream));
  return RLHF_OK;
}

int rlhf_ppo_gae(const float* rewards, const float* values, int64_t values_row_stride, const int32_t* kept,
                 int32_t B, int32_t N, float gamma, float lambda, float* out_advantages, float* out_returns,
                 void* stream) {
  if (!rewards || !values || !kept || !out_advantages || !out_returns)
    return fail(RLHF_EINVAL, "null pointer argument");
  if (B <= 0 || N <= 0) return fail(RLHF_EINVAL, "batch and response length must be positive");
  if (values_row_stride < N) return fail(RLHF_EINVAL, "values_row_stride smaller than the response length");
  HIP_OK(launch_ppo_gae(rewards, values, (long)values_row_stride, kept, B, N, gamma, lambda, out_advantages,
                        out_returns, (hipStream_t)stream));
  return RLHF_OK;
}

int rlhf_ppo_whiten(const float* x, const int32_t* kept, int32_t B, int32_t N, int32_t shift_mean, float* out,
                    void* stream) {
  if (!x || !out) return fail(RLHF_EINVAL, "null pointer argument");
  if (B <= 0 || N <= 0) return fail(RLHF_EINVAL, "batch and response length must be positive");
  HIP_OK(launch_ppo_whiten(x, kept, B, N, shift_mean ? 1 : 0, out, (hipStream_t)stream));
  return RLHF_OK;
}

int rlhf_ppo_loss(const float* new_logprobs, const float* old_logprobs, const float* advantages,
                  const float* new_values, const float* old_values, const float* returns, const int32_t* kept,
                  int32_t B, int32_t N, float cliprange, float cliprange_value, float vf_coef, float* d_logprobs,
                  float* d_values, float* stats, void* stream) {
  if (!new_logprobs || !old_logprobs || !advantages || !new_values || !old_values || !returns || !kept ||
      !d_logprobs || !d_values || !stats)
    return fail(RLHF_EINVAL, "null pointer argument");
  if (B <= 0 || N <= 0) return fail(RLHF_EINVAL, "batch and response length must be positive");
  if (!(cliprange >= 0.f) || !(cliprange_value >= 0.f) || !std::isfinite(cliprange) || !std::isfinite(cliprange_value) ||
      !std::isfinite(vf_coef))
    return fail(RLHF_EINVAL, "clip ranges must be finite and >= 0, the value coefficient finite");
  HIP_OK(launch_ppo_loss(new_logprobs, old_logprobs, advantages, new_values, old_values, returns, kept, B, N, cliprange,
                         cliprange_value, vf_coef, d_logprobs, d_values, stats, (hipStream_t)stream));
  return RLHF_OK;
}

int rlhf_attention_backward(const void* q, const void* k, const void* v, const void* d_out, const int32_t* cu_seqlens,
                            int32_t B, int32_t T, int32_t n_heads, int32_t head_dim, int32_t dtype, int32_t max_len,
                            float* lse_scratch, float* delta_scratch, void* dq, void* dk, void* dv, void* stream) {
  if (!q || !k || !v || !d_out || !cu_seqlens || !lse_scratch || !delta_scratch || !dq || !dk || !dv)
    return fail(RLHF_EINVAL, "null pointer argument");
  if (B <= 0 || T <= 0 || n_heads <= 0 || head_dim <= 0 || max_len <= 0)
    return fail(RLHF_EINVAL, "batch, rows, heads, head_dim and max_len must be positive");
  if (dtype != RLHF_DTYPE_FP32 && dtype != RLHF_DTYPE_BF16) return fail(RLHF_EUNSUPPORTED, "unknown dtype");
  if (head_dim > 256 || (head_dim % (dtype == RLHF_DTYPE_FP32 ? 4 : 8)) != 0)
    return fail(RLHF_EUNSUPPORTED, "head_dim must be <= 256 and a multiple of 4 (fp32) or 8 (fp16)");
  if ((size_t)4 * (2 * (size_t)head_dim + 2 * (size_t)max_len) * sizeof(float) > 150 * 1024)
    return fail(RLHF_EUNSUPPORTED, "max_len too large for the kernels' scratch");
  if ((((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)d_out | (uintptr_t)dq | (uintptr_t)dk | (uintptr_t)dv) & 15) != 0)
    return fail(RLHF_EINVAL, "matrices must be 16-byte aligned");
  HIP_OK(launch_attention_backward(dtype, q, k, v, d_out, cu_seqlens, B, T, n_heads, head_dim, max_len, lse_scratch,
                                   delta_scratch, dq, dk, dv, (hipStream_t)stream));
  return RLHF_OK;
}

int rlhf_attention_backward_noalloc(const void* q, const void* k, const void* v, const void* d_out,
                                    const int32_t* cu_seqlens, int32_t B, int32_t T, int32_t n_heads, int32_t head_dim,
                                    int32_t dtype, int32_t max_len, void* dq, void* dk, void* dv, void* stream) {
  if (T > 0 && n_heads > 0 && (size_t)T * (size_t)n_heads > kStaticScratchFloats)
    return fail(RLHF_EUNSUPPORTED, "rows * heads beyond the static scratch (1,048,576): use rlhf_attention_backward "
                                   "with caller scratch");
  int dev = -1;
  HIP_OK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(RLHF_EUNSUPPORTED, "device index beyond the per-device table");
  float* base = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_static_scratch_mu);
    if (!g_static_scratch_ptr[dev]) {
      // the array's name is a host-side stand-in: its device address on the current device comes from the runtime
      void* p = nullptr;
      HIP_OK(hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)));
      if (!p) return fail(RLHF_EHIP, "hipGetSymbolAddress returned a null address");
      g_static_scratch_ptr[dev] = (float*)p;
    }
    base = g_static_scratch_ptr[dev];
  }
  // Both halves are written by the first kernel for every (row, head) before the second reads them: nothing
  // has to start at zero, and what an earlier call left behind is never read.
  return rlhf_attention_backward(q, k, v, d_out, cu_seqlens, B, T, n_heads, head_dim, dtype, max_len, base,
                                 base + kStaticScratchFloats, dq, dk, dv, stream);
}

int rlhf_adamw_step(float* param, const float* grad, float* exp_avg, float* exp_avg_sq, uint16_t* param_bf16,
                    uint64_t n, int32_t step, double lr, double beta1, double beta2, double eps, double weight_decay,
                    double grad_scale, void* stream) {
  if (step < 1) return fail(RLHF_EINVAL, "step counts from 1");
  if (!(beta1 >= 0.0 && beta1 < 1.0) || !(beta2 >= 0.0 && beta2 < 1.0))
    return fail(RLHF_EINVAL, "beta1 and beta2 must be in [0, 1)");
  if (!(lr >= 0.0) || !(eps > 0.0) || !(weight_decay >= 0.0) || !std::isfinite(lr) || !std::isfinite(eps) ||
      !std::isfinite(weight_decay) || !std::isfinite(grad_scale))
    return fail(RLHF_EINVAL, "lr, weight_decay must be finite and >= 0, eps finite and > 0, grad_scale finite");
  if (n == 0) return RLHF_OK;  // nothing to update; the pointers may then be null
  if (!param || !grad || !exp_avg || !exp_avg_sq) return fail(RLHF_EINVAL, "null pointer argument");
  if ((((uintptr_t)param | (uintptr_t)grad | (uintptr_t)exp_avg | (uintptr_t)exp_avg_sq) & 15) != 0 ||
      ((uintptr_t)param_bf16 & 7) != 0)
    return fail(RLHF_EINVAL, "fp32 arrays must be 16-byte aligned, the bf16 array 8-byte aligned");
  const double bias1 = 1.0 - std::pow(beta1, (double)step);
  const double bias2 = 1.0 - std::pow(beta2, (double)step);
  HIP_OK(launch_adamw(param, grad, exp_avg, exp_avg_sq, param_bf16, (size_t)n, (float)(1.0 - lr * weight_decay),
                      (float)beta1, (float)(1.0 - beta1), (float)beta2, (float)(1.0 - beta2), (float)(lr / bias1),
                      (float)(1.0 / std::sqrt(bias2)), (float)eps, (float)grad_scale, (hipStream_t)stream));
  return RLHF_OK;
}

int rlhf_weight_image_bytes(const rlhf_model_config* cfg, size_t* out) {
  if (!cfg || !out) return fail(RLHF_EINVAL, "null argument");
  if (cfg->n_layers < 0 || cfg->d_model <= 0 || cfg->d_ff <= 0 || cfg->vocab <= 0)
    return fail(RLHF_EINVAL, "non-positive model dimension");
  *out = cfg->dtype == RLHF_DTYPE_BF16 ? weight_image_bytes_of(*cfg) : 0;
  return RLHF_OK;
}

int rlhf_refresh_weights(rlhf_handle* h, void* stream) {
  if (!h) return fail(RLHF_EINVAL, "null handle");
  if (h->cfg.dtype != RLHF_DTYPE_BF16) return RLHF_OK;  // fp32 mode reads the caller's arrays directly
  HIP_OK(convert_weight_image(h, (hipStream_t)stream));
  return RLHF_OK;
}

int rlhf_create(const rlhf_model_config* cfg, const rlhf_weights* w, void* weight_image, size_t weight_image_bytes,
                rlhf_handle** out) {
  if (out) *out = nullptr;
  if (!cfg || !w || !out) return fail(RLHF_EINVAL, "null argument");
  const rlhf_model_config& c = *cfg;
  if (c.n_layers < 0 || c.d_model <= 0 || c.n_heads <= 0 || c.head_dim <= 0 || c.d_ff <= 0 || c.vocab <= 0)
    return fail(RLHF_EINVAL, "non-positive model dimension");
  if (c.d_model != c.n_heads * c.head_dim) return fail(RLHF_EINVAL, "d_model != n_heads * head_dim");
  if (c.rotary_dims < 0 || (c.rotary_dims & 1) || c.rotary_dims > c.head_dim)
    return fail(RLHF_EINVAL, "rotary_dims must be even and <= head_dim");
  if (c.dtype != RLHF_DTYPE_FP32 && c.dtype != RLHF_DTYPE_BF16) return fail(RLHF_EUNSUPPORTED, "unknown dtype");
  if (c.head_dim > 256) return fail(RLHF_EUNSUPPORTED, "head_dim > 256");
  if (c.dtype == RLHF_DTYPE_BF16 && ((c.d_model % 8) || (c.d_ff % 8)))
    return fail(RLHF_EUNSUPPORTED, "bf16 needs d_model and d_ff to be multiples of 8");
  if (c.eos_id < 0 || c.eos_id >= c.vocab || c.pad_id < 0) return fail(RLHF_EINVAL, "bad eos/pad id");
  if (!(c.ln_eps > 0.f) || !(c.rope_base > 0.f)) return fail(RLHF_EINVAL, "ln_eps and rope_base must be > 0");
  if (!w->embed_in || !w->embed_out || !w->lnf_g || !w->lnf_b) return fail(RLHF_EINVAL, "null weight pointer");
  const void* const* per_layer[12] = {w->ln1_g, w->ln1_b, w->ln2_g, w->ln2_b, w->w_qkv, w->b_qkv,
                                      w->w_o,   w->b_o,   w->w_fc1, w->b_fc1, w->w_fc2, w->b_fc2};
  for (auto p : per_layer) {
    if (c.n_layers > 0 && !p) return fail(RLHF_EINVAL, "null per-layer pointer array");
    for (int l = 0; l < c.n_layers; ++l)
      if (!p[l]) return fail(RLHF_EINVAL, "null per-layer weight pointer");
  }
  rlhf_handle* h = new (std::nothrow) rlhf_handle();
  if (!h) return fail(RLHF_ENOMEM, "host allocation failed");
  h->cfg = c;
  h->w = *w;
  h->esz = c.dtype == RLHF_DTYPE_FP32 ? 4 : 2;
  std::vector<const void*>* dst[12] = {&h->ln1_g, &h->ln1_b, &h->ln2_g, &h->ln2_b, &h->w_qkv, &h->b_qkv,
                                       &h->w_o,   &h->b_o,   &h->w_fc1, &h->b_fc1, &h->w_fc2, &h->b_fc2};
  for (int i = 0; i < 12; ++i) dst[i]->assign(per_layer[i], per_layer[i] + c.n_layers);
  h->src_w_qkv = h->w_qkv; h->src_b_qkv = h->b_qkv; h->src_w_o = h->w_o; h->src_w_fc1 = h->w_fc1; h->src_w_fc2 = h->w_fc2;
  // rotary tables, evaluated in double on the host: angle(p, i) = p * base^(-2i/r)
  const int half = c.rotary_dims / 2;
  if (half > 0) {
    std::vector<float> cs((size_t)kMaxPos * half), sn((size_t)kMaxPos * half);
    for (int p = 0; p < kMaxPos; ++p)
      for (int i = 0; i < half; ++i) {
        const double ang = (double)p * std::pow((double)c.rope_base, -2.0 * i / c.rotary_dims);
        cs[(size_t)p * half + i] = (float)std::cos(ang);
        sn[(size_t)p * half + i] = (float)std::sin(ang);
      }
    hipError_t e = hipMalloc((void**)&h->rope_cos, cs.size() * 4);
    if (e == hipSuccess) e = hipMalloc((void**)&h->rope_sin, sn.size() * 4);
    if (e == hipSuccess) e = hipMemcpy(h->rope_cos, cs.data(), cs.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(h->rope_sin, sn.data(), sn.size() * 4, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
      rlhf_destroy(h);
      return fail(RLHF_EHIP, std::string("rotary tables: ") + hipGetErrorString(e));
    }
  }
  // bf16 mode: the matrix cores take fp16 operands; the five matrix families are converted into the caller's
  // image buffer (and again by rlhf_refresh_weights whenever the caller has changed its weights)
  h->embed_out_mm = w->embed_out;
  if (c.dtype == RLHF_DTYPE_BF16) {
    const size_t need = weight_image_bytes_of(c);
    if (!weight_image || ((uintptr_t)weight_image & 255) != 0 || weight_image_bytes < need) {
      rlhf_destroy(h);
      return fail(weight_image ? RLHF_ENOMEM : RLHF_EINVAL,
                  "bf16 mode needs a 256-byte aligned device buffer of rlhf_weight_image_bytes() bytes");
    }
    h->w16 = weight_image;
    hipError_t e = convert_weight_image(h, nullptr);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
      rlhf_destroy(h);
      return fail(RLHF_EHIP, std::string("fp16 weight conversion: ") + hipGetErrorString(e));
    }
  }
  {
    hipError_t e = hipStreamCreateWithFlags(&h->side, hipStreamNonBlocking);
    for (int i = 0; i < 8 && e == hipSuccess; ++i) {
      e = hipEventCreateWithFlags(&h->fork_ev[i], hipEventDisableTiming);
      if (e == hipSuccess) e = hipEventCreateWithFlags(&h->join_ev[i], hipEventDisableTiming);
    }
    if (e != hipSuccess) {
      rlhf_destroy(h);
      return fail(RLHF_EHIP, std::string("side stream: ") + hipGetErrorString(e));
    }
  }
  *out = h;
  return RLHF_OK;
}

void rlhf_destroy(rlhf_handle* h) {
  if (!h) return;
  if (h->rope_cos) (void)hipFree(h->rope_cos);
  if (h->rope_sin) (void)hipFree(h->rope_sin);
  for (hipEvent_t e : h->ev_pool) (void)hipEventDestroy(e);
  for (hipEvent_t e : h->ph)
    if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : h->fork_ev)
    if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : h->join_ev)
    if (e) (void)hipEventDestroy(e);
  if (h->side) (void)hipStreamDestroy(h->side);
  delete h;
}

int rlhf_workspace_bytes(const rlhf_handle* h, int32_t B, int32_t Lq, int32_t max_new, int32_t L_score,
                         size_t* out) {
  if (!h || !out) return fail(RLHF_EINVAL, "null argument");
  if (B <= 0) return fail(RLHF_EINVAL, "batch must be positive");
  size_t need = 0;
  if (Lq > 0 && max_new > 0) {
    Carver c(nullptr);
    carve_rollout(c, h->cfg, B, Lq, max_new, h->esz);
    need = std::max(need, c.off);
  }
  if (L_score > 0) {
    Carver c(nullptr);
    carve_score(c, h->cfg, B, L_score, h->esz);
    need = std::max(need, c.off);
  }
  *out = need + 256;
  return RLHF_OK;
}

namespace {
constexpr int kHeadChunk = 16384;  // rows whose logits and logit gradients exist at a time (3.3 GB of fp32 logits
                                   // at a 50k vocabulary): one chunk covers a rollout batch's response positions
struct HeadBwdWs {
  void *hl, *dz, *dzT, *hlT, *WT;
  float *logits, *dhl, *stats, *part;
  int chunk, chunk_pad, V_pad, splits;
};
HeadBwdWs carve_head_bwd(Carver& c, const rlhf_model_config& cfg, int T, size_t esz) {
  HeadBwdWs w;
  const size_t d = cfg.d_model, V = cfg.vocab;
  w.chunk = std::min(T, kHeadChunk);
  w.chunk_pad = (w.chunk + 127) & ~127;  // the row count of a chunk is the K of the weight-gradient product
  w.V_pad = (int)((V + 7) & ~(size_t)7);  // the vocabulary is the K of the input-gradient product
  w.splits = std::max(1, std::min(256, (T + 255) / 256));
  w.hl = c.take_bytes((size_t)w.chunk_pad * d * esz);
  w.logits = c.take<float>((size_t)w.chunk * V);
  w.dz = c.take_bytes((size_t)w.chunk_pad * w.V_pad * esz);
  w.dzT = c.take_bytes(V * (size_t)w.chunk_pad * esz);
  w.hlT = c.take_bytes(d * (size_t)w.chunk_pad * esz);
  w.WT = c.take_bytes(d * (size_t)w.V_pad * esz);
  w.dhl = c.take<float>((size_t)T * d);
  w.stats = c.take<float>((size_t)2 * T);
  w.part = c.take<float>((size_t)w.splits * 3 * d);
  return w;
}
}  // namespace

int rlhf_head_backward_workspace_bytes(const rlhf_handle* h, int32_t T, size_t* out) {
  if (!h || !out) return fail(RLHF_EINVAL, "null argument");
  if (T <= 0) return fail(RLHF_EINVAL, "row count must be positive");
  Carver c(nullptr);
  carve_head_bwd(c, h->cfg, T, h->esz);
  *out = c.off + 256;
  return RLHF_OK;
}

int rlhf_head_backward(rlhf_handle* h, const float* x_final, const int32_t* targets, const float* d_logprobs,
                       const float* d_values, int32_t T, float temperature, float grad_scale, float* d_x,
                       float* d_lnf_g, float* d_lnf_b, float* d_embed_out, float* d_value_w, float* d_value_b,
                       void* workspace, size_t workspace_bytes, void* stream) {
  if (!h) return fail(RLHF_EINVAL, "null handle");
  if (T <= 0) return fail(RLHF_EINVAL, "row count must be positive");
  if ((size_t)T > (size_t)1 << 30) return fail(RLHF_EUNSUPPORTED, "too many rows");
  if (!(temperature > 0.f) || !std::isfinite(temperature)) return fail(RLHF_EINVAL, "temperature must be > 0");
  if (!std::isfinite(grad_scale)) return fail(RLHF_EINVAL, "grad_scale must be finite");
  if (!x_final || !targets || !d_logprobs || !d_x || !d_lnf_g || !d_lnf_b || !d_embed_out || !workspace)
    return fail(RLHF_EINVAL, "null pointer argument");
  const rlhf_model_config& c = h->cfg;
  const bool has_value = h->w.value_w != nullptr;
  if (has_value && (!d_values || !d_value_w || !d_value_b))
    return fail(RLHF_EINVAL, "the model has a value head: d_values, d_value_w and d_value_b are required");
  Carver cv((void*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255));
  HeadBwdWs ws = carve_head_bwd(cv, c, T, h->esz);
  if (cv.off + ((char*)cv.base - (char*)workspace) > workspace_bytes)
    return fail(RLHF_ENOMEM, "workspace too small for rlhf_head_backward");
  hipStream_t s = (hipStream_t)stream;
  const int dt = c.dtype, d = c.d_model, V = c.vocab;
  const size_t esz = h->esz;

  // W^T [d, V_pad] (zero columns past V), and d_embed_out = 0: the chunks add into it
  LAUNCH("head_bwd_prep", launch_transpose_pad(dt, h->embed_out_mm, (size_t)d, ws.WT, (size_t)ws.V_pad, V, d, ws.V_pad, s));
  LAUNCH("head_bwd_prep", launch_fill_zero(d_embed_out, (size_t)V * d * sizeof(float), s));
  for (int r0 = 0; r0 < T; r0 += ws.chunk) {
    const int rows = std::min(ws.chunk, T - r0);
    const int rows_pad = (rows + 127) & ~127;
    // h = LN_f(x) for the chunk, rows past the chunk zero (they are columns of the K dimension below)
    if (rows_pad > rows)
      LAUNCH("head_bwd_prep", launch_fill_zero((char*)ws.hl + (size_t)rows * d * esz, (size_t)(rows_pad - rows) * d * esz, s));
    LAUNCH("final_ln", launch_final_ln(dt, x_final + (size_t)r0 * d, nullptr, 0, rows, nullptr, d, c.ln_eps, h->w.lnf_g,
                                       h->w.lnf_b, ws.hl, nullptr, 0.f, nullptr, s));
    GemmArgs lm;  // z = h W^T
    lm.A = ws.hl; lm.W = h->embed_out_mm; lm.bias = nullptr; lm.out = ws.logits;
    lm.M_max = rows; lm.M_dev = nullptr; lm.N = V; lm.K = d; lm.ldo = V; lm.epilogue = EPI_F32;
    LAUNCH("gemm_lm_head", launch_gemm(dt, lm, s));
    LAUNCH("softmax_grad", launch_softmax_grad(dt, ws.logits, V, ws.V_pad, targets + r0, d_logprobs + r0, rows, rows_pad,
                                               1.0f / temperature, grad_scale, ws.dz, s));
    GemmArgs gi;  // dL/dh = dz W: the product of dz [rows, V] with the rows of W^T
    gi.A = ws.dz; gi.W = ws.WT; gi.bias = nullptr; gi.out = ws.dhl + (size_t)r0 * d;
    gi.M_max = rows; gi.M_dev = nullptr; gi.N = d; gi.K = ws.V_pad; gi.ldo = d; gi.epilogue = EPI_F32;
    LAUNCH("gemm_head_dx", launch_gemm(dt, gi, s));
    // dL/dW += dz^T h: rows of dz^T [V, rows_pad] against rows of h^T [d, rows_pad]
    LAUNCH("head_bwd_transpose", launch_transpose_pad(dt, ws.dz, (size_t)ws.V_pad, ws.dzT, (size_t)rows_pad, rows_pad, V, rows_pad, s));
    LAUNCH("head_bwd_transpose", launch_transpose_pad(dt, ws.hl, (size_t)d, ws.hlT, (size_t)rows_pad, rows_pad, d, rows_pad, s));
    GemmArgs gw;
    gw.A = ws.dzT; gw.W = ws.hlT; gw.bias = nullptr; gw.out = d_embed_out;
    gw.M_max = V; gw.M_dev = nullptr; gw.N = d; gw.K = rows_pad; gw.ldo = d; gw.epilogue = EPI_BIAS_RESADD;
    LAUNCH("gemm_head_dw", launch_gemm(dt, gw, s));
  }
  LAUNCH("head_ln_backward", launch_head_ln_backward(dt, x_final, ws.dhl, d_values, grad_scale, h->w.value_w, h->w.lnf_g,
                                                     h->w.lnf_b, T, d, c.ln_eps, d_x, ws.stats, ws.part, ws.splits,
                                                     d_lnf_g, d_lnf_b, has_value ? d_value_w : nullptr,
                                                     has_value ? d_value_b : nullptr, s));
  return RLHF_OK;
}

namespace {
struct MlpBwdWs {
  void *m, *u, *f, *go, *df, *goT, *fT, *mT, *w1T, *w2T;
  float *dm, *stats, *part;
  void* slabs;         // fp32 partial results of the K-sliced weight-gradient products
  size_t slabs_bytes;
  float* lnpart;       // per-wave column sums of the one-pass LayerNorm backward
  int T_pad, splits;
};
MlpBwdWs carve_mlp_bwd(Carver& c, const rlhf_model_config& cfg, int T, size_t esz) {
  MlpBwdWs w;
  const size_t d = cfg.d_model, F = cfg.d_ff;
  w.T_pad = (T + 127) & ~127;  // the row count is the K of the weight-gradient products
  w.splits = std::max(1, std::min(256, (T + 255) / 256));
  const size_t Tp = (size_t)w.T_pad;
  w.m = c.take_bytes(Tp * d * esz);  // (Tp rows: operands of the weight-gradient products, whose K is padded)
  w.u = c.take_bytes((size_t)T * F * esz);
  w.f = c.take_bytes(Tp * F * esz);
  w.go = c.take_bytes(Tp * d * esz);
  w.df = c.take_bytes(Tp * F * esz);
  w.goT = c.take_bytes(d * Tp * esz);
  w.fT = c.take_bytes(F * Tp * esz);
  w.mT = c.take_bytes(d * Tp * esz);
  w.w1T = c.take_bytes(d * F * esz);
  w.w2T = c.take_bytes(F * d * esz);
  w.dm = c.take<float>((size_t)T * d);
  w.stats = c.take<float>((size_t)2 * T);
  w.part = c.take<float>((size_t)w.splits * std::max(3 * d, F));
  w.slabs_bytes = 8 * d * F * sizeof(float);
  w.slabs = c.take_bytes(w.slabs_bytes);
  w.lnpart = c.take<float>(ln_backward_rows_scratch_floats(T, (int)d));
  return w;
}
}  // namespace

int rlhf_mlp_backward_workspace_bytes(const rlhf_handle* h, int32_t T, size_t* out) {
  if (!h || !out) return fail(RLHF_EINVAL, "null argument");
  if (T <= 0) return fail(RLHF_EINVAL, "row count must be positive");
  Carver c(nullptr);
  carve_mlp_bwd(c, h->cfg, T, h->esz);
  *out = c.off + 256;
  return RLHF_OK;
}

// Shared work of a layer's two branches inside a whole backward pass (all optional): go16 = the fp16 copy of d_out,
// [T padded to 128 rows, d] with zero padding rows, made once for both branches together with the column sums that
// are d_b_fc2 and d_b_o (then neither is computed here); base = what d_x is added to (d_x = base + the branch's term);
// kept_u = the MLP branch's pre-activations kept by the forward pass (then FC1 is not recomputed).
struct BranchShare {
  const void* go16 = nullptr;
  const float* base = nullptr;
  const void* kept_u = nullptr;  // MLP branch: FC1's output before the GELU as the forward pass left it, [T, d_ff]
};
static int mlp_backward_impl(rlhf_handle* h, int32_t layer, const float* x_in, const float* d_out, int32_t T, float* d_x,
                             float* d_ln2_g, float* d_ln2_b, float* d_w_fc1, float* d_b_fc1, float* d_w_fc2,
                             float* d_b_fc2, void* workspace, size_t workspace_bytes, void* stream, BranchShare sh);

int rlhf_mlp_backward(rlhf_handle* h, int32_t layer, const float* x_in, const float* d_out, int32_t T, float* d_x,
                      float* d_ln2_g, float* d_ln2_b, float* d_w_fc1, float* d_b_fc1, float* d_w_fc2, float* d_b_fc2,
                      void* workspace, size_t workspace_bytes, void* stream) {
  return mlp_backward_impl(h, layer, x_in, d_out, T, d_x, d_ln2_g, d_ln2_b, d_w_fc1, d_b_fc1, d_w_fc2, d_b_fc2, workspace,
                           workspace_bytes, stream, BranchShare{});
}

static int mlp_backward_impl(rlhf_handle* h, int32_t layer, const float* x_in, const float* d_out, int32_t T, float* d_x,
                             float* d_ln2_g, float* d_ln2_b, float* d_w_fc1, float* d_b_fc1, float* d_w_fc2,
                             float* d_b_fc2, void* workspace, size_t workspace_bytes, void* stream, BranchShare sh) {
  if (!h) return fail(RLHF_EINVAL, "null handle");
  const rlhf_model_config& c = h->cfg;
  if (layer < 0 || layer >= c.n_layers) return fail(RLHF_EINVAL, "layer index out of range");
  if (T <= 0) return fail(RLHF_EINVAL, "row count must be positive");
  if ((size_t)T * (size_t)std::max(c.d_model, c.d_ff) >= ((size_t)1 << 32) - ((size_t)128 * std::max(c.d_model, c.d_ff)))
    return fail(RLHF_EUNSUPPORTED, "too many rows");
  if (!x_in || !d_out || !d_x || !d_ln2_g || !d_ln2_b || !d_w_fc1 || !d_b_fc1 || !d_w_fc2 || !d_b_fc2 || !workspace)
    return fail(RLHF_EINVAL, "null pointer argument");
  Carver cv((void*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255));
  MlpBwdWs ws = carve_mlp_bwd(cv, c, T, h->esz);
  if (cv.off + ((char*)cv.base - (char*)workspace) > workspace_bytes)
    return fail(RLHF_ENOMEM, "workspace too small for rlhf_mlp_backward");
  hipStream_t s = (hipStream_t)stream;
  const int dt = c.dtype, d = c.d_model, F = c.d_ff, l = layer, Tp = ws.T_pad;
  const size_t ld_w2 = h->ld_o2 ? (size_t)h->ld_o2 : (size_t)F;  // row stride of this layer's W_fc2

  auto gemm = [&](const void* A, const void* W, const void* bias, void* out, int M, int N, int K, int epi) {
    GemmArgs g;
    g.A = A; g.W = W; g.bias = bias; g.out = out; g.M_max = M; g.M_dev = nullptr;
    g.N = N; g.K = K; g.ldo = N; g.epilogue = epi;
    return g;
  };
  // ---- the branch's forward, recomputed from the layer input: m = LN2(x), u = m W1^T + b1, f = gelu(u)
  LAUNCH("final_ln", launch_final_ln(dt, x_in, nullptr, 0, T, nullptr, d, c.ln_eps, h->ln2_g[l], h->ln2_b[l], ws.m,
                                     nullptr, 0.f, nullptr, s));
  const void* u = sh.kept_u ? sh.kept_u : ws.u;
  if (!sh.kept_u)
    LAUNCH("gemm_mlp_fwd", launch_gemm(dt, gemm(ws.m, h->w_fc1[l], h->b_fc1[l], ws.u, T, F, d, EPI_BIAS), s));
  LAUNCH("gelu", launch_gelu(dt, u, ws.f, (size_t)T * F, s));
  // ---- FC2: db2 = sum_t G, dW2 = G^T f, df = G W2
  const void* go = sh.go16 ? sh.go16 : ws.go;
  if (!sh.go16) {
    LAUNCH("colsum", launch_colsum(0, d_out, T, d, ws.part, ws.splits, d_b_fc2, s));
    LAUNCH("convert", launch_convert_from_f32(dt, d_out, ws.go, (size_t)T * d, s));
  }
  auto dw_gemm = [&](const void* A, const void* W, void* out, int M, int N) {  // K = the rows: sliced
    GemmArgs g = gemm(A, W, nullptr, out, M, N, Tp, EPI_F32);
    g.long_k = true;
    g.splitk_ws = ws.slabs;
    g.splitk_ws_bytes = ws.slabs_bytes;
    return g;
  };
  // Weight gradients straight from the row-major activations (K-major operands) where the kernel takes the shape;
  // the rows T .. Tp-1 of those operands are zeroed first.  Otherwise from transposed, zero-padded copies.
  auto dw_kmajor = [&](const void* A, const void* W, void* out, int M, int N) {
    GemmArgs g = dw_gemm(A, W, out, M, N);
    g.k_major = true;
    return g;
  };
  const bool kmaj = gemm_takes_k_major(dt, dw_kmajor(go, ws.f, d_w_fc2, d, F)) &&
                    gemm_takes_k_major(dt, dw_kmajor(ws.df, ws.m, d_w_fc1, F, d));
  auto zero_tail = [&](void* buf, int width) {
    return Tp > T ? launch_fill_zero((char*)buf + (size_t)T * width * h->esz, (size_t)(Tp - T) * width * h->esz, s)
                  : hipSuccess;
  };
  if (kmaj) {
    if (!sh.go16) LAUNCH("mlp_bwd_zero", zero_tail(ws.go, d));
    LAUNCH("mlp_bwd_zero", zero_tail(ws.f, F));
    LAUNCH("gemm_mlp_dw", launch_gemm(dt, dw_kmajor(go, ws.f, d_w_fc2, d, F), s));
  } else {
    LAUNCH("mlp_bwd_transpose", launch_transpose_pad(dt, go, (size_t)d, ws.goT, (size_t)Tp, T, d, Tp, s));
    LAUNCH("mlp_bwd_transpose", launch_transpose_pad(dt, ws.f, (size_t)F, ws.fT, (size_t)Tp, T, F, Tp, s));
    LAUNCH("gemm_mlp_dw", launch_gemm(dt, dw_gemm(ws.goT, ws.fT, d_w_fc2, d, F), s));
  }
  LAUNCH("mlp_bwd_transpose", launch_transpose_pad(dt, h->w_fc2[l], ld_w2, ws.w2T, (size_t)d, d, F, d, s));
  LAUNCH("gemm_mlp_dx", launch_gemm(dt, gemm(go, ws.w2T, nullptr, ws.df, T, F, d, EPI_BIAS), s));
  // ---- GELU, then FC1: du = df * gelu'(u) (in place), db1 = sum_t du, dW1 = du^T m, dm = du W1
  if (gelu_backward_colsum_supported(dt, u, ws.df, F)) {
    LAUNCH("gelu", launch_gelu_backward_colsum(u, ws.df, T, F, ws.part, ws.splits, d_b_fc1, s));
  } else {
    LAUNCH("gelu", launch_gelu_backward(dt, u, ws.df, (size_t)T * F, s));
    LAUNCH("colsum", launch_colsum(dt, ws.df, T, F, ws.part, ws.splits, d_b_fc1, s));
  }
  if (kmaj) {
    LAUNCH("mlp_bwd_zero", zero_tail(ws.df, F));
    LAUNCH("mlp_bwd_zero", zero_tail(ws.m, d));
    LAUNCH("gemm_mlp_dw", launch_gemm(dt, dw_kmajor(ws.df, ws.m, d_w_fc1, F, d), s));
  } else {
    LAUNCH("mlp_bwd_transpose", launch_transpose_pad(dt, ws.df, (size_t)F, ws.fT, (size_t)Tp, T, F, Tp, s));
    LAUNCH("mlp_bwd_transpose", launch_transpose_pad(dt, ws.m, (size_t)d, ws.mT, (size_t)Tp, T, d, Tp, s));
    LAUNCH("gemm_mlp_dw", launch_gemm(dt, dw_gemm(ws.fT, ws.mT, d_w_fc1, F, d), s));
  }
  LAUNCH("mlp_bwd_transpose", launch_transpose_pad(dt, h->w_fc1[l], (size_t)d, ws.w1T, (size_t)F, F, d, F, s));
  LAUNCH("gemm_mlp_dx", launch_gemm(dt, gemm(ws.df, ws.w1T, nullptr, ws.dm, T, d, F, EPI_F32), s));
  // ---- LN2: the branch's term of dL/dx, and the gradients of its gain and bias
  if (sh.base && !(ln_backward_rows_supported(dt, d) && (((uintptr_t)x_in | (uintptr_t)d_x | (uintptr_t)sh.base) & 15) == 0))
    return fail(RLHF_EUNSUPPORTED, "accumulating LayerNorm backward: shape");
  if (ln_backward_rows_supported(dt, d) && (((uintptr_t)x_in | (uintptr_t)d_x) & 15) == 0)
    LAUNCH("ln_backward", launch_ln_backward_rows(x_in, ws.dm, h->ln2_g[l], T, d, c.ln_eps, d_x, ws.lnpart, d_ln2_g,
                                                  d_ln2_b, s, sh.base));
  else
    LAUNCH("head_ln_backward", launch_head_ln_backward(dt, x_in, ws.dm, nullptr, 1.0f, nullptr, h->ln2_g[l], h->ln2_b[l],
                                                       T, d, c.ln_eps, d_x, ws.stats, ws.part, ws.splits, d_ln2_g,
                                                       d_ln2_b, nullptr, nullptr, s));
  return RLHF_OK;
}

namespace {
struct AttnBwdWs {
  void *a, *qkv, *go, *dO, *att, *dqkv, *goT, *attT, *dqkvT, *aT, *woT, *wqkvT;
  float *da, *dwq, *dbq, *stats, *part, *lse, *delta;
  void* slabs;         // fp32 partial results of the K-sliced weight-gradient products
  size_t slabs_bytes;
  float* lnpart;       // per-wave column sums of the one-pass LayerNorm backward
  int T_pad, splits;
};
AttnBwdWs carve_attn_bwd(Carver& c, const rlhf_model_config& cfg, int T, size_t esz) {
  AttnBwdWs w;
  const size_t d = cfg.d_model;
  w.T_pad = (T + 127) & ~127;
  w.splits = std::max(1, std::min(256, (T + 255) / 256));
  const size_t Tp = (size_t)w.T_pad;
  w.a = c.take_bytes(Tp * d * esz);  // (Tp rows: operands of the weight-gradient products, whose K is padded)
  w.qkv = c.take_bytes((size_t)T * 3 * d * esz);
  w.go = c.take_bytes(Tp * d * esz);
  w.dO = c.take_bytes((size_t)T * d * esz);
  w.att = c.take_bytes(Tp * d * esz);
  w.dqkv = c.take_bytes(Tp * 3 * d * esz);
  w.goT = c.take_bytes(d * Tp * esz);
  w.attT = c.take_bytes(d * Tp * esz);
  w.dqkvT = c.take_bytes(3 * d * Tp * esz);
  w.aT = c.take_bytes(d * Tp * esz);
  w.woT = c.take_bytes(d * d * esz);
  w.wqkvT = c.take_bytes(3 * d * d * esz);
  w.da = c.take<float>((size_t)T * d);
  w.dwq = c.take<float>(3 * d * d);
  w.dbq = c.take<float>(3 * d);
  w.stats = c.take<float>((size_t)2 * T);
  w.part = c.take<float>((size_t)w.splits * 3 * d);
  w.lse = c.take<float>((size_t)T * cfg.n_heads);
  w.delta = c.take<float>((size_t)T * cfg.n_heads);
  w.slabs_bytes = 8 * 3 * d * d * sizeof(float);
  w.slabs = c.take_bytes(w.slabs_bytes);
  w.lnpart = c.take<float>(ln_backward_rows_scratch_floats(T, (int)d));
  return w;
}
}  // namespace

int rlhf_attention_branch_backward_workspace_bytes(const rlhf_handle* h, int32_t T, size_t* out) {
  if (!h || !out) return fail(RLHF_EINVAL, "null argument");
  if (T <= 0) return fail(RLHF_EINVAL, "row count must be positive");
  Carver c(nullptr);
  carve_attn_bwd(c, h->cfg, T, h->esz);
  *out = c.off + 256;
  return RLHF_OK;
}

// kept_q / kept_k / kept_v (optional, all or none): what the forward pass left of this layer's QKV product -- the
// rotated q rows [T, d] and the layer's K / V cache -- so that the product and the rotary turn are not recomputed.
static int attention_branch_backward_impl(rlhf_handle* h, int32_t layer, const float* x_in, const float* d_out,
                                          const int32_t* cu_seqlens, int32_t B, int32_t T, int32_t max_len, float* d_x,
                                          float* d_ln1_g, float* d_ln1_b, float* d_w_qkv, float* d_b_qkv, float* d_w_o,
                                          float* d_b_o, void* workspace, size_t workspace_bytes, void* stream,
                                          const void* kept_q, const void* kept_k, const void* kept_v,
                                          BranchShare sh = BranchShare{});

int rlhf_attention_branch_backward(rlhf_handle* h, int32_t layer, const float* x_in, const float* d_out,
                                   const int32_t* cu_seqlens, int32_t B, int32_t T, int32_t max_len, float* d_x,
                                   float* d_ln1_g, float* d_ln1_b, float* d_w_qkv, float* d_b_qkv, float* d_w_o,
                                   float* d_b_o, void* workspace, size_t workspace_bytes, void* stream) {
  return attention_branch_backward_impl(h, layer, x_in, d_out, cu_seqlens, B, T, max_len, d_x, d_ln1_g, d_ln1_b, d_w_qkv,
                                        d_b_qkv, d_w_o, d_b_o, workspace, workspace_bytes, stream, nullptr, nullptr,
                                        nullptr);
}

static int attention_branch_backward_impl(rlhf_handle* h, int32_t layer, const float* x_in, const float* d_out,
                                          const int32_t* cu_seqlens, int32_t B, int32_t T, int32_t max_len, float* d_x,
                                          float* d_ln1_g, float* d_ln1_b, float* d_w_qkv, float* d_b_qkv, float* d_w_o,
                                          float* d_b_o, void* workspace, size_t workspace_bytes, void* stream,
                                          const void* kept_q, const void* kept_k, const void* kept_v, BranchShare sh) {
  if (!h) return fail(RLHF_EINVAL, "null handle");
  const rlhf_model_config& c = h->cfg;
  if (layer < 0 || layer >= c.n_layers) return fail(RLHF_EINVAL, "layer index out of range");
  if (T <= 0 || B <= 0 || max_len <= 0) return fail(RLHF_EINVAL, "rows, batch and max_len must be positive");
  if (max_len > kMaxPos) return fail(RLHF_EUNSUPPORTED, "sequence longer than the rotary table");
  if ((size_t)T * 3 * (size_t)c.d_model >= ((size_t)1 << 32) - (size_t)384 * c.d_model)
    return fail(RLHF_EUNSUPPORTED, "too many rows");
  if (!x_in || !d_out || !cu_seqlens || !d_x || !d_ln1_g || !d_ln1_b || !d_w_qkv || !d_b_qkv || !d_w_o || !d_b_o ||
      !workspace)
    return fail(RLHF_EINVAL, "null pointer argument");
  const int dt = c.dtype, d = c.d_model, H = c.n_heads, hd = c.head_dim, l = layer;
  if ((hd % (dt == 0 ? 4 : 8)) != 0) return fail(RLHF_EUNSUPPORTED, "head_dim must be a multiple of 4 (fp32) or 8 (bf16)");
  if ((size_t)4 * (2 * (size_t)hd + 2 * (size_t)max_len) * sizeof(float) > 150 * 1024)
    return fail(RLHF_EUNSUPPORTED, "max_len too large for the attention kernels' scratch");
  Carver cv((void*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255));
  AttnBwdWs ws = carve_attn_bwd(cv, c, T, h->esz);
  if (cv.off + ((char*)cv.base - (char*)workspace) > workspace_bytes)
    return fail(RLHF_ENOMEM, "workspace too small for rlhf_attention_branch_backward");
  hipStream_t s = (hipStream_t)stream;
  const size_t esz = h->esz;
  const int Tp = ws.T_pad;
  const size_t ld_wo = h->ld_o2 ? (size_t)h->ld_o2 : (size_t)d;  // row stride of this layer's W_o
  const bool reordered = dt == 1;  // fp16 path: W_qkv's rows (and so the columns of qkv) are in the pair layout

  auto gemm = [&](const void* A, const void* W, const void* bias, void* out, int M, int N, int K, int epi) {
    GemmArgs g;
    g.A = A; g.W = W; g.bias = bias; g.out = out; g.M_max = M; g.M_dev = nullptr;
    g.N = N; g.K = K; g.ldo = N; g.epilogue = epi;
    return g;
  };
  // ---- the branch's forward, recomputed from the layer input: a = LN1(x), qkv = a Wqkv^T + b, rotary turn
  LAUNCH("final_ln", launch_final_ln(dt, x_in, nullptr, 0, T, nullptr, d, c.ln_eps, h->ln1_g[l], h->ln1_b[l], ws.a,
                                     nullptr, 0.f, nullptr, s));
  const bool kept = kept_q && kept_k && kept_v;
  if (kept && !attention_backward_takes_cache(dt, hd)) return fail(RLHF_EUNSUPPORTED, "kept K/V cache: head size");
  if (!kept) {
    LAUNCH("gemm_attn_fwd", launch_gemm(dt, gemm(ws.a, h->w_qkv[l], h->b_qkv[l], ws.qkv, T, 3 * d, d, EPI_BIAS), s));
    LAUNCH("rope_inplace", launch_rope_inplace(dt, ws.qkv, (size_t)3 * d, cu_seqlens, B, T, H, hd, c.rotary_dims,
                                               h->rope_cos, h->rope_sin, 0, s));
  }
  // ---- out-projection: dbo = sum_t G, do = G Wo
  const void* go = sh.go16 ? sh.go16 : ws.go;
  if (!sh.go16) {
    LAUNCH("colsum", launch_colsum(0, d_out, T, d, ws.part, ws.splits, d_b_o, s));
    LAUNCH("convert", launch_convert_from_f32(dt, d_out, ws.go, (size_t)T * d, s));
  }
  LAUNCH("attn_bwd_transpose", launch_transpose_pad(dt, h->w_o[l], ld_wo, ws.woT, (size_t)d, d, d, d, s));
  LAUNCH("gemm_attn_dx", launch_gemm(dt, gemm(go, ws.woT, nullptr, ws.dO, T, d, d, EPI_BIAS), s));
  // ---- attention core: (dq | dk | dv) into the sections of dqkv, and the forward output o
  char* qkv = (char*)ws.qkv;
  char* dqkv = (char*)ws.dqkv;
  if (kept)
    LAUNCH("attention_backward",
           launch_attention_backward(dt, kept_q, kept_k, kept_v, ws.dO, cu_seqlens, B, T, H, hd, max_len, ws.lse, ws.delta,
                                     dqkv, dqkv + (size_t)d * esz, dqkv + (size_t)2 * d * esz, s, (size_t)d, (size_t)d,
                                     (size_t)3 * d, ws.att, (size_t)d, true));
  else
    LAUNCH("attention_backward",
           launch_attention_backward(dt, qkv, qkv + (size_t)d * esz, qkv + (size_t)2 * d * esz, ws.dO, cu_seqlens, B, T, H,
                                     hd, max_len, ws.lse, ws.delta, dqkv, dqkv + (size_t)d * esz,
                                     dqkv + (size_t)2 * d * esz, s, (size_t)3 * d, (size_t)d, (size_t)3 * d, ws.att,
                                     (size_t)d));
  // ---- dWo = G^T o
  auto dw_gemm = [&](const void* A, const void* W, void* out, int M, int N) {  // K = the rows: sliced
    GemmArgs g = gemm(A, W, nullptr, out, M, N, Tp, EPI_F32);
    g.long_k = true;
    g.splitk_ws = ws.slabs;
    g.splitk_ws_bytes = ws.slabs_bytes;
    return g;
  };
  // Weight gradients straight from the row-major activations (K-major operands) where the kernel takes the shape;
  // the rows T .. Tp-1 of those operands are zeroed first.  Otherwise from transposed, zero-padded copies.
  auto dw_kmajor = [&](const void* A, const void* W, void* out, int M, int N) {
    GemmArgs g = dw_gemm(A, W, out, M, N);
    g.k_major = true;
    return g;
  };
  const bool kmaj = gemm_takes_k_major(dt, dw_kmajor(go, ws.att, d_w_o, d, d)) &&
                    gemm_takes_k_major(dt, dw_kmajor(ws.dqkv, ws.a, d_w_qkv, 3 * d, d));
  auto zero_tail = [&](void* buf, int width) {
    return Tp > T ? launch_fill_zero((char*)buf + (size_t)T * width * esz, (size_t)(Tp - T) * width * esz, s)
                  : hipSuccess;
  };
  if (kmaj) {
    if (!sh.go16) LAUNCH("attn_bwd_zero", zero_tail(ws.go, d));
    LAUNCH("attn_bwd_zero", zero_tail(ws.att, d));
    LAUNCH("gemm_attn_dw", launch_gemm(dt, dw_kmajor(go, ws.att, d_w_o, d, d), s));
  } else {
    LAUNCH("attn_bwd_transpose", launch_transpose_pad(dt, go, (size_t)d, ws.goT, (size_t)Tp, T, d, Tp, s));
    LAUNCH("attn_bwd_transpose", launch_transpose_pad(dt, ws.att, (size_t)d, ws.attT, (size_t)Tp, T, d, Tp, s));
    LAUNCH("gemm_attn_dw", launch_gemm(dt, dw_gemm(ws.goT, ws.attT, d_w_o, d, d), s));
  }
  // ---- back through the rotary turn, then the QKV product: dbqkv, dWqkv, da
  LAUNCH("rope_inplace", launch_rope_inplace(dt, ws.dqkv, (size_t)3 * d, cu_seqlens, B, T, H, hd, c.rotary_dims,
                                             h->rope_cos, h->rope_sin, 1, s));
  LAUNCH("colsum", launch_colsum(dt, ws.dqkv, T, 3 * d, ws.part, ws.splits, reordered ? ws.dbq : d_b_qkv, s));
  if (kmaj) {
    LAUNCH("attn_bwd_zero", zero_tail(ws.dqkv, 3 * d));
    LAUNCH("attn_bwd_zero", zero_tail(ws.a, d));
    LAUNCH("gemm_attn_dw", launch_gemm(dt, dw_kmajor(ws.dqkv, ws.a, reordered ? ws.dwq : d_w_qkv, 3 * d, d), s));
  } else {
    LAUNCH("attn_bwd_transpose", launch_transpose_pad(dt, ws.dqkv, (size_t)3 * d, ws.dqkvT, (size_t)Tp, T, 3 * d, Tp, s));
    LAUNCH("attn_bwd_transpose", launch_transpose_pad(dt, ws.a, (size_t)d, ws.aT, (size_t)Tp, T, d, Tp, s));
    LAUNCH("gemm_attn_dw", launch_gemm(dt, dw_gemm(ws.dqkvT, ws.aT, reordered ? ws.dwq : d_w_qkv, 3 * d, d), s));
  }
  if (reordered) {
    LAUNCH("qkv_rows", launch_qkv_rows_to_caller_order(ws.dwq, d_w_qkv, d, hd, c.rotary_dims, d, s));
    LAUNCH("qkv_rows", launch_qkv_rows_to_caller_order(ws.dbq, d_b_qkv, d, hd, c.rotary_dims, 1, s));
  }
  LAUNCH("attn_bwd_transpose", launch_transpose_pad(dt, h->w_qkv[l], (size_t)d, ws.wqkvT, (size_t)3 * d, 3 * d, d, 3 * d, s));
  LAUNCH("gemm_attn_dx", launch_gemm(dt, gemm(ws.dqkv, ws.wqkvT, nullptr, ws.da, T, d, 3 * d, EPI_F32), s));
  // ---- LN1: the branch's term of dL/dx, and the gradients of its gain and bias
  if (sh.base && !(ln_backward_rows_supported(dt, d) && (((uintptr_t)x_in | (uintptr_t)d_x | (uintptr_t)sh.base) & 15) == 0))
    return fail(RLHF_EUNSUPPORTED, "accumulating LayerNorm backward: shape");
  if (ln_backward_rows_supported(dt, d) && (((uintptr_t)x_in | (uintptr_t)d_x) & 15) == 0)
    LAUNCH("ln_backward", launch_ln_backward_rows(x_in, ws.da, h->ln1_g[l], T, d, c.ln_eps, d_x, ws.lnpart, d_ln1_g,
                                                  d_ln1_b, s, sh.base));
  else
    LAUNCH("head_ln_backward", launch_head_ln_backward(dt, x_in, ws.da, nullptr, 1.0f, nullptr, h->ln1_g[l], h->ln1_b[l],
                                                       T, d, c.ln_eps, d_x, ws.stats, ws.part, ws.splits, d_ln1_g,
                                                       d_ln1_b, nullptr, nullptr, s));
  return RLHF_OK;
}

int rollout_generate(rlhf_handle* h, const int32_t* queries, const uint8_t* pad_mask, int32_t B, int32_t Lq,
                     uint64_t seed, uint64_t seq_id_base, float temperature, int32_t max_new_tokens,
                     int32_t* out_tokens, float* out_logprobs, int32_t* out_lengths, uint8_t* out_mask,
                     void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_common(h, B, Lq);
  if (rc) return rc;
  if (max_new_tokens <= 0) return fail(RLHF_EINVAL, "max_new_tokens must be > 0");
  if (!(temperature > 0.f) || !std::isfinite(temperature)) return fail(RLHF_EINVAL, "temperature must be > 0");
  if (!queries || !pad_mask || !out_tokens || !out_logprobs || !out_lengths || !workspace)
    return fail(RLHF_EINVAL, "null pointer argument");
  if ((long)Lq + max_new_tokens > kMaxPos) return fail(RLHF_EUNSUPPORTED, "Lq + max_new_tokens too large");
  const rlhf_model_config& c = h->cfg;
  const int N = max_new_tokens;
  Carver cv((void*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255));
  RolloutWs ws = carve_rollout(cv, c, B, Lq, N, h->esz);
  if (cv.off + ((char*)cv.base - (char*)workspace) > workspace_bytes)
    return fail(RLHF_ENOMEM, "workspace too small for rollout_generate");
  hipStream_t s = (hipStream_t)stream;
  const int dt = c.dtype, d = c.d_model;
  for (int i = 0; i < 3; ++i)
    if (!h->ph[i]) HIP_OK(hipEventCreate(&h->ph[i]));
  h->ph_valid = false;
  HIP_OK(hipEventRecord(h->ph[0], s));

  const Meta& m = ws.meta;
  LAUNCH("copy_queries", launch_copy_queries(queries, pad_mask, B, Lq, N, c.pad_id, out_tokens, out_mask, s));
  LAUNCH("row_spans", launch_row_spans(pad_mask, B, Lq, N - 1, m.start, m.len, m.cu, m.kvoff, m.total, s));
  LAUNCH("pack_embed", launch_pack_embed(dt, queries, B, Lq, m.start, m.len, m.cu, h->w.embed_in, d, c.vocab,
                                         m.pos, m.rowid, m.tok, ws.acts.x, s));
  PassArgs p;
  p.mode = 0;
  p.rows_max = B * Lq;
  p.rows_dev = m.total;
  p.pos = m.pos;
  p.pos_add = 0;
  p.rowid = m.rowid;
  p.kvoff = m.kvoff;
  p.len = m.len;
  p.cu = m.cu;
  p.B = B;
  p.Lmax = Lq;
  p.ctx_add = 0;
  p.ctx_max = Lq + N;
  p.kv_extra = N - 1;
  p.kv = ws.kv;
  p.kv_slots = ws.kv_slots;
  p.kv_per_layer = true;
  p.last = c.n_layers > 0 ? &ws.last : nullptr;
  rc = run_layers(h, ws.acts, p, s);
  if (rc) return rc;
  p.last = nullptr;

  SampleArgs sa;
  sa.logits = ws.logits;
  sa.B = B; sa.V = c.vocab; sa.Lq = Lq; sa.N = N;
  sa.seed = seed; sa.seq_base = seq_id_base; sa.temperature = temperature;
  sa.eos_id = c.eos_id; sa.pad_id = c.pad_id;
  sa.len = m.len; sa.finished = ws.finished; sa.cur_tok = ws.cur_tok;
  sa.out_tokens = out_tokens; sa.out_logprobs = out_logprobs; sa.out_lengths = out_lengths; sa.out_mask = out_mask;

  GemmArgs lm;
  lm.A = ws.hl; lm.W = h->embed_out_mm; lm.bias = nullptr; lm.out = ws.logits;
  lm.M_max = B; lm.M_dev = nullptr; lm.N = c.vocab; lm.K = d; lm.ldo = c.vocab; lm.epilogue = EPI_F32;

  // last real position of every sequence: row b of the gathered rows (packed row cu[b+1] - 1 when
  // the model has no layers)
  if (c.n_layers > 0)
    LAUNCH("final_ln", launch_final_ln(dt, ws.last.x, nullptr, 0, B, nullptr, d, c.ln_eps, h->w.lnf_g, h->w.lnf_b,
                                       ws.hl, nullptr, 0.f, nullptr, s));
  else
    LAUNCH("final_ln", launch_final_ln(dt, ws.acts.x, m.cu + 1, -1, B, nullptr, d, c.ln_eps, h->w.lnf_g, h->w.lnf_b,
                                       ws.hl, nullptr, 0.f, nullptr, s));
  LAUNCH("gemm_lm_head_decode", launch_gemm(dt, lm, s));
  sa.step = 0;
  LAUNCH("sampler", launch_sampler(sa, s));
  HIP_OK(hipEventRecord(h->ph[1], s));

  // decode: pass t feeds the token sampled at step t (position len + t) and samples step t + 1
  p.mode = 1;
  p.rows_max = B;
  p.rows_dev = nullptr;
  p.pos = m.len;
  p.rowid = nullptr;
  for (int t = 0; t + 1 < N; ++t) {
    LAUNCH("embed_rows", launch_embed_rows(dt, ws.cur_tok, B, h->w.embed_in, d, c.vocab, ws.acts.x, s));
    p.pos_add = t;
    p.ctx_add = t + 1;
    rc = run_layers(h, ws.acts, p, s);
    if (rc) return rc;
    LAUNCH("final_ln", launch_final_ln(dt, ws.acts.x, nullptr, 0, B, nullptr, d, c.ln_eps, h->w.lnf_g, h->w.lnf_b,
                                       ws.hl, nullptr, 0.f, nullptr, s));
    LAUNCH("gemm_lm_head_decode", launch_gemm(dt, lm, s));
    sa.step = t + 1;
    LAUNCH("sampler", launch_sampler(sa, s));
  }
  HIP_OK(hipEventRecord(h->ph[2], s));
  h->ph_valid = true;
  return RLHF_OK;
}

// keep_q / keep_kv (training forward, with keep): buffers of [layers][keep_rows][d] and [layers][2][keep_rows * d]
// elements that receive every layer's rotated q rows and its K / V cache.
static int score_forward(rlhf_handle* h, const int32_t* tokens, const uint8_t* mask, int B, int L, ScoreWs& ws,
                         hipStream_t s, float* keep = nullptr, size_t keep_rows = 0, char* keep_q = nullptr,
                         char* keep_kv = nullptr, char* keep_u = nullptr, size_t keep_u_stride = 0,
                         int keep_u_layers = 0) {
  const rlhf_model_config& c = h->cfg;
  const Meta& m = ws.meta;
  LAUNCH("row_spans", launch_row_spans(mask, B, L, 0, m.start, m.len, m.cu, m.kvoff, m.total, s));
  LAUNCH("pack_embed", launch_pack_embed(c.dtype, tokens, B, L, m.start, m.len, m.cu, h->w.embed_in, c.d_model,
                                         c.vocab, m.pos, m.rowid, m.tok, ws.acts.x, s));
  PassArgs p;
  p.mode = 0;
  p.rows_max = B * L;
  p.rows_dev = m.total;
  p.pos = m.pos;
  p.pos_add = 0;
  p.rowid = m.rowid;
  p.kvoff = m.cu;  // the single-layer K/V scratch is indexed like the packed rows
  p.len = m.len;
  p.cu = m.cu;
  p.B = B;
  p.Lmax = L;
  p.ctx_add = 0;
  p.ctx_max = L;
  p.kv_extra = 0;
  p.kv = ws.kv;
  p.kv_slots = ws.Tmax;
  p.kv_per_layer = false;
  p.keep = keep;
  p.keep_rows = keep_rows ? keep_rows : (size_t)B * L;  // rows copied per layer = row stride of the kept slices
  p.keep_stride = p.keep_rows * c.d_model;
  if (keep && keep_q && keep_kv) {
    p.kv = keep_kv;
    p.kv_slots = p.keep_rows;
    p.kv_per_layer = true;
    p.q_keep = keep_q;
    p.q_keep_stride = p.keep_rows * c.d_model * h->esz;
  }
  if (keep && keep_u && keep_u_layers > 0) {
    p.u_keep = keep_u;
    p.u_keep_stride = keep_u_stride;
    p.u_keep_layers = keep_u_layers;
  }
  ws.sel_layers = false;
  if (ws.sel_rows) {
    LAUNCH("select_rows", launch_select_rows(ws.first_col, B, m.start, m.len, m.cu, m.tok, ws.sel_rows, ws.sel, ws.tgt,
                                             ws.n_sel, ws.sel_off, s));
    if (!keep && c.n_layers > 0) {  // a training forward keeps the final layer's output for every row
      p.sel = ws.sel;
      p.n_sel = ws.n_sel;
      p.sel_rows = ws.sel_rows;
      p.selz = &ws.z;
      ws.sel_layers = true;
    }
  }
  return run_layers(h, ws.acts, p, s);
}

// After score_forward: final LayerNorm + value head, LM head + log-softmax of the next token, and the packed ->
// padded [B, L] outputs.
static int score_tail(rlhf_handle* h, int B, int L, float temperature, ScoreWs& ws, float* out_logprobs,
                      float* out_values, hipStream_t s) {
  const rlhf_model_config& c = h->cfg;
  const Meta& m = ws.meta;
  const int dt = c.dtype, d = c.d_model;
  const int Tmax = B * L;
  const bool want_val = out_values && h->w.value_w;
  LseArgs la;
  la.inv_temperature = 1.0f / temperature;
  la.pmax = ws.pmax; la.psum = ws.psum; la.ztgt = ws.ztgt; la.vocab = c.vocab;
  GemmArgs lf;
  lf.W = h->embed_out_mm; lf.bias = nullptr; lf.out = nullptr; lf.M_sub = 0;
  lf.N = c.vocab; lf.K = d; lf.ldo = c.vocab; lf.epilogue = EPI_LSE; lf.lse = &la;
  if (ws.sel_rows) {
    // Scoring from a first column on: the LM head runs on the selected rows only.  Their final LayerNorm (and
    // value head) reads the final layer's output where it is: the selected rows' own buffer, or, after a forward
    // that ran every row through the final layer, the packed rows through the selection.
    if (ws.sel_layers) {
      LAUNCH("final_ln", launch_final_ln(dt, ws.z.x, nullptr, 0, ws.sel_rows, ws.n_sel, d, c.ln_eps, h->w.lnf_g,
                                         h->w.lnf_b, ws.z.a, want_val ? h->w.value_w : nullptr,
                                         h->value_b_dev ? 0.f : h->w.value_b, ws.val_sel, s));
    } else {
      LAUNCH("final_ln", launch_final_ln(dt, ws.acts.x, ws.sel, 0, ws.sel_rows, ws.n_sel, d, c.ln_eps, h->w.lnf_g,
                                         h->w.lnf_b, ws.z.a, want_val ? h->w.value_w : nullptr,
                                         h->value_b_dev ? 0.f : h->w.value_b, ws.val_sel, s));
    }
    la.tok = nullptr; la.pos = nullptr; la.T_dev = ws.n_sel; la.stride = ws.sel_rows;
    la.tgt = ws.tgt; la.dst = ws.sel;
    if (want_val) { la.val_in = ws.val_sel; la.val_out = ws.val; }
    lf.A = ws.z.a; lf.M_max = ws.sel_rows; lf.M_dev = ws.n_sel;
    LAUNCH("gemm_lm_head", launch_gemm(dt, lf, s));
    LAUNCH("lse_gather", launch_lse_combine(la, ws.sel_rows, ws.nparts, ws.lp, s));
    LAUNCH("unpack_scores", launch_unpack_scores(ws.lp, want_val ? ws.val : nullptr, B, L, m.start, m.len, m.cu,
                                                 out_logprobs, want_val ? out_values : nullptr, s,
                                                 want_val ? h->value_b_dev : nullptr, ws.first_col));
    return RLHF_OK;
  }
  // final LayerNorm of every packed row (into the LN1 buffer, free by now) + value head
  LAUNCH("final_ln", launch_final_ln(dt, ws.acts.x, nullptr, 0, Tmax, m.total, d, c.ln_eps, h->w.lnf_g,
                                     h->w.lnf_b, ws.acts.a, want_val ? h->w.value_w : nullptr,
                                     h->value_b_dev ? 0.f : h->w.value_b, ws.val, s));
  // LM head + log-softmax.  With enough rows for the large-M kernel the logits never leave the
  // accumulators: its epilogue reduces every part of a row (one wave's columns) to (max, sum of exp) and
  // picks out the target token's logit, and a small kernel combines the parts.  Otherwise the
  // logits of a chunk of rows are materialised and reduced by a second kernel.
  la.tok = m.tok; la.pos = m.pos; la.T_dev = m.total; la.stride = Tmax;
  lf.A = ws.acts.a; lf.M_max = Tmax; lf.M_dev = m.total;
  const bool fused_lm = ws.fused_lm;
  if (fused_lm) {
    LAUNCH("gemm_lm_head", launch_gemm(dt, lf, s));
    LAUNCH("lse_gather", launch_lse_combine(la, Tmax, ws.nparts, ws.lp, s));
  }
  for (int t0 = 0; t0 < Tmax && !fused_lm; t0 += ws.chunk) {
    const int rows = std::min(ws.chunk, Tmax - t0);
    GemmArgs lm;
    lm.A = (const char*)ws.acts.a + (size_t)t0 * d * h->esz;
    lm.W = h->embed_out_mm; lm.bias = nullptr; lm.out = ws.logits;
    lm.M_max = rows; lm.M_dev = m.total; lm.M_sub = t0;  // rows past the device-side token count are skipped
    lm.N = c.vocab; lm.K = d; lm.ldo = c.vocab; lm.epilogue = EPI_F32;
    LAUNCH("gemm_lm_head", launch_gemm(dt, lm, s));
    LAUNCH("lse_gather", launch_lse_gather(ws.logits, rows, t0, m.total, c.vocab, temperature, m.tok, m.pos, ws.lp,
                                           s));
  }
  LAUNCH("unpack_scores", launch_unpack_scores(ws.lp, want_val ? ws.val : nullptr, B, L, m.start, m.len, m.cu,
                                               out_logprobs, want_val ? out_values : nullptr, s,
                                               want_val ? h->value_b_dev : nullptr, ws.first_col));
  return RLHF_OK;
}

int score_sequences(rlhf_handle* h, const int32_t* tokens, const uint8_t* mask, int32_t B, int32_t L,
                    float temperature, float* out_logprobs, float* out_values, void* workspace,
                    size_t workspace_bytes, void* stream) {
  int rc = check_common(h, B, L);
  if (rc) return rc;
  if (!tokens || !mask || !out_logprobs || !workspace) return fail(RLHF_EINVAL, "null pointer argument");
  if (!(temperature > 0.f) || !std::isfinite(temperature)) return fail(RLHF_EINVAL, "temperature must be > 0");
  Carver cv((void*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255));
  ScoreWs ws = carve_score(cv, h->cfg, B, L, h->esz);
  if (cv.off + ((char*)cv.base - (char*)workspace) > workspace_bytes)
    return fail(RLHF_ENOMEM, "workspace too small for score_sequences");
  hipStream_t s = (hipStream_t)stream;
  rc = score_forward(h, tokens, mask, B, L, ws, s);
  if (rc) return rc;
  return score_tail(h, B, L, temperature, ws, out_logprobs, out_values, s);
}

int rlhf_score_responses_workspace_bytes(const rlhf_handle* h, int32_t B, int32_t L, int32_t first_col, size_t* out) {
  if (!h || !out) return fail(RLHF_EINVAL, "null argument");
  int rc = check_common(h, B, L);
  if (rc) return rc;
  Carver c(nullptr);
  carve_score(c, h->cfg, B, L, h->esz, first_col);
  *out = c.off + 256;
  return RLHF_OK;
}

int score_responses(rlhf_handle* h, const int32_t* tokens, const uint8_t* mask, int32_t B, int32_t L, int32_t first_col,
                    float temperature, float* out_logprobs, float* out_values, void* workspace,
                    size_t workspace_bytes, void* stream) {
  int rc = check_common(h, B, L);
  if (rc) return rc;
  if (!tokens || !mask || !out_logprobs || !workspace) return fail(RLHF_EINVAL, "null pointer argument");
  if (!(temperature > 0.f) || !std::isfinite(temperature)) return fail(RLHF_EINVAL, "temperature must be > 0");
  if (first_col < 0 || first_col > L) return fail(RLHF_EINVAL, "first_col must be in [0, L]");
  Carver cv((void*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255));
  ScoreWs ws = carve_score(cv, h->cfg, B, L, h->esz, first_col);
  if (cv.off + ((char*)cv.base - (char*)workspace) > workspace_bytes)
    return fail(RLHF_ENOMEM, "workspace too small for score_responses");
  hipStream_t s = (hipStream_t)stream;
  rc = score_forward(h, tokens, mask, B, L, ws, s);
  if (rc) return rc;
  return score_tail(h, B, L, temperature, ws, out_logprobs, out_values, s);
}

int rlhf_forward_keep(rlhf_handle* h, const int32_t* tokens, const uint8_t* mask, int32_t B, int32_t L, float* x_keep,
                      int32_t* cu_seqlens, int32_t* packed_tokens, void* workspace, size_t workspace_bytes,
                      void* stream) {
  int rc = check_common(h, B, L);
  if (rc) return rc;
  if (!tokens || !mask || !x_keep || !cu_seqlens || !packed_tokens || !workspace)
    return fail(RLHF_EINVAL, "null pointer argument");
  const rlhf_model_config& c = h->cfg;
  Carver cv((void*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255));
  ScoreWs ws = carve_score(cv, c, B, L, h->esz);
  if (cv.off + ((char*)cv.base - (char*)workspace) > workspace_bytes)
    return fail(RLHF_ENOMEM, "workspace too small for rlhf_forward_keep");
  hipStream_t s = (hipStream_t)stream;
  rc = score_forward(h, tokens, mask, B, L, ws, s, x_keep);
  if (rc) return rc;
  HIP_OK(hipMemcpyAsync(cu_seqlens, ws.meta.cu, (size_t)(B + 1) * sizeof(int32_t), hipMemcpyDeviceToDevice, s));
  HIP_OK(hipMemcpyAsync(packed_tokens, ws.meta.tok, (size_t)B * L * sizeof(int32_t), hipMemcpyDeviceToDevice, s));
  return RLHF_OK;
}

int rlhf_policy_backward_workspace_bytes(const rlhf_handle* h, int32_t T, size_t* out) {
  if (!h || !out) return fail(RLHF_EINVAL, "null argument");
  if (T <= 0) return fail(RLHF_EINVAL, "row count must be positive");
  size_t a = 0, b = 0, c = 0;
  int rc = rlhf_head_backward_workspace_bytes(h, T, &a);
  if (rc) return rc;
  if (h->cfg.n_layers > 0) {
    rc = rlhf_mlp_backward_workspace_bytes(h, T, &b);
    if (rc) return rc;
    rc = rlhf_attention_branch_backward_workspace_bytes(h, T, &c);
    if (rc) return rc;
  }
  // four [T, d] float buffers, the shared fp16 copy of the stream's gradient (rows padded to 128) and its column-sum scratch
  const size_t Tp = ((size_t)T + 127) & ~(size_t)127;
  *out = std::max(a, std::max(b, c)) + (size_t)4 * T * h->cfg.d_model * sizeof(float) + Tp * h->cfg.d_model * h->esz +
         (size_t)256 * h->cfg.d_model * sizeof(float) + 4096;
  return RLHF_OK;
}

// sel (optional): the sel_rows packed rows (*n_sel of them real) outside which targets, d_logprobs and d_values
// carry nothing: the output heads' backward pass then runs on those rows only.
static int policy_backward_impl(rlhf_handle* h, const float* x_keep, int64_t x_keep_layer_stride,
                                const int32_t* cu_seqlens, const int32_t* packed_tokens, int32_t B, int32_t T,
                                int32_t max_len, const int32_t* targets, const float* d_logprobs, const float* d_values,
                                float temperature, float grad_scale, const rlhf_grads* g, void* workspace,
                                size_t workspace_bytes, void* stream, const int* sel, int sel_rows, const int* n_sel,
                                const char* kept_q = nullptr, const char* kept_kv = nullptr,
                                const char* kept_u = nullptr, size_t kept_u_stride = 0, int kept_u_layers = 0);

int rlhf_policy_backward(rlhf_handle* h, const float* x_keep, int64_t x_keep_layer_stride, const int32_t* cu_seqlens,
                         const int32_t* packed_tokens, int32_t B, int32_t T, int32_t max_len, const int32_t* targets,
                         const float* d_logprobs, const float* d_values, float temperature, float grad_scale,
                         const rlhf_grads* g, void* workspace, size_t workspace_bytes, void* stream) {
  return policy_backward_impl(h, x_keep, x_keep_layer_stride, cu_seqlens, packed_tokens, B, T, max_len, targets,
                              d_logprobs, d_values, temperature, grad_scale, g, workspace, workspace_bytes, stream,
                              nullptr, 0, nullptr);
}

static int policy_backward_impl(rlhf_handle* h, const float* x_keep, int64_t x_keep_layer_stride,
                                const int32_t* cu_seqlens, const int32_t* packed_tokens, int32_t B, int32_t T,
                                int32_t max_len, const int32_t* targets, const float* d_logprobs, const float* d_values,
                                float temperature, float grad_scale, const rlhf_grads* g, void* workspace,
                                size_t workspace_bytes, void* stream, const int* sel, int sel_rows, const int* n_sel,
                                const char* kept_q, const char* kept_kv, const char* kept_u, size_t kept_u_stride,
                                int kept_u_layers) {
  // kept_q / kept_kv: what score_forward's keep_q / keep_kv received, with keep_rows = x_keep_layer_stride / d_model
  if (!h || !g) return fail(RLHF_EINVAL, "null argument");
  const rlhf_model_config& c = h->cfg;
  if (T <= 0 || B <= 0) return fail(RLHF_EINVAL, "rows and batch must be positive");
  if (!x_keep || !cu_seqlens || !packed_tokens || !workspace || !g->embed_in)
    return fail(RLHF_EINVAL, "null pointer argument");
  if (x_keep_layer_stride < (int64_t)T * c.d_model) return fail(RLHF_EINVAL, "x_keep_layer_stride smaller than T * d_model");
  float* const* per_layer[12] = {g->ln1_g, g->ln1_b, g->ln2_g, g->ln2_b, g->w_qkv, g->b_qkv,
                                 g->w_o,   g->b_o,   g->w_fc1, g->b_fc1, g->w_fc2, g->b_fc2};
  for (auto p : per_layer) {
    if (c.n_layers > 0 && !p) return fail(RLHF_EINVAL, "null per-layer gradient pointer array");
    for (int l = 0; l < c.n_layers; ++l)
      if (!p[l]) return fail(RLHF_EINVAL, "null per-layer gradient pointer");
  }
  if (c.d_model > 8192) return fail(RLHF_EUNSUPPORTED, "d_model > 8192");
  size_t need = 0;
  int rc = rlhf_policy_backward_workspace_bytes(h, T, &need);
  if (rc) return rc;
  if (workspace_bytes < need) return fail(RLHF_ENOMEM, "workspace too small for rlhf_policy_backward");
  hipStream_t s = (hipStream_t)stream;
  const size_t n = (size_t)T * c.d_model;
  char* base = (char*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255);
  const size_t buf = (n * sizeof(float) + 255) & ~(size_t)255;
  float* dx = (float*)base;                 // gradient of the residual stream at the current depth
  float* dx_m = (float*)(base + buf);       // MLP branch term
  float* dx_a = (float*)(base + 2 * buf);   // attention branch term
  float* dx_n = (float*)(base + 3 * buf);   // their sum with dx: the gradient one layer down
  // shared by a layer's two branches: the fp16 copy of dx (zero padding rows) and the scratch of its column sums
  const size_t Tp = ((size_t)T + 127) & ~(size_t)127;
  const size_t go_bytes = (Tp * c.d_model * h->esz + 255) & ~(size_t)255;
  const size_t part_bytes = ((size_t)256 * c.d_model * sizeof(float) + 255) & ~(size_t)255;
  char* go16 = base + 4 * buf;
  float* go_part = (float*)(go16 + go_bytes);
  char* sub = go16 + go_bytes + part_bytes;
  const size_t sub_bytes = workspace_bytes - (size_t)(sub - (char*)workspace);
  // one conversion and one set of column sums of dx per layer for both branches, and each branch's LayerNorm
  // backward adding onto the running sum (dx + MLP term, then + attention term) -- where the one-pass kernel runs
  const bool share = c.dtype == 1 && c.n_layers > 0 && ln_backward_rows_supported(c.dtype, c.d_model) && (c.d_model & 3) == 0;
  const int go_splits = std::max(1, std::min(256, (T + 255) / 256));
  if (share && Tp > (size_t)T)
    LAUNCH("convert", launch_fill_zero(go16 + (size_t)T * c.d_model * h->esz, (Tp - T) * c.d_model * h->esz, s));
  const float* x_final = x_keep + (size_t)c.n_layers * x_keep_layer_stride;
  if (sel && sel_rows > 0 && sel_rows < T) {
    // the heads on the selected rows: their inputs gathered into the (still free) branch buffers, the input
    // gradient scattered back into a zeroed dx
    const size_t rb = (size_t)c.d_model * sizeof(float);
    float *x_sel = dx_m, *dx_sel = dx_a;
    int* t_sel = (int*)dx_n;
    float *gl_sel = dx_n + sel_rows, *gv_sel = dx_n + 2 * (size_t)sel_rows;
    LAUNCH("gather_sel", launch_gather_rows_strided(x_final, rb, sel, sel_rows, rb, x_sel, rb, s));
    LAUNCH("gather_sel", launch_gather_row_scalars(sel, n_sel, sel_rows, targets, d_logprobs, d_values, t_sel, gl_sel,
                                                   gv_sel, s));
    rc = rlhf_head_backward(h, x_sel, t_sel, gl_sel, gv_sel, sel_rows, temperature, grad_scale, dx_sel, g->lnf_g,
                            g->lnf_b, g->embed_out, g->value_w, g->value_b, sub, sub_bytes, stream);
    if (rc) return rc;
    LAUNCH("gather_sel", launch_fill_zero(dx, n * sizeof(float), s));
    LAUNCH("gather_sel", launch_scatter_rows(dx_sel, sel, n_sel, sel_rows, rb, dx, s));
  } else {
    rc = rlhf_head_backward(h, x_final, targets, d_logprobs, d_values, T, temperature, grad_scale, dx, g->lnf_g,
                            g->lnf_b, g->embed_out, g->value_w, g->value_b, sub, sub_bytes, stream);
    if (rc) return rc;
  }
  for (int l = c.n_layers - 1; l >= 0; --l) {
    const float* xl = x_keep + (size_t)l * x_keep_layer_stride;
    if (share) {
      LAUNCH("convert", launch_convert_colsum(dx, T, c.d_model, go_part, go_splits, g->b_fc2[l], go16, s));
      HIP_OK(hipMemcpyAsync(g->b_o[l], g->b_fc2[l], (size_t)c.d_model * sizeof(float), hipMemcpyDeviceToDevice, s));
    }
    BranchShare sm, sa;
    if (share) {
      sm.go16 = sa.go16 = go16;
      sm.base = dx;    // dx_m = dx + MLP term
      sa.base = dx_m;  // dx_n = dx_m + attention term
    }
    if (kept_u && l < kept_u_layers) sm.kept_u = kept_u + (size_t)l * kept_u_stride;
    rc = mlp_backward_impl(h, l, xl, dx, T, dx_m, g->ln2_g[l], g->ln2_b[l], g->w_fc1[l], g->b_fc1[l], g->w_fc2[l],
                           g->b_fc2[l], sub, sub_bytes, stream, sm);
    if (rc) return rc;
    const size_t plane = (size_t)x_keep_layer_stride * h->esz;  // bytes of one layer's q rows, K plane or V plane
    const char* kq = kept_q && kept_kv ? kept_q + (size_t)l * plane : nullptr;
    const char* kk = kq ? kept_kv + (size_t)l * 2 * plane : nullptr;
    rc = attention_branch_backward_impl(h, l, xl, dx, cu_seqlens, B, T, max_len, share ? dx_n : dx_a, g->ln1_g[l],
                                        g->ln1_b[l], g->w_qkv[l], g->b_qkv[l], g->w_o[l], g->b_o[l], sub, sub_bytes, stream,
                                        kq, kk, kk ? kk + plane : nullptr, sa);
    if (rc) return rc;
    if (!share) LAUNCH("add3", launch_add3(dx, dx_a, dx_m, dx_n, n, s));
    std::swap(dx, dx_n);
  }
  LAUNCH("embed_backward", launch_embed_backward(packed_tokens, dx, T, c.d_model, c.vocab, g->embed_in, s));
  return RLHF_OK;
}

namespace {
struct UpdateWs {
  ScoreWs score;
  char *q_keep = nullptr, *kv_keep = nullptr;  // every layer's rotated q rows and K / V cache (where the backward
                                               // pass's attention kernels read that layout), else null
  char* u_keep = nullptr;      // FC1 pre-activations of the first u_layers layers: whatever workspace the caller
  size_t u_stride = 0;         // gave beyond the minimum
  int u_layers = 0;
  float *x_keep, *lp_full, *val_full, *new_lp, *new_v, *d_lp, *d_v, *gl, *gv;
  int32_t* targets;
  void* bwd;
  size_t bwd_bytes;
};
UpdateWs carve_update(Carver& c, const rlhf_handle* h, int Bm, int L, int N, int T_max) {
  UpdateWs w;
  const rlhf_model_config& cfg = h->cfg;
  w.score = carve_score(c, cfg, Bm, L, h->esz, L - N);  // log-probs and values are read from column L - N - 1 on
  w.x_keep = c.take<float>((size_t)(cfg.n_layers + 1) * T_max * cfg.d_model);
  if (cfg.n_layers > 0 && attention_backward_takes_cache(cfg.dtype, cfg.head_dim)) {
    w.q_keep = (char*)c.take_bytes((size_t)cfg.n_layers * T_max * cfg.d_model * h->esz);
    w.kv_keep = (char*)c.take_bytes((size_t)cfg.n_layers * 2 * T_max * cfg.d_model * h->esz);
  }
  w.lp_full = c.take<float>((size_t)Bm * L);
  w.val_full = c.take<float>((size_t)Bm * L);
  w.new_lp = c.take<float>((size_t)Bm * N);
  w.new_v = c.take<float>((size_t)Bm * N);
  w.d_lp = c.take<float>((size_t)Bm * N);
  w.d_v = c.take<float>((size_t)Bm * N);
  w.gl = c.take<float>((size_t)T_max);
  w.gv = c.take<float>((size_t)T_max);
  w.targets = c.take<int32_t>((size_t)T_max);
  size_t b = 0;
  (void)rlhf_policy_backward_workspace_bytes(h, T_max, &b);
  w.bwd_bytes = b;
  w.bwd = c.take_bytes(b);
  return w;
}
}  // namespace

int rlhf_ppo_update_workspace_bytes(const rlhf_handle* h, int32_t B_minibatch, int32_t L, int32_t N, int32_t T_max,
                                    size_t* out) {
  if (!h || !out) return fail(RLHF_EINVAL, "null argument");
  if (B_minibatch <= 0 || L <= 0 || N <= 0 || N > L || T_max <= 0 || (size_t)T_max > (size_t)B_minibatch * L)
    return fail(RLHF_EINVAL, "bad mini-batch shape");
  Carver c(nullptr);
  carve_update(c, h, B_minibatch, L, N, T_max);
  *out = c.off + 256;
  return RLHF_OK;
}

int rlhf_ppo_update(rlhf_handle* h, const rlhf_ppo_update_config* cfg, const rlhf_train_state* st,
                    const int32_t* tokens, const uint8_t* mask, int32_t B, int32_t Lq, int32_t N,
                    const float* old_logprobs, const float* advantages, const float* old_values, const float* returns,
                    const int32_t* kept, const int32_t* minibatch_tokens, int32_t max_len, float* out_stats,
                    void* workspace, size_t workspace_bytes, void* stream) {
  if (!h || !cfg || !st) return fail(RLHF_EINVAL, "null argument");
  const rlhf_model_config& c = h->cfg;
  if (!tokens || !mask || !old_logprobs || !advantages || !old_values || !returns || !kept || !minibatch_tokens ||
      !out_stats || !workspace)
    return fail(RLHF_EINVAL, "null pointer argument");
  if (B <= 0 || Lq <= 0 || N <= 0) return fail(RLHF_EINVAL, "batch, query length and response length must be positive");
  if (cfg->epochs <= 0 || cfg->n_minibatches <= 0 || B % cfg->n_minibatches != 0)
    return fail(RLHF_EINVAL, "epochs and n_minibatches must be positive and n_minibatches must divide the batch");
  if (cfg->first_step < 1) return fail(RLHF_EINVAL, "first_step counts from 1");
  if (!(cfg->temperature > 0.f) || !std::isfinite(cfg->temperature)) return fail(RLHF_EINVAL, "temperature must be > 0");
  if (!(cfg->grad_scale > 0.f) || !std::isfinite(cfg->grad_scale)) return fail(RLHF_EINVAL, "grad_scale must be finite and > 0");
  if (!h->w.value_w) return fail(RLHF_EUNSUPPORTED, "the update trains the value head as well: the model needs one");
  const int L = Lq + N, Bm = B / cfg->n_minibatches;
  int rc = check_common(h, Bm, L);
  if (rc) return rc;
  int T_max = 0;
  for (int j = 0; j < cfg->n_minibatches; ++j) {
    if (minibatch_tokens[j] <= 0 || (size_t)minibatch_tokens[j] > (size_t)Bm * L)
      return fail(RLHF_EINVAL, "minibatch_tokens: every mini-batch needs between 1 and B_minibatch * L real tokens");
    T_max = std::max(T_max, minibatch_tokens[j]);
  }
  const bool bf16 = c.dtype == RLHF_DTYPE_BF16;
  // ---- every trainable tensor: the caller's weight array, its gradient buffer and optimizer state
  struct Tensor { void* weight; float *grad, *master, *m, *v; size_t n; };
  std::vector<Tensor> ts;
  const size_t d = c.d_model, F = c.d_ff, V = c.vocab;
  auto add = [&](const void* wt, float* g, float* ms, float* m, float* v, size_t n) {
    ts.push_back(Tensor{(void*)wt, g, ms, m, v, n});
  };
  const rlhf_grads &G = st->grads, &P = st->master, &M1 = st->exp_avg, &M2 = st->exp_avg_sq;
  add(h->w.embed_in, G.embed_in, P.embed_in, M1.embed_in, M2.embed_in, V * d);
  add(h->w.embed_out, G.embed_out, P.embed_out, M1.embed_out, M2.embed_out, V * d);
  add(h->w.lnf_g, G.lnf_g, P.lnf_g, M1.lnf_g, M2.lnf_g, d);
  add(h->w.lnf_b, G.lnf_b, P.lnf_b, M1.lnf_b, M2.lnf_b, d);
  add(h->w.value_w, G.value_w, P.value_w, M1.value_w, M2.value_w, d);
  float* const* gl_[12] = {G.ln1_g, G.ln1_b, G.ln2_g, G.ln2_b, G.w_qkv, G.b_qkv, G.w_o, G.b_o, G.w_fc1, G.b_fc1, G.w_fc2, G.b_fc2};
  float* const* pl_[12] = {P.ln1_g, P.ln1_b, P.ln2_g, P.ln2_b, P.w_qkv, P.b_qkv, P.w_o, P.b_o, P.w_fc1, P.b_fc1, P.w_fc2, P.b_fc2};
  float* const* ml_[12] = {M1.ln1_g, M1.ln1_b, M1.ln2_g, M1.ln2_b, M1.w_qkv, M1.b_qkv, M1.w_o, M1.b_o, M1.w_fc1, M1.b_fc1, M1.w_fc2, M1.b_fc2};
  float* const* vl_[12] = {M2.ln1_g, M2.ln1_b, M2.ln2_g, M2.ln2_b, M2.w_qkv, M2.b_qkv, M2.w_o, M2.b_o, M2.w_fc1, M2.b_fc1, M2.w_fc2, M2.b_fc2};
  const std::vector<const void*>* wl_[12] = {&h->ln1_g, &h->ln1_b, &h->ln2_g, &h->ln2_b, &h->src_w_qkv, &h->src_b_qkv,
                                            &h->src_w_o, &h->b_o, &h->src_w_fc1, &h->b_fc1, &h->src_w_fc2, &h->b_fc2};
  const size_t nl_[12] = {d, d, d, d, 3 * d * d, 3 * d, d * d, d, F * d, F, d * F, d};
  for (int i = 0; i < 12; ++i) {
    if (c.n_layers > 0 && (!gl_[i] || !ml_[i] || !vl_[i] || (bf16 && !pl_[i])))
      return fail(RLHF_EINVAL, "null per-layer array in the training state");
    for (int l = 0; l < c.n_layers; ++l)
      add((*wl_[i])[l], gl_[i][l], bf16 ? pl_[i][l] : nullptr, ml_[i][l], vl_[i][l], nl_[i]);
  }
  for (const Tensor& t : ts)
    if (!t.weight || !t.grad || !t.m || !t.v || (bf16 && !t.master))
      return fail(RLHF_EINVAL, "null tensor in the training state");
  if (!G.value_b || !P.value_b || !M1.value_b || !M2.value_b)
    return fail(RLHF_EINVAL, "the value bias needs a gradient, a master copy and both moments (device floats)");
  Carver cv((void*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255));
  UpdateWs ws = carve_update(cv, h, Bm, L, N, T_max);
  if (cv.off + ((char*)cv.base - (char*)workspace) > workspace_bytes)
    return fail(RLHF_ENOMEM, "workspace too small for rlhf_ppo_update");
  if (bf16 && c.n_layers > 0) {  // what the caller gave beyond the minimum keeps FC1 pre-activations, layer by layer
    const size_t used = ((cv.off + 255) & ~(size_t)255) + (size_t)((char*)cv.base - (char*)workspace);
    ws.u_stride = (((size_t)T_max * c.d_ff * h->esz) + 255) & ~(size_t)255;
    ws.u_layers = (int)std::min<size_t>((size_t)c.n_layers, (workspace_bytes - used) / ws.u_stride);
    ws.u_keep = ws.u_layers > 0 ? (char*)workspace + used : nullptr;
  }
  hipStream_t s = (hipStream_t)stream;
  // from here on the value head's bias is the device scalar the optimizer updates
  h->value_b_dev = P.value_b;
  int step = cfg->first_step;
  for (int ep = 0; ep < cfg->epochs; ++ep) {
    for (int j = 0; j < cfg->n_minibatches; ++j, ++step) {
      const size_t r0 = (size_t)j * Bm;
      const int32_t* tok_j = tokens + r0 * L;
      const uint8_t* mask_j = mask + r0 * L;
      const int T = minibatch_tokens[j];
      // forward with the current weights, keeping the layer inputs (packed rows: slices of T rows)
      rc = score_forward(h, tok_j, mask_j, Bm, L, ws.score, s, ws.x_keep, (size_t)T, ws.q_keep, ws.kv_keep, ws.u_keep,
                         ws.u_stride, ws.u_layers);
      if (rc) return rc;
      rc = score_tail(h, Bm, L, cfg->temperature, ws.score, ws.lp_full, ws.val_full, s);
      if (rc) return rc;
      LAUNCH("ppo_glue", launch_ppo_slice(ws.lp_full, ws.val_full, Bm, L, Lq, N, ws.new_lp, ws.new_v, s));
      float* stats = out_stats + ((size_t)ep * cfg->n_minibatches + j) * 8;
      LAUNCH("ppo_loss", launch_ppo_loss(ws.new_lp, old_logprobs + r0 * N, advantages + r0 * N, ws.new_v,
                                         old_values + r0 * N, returns + r0 * N, kept + r0, Bm, N, cfg->cliprange,
                                         cfg->cliprange_value, cfg->vf_coef, ws.d_lp, ws.d_v, stats, s));
      const Meta& m = ws.score.meta;
      LAUNCH("ppo_glue", launch_ppo_pack_grads(tok_j, Bm, L, Lq, N, m.start, m.len, m.cu, ws.d_lp, ws.d_v, ws.targets,
                                               ws.gl, ws.gv, s));
      rc = policy_backward_impl(h, ws.x_keep, (int64_t)T * c.d_model, m.cu, m.tok, Bm, T, max_len, ws.targets, ws.gl,
                                ws.gv, cfg->temperature, cfg->grad_scale, &G, ws.bwd, ws.bwd_bytes, stream,
                                ws.score.sel_rows ? ws.score.sel : nullptr, ws.score.sel_rows, ws.score.n_sel,
                                ws.q_keep, ws.kv_keep, ws.u_keep, ws.u_stride, ws.u_layers);
      if (rc) return rc;
      // AdamW on every tensor; a bf16 model keeps fp32 masters and gets its storage arrays rewritten
      const double inv_scale = 1.0 / (double)cfg->grad_scale;
      for (const Tensor& t : ts) {
        rc = rlhf_adamw_step(bf16 ? t.master : (float*)t.weight, t.grad, t.m, t.v, bf16 ? (uint16_t*)t.weight : nullptr,
                             t.n, step, cfg->lr, cfg->beta1, cfg->beta2, cfg->eps, cfg->weight_decay, inv_scale, stream);
        if (rc) return rc;
      }
      rc = rlhf_adamw_step(P.value_b, G.value_b, M1.value_b, M2.value_b, nullptr, 1, step, cfg->lr, cfg->beta1,
                           cfg->beta2, cfg->eps, cfg->weight_decay, inv_scale, stream);
      if (rc) return rc;
      rc = rlhf_refresh_weights(h, stream);
      if (rc) return rc;
    }
  }
  return RLHF_OK;
}

int rlhf_debug_logits_rows(rlhf_handle* h, const int32_t* tokens, const uint8_t* mask, int32_t B, int32_t L,
                           const int32_t* rows_bt, int32_t n, float* out_logits, void* workspace,
                           size_t workspace_bytes, void* stream) {
  int rc = check_common(h, B, L);
  if (rc) return rc;
  if (!tokens || !mask || !rows_bt || !out_logits || !workspace) return fail(RLHF_EINVAL, "null pointer argument");
  if (n <= 0 || (size_t)n > (size_t)B * L) return fail(RLHF_EINVAL, "bad row count");
  for (int i = 0; i < n; ++i)
    if (rows_bt[2 * i] < 0 || rows_bt[2 * i] >= B || rows_bt[2 * i + 1] < 0 || rows_bt[2 * i + 1] >= L)
      return fail(RLHF_EINVAL, "row index out of range");
  const rlhf_model_config& c = h->cfg;
  Carver cv((void*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255));
  ScoreWs ws = carve_score(cv, c, B, L, h->esz);
  if (cv.off + ((char*)cv.base - (char*)workspace) > workspace_bytes)
    return fail(RLHF_ENOMEM, "workspace too small");
  hipStream_t s = (hipStream_t)stream;
  rc = score_forward(h, tokens, mask, B, L, ws, s);
  if (rc) return rc;
  HIP_OK(hipMemcpyAsync(ws.rows_dev, rows_bt, sizeof(int32_t) * 2 * n, hipMemcpyHostToDevice, s));
  HIP_OK(hipStreamSynchronize(s));  // rows_bt is pageable host memory: the one host sync of this debug call
  LAUNCH("rows_to_packed", launch_rows_to_packed(ws.rows_dev, n, ws.meta.start, ws.meta.cu, ws.idx, s));
  LAUNCH("final_ln", launch_final_ln(c.dtype, ws.acts.x, ws.idx, 0, n, nullptr, c.d_model, c.ln_eps, h->w.lnf_g,
                                     h->w.lnf_b, ws.acts.a, nullptr, 0.f, nullptr, s));
  GemmArgs lm;
  lm.A = ws.acts.a; lm.W = h->embed_out_mm; lm.bias = nullptr; lm.out = out_logits;
  lm.M_max = n; lm.M_dev = nullptr; lm.N = c.vocab; lm.K = c.d_model; lm.ldo = c.vocab; lm.epilogue = EPI_F32;
  LAUNCH("gemm_lm_head", launch_gemm(c.dtype, lm, s));
  return RLHF_OK;
}

int rlhf_profile_enable(rlhf_handle* h, int32_t on) {
  if (!h) return fail(RLHF_EINVAL, "null handle");
  h->prof_on = on != 0;
  h->prof_names.clear();
  h->prof_ev.clear();
  h->ev_used = 0;
  return RLHF_OK;
}

int rlhf_profile_read(rlhf_handle* h, int32_t cap, const char** names, double* total_ms, int64_t* launches,
                      int32_t* n_out) {
  if (!h || !n_out) return fail(RLHF_EINVAL, "null argument");
  std::map<std::string, std::pair<double, int64_t>> agg;
  std::map<std::string, const char*> ptr;
  const size_t n = std::min(h->prof_names.size(), h->prof_ev.size() / 2);
  if (n) HIP_OK(hipEventSynchronize(h->prof_ev[2 * n - 1]));
  for (size_t i = 0; i < n; ++i) {
    float ms = 0.f;
    HIP_OK(hipEventElapsedTime(&ms, h->prof_ev[2 * i], h->prof_ev[2 * i + 1]));
    auto& a = agg[h->prof_names[i]];
    a.first += ms;
    a.second += 1;
    ptr[h->prof_names[i]] = h->prof_names[i];
  }
  int k = 0;
  for (auto& kv : agg) {
    if (k < cap) {
      if (names) names[k] = ptr[kv.first];
      if (total_ms) total_ms[k] = kv.second.first;
      if (launches) launches[k] = kv.second.second;
    }
    ++k;
  }
  *n_out = k;
  h->prof_names.clear();
  h->prof_ev.clear();
  h->ev_used = 0;
  return RLHF_OK;
}

int rlhf_last_rollout_phases(rlhf_handle* h, double* prefill_ms, double* decode_ms) {
  if (!h || !prefill_ms || !decode_ms) return fail(RLHF_EINVAL, "null argument");
  if (!h->ph_valid) return fail(RLHF_EINVAL, "no completed rollout_generate on this handle");
  HIP_OK(hipEventSynchronize(h->ph[2]));
  float a = 0.f, b = 0.f;
  HIP_OK(hipEventElapsedTime(&a, h->ph[0], h->ph[1]));
  HIP_OK(hipEventElapsedTime(&b, h->ph[1], h->ph[2]));
  *prefill_ms = a;
  *decode_ms = b;
  return RLHF_OK;
}

}  // extern "C"
