// Stand-alone driver for the few-rows (decode) products of a model layer: the QKV, out-projection, FC1, FC2 and
// LM-head shapes at M rows (the batch), through the library's own launch_gemm.  Each shape is checked on sampled
// outputs against a double-precision dot product on the host, then timed with HIP events twice: on one weight
// matrix (warm: it stays in the caches) and rotating over more than 1 GB of weight copies (cold: every launch
// streams its weights from HBM, as a decode pass does).  Like the other drivers it exists because hardware
// counters (rocprofv3 --pmc) can be collected on a small native process where they cannot on the Python benchmark.
//   usage: dec_driver [M=256] [d_model=2560] [reps=96] [max_split=0] [timed_phase=0] [pad_a=0] [pad_w=0]
//   (pad_a / pad_w: elements added to the row strides of A / W, to see what the address-to-channel mapping costs)
//   (timed_phase 1 times the partial products alone, as the decode loop runs them: their reductions are folded
//   into the kernels that consume them)
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "common.h"

using namespace rlhf;

#define CK(x)                                                                               \
  do {                                                                                      \
    hipError_t e_ = (x);                                                                    \
    if (e_ != hipSuccess) {                                                                 \
      printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__);         \
      return 1;                                                                             \
    }                                                                                       \
  } while (0)

static uint16_t f2h(float f) { _Float16 h = (_Float16)f; uint16_t u; memcpy(&u, &h, 2); return u; }
static float h2f(uint16_t u) { _Float16 h; memcpy(&h, &u, 2); return (float)h; }
static uint16_t f2bf(float f) { unsigned u; memcpy(&u, &f, 4); u += 0x7FFF + ((u >> 16) & 1); return (uint16_t)(u >> 16); }
static float bf2f(uint16_t h) { unsigned u = ((unsigned)h) << 16; float f; memcpy(&f, &u, 4); return f; }

int main(int argc, char** argv) {
  const int M = argc > 1 ? atoi(argv[1]) : 256;
  const int d = argc > 2 ? atoi(argv[2]) : 2560, F = 4 * d, V = 50304;
  const int reps = argc > 3 ? atoi(argv[3]) : 96;
  const int max_split = argc > 4 ? atoi(argv[4]) : 0;
  const int timed_phase = argc > 5 ? atoi(argv[5]) : 0;
  const int pad_a = argc > 6 ? atoi(argv[6]) : 0, pad_w = argc > 7 ? atoi(argv[7]) : 0;
  if (M <= 0 || M > 512 || d % 64 != 0) { printf("M must be 1..512 and d_model a multiple of 64\n"); return 1; }
  struct Shape { const char* name; int N, K, epi; } shapes[] = {
      {"qkv", 3 * d, d, EPI_BIAS}, {"out", d, d, EPI_BIAS_RESADD}, {"fc1", F, d, EPI_BIAS_GELU}, {"fc2", d, F, EPI_BIAS_RESADD},
      {"lm_head", V, d, EPI_F32}};
  const size_t wmax = (size_t)std::max(F, V) * (d + pad_w) + (size_t)d * (F + pad_w);  // elements of the largest matrix, padded
  const int R = (int)(((size_t)1200 << 20) / (wmax * 2)) + 1;  // copies: more than 1.2 GB in all
  std::vector<uint16_t> hA((size_t)M * (F + pad_a)), hW(wmax), hb(std::max(F, V));
  srand(1);
  for (auto& x : hA) x = f2h((rand() % 2001 - 1000) / 1000.0f);
  for (auto& x : hW) x = f2h((rand() % 2001 - 1000) / 25000.0f);
  for (auto& x : hb) x = f2bf((rand() % 2001 - 1000) / 5000.0f);
  uint16_t *dA, *dW, *db; void *dO, *dsk;
  const size_t skb = (size_t)16 * 512 * F * 4;
  CK(hipMalloc(&dA, hA.size() * 2)); CK(hipMalloc(&dW, wmax * 2 * R)); CK(hipMalloc(&db, hb.size() * 2));
  CK(hipMalloc(&dO, (size_t)M * std::max(F, V) * 4)); CK(hipMalloc(&dsk, skb));
  CK(hipMemcpy(dA, hA.data(), hA.size() * 2, hipMemcpyHostToDevice));
  for (int r = 0; r < R; ++r) CK(hipMemcpy(dW + (size_t)r * wmax, hW.data(), wmax * 2, hipMemcpyHostToDevice));
  CK(hipMemcpy(db, hb.data(), hb.size() * 2, hipMemcpyHostToDevice));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  int bad = 0;
  for (auto& s : shapes) {
    GemmArgs g;
    g.A = dA; g.W = dW; g.bias = s.epi == EPI_F32 ? nullptr : db; g.out = dO;
    g.M_max = M; g.M_dev = nullptr; g.N = s.N; g.K = s.K; g.ldo = s.N; g.epilogue = s.epi;
    g.splitk_ws = dsk; g.splitk_ws_bytes = skb; g.max_split = max_split;
    g.lda = s.K + pad_a; g.ldw = s.K + pad_w;
    const int ks = gemm_splitk_factor(1, g);
    const bool f32out = s.epi == EPI_BIAS_RESADD || s.epi == EPI_F32;
    // the residual epilogue adds into the output: start from a known value
    std::vector<float> init((size_t)M * s.N, 0.25f);
    if (f32out) CK(hipMemcpy(dO, init.data(), init.size() * 4, hipMemcpyHostToDevice));
    CK(launch_gemm(1, g, 0)); CK(hipDeviceSynchronize());
    std::vector<uint16_t> ho16; std::vector<float> ho32;
    if (f32out) { ho32.resize((size_t)M * s.N); CK(hipMemcpy(ho32.data(), dO, ho32.size() * 4, hipMemcpyDeviceToHost)); }
    else { ho16.resize((size_t)M * s.N); CK(hipMemcpy(ho16.data(), dO, ho16.size() * 2, hipMemcpyDeviceToHost)); }
    double maxerr = 0;
    for (int t = 0; t < 600; ++t) {
      const int r = t < 8 ? (t % 2 ? M - 1 : 0) : rand() % M, c = t < 8 ? (t % 4 < 2 ? 0 : s.N - 1) : rand() % s.N;
      double acc = 0;
      for (int k = 0; k < s.K; ++k) acc += (double)h2f(hA[(size_t)r * g.lda + k]) * h2f(hW[(size_t)c * g.ldw + k]);
      if (s.epi != EPI_F32) acc += bf2f(hb[c]);
      if (s.epi == EPI_BIAS_GELU) acc = 0.5 * acc * (1 + erf(acc / sqrt(2.0)));
      if (s.epi == EPI_BIAS_RESADD) acc += 0.25;
      const double got = f32out ? ho32[(size_t)r * s.N + c] : h2f(ho16[(size_t)r * s.N + c]);
      const double tol = f32out ? 4e-3 : 8e-3 * fmax(1.0, fabs(acc));
      const double err = fabs(got - acc);
      if (err > maxerr) maxerr = err;
      if (err > tol) { printf("MISMATCH %s r=%d c=%d got %f want %f\n", s.name, r, c, got, acc); ++bad; break; }
    }
    float ms_w = 0, ms_c = 0;
    if (ks > 1) g.phase = timed_phase;
    for (int mode = 0; mode < 2; ++mode) {
      for (int i = 0; i < 8; ++i) { g.W = dW + (mode ? (size_t)(i % R) * wmax : 0); CK(launch_gemm(1, g, 0)); }
      CK(hipEventRecord(e0, 0));
      for (int i = 0; i < reps; ++i) { g.W = dW + (mode ? (size_t)(i % R) * wmax : 0); CK(launch_gemm(1, g, 0)); }
      CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1));
      float ms; CK(hipEventElapsedTime(&ms, e0, e1)); (mode ? ms_c : ms_w) = ms / reps;
    }
    const double wb = 2.0 * s.N * s.K, fl = 2.0 * M * s.N * s.K;
    printf("%-7s M=%d N=%d K=%d split %d: warm %.1f us  cold %.1f us (%.2f TB/s of weights, %.0f TFLOP/s)  max |err| %.2e\n",
           s.name, M, s.N, s.K, ks, ms_w * 1e3, ms_c * 1e3, wb / ms_c / 1e9, fl / ms_c / 1e9, maxerr);
    fflush(stdout);
  }
  return bad ? 2 : 0;
}
