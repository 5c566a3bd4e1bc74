// Stand-alone driver for the library's GEMM path at the per-layer shapes of a model: runs QKV (with the
// epilogue the library runs it with: bias, rotary turn, q rows and K/V cache slots stored; sequences of 352
// rows each), FC1 and the fused out-projection + FC2 product on seeded random operands, checks sampled outputs against a
// double-precision dot product on the host, times them with HIP events, and runs a plain copy kernel of
// known size next to them.  It exists because hardware counters (rocprofv3 --pmc) can be collected on a
// small native process where they cannot on the Python benchmark; the copy kernel is the yardstick the
// FETCH_SIZE / WRITE_SIZE readings are scaled by.
//   usage: gemm_driver [M=83373] [reps=3] [d_model=2560]
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

// yardstick: reads `n` 16-byte words and writes them elsewhere
typedef __attribute__((ext_vector_type(4))) unsigned u4_t;
__global__ void __launch_bounds__(256) copy_yardstick_kernel(const u4_t* __restrict__ src, u4_t* __restrict__ dst, size_t n) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t st = (size_t)gridDim.x * 256;
  for (; i < n; i += st) dst[i] = src[i];
}

int main(int argc, char** argv) {
  const int M = argc > 1 ? atoi(argv[1]) : 83373;
  const int reps = argc > 2 ? atoi(argv[2]) : 3;
  const int d = argc > 3 ? atoi(argv[3]) : 2560, F = 4 * d;
  if (M <= 512 || d % 128 != 0) { printf("M must exceed 512 and d_model be a multiple of 128\n"); return 1; }
  struct Shape { const char* name; int N, K, epi; bool bias2; } shapes[] = {
      {"qkv", 3 * d, d, EPI_QKV, false}, {"fc1", F, d, EPI_BIAS_GELU, false}, {"out+fc2", d, d + F, EPI_BIAS_RESADD, true}};
  const size_t maxA = (size_t)M * (d + F), maxW = (size_t)F * d * 3, maxO = (size_t)M * F;
  std::vector<uint16_t> hA(maxA), hW(maxW), hb(F), hb2(F);
  srand(1);
  for (auto& x : hA) x = f2h((rand() % 2001 - 1000) / 1000.0f);
  for (auto& x : hW) x = f2h((rand() % 2001 - 1000) / 25000.0f);
  for (auto& x : hb) x = f2bf((rand() % 2001 - 1000) / 5000.0f);
  for (auto& x : hb2) x = f2bf((rand() % 2001 - 1000) / 5000.0f);
  uint16_t *dA, *dW, *db, *db2; void* dO; int* dM;
  CK(hipMalloc(&dA, maxA * 2)); CK(hipMalloc(&dW, maxW * 2)); CK(hipMalloc(&db, F * 2)); CK(hipMalloc(&db2, F * 2));
  CK(hipMalloc(&dO, maxO * 4)); CK(hipMalloc(&dM, 4));
  CK(hipMemcpy(dA, hA.data(), maxA * 2, hipMemcpyHostToDevice)); CK(hipMemcpy(dW, hW.data(), maxW * 2, hipMemcpyHostToDevice));
  CK(hipMemcpy(db, hb.data(), F * 2, hipMemcpyHostToDevice)); CK(hipMemcpy(db2, hb2.data(), F * 2, hipMemcpyHostToDevice));
  CK(hipMemcpy(dM, &M, 4, hipMemcpyHostToDevice));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  // packing for the QKV epilogue: sequences of Ls rows (the last one shorter), heads of 80 (2.8B shape) or 64
  const int hd = d % 80 == 0 ? 80 : 64, H = d / hd, r = hd / 4, Ls = 352, nseq = (M + Ls - 1) / Ls, maxpos = 512;
  std::vector<int> hpos(M + 1000, 0), hrow(M + 1000, 0), hkv(nseq + 1), hlen(nseq);
  for (int t = 0; t < M; ++t) { hpos[t] = t % Ls; hrow[t] = t / Ls; }
  for (int b = 0; b <= nseq; ++b) hkv[b] = std::min(b * Ls, M);
  for (int b = 0; b < nseq; ++b) hlen[b] = hkv[b + 1] - hkv[b];
  std::vector<float> hcs((size_t)maxpos * (r / 2)), hsn((size_t)maxpos * (r / 2));
  for (int p = 0; p < maxpos; ++p)
    for (int i = 0; i < r / 2; ++i) { const double a = p * pow(10000.0, -2.0 * i / r); hcs[(size_t)p * (r / 2) + i] = (float)cos(a); hsn[(size_t)p * (r / 2) + i] = (float)sin(a); }
  int *dpos, *drow, *dkv, *dlen; float *dcs, *dsn; uint16_t *dq, *dkc, *dvc;
  CK(hipMalloc(&dpos, hpos.size() * 4)); CK(hipMalloc(&drow, hrow.size() * 4)); CK(hipMalloc(&dkv, hkv.size() * 4)); CK(hipMalloc(&dlen, hlen.size() * 4));
  CK(hipMalloc(&dcs, hcs.size() * 4)); CK(hipMalloc(&dsn, hsn.size() * 4));
  CK(hipMalloc(&dq, (size_t)(M + 1000) * d * 2)); CK(hipMalloc(&dkc, (size_t)(M + 1000) * d * 2)); CK(hipMalloc(&dvc, (size_t)(M + 1000) * d * 2));
  CK(hipMemcpy(dpos, hpos.data(), hpos.size() * 4, hipMemcpyHostToDevice)); CK(hipMemcpy(drow, hrow.data(), hrow.size() * 4, hipMemcpyHostToDevice));
  CK(hipMemcpy(dkv, hkv.data(), hkv.size() * 4, hipMemcpyHostToDevice)); CK(hipMemcpy(dlen, hlen.data(), hlen.size() * 4, hipMemcpyHostToDevice));
  CK(hipMemcpy(dcs, hcs.data(), hcs.size() * 4, hipMemcpyHostToDevice)); CK(hipMemcpy(dsn, hsn.data(), hsn.size() * 4, hipMemcpyHostToDevice));
  QkvArgs qa;
  qa.pos = dpos; qa.rowid = drow; qa.kvoff = dkv; qa.len = dlen; qa.cos_t = dcs; qa.sin_t = dsn; qa.q = dq; qa.kc = dkc; qa.vc = dvc;
  qa.kv_extra = 0; qa.pos_add = 0; qa.H = H; qa.hd = hd; qa.r = r;
  int bad = 0;
  for (auto& s : shapes) {
    GemmArgs g;
    g.A = dA; g.W = dW; g.bias = db; g.bias2 = s.bias2 ? db2 : nullptr; g.out = dO;
    g.M_max = M + 1000; g.M_dev = dM; g.N = s.N; g.K = s.K; g.ldo = s.N; g.epilogue = s.epi;
    if (s.epi == EPI_QKV) {
      g.qkv = &qa;
      if (!gemm_takes_qkv(1, g, H, hd, r)) { printf("the QKV epilogue does not take this shape\n"); return 1; }
    }
    CK(hipMemset(dO, 0, maxO * 4));
    CK(launch_gemm(1, g, 0)); CK(hipDeviceSynchronize());
    const bool f32out = s.epi == EPI_BIAS_RESADD;
    std::vector<uint16_t> ho16; std::vector<float> ho32;
    if (s.epi == EPI_QKV) {
      // checked on the V section (no rotary turn): value (t, head h, e) sits at cache row kvoff[b]*H + h*len[b] + pos
      std::vector<uint16_t> hv((size_t)M * d);
      CK(hipMemcpy(hv.data(), dvc, hv.size() * 2, hipMemcpyDeviceToHost));
      double maxerr = 0;
      for (int t = 0; t < 400 && !bad; ++t) {
        const int row = t < 4 ? (t % 2 ? M - 1 : 0) : rand() % M, c = 2 * d + (t < 4 ? (t < 2 ? 0 : d - 1) : rand() % d);
        double acc = 0;
        for (int k = 0; k < s.K; ++k) acc += (double)h2f(hA[(size_t)row * s.K + k]) * h2f(hW[(size_t)c * s.K + k]);
        acc += bf2f(hb[c]);
        const int b = hrow[row], hh = (c - 2 * d) / hd, e = (c - 2 * d) % hd;
        const size_t slot = (size_t)hkv[b] * H + (size_t)hh * hlen[b] + hpos[row];
        const double got = h2f(hv[slot * hd + e]), err = fabs(got - acc);
        if (err > maxerr) maxerr = err;
        if (err > 8e-3 * fmax(1.0, fabs(acc))) { printf("MISMATCH %s r=%d c=%d got %f want %f\n", s.name, row, c, got, acc); ++bad; }
      }
      CK(hipEventRecord(e0, 0));
      for (int i = 0; i < reps; ++i) CK(launch_gemm(1, g, 0));
      CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1));
      float ms; CK(hipEventElapsedTime(&ms, e0, e1)); ms /= reps;
      printf("%-8s M=%d N=%d K=%d: %.3f ms  %.1f TFLOP/s  algorithmic HBM bytes %.3f GB  max |err| %.2e\n", s.name, M, s.N,
             s.K, ms, 2.0 * M * s.N * s.K / ms / 1e9, (2.0 * ((double)M * s.K + (double)s.N * s.K) + 2.0 * M * s.N) / 1e9, maxerr);
      continue;
    }
    if (f32out) { ho32.resize((size_t)M * s.N); CK(hipMemcpy(ho32.data(), dO, ho32.size() * 4, hipMemcpyDeviceToHost)); }
    else { ho16.resize((size_t)M * s.N); CK(hipMemcpy(ho16.data(), dO, ho16.size() * 2, hipMemcpyDeviceToHost)); }
    double maxerr = 0;
    for (int t = 0; t < 400; ++t) {
      const int r = t < 8 ? (t % 2 ? M - 1 : 0) : rand() % M, c = t < 8 ? (t % 4 < 2 ? 0 : s.N - 1) : rand() % s.N;
      double acc = 0;
      for (int k = 0; k < s.K; ++k) acc += (double)h2f(hA[(size_t)r * s.K + k]) * h2f(hW[(size_t)c * s.K + k]);
      acc += bf2f(hb[c]) + (s.bias2 ? bf2f(hb2[c]) : 0.f);
      if (s.epi == EPI_BIAS_GELU) acc = 0.5 * acc * (1 + erf(acc / sqrt(2.0)));
      const double got = f32out ? ho32[(size_t)r * s.N + c] : h2f(ho16[(size_t)r * s.N + c]);
      const double tol = f32out ? 4e-3 : 8e-3 * fmax(1.0, fabs(acc));
      const double err = fabs(got - acc);
      if (err > maxerr) maxerr = err;
      if (err > tol) { printf("MISMATCH %s r=%d c=%d got %f want %f\n", s.name, r, c, got, acc); ++bad; break; }
    }
    CK(hipEventRecord(e0, 0));
    for (int i = 0; i < reps; ++i) CK(launch_gemm(1, g, 0));
    CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1));
    float ms; CK(hipEventElapsedTime(&ms, e0, e1)); ms /= reps;
    const double fl = 2.0 * M * s.N * s.K;
    const double bytes = 2.0 * ((double)M * s.K + (double)s.N * s.K) + (f32out ? 8.0 : 2.0) * M * s.N;
    printf("%-8s M=%d N=%d K=%d: %.3f ms  %.1f TFLOP/s  algorithmic HBM bytes %.3f GB  max |err| %.2e\n", s.name, M, s.N,
           s.K, ms, fl / ms / 1e9, bytes / 1e9, maxerr);
  }
  {
    // the weight-gradient form: out [d, F] = A^T W with both operands K-major ([K, d] and [K, F] row-major, K = the
    // rows rounded down to 128), K cut into slices whose fp32 slabs are summed -- as the backward pass runs dW_fc2
    const int Kk = (M / 128) * 128;
    const uint16_t *hAt = hA.data(), *hWt = hA.data() + (size_t)Kk * d;  // the same host data, read as [Kk, d] | [Kk, F]
    void* dslab;
    const size_t slab_bytes = (size_t)8 * d * F * 4;
    CK(hipMalloc(&dslab, slab_bytes));
    GemmArgs g;
    g.A = dA; g.W = dA + (size_t)Kk * d; g.bias = nullptr; g.out = dO;
    g.M_max = d; g.M_dev = nullptr; g.N = F; g.K = Kk; g.ldo = F; g.epilogue = EPI_F32;
    g.k_major = true; g.long_k = true; g.splitk_ws = dslab; g.splitk_ws_bytes = slab_bytes;
    if (!gemm_takes_k_major(1, g)) { printf("the K-major form does not take this shape\n"); return 1; }
    CK(launch_gemm(1, g, 0)); CK(hipDeviceSynchronize());
    std::vector<float> ho((size_t)d * F);
    CK(hipMemcpy(ho.data(), dO, ho.size() * 4, hipMemcpyDeviceToHost));
    double maxerr = 0, maxabs = 0;
    for (int t = 0; t < 200; ++t) {
      const int m = t < 4 ? (t % 2 ? d - 1 : 0) : rand() % d, n = t < 4 ? (t < 2 ? 0 : F - 1) : rand() % F;
      double acc = 0;
      for (int k = 0; k < Kk; ++k) acc += (double)h2f(hAt[(size_t)k * d + m]) * h2f(hWt[(size_t)k * F + n]);
      const double err = fabs(ho[(size_t)m * F + n] - acc);
      if (err > maxerr) maxerr = err;
      if (fabs(acc) > maxabs) maxabs = fabs(acc);
      if (err > 2e-3 * fmax(1.0, fabs(acc)) + 2e-2) { printf("MISMATCH k-major m=%d n=%d got %f want %f\n", m, n, ho[(size_t)m * F + n], acc); ++bad; break; }
    }
    CK(hipEventRecord(e0, 0));
    for (int i = 0; i < reps; ++i) CK(launch_gemm(1, g, 0));
    CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1));
    float ms; CK(hipEventElapsedTime(&ms, e0, e1)); ms /= reps;
    printf("dW k-major M=%d N=%d K=%d: %.3f ms  %.1f TFLOP/s  max |err| %.2e (largest |value| %.1f)\n", d, F, Kk, ms,
           2.0 * d * F * (double)Kk / ms / 1e9, maxerr, maxabs);
    CK(hipFree(dslab));
  }
  {
    const size_t n = (size_t)1 << 26;  // 1 GiB read + 1 GiB written
    u4_t *src = (u4_t*)dA, *dst = (u4_t*)dO;
    if (maxA * 2 < n * 16 || maxO * 4 < n * 16) { printf("copy yardstick skipped: buffers smaller than 1 GiB\n"); }
    else {
      CK(hipEventRecord(e0, 0));
      for (int i = 0; i < reps; ++i) hipLaunchKernelGGL(copy_yardstick_kernel, dim3(8192), dim3(256), 0, 0, src, dst, n);
      CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1));
      float ms; CK(hipEventElapsedTime(&ms, e0, e1)); ms /= reps;
      printf("copy yardstick: 1.074 GB read + 1.074 GB written per launch, %.3f ms (%.2f TB/s)\n", ms, 2.0 * n * 16 / ms / 1e9);
    }
  }
  return bad ? 2 : 0;
}
