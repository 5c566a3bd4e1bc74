// Stand-alone driver for the decode attention kernel at the 2.8B shape (batch 256, 32 heads of 80): fills
// a K/V cache laid out as the library lays it out, runs one decode step's attention, checks sampled
// (sequence, head) outputs against a double-precision softmax on the host, times the kernel and runs a
// plain copy kernel of known size next to it; it also runs and checks the packed causal (prefill /
// scoring) attention kernel on the same cache.  Like gemm_driver it exists for hardware-counter runs
// (rocprofv3 --pmc), which work on a small native process but not on the Python benchmark.
//   usage: attn_driver [batch=256] [reps=5] [layers=1]
//   (layers > 1: the decode kernel is also timed rotating over that many layers' caches, as a decode pass does)
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

static float h2f(uint16_t u) { _Float16 h; memcpy(&h, &u, 2); return (float)h; }

// values in [-1, 1) from a hash of the element index
__global__ void __launch_bounds__(256) fill_f16_kernel(_Float16* p, size_t n, unsigned salt) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t st = (size_t)gridDim.x * 256;
  for (; i < n; i += st) {
    unsigned x = (unsigned)i * 2654435761u ^ (unsigned)(i >> 32) ^ salt;
    x ^= x >> 15; x *= 2246822519u; x ^= x >> 13;
    p[i] = (_Float16)((float)(x & 0xFFFF) / 32768.0f - 1.0f);
  }
}
typedef __attribute__((ext_vector_type(4))) unsigned u4_t;
__global__ void __launch_bounds__(256) copy_yardstick_kernel(const u4_t* __restrict__ src, u4_t* __restrict__ dst, size_t n) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t st = (size_t)gridDim.x * 256;
  for (; i < n; i += st) dst[i] = src[i];
}

int main(int argc, char** argv) {
  const int B = argc > 1 ? atoi(argv[1]) : 256;
  const int reps = argc > 2 ? atoi(argv[2]) : 5;
  const int layers = argc > 3 ? atoi(argv[3]) : 1;
  if (layers < 1 || layers > 64) { printf("layers out of range\n"); return 1; }
  const int H = 32, HD = 80, d = H * HD, N = 53, step = 26;  // mid-rollout decode step
  if (B <= 0 || B > 4096) { printf("batch out of range\n"); return 1; }
  std::vector<int> len(B), kvoff(B + 1);
  srand(7);
  long slots = 0;
  double ctx_sum = 0;
  for (int b = 0; b < B; ++b) {
    len[b] = 96 + rand() % 417;  // query lengths 96..512
    kvoff[b] = (int)slots;
    slots += len[b] + N - 1;
    ctx_sum += len[b] + step + 1;
  }
  kvoff[B] = (int)slots;
  const size_t plane = (size_t)slots * d;  // halfs in the K (or V) plane of one layer
  _Float16 *dK, *dV, *dq, *dout;
  int *dlen, *dkvoff;
  CK(hipMalloc(&dK, plane * 2)); CK(hipMalloc(&dV, plane * 2));
  CK(hipMalloc(&dq, (size_t)B * d * 2)); CK(hipMalloc(&dout, (size_t)B * d * 2));
  CK(hipMalloc(&dlen, B * 4)); CK(hipMalloc(&dkvoff, (B + 1) * 4));
  hipLaunchKernelGGL(fill_f16_kernel, dim3(4096), dim3(256), 0, 0, dK, plane, 1u);
  hipLaunchKernelGGL(fill_f16_kernel, dim3(4096), dim3(256), 0, 0, dV, plane, 2u);
  hipLaunchKernelGGL(fill_f16_kernel, dim3(256), dim3(256), 0, 0, dq, (size_t)B * d, 3u);
  CK(hipMemcpy(dlen, len.data(), B * 4, hipMemcpyHostToDevice));
  CK(hipMemcpy(dkvoff, kvoff.data(), (B + 1) * 4, hipMemcpyHostToDevice));
  CK(hipDeviceSynchronize());
  const int ctx_max = 512 + N;
  CK(launch_attn_decode(1, dq, dK, dV, N - 1, B, dlen, step + 1, ctx_max, dkvoff, H, HD, dout, 0));
  CK(hipDeviceSynchronize());
  // ---- check sampled (sequence, head) pairs
  std::vector<uint16_t> hq((size_t)B * d), ho((size_t)B * d);
  CK(hipMemcpy(hq.data(), dq, hq.size() * 2, hipMemcpyDeviceToHost));
  CK(hipMemcpy(ho.data(), dout, ho.size() * 2, hipMemcpyDeviceToHost));
  double maxerr = 0;
  int bad = 0;
  for (int t = 0; t < 24; ++t) {
    const int b = t == 0 ? 0 : (t == 1 ? B - 1 : rand() % B), h = t == 0 ? 0 : (t == 1 ? H - 1 : rand() % H);
    const int ctx = len[b] + step + 1;
    const size_t base = ((size_t)kvoff[b] * H + (size_t)h * (len[b] + N - 1)) * HD;
    std::vector<uint16_t> hk((size_t)ctx * HD), hv((size_t)ctx * HD);
    CK(hipMemcpy(hk.data(), dK + base, hk.size() * 2, hipMemcpyDeviceToHost));
    CK(hipMemcpy(hv.data(), dV + base, hv.size() * 2, hipMemcpyDeviceToHost));
    std::vector<double> sc(ctx);
    double mx = -1e300;
    for (int j = 0; j < ctx; ++j) {
      double s = 0;
      for (int e = 0; e < HD; ++e) s += (double)h2f(hq[(size_t)b * d + h * HD + e]) * h2f(hk[(size_t)j * HD + e]);
      sc[j] = s / sqrt((double)HD);
      if (sc[j] > mx) mx = sc[j];
    }
    double den = 0;
    for (int j = 0; j < ctx; ++j) { sc[j] = exp(sc[j] - mx); den += sc[j]; }
    for (int e = 0; e < HD; ++e) {
      double o = 0;
      for (int j = 0; j < ctx; ++j) o += sc[j] * h2f(hv[(size_t)j * HD + e]);
      o /= den;
      const double err = fabs(o - h2f(ho[(size_t)b * d + h * HD + e]));
      if (err > maxerr) maxerr = err;
      if (err > 2e-3) { if (!bad) printf("MISMATCH b=%d h=%d e=%d got %f want %f\n", b, h, e, h2f(ho[(size_t)b * d + h * HD + e]), o); ++bad; }
    }
  }
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  CK(hipEventRecord(e0, 0));
  for (int i = 0; i < reps; ++i) CK(launch_attn_decode(1, dq, dK, dV, N - 1, B, dlen, step + 1, ctx_max, dkvoff, H, HD, dout, 0));
  CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1));
  float ms; CK(hipEventElapsedTime(&ms, e0, e1)); ms /= reps;
  const double bytes = ctx_sum * 2.0 * d * 2.0;  // K and V rows of every sequence's context, fp16
  printf("attn_decode B=%d H=%d hd=%d mean context %.1f: %.1f us  algorithmic K/V bytes %.3f GB  %.2f TB/s  max |err| %.2e\n",
         B, H, HD, ctx_sum / B, ms * 1e3, bytes / 1e9, bytes / ms / 1e9, maxerr);
  if (layers > 1) {  // one cache per layer, visited in turn: every launch finds its K / V cold in the caches and TLBs
    _Float16* dKV;
    CK(hipMalloc(&dKV, (size_t)layers * 2 * plane * 2));
    for (int l = 0; l < layers; ++l) {
      CK(hipMemcpy(dKV + (size_t)l * 2 * plane, dK, plane * 2, hipMemcpyDeviceToDevice));
      CK(hipMemcpy(dKV + (size_t)l * 2 * plane + plane, dV, plane * 2, hipMemcpyDeviceToDevice));
    }
    CK(hipDeviceSynchronize());
    const int n = reps * layers;
    for (int i = 0; i < layers; ++i)
      CK(launch_attn_decode(1, dq, dKV + (size_t)i * 2 * plane, dKV + (size_t)i * 2 * plane + plane, N - 1, B, dlen, step + 1,
                            ctx_max, dkvoff, H, HD, dout, 0));
    CK(hipEventRecord(e0, 0));
    for (int i = 0; i < n; ++i) {
      const size_t o = (size_t)(i % layers) * 2 * plane;
      CK(launch_attn_decode(1, dq, dKV + o, dKV + o + plane, N - 1, B, dlen, step + 1, ctx_max, dkvoff, H, HD, dout, 0));
    }
    CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1));
    float msl; CK(hipEventElapsedTime(&msl, e0, e1)); msl /= n;
    printf("attn_decode rotating over %d layers' caches (%.1f GB): %.1f us  %.2f TB/s\n", layers,
           (double)layers * 2 * plane * 2 / 1e9, msl * 1e3, bytes / msl / 1e9);
    CK(hipFree(dKV));
  }
  // ---- the packed causal (prefill / scoring) kernel on the same cache: every sequence attends over
  //      all len + 52 rows of its slab, queries packed back to back as the library packs them
  {
    std::vector<int> plen(B), cu(B + 1);
    long T = 0;
    double pair_sum = 0;
    int Lmax = 0;
    for (int b = 0; b < B; ++b) {
      plen[b] = len[b] + N - 1;  // every row of the sequence's slab
      cu[b] = (int)T;
      T += plen[b];
      pair_sum += 0.5 * plen[b] * (plen[b] + 1.0);
      if (plen[b] > Lmax) Lmax = plen[b];
    }
    cu[B] = (int)T;
    _Float16 *dq2, *dout2;
    int *dplen, *dcu;
    CK(hipMalloc(&dq2, (size_t)T * d * 2)); CK(hipMalloc(&dout2, (size_t)T * d * 2));
    CK(hipMalloc(&dplen, B * 4)); CK(hipMalloc(&dcu, (B + 1) * 4));
    hipLaunchKernelGGL(fill_f16_kernel, dim3(4096), dim3(256), 0, 0, dq2, (size_t)T * d, 4u);
    CK(hipMemcpy(dplen, plen.data(), B * 4, hipMemcpyHostToDevice));
    CK(hipMemcpy(dcu, cu.data(), (B + 1) * 4, hipMemcpyHostToDevice));
    CK(launch_attn_prefill(1, dq2, dK, dV, 0, B, Lmax, dplen, dcu, dkvoff, H, HD, dout2, d, 0));
    CK(hipDeviceSynchronize());
    double perr = 0;
    for (int t = 0; t < 12; ++t) {
      const int b = t == 0 ? 0 : rand() % B, h = rand() % H;
      const int qi = t == 0 ? plen[b] - 1 : rand() % plen[b];
      const size_t base = ((size_t)kvoff[b] * H + (size_t)h * plen[b]) * HD;
      std::vector<uint16_t> hk((size_t)(qi + 1) * HD), hv((size_t)(qi + 1) * HD), hq1(HD), ho1(HD);
      CK(hipMemcpy(hk.data(), dK + base, hk.size() * 2, hipMemcpyDeviceToHost));
      CK(hipMemcpy(hv.data(), dV + base, hv.size() * 2, hipMemcpyDeviceToHost));
      CK(hipMemcpy(hq1.data(), dq2 + ((size_t)cu[b] + qi) * d + h * HD, HD * 2, hipMemcpyDeviceToHost));
      CK(hipMemcpy(ho1.data(), dout2 + ((size_t)cu[b] + qi) * d + h * HD, HD * 2, hipMemcpyDeviceToHost));
      std::vector<double> sc(qi + 1);
      double mx = -1e300, den = 0;
      for (int j = 0; j <= qi; ++j) {
        double sdot = 0;
        for (int e = 0; e < HD; ++e) sdot += (double)h2f(hq1[e]) * h2f(hk[(size_t)j * HD + e]);
        sc[j] = sdot / sqrt((double)HD);
        if (sc[j] > mx) mx = sc[j];
      }
      for (int j = 0; j <= qi; ++j) { sc[j] = exp(sc[j] - mx); den += sc[j]; }
      for (int e = 0; e < HD; ++e) {
        double o = 0;
        for (int j = 0; j <= qi; ++j) o += sc[j] * h2f(hv[(size_t)j * HD + e]);
        const double err = fabs(o / den - h2f(ho1[e]));
        if (err > perr) perr = err;
        if (err > 4e-3) { if (!bad) printf("PREFILL MISMATCH b=%d h=%d q=%d e=%d\n", b, h, qi, e); ++bad; }
      }
    }
    CK(hipEventRecord(e0, 0));
    for (int i = 0; i < reps; ++i) CK(launch_attn_prefill(1, dq2, dK, dV, 0, B, Lmax, dplen, dcu, dkvoff, H, HD, dout2, d, 0));
    CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1));
    CK(hipEventElapsedTime(&ms, e0, e1)); ms /= reps;
    const double fl = 4.0 * d * pair_sum;  // QK^T and PV over the causal (query, key) pairs
    printf("attn_prefill B=%d H=%d hd=%d tokens %ld mean length %.1f: %.1f us  %.1f TFLOP/s  max |err| %.2e\n", B, H, HD, T,
           (double)T / B, ms * 1e3, fl / ms / 1e9, perr);
  }
  {
    const size_t n = (size_t)1 << 24;  // 256 MiB read + 256 MiB written
    if (plane * 2 < n * 16) printf("copy yardstick skipped: cache plane smaller than 256 MiB\n");
    else {
      CK(hipEventRecord(e0, 0));
      for (int i = 0; i < reps; ++i) hipLaunchKernelGGL(copy_yardstick_kernel, dim3(8192), dim3(256), 0, 0, (const u4_t*)dK, (u4_t*)dV, n);
      CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1));
      CK(hipEventElapsedTime(&ms, e0, e1)); ms /= reps;
      printf("copy yardstick: 268.4 MB read + 268.4 MB written per launch, %.3f ms (%.2f TB/s)\n", ms, 2.0 * n * 16 / ms / 1e9);
    }
  }
  return bad ? 2 : 0;
}
