// Measured ceilings of the GPU this process runs on, next to which the library's kernels are reported:
//   * streaming read: 2 GiB read once per launch, one 256-thread block per ~100 KB run, four 16-byte loads in
//     flight per lane (the access pattern of the decode attention kernel's K/V streams);
//   * matrix cores: a loop of v_mfma_f32_32x32x16_f16 on 16 independent accumulators per wave, four waves on each
//     of 256 CUs, nothing else in the loop -- once on all-zero operands (the chip holds its clock) and once on
//     random fp16 operands (it does not: under matrix-core load with real data the clock drops, and that rate,
//     not the data-sheet peak, is what a product on real data can at best sustain).
// Prints one JSON object on stdout.   usage: ceilings_driver [mfma_iters=300000]
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <vector>

typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

#define CK(x)                                                                       \
  do {                                                                              \
    hipError_t e_ = (x);                                                            \
    if (e_ != hipSuccess) {                                                         \
      fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
      return 1;                                                                     \
    }                                                                               \
  } while (0)

__global__ void __launch_bounds__(256) stream_read_kernel(const u32x4_t* __restrict__ p, size_t run16, unsigned* out) {
  const u32x4_t* r = p + (size_t)blockIdx.x * run16;
  u32x4_t a = {0, 0, 0, 0};
  size_t i = threadIdx.x;
  for (; i + 768 < run16; i += 1024) {
    const u32x4_t v0 = r[i], v1 = r[i + 256], v2 = r[i + 512], v3 = r[i + 768];
    a ^= v0 ^ v1 ^ v2 ^ v3;
  }
  for (; i < run16; i += 256) a ^= r[i];
  if (a[0] == 0x12345 && a[1] == 77) out[0] = a[2];  // never true for the fill pattern: keeps the loads alive
}

__global__ void __launch_bounds__(256) mfma_loop_kernel(const f16x8_t* __restrict__ in, float* out, int iters) {
  f16x8_t a[4], b[4];
  for (int i = 0; i < 4; ++i) {
    a[i] = in[(threadIdx.x * 8 + i) & 4095];
    b[i] = in[(threadIdx.x * 8 + 4 + i) & 4095];
  }
  f32x16_t acc[16];
  for (int j = 0; j < 16; ++j)
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[j * 4 + i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(b[j], a[i], acc[j * 4 + i], 0, 0, 0);
  }
  float s = 0;
  for (int j = 0; j < 16; ++j)
    for (int e = 0; e < 16; ++e) s += acc[j][e];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

int main(int argc, char** argv) {
  const int iters = argc > 1 ? atoi(argv[1]) : 300000;
  if (iters <= 0 || iters > 4000000) { fprintf(stderr, "mfma_iters must be 1..4000000\n"); return 1; }
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  float ms;
  // ---- streaming read
  const size_t bytes = (size_t)2 << 30, n16 = bytes / 16, run16 = 100 * 1024 / 16;
  const int nb = (int)(n16 / run16);
  u32x4_t* d;
  unsigned* o;
  CK(hipMalloc(&d, bytes));
  CK(hipMalloc(&o, 64));
  CK(hipMemset(d, 1, bytes));
  hipLaunchKernelGGL(stream_read_kernel, dim3(nb), dim3(256), 0, 0, d, run16, o);
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0));
  for (int r = 0; r < 10; ++r) hipLaunchKernelGGL(stream_read_kernel, dim3(nb), dim3(256), 0, 0, d, run16, o);
  CK(hipEventRecord(e1));
  CK(hipEventSynchronize(e1));
  CK(hipEventElapsedTime(&ms, e0, e1));
  const double stream_gbps = 10.0 * nb * run16 * 16 / ms / 1e6;
  CK(hipFree(d));
  // ---- matrix-core loop, zero and random operands
  double tf[2];
  for (int mode = 0; mode < 2; ++mode) {
    std::vector<_Float16> h(4096 * 8);
    srand(3);
    for (auto& x : h) x = mode ? (_Float16)((rand() % 2001 - 1000) / 1000.0f) : (_Float16)0.0f;
    f16x8_t* din;
    float* dout;
    CK(hipMalloc(&din, h.size() * 2));
    CK(hipMalloc(&dout, 256 * 256 * 4));
    CK(hipMemcpy(din, h.data(), h.size() * 2, hipMemcpyHostToDevice));
    hipLaunchKernelGGL(mfma_loop_kernel, dim3(256), dim3(256), 0, 0, din, dout, iters / 10 + 1);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL(mfma_loop_kernel, dim3(256), dim3(256), 0, 0, din, dout, iters);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    CK(hipEventElapsedTime(&ms, e0, e1));
    tf[mode] = 256.0 * 4 * iters * 16 * 32768.0 / ms / 1e9;  // blocks x waves x iterations x 16 instructions x flop each
    CK(hipFree(din));
    CK(hipFree(dout));
  }
  printf("{\"stream_read_GBps\": %.1f, \"mfma_f16_zero_TFLOPs\": %.1f, \"mfma_f16_random_TFLOPs\": %.1f, "
         "\"stream_read_bytes\": %zu, \"mfma_iters\": %d}\n",
         stream_gbps, tf[0], tf[1], (size_t)nb * run16 * 16, iters);
  return 0;
}
