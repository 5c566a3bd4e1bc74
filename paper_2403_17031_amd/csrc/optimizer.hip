// AdamW step of the PPO update, fused over everything an update touches: fp32 master weights, both
// moments, and the bf16 storage copy of the weights (a bf16 model's matrices reach the forward passes through
// the fp16 image that rlhf_refresh_weights rebuilds from that copy).  Pure streaming work
// (16 bytes read, 12 to 14 written per element): 4 elements per lane, 16-byte accesses, grid sized
// for 64 blocks per CU (measured best of 8 / 16 / 64) with a grid-stride loop, so any length fits one launch.
#include "common.h"

namespace rlhf {

typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;  // NaN stays NaN
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// decay = 1 - lr * weight_decay; omb1 = 1 - beta1; omb2 = 1 - beta2; step_size = lr / (1 - beta1^t);
// inv_sqrt_bias2 = 1 / sqrt(1 - beta2^t): formed once on the host in double (1 - 0.999 in fp32 would
// already be off by 1.3e-5 relative).
__global__ void __launch_bounds__(256)
    adamw_kernel(float* __restrict__ p, const float* __restrict__ g, float* __restrict__ m, float* __restrict__ v,
                 uint16_t* __restrict__ p_bf16, size_t n, float decay, float beta1, float omb1, float beta2,
                 float omb2, float step_size, float inv_sqrt_bias2, float eps, float grad_scale) {
  const size_t n4 = n >> 2;
  const size_t stride = (size_t)gridDim.x * 256;
  auto upd = [&](float pv, float gv, float& mv, float& vv) {
    gv *= grad_scale;
    pv *= decay;
    mv = beta1 * mv + omb1 * gv;
    vv = beta2 * vv + omb2 * gv * gv;
    const float denom = sqrtf(vv) * inv_sqrt_bias2 + eps;
    return pv - step_size * (mv / denom);
  };
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
    f32x4_t pv = ((const f32x4_t*)p)[i];
    const f32x4_t gv = ((const f32x4_t*)g)[i];
    f32x4_t mv = ((const f32x4_t*)m)[i], vv = ((const f32x4_t*)v)[i];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float m1 = mv[u], v1 = vv[u];
      pv[u] = upd(pv[u], gv[u], m1, v1);
      mv[u] = m1;
      vv[u] = v1;
    }
    ((f32x4_t*)p)[i] = pv;
    ((f32x4_t*)m)[i] = mv;
    ((f32x4_t*)v)[i] = vv;
    if (p_bf16) {
      u32x2_t o;
      o[0] = f32_to_bf16_rne(pv[0]) | (f32_to_bf16_rne(pv[1]) << 16);
      o[1] = f32_to_bf16_rne(pv[2]) | (f32_to_bf16_rne(pv[3]) << 16);
      ((u32x2_t*)p_bf16)[i] = o;
    }
  }
  // ragged tail (n not a multiple of 4): one element per thread of block 0
  if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
    const size_t i = (n4 << 2) + threadIdx.x;
    float mv = m[i], vv = v[i];
    const float pv = upd(p[i], g[i], mv, vv);
    p[i] = pv;
    m[i] = mv;
    v[i] = vv;
    if (p_bf16) p_bf16[i] = (uint16_t)f32_to_bf16_rne(pv);
  }
}

hipError_t launch_adamw(float* p, const float* g, float* m, float* v, uint16_t* p_bf16, size_t n, float decay,
                        float beta1, float omb1, float beta2, float omb2, float step_size, float inv_sqrt_bias2,
                        float eps, float grad_scale, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const size_t want = ((n >> 2) + 255) / 256;
  const unsigned blocks = (unsigned)std::min<size_t>(std::max<size_t>(want, 1), 256 * 64);
  hipLaunchKernelGGL(adamw_kernel, dim3(blocks), dim3(256), 0, s, p, g, m, v, p_bf16, n, decay, beta1, omb1, beta2, omb2,
                     step_size, inv_sqrt_bias2, eps, grad_scale);
  return hipGetLastError();
}

}  // namespace rlhf
