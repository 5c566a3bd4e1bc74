// Causal self-attention over packed variable-length sequences (prefill / scoring) and single-query
// attention against the KV cache (decode).  K and V live in a [head][slot][head_dim] layout, a
// sequence's keys occupying consecutive slots, so one (sequence, head) pair reads one contiguous
// run of memory.
#include "common.h"

namespace rlhf {

// =================================================================================================
// Generic tile kernel (any storage type, any head_dim <= 256): 32 queries x 32 keys per step,
// fp32 throughout, online softmax.  Used for fp32 check mode and as the fallback.
// =================================================================================================
template <typename T>
__global__ void __launch_bounds__(256)
    attn_prefill_generic(const T* __restrict__ q, const T* __restrict__ kc, const T* __restrict__ vc,
                         long kv_head_stride, const int* __restrict__ len, const int* __restrict__ cu,
                         const int* __restrict__ kvoff, int H, int hd, float scale, T* __restrict__ out) {
  extern __shared__ float smem[];
  const int b = blockIdx.z, h = blockIdx.y, q0 = blockIdx.x * 32;
  const int n = len[b];
  if (q0 >= n) return;
  float* Qs = smem;                 // [32][hd]
  float* Ks = Qs + 32 * hd;         // [32][hd+1]
  float* Vs = Ks + 32 * (hd + 1);   // [32][hd]
  float* Ss = Vs + 32 * hd;         // [32][33]
  float* row_m = Ss + 32 * 33;      // [32]
  float* row_l = row_m + 32;        // [32]
  float* row_a = row_l + 32;        // [32]
  const int tid = threadIdx.x;
  const int d = H * hd;
  const T* qb = q + ((size_t)cu[b]) * d + (size_t)h * hd;
  const T* kb = kc + (size_t)h * kv_head_stride + (size_t)kvoff[b] * hd;
  const T* vb = vc + (size_t)h * kv_head_stride + (size_t)kvoff[b] * hd;
  for (int c = tid; c < 32 * hd; c += 256) {
    const int r = c / hd, e = c - r * hd;
    const int qi = min(q0 + r, n - 1);
    Qs[c] = to_f32(qb[(size_t)qi * d + e]) * scale;
  }
  if (tid < 32) {
    row_m[tid] = -INFINITY;
    row_l[tid] = 0.f;
  }
  const int qi = tid >> 3, sub = tid & 7;
  float acc[32];
#pragma unroll
  for (int k = 0; k < 32; ++k) acc[k] = 0.f;
  const int q_last = min(q0 + 31, n - 1);
  for (int k0 = 0; k0 <= q_last; k0 += 32) {
    __syncthreads();
    for (int c = tid; c < 32 * hd; c += 256) {
      const int r = c / hd, e = c - r * hd;
      const int kj = min(k0 + r, n - 1);
      Ks[r * (hd + 1) + e] = to_f32(kb[(size_t)kj * hd + e]);
      Vs[c] = to_f32(vb[(size_t)kj * hd + e]);
    }
    __syncthreads();
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const int j = sub * 4 + jj;
      float s = 0.f;
      for (int e = 0; e < hd; ++e) s = fmaf(Qs[qi * hd + e], Ks[j * (hd + 1) + e], s);
      const bool ok = (k0 + j <= q0 + qi) && (k0 + j < n);
      Ss[qi * 33 + j] = ok ? s : -INFINITY;
    }
    __syncthreads();
    if (tid < 32) {
      float m = row_m[tid];
      float mx = m;
      for (int j = 0; j < 32; ++j) mx = fmaxf(mx, Ss[tid * 33 + j]);
      const float alpha = (m == -INFINITY) ? 0.f : expf(m - mx);
      float l = row_l[tid] * alpha;
      for (int j = 0; j < 32; ++j) {
        const float p = expf(Ss[tid * 33 + j] - mx);
        Ss[tid * 33 + j] = p;
        l += p;
      }
      row_m[tid] = mx;
      row_l[tid] = l;
      row_a[tid] = alpha;
    }
    __syncthreads();
    const float alpha = row_a[qi];
#pragma unroll
    for (int k = 0; k < 32; ++k) {
      const int e = sub + 8 * k;
      if (e < hd) {
        float o = acc[k] * alpha;
        for (int j = 0; j < 32; ++j) o = fmaf(Ss[qi * 33 + j], Vs[j * hd + e], o);
        acc[k] = o;
      }
    }
  }
  if (q0 + qi < n) {
    const float inv = 1.0f / row_l[qi];
    T* ob = out + ((size_t)cu[b] + q0 + qi) * d + (size_t)h * hd;
#pragma unroll
    for (int k = 0; k < 32; ++k) {
      const int e = sub + 8 * k;
      if (e < hd) ob[e] = from_f32<T>(acc[k] * inv);
    }
  }
}

hipError_t launch_attn_prefill(int dtype, const void* q, const void* kc, const void* vc, long kv_head_stride,
                               int B, int Lmax, const int* len, const int* cu, const int* kvoff, int H, int hd,
                               void* out, hipStream_t s) {
  if (hd > 256) return hipErrorInvalidValue;
  const size_t sh = sizeof(float) * (32 * hd + 32 * (hd + 1) + 32 * hd + 32 * 33 + 96);
  const float scale = 1.0f / sqrtf((float)hd);
  dim3 grid((Lmax + 31) / 32, H, B);
  if (dtype == 0) {
    if (sh > 65536)
      (void)hipFuncSetAttribute((const void*)attn_prefill_generic<float>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)sh);
    hipLaunchKernelGGL(attn_prefill_generic<float>, grid, dim3(256), sh, s, (const float*)q, (const float*)kc,
                       (const float*)vc, kv_head_stride, len, cu, kvoff, H, hd, scale, (float*)out);
  } else {
    if (sh > 65536)
      (void)hipFuncSetAttribute((const void*)attn_prefill_generic<half_t>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)sh);
    hipLaunchKernelGGL(attn_prefill_generic<half_t>, grid, dim3(256), sh, s, (const half_t*)q, (const half_t*)kc,
                       (const half_t*)vc, kv_head_stride, len, cu, kvoff, H, hd, scale, (half_t*)out);
  }
  return hipGetLastError();
}

// =================================================================================================
// Decode attention: one block per (head, sequence).
// =================================================================================================
template <typename T>
__global__ void __launch_bounds__(256)
    attn_decode_generic(const T* __restrict__ q, const T* __restrict__ kc, const T* __restrict__ vc,
                        long kv_head_stride, const int* __restrict__ len, int ctx_add,
                        const int* __restrict__ kvoff, int H, int hd, float scale, T* __restrict__ out) {
  extern __shared__ float smem[];
  __shared__ float red[8];
  const int h = blockIdx.x, b = blockIdx.y;
  const int ctx = len[b] + ctx_add;
  const int tid = threadIdx.x;
  float* qs = smem;        // [hd]
  float* part = qs + hd;   // [256]  (G x hd partial outputs, G*hd <= 256)
  float* sc = part + 256;  // [ctx]
  const int d = H * hd;
  const T* kb = kc + (size_t)h * kv_head_stride + (size_t)kvoff[b] * hd;
  const T* vb = vc + (size_t)h * kv_head_stride + (size_t)kvoff[b] * hd;
  for (int e = tid; e < hd; e += 256) qs[e] = to_f32(q[(size_t)b * d + (size_t)h * hd + e]) * scale;
  __syncthreads();
  float mx = -INFINITY;
  for (int j = tid; j < ctx; j += 256) {
    const T* kr = kb + (size_t)j * hd;
    float s = 0.f;
    for (int e = 0; e < hd; ++e) s = fmaf(qs[e], to_f32(kr[e]), s);
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  if ((tid & 63) == 0) red[tid >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  float sum = 0.f;
  for (int j = tid; j < ctx; j += 256) {
    const float p = expf(sc[j] - mx);
    sc[j] = p;
    sum += p;
  }
  sum = wave_sum(sum);
  if ((tid & 63) == 0) red[4 + (tid >> 6)] = sum;
  __syncthreads();
  sum = red[4] + red[5] + red[6] + red[7];
  const int G = 256 / hd;
  const int g = tid / hd, e = tid - g * hd;
  if (g < G) {
    float o = 0.f;
    for (int j = g; j < ctx; j += G) o = fmaf(sc[j], to_f32(vb[(size_t)j * hd + e]), o);
    part[g * hd + e] = o;
  }
  __syncthreads();
  if (tid < hd) {
    float o = 0.f;
    for (int gg = 0; gg < G; ++gg) o += part[gg * hd + tid];
    out[(size_t)b * d + (size_t)h * hd + tid] = from_f32<T>(o / sum);
  }
}

hipError_t launch_attn_decode(int dtype, const void* q, const void* kc, const void* vc, long kv_head_stride,
                              int B, const int* len, int ctx_add, int ctx_max, const int* kvoff, int H, int hd,
                              void* out, hipStream_t s) {
  if (hd > 256) return hipErrorInvalidValue;
  const size_t sh = sizeof(float) * (hd + 256 + ctx_max);
  if (sh > 65536) return hipErrorInvalidValue;
  const float scale = 1.0f / sqrtf((float)hd);
  dim3 grid(H, B);
  if (dtype == 0)
    hipLaunchKernelGGL(attn_decode_generic<float>, grid, dim3(256), sh, s, (const float*)q, (const float*)kc,
                       (const float*)vc, kv_head_stride, len, ctx_add, kvoff, H, hd, scale, (float*)out);
  else
    hipLaunchKernelGGL(attn_decode_generic<half_t>, grid, dim3(256), sh, s, (const half_t*)q, (const half_t*)kc,
                       (const half_t*)vc, kv_head_stride, len, ctx_add, kvoff, H, hd, scale, (half_t*)out);
  return hipGetLastError();
}

}  // namespace rlhf
