// Backward pass through packed causal softmax attention: dQ, dK, dV from Q, K, V and dO.
// First form: one wave per (row, head), no matrix cores, every sum in a fixed order (no atomics).
//   attn_bwd_q_kernel : for query row i -- scores against keys j <= i, their log-sum-exp, P_ij,
//                       dP_ij = dO_i . V_j, delta_i = sum_j P_ij dP_ij, dS_ij = P_ij (dP_ij - delta_i),
//                       dQ_i = scale * sum_j dS_ij K_j; keeps lse_i and delta_i for the second kernel.
//   attn_bwd_kv_kernel: for key row j -- the same P_ij and dS_ij for the queries i >= j of its
//                       sequence (from lse_i, delta_i), dV_j = sum_i P_ij dO_i, dK_j = scale * sum_i dS_ij Q_i.
// Dot products run with lanes over partner rows (each lane reads one partner row, 16 bytes at a
// time, against this row's vector broadcast from LDS); the weighted row sums run with lanes over
// the head's dims (partner rows read coalesced, one after the other).
#include <algorithm>

#include "common.h"

namespace rlhf {

namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;

__device__ __forceinline__ float dot_row(const float* __restrict__ a, const float* __restrict__ row, int hd) {
  float s = 0.f;
  for (int c = 0; c < hd; c += 4) {
    const f32x4_t v = *(const f32x4_t*)(row + c);
#pragma unroll
    for (int e = 0; e < 4; ++e) s = fmaf(a[c + e], v[e], s);
  }
  return s;
}
__device__ __forceinline__ float dot_row(const float* __restrict__ a, const half_t* __restrict__ row, int hd) {
  float s = 0.f;
  for (int c = 0; c < hd; c += 8) {
    const f16x8_t v = *(const f16x8_t*)(row + c);
#pragma unroll
    for (int e = 0; e < 8; ++e) s = fmaf(a[c + e], (float)v[e], s);
  }
  return s;
}

template <typename T>
struct __attribute__((aligned(2 * sizeof(T)))) pair2 {  // two neighbouring elements, moved as one word
  T a, b;
};

// sequence of packed row t: the largest b with cu[b] <= t (cu has B + 1 entries, cu[0] = 0)
__device__ __forceinline__ int find_seq(const int* __restrict__ cu, int B, int t) {
  int lo = 0, hi = B;  // invariant: cu[lo] <= t, and t < cu[hi] or hi == B
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu[mid] <= t) lo = mid; else hi = mid;
  }
  return lo;
}

template <typename T>
__global__ void __launch_bounds__(256)
    attn_bwd_q_kernel(const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v,
                      const T* __restrict__ g, const int* __restrict__ cu, int B, int Tn, int H, int hd, float scale,
                      int max_len, float* __restrict__ lse, float* __restrict__ delta, T* __restrict__ dq) {
  extern __shared__ float sm[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, h = blockIdx.y;
  const int t_raw = blockIdx.x * 4 + wave;
  const bool live = t_raw < Tn && t_raw < cu[B];
  const int t = live ? t_raw : 0;
  const int b = find_seq(cu, B, t), s0 = min(max(cu[b], 0), t);  // clamped: a malformed cu must not lead out of bounds
  const int nk = min(t - s0 + 1, max_len);  // keys 0 .. i of the sequence
  const size_t d = (size_t)H * hd, col = (size_t)h * hd;
  float* qs = sm + (size_t)wave * (2 * hd + 2 * max_len);
  float* gs = qs + hd;
  float* p = gs + hd;
  float* ds = p + max_len;
  for (int e = lane; e < hd; e += 64) {
    qs[e] = to_f32(q[t * d + col + e]);
    gs[e] = to_f32(g[t * d + col + e]);
  }
  __syncthreads();
  float mx = -INFINITY;
  for (int j = lane; j < nk; j += 64) {
    const float s = dot_row(qs, k + (size_t)(s0 + j) * d + col, hd) * scale;
    p[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int j = lane; j < nk; j += 64) sum += __expf(p[j] - mx);
  sum = wave_sum(sum);
  const float l = mx + __logf(sum);
  float dl = 0.f;
  for (int j = lane; j < nk; j += 64) {
    const float pj = __expf(p[j] - l);
    const float dp = dot_row(gs, v + (size_t)(s0 + j) * d + col, hd);
    p[j] = pj;
    ds[j] = dp;
    dl = fmaf(pj, dp, dl);
  }
  dl = wave_sum(dl);
  for (int j = lane; j < nk; j += 64) ds[j] = p[j] * (ds[j] - dl);
  __syncthreads();
  for (int e = 2 * lane; e < hd; e += 128) {  // two dims per lane: head sizes up to 128 take one sweep
    const T* kc = k + (size_t)s0 * d + col + e;
    float a0 = 0.f, a1 = 0.f, b0 = 0.f, b1 = 0.f;
    int j = 0;
    for (; j + 1 < nk; j += 2) {
      const pair2<T> x = *(const pair2<T>*)(kc + (size_t)j * d), y = *(const pair2<T>*)(kc + (size_t)(j + 1) * d);
      a0 = fmaf(ds[j], to_f32(x.a), a0);
      a1 = fmaf(ds[j], to_f32(x.b), a1);
      b0 = fmaf(ds[j + 1], to_f32(y.a), b0);
      b1 = fmaf(ds[j + 1], to_f32(y.b), b1);
    }
    if (j < nk) {
      const pair2<T> x = *(const pair2<T>*)(kc + (size_t)j * d);
      a0 = fmaf(ds[j], to_f32(x.a), a0);
      a1 = fmaf(ds[j], to_f32(x.b), a1);
    }
    if (live) {
      pair2<T> o;
      o.a = from_f32<T>((a0 + b0) * scale);
      o.b = from_f32<T>((a1 + b1) * scale);
      *(pair2<T>*)(dq + t * d + col + e) = o;
    }
  }
  if (live && lane == 0) {
    lse[(size_t)t * H + h] = l;
    delta[(size_t)t * H + h] = dl;
  }
}

template <typename T>
__global__ void __launch_bounds__(256)
    attn_bwd_kv_kernel(const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v,
                       const T* __restrict__ g, const int* __restrict__ cu, int B, int Tn, int H, int hd, float scale,
                       int max_len, const float* __restrict__ lse, const float* __restrict__ delta,
                       T* __restrict__ dk, T* __restrict__ dv) {
  extern __shared__ float sm[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, h = blockIdx.y;
  const int t_raw = blockIdx.x * 4 + wave;
  const bool live = t_raw < Tn && t_raw < cu[B];
  const int t = live ? t_raw : 0;
  const int b = find_seq(cu, B, t), s0 = min(max(cu[b], 0), t);
  const int n = min(cu[b + 1] - s0, max_len);
  const int j = t - s0;
  const int nq = max(min(n - j, Tn - t), 0);  // queries j .. n-1 of the sequence see this key
  const size_t d = (size_t)H * hd, col = (size_t)h * hd;
  float* ks = sm + (size_t)wave * (2 * hd + 2 * max_len);
  float* vs = ks + hd;
  float* p = vs + hd;
  float* ds = p + max_len;
  for (int e = lane; e < hd; e += 64) {
    ks[e] = to_f32(k[t * d + col + e]);
    vs[e] = to_f32(v[t * d + col + e]);
  }
  __syncthreads();
  for (int ii = lane; ii < nq; ii += 64) {
    const size_t r = (size_t)(t + ii);
    const float s = dot_row(ks, q + r * d + col, hd) * scale;
    const float pr = __expf(s - lse[r * H + h]);
    const float dp = dot_row(vs, g + r * d + col, hd);
    p[ii] = pr;
    ds[ii] = pr * (dp - delta[r * H + h]);
  }
  __syncthreads();
  for (int e = 2 * lane; e < hd; e += 128) {
    const T* gc = g + (size_t)t * d + col + e;
    const T* qc = q + (size_t)t * d + col + e;
    float av0 = 0.f, av1 = 0.f, ak0 = 0.f, ak1 = 0.f;
    for (int ii = 0; ii < nq; ++ii) {
      const pair2<T> x = *(const pair2<T>*)(gc + (size_t)ii * d), y = *(const pair2<T>*)(qc + (size_t)ii * d);
      av0 = fmaf(p[ii], to_f32(x.a), av0);
      av1 = fmaf(p[ii], to_f32(x.b), av1);
      ak0 = fmaf(ds[ii], to_f32(y.a), ak0);
      ak1 = fmaf(ds[ii], to_f32(y.b), ak1);
    }
    if (live) {
      pair2<T> o;
      o.a = from_f32<T>(av0);
      o.b = from_f32<T>(av1);
      *(pair2<T>*)(dv + t * d + col + e) = o;
      o.a = from_f32<T>(ak0 * scale);
      o.b = from_f32<T>(ak1 * scale);
      *(pair2<T>*)(dk + t * d + col + e) = o;
    }
  }
}

}  // namespace

// dtype 0: float, 1: fp16.  head_dim a multiple of 4 (float) or 8 (fp16); the longest sequence at
// most max_len rows (longer ones are cut off at max_len: wrong results, but no access out of bounds).
hipError_t launch_attention_backward(int dtype, const void* q, const void* k, const void* v, const void* g,
                                     const int* cu, int B, int Tn, int H, int hd, int max_len, float* lse,
                                     float* delta, void* dq, void* dk, void* dv, hipStream_t s) {
  if (Tn <= 0) return hipSuccess;
  if (hd <= 0 || (hd % (dtype == 0 ? 4 : 8)) != 0 || max_len <= 0) return hipErrorInvalidValue;
  const size_t sh = (size_t)4 * (2 * (size_t)hd + 2 * (size_t)max_len) * sizeof(float);
  if (sh > 150 * 1024) return hipErrorInvalidValue;
  const float scale = 1.0f / sqrtf((float)hd);
  dim3 grid((Tn + 3) / 4, H);
  if (dtype == 0) {
    if (sh > 65536) {
      (void)hipFuncSetAttribute((const void*)attn_bwd_q_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh);
      (void)hipFuncSetAttribute((const void*)attn_bwd_kv_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh);
    }
    hipLaunchKernelGGL(attn_bwd_q_kernel<float>, grid, dim3(256), sh, s, (const float*)q, (const float*)k,
                       (const float*)v, (const float*)g, cu, B, Tn, H, hd, scale, max_len, lse, delta, (float*)dq);
    hipLaunchKernelGGL(attn_bwd_kv_kernel<float>, grid, dim3(256), sh, s, (const float*)q, (const float*)k,
                       (const float*)v, (const float*)g, cu, B, Tn, H, hd, scale, max_len, lse, delta, (float*)dk,
                       (float*)dv);
  } else {
    if (sh > 65536) {
      (void)hipFuncSetAttribute((const void*)attn_bwd_q_kernel<half_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh);
      (void)hipFuncSetAttribute((const void*)attn_bwd_kv_kernel<half_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh);
    }
    hipLaunchKernelGGL(attn_bwd_q_kernel<half_t>, grid, dim3(256), sh, s, (const half_t*)q, (const half_t*)k,
                       (const half_t*)v, (const half_t*)g, cu, B, Tn, H, hd, scale, max_len, lse, delta, (half_t*)dq);
    hipLaunchKernelGGL(attn_bwd_kv_kernel<half_t>, grid, dim3(256), sh, s, (const half_t*)q, (const half_t*)k,
                       (const half_t*)v, (const half_t*)g, cu, B, Tn, H, hd, scale, max_len, lse, delta, (half_t*)dk,
                       (half_t*)dv);
  }
  return hipGetLastError();
}

}  // namespace rlhf
