// Row bookkeeping, embedding gather, LayerNorm (+ value head), partial rotary + KV store, the
// Gumbel-max sampler, log-sum-exp + target gather, and output scatter.  All bandwidth-bound.
#include <algorithm>

#include "common.h"

namespace rlhf {

// =================================================================================================
// Row spans: one wave per row finds the first real slot and the number of real slots.
// =================================================================================================
__global__ void row_span_kernel(const uint8_t* __restrict__ mask, int L, int* __restrict__ start,
                                int* __restrict__ len) {
  const int b = blockIdx.x;
  const uint8_t* row = mask + (size_t)b * L;
  int cnt = 0, first = L;
  for (int c = threadIdx.x; c < L; c += 64) {
    if (row[c]) {
      cnt++;
      first = min(first, c);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    cnt += __shfl_xor(cnt, o, 64);
    first = min(first, __shfl_xor(first, o, 64));
  }
  if (threadIdx.x == 0) {
    len[b] = cnt;
    start[b] = cnt ? first : 0;
  }
}

// Exclusive prefix sums over B rows (B is at most a few thousand: one thread walks them).
__global__ void row_scan_kernel(const int* __restrict__ len, int B, int kv_extra, int* __restrict__ cu,
                                int* __restrict__ kvoff, int* __restrict__ total) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  int a = 0, k = 0;
  for (int b = 0; b < B; ++b) {
    cu[b] = a;
    kvoff[b] = k;
    a += len[b];
    k += len[b] + kv_extra;
  }
  cu[B] = a;
  kvoff[B] = k;
  total[0] = a;
  total[1] = k;
}

hipError_t launch_row_spans(const uint8_t* mask, int B, int L, int kv_extra, int* start, int* len, int* cu,
                            int* kvoff, int* total, hipStream_t s) {
  hipLaunchKernelGGL(row_span_kernel, dim3(B), dim3(64), 0, s, mask, L, start, len);
  hipLaunchKernelGGL(row_scan_kernel, dim3(1), dim3(64), 0, s, len, B, kv_extra, cu, kvoff, total);
  return hipGetLastError();
}

// =================================================================================================
// Pack + embed
// =================================================================================================
template <typename T>
__global__ void pack_embed_kernel(const int32_t* __restrict__ tokens, int L, const int* __restrict__ start,
                                  const int* __restrict__ len, const int* __restrict__ cu,
                                  const T* __restrict__ embed, int d, int vocab, int* __restrict__ pos,
                                  int* __restrict__ rowid, int* __restrict__ tok, float* __restrict__ x) {
  const int i = blockIdx.x, b = blockIdx.y;
  if (i >= len[b]) return;
  const int t = cu[b] + i;
  // ids outside the vocabulary are a caller error; clamping keeps every access in bounds
  const int id = min(max(tokens[(size_t)b * L + start[b] + i], 0), vocab - 1);
  if (threadIdx.x == 0) {
    pos[t] = i;
    rowid[t] = b;
    tok[t] = id;
  }
  const T* e = embed + (size_t)id * d;
  float* xr = x + (size_t)t * d;
  for (int c = threadIdx.x; c < d; c += blockDim.x) xr[c] = to_f32(e[c]);
}

hipError_t launch_pack_embed(int dtype, const int32_t* tokens, int B, int L, const int* start, const int* len,
                             const int* cu, const void* embed, int d, int vocab, int* pos, int* rowid, int* tok,
                             float* x, hipStream_t s) {
  dim3 grid(L, B), block(256);
  if (dtype == 0)
    hipLaunchKernelGGL(pack_embed_kernel<float>, grid, block, 0, s, tokens, L, start, len, cu,
                       (const float*)embed, d, vocab, pos, rowid, tok, x);
  else
    hipLaunchKernelGGL(pack_embed_kernel<bf16_t>, grid, block, 0, s, tokens, L, start, len, cu,
                       (const bf16_t*)embed, d, vocab, pos, rowid, tok, x);
  return hipGetLastError();
}

template <typename T>
__global__ void embed_rows_kernel(const int32_t* __restrict__ tok, const T* __restrict__ embed, int d, int vocab,
                                  float* __restrict__ x) {
  const int b = blockIdx.x;
  const T* e = embed + (size_t)min(max(tok[b], 0), vocab - 1) * d;  // an id outside the table never leaves it
  float* xr = x + (size_t)b * d;
  for (int c = threadIdx.x; c < d; c += blockDim.x) xr[c] = to_f32(e[c]);
}

hipError_t launch_embed_rows(int dtype, const int32_t* tok, int B, const void* embed, int d, int vocab, float* x,
                             hipStream_t s) {
  if (dtype == 0)
    hipLaunchKernelGGL(embed_rows_kernel<float>, dim3(B), dim3(256), 0, s, tok, (const float*)embed, d, vocab, x);
  else
    hipLaunchKernelGGL(embed_rows_kernel<bf16_t>, dim3(B), dim3(256), 0, s, tok, (const bf16_t*)embed, d, vocab, x);
  return hipGetLastError();
}

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

// out row r = in row src[r] + src_add, rows of `chunks` 16-byte pieces (any element type).
__global__ void __launch_bounds__(256)
    gather_rows_kernel(const u32x4_t* __restrict__ in, const int* __restrict__ src, int src_add, int chunks,
                       u32x4_t* __restrict__ out) {
  const size_t sr = (size_t)max(src[blockIdx.x] + src_add, 0);
  for (int c = threadIdx.x; c < chunks; c += 256) out[(size_t)blockIdx.x * chunks + c] = in[sr * chunks + c];
}

hipError_t launch_gather_rows(const void* in, const int* src, int src_add, int rows, size_t row_bytes, void* out,
                              hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if ((row_bytes & 15) != 0 || row_bytes / 16 > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(gather_rows_kernel, dim3(rows), dim3(256), 0, s, (const u32x4_t*)in, src, src_add,
                     (int)(row_bytes / 16), (u32x4_t*)out);
  return hipGetLastError();
}

// =================================================================================================
// LayerNorm: one block per row, fp32 statistics (mean, then centred second moment), up to two
// affine outputs from the same statistics, optional value-head dot product on the first output.
// =================================================================================================
__device__ __forceinline__ float block_sum_256(float v, float* sh) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6;
  __syncthreads();  // protects sh against the previous use
  if ((threadIdx.x & 63) == 0) sh[w] = v;
  __syncthreads();
  return sh[0] + sh[1] + sh[2] + sh[3];
}

template <typename WT, typename AT>
__global__ void __launch_bounds__(256)
    layernorm_kernel(const float* __restrict__ x, const int* __restrict__ src, int src_add,
                     const int* __restrict__ rows_dev, int d, float eps, const WT* __restrict__ g1,
                     const WT* __restrict__ b1, AT* __restrict__ out1, const WT* __restrict__ g2,
                     const WT* __restrict__ b2, AT* __restrict__ out2, const WT* __restrict__ value_w,
                     float value_b, float* __restrict__ val) {
  __shared__ float sh[4];
  const int r = blockIdx.x;
  if (rows_dev && r >= *rows_dev) return;
  const int sr = src ? max(src[r] + src_add, 0) : r;  // an empty first sequence would give -1
  const float* xr = x + (size_t)sr * d;
  float s = 0.f;
  for (int c = threadIdx.x; c < d; c += 256) s += xr[c];
  const float mean = block_sum_256(s, sh) / (float)d;
  float q = 0.f;
  for (int c = threadIdx.x; c < d; c += 256) {
    const float u = xr[c] - mean;
    q += u * u;
  }
  const float rstd = 1.0f / sqrtf(block_sum_256(q, sh) / (float)d + eps);
  float vd = 0.f;
  for (int c = threadIdx.x; c < d; c += 256) {
    const float n = (xr[c] - mean) * rstd;
    const float h1 = n * to_f32(g1[c]) + to_f32(b1[c]);
    out1[(size_t)r * d + c] = from_f32<AT>(h1);
    if (out2) out2[(size_t)r * d + c] = from_f32<AT>(n * to_f32(g2[c]) + to_f32(b2[c]));
    if (val) vd += h1 * to_f32(value_w[c]);
  }
  if (val) {
    vd = block_sum_256(vd, sh);
    if (threadIdx.x == 0) val[r] = vd + value_b;
  }
}

// Vectorised form for bf16 parameters / fp16 outputs: d a multiple of 4 and at most 4096; the row
// lives in registers (up to four float4 per thread), parameters and outputs move 8 bytes at a time.
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

__device__ __forceinline__ f32x4_t bf16x4_to_f32(u32x2_t v) {
  f32x4_t r;
  r[0] = __uint_as_float(v[0] << 16);
  r[1] = __uint_as_float(v[0] & 0xFFFF0000u);
  r[2] = __uint_as_float(v[1] << 16);
  r[3] = __uint_as_float(v[1] & 0xFFFF0000u);
  return r;
}

// Sum of ks fp32 partial slabs at one float4 position, added in slab order.  The usual split factors
// are unrolled completely so that all loads are in flight before the chain of additions starts.
template <int KS>
__device__ __forceinline__ f32x4_t sum_slabs_n(const f32x4_t* __restrict__ p, size_t slab4) {
  f32x4_t v[KS];
#pragma unroll
  for (int z = 0; z < KS; ++z) v[z] = p[z * slab4];
  f32x4_t t = v[0];
#pragma unroll
  for (int z = 1; z < KS; ++z) t += v[z];
  return t;
}
__device__ __forceinline__ f32x4_t sum_slabs(const f32x4_t* __restrict__ p, size_t slab4, int ks) {
  switch (ks) {
    case 2: return sum_slabs_n<2>(p, slab4);
    case 4: return sum_slabs_n<4>(p, slab4);
    case 8: return sum_slabs_n<8>(p, slab4);
    case 16: return sum_slabs_n<16>(p, slab4);
    default: break;
  }
  f32x4_t t = p[0];
  for (int z = 1; z < ks; ++z) t += p[z * slab4];
  return t;
}

// One block per row (few rows: decode).
__global__ void __launch_bounds__(256)
    layernorm_vec_block_kernel(const float* x, const int* __restrict__ src, int src_add,
                         const int* __restrict__ rows_dev, int d, float eps, const bf16_t* __restrict__ g1,
                         const bf16_t* __restrict__ b1, half_t* __restrict__ out1, const bf16_t* __restrict__ g2,
                         const bf16_t* __restrict__ b2, half_t* __restrict__ out2,
                         const bf16_t* __restrict__ value_w, float value_b, float* __restrict__ val,
                         PendingResidual pend, float* xw) {
  __shared__ float sh[4];
  const int r = blockIdx.x;
  if (rows_dev && r >= *rows_dev) return;
  const int sr = src ? max(src[r] + src_add, 0) : r;
  const f32x4_t* xr = (const f32x4_t*)(x + (size_t)sr * d);
  const int nv = d >> 2;
  f32x4_t v[4];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = threadIdx.x + 256 * i;
    if (c < nv) {
      v[i] = xr[c];
      if (xw) {
        // two split-K products whose reduction was left to this kernel: x <- (x + (sum_z A_z + bias_a))
        // + (sum_z B_z + bias_b), slabs in index order, the order of the stand-alone reduction
        const size_t o = (size_t)r * nv + c;
        const size_t slab4 = pend.slab >> 2;
        const f32x4_t ta = sum_slabs((const f32x4_t*)pend.part_a + o, slab4, pend.ks_a);
        const f32x4_t tb = sum_slabs((const f32x4_t*)pend.part_b + o, slab4, pend.ks_b);
        v[i] += ta + bf16x4_to_f32(((const u32x2_t*)pend.bias_a)[c]);
        v[i] += tb + bf16x4_to_f32(((const u32x2_t*)pend.bias_b)[c]);
        ((f32x4_t*)(xw + (size_t)r * d))[c] = v[i];
      }
      s += v[i][0] + v[i][1] + v[i][2] + v[i][3];
    }
  }
  const float mean = block_sum_256(s, sh) / (float)d;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = threadIdx.x + 256 * i;
    if (c < nv) {
      v[i] -= mean;
      q += v[i][0] * v[i][0] + v[i][1] * v[i][1] + v[i][2] * v[i][2] + v[i][3] * v[i][3];
    }
  }
  const float rstd = 1.0f / sqrtf(block_sum_256(q, sh) / (float)d + eps);
  float vd = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = threadIdx.x + 256 * i;
    if (c < nv) {
      const f32x4_t n = v[i] * rstd;
      const f32x4_t h1 = n * bf16x4_to_f32(((const u32x2_t*)g1)[c]) + bf16x4_to_f32(((const u32x2_t*)b1)[c]);
      f16x4_t o;
#pragma unroll
      for (int u = 0; u < 4; ++u) o[u] = from_f32<half_t>(h1[u]);
      ((f16x4_t*)(out1 + (size_t)r * d))[c] = o;
      if (out2) {
        const f32x4_t h2 = n * bf16x4_to_f32(((const u32x2_t*)g2)[c]) + bf16x4_to_f32(((const u32x2_t*)b2)[c]);
#pragma unroll
        for (int u = 0; u < 4; ++u) o[u] = from_f32<half_t>(h2[u]);
        ((f16x4_t*)(out2 + (size_t)r * d))[c] = o;
      }
      if (val) {
        const f32x4_t w = bf16x4_to_f32(((const u32x2_t*)value_w)[c]);
        vd += h1[0] * w[0] + h1[1] * w[1] + h1[2] * w[2] + h1[3] * w[3];
      }
    }
  }
  if (val) {
    vd = block_sum_256(vd, sh);
    if (threadIdx.x == 0) val[r] = vd + value_b;
  }
}

// One wave per row, four rows per block: no block-wide synchronisation, only wave shuffles.
template <int NV>  // float4 chunks per lane: d <= 256 * NV
__global__ void __launch_bounds__(256)
    layernorm_vec_kernel(const float* __restrict__ x, const int* __restrict__ src, int src_add, int rows_max,
                         const int* __restrict__ rows_dev, int d, float eps, const bf16_t* __restrict__ g1,
                         const bf16_t* __restrict__ b1, half_t* __restrict__ out1, const bf16_t* __restrict__ g2,
                         const bf16_t* __restrict__ b2, half_t* __restrict__ out2,
                         const bf16_t* __restrict__ value_w, float value_b, float* __restrict__ val) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= (rows_dev ? min(*rows_dev, rows_max) : rows_max)) return;
  const int sr = src ? max(src[r] + src_add, 0) : r;
  const f32x4_t* xr = (const f32x4_t*)(x + (size_t)sr * d);
  const int nv = d >> 2;
  f32x4_t v[NV];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = lane + 64 * i;
    if (c < nv) {
      v[i] = xr[c];
      s += v[i][0] + v[i][1] + v[i][2] + v[i][3];
    }
  }
  const float mean = wave_sum(s) / (float)d;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = lane + 64 * i;
    if (c < nv) {
      v[i] -= mean;
      q += v[i][0] * v[i][0] + v[i][1] * v[i][1] + v[i][2] * v[i][2] + v[i][3] * v[i][3];
    }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)d + eps);
  float vd = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = lane + 64 * i;
    if (c < nv) {
      const f32x4_t n = v[i] * rstd;
      const f32x4_t h1 = n * bf16x4_to_f32(((const u32x2_t*)g1)[c]) + bf16x4_to_f32(((const u32x2_t*)b1)[c]);
      f16x4_t o;
#pragma unroll
      for (int u = 0; u < 4; ++u) o[u] = from_f32<half_t>(h1[u]);
      ((f16x4_t*)(out1 + (size_t)r * d))[c] = o;
      if (out2) {
        const f32x4_t h2 = n * bf16x4_to_f32(((const u32x2_t*)g2)[c]) + bf16x4_to_f32(((const u32x2_t*)b2)[c]);
#pragma unroll
        for (int u = 0; u < 4; ++u) o[u] = from_f32<half_t>(h2[u]);
        ((f16x4_t*)(out2 + (size_t)r * d))[c] = o;
      }
      if (val) {
        const f32x4_t w = bf16x4_to_f32(((const u32x2_t*)value_w)[c]);
        vd += h1[0] * w[0] + h1[1] * w[1] + h1[2] * w[2] + h1[3] * w[3];
      }
    }
  }
  if (val) {
    vd = wave_sum(vd);
    if (lane == 0) val[r] = vd + value_b;
  }
}

// Same, with 8 consecutive elements per lane: two 16-byte loads, and one 16-byte fp16 store per
// output instead of two 8-byte ones.
template <int NV8>  // 8-element chunks per lane: d <= 512 * NV8
__global__ void __launch_bounds__(256)
    layernorm_vec8_kernel(const float* __restrict__ x, const int* __restrict__ src, int src_add, int rows_max,
                          const int* __restrict__ rows_dev, int d, float eps, const bf16_t* __restrict__ g1,
                          const bf16_t* __restrict__ b1, half_t* __restrict__ out1, const bf16_t* __restrict__ g2,
                          const bf16_t* __restrict__ b2, half_t* __restrict__ out2,
                          const bf16_t* __restrict__ value_w, float value_b, float* __restrict__ val) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= (rows_dev ? min(*rows_dev, rows_max) : rows_max)) return;
  const int sr = src ? max(src[r] + src_add, 0) : r;
  const f32x4_t* xr = (const f32x4_t*)(x + (size_t)sr * d);
  const int nv = d >> 3;
  f32x4_t v[NV8][2];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NV8; ++i) {
    const int c = lane + 64 * i;
    if (c < nv) {
      v[i][0] = xr[2 * c];
      v[i][1] = xr[2 * c + 1];
      s += (v[i][0][0] + v[i][0][1] + v[i][0][2] + v[i][0][3]) + (v[i][1][0] + v[i][1][1] + v[i][1][2] + v[i][1][3]);
    }
  }
  const float mean = wave_sum(s) / (float)d;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < NV8; ++i) {
    const int c = lane + 64 * i;
    if (c < nv) {
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        v[i][hh] -= mean;
        q += v[i][hh][0] * v[i][hh][0] + v[i][hh][1] * v[i][hh][1] + v[i][hh][2] * v[i][hh][2] +
             v[i][hh][3] * v[i][hh][3];
      }
    }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)d + eps);
  float vd = 0.f;
#pragma unroll
  for (int i = 0; i < NV8; ++i) {
    const int c = lane + 64 * i;
    if (c < nv) {
      f16x8_t o1, o2;
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const f32x4_t n = v[i][hh] * rstd;
        const int c4 = 2 * c + hh;
        const f32x4_t h1 = n * bf16x4_to_f32(((const u32x2_t*)g1)[c4]) + bf16x4_to_f32(((const u32x2_t*)b1)[c4]);
#pragma unroll
        for (int u = 0; u < 4; ++u) o1[4 * hh + u] = from_f32<half_t>(h1[u]);
        if (out2) {
          const f32x4_t h2 = n * bf16x4_to_f32(((const u32x2_t*)g2)[c4]) + bf16x4_to_f32(((const u32x2_t*)b2)[c4]);
#pragma unroll
          for (int u = 0; u < 4; ++u) o2[4 * hh + u] = from_f32<half_t>(h2[u]);
        }
        if (val) {
          const f32x4_t w = bf16x4_to_f32(((const u32x2_t*)value_w)[c4]);
          vd += h1[0] * w[0] + h1[1] * w[1] + h1[2] * w[2] + h1[3] * w[3];
        }
      }
      ((f16x8_t*)(out1 + (size_t)r * d))[c] = o1;
      if (out2) ((f16x8_t*)(out2 + (size_t)r * d))[c] = o2;
    }
  }
  if (val) {
    vd = wave_sum(vd);
    if (lane == 0) val[r] = vd + value_b;
  }
}

template <typename M>
static hipError_t ln_launch(const float* x, const int* src, int src_add, int rows_max, const int* rows_dev, int d,
                            float eps, const void* g1, const void* b1, void* out1, const void* g2,
                            const void* b2, void* out2, const void* vw, float vb, float* val, hipStream_t s) {
  if (rows_max <= 0) return hipSuccess;
  typedef typename M::W WT;
  typedef typename M::A AT;
  if (sizeof(AT) == 2 && (d & 3) == 0 && d <= 4096) {
    const dim3 grid((rows_max + 3) / 4);
    if (rows_max <= 2048)
      hipLaunchKernelGGL(layernorm_vec_block_kernel, dim3(rows_max), dim3(256), 0, s, x, src, src_add, rows_dev, d,
                         eps, (const bf16_t*)g1, (const bf16_t*)b1, (half_t*)out1, (const bf16_t*)g2,
                         (const bf16_t*)b2, (half_t*)out2, (const bf16_t*)vw, vb, val, PendingResidual{},
                         (float*)nullptr);
    else if ((d & 7) == 0 && d > 1024)
      hipLaunchKernelGGL(layernorm_vec8_kernel<8>, grid, dim3(256), 0, s, x, src, src_add, rows_max, rows_dev, d,
                         eps, (const bf16_t*)g1, (const bf16_t*)b1, (half_t*)out1, (const bf16_t*)g2,
                         (const bf16_t*)b2, (half_t*)out2, (const bf16_t*)vw, vb, val);
    else if (d <= 1024)
      hipLaunchKernelGGL(layernorm_vec_kernel<4>, grid, dim3(256), 0, s, x, src, src_add, rows_max, rows_dev, d,
                         eps, (const bf16_t*)g1, (const bf16_t*)b1, (half_t*)out1, (const bf16_t*)g2,
                         (const bf16_t*)b2, (half_t*)out2, (const bf16_t*)vw, vb, val);
    else
      hipLaunchKernelGGL(layernorm_vec_kernel<16>, grid, dim3(256), 0, s, x, src, src_add, rows_max, rows_dev, d,
                         eps, (const bf16_t*)g1, (const bf16_t*)b1, (half_t*)out1, (const bf16_t*)g2,
                         (const bf16_t*)b2, (half_t*)out2, (const bf16_t*)vw, vb, val);
    return hipGetLastError();
  }
  hipLaunchKernelGGL((layernorm_kernel<WT, AT>), dim3(rows_max), dim3(256), 0, s, x, src, src_add, rows_dev, d,
                     eps, (const WT*)g1, (const WT*)b1, (AT*)out1, (const WT*)g2, (const WT*)b2, (AT*)out2,
                     (const WT*)vw, vb, val);
  return hipGetLastError();
}

hipError_t launch_layernorm(int dtype, const float* x, int rows_max, const int* rows_dev, int d, float eps,
                            const void* g1, const void* b1, void* out1, const void* g2, const void* b2,
                            void* out2, hipStream_t s) {
  if (dtype == 0)
    return ln_launch<ModeF32>(x, nullptr, 0, rows_max, rows_dev, d, eps, g1, b1, out1, g2, b2, out2, nullptr, 0.f,
                            nullptr, s);
  return ln_launch<ModeBF16>(x, nullptr, 0, rows_max, rows_dev, d, eps, g1, b1, out1, g2, b2, out2, nullptr, 0.f,
                           nullptr, s);
}

bool layernorm_pending_supported(int dtype, int rows_max, int d) {
  return dtype == 1 && (d & 3) == 0 && d <= 4096 && rows_max <= 2048;
}

hipError_t launch_layernorm_pending(float* x, int rows_max, const int* rows_dev, int d, float eps, const void* g1,
                                    const void* b1, void* out1, const void* g2, const void* b2, void* out2,
                                    const PendingResidual& pend, hipStream_t s) {
  if (!layernorm_pending_supported(1, rows_max, d) || (pend.slab & 3) != 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(layernorm_vec_block_kernel, dim3(rows_max), dim3(256), 0, s, x, (const int*)nullptr, 0,
                     rows_dev, d, eps, (const bf16_t*)g1, (const bf16_t*)b1, (half_t*)out1, (const bf16_t*)g2,
                     (const bf16_t*)b2, (half_t*)out2, (const bf16_t*)nullptr, 0.f, (float*)nullptr, pend, x);
  return hipGetLastError();
}

hipError_t launch_final_ln(int dtype, const float* x, const int* src, int src_add, int rows_max,
                           const int* rows_dev, int d, float eps, const void* g, const void* b, void* out,
                           const void* value_w, float value_b, float* val, hipStream_t s) {
  if (!value_w) val = nullptr;
  if (dtype == 0)
    return ln_launch<ModeF32>(x, src, src_add, rows_max, rows_dev, d, eps, g, b, out, nullptr, nullptr, nullptr,
                            value_w, value_b, val, s);
  return ln_launch<ModeBF16>(x, src, src_add, rows_max, rows_dev, d, eps, g, b, out, nullptr, nullptr, nullptr,
                           value_w, value_b, val, s);
}

// =================================================================================================
// Partial rotary + K/V store.  One block per packed row.
// =================================================================================================
template <typename T>
__global__ void __launch_bounds__(256)
    rope_kv_kernel(const T* __restrict__ qkv, const int* __restrict__ rows_dev, const int* __restrict__ pos,
                   int pos_add, const int* __restrict__ rowid, const int* __restrict__ kvoff,
                   const int* __restrict__ len, int H, int hd,
                   int r, const float* __restrict__ cos_t, const float* __restrict__ sin_t, T* __restrict__ q,
                   T* __restrict__ kc, T* __restrict__ vc, long kv_extra) {
  // fp16 (bf16-model) path: the rows of W_qkv were reordered when the handle was created so that
  // the two dims of a rotary pair are neighbours (see launch_qkv_weights_f16)
  constexpr bool ADJ = sizeof(T) == 2;
  const int t = blockIdx.x;
  if (rows_dev && t >= *rows_dev) return;
  const int d = H * hd;
  const int p = pos[t] + pos_add;
  const int b = rowid ? rowid[t] : t;
  const long seq_base = (long)kvoff[b] * H;          // sequence b owns slots [kvoff[b]*H, kvoff[b+1]*H)
  const long seq_len = len[b] + kv_extra;             // slots per head inside that slab
  const T* src = qkv + (size_t)t * 3 * d;
  const int half = r >> 1;
  const float* cs = cos_t + (size_t)p * half;
  const float* sn = sin_t + (size_t)p * half;
  for (int c = threadIdx.x; c < d; c += 256) {
    const int h = c / hd, e = c - h * hd;
    float qv = to_f32(src[c]), kv = to_f32(src[d + c]);
    if (ADJ) {  // pair (2i, 2i+1) turns by angle i
      if (e < r) {
        const float co = cs[e >> 1], si = (e & 1) ? sn[e >> 1] : -sn[e >> 1];
        const int cp = c - e + (e ^ 1);
        qv = qv * co + to_f32(src[cp]) * si;
        kv = kv * co + to_f32(src[d + cp]) * si;
      }
    } else if (e < half) {
      const float co = cs[e], si = sn[e];
      qv = qv * co - to_f32(src[c + half]) * si;
      kv = kv * co - to_f32(src[d + c + half]) * si;
    } else if (e < r) {
      const float co = cs[e - half], si = sn[e - half];
      qv = qv * co + to_f32(src[c - half]) * si;
      kv = kv * co + to_f32(src[d + c - half]) * si;
    }
    q[(size_t)t * d + c] = from_f32<T>(qv);
    const size_t o = (size_t)(seq_base + h * seq_len + p) * hd + e;
    kc[o] = from_f32<T>(kv);
    vc[o] = src[2 * d + c];
  }
}

// fp16 form moving 16 bytes (8 dims) per access; head_dim a multiple of 8.  Only the chunks that
// overlap the rotary dims do per-element work (the rotation partner is fetched as a scalar).
// A block takes RPB consecutive packed rows, so that the K / V stores of one head are RPB adjacent
// 2*hd-byte rows written by one CU.  Two passes: (1) one thread per (row, q|k, head) loads the
// head's rotary dims (the first ceil(R/8) 16-byte chunks), rotates them in registers and stores
// them; (2) every other chunk (rest of q and k, all of v) is a 16-byte copy.  R is a template
// parameter so the rotation pairs (2i, 2i + 1: the reordered layout of the fp16 path) are register-to-register.
template <int RPB, int R>
__global__ void __launch_bounds__(256)
    rope_kv_vec_kernel(const half_t* __restrict__ qkv, int rows_max, const int* __restrict__ rows_dev,
                       const int* __restrict__ pos, int pos_add, const int* __restrict__ rowid,
                       const int* __restrict__ kvoff, const int* __restrict__ len, int H, int hd,
                       const float* __restrict__ cos_t, const float* __restrict__ sin_t, half_t* __restrict__ q,
                       half_t* __restrict__ kc, half_t* __restrict__ vc, long kv_extra) {
  constexpr int HALF = R / 2, RC = (R + 7) / 8;
  __shared__ int s_pos[RPB];
  __shared__ long s_base[RPB], s_len[RPB];
  const int t0 = blockIdx.x * RPB;
  const int rows = min(rows_dev ? *rows_dev : rows_max, rows_max);
  if (t0 >= rows) return;
  const int nr = min(RPB, rows - t0);
  if (threadIdx.x < nr) {
    const int t = t0 + threadIdx.x;
    const int p = pos[t] + pos_add;
    const int b = rowid ? rowid[t] : t;
    s_pos[threadIdx.x] = p;
    s_len[threadIdx.x] = len[b] + kv_extra;             // slots per head in sequence b's slab
    s_base[threadIdx.x] = (long)kvoff[b] * H + p;       // slab start (in slots) + position
  }
  __syncthreads();
  const int d = H * hd, cph = hd >> 3;
  auto dst_of = [&](int sec, int rr, int h) -> half_t* {
    return sec == 0 ? q + (size_t)(t0 + rr) * d + h * hd
                    : (sec == 1 ? kc : vc) + (size_t)(s_base[rr] + h * s_len[rr]) * hd;
  };
  // ---- pass 1: rotary part of every q and k head
  for (int c = threadIdx.x; c < nr * 2 * H; c += 256) {
    const int rr = c / (2 * H), w = c - rr * 2 * H;
    const int sec = w / H, h = w - sec * H;
    const half_t* hb = qkv + (size_t)(t0 + rr) * 3 * d + sec * d + h * hd;
    f16x8_t v[RC];
#pragma unroll
    for (int i = 0; i < RC; ++i) v[i] = *(const f16x8_t*)(hb + 8 * i);
    const float* cs = cos_t + (size_t)s_pos[rr] * HALF;
    const float* sn = sin_t + (size_t)s_pos[rr] * HALF;
#pragma unroll
    for (int i = 0; i < HALF; ++i) {
      const float co = cs[i], si = sn[i];
      const float lo = (float)v[(2 * i) >> 3][(2 * i) & 7], hi = (float)v[(2 * i + 1) >> 3][(2 * i + 1) & 7];
      v[(2 * i) >> 3][(2 * i) & 7] = from_f32<half_t>(lo * co - hi * si);
      v[(2 * i + 1) >> 3][(2 * i + 1) & 7] = from_f32<half_t>(hi * co + lo * si);
    }
    half_t* dst = dst_of(sec, rr, h);
#pragma unroll
    for (int i = 0; i < RC; ++i) *(f16x8_t*)(dst + 8 * i) = v[i];
  }
  // ---- pass 2: plain copies, chunk fastest, then row, then head, then section
  const int qk_cph = cph - RC;                    // untouched chunks per q / k head
  const int per_qk = nr * qk_cph, per_v = nr * cph;
  const int total = 2 * H * per_qk + H * per_v;
  for (int c = threadIdx.x; c < total; c += 256) {
    int sec, h, rr, ch;
    if (c < 2 * H * per_qk) {
      const int sh = c / per_qk, w = c - sh * per_qk;
      sec = sh / H; h = sh - sec * H;
      rr = w / qk_cph; ch = RC + (w - rr * qk_cph);
    } else {
      const int c2 = c - 2 * H * per_qk;
      sec = 2; h = c2 / per_v;
      const int w = c2 - h * per_v;
      rr = w / cph; ch = w - rr * cph;
    }
    const f16x8_t v = *(const f16x8_t*)(qkv + (size_t)(t0 + rr) * 3 * d + sec * d + h * hd + 8 * ch);
    *(f16x8_t*)(dst_of(sec, rr, h) + 8 * ch) = v;
  }
}

template <int RPB>
static bool launch_rope_vec(int r, dim3 grid, hipStream_t s, const half_t* qkv, int rows_max, const int* rows_dev,
                            const int* pos, int pos_add, const int* rowid, const int* kvoff, const int* len, int H,
                            int hd, const float* cos_t, const float* sin_t, half_t* q, half_t* kc, half_t* vc,
                            long kv_extra) {
#define RLHF_ROPE_CASE(RR)                                                                                     \
  case RR:                                                                                                     \
    hipLaunchKernelGGL((rope_kv_vec_kernel<RPB, RR>), grid, dim3(256), 0, s, qkv, rows_max, rows_dev, pos,     \
                       pos_add, rowid, kvoff, len, H, hd, cos_t, sin_t, q, kc, vc, kv_extra);                  \
    return true;
  switch (r) {
    RLHF_ROPE_CASE(4) RLHF_ROPE_CASE(16) RLHF_ROPE_CASE(20) RLHF_ROPE_CASE(32) RLHF_ROPE_CASE(64)
    default: return false;
  }
#undef RLHF_ROPE_CASE
}

// Many-rows form (prefill, scoring): block (RPB consecutive packed rows) x (HPB heads).  The q, k and v
// slices of those heads are loaded into LDS as RPB*3 contiguous segments of HPB*HD halfs, the rotary
// pairs are turned there, and the result leaves in 16-byte chunks: q as one contiguous segment per
// row, K and V as HD-long rows of which the RPB rows of one head are adjacent in a sequence's slab.
// All index arithmetic divides by compile-time constants.
template <int HD, int R, int HPB, int RPB>
__global__ void __launch_bounds__(256)
    rope_kv_tile_kernel(const half_t* __restrict__ qkv, int rows_max, const int* __restrict__ rows_dev,
                        const int* __restrict__ pos, int pos_add, const int* __restrict__ rowid,
                        const int* __restrict__ kvoff, const int* __restrict__ len, int H,
                        const float* __restrict__ cos_t, const float* __restrict__ sin_t, half_t* __restrict__ q,
                        half_t* __restrict__ kc, half_t* __restrict__ vc, long kv_extra) {
  constexpr int SEG = HPB * HD, SEGC = SEG / 8, CPH = HD / 8, HALF = R / 2;
  __shared__ __attribute__((aligned(16))) half_t tile[RPB * 3 * SEG];
  __shared__ int s_pos[RPB];
  __shared__ long s_base[RPB], s_len[RPB];
  const int t0 = blockIdx.x * RPB, h0 = blockIdx.y * HPB;
  const int rows = min(rows_dev ? *rows_dev : rows_max, rows_max);
  if (t0 >= rows) return;
  const int nr = min(RPB, rows - t0);
  const int d = H * HD;
  if (threadIdx.x < nr) {
    const int t = t0 + threadIdx.x;
    const int p = pos[t] + pos_add;
    const int b = rowid ? rowid[t] : t;
    s_pos[threadIdx.x] = p;
    s_len[threadIdx.x] = len[b] + kv_extra;
    s_base[threadIdx.x] = (long)kvoff[b] * H + p;
  }
  for (int c = threadIdx.x; c < nr * 3 * SEGC; c += 256) {
    const int rs = c / SEGC, ch = c - rs * SEGC;  // rs = row * 3 + section
    const int rr = rs / 3, sec = rs - rr * 3;
    *(f16x8_t*)(tile + rs * SEG + 8 * ch) =
        *(const f16x8_t*)(qkv + (size_t)(t0 + rr) * 3 * d + sec * d + h0 * HD + 8 * ch);
  }
  __syncthreads();
  for (int c = threadIdx.x; c < nr * 2 * HPB * HALF; c += 256) {
    const int u = c / HALF, i = c - u * HALF;     // u = (row * 2 + section) * HPB + head
    const int rs2 = u / HPB, hl = u - rs2 * HPB;
    const int rr = rs2 >> 1, sec = rs2 & 1;
    half_t* hb = tile + (rr * 3 + sec) * SEG + hl * HD;
    const float co = cos_t[(size_t)s_pos[rr] * HALF + i], si = sin_t[(size_t)s_pos[rr] * HALF + i];
    const float lo = (float)hb[2 * i], hi = (float)hb[2 * i + 1];
    hb[2 * i] = from_f32<half_t>(lo * co - hi * si);
    hb[2 * i + 1] = from_f32<half_t>(hi * co + lo * si);
  }
  __syncthreads();
  for (int c = threadIdx.x; c < nr * SEGC; c += 256) {  // q
    const int rr = c / SEGC, ch = c - rr * SEGC;
    *(f16x8_t*)(q + (size_t)(t0 + rr) * d + h0 * HD + 8 * ch) = *(const f16x8_t*)(tile + rr * 3 * SEG + 8 * ch);
  }
  for (int c = threadIdx.x; c < 2 * HPB * nr * CPH; c += 256) {  // k, v: chunk, then row, then head, then section
    const int w = c / CPH, ch = c - w * CPH;
    const int sh = w / nr, rr = w - sh * nr;
    const int sec = 1 + sh / HPB, hl = sh - (sec - 1) * HPB;
    half_t* dst = (sec == 1 ? kc : vc) + (size_t)(s_base[rr] + (h0 + hl) * s_len[rr]) * HD + 8 * ch;
    *(f16x8_t*)dst = *(const f16x8_t*)(tile + (rr * 3 + sec) * SEG + hl * HD + 8 * ch);
  }
}

template <int HD, int R, int HPB>
static void launch_rope_tile(hipStream_t s, const half_t* qkv, int rows_max, const int* rows_dev, const int* pos,
                             int pos_add, const int* rowid, const int* kvoff, const int* len, int H,
                             const float* cos_t, const float* sin_t, half_t* q, half_t* kc, half_t* vc,
                             long kv_extra) {
  hipLaunchKernelGGL((rope_kv_tile_kernel<HD, R, HPB, 8>), dim3((rows_max + 7) / 8, H / HPB), dim3(256), 0, s, qkv,
                     rows_max, rows_dev, pos, pos_add, rowid, kvoff, len, H, cos_t, sin_t, q, kc, vc, kv_extra);
}

// The head shapes of the model family (rotary on a quarter of the head); other shapes take the
// general kernels.
static bool try_rope_tile(hipStream_t s, const half_t* qkv, int rows_max, const int* rows_dev, const int* pos,
                          int pos_add, const int* rowid, const int* kvoff, const int* len, int H, int hd, int r,
                          const float* cos_t, const float* sin_t, half_t* q, half_t* kc, half_t* vc,
                          long kv_extra) {
#define RLHF_TILE(HD_, R_, HPB_)                                                                              \
  if (hd == HD_ && r == R_ && H % HPB_ == 0) {                                                                \
    launch_rope_tile<HD_, R_, HPB_>(s, qkv, rows_max, rows_dev, pos, pos_add, rowid, kvoff, len, H, cos_t,    \
                                    sin_t, q, kc, vc, kv_extra);                                              \
    return true;                                                                                              \
  }
  RLHF_TILE(80, 20, 8) RLHF_TILE(128, 32, 8) RLHF_TILE(256, 64, 4) RLHF_TILE(64, 16, 4) RLHF_TILE(16, 4, 1)
#undef RLHF_TILE
  return false;
}

hipError_t launch_rope_kv(int dtype, const void* qkv, int rows_max, const int* rows_dev, const int* pos,
                          int pos_add, const int* rowid, const int* kvoff, const int* len, int H, int hd, int r,
                          const float* cos_t, const float* sin_t, void* q, void* kc, void* vc,
                          long kv_extra, hipStream_t s) {
  if (rows_max <= 0) return hipSuccess;
  if (dtype == 0)
    hipLaunchKernelGGL(rope_kv_kernel<float>, dim3(rows_max), dim3(256), 0, s, (const float*)qkv, rows_dev, pos,
                       pos_add, rowid, kvoff, len, H, hd, r, cos_t, sin_t, (float*)q, (float*)kc, (float*)vc,
                       kv_extra);
  else if (rows_max > 2048 &&
           try_rope_tile(s, (const half_t*)qkv, rows_max, rows_dev, pos, pos_add, rowid, kvoff, len, H, hd, r, cos_t,
                         sin_t, (half_t*)q, (half_t*)kc, (half_t*)vc, kv_extra)) {
  }
  else if ((hd & 7) == 0 && r <= hd &&
           (rows_max > 2048
                ? launch_rope_vec<8>(r, dim3((rows_max + 7) / 8), s, (const half_t*)qkv, rows_max, rows_dev, pos,
                                     pos_add, rowid, kvoff, len, H, hd, cos_t, sin_t, (half_t*)q, (half_t*)kc,
                                     (half_t*)vc, kv_extra)
                : launch_rope_vec<1>(r, dim3(rows_max), s, (const half_t*)qkv, rows_max, rows_dev, pos, pos_add,
                                     rowid, kvoff, len, H, hd, cos_t, sin_t, (half_t*)q, (half_t*)kc, (half_t*)vc,
                                     kv_extra))) {
  }
  else
    hipLaunchKernelGGL(rope_kv_kernel<half_t>, dim3(rows_max), dim3(256), 0, s, (const half_t*)qkv, rows_dev,
                       pos, pos_add, rowid, kvoff, len, H, hd, r, cos_t, sin_t, (half_t*)q, (half_t*)kc, (half_t*)vc,
                       kv_extra);
  return hipGetLastError();
}

// Decode form fed by a split-K product: block (t, g) owns HPB heads of row t.  The q, k and v slices
// of those heads are formed from the fp32 partial slabs (added in slab order) plus the bias and
// rounded to fp16 exactly as the stand-alone reduction would have stored them; the rotary pairs
// are then turned in LDS and the slices copied out in 16-byte chunks.
template <int HPB>
__global__ void __launch_bounds__(256)
    rope_kv_splitk_kernel(const float* __restrict__ part, int ksplit, size_t slab, const bf16_t* __restrict__ bias,
                          const int* __restrict__ rows_dev, const int* __restrict__ pos, int pos_add,
                          const int* __restrict__ rowid, const int* __restrict__ kvoff, const int* __restrict__ len,
                          int H, int hd, int r, const float* __restrict__ cos_t, const float* __restrict__ sin_t,
                          half_t* __restrict__ q, half_t* __restrict__ kc, half_t* __restrict__ vc, long kv_extra) {
  __shared__ __attribute__((aligned(16))) half_t s_row[3 * HPB * 256];
  const int t = blockIdx.x, h0 = blockIdx.y * HPB;
  if (rows_dev && t >= *rows_dev) return;
  const int d = H * hd, q4 = hd >> 2, half = r >> 1;
  const size_t rb = ((size_t)t * 3 * d) >> 2, slab4 = slab >> 2;
  for (int c = threadIdx.x; c < 3 * HPB * q4; c += 256) {
    const int u = c / q4, j = c - u * q4;          // unit u = sec * HPB + local head
    const int sec = u / HPB, hl = u - sec * HPB;
    const int col4 = (sec * d + (h0 + hl) * hd) / 4 + j;
    f32x4_t v = sum_slabs((const f32x4_t*)part + rb + col4, slab4, ksplit);
    v += bf16x4_to_f32(((const u32x2_t*)bias)[col4]);
    f16x4_t o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = from_f32<half_t>(v[e]);
    ((f16x4_t*)s_row)[u * q4 + j] = o;
  }
  __syncthreads();
  const int p = pos[t] + pos_add;
  for (int c = threadIdx.x; c < 2 * HPB * half; c += 256) {  // q and k units only
    const int u = c / half, i = c - u * half;
    half_t* hb = s_row + u * hd;
    const float co = cos_t[(size_t)p * half + i], si = sin_t[(size_t)p * half + i];
    const float lo = (float)hb[2 * i], hi = (float)hb[2 * i + 1];
    hb[2 * i] = from_f32<half_t>(lo * co - hi * si);
    hb[2 * i + 1] = from_f32<half_t>(hi * co + lo * si);
  }
  __syncthreads();
  const int b = rowid ? rowid[t] : t;
  const long slot0 = (long)kvoff[b] * H + p, seq_len = len[b] + kv_extra;
  const int cph = hd >> 3;
  for (int c = threadIdx.x; c < 3 * HPB * cph; c += 256) {
    const int u = c / cph, ch = c - u * cph;
    const int sec = u / HPB, h = h0 + (u - sec * HPB);
    half_t* dst = sec == 0 ? q + (size_t)t * d + h * hd : (sec == 1 ? kc : vc) + (size_t)(slot0 + h * seq_len) * hd;
    *(f16x8_t*)(dst + 8 * ch) = *(const f16x8_t*)(s_row + u * hd + 8 * ch);
  }
}

bool rope_kv_splitk_supported(int dtype, int H, int hd, int r) {
  return dtype == 1 && (hd & 7) == 0 && hd <= 256 && (r & 1) == 0 && r <= hd && ((3 * H * hd) & 3) == 0;
}

hipError_t launch_rope_kv_splitk(const float* part, int ksplit, size_t slab, const void* bias, int rows_max,
                                 const int* rows_dev, const int* pos, int pos_add, const int* rowid,
                                 const int* kvoff, const int* len, int H, int hd, int r, const float* cos_t,
                                 const float* sin_t, void* q, void* kc, void* vc, long kv_extra, hipStream_t s) {
  if (rows_max <= 0) return hipSuccess;
  if (!rope_kv_splitk_supported(1, H, hd, r) || (slab & 3) != 0 || ksplit < 1) return hipErrorInvalidValue;
  if ((H & 3) == 0)
    hipLaunchKernelGGL(rope_kv_splitk_kernel<4>, dim3(rows_max, H / 4), dim3(256), 0, s, part, ksplit, slab,
                       (const bf16_t*)bias, rows_dev, pos, pos_add, rowid, kvoff, len, H, hd, r, cos_t, sin_t,
                       (half_t*)q, (half_t*)kc, (half_t*)vc, kv_extra);
  else
    hipLaunchKernelGGL(rope_kv_splitk_kernel<1>, dim3(rows_max, H), dim3(256), 0, s, part, ksplit, slab,
                       (const bf16_t*)bias, rows_dev, pos, pos_add, rowid, kvoff, len, H, hd, r, cos_t, sin_t,
                       (half_t*)q, (half_t*)kc, (half_t*)vc, kv_extra);
  return hipGetLastError();
}

// =================================================================================================
// Sampling noise: counter hash keyed (seed, sequence, step, token id) -> Gumbel variate.
// Integer part: 64-bit xor-shift-multiply finaliser, applied three times (row key, step key,
// token).  The top 32 bits k give u = (k + 1/2) / 2^32 in (0,1), g = -ln(-ln u).
// =================================================================================================
__device__ __forceinline__ uint64_t fmix64(uint64_t x) {
  x ^= x >> 30;
  x *= 0xBF58476D1CE4E5B9ull;
  x ^= x >> 27;
  x *= 0x94D049BB133111EBull;
  x ^= x >> 31;
  return x;
}
#define RLHF_GOLDEN 0x9E3779B97F4A7C15ull

__device__ __forceinline__ uint64_t noise_step_key(uint64_t seed, uint64_t seq, uint32_t step) {
  const uint64_t kr = fmix64(seed + RLHF_GOLDEN * (seq + 1));
  return fmix64(kr + RLHF_GOLDEN * (uint64_t)(step + 1));
}

__device__ __forceinline__ float gumbel_from_key(uint64_t step_key, uint32_t v) {
  const uint32_t k = (uint32_t)(fmix64(step_key + RLHF_GOLDEN * (uint64_t)(v + 1)) >> 32);
  float E;  // E = -ln u, evaluated so that u close to 1 keeps its relative accuracy
  if (k < 0x80000000u) {
    E = -logf((float)k * 2.3283064365386963e-10f + 1.1641532182693481e-10f);
  } else {
    const float c = (float)(0u - k);  // 2^32 - k, in [1, 2^31]
    E = -log1pf(-(c - 0.5f) * 2.3283064365386963e-10f);
  }
  return -logf(E);
}

// One block per row.  Single pass over the logits: running (max, sum exp) for the log-sum-exp and
// running best perturbed score; ties resolve to the lowest token id at every merge.
__global__ void __launch_bounds__(1024) sampler_kernel(SampleArgs a) {
  __shared__ float sm[16], ss[16], sb[16];
  __shared__ int si[16];
  const int b = blockIdx.x;
  const float* row = a.logits + (size_t)b * a.V;
  const uint64_t key = noise_step_key(a.seed, a.seq_base + (uint64_t)b, (uint32_t)a.step);
  float m = -INFINITY, s = 0.f, best = -INFINITY;
  int bi = 0x7FFFFFFF;
  for (int v = threadIdx.x; v < a.V; v += 1024) {
    const float z = row[v] / a.temperature;
    if (z > m) {
      s = s * expf(m - z) + 1.0f;
      m = z;
    } else {
      s += expf(z - m);
    }
    const float sc = z + gumbel_from_key(key, (uint32_t)v);
    if (sc > best) {  // v increases within a thread, so '>' keeps the lowest id among equals
      best = sc;
      bi = v;
    }
  }
  // wave merge
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float m2 = __shfl_xor(m, o, 64), s2 = __shfl_xor(s, o, 64), b2 = __shfl_xor(best, o, 64);
    const int i2 = __shfl_xor(bi, o, 64);
    const float mn = fmaxf(m, m2);
    s = (m == -INFINITY ? 0.f : s * expf(m - mn)) + (m2 == -INFINITY ? 0.f : s2 * expf(m2 - mn));
    m = mn;
    if (b2 > best || (b2 == best && i2 < bi)) {
      best = b2;
      bi = i2;
    }
  }
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
    sm[w] = m;
    ss[w] = s;
    sb[w] = best;
    si[w] = bi;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int j = 1; j < 16; ++j) {
      const float mn = fmaxf(m, sm[j]);
      s = (m == -INFINITY ? 0.f : s * expf(m - mn)) + (sm[j] == -INFINITY ? 0.f : ss[j] * expf(sm[j] - mn));
      m = mn;
      if (sb[j] > best || (sb[j] == best && si[j] < bi)) {
        best = sb[j];
        bi = si[j];
      }
    }
    // A row without a single comparable score (every logit NaN) leaves bi at its start value: stop the row
    // with EOS and a zero log-prob rather than index past the row and feed an id outside the table onwards.
    const bool none = bi < 0 || bi >= a.V;
    if (none) bi = a.eos_id;
    const float ztok = row[bi] / a.temperature;
    const float lp = none ? 0.f : ztok - (m + logf(s));
    int fin = (a.step == 0) ? (a.len[b] == 0 ? 1 : 0) : a.finished[b];
    if (a.step == 0) a.out_lengths[b] = (a.len[b] == 0) ? 0 : a.N;
    const size_t to = (size_t)b * (a.Lq + a.N) + a.Lq + a.step;
    if (a.out_mask) a.out_mask[to] = fin ? 0 : 1;
    if (fin) {
      a.out_tokens[to] = a.pad_id;
      a.out_logprobs[(size_t)b * a.N + a.step] = 0.f;
    } else {
      a.out_tokens[to] = bi;
      a.out_logprobs[(size_t)b * a.N + a.step] = lp;
      if (bi == a.eos_id) {
        fin = 1;
        a.out_lengths[b] = a.step + 1;
      }
    }
    a.finished[b] = fin;
    a.cur_tok[b] = bi;  // fed back either way; what follows EOS never reaches a kept output
  }
}

hipError_t launch_sampler(const SampleArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(sampler_kernel, dim3(a.B), dim3(1024), 0, s, a);
  return hipGetLastError();
}

__global__ void copy_queries_kernel(const int32_t* __restrict__ queries, const uint8_t* __restrict__ pad_mask,
                                    int Lq, int N, int pad_id, int32_t* __restrict__ out,
                                    uint8_t* __restrict__ out_mask) {
  const int b = blockIdx.x;
  for (int c = threadIdx.x; c < Lq + N; c += blockDim.x) {
    out[(size_t)b * (Lq + N) + c] = c < Lq ? queries[(size_t)b * Lq + c] : pad_id;
    if (out_mask) out_mask[(size_t)b * (Lq + N) + c] = c < Lq ? (pad_mask[(size_t)b * Lq + c] ? 1 : 0) : 0;
  }
}

hipError_t launch_copy_queries(const int32_t* queries, const uint8_t* pad_mask, int B, int Lq, int N, int pad_id,
                               int32_t* out_tokens, uint8_t* out_mask, hipStream_t s) {
  hipLaunchKernelGGL(copy_queries_kernel, dim3(B), dim3(256), 0, s, queries, pad_mask, Lq, N, pad_id, out_tokens,
                     out_mask);
  return hipGetLastError();
}

// =================================================================================================
// Scoring: log-sum-exp of logits/T and the target-token logit, one block per packed row.
// =================================================================================================
__global__ void __launch_bounds__(256)
    lse_gather_kernel(const float* __restrict__ logits, int t0, const int* __restrict__ T_dev, int V,
                      float temperature, const int* __restrict__ tok, const int* __restrict__ pos,
                      float* __restrict__ lp_packed) {
  __shared__ float sm[4], ss[4];
  const int t = t0 + blockIdx.x;
  const int T = *T_dev;
  if (t + 1 >= T) return;
  if (pos[t + 1] != pos[t] + 1) return;  // t is the last token of its sequence: nothing to predict
  const float* row = logits + (size_t)blockIdx.x * V;
  float m = -INFINITY, s = 0.f;
  for (int v = threadIdx.x; v < V; v += 256) {
    const float z = row[v] / temperature;
    if (z > m) {
      s = s * expf(m - z) + 1.0f;
      m = z;
    } else {
      s += expf(z - m);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float m2 = __shfl_xor(m, o, 64), s2 = __shfl_xor(s, o, 64);
    const float mn = fmaxf(m, m2);
    s = (m == -INFINITY ? 0.f : s * expf(m - mn)) + (m2 == -INFINITY ? 0.f : s2 * expf(m2 - mn));
    m = mn;
  }
  if ((threadIdx.x & 63) == 0) {
    sm[threadIdx.x >> 6] = m;
    ss[threadIdx.x >> 6] = s;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int j = 1; j < 4; ++j) {
      const float mn = fmaxf(m, sm[j]);
      s = (m == -INFINITY ? 0.f : s * expf(m - mn)) + (sm[j] == -INFINITY ? 0.f : ss[j] * expf(sm[j] - mn));
      m = mn;
    }
    const float zt = row[tok[t + 1]] / temperature;
    lp_packed[t + 1] = zt - (m + logf(s));
  }
}

hipError_t launch_lse_gather(const float* logits, int rows_max, int t0, const int* T_dev, int V,
                             float temperature, const int* tok, const int* pos, float* lp_packed,
                             hipStream_t s) {
  if (rows_max <= 0) return hipSuccess;
  hipLaunchKernelGGL(lse_gather_kernel, dim3(rows_max), dim3(256), 0, s, logits, t0, T_dev, V, temperature, tok,
                     pos, lp_packed);
  return hipGetLastError();
}

// Scoring with the fused LM head: the per-part statistics of a row are combined by four threads (one per wave of
// the block, each taking every fourth part; rows along the lanes so that the reads coalesce) and then across the
// waves through LDS, in a fixed order.
__global__ void __launch_bounds__(256)
    lse_combine_kernel(LseArgs a, int nparts, float* __restrict__ lp_packed) {
  __shared__ float sm[4][64], ss[4][64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int t = blockIdx.x * 64 + lane;
  const int T = *a.T_dev;
  const bool row = t < T;
  float m = -INFINITY, s = 0.f;
  if (row) {
    for (int p = w; p < nparts; p += 4) {  // online: rescale the running sum when the maximum moves
      const float pm = a.pmax[(size_t)p * a.stride + t];
      if (pm > -INFINITY) {
        const float ps = a.psum[(size_t)p * a.stride + t];
        const float mn = fmaxf(m, pm);
        s = s * expf(m - mn) + ps * expf(pm - mn);
        m = mn;
      }
    }
  }
  sm[w][lane] = m;
  ss[w][lane] = s;
  __syncthreads();
  if (w != 0 || !row) return;
  m = fmaxf(fmaxf(sm[0][lane], sm[1][lane]), fmaxf(sm[2][lane], sm[3][lane]));
  s = 0.f;
#pragma unroll
  for (int k = 0; k < 4; ++k)
    if (sm[k][lane] > -INFINITY) s += ss[k][lane] * expf(sm[k][lane] - m);
  if (a.tgt) {
    if (a.val_out) a.val_out[a.dst[t]] = a.val_in[t];
    if (a.tgt[t] < 0) return;
  } else {
    if (t + 1 >= T) return;
    if (a.pos[t + 1] != a.pos[t] + 1) return;  // t is the last token of its sequence: nothing to predict
  }
  lp_packed[(a.tgt ? a.dst[t] : t) + 1] = a.ztgt[t] - (m + logf(s));
}

hipError_t launch_lse_combine(const LseArgs& a, int rows_max, int nparts, float* lp_packed, hipStream_t s) {
  if (rows_max <= 0) return hipSuccess;
  hipLaunchKernelGGL(lse_combine_kernel, dim3((rows_max + 63) / 64), dim3(256), 0, s, a, nparts, lp_packed);
  return hipGetLastError();
}

__global__ void unpack_scores_kernel(const float* __restrict__ lp_packed, const float* __restrict__ val_packed,
                                     int L, const int* __restrict__ start, const int* __restrict__ len,
                                     const int* __restrict__ cu, float* __restrict__ out_lp,
                                     float* __restrict__ out_val, const float* __restrict__ val_bias_dev,
                                     int first_col) {
  const int b = blockIdx.y;
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= L) return;
  const int i = c - start[b];
  const bool real = i >= 0 && i < len[b];
  const size_t o = (size_t)b * L + c;
  out_lp[o] = (real && i >= 1 && c >= first_col) ? lp_packed[cu[b] + i] : 0.f;
  if (out_val)
    out_val[o] = (real && c >= first_col - 1) ? val_packed[cu[b] + i] + (val_bias_dev ? *val_bias_dev : 0.f) : 0.f;
}

hipError_t launch_unpack_scores(const float* lp_packed, const float* val_packed, int B, int L, const int* start,
                                const int* len, const int* cu, float* out_lp, float* out_val, hipStream_t s,
                                const float* val_bias_dev, int first_col) {
  hipLaunchKernelGGL(unpack_scores_kernel, dim3((L + 255) / 256, B), dim3(256), 0, s, lp_packed, val_packed, L,
                     start, len, cu, out_lp, out_val, val_bias_dev, first_col);
  return hipGetLastError();
}

// The packed rows from padded column first_col - 1 on, sequence by sequence (see common.h).  One block: a
// block-wide prefix sum over the sequences' counts (1024 sequences at a time) gives the offsets, then each wave
// fills the entries of every 16th sequence.
__global__ void __launch_bounds__(1024)
    select_rows_kernel(int first_col, int B, const int* __restrict__ start, const int* __restrict__ len,
                       const int* __restrict__ cu, const int* __restrict__ tok, int rows_max, int* __restrict__ sel,
                       int* __restrict__ tgt, int* __restrict__ n_sel, int* __restrict__ off) {
  __shared__ int sc[1024];
  __shared__ int carry;
  const int tid = threadIdx.x;
  if (tid == 0) carry = 0;
  __syncthreads();
  for (int base = 0; base < B; base += 1024) {
    const int b = base + tid;
    int cnt = 0;
    if (b < B) cnt = len[b] - min(max(first_col - 1 - start[b], 0), len[b]);
    sc[tid] = cnt;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
      const int v = tid >= o ? sc[tid - o] : 0;
      __syncthreads();
      sc[tid] += v;
      __syncthreads();
    }
    if (b < B) off[b] = carry + sc[tid] - cnt;
    __syncthreads();
    if (tid == 1023) carry += sc[1023];
    __syncthreads();
  }
  const int total = min(carry, rows_max);
  if (tid == 0) {
    off[B] = carry;
    *n_sel = total;
  }
  const int wave = tid >> 6, lane = tid & 63;
  for (int b = wave; b < B; b += 16) {
    const int i0 = min(max(first_col - 1 - start[b], 0), len[b]);
    const int cnt = len[b] - i0, o = off[b];
    for (int k = lane; k < cnt && o + k < rows_max; k += 64) {
      const int t = cu[b] + i0 + k;
      sel[o + k] = t;
      tgt[o + k] = k + 1 < cnt ? tok[t + 1] : -1;
    }
  }
  for (int j = total + tid; j < rows_max; j += 1024) {
    sel[j] = 0;
    tgt[j] = -1;
  }
}

hipError_t launch_select_rows(int first_col, int B, const int* start, const int* len, const int* cu, const int* tok,
                              int rows_max, int* sel, int* tgt, int* n_sel, int* off, hipStream_t s) {
  hipLaunchKernelGGL(select_rows_kernel, dim3(1), dim3(1024), 0, s, first_col, B, start, len, cu, tok, rows_max, sel,
                     tgt, n_sel, off);
  return hipGetLastError();
}

__global__ void __launch_bounds__(256)
    gather_rows_strided_kernel(const u32x4_t* __restrict__ in, size_t in_chunks, const int* __restrict__ src,
                               int chunks, u32x4_t* __restrict__ out, size_t out_chunks) {
  const size_t sr = (size_t)max(src[blockIdx.x], 0);
  for (int c = threadIdx.x; c < chunks; c += 256) out[(size_t)blockIdx.x * out_chunks + c] = in[sr * in_chunks + c];
}

hipError_t launch_gather_rows_strided(const void* in, size_t in_stride, const int* src, int rows, size_t row_bytes,
                                      void* out, size_t out_stride, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (((row_bytes | in_stride | out_stride) & 15) != 0 || row_bytes / 16 > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(gather_rows_strided_kernel, dim3(rows), dim3(256), 0, s, (const u32x4_t*)in, in_stride / 16, src,
                     (int)(row_bytes / 16), (u32x4_t*)out, out_stride / 16);
  return hipGetLastError();
}

// Per-row scalars of the selected rows (a target id and two gradients); entries past *n_sel get (-1, 0, 0).
__global__ void gather_row_scalars_kernel(const int* __restrict__ sel, const int* __restrict__ n_sel, int rows,
                                          const int* __restrict__ tgt, const float* __restrict__ a,
                                          const float* __restrict__ b, int* __restrict__ tgt_out,
                                          float* __restrict__ a_out, float* __restrict__ b_out) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= rows) return;
  const bool ok = j < *n_sel;
  const int t = ok ? sel[j] : 0;
  tgt_out[j] = ok ? tgt[t] : -1;
  a_out[j] = ok ? a[t] : 0.f;
  if (b_out) b_out[j] = ok && b ? b[t] : 0.f;
}

hipError_t launch_gather_row_scalars(const int* sel, const int* n_sel, int rows, const int* tgt, const float* a,
                                     const float* b, int* tgt_out, float* a_out, float* b_out, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(gather_row_scalars_kernel, dim3((rows + 255) / 256), dim3(256), 0, s, sel, n_sel, rows, tgt, a, b,
                     tgt_out, a_out, b_out);
  return hipGetLastError();
}

// out row sel[j] = in row j for j < *n_sel (rows of `chunks` 16-byte pieces); the selected rows are distinct.
__global__ void __launch_bounds__(256)
    scatter_rows_kernel(const u32x4_t* __restrict__ in, const int* __restrict__ sel, const int* __restrict__ n_sel,
                        int chunks, u32x4_t* __restrict__ out) {
  if ((int)blockIdx.x >= *n_sel) return;
  const size_t dr = (size_t)max(sel[blockIdx.x], 0);
  for (int c = threadIdx.x; c < chunks; c += 256) out[dr * chunks + c] = in[(size_t)blockIdx.x * chunks + c];
}

hipError_t launch_scatter_rows(const void* in, const int* sel, const int* n_sel, int rows, size_t row_bytes, void* out,
                               hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if ((row_bytes & 15) != 0 || row_bytes / 16 > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(scatter_rows_kernel, dim3(rows), dim3(256), 0, s, (const u32x4_t*)in, sel, n_sel,
                     (int)(row_bytes / 16), (u32x4_t*)out);
  return hipGetLastError();
}

__global__ void rows_to_packed_kernel(const int32_t* __restrict__ rows_bt, int n, const int* __restrict__ start,
                                      const int* __restrict__ cu, int* __restrict__ idx) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int b = rows_bt[2 * i], c = rows_bt[2 * i + 1];
  idx[i] = cu[b] + (c - start[b]);
}

hipError_t launch_rows_to_packed(const int32_t* rows_bt, int n, const int* start, const int* cu, int* idx,
                                 hipStream_t s) {
  hipLaunchKernelGGL(rows_to_packed_kernel, dim3((n + 63) / 64), dim3(64), 0, s, rows_bt, n, start, cu, idx);
  return hipGetLastError();
}

// =================================================================================================
// One-time weight conversion bf16 -> fp16.
// =================================================================================================
__global__ void bf16_to_f16_kernel(const bf16_t* __restrict__ src, half_t* __restrict__ dst, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = (half_t)to_f32(src[i]);
}

hipError_t launch_bf16_to_f16(const void* src, void* dst, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const int blocks = (int)std::min<size_t>((n + 255) / 256, 65536);
  hipLaunchKernelGGL(bf16_to_f16_kernel, dim3(blocks), dim3(256), 0, s, (const bf16_t*)src, (half_t*)dst, n);
  return hipGetLastError();
}

__global__ void bf16_to_f16_2d_kernel(const bf16_t* __restrict__ src, half_t* __restrict__ dst, size_t rows,
                                      size_t cols, size_t dst_ld) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x, n = rows * cols;
  for (; i < n; i += stride) {
    const size_t r = i / cols, c = i - r * cols;
    dst[r * dst_ld + c] = (half_t)to_f32(src[i]);
  }
}

hipError_t launch_bf16_to_f16_2d(const void* src, void* dst, size_t rows, size_t cols, size_t dst_ld,
                                 hipStream_t s) {
  if (rows * cols == 0) return hipSuccess;
  const int blocks = (int)std::min<size_t>((rows * cols + 255) / 256, 65536);
  hipLaunchKernelGGL(bf16_to_f16_2d_kernel, dim3(blocks), dim3(256), 0, s, (const bf16_t*)src, (half_t*)dst, rows,
                     cols, dst_ld);
  return hipGetLastError();
}

// W_qkv and its bias for the fp16 path: [q | k | v] sections of H heads.  Inside every q and k head
// the rotary dims are reordered so that the pair (i, i + r/2) sits at (2i, 2i + 1); q.k is unchanged
// by a reordering common to both, and neighbours can be turned by whoever holds two adjacent
// columns (a GEMM epilogue lane) without any exchange.  One block per output row.
__global__ void __launch_bounds__(256)
    qkv_weights_f16_kernel(const bf16_t* __restrict__ w, const bf16_t* __restrict__ b, half_t* __restrict__ w16,
                           bf16_t* __restrict__ b_out, int d, int hd, int r) {
  const int n = blockIdx.x;  // destination row, 0 .. 3d-1
  const int sec = n / d, e = (n - sec * d) % hd;
  int src = n;
  if (sec < 2 && e < r) src = n - e + ((e & 1) ? (e >> 1) + (r >> 1) : (e >> 1));
  for (int c = threadIdx.x; c < d; c += 256) w16[(size_t)n * d + c] = (half_t)to_f32(w[(size_t)src * d + c]);
  if (threadIdx.x == 0) b_out[n] = b[src];
}

hipError_t launch_qkv_weights_f16(const void* w, const void* b, void* w16, void* b_out, int d, int hd, int r,
                                  hipStream_t s) {
  hipLaunchKernelGGL(qkv_weights_f16_kernel, dim3(3 * d), dim3(256), 0, s, (const bf16_t*)w, (const bf16_t*)b,
                     (half_t*)w16, (bf16_t*)b_out, d, hd, r);
  return hipGetLastError();
}

}  // namespace rlhf
