// Backward pass through the output heads (final LayerNorm, LM head with temperature, value head):
// the element-wise and reduction kernels around the three matrix products, which run on the
// library's GEMM kernels.  Sums over rows are taken in a fixed order (no floating-point atomics).
#include <algorithm>

#include "common.h"

namespace rlhf {

namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

__device__ __forceinline__ float block_sum(float v, float* sh) {  // 256 threads; sh: 4 floats
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  return (sh[0] + sh[1]) + (sh[2] + sh[3]);
}
__device__ __forceinline__ float block_max(float v, float* sh) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
}

// dst[c][r] = src[r][c] for r < R, c < C; dst columns R .. R_pad-1 are zeroed.  32 x 32 tiles.
template <typename T>
__global__ void __launch_bounds__(256)
    transpose_pad_kernel(const T* __restrict__ src, size_t ld_src, T* __restrict__ dst, size_t ld_dst, int R, int C,
                         int R_pad) {
  __shared__ T tile[32][33];
  const int r0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = r0 + ty + 8 * i, c = c0 + tx;
    T v = from_f32<T>(0.f);
    if (r < R && c < C) v = src[(size_t)r * ld_src + c];
    tile[ty + 8 * i][tx] = v;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = c0 + ty + 8 * i, r = r0 + tx;
    if (c < C && r < R_pad) dst[(size_t)c * ld_dst + r] = tile[tx][ty + 8 * i];
  }
}

// fp16 form with 8-byte accesses: 64 x 64 tiles, a thread moves 4 consecutive halfs on both sides.
// Needs ld_src, ld_dst multiples of 4, and R_pad, C multiples of 4 (so every quad is inside or outside as a whole); src
// rows R .. R_pad-1 are not read (the destination gets zeros there).
__global__ void __launch_bounds__(256)
    transpose_pad_f16x4_kernel(const half_t* __restrict__ src, size_t ld_src, half_t* __restrict__ dst, size_t ld_dst,
                               int R, int C, int R_pad) {
  __shared__ half_t tile[64][64 + 4];
  const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
  const int tq = threadIdx.x & 15, tr = threadIdx.x >> 4;  // quad within a row of the tile, row within a pass
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = r0 + tr + 16 * i, c = c0 + 4 * tq;
    f16x4_t v = {0, 0, 0, 0};
    if (r < R && c < C) v = *(const f16x4_t*)(src + (size_t)r * ld_src + c);
    *(f16x4_t*)&tile[tr + 16 * i][4 * tq] = v;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = c0 + tr + 16 * i, r = r0 + 4 * tq;
    if (c < C && r < R_pad) {
      const f16x4_t v = {tile[4 * tq][tr + 16 * i], tile[4 * tq + 1][tr + 16 * i], tile[4 * tq + 2][tr + 16 * i],
                         tile[4 * tq + 3][tr + 16 * i]};
      *(f16x4_t*)(dst + (size_t)c * ld_dst + r) = v;
    }
  }
}

// fp16 form with 16-byte accesses on both sides: 64 x 64 tiles, a thread moves 8 consecutive halfs.
// Needs ld_src, ld_dst, R_pad and C multiples of 8 and 16-byte aligned bases.  The LDS row stride of
// 66 halfs (33 words) spreads the 8 rows a thread gathers over different banks.
__global__ void __launch_bounds__(256)
    transpose_pad_f16x8_kernel(const half_t* __restrict__ src, size_t ld_src, half_t* __restrict__ dst, size_t ld_dst,
                               int R, int C, int R_pad) {
  __shared__ uint32_t tile[64 * 33];
  const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
  const int to = threadIdx.x & 7, tr = threadIdx.x >> 3;  // octet within a tile row, row within a pass
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int r = r0 + tr + 32 * i, c = c0 + 8 * to;
    u32x4_t v = {0, 0, 0, 0};
    if (r < R && c < C) v = *(const u32x4_t*)(src + (size_t)r * ld_src + c);
    uint32_t* t = tile + (tr + 32 * i) * 33 + 4 * to;
    t[0] = v[0]; t[1] = v[1]; t[2] = v[2]; t[3] = v[3];
  }
  __syncthreads();
  const uint16_t* th = (const uint16_t*)tile;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int cl = tr + 32 * i, c = c0 + cl, r = r0 + 8 * to;
    if (c < C && r < R_pad) {
      u32x4_t v;
#pragma unroll
      for (int k = 0; k < 4; ++k)
        v[k] = (uint32_t)th[(8 * to + 2 * k) * 66 + cl] | ((uint32_t)th[(8 * to + 2 * k + 1) * 66 + cl] << 16);
      *(u32x4_t*)(dst + (size_t)c * ld_dst + r) = v;
    }
  }
}

template <typename T>
__global__ void __launch_bounds__(256) fill_zero_kernel(T* __restrict__ p, size_t n) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n; i += stride) p[i] = from_f32<T>(0.f);
}

// Row r of a chunk: dz[r][v] = gl[r] * scale / T * (onehot(y_r)[v] - softmax(logits[r] / T)[v]);
// rows past `rows` (padding), rows without a target and columns V .. V_pad-1 are zero.
// One block of 1024 threads per row; the row is read once and kept in registers (up to NPT values
// per thread, i.e. vocabularies up to 1024 * NPT), longer rows are re-read from memory.
constexpr int SG_THREADS = 1024, SG_NPT = 64;
__device__ __forceinline__ float block_sum_1024(float v, float* sh) {  // sh: 16 floats
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) t += sh[i];
  return t;
}
__device__ __forceinline__ float block_max_1024(float v, float* sh) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = sh[0];
#pragma unroll
  for (int i = 1; i < 16; ++i) t = fmaxf(t, sh[i]);
  return t;
}
// store 4 consecutive values of type T (16 or 8 bytes)
__device__ __forceinline__ void store4(float* p, float a, float b, float c, float d) {
  *(f32x4_t*)p = (f32x4_t){a, b, c, d};
}
__device__ __forceinline__ void store4(half_t* p, float a, float b, float c, float d) {
  *(f16x4_t*)p = (f16x4_t){from_f32<half_t>(a), from_f32<half_t>(b), from_f32<half_t>(c), from_f32<half_t>(d)};
}
// MODE 0: rows re-read from memory, any V.  MODE 1: the row is read once, 4 consecutive values per
// access (V a multiple of 4 -- rows are then 16-byte aligned -- and at most 4 * 1024 * NQ values).
template <typename T, int MODE>
__global__ void __launch_bounds__(SG_THREADS)
    softmax_grad_kernel(const float* __restrict__ logits, int V, int V_pad, const int* __restrict__ targets,
                        const float* __restrict__ gl, int rows, float inv_temp, float scale, T* __restrict__ dz) {
  constexpr int NQ = SG_NPT / 4;  // quads per thread
  __shared__ float sh[16];
  const int r = blockIdx.x;
  T* out = dz + (size_t)r * V_pad;
  const int y = r < rows ? targets[r] : -1;
  if (y < 0 || y >= V) {  // block-uniform
    for (int v = threadIdx.x; v < V_pad; v += SG_THREADS) out[v] = from_f32<T>(0.f);
    return;
  }
  const float* z = logits + (size_t)r * V;
  f32x4_t zr[MODE == 1 ? NQ : 1];
  float mx = -INFINITY;
  if (MODE == 1) {
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
      const int v = 4 * (threadIdx.x + i * SG_THREADS);
      zr[i] = (f32x4_t){-INFINITY, -INFINITY, -INFINITY, -INFINITY};
      if (v < V) zr[i] = *(const f32x4_t*)(z + v) * inv_temp;
      mx = fmaxf(fmaxf(mx, fmaxf(zr[i][0], zr[i][1])), fmaxf(zr[i][2], zr[i][3]));
    }
  } else {
    for (int v = threadIdx.x; v < V; v += SG_THREADS) mx = fmaxf(mx, z[v] * inv_temp);
  }
  mx = block_max_1024(mx, sh);
  float sum = 0.f;
  if (MODE == 1) {
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        zr[i][u] = __expf(zr[i][u] - mx);  // exp(-inf) = 0 past the end of the row
        sum += zr[i][u];
      }
    }
  } else {
    for (int v = threadIdx.x; v < V; v += SG_THREADS) sum += __expf(z[v] * inv_temp - mx);
  }
  sum = block_sum_1024(sum, sh);
  const float c = gl[r] * scale * inv_temp, ci = -c / sum;
  if (MODE == 1) {
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
      const int v = 4 * (threadIdx.x + i * SG_THREADS);
      if (v < V) {
        float o[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) o[u] = zr[i][u] * ci + (v + u == y ? c : 0.f);
        store4(out + v, o[0], o[1], o[2], o[3]);
      } else if (v < V_pad) {  // V_pad - V < 8 and both are multiples of 4: one quad at most
        store4(out + v, 0.f, 0.f, 0.f, 0.f);
      }
    }
  } else {
    for (int v = threadIdx.x; v < V_pad; v += SG_THREADS) {
      float g = 0.f;
      if (v < V) g = __expf(z[v] * inv_temp - mx) * ci + (v == y ? c : 0.f);
      out[v] = from_f32<T>(g);
    }
  }
}

// One block per row: statistics of x, dy = dhl + gv * scale * w_v, and the LayerNorm input gradient
//   dx = rstd * (u - mean(u) - xh * mean(u * xh)),  u = dy * g,  xh = (x - mean) * rstd.
// mean and rstd are kept for the column sums.
template <typename W>
__global__ void __launch_bounds__(256)
    ln_backward_kernel(const float* __restrict__ x, const float* __restrict__ dhl, const float* __restrict__ gv,
                       float scale, const W* __restrict__ value_w, const W* __restrict__ g, int d, float eps,
                       float* __restrict__ dx, float* __restrict__ stats) {
  __shared__ float sh[4];
  const size_t t = blockIdx.x;
  const float* xr = x + t * d;
  const float* dr = dhl + t * d;
  float s = 0.f;
  for (int c = threadIdx.x; c < d; c += 256) s += xr[c];
  const float mean = block_sum(s, sh) / (float)d;
  float q = 0.f;
  for (int c = threadIdx.x; c < d; c += 256) {
    const float e = xr[c] - mean;
    q += e * e;
  }
  const float rstd = 1.0f / sqrtf(block_sum(q, sh) / (float)d + eps);
  const float gvt = value_w ? gv[t] * scale : 0.f;
  float su = 0.f, sux = 0.f;
  for (int c = threadIdx.x; c < d; c += 256) {
    const float dy = dr[c] + (value_w ? gvt * to_f32(value_w[c]) : 0.f);
    const float u = dy * to_f32(g[c]), xh = (xr[c] - mean) * rstd;
    su += u;
    sux += u * xh;
  }
  const float mu = block_sum(su, sh) / (float)d;
  const float mux = block_sum(sux, sh) / (float)d;
  for (int c = threadIdx.x; c < d; c += 256) {
    const float dy = dr[c] + (value_w ? gvt * to_f32(value_w[c]) : 0.f);
    const float u = dy * to_f32(g[c]), xh = (xr[c] - mean) * rstd;
    dx[t * d + c] = rstd * (u - mu - xh * mux);
  }
  if (threadIdx.x == 0) {
    stats[2 * t] = mean;
    stats[2 * t + 1] = rstd;
  }
}

// The layers' LayerNorm backward in one pass over the data: a wave owns a run of consecutive rows, holds a row of x
// and of dy in registers (NV float4 per lane, d = 256 * NV), forms the row's statistics and dx, and keeps the column
// sums sum dy * xh and sum dy of its rows in registers; they go to part [waves][2][d], which
// ln_backward_rows_final_kernel adds in wave order.  x, dy read once, dx written once.
template <int NV>
__global__ void __launch_bounds__(256)
    ln_backward_rows_kernel(const float* __restrict__ x, const float* __restrict__ dyp, const bf16_t* __restrict__ g,
                            int T, float eps, float* __restrict__ dx, float* __restrict__ part, int rows_per_wave,
                            const float* __restrict__ base) {
  constexpr int d = 256 * NV;
  const int lane = threadIdx.x & 63;
  const int gw = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int t0 = gw * rows_per_wave, t1 = min(T, t0 + rows_per_wave);
  f32x4_t sg[NV], sb[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    sg[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    sb[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  }
  for (int t = t0; t < t1; ++t) {
    const f32x4_t* xr = (const f32x4_t*)(x + (size_t)t * d);
    const f32x4_t* dr = (const f32x4_t*)(dyp + (size_t)t * d);
    f32x4_t xv[NV], dv[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      xv[j] = xr[lane + 64 * j];
      dv[j] = dr[lane + 64 * j];
    }
    float a = 0.f;
#pragma unroll
    for (int j = 0; j < NV; ++j) a += (xv[j][0] + xv[j][1]) + (xv[j][2] + xv[j][3]);
    const float mean = wave_sum(a) / (float)d;
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < NV; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        xv[j][e] -= mean;
        q += xv[j][e] * xv[j][e];
      }
    const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)d + eps);
    float su = 0.f, sux = 0.f;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const u32x2_t gb = *(const u32x2_t*)(g + 4 * (lane + 64 * j));
      const float gf[4] = {__uint_as_float(gb[0] << 16), __uint_as_float(gb[0] & 0xFFFF0000u),
                           __uint_as_float(gb[1] << 16), __uint_as_float(gb[1] & 0xFFFF0000u)};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        xv[j][e] *= rstd;  // xh
        sg[j][e] += dv[j][e] * xv[j][e];
        sb[j][e] += dv[j][e];
        dv[j][e] *= gf[e];  // u = dy * g, in place: dy itself is not needed again
        su += dv[j][e];
        sux += dv[j][e] * xv[j][e];
      }
    }
    const float mu = wave_sum(su) / (float)d, mux = wave_sum(sux) / (float)d;
    f32x4_t* o = (f32x4_t*)(dx + (size_t)t * d);
    const f32x4_t* bs = base ? (const f32x4_t*)(base + (size_t)t * d) : nullptr;  // dx = base + this term
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      f32x4_t r;
#pragma unroll
      for (int e = 0; e < 4; ++e) r[e] = rstd * (dv[j][e] - mu - xv[j][e] * mux);
      if (bs) r += bs[lane + 64 * j];
      o[lane + 64 * j] = r;
    }
  }
  f32x4_t* p = (f32x4_t*)(part + (size_t)gw * 2 * d);
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    p[lane + 64 * j] = sg[j];
    p[d / 4 + lane + 64 * j] = sb[j];
  }
}

__global__ void __launch_bounds__(256)
    ln_backward_rows_final_kernel(const float* __restrict__ part, int waves, int d, float* __restrict__ d_g,
                                  float* __restrict__ d_b) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= 2 * d) return;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;  // four interleaved chains, added at the end: a fixed order
  int w = 0;
  for (; w + 4 <= waves; w += 4) {
    s0 += part[(size_t)w * 2 * d + c];
    s1 += part[(size_t)(w + 1) * 2 * d + c];
    s2 += part[(size_t)(w + 2) * 2 * d + c];
    s3 += part[(size_t)(w + 3) * 2 * d + c];
  }
  for (; w < waves; ++w) s0 += part[(size_t)w * 2 * d + c];
  const float r = (s0 + s1) + (s2 + s3);
  if (c < d) d_g[c] = r;
  else d_b[c - d] = r;
}

// Column sums over a range of rows: block (column block, row split) leaves, for each of its 256
// columns, sum dy * xh, sum dy and sum gv * h over its rows (h = the final LayerNorm's output in the
// activation type A, as the forward pass produces it).  part: [splits][3][d].
template <typename W, typename A>
__global__ void __launch_bounds__(256)
    head_colsum_kernel(const float* __restrict__ x, const float* __restrict__ dhl, const float* __restrict__ gv,
                       float scale, const W* __restrict__ value_w, const W* __restrict__ g, const W* __restrict__ b,
                       const float* __restrict__ stats, int T, int d, int rows_per_split, float* __restrict__ part) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  const int t0 = blockIdx.y * rows_per_split, t1 = min(T, t0 + rows_per_split);
  if (c >= d) return;
  const float gc = to_f32(g[c]), bc = to_f32(b[c]), wv = value_w ? to_f32(value_w[c]) : 0.f;
  float sg = 0.f, sb = 0.f, sw = 0.f;
  for (int t = t0; t < t1; ++t) {
    const float gvt = value_w ? gv[t] * scale : 0.f;
    const float dy = dhl[(size_t)t * d + c] + gvt * wv;
    const float xh = (x[(size_t)t * d + c] - stats[2 * t]) * stats[2 * t + 1];
    sg += dy * xh;
    sb += dy;
    sw += gvt * to_f32(from_f32<A>(xh * gc + bc));
  }
  float* p = part + (size_t)blockIdx.y * 3 * d;
  p[c] = sg;
  p[d + c] = sb;
  p[2 * d + c] = sw;
}

// Adds the row splits in index order; thread block 0 also sums gv over all rows (fixed order:
// per-thread strided partial sums, then the block tree).
__global__ void __launch_bounds__(256)
    head_colsum_final_kernel(const float* __restrict__ part, int splits, int d, const float* __restrict__ gv,
                             float scale, int T, float* __restrict__ d_g, float* __restrict__ d_b,
                             float* __restrict__ d_wv, float* __restrict__ d_bv) {
  __shared__ float sh[4];
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c < d) {
    float sg = 0.f, sb = 0.f, sw = 0.f;
    for (int z = 0; z < splits; ++z) {
      const float* p = part + (size_t)z * 3 * d;
      sg += p[c];
      sb += p[d + c];
      sw += p[2 * d + c];
    }
    d_g[c] = sg;
    d_b[c] = sb;
    if (d_wv) d_wv[c] = sw;
  }
  if (blockIdx.x == 0 && d_bv) {
    float s = 0.f;
    for (int t = threadIdx.x; t < T; t += 256) s += gv[t];
    s = block_sum(s, sh);
    if (threadIdx.x == 0) *d_bv = s * scale;
  }
}

// f = gelu(u) (exact erf form), element-wise.
template <typename T>
__global__ void __launch_bounds__(256) gelu_kernel(const T* __restrict__ u, T* __restrict__ f, size_t n) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n; i += stride) {
    const float x = to_f32(u[i]);
    f[i] = from_f32<T>(0.5f * x * (1.0f + erff(x * 0.70710678118654752f)));
  }
}
// du = df * gelu'(u), gelu'(u) = Phi(u) + u * phi(u); in place on df.
template <typename T>
__global__ void __launch_bounds__(256) gelu_backward_kernel(const T* __restrict__ u, T* __restrict__ df, size_t n) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n; i += stride) {
    const float x = to_f32(u[i]);
    const float Phi = 0.5f * (1.0f + erff(x * 0.70710678118654752f));
    const float phi = 0.3989422804014327f * __expf(-0.5f * x * x);
    df[i] = from_f32<T>(to_f32(df[i]) * (Phi + x * phi));
  }
}
// fp16 forms, 8 values per access.  Phi(x) ~ 1 / (1 + exp(-x (c1 + c3 x^2 + c5 x^4))) with the coefficients
// the forward pass's fp16 GELU epilogue uses (absolute error below 2.6e-5, under fp16's own rounding).
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
__device__ __forceinline__ float phi_cdf_fast(float x) {
  const float s = fminf(x * x, 64.0f);
  float p = fmaf(1.01426504e-3f, s, -1.06775735e-1f);
  p = fmaf(p, s, -2.30112140f);
  return __frcp_rn(1.0f + __builtin_amdgcn_exp2f(x * p));
}
__global__ void __launch_bounds__(256)
    gelu_f16x8_kernel(const half_t* __restrict__ u, half_t* __restrict__ f, size_t n8) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n8; i += stride) {
    const f16x8_t v = ((const f16x8_t*)u)[i];
    f16x8_t o;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float x = (float)v[e];
      o[e] = from_f32<half_t>(x * phi_cdf_fast(x));
    }
    ((f16x8_t*)f)[i] = o;
  }
}
__global__ void __launch_bounds__(256)
    gelu_backward_f16x8_kernel(const half_t* __restrict__ u, half_t* __restrict__ df, size_t n8) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n8; i += stride) {
    const f16x8_t v = ((const f16x8_t*)u)[i];
    f16x8_t g = ((const f16x8_t*)df)[i];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float x = (float)v[e];
      const float phi = 0.3989422804014327f * __builtin_amdgcn_exp2f(-0.72134752044448170f * x * x);
      g[e] = from_f32<half_t>((float)g[e] * (phi_cdf_fast(x) + x * phi));
    }
    ((f16x8_t*)df)[i] = g;
  }
}
// df *= gelu'(u) on a [R, C] fp16 matrix and, in the same pass, the column sums of the result (of the rounded values,
// as a separate pass over the stored matrix would see them): part [splits][C], rows added in increasing order.
__global__ void __launch_bounds__(256)
    gelu_backward_colsum_kernel(const half_t* __restrict__ u, half_t* __restrict__ df, int R, int C, int rows_per_split,
                                float* __restrict__ part) {
  const int c0 = (blockIdx.x * 256 + threadIdx.x) * 8;
  if (c0 >= C) return;
  const int r0 = blockIdx.y * rows_per_split, r1 = min(R, r0 + rows_per_split);
  float s[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) s[i] = 0.f;
  for (int r = r0; r < r1; r += 2) {
    f16x8_t v[2], g[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const size_t o = (size_t)min(r + k, r1 - 1) * C + c0;
      v[k] = *(const f16x8_t*)(u + o);
      g[k] = *(const f16x8_t*)(df + o);
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      if (r + k < r1) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float x = (float)v[k][e];
          const float phi = 0.3989422804014327f * __builtin_amdgcn_exp2f(-0.72134752044448170f * x * x);
          g[k][e] = from_f32<half_t>((float)g[k][e] * (phi_cdf_fast(x) + x * phi));
          s[e] += (float)g[k][e];
        }
        *(f16x8_t*)(df + (size_t)(r + k) * C + c0) = g[k];
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) part[(size_t)blockIdx.y * C + c0 + i] = s[i];
}
template <typename T>
__global__ void __launch_bounds__(256) convert_kernel(const float* __restrict__ src, T* __restrict__ dst, size_t n) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n; i += stride) dst[i] = from_f32<T>(src[i]);
}
// Column sums of a [R, C] matrix in two stages with a fixed order: block (column block, row split)
// sums its rows for 256 columns into part [splits][C]; the second kernel adds the splits.
template <typename T>
__global__ void __launch_bounds__(256)
    colsum_part_kernel(const T* __restrict__ a, int R, int C, int rows_per_split, float* __restrict__ part) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C) return;
  const int r0 = blockIdx.y * rows_per_split, r1 = min(R, r0 + rows_per_split);
  float s = 0.f;
  for (int r = r0; r < r1; ++r) s += to_f32(a[(size_t)r * C + c]);
  part[(size_t)blockIdx.y * C + c] = s;
}
// The same with 16-byte accesses: a thread owns 16 bytes' worth of neighbouring columns (4 floats or 8 halfs) and
// keeps four rows' loads in flight; rows are still added in increasing order.
template <typename T>
__global__ void __launch_bounds__(256)
    colsum_part_vec_kernel(const T* __restrict__ a, int R, int C, int rows_per_split, float* __restrict__ part) {
  constexpr int V = 16 / sizeof(T);
  const int c0 = (blockIdx.x * 256 + threadIdx.x) * V;
  if (c0 >= C) return;
  const int r0 = blockIdx.y * rows_per_split, r1 = min(R, r0 + rows_per_split);
  float s[V];
#pragma unroll
  for (int i = 0; i < V; ++i) s[i] = 0.f;
  const u32x4_t zero = {0u, 0u, 0u, 0u};
  for (int r = r0; r < r1; r += 4) {
    u32x4_t v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = r + k < r1 ? *(const u32x4_t*)(a + (size_t)(r + k) * C + c0) : zero;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const T* e = (const T*)&v[k];
#pragma unroll
      for (int i = 0; i < V; ++i) s[i] += to_f32(e[i]);
    }
  }
#pragma unroll
  for (int i = 0; i < V; ++i) part[(size_t)blockIdx.y * C + c0 + i] = s[i];
}
// Column sums of a float [R, C] matrix as above and, in the same pass, its fp16 copy.
__global__ void __launch_bounds__(256)
    convert_colsum_part_kernel(const float* __restrict__ a, int R, int C, int rows_per_split, float* __restrict__ part,
                               half_t* __restrict__ out) {
  const int c0 = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (c0 >= C) return;
  const int r0 = blockIdx.y * rows_per_split, r1 = min(R, r0 + rows_per_split);
  f32x4_t s = {0.f, 0.f, 0.f, 0.f};
  for (int r = r0; r < r1; r += 4) {
    f32x4_t v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
      v[k] = r + k < r1 ? *(const f32x4_t*)(a + (size_t)(r + k) * C + c0) : f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      s += v[k];
      if (r + k < r1) {
        const f16x4_t hv = {from_f32<half_t>(v[k][0]), from_f32<half_t>(v[k][1]), from_f32<half_t>(v[k][2]),
                            from_f32<half_t>(v[k][3])};
        *(f16x4_t*)(out + (size_t)(r + k) * C + c0) = hv;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) part[(size_t)blockIdx.y * C + c0 + i] = s[i];
}
__global__ void __launch_bounds__(256)
    colsum_final_kernel(const float* __restrict__ part, int splits, int C, float* __restrict__ out) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C) return;
  float s = 0.f;
  for (int z = 0; z < splits; ++z) s += part[(size_t)z * C + c];
  out[c] = s;
}

// Gradient of the input embedding: out[v][:] = sum over packed rows t with tok[t] == v of dx[t][:], rows added
// in increasing t (a fixed order: no atomics).  One block per vocabulary entry scans the token list 256 rows at a
// time; a thread keeps up to 32 columns (d <= 8192) in registers.
__global__ void __launch_bounds__(256)
    embed_backward_kernel(const int* __restrict__ tok, const float* __restrict__ dx, int T, int d,
                          float* __restrict__ out) {
  __shared__ int hits[256];
  const int v = blockIdx.x, tid = threadIdx.x;
  float acc[32];
#pragma unroll
  for (int i = 0; i < 32; ++i) acc[i] = 0.f;
  for (int t0 = 0; t0 < T; t0 += 256) {
    const int t = t0 + tid;
    const int match = (t < T && tok[t] == v) ? 1 : 0;
    if (__syncthreads_or(match)) {
      hits[tid] = match;
      __syncthreads();
      for (int i = 0; i < 256; ++i) {
        if (!hits[i]) continue;
        const float* row = dx + (size_t)(t0 + i) * d;
#pragma unroll
        for (int u = 0; u < 32; ++u) {
          const int c = tid + 256 * u;
          if (c < d) acc[u] += row[c];
        }
      }
      __syncthreads();
    }
  }
#pragma unroll
  for (int u = 0; u < 32; ++u) {
    const int c = tid + 256 * u;
    if (c < d) out[(size_t)v * d + c] = acc[u];
  }
}

__global__ void __launch_bounds__(256)
    add3_kernel(const float* __restrict__ a, const float* __restrict__ b, const float* __restrict__ c,
                float* __restrict__ out, size_t n) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n; i += stride) out[i] = (a[i] + b[i]) + c[i];
}

}  // namespace

hipError_t launch_embed_backward(const int* tok, const float* dx, int T, int d, int V, float* out, hipStream_t s) {
  if (V <= 0) return hipSuccess;
  if (d > 8192) return hipErrorInvalidValue;
  hipLaunchKernelGGL(embed_backward_kernel, dim3(V), dim3(256), 0, s, tok, dx, T, d, out);
  return hipGetLastError();
}
hipError_t launch_add3(const float* a, const float* b, const float* c, float* out, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const int blocks = (int)std::min<size_t>((n + 255) / 256, 65536);
  hipLaunchKernelGGL(add3_kernel, dim3(blocks), dim3(256), 0, s, a, b, c, out, n);
  return hipGetLastError();
}

// f[r][0..cols) = gelu(u[r][0..cols)) for r < rows, fp16, row strides ld_u / ld_f in elements (all multiples of 8).
__global__ void __launch_bounds__(256)
    gelu_rows_f16x8_kernel(const half_t* __restrict__ u, size_t ld_u, half_t* __restrict__ f, size_t ld_f, int rows,
                           int cols8) {
  const size_t n = (size_t)rows * cols8, stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
    const size_t r = i / cols8, c = i - r * cols8;
    const f16x8_t v = *(const f16x8_t*)(u + r * ld_u + c * 8);
    f16x8_t o;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float x = (float)v[e];
      o[e] = from_f32<half_t>(x * phi_cdf_fast(x));
    }
    *(f16x8_t*)(f + r * ld_f + c * 8) = o;
  }
}
hipError_t launch_gelu_rows_f16(const void* u, size_t ld_u, void* f, size_t ld_f, int rows, int cols, hipStream_t s) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  if (((cols | ld_u | ld_f) & 7) != 0 || (((uintptr_t)u | (uintptr_t)f) & 15) != 0) return hipErrorInvalidValue;
  const size_t n = (size_t)rows * (cols / 8);
  hipLaunchKernelGGL(gelu_rows_f16x8_kernel, dim3((int)std::min<size_t>((n + 255) / 256, 65536)), dim3(256), 0, s,
                     (const half_t*)u, ld_u, (half_t*)f, ld_f, rows, cols / 8);
  return hipGetLastError();
}
hipError_t launch_gelu(int dtype, const void* u, void* f, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const int blocks = (int)std::min<size_t>((n + 255) / 256, 65536);
  if (dtype == 0) hipLaunchKernelGGL(gelu_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float*)u, (float*)f, n);
  else if ((n & 7) == 0 && (((uintptr_t)u | (uintptr_t)f) & 15) == 0)
    hipLaunchKernelGGL(gelu_f16x8_kernel, dim3((int)std::min<size_t>((n / 8 + 255) / 256, 65536)), dim3(256), 0, s,
                       (const half_t*)u, (half_t*)f, n / 8);
  else hipLaunchKernelGGL(gelu_kernel<half_t>, dim3(blocks), dim3(256), 0, s, (const half_t*)u, (half_t*)f, n);
  return hipGetLastError();
}
hipError_t launch_gelu_backward(int dtype, const void* u, void* df, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const int blocks = (int)std::min<size_t>((n + 255) / 256, 65536);
  if (dtype == 0)
    hipLaunchKernelGGL(gelu_backward_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float*)u, (float*)df, n);
  else if ((n & 7) == 0 && (((uintptr_t)u | (uintptr_t)df) & 15) == 0)
    hipLaunchKernelGGL(gelu_backward_f16x8_kernel, dim3((int)std::min<size_t>((n / 8 + 255) / 256, 65536)), dim3(256),
                       0, s, (const half_t*)u, (half_t*)df, n / 8);
  else
    hipLaunchKernelGGL(gelu_backward_kernel<half_t>, dim3(blocks), dim3(256), 0, s, (const half_t*)u, (half_t*)df, n);
  return hipGetLastError();
}
bool gelu_backward_colsum_supported(int dtype, const void* u, const void* df, int C) {
  return dtype == 1 && (C & 7) == 0 && (((uintptr_t)u | (uintptr_t)df) & 15) == 0;
}
hipError_t launch_gelu_backward_colsum(const void* u, void* df, int R, int C, float* part, int splits, float* sums,
                                       hipStream_t s) {
  if (R <= 0 || C <= 0) return hipSuccess;
  const int rps = (R + splits - 1) / splits;
  hipLaunchKernelGGL(gelu_backward_colsum_kernel, dim3((C / 8 + 255) / 256, splits), dim3(256), 0, s, (const half_t*)u,
                     (half_t*)df, R, C, rps, part);
  hipLaunchKernelGGL(colsum_final_kernel, dim3((C + 255) / 256), dim3(256), 0, s, part, splits, C, sums);
  return hipGetLastError();
}
hipError_t launch_convert_from_f32(int dtype, const float* src, void* dst, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const int blocks = (int)std::min<size_t>((n + 255) / 256, 65536);
  if (dtype == 0) hipLaunchKernelGGL(convert_kernel<float>, dim3(blocks), dim3(256), 0, s, src, (float*)dst, n);
  else hipLaunchKernelGGL(convert_kernel<half_t>, dim3(blocks), dim3(256), 0, s, src, (half_t*)dst, n);
  return hipGetLastError();
}
hipError_t launch_convert_colsum(const float* a, int R, int C, float* part, int splits, float* sums, void* out_f16,
                                 hipStream_t s) {
  if (C <= 0 || R <= 0) return hipSuccess;
  if ((C & 3) != 0 || (((uintptr_t)a | (uintptr_t)out_f16) & 15) != 0) return hipErrorInvalidValue;
  const int rps = (R + splits - 1) / splits;
  hipLaunchKernelGGL(convert_colsum_part_kernel, dim3((C / 4 + 255) / 256, splits), dim3(256), 0, s, a, R, C, rps, part,
                     (half_t*)out_f16);
  hipLaunchKernelGGL(colsum_final_kernel, dim3((C + 255) / 256), dim3(256), 0, s, part, splits, C, sums);
  return hipGetLastError();
}
// elem: 0 = float matrix, 1 = fp16 matrix.  part: [splits][C] floats of scratch.
hipError_t launch_colsum(int elem, const void* a, int R, int C, float* part, int splits, float* out, hipStream_t s) {
  if (C <= 0) return hipSuccess;
  const int rps = (std::max(R, 1) + splits - 1) / splits;
  dim3 grid((C + 255) / 256, splits);
  const int V = elem == 0 ? 4 : 8;
  if (C % V == 0 && ((uintptr_t)a & 15) == 0) {
    dim3 vgrid((C / V + 255) / 256, splits);
    if (elem == 0)
      hipLaunchKernelGGL(colsum_part_vec_kernel<float>, vgrid, dim3(256), 0, s, (const float*)a, R, C, rps, part);
    else
      hipLaunchKernelGGL(colsum_part_vec_kernel<half_t>, vgrid, dim3(256), 0, s, (const half_t*)a, R, C, rps, part);
  } else if (elem == 0)
    hipLaunchKernelGGL(colsum_part_kernel<float>, grid, dim3(256), 0, s, (const float*)a, R, C, rps, part);
  else hipLaunchKernelGGL(colsum_part_kernel<half_t>, grid, dim3(256), 0, s, (const half_t*)a, R, C, rps, part);
  hipLaunchKernelGGL(colsum_final_kernel, dim3((C + 255) / 256), dim3(256), 0, s, part, splits, C, out);
  return hipGetLastError();
}

hipError_t launch_transpose_pad(int dtype, const void* src, size_t ld_src, void* dst, size_t ld_dst, int R, int C,
                                int R_pad, hipStream_t s) {
  if (R_pad <= 0 || C <= 0) return hipSuccess;
  dim3 grid((R_pad + 31) / 32, (C + 31) / 32);
  if (dtype == 0)
    hipLaunchKernelGGL(transpose_pad_kernel<float>, grid, dim3(256), 0, s, (const float*)src, ld_src, (float*)dst,
                       ld_dst, R, C, R_pad);
  else if ((ld_src & 7) == 0 && (ld_dst & 7) == 0 && (R_pad & 7) == 0 && (C & 7) == 0 &&
           (((uintptr_t)src | (uintptr_t)dst) & 15) == 0)
    hipLaunchKernelGGL(transpose_pad_f16x8_kernel, dim3((R_pad + 63) / 64, (C + 63) / 64), dim3(256), 0, s,
                       (const half_t*)src, ld_src, (half_t*)dst, ld_dst, R, C, R_pad);
  else if ((ld_src & 3) == 0 && (ld_dst & 3) == 0 && (R_pad & 3) == 0 && (C & 3) == 0 && (R & 3) == 0 &&
           (((uintptr_t)src | (uintptr_t)dst) & 7) == 0)
    hipLaunchKernelGGL(transpose_pad_f16x4_kernel, dim3((R_pad + 63) / 64, (C + 63) / 64), dim3(256), 0, s,
                       (const half_t*)src, ld_src, (half_t*)dst, ld_dst, R, C, R_pad);
  else
    hipLaunchKernelGGL(transpose_pad_kernel<half_t>, grid, dim3(256), 0, s, (const half_t*)src, ld_src, (half_t*)dst,
                       ld_dst, R, C, R_pad);
  return hipGetLastError();
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  const size_t n = bytes / 4;  // callers pass multiples of 4 bytes
  const int blocks = (int)std::min<size_t>((n + 255) / 256, 65536);
  hipLaunchKernelGGL(fill_zero_kernel<float>, dim3(blocks), dim3(256), 0, s, (float*)p, n);
  return hipGetLastError();
}

hipError_t launch_softmax_grad(int dtype, const float* logits, int V, int V_pad, const int* targets, const float* gl,
                               int rows, int rows_pad, float inv_temp, float scale, void* dz, hipStream_t s) {
  if (rows_pad <= 0) return hipSuccess;
  const int mode = ((V & 3) == 0 && V_pad <= SG_THREADS * SG_NPT) ? 1 : 0;
#define RLHF_SG(TT, MD)                                                                                          \
  hipLaunchKernelGGL((softmax_grad_kernel<TT, MD>), dim3(rows_pad), dim3(SG_THREADS), 0, s, logits, V, V_pad, targets, \
                     gl, rows, inv_temp, scale, (TT*)dz)
  if (dtype == 0) {
    if (mode) RLHF_SG(float, 1); else RLHF_SG(float, 0);
  } else {
    if (mode) RLHF_SG(half_t, 1); else RLHF_SG(half_t, 0);
  }
#undef RLHF_SG
  return hipGetLastError();
}

bool ln_backward_rows_supported(int dtype, int d) { return dtype == 1 && d % 256 == 0 && d / 256 >= 1 && d / 256 <= 16; }
size_t ln_backward_rows_scratch_floats(int T, int d) {
  const int rpw = std::max(1, (T + 2047) / 2048), waves = ((T + rpw - 1) / rpw + 3) & ~3;
  return (size_t)waves * 2 * d;
}
hipError_t launch_ln_backward_rows(const float* x, const float* dy, const void* g, int T, int d, float eps, float* dx,
                                   float* part, float* d_g, float* d_b, hipStream_t s, const float* base) {
  if (T <= 0) return hipSuccess;
  const int rpw = std::max(1, (T + 2047) / 2048), waves = ((T + rpw - 1) / rpw + 3) & ~3;
#define RLHF_LNB(NV)                                                                                             \
  case NV:                                                                                                       \
    hipLaunchKernelGGL(ln_backward_rows_kernel<NV>, dim3(waves / 4), dim3(256), 0, s, x, dy, (const bf16_t*)g, T, \
                       eps, dx, part, rpw, base);                                                                \
    break;
  switch (d / 256) {
    RLHF_LNB(1) RLHF_LNB(2) RLHF_LNB(3) RLHF_LNB(4) RLHF_LNB(5) RLHF_LNB(6) RLHF_LNB(7) RLHF_LNB(8)
    RLHF_LNB(9) RLHF_LNB(10) RLHF_LNB(11) RLHF_LNB(12) RLHF_LNB(13) RLHF_LNB(14) RLHF_LNB(15) RLHF_LNB(16)
    default: return hipErrorInvalidValue;
  }
#undef RLHF_LNB
  hipLaunchKernelGGL(ln_backward_rows_final_kernel, dim3((2 * d + 255) / 256), dim3(256), 0, s, part, waves, d, d_g, d_b);
  return hipGetLastError();
}

hipError_t launch_head_ln_backward(int dtype, const float* x, const float* dhl, const float* gv, float scale,
                                   const void* value_w, const void* g, const void* b, int T, int d, float eps,
                                   float* dx, float* stats, float* part, int splits, float* d_g, float* d_b,
                                   float* d_wv, float* d_bv, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  const int rps = (T + splits - 1) / splits;
  dim3 cgrid((d + 255) / 256, splits);
  if (dtype == 0) {
    hipLaunchKernelGGL(ln_backward_kernel<float>, dim3(T), dim3(256), 0, s, x, dhl, gv, scale, (const float*)value_w,
                       (const float*)g, d, eps, dx, stats);
    hipLaunchKernelGGL((head_colsum_kernel<float, float>), cgrid, dim3(256), 0, s, x, dhl, gv, scale,
                       (const float*)value_w, (const float*)g, (const float*)b, stats, T, d, rps, part);
  } else {
    hipLaunchKernelGGL(ln_backward_kernel<bf16_t>, dim3(T), dim3(256), 0, s, x, dhl, gv, scale,
                       (const bf16_t*)value_w, (const bf16_t*)g, d, eps, dx, stats);
    hipLaunchKernelGGL((head_colsum_kernel<bf16_t, half_t>), cgrid, dim3(256), 0, s, x, dhl, gv, scale,
                       (const bf16_t*)value_w, (const bf16_t*)g, (const bf16_t*)b, stats, T, d, rps, part);
  }
  hipLaunchKernelGGL(head_colsum_final_kernel, dim3((d + 255) / 256), dim3(256), 0, s, part, splits, d, gv, scale, T,
                     d_g, d_b, d_wv, d_bv);
  return hipGetLastError();
}

}  // namespace rlhf
