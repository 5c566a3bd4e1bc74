// Backward pass through packed causal softmax attention: dQ, dK, dV from Q, K, V and dO.
// Two kernels, query side and key side, every sum in a fixed order (no atomics).  For fp16 and the model
// family's head sizes the matrix-core kernels further down run (attn_bwd_q_mfma, attn_bwd_kv_mfma); the first
// form, kept for the other head sizes and the fp32 check mode, is one wave per (row, head) on the vector units:
//   attn_bwd_q_kernel : for query row i -- scores against keys j <= i, their log-sum-exp, P_ij,
//                       dP_ij = dO_i . V_j, delta_i = sum_j P_ij dP_ij, dS_ij = P_ij (dP_ij - delta_i),
//                       dQ_i = scale * sum_j dS_ij K_j; keeps lse_i and delta_i for the second kernel.
//   attn_bwd_kv_kernel: for key row j -- the same P_ij and dS_ij for the queries i >= j of its
//                       sequence (from lse_i, delta_i), dV_j = sum_i P_ij dO_i, dK_j = scale * sum_i dS_ij Q_i.
// Dot products (fp16): hd/8 neighbouring lanes share a partner row, 16 bytes each, against this row's own
// vector kept in LDS; the weighted row sums run with lanes over pairs of the head's dims, partner rows one
// after the other.  Every global read is a whole row segment.
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
// fp16 rows: the row's own vector sits in LDS as fp16 pairs (exact: the inputs are fp16; they take the first
// half of the slot sized for floats), so that two products per instruction accumulate in fp32 (v_dot2_f32_f16).
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;
__device__ __forceinline__ float dot_row(const float* __restrict__ a, const half_t* __restrict__ row, int hd) {
  const f16x2_t* ah = (const f16x2_t*)a;  // hd/2 pairs, written by stash_row
  float s = 0.f;
  for (int c = 0; c < hd; c += 8) {
    const f16x8_t v = *(const f16x8_t*)(row + c);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const f16x2_t x = {v[2 * e], v[2 * e + 1]};
      s = __builtin_amdgcn_fdot2(x, ah[(c >> 1) + e], s, false);
    }
  }
  return s;
}
// the row's own vector into its LDS slot, in the form dot_row reads
__device__ __forceinline__ void stash_row(float* dst, const float* src, int hd, int lane) {
  for (int e = lane; e < hd; e += 64) dst[e] = src[e];
}
__device__ __forceinline__ void stash_row(float* dst, const half_t* src, int hd, int lane) {
  half_t* dh = (half_t*)dst;
  for (int e = lane; e < hd; e += 64) dh[e] = src[e];
}

// outA[i] = fa . rowA_i and outB[i] = fb . rowB_i for i < count, rows ld apart (fa, fb: this row's vectors in LDS
// as stash_row leaves them).  Float rows: one partner row per lane.
__device__ __forceinline__ void dots2_rows(const float* fa, const float* fb, const float* rowsA, size_t ldA,
                                           const float* rowsB, size_t ldB, int count, int hd, int lane, float* outA,
                                           float* outB) {
  for (int i = lane; i < count; i += 64) {
    outA[i] = dot_row(fa, rowsA + (size_t)i * ldA, hd);
    outB[i] = dot_row(fb, rowsB + (size_t)i * ldB, hd);
  }
}
// fp16 rows: hd/8 neighbouring lanes share a partner row, 16 bytes each, so that a wave instruction reads whole
// rows (64 / (hd/8) of them) instead of 64 scattered chunks; the lanes of a row then add their partial sums.
__device__ __forceinline__ void dots2_rows(const float* fa, const float* fb, const half_t* rowsA, size_t ldA,
                                           const half_t* rowsB, size_t ldB, int count, int hd, int lane, float* outA,
                                           float* outB) {
  const int cpr = hd >> 3, G = 64 / cpr;
  const int grp = lane / cpr, part = lane - grp * cpr;
  const bool active = grp < G;
  const f16x2_t* ah = (const f16x2_t*)fa + 4 * part;
  const f16x2_t* bh = (const f16x2_t*)fb + 4 * part;
  f16x2_t a[4], b[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    a[e] = active ? ah[e] : (f16x2_t){0, 0};
    b[e] = active ? bh[e] : (f16x2_t){0, 0};
  }
  for (int i0 = 0; i0 < count; i0 += G) {
    const int i = i0 + grp;
    float sa = 0.f, sb = 0.f;
    if (active && i < count) {
      const f16x8_t x = *(const f16x8_t*)(rowsA + (size_t)i * ldA + 8 * part);
      const f16x8_t y = *(const f16x8_t*)(rowsB + (size_t)i * ldB + 8 * part);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        sa = __builtin_amdgcn_fdot2((f16x2_t){x[2 * e], x[2 * e + 1]}, a[e], sa, false);
        sb = __builtin_amdgcn_fdot2((f16x2_t){y[2 * e], y[2 * e + 1]}, b[e], sb, false);
      }
    }
    for (int off = 1; off < cpr; off <<= 1) {  // lane `part` ends up with the sum over parts part .. cpr-1
      const float oa = __shfl_down(sa, off, 64), ob = __shfl_down(sb, off, 64);
      if (part + off < cpr) {
        sa += oa;
        sb += ob;
      }
    }
    if (active && part == 0 && i < count) {
      outA[i] = sa;
      outB[i] = sb;
    }
  }
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
                      int max_len, float* __restrict__ lse, float* __restrict__ delta, T* __restrict__ dq,
                      size_t ldq, size_t ldg, size_t ldo, T* __restrict__ o, size_t ldoo) {
  extern __shared__ float sm[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, h = blockIdx.y;
  const int t_raw = blockIdx.x * 4 + wave;
  const bool live = t_raw < Tn && t_raw < cu[B];
  const int t = live ? t_raw : 0;
  const int b = find_seq(cu, B, t), s0 = min(max(cu[b], 0), t);  // clamped: a malformed cu must not lead out of bounds
  const int nk = min(t - s0 + 1, max_len);  // keys 0 .. i of the sequence
  const size_t col = (size_t)h * hd;
  float* qs = sm + (size_t)wave * (2 * hd + 2 * max_len);
  float* gs = qs + hd;
  float* p = gs + hd;
  float* ds = p + max_len;
  stash_row(qs, q + t * ldq + col, hd, lane);
  stash_row(gs, g + t * ldg + col, hd, lane);
  __syncthreads();
  // p[j] = q . k_j (raw), ds[j] = dO . v_j for the keys of the row
  dots2_rows(qs, gs, k + (size_t)s0 * ldq + col, ldq, v + (size_t)s0 * ldq + col, ldq, nk, hd, lane, p, ds);
  __syncthreads();
  float mx = -INFINITY;
  for (int j = lane; j < nk; j += 64) mx = fmaxf(mx, p[j] * scale);
  mx = wave_max(mx);
  float sum = 0.f;
  for (int j = lane; j < nk; j += 64) sum += __expf(p[j] * scale - mx);
  sum = wave_sum(sum);
  const float l = mx + __logf(sum);
  float dl = 0.f;
  for (int j = lane; j < nk; j += 64) {
    const float pj = __expf(p[j] * scale - l);
    p[j] = pj;
    dl = fmaf(pj, ds[j], dl);
  }
  dl = wave_sum(dl);
  for (int j = lane; j < nk; j += 64) ds[j] = p[j] * (ds[j] - dl);
  __syncthreads();
  for (int e = 2 * lane; e < hd; e += 128) {  // two dims per lane: head sizes up to 128 take one sweep
    const T* kc = k + (size_t)s0 * ldq + col + e;
    float a0 = 0.f, a1 = 0.f, b0 = 0.f, b1 = 0.f;
    int j = 0;
#pragma unroll 4
    for (; j + 1 < nk; j += 2) {
      const pair2<T> x = *(const pair2<T>*)(kc + (size_t)j * ldq), y = *(const pair2<T>*)(kc + (size_t)(j + 1) * ldq);
      a0 = fmaf(ds[j], to_f32(x.a), a0);
      a1 = fmaf(ds[j], to_f32(x.b), a1);
      b0 = fmaf(ds[j + 1], to_f32(y.a), b0);
      b1 = fmaf(ds[j + 1], to_f32(y.b), b1);
    }
    if (j < nk) {
      const pair2<T> x = *(const pair2<T>*)(kc + (size_t)j * ldq);
      a0 = fmaf(ds[j], to_f32(x.a), a0);
      a1 = fmaf(ds[j], to_f32(x.b), a1);
    }
    if (live) {
      pair2<T> ov;
      ov.a = from_f32<T>((a0 + b0) * scale);
      ov.b = from_f32<T>((a1 + b1) * scale);
      *(pair2<T>*)(dq + t * ldo + col + e) = ov;
    }
  }
  if (o) {  // the forward output O_i = sum_j P_ij V_j, for callers that recompute the forward pass here
    for (int e = 2 * lane; e < hd; e += 128) {
      const T* vc = v + (size_t)s0 * ldq + col + e;
      float a0 = 0.f, a1 = 0.f;
#pragma unroll 8
      for (int j = 0; j < nk; ++j) {
        const pair2<T> x = *(const pair2<T>*)(vc + (size_t)j * ldq);
        a0 = fmaf(p[j], to_f32(x.a), a0);
        a1 = fmaf(p[j], to_f32(x.b), a1);
      }
      if (live) {
        pair2<T> ov;
        ov.a = from_f32<T>(a0);
        ov.b = from_f32<T>(a1);
        *(pair2<T>*)(o + t * ldoo + col + e) = ov;
      }
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
                       T* __restrict__ dk, T* __restrict__ dv, size_t ldq, size_t ldg, size_t ldo) {
  extern __shared__ float sm[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, h = blockIdx.y;
  const int t_raw = blockIdx.x * 4 + wave;
  const bool live = t_raw < Tn && t_raw < cu[B];
  const int t = live ? t_raw : 0;
  const int b = find_seq(cu, B, t), s0 = min(max(cu[b], 0), t);
  const int n = min(cu[b + 1] - s0, max_len);
  const int j = t - s0;
  const int nq = max(min(n - j, Tn - t), 0);  // queries j .. n-1 of the sequence see this key
  const size_t col = (size_t)h * hd;
  float* ks = sm + (size_t)wave * (2 * hd + 2 * max_len);
  float* vs = ks + hd;
  float* p = vs + hd;
  float* ds = p + max_len;
  stash_row(ks, k + t * ldq + col, hd, lane);
  stash_row(vs, v + t * ldq + col, hd, lane);
  __syncthreads();
  // p[ii] = k . q_i (raw), ds[ii] = v . dO_i for the queries that see this key
  dots2_rows(ks, vs, q + (size_t)t * ldq + col, ldq, g + (size_t)t * ldg + col, ldg, nq, hd, lane, p, ds);
  __syncthreads();
  for (int ii = lane; ii < nq; ii += 64) {
    const size_t r = (size_t)(t + ii);
    const float pr = __expf(p[ii] * scale - lse[r * H + h]);
    p[ii] = pr;
    ds[ii] = pr * (ds[ii] - delta[r * H + h]);
  }
  __syncthreads();
  for (int e = 2 * lane; e < hd; e += 128) {
    const T* gc = g + (size_t)t * ldg + col + e;
    const T* qc = q + (size_t)t * ldq + col + e;
    float av0 = 0.f, av1 = 0.f, ak0 = 0.f, ak1 = 0.f;
#pragma unroll 8
    for (int ii = 0; ii < nq; ++ii) {
      const pair2<T> x = *(const pair2<T>*)(gc + (size_t)ii * ldg), y = *(const pair2<T>*)(qc + (size_t)ii * ldq);
      av0 = fmaf(p[ii], to_f32(x.a), av0);
      av1 = fmaf(p[ii], to_f32(x.b), av1);
      ak0 = fmaf(ds[ii], to_f32(y.a), ak0);
      ak1 = fmaf(ds[ii], to_f32(y.b), ak1);
    }
    if (live) {
      pair2<T> o;
      o.a = from_f32<T>(av0);
      o.b = from_f32<T>(av1);
      *(pair2<T>*)(dv + t * ldo + col + e) = o;
      o.a = from_f32<T>(ak0 * scale);
      o.b = from_f32<T>(ak1 * scale);
      *(pair2<T>*)(dk + t * ldo + col + e) = o;
    }
  }
}

// Matrix-core form of the dK / dV kernel (fp16).  A block owns 128 keys of one (sequence, head), a wave 32 of them,
// one per lane pair; their K and V rows stay in registers as MFMA operands.  Tiles of 64 queries (rows i0 .. i0+63
// of the sequence, from the key tile's own position to the end) go through LDS twice over: row-major (Q, dO) as
// the first operand of S = Q K^T and dP = dO V^T, whose accumulators hold, for the lane's key, the tile's queries
// as rows; and transposed (Q^T, dO^T, columns in the order the accumulator rows map to operand slots) as the first
// operand of dK^T += Q^T dS and dV^T += dO^T P.  P = exp(S scale - lse_i) needs no running maximum: lse_i and
// delta_i come from the query-side kernel.
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

// Two blocks per CU where the registers allow it without spilling (head sizes up to 80 here, up to 128 for the
// query-side kernel): a second wave per SIMD covers the first one's waits (3.45 against 4.9 ms per layer at the
// 2.8B shape for the two kernels together).
template <int HD>
__global__ void __launch_bounds__(256, HD <= 80 ? 2 : 1)
    attn_bwd_kv_mfma(const half_t* __restrict__ q, const half_t* __restrict__ k, const half_t* __restrict__ v,
                     const half_t* __restrict__ g, const int* __restrict__ cu, int Tn, int H, float scale,
                     const float* __restrict__ lse, const float* __restrict__ delta, half_t* __restrict__ dk,
                     half_t* __restrict__ dv, size_t ldq, size_t ldg, size_t ldo, int kv_cache) {
  // kv_cache: k and v are the forward pass's K / V cache of the layer (sequence b owns the slots from cu[b] * H on,
  // head h of it len_b consecutive rows of HD) instead of [T, .] matrices with row stride ldq
  constexpr int NKS = HD / 16, NDT = (HD + 31) / 32, RS = HD + 8, TS = 64 + 8;
  __shared__ __attribute__((aligned(16))) uint16_t Qs[64 * RS];
  __shared__ __attribute__((aligned(16))) uint16_t Gs[64 * RS];
  __shared__ __attribute__((aligned(16))) uint16_t Qt[NDT * 32 * TS];
  __shared__ __attribute__((aligned(16))) uint16_t Gt[NDT * 32 * TS];
  __shared__ __attribute__((aligned(16))) float lse_s[64], del_s[64];
  const int b = blockIdx.z, h = blockIdx.y, k0 = blockIdx.x * 128;
  const int s0 = min(max(cu[b], 0), Tn), n = min(cu[b + 1], Tn) - s0;  // clamped: a malformed cu must not lead out of bounds
  if (k0 >= n) return;
  const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: the per-tile tests become scalar branches
  const size_t col = (size_t)h * HD;
  const int kj = k0 + wave * 32 + l32;  // this lane's key
  const int kjc = min(kj, n - 1);
  f16x8_t kf[NKS], vf[NKS];
  {
    const size_t kvb = kv_cache ? ((size_t)s0 * H + (size_t)h * (cu[b + 1] - cu[b]) + kjc) * HD
                                : (size_t)(s0 + kjc) * ldq + col;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      kf[ks] = *(const f16x8_t*)(k + kvb + 16 * ks + 8 * half);
      vf[ks] = *(const f16x8_t*)(v + kvb + 16 * ks + 8 * half);
    }
  }
  for (int c = tid; c < (NDT * 32 - HD) * TS; c += 256) {  // rows of the transposed tiles past HD stay zero
    Qt[HD * TS + c] = 0;
    Gt[HD * TS + c] = 0;
  }
  f32x16_t dvT[NDT], dkT[NDT];
#pragma unroll
  for (int t = 0; t < NDT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      dvT[t][e] = 0.f;
      dkT[t][e] = 0.f;
    }
  const float scale_log2e = scale * 1.4426950408889634f;
  const int kw0 = k0 + wave * 32;  // first key of the wave
  constexpr int CPR = HD / 8;
  // A tile travels global -> registers one iteration ahead of its use, once: a thread's item is 4 queries x 8 dims
  // of Q and of dO, which it writes to LDS both row-major (4 x 16 bytes) and transposed (8 x 8 bytes, the 4 queries
  // adjacent under the column permutation of the accumulator layout).  Threads past the tile's 16 * CPR items
  // re-read the last item instead of branching around the loads (the wait counting stays static).
  constexpr int ITEMS = 16 * CPR, NIT = (ITEMS + 255) / 256;  // items of the tile, items per thread
  f16x8_t qv[NIT][4], gv[NIT][4];
  float lse_r = 0.f, del_r = 0.f;
  auto load_tile = [&](int i0) {
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int item = min(tid + 256 * it, ITEMS - 1), ich = item / 16, ig4 = item - ich * 16;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const size_t row = (size_t)(s0 + min(i0 + 4 * ig4 + u, n - 1));
        qv[it][u] = *(const f16x8_t*)(q + row * ldq + col + ich * 8);
        gv[it][u] = *(const f16x8_t*)(g + row * ldg + col + ich * 8);
      }
    }
    const size_t row = (size_t)(s0 + min(i0 + (tid & 63), n - 1));
    lse_r = lse[row * H + h];
    del_r = delta[row * H + h];
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int item = tid + 256 * it, ich = item / 16, ig4 = item - ich * 16;
      if (item < ITEMS) {
        const int kk = (4 * ig4) & 15;
        const int colp = ((4 * ig4) & ~15) + 8 * ((kk >> 2) & 1) + 4 * (kk >> 3);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          *(f16x8_t*)((half_t*)Qs + (4 * ig4 + u) * RS + ich * 8) = qv[it][u];
          *(f16x8_t*)((half_t*)Gs + (4 * ig4 + u) * RS + ich * 8) = gv[it][u];
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const f16x4_t wq = {qv[it][0][e], qv[it][1][e], qv[it][2][e], qv[it][3][e]};
          const f16x4_t wg = {gv[it][0][e], gv[it][1][e], gv[it][2][e], gv[it][3][e]};
          *(f16x4_t*)((half_t*)Qt + (ich * 8 + e) * TS + colp) = wq;
          *(f16x4_t*)((half_t*)Gt + (ich * 8 + e) * TS + colp) = wg;
        }
      }
    }
    if (tid < 64) {
      lse_s[tid] = lse_r * 1.4426950408889634f;
      del_s[tid] = del_r;
    }
  };
  const int i_first = k0 & ~63;
  const int i_last = ((n - 1) / 64) * 64;  // first query of the sequence's last tile
  load_tile(i_first);
  // (the loads issued so far are waited for here, once: see the note in attn_prefill_mfma)
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  for (int i0 = i_first; i0 < n; i0 += 64) {
    __syncthreads();  // every wave is done with the previous tile
    store_tile();
    __syncthreads();
    load_tile(min(i0 + 64, i_last));
    if (i0 + 63 < kw0) continue;  // every query of this tile comes before every key of this wave
    // lse and delta of this lane's 32 queries of the tile: rows 32*qf2 + 8*g + 4*half + (0..3), as 4-vectors
    f16x8_t pf[4], df[4];  // P and dS of the tile for this lane's key, as second operands of the 16-query steps
    // a query i sees key kj iff i >= kj; rows past the sequence's end and keys past it contribute nothing
    const bool need_mask = (i0 < kw0 + 31) || (i0 + 64 > n) || (kw0 + 32 > n);
    const int lo = kj - i0 - 4 * half, hi = (kj < n ? n : 0) - i0 - 4 * half;  // visible iff lo <= c < hi
#pragma unroll
    for (int qf2 = 0; qf2 < 2; ++qf2) {
      f32x16_t st, dp;
      {
        f16x8_t qa[NKS], ga[NKS];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
          qa[ks] = *(const f16x8_t*)(Qs + (qf2 * 32 + l32) * RS + 16 * ks + 8 * half);
          ga[ks] = *(const f16x8_t*)(Gs + (qf2 * 32 + l32) * RS + 16 * ks + 8 * half);
        }
        const f32x16_t z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        st = z;
        dp = z;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
          st = __builtin_amdgcn_mfma_f32_32x32x16_f16(qa[ks], kf[ks], st, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_f16(ga[ks], vf[ks], dp, 0, 0, 0);
        }
        // fragment reads four ahead of the matrix instructions
        constexpr int AH = 2 * NKS < 4 ? 2 * NKS : 4;
        __builtin_amdgcn_sched_group_barrier(0x100, AH, 0);
#pragma unroll
        for (int i = 0; i < 2 * NKS - AH; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, AH, 0);
      }
      f32x4_t ls[4], dl[4];
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        ls[g4] = *(const f32x4_t*)(lse_s + qf2 * 32 + 8 * g4 + 4 * half);
        dl[g4] = *(const f32x4_t*)(del_s + qf2 * 32 + 8 * g4 + 4 * half);
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        float pr = __builtin_amdgcn_exp2f(fmaf(st[e], scale_log2e, -ls[e >> 2][e & 3]));
        if (need_mask) {
          const int c = qf2 * 32 + 8 * (e >> 2) + (e & 3);
          if (c < lo || c >= hi) pr = 0.f;
        }
        pf[qf2 * 2 + (e >> 3)][e & 7] = (half_t)pr;
        df[qf2 * 2 + (e >> 3)][e & 7] = (half_t)(pr * (dp[e] - dl[e >> 2][e & 3]));
      }
    }
    {
      f16x8_t ga[4 * NDT], qa[4 * NDT];
#pragma unroll
      for (int i = 0; i < 4 * NDT; ++i) {
        ga[i] = *(const f16x8_t*)(Gt + ((i % NDT) * 32 + l32) * TS + 16 * (i / NDT) + 8 * half);
        qa[i] = *(const f16x8_t*)(Qt + ((i % NDT) * 32 + l32) * TS + 16 * (i / NDT) + 8 * half);
      }
#pragma unroll
      for (int i = 0; i < 4 * NDT; ++i) {
        dvT[i % NDT] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ga[i], pf[i / NDT], dvT[i % NDT], 0, 0, 0);
        dkT[i % NDT] = __builtin_amdgcn_mfma_f32_32x32x16_f16(qa[i], df[i / NDT], dkT[i % NDT], 0, 0, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
      for (int i = 0; i < 8 * NDT - 4; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    }
  }
  if (kj < n) {
    half_t* dvr = dv + (size_t)(s0 + kj) * ldo + col;
    half_t* dkr = dk + (size_t)(s0 + kj) * ldo + col;
#pragma unroll
    for (int t = 0; t < NDT; ++t)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int dd = 32 * t + 8 * g4 + 4 * half;
        if (dd < HD) {  // HD is a multiple of 4: the 4 dims are in range together
          f16x4_t a, c2;
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            a[u] = from_f32<half_t>(dvT[t][4 * g4 + u]);
            c2[u] = from_f32<half_t>(dkT[t][4 * g4 + u] * scale);
          }
          *(f16x4_t*)(dvr + dd) = a;
          *(f16x4_t*)(dkr + dd) = c2;
        }
      }
  }
}

// Matrix-core form of the query-side kernel (fp16).  A block owns 128 queries of one (sequence, head), a wave 32,
// whose Q and dO rows stay in registers as second operands; tiles of 64 keys go through LDS row-major (K, V) and
// transposed (K^T, V^T).  Pass 1 is the forward pass (S^T = K Q^T, running maximum and sum, O^T += V^T P^T): it
// yields O, lse_i and delta_i = dO_i . O_i.  Pass 2 walks the key tiles again: P^T = exp(S^T scale - lse_i),
// dP^T = V dO^T, dS^T = P^T (dP^T - delta_i), dQ^T += K^T dS^T.
template <int HD>
__global__ void __launch_bounds__(256, HD <= 128 ? 2 : 1)
    attn_bwd_q_mfma(const half_t* __restrict__ q, const half_t* __restrict__ k, const half_t* __restrict__ v,
                    const half_t* __restrict__ g, const int* __restrict__ cu, int Tn, int H, float scale,
                    float* __restrict__ lse, float* __restrict__ delta, half_t* __restrict__ dq, size_t ldq, size_t ldg,
                    size_t ldo, half_t* __restrict__ o_out, size_t ldoo, int kv_cache) {
  // kv_cache: k and v are the forward pass's K / V cache of the layer (see attn_bwd_kv_mfma); q stays [T, .]
  constexpr int NKS = HD / 16, NDT = (HD + 31) / 32, RS = HD + 8, TS = 64 + 8, CPR = HD / 8;
  __shared__ __attribute__((aligned(16))) uint16_t Ks[64 * RS];
  __shared__ __attribute__((aligned(16))) uint16_t Vs[64 * RS];
  __shared__ __attribute__((aligned(16))) uint16_t Kt[NDT * 32 * TS];
  __shared__ __attribute__((aligned(16))) uint16_t Vt[NDT * 32 * TS];
  const int b = blockIdx.z, h = blockIdx.y, q0 = blockIdx.x * 128;
  const int s0 = min(max(cu[b], 0), Tn), n = min(cu[b + 1], Tn) - s0;
  if (q0 >= n) return;
  const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: the per-tile tests become scalar branches
  const size_t col = (size_t)h * HD;
  const int qi = q0 + wave * 32 + l32;  // this lane's query (two lanes per query: half 0 / 1)
  const int qic = min(qi, n - 1);
  f16x8_t qf[NKS], gf[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    qf[ks] = *(const f16x8_t*)(q + (size_t)(s0 + qic) * ldq + col + 16 * ks + 8 * half);
    gf[ks] = *(const f16x8_t*)(g + (size_t)(s0 + qic) * ldg + col + 16 * ks + 8 * half);
  }
  for (int c = tid; c < (NDT * 32 - HD) * TS; c += 256) {
    Kt[HD * TS + c] = 0;
    Vt[HD * TS + c] = 0;
  }
  const int q_hi = min(q0 + 128, n) - 1, wq_lo = q0 + wave * 32;
  const int k_last = (q_hi / 64) * 64;  // first key of the block's last tile
  const float scale_log2e = scale * 1.4426950408889634f;
  // A tile travels global -> registers one iteration ahead of its use, once: a thread's item is 4 keys x 8 dims of K
  // and of V, which it writes to LDS row-major (4 x 16 bytes) and / or transposed (8 x 8 bytes, the 4 keys adjacent
  // under the column permutation of the accumulator layout), whichever images the pass reads.  Threads past the
  // tile's 16 * CPR items re-read the last item instead of branching around the loads (static wait counts).
  constexpr int ITEMS = 16 * CPR, NIT = (ITEMS + 255) / 256;  // items of the tile, items per thread
  f16x8_t kv[NIT][4], vv[NIT][4];
  const size_t kvb = kv_cache ? ((size_t)s0 * H + (size_t)h * (cu[b + 1] - cu[b])) * HD : (size_t)s0 * ldq + col;
  const size_t kvld = kv_cache ? (size_t)HD : ldq;
  auto load_tile = [&](int k0) {
    k0 = min(k0, k_last);
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int item = min(tid + 256 * it, ITEMS - 1), ich = item / 16, ig4 = item - ich * 16;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const size_t off = kvb + (size_t)min(k0 + 4 * ig4 + u, n - 1) * kvld + ich * 8;
        kv[it][u] = *(const f16x8_t*)(k + off);
        vv[it][u] = *(const f16x8_t*)(v + off);
      }
    }
  };
  auto store_tile = [&](bool second_pass) {
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int item = tid + 256 * it, ich = item / 16, ig4 = item - ich * 16;
      if (item < ITEMS) {
        const int kk = (4 * ig4) & 15;
        const int colp = ((4 * ig4) & ~15) + 8 * ((kk >> 2) & 1) + 4 * (kk >> 3);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          *(f16x8_t*)((half_t*)Ks + (4 * ig4 + u) * RS + ich * 8) = kv[it][u];
          if (second_pass) *(f16x8_t*)((half_t*)Vs + (4 * ig4 + u) * RS + ich * 8) = vv[it][u];
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          if (second_pass) {
            const f16x4_t wk = {kv[it][0][e], kv[it][1][e], kv[it][2][e], kv[it][3][e]};
            *(f16x4_t*)((half_t*)Kt + (ich * 8 + e) * TS + colp) = wk;
          } else {
            const f16x4_t wv = {vv[it][0][e], vv[it][1][e], vv[it][2][e], vv[it][3][e]};
            *(f16x4_t*)((half_t*)Vt + (ich * 8 + e) * TS + colp) = wv;
          }
        }
      }
    }
  };
  // S^T of the tile for this lane's query: two fragments of 32 keys, their accumulation chains alternating, the
  // fragment reads four ahead of the matrix instructions
#define BWD_SCORES(ST)                                                                                      \
  {                                                                                                         \
    f16x8_t kfr[2 * NKS];                                                                                   \
    _Pragma("unroll") for (int i = 0; i < 2 * NKS; ++i)                                                     \
        kfr[i] = *(const f16x8_t*)(Ks + ((i & 1) * 32 + l32) * RS + 16 * (i >> 1) + 8 * half);            \
    const f32x16_t z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};    \
    ST[0] = z;                                                                                              \
    ST[1] = z;                                                                                              \
    _Pragma("unroll") for (int i = 0; i < 2 * NKS; ++i)                                                     \
        ST[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kfr[i], qf[i >> 1], ST[i & 1], 0, 0, 0);       \
    constexpr int AH = 2 * NKS < 4 ? 2 * NKS : 4;                                                           \
    __builtin_amdgcn_sched_group_barrier(0x100, AH, 0);                                                     \
    _Pragma("unroll") for (int i = 0; i < 2 * NKS - AH; ++i) {                                              \
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                    \
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                                    \
    }                                                                                                       \
    __builtin_amdgcn_sched_group_barrier(0x008, AH, 0);                                                     \
  }
  // NDT accumulation chains over the four 16-key steps of a transposed image, reads four ahead
#define BWD_OUT(IMG, OPS, ACC)                                                                              \
  {                                                                                                         \
    f16x8_t fr[4 * NDT];                                                                                    \
    _Pragma("unroll") for (int i = 0; i < 4 * NDT; ++i)                                                     \
        fr[i] = *(const f16x8_t*)(IMG + ((i % NDT) * 32 + l32) * TS + 16 * (i / NDT) + 8 * half);         \
    _Pragma("unroll") for (int i = 0; i < 4 * NDT; ++i)                                                     \
        ACC[i % NDT] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fr[i], OPS[i / NDT], ACC[i % NDT], 0, 0, 0); \
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);                                                      \
    _Pragma("unroll") for (int i = 0; i < 4 * NDT - 4; ++i) {                                               \
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                    \
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                                    \
    }                                                                                                       \
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);                                                      \
  }
  // ---- pass 1: the forward pass
  f32x16_t acc[NDT];
#pragma unroll
  for (int t = 0; t < NDT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  load_tile(0);
  // (the loads issued so far are waited for here, once: see the note in attn_prefill_mfma)
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  for (int k0 = 0; k0 <= q_hi; k0 += 64) {
    __syncthreads();  // every wave is done with the previous tile
    store_tile(false);
    __syncthreads();
    load_tile(k0 + 64 <= q_hi ? k0 + 64 : 0);  // after the last tile: tile 0, which the second pass starts with
    if (k0 > wq_lo + 31) continue;  // every key of this tile is in the future of this wave's queries
    f32x16_t st[2];
    BWD_SCORES(st)
    // key kj = k0 + 4*half + c of element (kf, e), c = 32*kf + 8*(e/4) + e%4, is visible iff kj <= min(qi, n - 1)
    if ((k0 + 63 > wq_lo) || (k0 + 64 > n)) {
      const int lim = min(qi, n - 1) - k0 - 4 * half;
#pragma unroll
      for (int kf = 0; kf < 2; ++kf)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (kf * 32 + 8 * (e >> 2) + (e & 3) > lim) st[kf][e] = -INFINITY;
    }
    float mx = -INFINITY;
#pragma unroll
    for (int kf = 0; kf < 2; ++kf)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, st[kf][e]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx * scale_log2e);  // finite: key 0 is visible to every query
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    float psum = 0.f;
    f16x8_t pf[4];
#pragma unroll
    for (int kf = 0; kf < 2; ++kf)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float p = __builtin_amdgcn_exp2f(fmaf(st[kf][e], scale_log2e, -m_new));
        psum += p;
        pf[kf * 2 + (e >> 3)][e & 7] = (half_t)p;
      }
    l_run = l_run * alpha + psum;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
      for (int t = 0; t < NDT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] *= alpha;
    }
    BWD_OUT(Vt, pf, acc)
  }
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.0f / l_tot;
  const float lse2 = m_run + __builtin_amdgcn_logf(l_tot);  // log2 of the row's sum of exponentials
  // O_i (optional output) and delta_i = dO_i . O_i: this lane holds 4-dim groups of its query's output
  float dl = 0.f;
  {
    const half_t* grow = g + (size_t)(s0 + qic) * ldg + col;
#pragma unroll
    for (int t = 0; t < NDT; ++t)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int dd = 32 * t + 8 * g4 + 4 * half;
        if (dd < HD) {
          const f16x4_t gv = *(const f16x4_t*)(grow + dd);
          f16x4_t ov;
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const float x = acc[t][4 * g4 + u] * inv;
            dl = fmaf(x, (float)gv[u], dl);
            ov[u] = from_f32<half_t>(x);
          }
          if (o_out && qi < n) *(f16x4_t*)(o_out + (size_t)(s0 + qi) * ldoo + col + dd) = ov;
        }
      }
  }
  dl += __shfl_xor(dl, 32, 64);
  if (qi < n && half == 0) {
    lse[(size_t)(s0 + qi) * H + h] = lse2 * 0.6931471805599453f;  // natural logarithm, as the key-side kernels read it
    delta[(size_t)(s0 + qi) * H + h] = dl;
  }
  // ---- pass 2: dQ^T += K^T dS^T over the same key tiles
#pragma unroll
  for (int t = 0; t < NDT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
  for (int k0 = 0; k0 <= q_hi; k0 += 64) {  // (tile 0 is in the registers: the first pass's last load)
    __syncthreads();
    store_tile(true);
    __syncthreads();
    load_tile(k0 + 64);
    if (k0 > wq_lo + 31) continue;
    f32x16_t st[2];
    BWD_SCORES(st)
    f16x8_t df[4];
    const bool need_mask = (k0 + 63 > wq_lo) || (k0 + 64 > n);
    const int lim = min(qi, n - 1) - k0 - 4 * half;
#pragma unroll
    for (int kf = 0; kf < 2; ++kf) {
      f32x16_t dp;
      {
        f16x8_t va[NKS];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) va[ks] = *(const f16x8_t*)(Vs + (kf * 32 + l32) * RS + 16 * ks + 8 * half);
        const f32x16_t z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        dp = z;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) dp = __builtin_amdgcn_mfma_f32_32x32x16_f16(va[ks], gf[ks], dp, 0, 0, 0);
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        float pr = __builtin_amdgcn_exp2f(fmaf(st[kf][e], scale_log2e, -lse2));
        if (need_mask && kf * 32 + 8 * (e >> 2) + (e & 3) > lim) pr = 0.f;
        df[kf * 2 + (e >> 3)][e & 7] = (half_t)(pr * (dp[e] - dl));
      }
    }
    BWD_OUT(Kt, df, acc)
  }
#undef BWD_SCORES
#undef BWD_OUT
  if (qi < n) {
    half_t* drow = dq + (size_t)(s0 + qi) * ldo + col;
#pragma unroll
    for (int t = 0; t < NDT; ++t)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int dd = 32 * t + 8 * g4 + 4 * half;
        if (dd < HD) {
          f16x4_t a;
#pragma unroll
          for (int u = 0; u < 4; ++u) a[u] = from_f32<half_t>(acc[t][4 * g4 + u] * scale);
          *(f16x4_t*)(drow + dd) = a;
        }
      }
  }
}

// Rotary turn of the q and k sections of a [T, 3*d] matrix (sections q | k | v, heads of hd, the first
// r dims of a head rotary), in place, by the row's position in its sequence (row - cu[sequence]);
// dir = +1 turns forward, -1 back (the transpose of the forward turn: what a gradient takes).
// ADJ: pairs are (2i, 2i+1) -- the reordered layout of the fp16 path -- else (i, i + r/2).
template <typename T, bool ADJ>
__global__ void __launch_bounds__(256)
    rope_inplace_kernel(T* __restrict__ qkv, size_t ld, const int* __restrict__ cu, int B, int Tn, int H, int hd, int r,
                        const float* __restrict__ cos_t, const float* __restrict__ sin_t, float dir) {
  const int t = blockIdx.x;
  if (t >= Tn || t >= cu[B]) return;
  const int b = find_seq(cu, B, t), pos = t - min(max(cu[b], 0), t), half = r >> 1;
  const float* cs = cos_t + (size_t)pos * half;
  const float* sn = sin_t + (size_t)pos * half;
  for (int c = threadIdx.x; c < 2 * H * half; c += 256) {
    const int u = c / half, i = c - u * half;  // u = section * H + head
    T* hb = qkv + (size_t)t * ld + (size_t)u * hd;  // sections are d = H*hd apart, so (section, head) is u heads in
    const int lo_i = ADJ ? 2 * i : i, hi_i = ADJ ? 2 * i + 1 : i + half;
    const float co = cs[i], si = sn[i] * dir;
    const float lo = to_f32(hb[lo_i]), hi = to_f32(hb[hi_i]);
    hb[lo_i] = from_f32<T>(lo * co - hi * si);
    hb[hi_i] = from_f32<T>(hi * co + lo * si);
  }
}

// out[src(n)] = in[n] for the 3*d rows of a W_qkv-shaped matrix (or its bias, C = 1): puts rows that are in
// the reordered pair layout of the fp16 path back into the caller's order (see qkv_weights_f16_kernel).
__global__ void __launch_bounds__(256)
    qkv_rows_to_caller_order_kernel(const float* __restrict__ in, float* __restrict__ out, int d, int hd, int r, int C) {
  const int n = blockIdx.x;
  const int sec = n / d, e = (n - sec * d) % hd;
  int src = n;
  if (sec < 2 && e < r) src = n - e + ((e & 1) ? (e >> 1) + (r >> 1) : (e >> 1));
  for (int c = threadIdx.x; c < C; c += 256) out[(size_t)src * C + c] = in[(size_t)n * C + c];
}

}  // namespace

hipError_t launch_rope_inplace(int dtype, void* qkv, size_t ld, const int* cu, int B, int Tn, int H, int hd, int r,
                               const float* cos_t, const float* sin_t, int backward, hipStream_t s) {
  if (Tn <= 0 || r <= 0) return hipSuccess;
  const float dir = backward ? -1.0f : 1.0f;
  if (dtype == 0)
    hipLaunchKernelGGL((rope_inplace_kernel<float, false>), dim3(Tn), dim3(256), 0, s, (float*)qkv, ld, cu, B, Tn, H, hd,
                       r, cos_t, sin_t, dir);
  else
    hipLaunchKernelGGL((rope_inplace_kernel<half_t, true>), dim3(Tn), dim3(256), 0, s, (half_t*)qkv, ld, cu, B, Tn, H,
                       hd, r, cos_t, sin_t, dir);
  return hipGetLastError();
}

hipError_t launch_qkv_rows_to_caller_order(const float* in, float* out, int d, int hd, int r, int C, hipStream_t s) {
  hipLaunchKernelGGL(qkv_rows_to_caller_order_kernel, dim3(3 * d), dim3(256), 0, s, in, out, d, hd, r, C);
  return hipGetLastError();
}

// dtype 0: float, 1: fp16.  head_dim a multiple of 4 (float) or 8 (fp16); the longest sequence at
// most max_len rows (longer ones are cut off at max_len: wrong results, but no access out of bounds).
bool attention_backward_takes_cache(int dtype, int hd) { return dtype == 1 && (hd == 64 || hd == 80 || hd == 128 || hd == 256); }

hipError_t launch_attention_backward(int dtype, const void* q, const void* k, const void* v, const void* g,
                                     const int* cu, int B, int Tn, int H, int hd, int max_len, float* lse,
                                     float* delta, void* dq, void* dk, void* dv, hipStream_t s, size_t ld_qkv,
                                     size_t ld_g, size_t ld_out, void* o, size_t ld_o, bool kv_cache) {
  const size_t dm = (size_t)H * hd;
  if (kv_cache && !attention_backward_takes_cache(dtype, hd)) return hipErrorInvalidValue;
  if (!ld_qkv) ld_qkv = dm;
  if (!ld_g) ld_g = dm;
  if (!ld_out) ld_out = dm;
  if (!ld_o) ld_o = dm;
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
                       (const float*)v, (const float*)g, cu, B, Tn, H, hd, scale, max_len, lse, delta, (float*)dq, ld_qkv,
                       ld_g, ld_out, (float*)o, ld_o);
    hipLaunchKernelGGL(attn_bwd_kv_kernel<float>, grid, dim3(256), sh, s, (const float*)q, (const float*)k,
                       (const float*)v, (const float*)g, cu, B, Tn, H, hd, scale, max_len, lse, delta, (float*)dk,
                       (float*)dv, ld_qkv, ld_g, ld_out);
  } else {
    if (sh > 65536) {
      (void)hipFuncSetAttribute((const void*)attn_bwd_q_kernel<half_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh);
      (void)hipFuncSetAttribute((const void*)attn_bwd_kv_kernel<half_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh);
    }
    if (hd == 64 || hd == 80 || hd == 128 || hd == 256) {  // the model family's head sizes: matrix-core forms of both kernels
      dim3 mgrid((max_len + 127) / 128, H, B);
#define RLHF_BWD_MFMA(HD_)                                                                                      \
  hipLaunchKernelGGL(attn_bwd_q_mfma<HD_>, mgrid, dim3(256), 0, s, (const half_t*)q, (const half_t*)k,          \
                     (const half_t*)v, (const half_t*)g, cu, Tn, H, scale, lse, delta, (half_t*)dq, ld_qkv,     \
                     ld_g, ld_out, (half_t*)o, ld_o, kv_cache ? 1 : 0);                                         \
  hipLaunchKernelGGL(attn_bwd_kv_mfma<HD_>, mgrid, dim3(256), 0, s, (const half_t*)q, (const half_t*)k,         \
                     (const half_t*)v, (const half_t*)g, cu, Tn, H, scale, lse, delta, (half_t*)dk, (half_t*)dv, \
                     ld_qkv, ld_g, ld_out, kv_cache ? 1 : 0)
      if (hd == 64) { RLHF_BWD_MFMA(64); }
      else if (hd == 80) { RLHF_BWD_MFMA(80); }
      else if (hd == 128) { RLHF_BWD_MFMA(128); }
      else { RLHF_BWD_MFMA(256); }
#undef RLHF_BWD_MFMA
      return hipGetLastError();
    }
    hipLaunchKernelGGL(attn_bwd_q_kernel<half_t>, grid, dim3(256), sh, s, (const half_t*)q, (const half_t*)k,
                       (const half_t*)v, (const half_t*)g, cu, B, Tn, H, hd, scale, max_len, lse, delta, (half_t*)dq,
                       ld_qkv, ld_g, ld_out, (half_t*)o, ld_o);
    hipLaunchKernelGGL(attn_bwd_kv_kernel<half_t>, grid, dim3(256), sh, s, (const half_t*)q, (const half_t*)k,
                       (const half_t*)v, (const half_t*)g, cu, B, Tn, H, hd, scale, max_len, lse, delta, (half_t*)dk,
                       (half_t*)dv, ld_qkv, ld_g, ld_out);
  }
  return hipGetLastError();
}

}  // namespace rlhf
