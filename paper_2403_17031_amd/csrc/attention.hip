// Causal self-attention over packed variable-length sequences (prefill / scoring) and single-query
// attention against the KV cache (decode).  K and V live in a [head][slot][head_dim] layout, a
// sequence's keys occupying consecutive slots, so one (sequence, head) pair reads one contiguous
// run of memory.
#include <algorithm>

#include "common.h"

namespace rlhf {

// =================================================================================================
// Generic tile kernel (any storage type, any head_dim <= 256): 32 queries x 32 keys per step,
// fp32 throughout, online softmax.  Used for fp32 check mode and as the fallback.
// =================================================================================================
template <typename T>
__global__ void __launch_bounds__(256)
    attn_prefill_generic(const T* __restrict__ q, const T* __restrict__ kc, const T* __restrict__ vc,
                         long kv_extra, const int* __restrict__ len, const int* __restrict__ cu,
                         const int* __restrict__ kvoff, int H, int hd, float scale, T* __restrict__ out, int out_ld) {
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
  const T* kb = kc + ((size_t)kvoff[b] * H + (size_t)h * (len[b] + kv_extra)) * hd;
  const T* vb = vc + ((size_t)kvoff[b] * H + (size_t)h * (len[b] + kv_extra)) * hd;
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
    T* ob = out + ((size_t)cu[b] + q0 + qi) * out_ld + (size_t)h * hd;
#pragma unroll
    for (int k = 0; k < 32; ++k) {
      const int e = sub + 8 * k;
      if (e < hd) ob[e] = from_f32<T>(acc[k] * inv);
    }
  }
}


// =================================================================================================
// MFMA flash attention (fp16 operands, fp32 softmax and accumulation), head_dim HD a multiple of 16.
//
// Block = 4 waves; wave w owns 32 queries, all work is per wave except the shared K / V tile.
// Scores are produced transposed, S^T[key][q] = K Q^T, so that a lane holds one query (lane % 32)
// and 16 of each 32 keys: the running max / sum are per-lane scalars, shared with lane ^ 32 only.
// The probabilities then feed O^T[d][q] = V^T P^T straight from registers: the accumulator layout
// of S^T is the operand layout of P^T up to a fixed permutation of the 16 keys of a k-step, and
// the V tile is stored in LDS transposed with that same permutation applied.
// =================================================================================================
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

constexpr int FA_BQ = 128, FA_BK = 64;
constexpr int FA_VT_STRIDE = FA_BK + 8;  // halfs per V^T row: 144 B, odd multiple of 16 B

template <int HD>
__global__ void __launch_bounds__(256, (HD <= 80 ? 3 : HD <= 128 ? 2 : 1))
    attn_prefill_mfma(const half_t* __restrict__ q, const half_t* __restrict__ kc, const half_t* __restrict__ vc,
                      long kv_extra, const int* __restrict__ len, const int* __restrict__ cu,
                      const int* __restrict__ kvoff, int H, float scale_log2e, half_t* __restrict__ out, int out_ld) {
  constexpr int NKS = HD / 16;         // k-steps of the Q K^T contraction
  constexpr int NDT = (HD + 31) / 32;  // 32-row tiles of O^T
  constexpr int K_STRIDE = HD + 8;     // halfs per K row: odd multiple of 16 B for every HD used
  __shared__ __attribute__((aligned(16))) uint16_t Ks[FA_BK * K_STRIDE];
  __shared__ __attribute__((aligned(16))) uint16_t Vt[NDT * 32 * FA_VT_STRIDE];
  const int b = blockIdx.z, h = blockIdx.y, q0 = blockIdx.x * FA_BQ;
  const int n = len[b];
  if (q0 >= n) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: the per-tile branches below are scalar
  const int half = lane >> 5, l32 = lane & 31;
  const int d = H * HD;
  const half_t* kb = kc + ((size_t)kvoff[b] * H + (size_t)h * (len[b] + kv_extra)) * HD;
  const half_t* vb = vc + ((size_t)kvoff[b] * H + (size_t)h * (len[b] + kv_extra)) * HD;

  // rows of V^T beyond HD are never loaded: zero them once
  for (int c = tid; c < (NDT * 32 - HD) * FA_VT_STRIDE; c += 256) Vt[HD * FA_VT_STRIDE + c] = 0;

  // this lane's query and its Q fragments (kept in registers for the whole block)
  const int qi = q0 + wave * 32 + l32;
  const half_t* qrow = q + ((size_t)cu[b] + min(qi, n - 1)) * d + (size_t)h * HD;
  f16x8_t qf[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) qf[ks] = *(const f16x8_t*)(qrow + 16 * ks + 8 * half);

  f32x16_t o[NDT];
#pragma unroll
  for (int t = 0; t < NDT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[t][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;  // l_run: sum over this lane's keys only

  const int q_hi = min(q0 + FA_BQ, n) - 1;           // last query of the block
  const int wq_lo = q0 + wave * 32;                  // first query of the wave
  // The next K / V tile travels global -> registers while the current one is being multiplied.
  //   K: row-major 16-byte chunks, keys past the sequence clamped (their scores are masked below).
  //   V: stored transposed.  A thread takes 4 consecutive keys x 8 dims and writes 8 eight-byte
  //      words, one per dim: keys 4g..4g+3 stay adjacent under the column permutation
  //      (key kk of a 16-key group goes to column 8*((kk>>2)&1) + (kk&3) + 4*(kk>>3)).
  constexpr int KCH = FA_BK * (HD / 8);             // 16-byte chunks of a K tile
  constexpr int NKR = (KCH + 255) / 256;            // ... per thread
  constexpr int VIT = (FA_BK / 4) * (HD / 8);       // V items (4 keys x 8 dims)
  constexpr int NVR = (VIT + 255) / 256;            // ... per thread
  u32x4_t kreg[NKR];
  f16x8_t vreg[NVR][4];
  auto load_tile = [&](int k0) {
#pragma unroll
    for (int i = 0; i < NKR; ++i) {
      const int c = tid + 256 * i;
      if (c < KCH) {
        const int r = c / (HD / 8), ch = c - r * (HD / 8);
        kreg[i] = *(const u32x4_t*)(kb + (size_t)min(k0 + r, n - 1) * HD + ch * 8);
      }
    }
#pragma unroll
    for (int i = 0; i < NVR; ++i) {
      const int c = tid + 256 * i;
      if (c < VIT) {
        const int ch = c / (FA_BK / 4), g4 = c - ch * (FA_BK / 4);
#pragma unroll
        for (int u = 0; u < 4; ++u)
          vreg[i][u] = *(const f16x8_t*)(vb + (size_t)min(k0 + 4 * g4 + u, n - 1) * HD + ch * 8);
      }
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int i = 0; i < NKR; ++i) {
      const int c = tid + 256 * i;
      if (c < KCH) {
        const int r = c / (HD / 8), ch = c - r * (HD / 8);
        *(u32x4_t*)(Ks + r * K_STRIDE + ch * 8) = kreg[i];
      }
    }
#pragma unroll
    for (int i = 0; i < NVR; ++i) {
      const int c = tid + 256 * i;
      if (c < VIT) {
        const int ch = c / (FA_BK / 4), g4 = c - ch * (FA_BK / 4);
        const int kk = (4 * g4) & 15;
        const int col = ((4 * g4) & ~15) + 8 * ((kk >> 2) & 1) + 4 * (kk >> 3);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          f16x4_t w = {vreg[i][0][e], vreg[i][1][e], vreg[i][2][e], vreg[i][3][e]};
          *(f16x4_t*)((half_t*)Vt + (ch * 8 + e) * FA_VT_STRIDE + col) = w;
        }
      }
    }
  };
  load_tile(0);
  // Everything loaded so far (the Q fragments, tile 0) is waited for here, once: otherwise the compiler's wait
  // bookkeeping carries the Q loads as possibly pending around the loop and, since loads retire in order, makes
  // every iteration wait for the tile it has just prefetched before the first matrix instruction that reads Q.
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  for (int k0 = 0; k0 <= q_hi; k0 += FA_BK) {
    __syncthreads();  // every wave is done with the previous tile
    store_tile();
    __syncthreads();
    if (k0 + FA_BK <= q_hi) load_tile(k0 + FA_BK);
    if (k0 > wq_lo + 31) continue;  // every key of this tile is in the future of this wave's queries

    // ---- S^T = K Q^T for the two 32-key fragments.  The two accumulation chains alternate, and the fragment
    //      reads run three ahead of the matrix instructions (scheduling groups: left to itself the compiler
    //      waits for every read right before the instruction that uses it; four ahead costs the registers that
    //      keep head sizes up to 80 from running three blocks per CU: 730 against 785 us at the 2.8B shape)
    f32x16_t st[2];
#pragma unroll
    for (int kf = 0; kf < 2; ++kf)
#pragma unroll
      for (int e = 0; e < 16; ++e) st[kf][e] = 0.f;
    {
      f16x8_t kfr[2 * NKS];
#pragma unroll
      for (int i = 0; i < 2 * NKS; ++i)
        kfr[i] = *(const f16x8_t*)(Ks + ((i & 1) * 32 + l32) * K_STRIDE + 16 * (i >> 1) + 8 * half);
#pragma unroll
      for (int i = 0; i < 2 * NKS; ++i)
        st[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kfr[i], qf[i >> 1], st[i & 1], 0, 0, 0);
      constexpr int AHEAD = 2 * NKS < 3 ? 2 * NKS : 3;
      __builtin_amdgcn_sched_group_barrier(0x100, AHEAD, 0);
#pragma unroll
      for (int i = 0; i < 2 * NKS - AHEAD; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, AHEAD, 0);
    }
    // ---- mask (only tiles that touch the diagonal or the end of the sequence), scale, running max
    //      Key kj = k0 + 4*half + c of element (kf, e), c = 32*kf + 8*(e/4) + e%4 a constant, is visible iff
    //      kj <= min(qi, n - 1), i.e. c <= lim with lim formed once per tile: a compare and a select per element
    //      (the branch is wave-uniform).
    const bool need_mask = (k0 + FA_BK - 1 > wq_lo) || (k0 + FA_BK > n);
    if (need_mask) {
      const int lim = min(qi, n - 1) - k0 - 4 * half;
#pragma unroll
      for (int kf = 0; kf < 2; ++kf)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (kf * 32 + 8 * (e >> 2) + (e & 3) > lim) st[kf][e] = -INFINITY;
    }
    float mx = -INFINITY;  // raw dot products: the (positive) scale is applied inside the exponent's FMA
#pragma unroll
    for (int kf = 0; kf < 2; ++kf)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, st[kf][e]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx * scale_log2e);  // finite: key 0 is visible to every query
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);  // arguments <= 0: the bare instruction will do
    m_run = m_new;
    float psum = 0.f;
    f16x8_t pf[4];  // P^T operand of each 16-key step
#pragma unroll
    for (int kf = 0; kf < 2; ++kf)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float p = __builtin_amdgcn_exp2f(fmaf(st[kf][e], scale_log2e, -m_new));
        psum += p;
        pf[kf * 2 + (e >> 3)][e & 7] = (half_t)p;
      }
    l_run = l_run * alpha + psum;
    // ---- O^T = alpha * O^T + V^T P^T
    // once the running maxima have settled (usually after the first tiles) alpha is 1 in every lane
    // and the rescaling of the accumulators is skipped for the whole wave
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
      for (int t = 0; t < NDT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[t][e] *= alpha;
    }
    //      (the NDT accumulation chains alternate; fragment reads three ahead as above)
    {
      f16x8_t vfr[4 * NDT];
#pragma unroll
      for (int i = 0; i < 4 * NDT; ++i)
        vfr[i] = *(const f16x8_t*)(Vt + ((i % NDT) * 32 + l32) * FA_VT_STRIDE + 16 * (i / NDT) + 8 * half);
#pragma unroll
      for (int i = 0; i < 4 * NDT; ++i)
        o[i % NDT] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vfr[i], pf[i / NDT], o[i % NDT], 0, 0, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
#pragma unroll
      for (int i = 0; i < 4 * NDT - 3; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 3, 0);
    }
  }
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (qi < n) {
    const float inv = 1.0f / l_tot;
    half_t* orow = out + ((size_t)cu[b] + qi) * out_ld + (size_t)h * HD;
#pragma unroll
    for (int t = 0; t < NDT; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int dd = 32 * t + 8 * g + 4 * half;
        if (dd < HD) {  // HD is a multiple of 4, so the 4 columns are in range together
          f16x4_t v;
#pragma unroll
          for (int u = 0; u < 4; ++u) v[u] = from_f32<half_t>(o[t][4 * g + u] * inv);
          *(f16x4_t*)(orow + dd) = v;
        }
      }
  }
}

template <int HD>
static void launch_fa(const void* q, const void* kc, const void* vc, long kv_extra, int B, int Lmax,
                      const int* len, const int* cu, const int* kvoff, int H, void* out, int out_ld, hipStream_t s) {
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)HD);
  dim3 grid((Lmax + FA_BQ - 1) / FA_BQ, H, B);
  hipLaunchKernelGGL(attn_prefill_mfma<HD>, grid, dim3(256), 0, s, (const half_t*)q, (const half_t*)kc,
                     (const half_t*)vc, kv_extra, len, cu, kvoff, H, scale_log2e, (half_t*)out, out_ld);
}

hipError_t launch_attn_prefill(int dtype, const void* q, const void* kc, const void* vc, long kv_extra,
                               int B, int Lmax, const int* len, const int* cu, const int* kvoff, int H, int hd,
                               void* out, int out_ld, hipStream_t s) {
  if (hd > 256) return hipErrorInvalidValue;
  if (dtype == 1) {
    switch (hd) {
      case 16: launch_fa<16>(q, kc, vc, kv_extra, B, Lmax, len, cu, kvoff, H, out, out_ld, s); return hipGetLastError();
      case 64: launch_fa<64>(q, kc, vc, kv_extra, B, Lmax, len, cu, kvoff, H, out, out_ld, s); return hipGetLastError();
      case 80: launch_fa<80>(q, kc, vc, kv_extra, B, Lmax, len, cu, kvoff, H, out, out_ld, s); return hipGetLastError();
      case 128: launch_fa<128>(q, kc, vc, kv_extra, B, Lmax, len, cu, kvoff, H, out, out_ld, s); return hipGetLastError();
      case 256: launch_fa<256>(q, kc, vc, kv_extra, B, Lmax, len, cu, kvoff, H, out, out_ld, s); return hipGetLastError();
      default: break;  // other head sizes: generic kernel below
    }
  }
  const size_t sh = sizeof(float) * (32 * hd + 32 * (hd + 1) + 32 * hd + 32 * 33 + 96);
  const float scale = 1.0f / sqrtf((float)hd);
  dim3 grid((Lmax + 31) / 32, H, B);
  if (dtype == 0) {
    if (sh > 65536)
      (void)hipFuncSetAttribute((const void*)attn_prefill_generic<float>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)sh);
    hipLaunchKernelGGL(attn_prefill_generic<float>, grid, dim3(256), sh, s, (const float*)q, (const float*)kc,
                       (const float*)vc, kv_extra, len, cu, kvoff, H, hd, scale, (float*)out, out_ld);
  } else {
    if (sh > 65536)
      (void)hipFuncSetAttribute((const void*)attn_prefill_generic<half_t>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)sh);
    hipLaunchKernelGGL(attn_prefill_generic<half_t>, grid, dim3(256), sh, s, (const half_t*)q, (const half_t*)kc,
                       (const half_t*)vc, kv_extra, len, cu, kvoff, H, hd, scale, (half_t*)out, out_ld);
  }
  return hipGetLastError();
}

// =================================================================================================
// Decode attention: one block per (head, sequence).
// =================================================================================================
template <typename T>
__global__ void __launch_bounds__(256)
    attn_decode_generic(const T* __restrict__ q, const T* __restrict__ kc, const T* __restrict__ vc,
                        long kv_extra, const int* __restrict__ len, int ctx_add,
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
  const T* kb = kc + ((size_t)kvoff[b] * H + (size_t)h * (len[b] + kv_extra)) * hd;
  const T* vb = vc + ((size_t)kvoff[b] * H + (size_t)h * (len[b] + kv_extra)) * hd;
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
    out[(size_t)b * d + (size_t)h * hd + tid] = from_f32<T>(sum > 0.f ? o / sum : 0.f);  // empty context: zero row
  }
}


// =================================================================================================
// Decode attention for fp16 caches, head_dim HD a multiple of 8.  HBM-bound: a (sequence, head)
// pair owns one contiguous run of ctx*HD halfs of K and of V, which the block reads as a flat
// stream of 16-byte chunks, 64 lanes x 16 B per wave instruction.
//   lane = (g, part): part = chunk within a row (HD/8 per row), g = row within the wave's group
//   of G = 64 / (HD/8) rows.  Phase 1: 8-element partial dot products (v_dot2_f32_f16) combined
//   across the lanes of a row (butterfly when HD/8 is a power of two, else through LDS).
//   Phase 2: softmax over the scores in LDS.  Phase 3: the same flat stream over V, each lane
//   accumulating its 8 output dims in fp32; groups and waves are summed through LDS.
// =================================================================================================
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;

template <int HD>
__global__ void __launch_bounds__(256)
    attn_decode_f16(const half_t* __restrict__ q, const half_t* __restrict__ kc, const half_t* __restrict__ vc,
                    long kv_extra, const int* __restrict__ len, int ctx_add, const int* __restrict__ kvoff,
                    int H, float scale, half_t* __restrict__ out) {
  constexpr int CPR = HD / 8;             // 16-byte chunks per row
  constexpr int G = 64 / CPR;             // rows per wave instruction
  constexpr int ACTIVE = G * CPR;         // lanes that carry a chunk
  constexpr bool POW2 = (CPR & (CPR - 1)) == 0;
  extern __shared__ float smem[];
  __shared__ float red[8];
  const int h = blockIdx.x, b = blockIdx.y;
  const int ctx = len[b] + ctx_add;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane / CPR, part = lane - g * CPR;
  const bool active = lane < ACTIVE;
  float* sc = smem;                              // [ctx_pad] scores, then probabilities
  const int ctx_pad = (ctx + 3) & ~3;
  float* scratch = sc + ctx_pad;                 // partial dots (non-power-of-two CPR) / output partials
  const int d = H * HD;
  const half_t* kb = kc + ((size_t)kvoff[b] * H + (size_t)h * (len[b] + kv_extra)) * HD;
  const half_t* vb = vc + ((size_t)kvoff[b] * H + (size_t)h * (len[b] + kv_extra)) * HD;

  // this lane's 8 query values, as 4 packed pairs
  f16x2_t qv[4];
  {
    const half_t* qp = q + (size_t)b * d + (size_t)h * HD + part * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) qv[i] = active ? *(const f16x2_t*)(qp + 2 * i) : (f16x2_t){0, 0};
  }
  const int n_it = (ctx + G - 1) / G;  // wave instructions needed to cover ctx rows
  // ---- phase 1: scores.  Four wave-loads are issued before the first is consumed: with one load
  //      per wave in flight a CU holds too few bytes in flight to cover the HBM round trip.
  for (int it0 = wave; it0 < n_it; it0 += 16) {
    u32x4_t kv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = (it0 + 4 * u) * G + g;
      kv[u] = (u32x4_t){0, 0, 0, 0};
      if (active && j < ctx) kv[u] = *(const u32x4_t*)(kb + (size_t)j * HD + part * 8);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int it = it0 + 4 * u;
      const int j = it * G + g;
      float pd = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t w = kv[u][i];
        f16x2_t kk;
        __builtin_memcpy(&kk, &w, 4);
        pd = __builtin_amdgcn_fdot2(kk, qv[i], pd, false);
      }
      if (POW2) {
#pragma unroll
        for (int o = CPR >> 1; o > 0; o >>= 1) pd += __shfl_xor(pd, o, 64);
        if (part == 0 && j < ctx) sc[j] = pd * scale;
      } else {
        if (active && it < n_it) scratch[it * ACTIVE + lane] = pd;  // row j's CPR partials are contiguous
      }
    }
  }
  __syncthreads();
  if (!POW2) {
    for (int j = tid; j < ctx; j += 256) {
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < CPR; ++c) s += scratch[j * CPR + c];  // (j/G)*ACTIVE + (j%G)*CPR == j*CPR
      sc[j] = s * scale;
    }
    __syncthreads();
  }
  // ---- phase 2: softmax
  float mx = -INFINITY;
  for (int j = tid; j < ctx; j += 256) mx = fmaxf(mx, sc[j]);
  mx = wave_max(mx);
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  float sum = 0.f;
  for (int j = tid; j < ctx; j += 256) {
    const float p = __expf(sc[j] - mx);
    sc[j] = p;
    sum += p;
  }
  sum = wave_sum(sum);
  if (lane == 0) red[4 + wave] = sum;
  __syncthreads();
  const float den = red[4] + red[5] + red[6] + red[7];
  const float inv = den > 0.f ? 1.0f / den : 0.f;  // an empty context (all-pad sequence) gives a zero row
  // ---- phase 3: out = sum_j p_j V[j]
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int it0 = wave; it0 < n_it; it0 += 16) {
    u32x4_t vv[4];
    float pj[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = (it0 + 4 * u) * G + g;
      const bool ok = active && j < ctx;
      vv[u] = (u32x4_t){0, 0, 0, 0};
      if (ok) vv[u] = *(const u32x4_t*)(vb + (size_t)j * HD + part * 8);
      pj[u] = ok ? sc[j] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t w = vv[u][i];
        f16x2_t x;
        __builtin_memcpy(&x, &w, 4);
        acc[2 * i] = fmaf(pj[u], (float)x[0], acc[2 * i]);
        acc[2 * i + 1] = fmaf(pj[u], (float)x[1], acc[2 * i + 1]);
      }
    }
  }
  __syncthreads();  // the partial-dot scratch is dead; reuse it for [wave][g][HD] output partials
  if (active) {
#pragma unroll
    for (int i = 0; i < 8; ++i) scratch[(wave * G + g) * HD + part * 8 + i] = acc[i];
  }
  __syncthreads();
  for (int e = tid; e < HD; e += 256) {
    float o = 0.f;
#pragma unroll
    for (int r = 0; r < 4 * G; ++r) o += scratch[r * HD + e];
    out[(size_t)b * d + (size_t)h * HD + e] = from_f32<half_t>(o * inv);
  }
}

template <int HD>
static hipError_t launch_dec(const void* q, const void* kc, const void* vc, long kv_extra, int B,
                             const int* len, int ctx_add, int ctx_max, const int* kvoff, int H, void* out,
                             hipStream_t s) {
  constexpr int CPR = HD / 8, G = 64 / CPR;
  const size_t part = ((CPR & (CPR - 1)) == 0) ? 0 : (size_t)((ctx_max + G - 1) / G) * G * CPR;
  const size_t sh = sizeof(float) * (((ctx_max + 3) & ~3) + std::max(part, (size_t)4 * G * HD));
  if (sh > 160 * 1024) return hipErrorInvalidValue;
  if (sh > 65536)
    (void)hipFuncSetAttribute((const void*)attn_decode_f16<HD>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh);
  hipLaunchKernelGGL(attn_decode_f16<HD>, dim3(H, B), dim3(256), sh, s, (const half_t*)q, (const half_t*)kc,
                     (const half_t*)vc, kv_extra, len, ctx_add, kvoff, H, 1.0f / sqrtf((float)HD),
                     (half_t*)out);
  return hipGetLastError();
}

hipError_t launch_attn_decode(int dtype, const void* q, const void* kc, const void* vc, long kv_extra,
                              int B, const int* len, int ctx_add, int ctx_max, const int* kvoff, int H, int hd,
                              void* out, hipStream_t s) {
  if (hd > 256) return hipErrorInvalidValue;
  if (dtype == 1) {
    switch (hd) {
      case 16: return launch_dec<16>(q, kc, vc, kv_extra, B, len, ctx_add, ctx_max, kvoff, H, out, s);
      case 64: return launch_dec<64>(q, kc, vc, kv_extra, B, len, ctx_add, ctx_max, kvoff, H, out, s);
      case 80: return launch_dec<80>(q, kc, vc, kv_extra, B, len, ctx_add, ctx_max, kvoff, H, out, s);
      case 128: return launch_dec<128>(q, kc, vc, kv_extra, B, len, ctx_add, ctx_max, kvoff, H, out, s);
      case 256: return launch_dec<256>(q, kc, vc, kv_extra, B, len, ctx_add, ctx_max, kvoff, H, out, s);
      default: break;  // other head sizes: generic kernel below
    }
  }
  const size_t sh = sizeof(float) * (hd + 256 + ctx_max);
  if (sh > 65536) return hipErrorInvalidValue;
  const float scale = 1.0f / sqrtf((float)hd);
  dim3 grid(H, B);
  if (dtype == 0)
    hipLaunchKernelGGL(attn_decode_generic<float>, grid, dim3(256), sh, s, (const float*)q, (const float*)kc,
                       (const float*)vc, kv_extra, len, ctx_add, kvoff, H, hd, scale, (float*)out);
  else
    hipLaunchKernelGGL(attn_decode_generic<half_t>, grid, dim3(256), sh, s, (const half_t*)q, (const half_t*)kc,
                       (const half_t*)vc, kv_extra, len, ctx_add, kvoff, H, hd, scale, (half_t*)out);
  return hipGetLastError();
}

}  // namespace rlhf
