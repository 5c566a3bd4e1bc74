// C[M,N] = A[M,K] * W[N,K]^T (+ bias, + epilogue).  Both operands are K-contiguous, which is the
// natural operand order of the CDNA matrix cores: every lane loads 8 consecutive K elements of one
// row of A and of one row of W.
//
//  * bf16 mode (fp16 operands), many rows: v_mfma_f32_32x32x16_f16, 256x256 block tile, 8 waves
//    (2x4) of 128x64, K step 64 (a tile row is one full 128-byte line), two 64 KB LDS stages
//    filled directly from global memory, XOR-swizzled 16-byte chunks (conflict-free ds_read_b128),
//    workgroup ids remapped so that the 32 tiles resident on one XCD share A and W panels in that
//    XCD's L2.  Few rows (decode): 128x64 tiles staged through registers, split over K.
//  * fp32: plain FMA tile kernel (check mode only; not tuned).
#include <algorithm>
#include <type_traits>

#include "common.h"

namespace rlhf {

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

// GELU for fp16 outputs: x * Phi(x) with Phi(x) ~ 1 / (1 + exp(-x * (c1 + c3 x^2 + c5 x^4))), the
// coefficients fitted to the erf form over [-9, 9]: absolute error below 2.6e-5 everywhere (the
// fp16 result itself is rounded to 2^-11 relative), one exp and one reciprocal per element.  x^2 is
// capped at 64: beyond |x| = 8 the polynomial would bend back, and the sigmoid is saturated there.
// The constants carry the factor -log2(e) of the base-2 exponential.
__device__ __forceinline__ float gelu_f16out(float x) {
  const float s = fminf(x * x, 64.0f);
  float p = fmaf(1.01426504e-3f, s, -1.06775735e-1f);
  p = fmaf(p, s, -2.30112140f);
  const float e = __builtin_amdgcn_exp2f(x * p);  // exp(-u); inf for very negative x gives 1/inf = 0
  return x * __frcp_rn(1.0f + e);
}

template <int EPI, typename T>
__device__ __forceinline__ void epilogue_store(void* out, size_t idx, float acc, float bias) {
  if (EPI == EPI_BIAS) {
    ((T*)out)[idx] = from_f32<T>(acc + bias);
  } else if (EPI == EPI_BIAS_GELU) {
    ((T*)out)[idx] = from_f32<T>(gelu_erf(acc + bias));
  } else if (EPI == EPI_BIAS_RESADD) {
    ((float*)out)[idx] += acc + bias;
  } else {
    ((float*)out)[idx] = acc;
  }
}

// =================================================================================================
// fp16-operand MFMA kernel
// =================================================================================================
constexpr int TK = 64;
constexpr int GROUP_M = 4;  // m-tiles per scheduling group

// LDS position (in halfs) of logical 16-byte chunk c (0..7) of tile row r (A rows first, then W
// rows): rows are 128 B apart; the chunk index is XORed with bits 1..3 of the row so that 16
// consecutive rows reading the same logical chunk hit 16 different 16-byte bank groups.
__device__ __forceinline__ int lds_pos(int r, int c) { return r * TK + ((c ^ ((r >> 1) & 7)) << 3); }

// MT x NT: 32x32 accumulator tiles per wave along M and N; the block is 2x2 waves.
// PF: k-steps of global loads kept in flight in registers; OCC: blocks per CU the register
// allocation is sized for.
template <int EPI, int MT, int NT, int PF, int OCC>
__global__ void __launch_bounds__(256, OCC)
    gemm_f16_kernel(const half_t* __restrict__ A, const half_t* __restrict__ W, const bf16_t* __restrict__ bias,
                    void* __restrict__ out, int M_max, const int* __restrict__ M_dev, int M_sub, int N, int K,
                    int ldo, int nb_m, int nb_n, int ksplit, int lda, int ldw) {
  constexpr int TM = 64 * MT, TN = 64 * NT;
  constexpr int NLD = (TM + TN) / 32;  // 16-byte chunks per thread per k-step
  constexpr int NLD_A = TM / 32;
  __shared__ __attribute__((aligned(16))) uint16_t lds[(TM + TN) * TK];
  const int M = M_dev ? min(M_max, *M_dev - M_sub) : M_max;

  // ---- tile assignment: workgroup w runs on XCD w % 8; give each XCD a contiguous run of tiles,
  //      ordered so that consecutive tiles walk GROUP_M m-tiles for each n-tile.
  //      The split uses the device-side row count, so that tiles past it do not leave XCDs idle.
  nb_m = min(nb_m, (M + TM - 1) / TM);
  const int total = nb_m * nb_n;
  const int per_xcd = (total + 7) >> 3;
  if ((int)(blockIdx.x >> 3) >= per_xcd) return;
  const int lt = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (lt >= total) return;
  const int group_sz = GROUP_M * nb_n;
  const int grp = lt / group_sz, rem = lt - grp * group_sz;
  const int gm = min(GROUP_M, nb_m - grp * GROUP_M);
  const int tm = grp * GROUP_M + rem % gm, tn = rem / gm;
  const int m0 = tm * TM, n0 = tn * TN;
  if (m0 >= M) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave >> 1) * (32 * MT), wn = (wave & 1) * (32 * NT);

  // ---- global -> register staging: a row of the tile is one full 128-byte line, read by 8
  //      consecutive lanes; thread handles rows ld_r + 32*i (A rows first, then W rows)
  const int ld_r = tid >> 3, ld_c = tid & 7;
  // element offset of this thread's chunk i from A (i < NLD_A) or W, recomputed per use: keeping
  // NLD offsets live would push the kernel past 256 registers and into scratch
  auto goff = [&](int i) -> uint32_t {
    const int r = ld_r + 32 * (i < NLD_A ? i : i - NLD_A);
    return (uint32_t)((i < NLD_A ? min(m0 + r, M - 1) * lda : min(n0 + r, N - 1) * ldw) + ld_c * 8);
  };
  const int st_off = lds_pos(ld_r, ld_c);  // + 32*i rows: (r>>1)&7 is unchanged by adding 32*i
  u32x4_t stage[PF][NLD];
  // Full K tiles load unconditionally (a select on the loaded value would force the wave to wait
  // for the data right away); only a ragged last tile takes the guarded form.
  auto load_global = [&](int set, int k0) {
    if (k0 + TK <= K) {
#pragma unroll
      for (int i = 0; i < NLD; ++i) stage[set][i] = *(const u32x4_t*)((i < NLD_A ? A : W) + goff(i) + k0);
    } else {
      const bool kok = k0 + ld_c * 8 < K;
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        u32x4_t z = {0, 0, 0, 0};
        if (kok) z = *(const u32x4_t*)((i < NLD_A ? A : W) + goff(i) + k0);
        stage[set][i] = z;
      }
    }
  };
  auto store_lds = [&](int set) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) *(u32x4_t*)(lds + st_off + 32 * i * TK) = stage[set][i];
  };

  // ---- fragment addressing: lane reads row (lane & 31) of a 32-row fragment, logical chunk
  //      2*ks + (lane >> 5); the swizzle key depends on (lane & 31) >> 1 only.
  const int key = ((lane & 31) >> 1) & 7;
  const int fr = (lane & 31) * TK;
  const int a_off = wm * TK + fr, w_off = (TM + wn) * TK + fr;

  f32x16_t acc[NT][MT];  // [j over N][i over M]
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[j][i][e] = 0.f;

  // split-K: block z = blockIdx.y owns k-steps [kt0, nk); its fp32 partial sums go to slab z of
  // `out` ([ksplit][M_max][ldo]) and a second kernel adds the slabs in a fixed order
  const int nk_all = (K + TK - 1) / TK;
  const int per_split = (nk_all + ksplit - 1) / ksplit;
  const int kt0 = blockIdx.y * per_split;
  const int nk = min(nk_all, kt0 + per_split);
  if (ksplit > 1) out = (float*)out + (size_t)blockIdx.y * M_max * ldo;
#pragma unroll
  for (int p = 0; p < PF; ++p)
    if (kt0 + p < nk) load_global(p, (kt0 + p) * TK);
  for (int kt = kt0; kt < nk; kt += PF) {
#pragma unroll
   for (int p = 0; p < PF; ++p) {
    if (kt + p >= nk) break;
    store_lds(p);
    __syncthreads();
    if (kt + p + PF < nk) load_global(p, (kt + p + PF) * TK);  // in flight for PF k-steps of math
    // Fragments are double-buffered by hand and the scheduler is fenced, so that the LDS reads of
    // sub-step ks+1 are in flight while the matrix instructions of sub-step ks issue (left alone,
    // the compiler re-reads into one register quad and waits before every few MFMAs).
    constexpr int FB = (MT * NT > 8) ? 2 : 1;  // fragment buffers: two when one wave owns the SIMD
    f16x8_t fa[FB][MT], fw[FB][NT];
    auto load_frags = [&](int buf, int ks) {
      const int ch = ((2 * ks + (lane >> 5)) ^ key) << 3;
#pragma unroll
      for (int i = 0; i < MT; ++i) fa[buf][i] = *(const f16x8_t*)(lds + a_off + i * 32 * TK + ch);
#pragma unroll
      for (int j = 0; j < NT; ++j) fw[buf][j] = *(const f16x8_t*)(lds + w_off + j * 32 * TK + ch);
    };
    if (FB == 2) load_frags(0, 0);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      if (FB == 2) {
        if (ks < 3) load_frags((ks + 1) & 1, ks + 1);
      } else {
        load_frags(0, ks);
      }
      __builtin_amdgcn_sched_barrier(0);
      // weights as the first operand: accumulator element e of a lane is then
      // (n = 8*(e/4) + 4*(lane/32) + e%4, m = lane%32), i.e. 4 consecutive output columns per lane
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int i = 0; i < MT; ++i)
          acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fw[ks & (FB - 1)][j], fa[ks & (FB - 1)][i], acc[j][i],
                                                             0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
   }
  }

  // ---- epilogue
  const bool vec_ok = (ldo & 3) == 0;
#pragma unroll
  for (int j = 0; j < NT; ++j) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int nb = n0 + wn + 32 * j + 8 * g + 4 * (lane >> 5);
      if (nb >= N) continue;
      float bv[4] = {0.f, 0.f, 0.f, 0.f};
      if (EPI != EPI_F32 && bias) {
#pragma unroll
        for (int u = 0; u < 4; ++u) bv[u] = (nb + u < N) ? to_f32(bias[nb + u]) : 0.f;
      }
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        const int row = m0 + wm + 32 * i + (lane & 31);
        if (row >= M) continue;
        const size_t o = (size_t)row * ldo + nb;
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = acc[j][i][4 * g + u] + bv[u];
        if (vec_ok && nb + 4 <= N) {
          if (EPI == EPI_BIAS || EPI == EPI_BIAS_GELU) {
            f16x4_t h;
#pragma unroll
            for (int u = 0; u < 4; ++u) h[u] = from_f32<half_t>(EPI == EPI_BIAS_GELU ? gelu_f16out(v[u]) : v[u]);
            *(f16x4_t*)((half_t*)out + o) = h;
          } else if (EPI == EPI_BIAS_RESADD) {
            f32x4_t x = *(f32x4_t*)((float*)out + o);
#pragma unroll
            for (int u = 0; u < 4; ++u) x[u] += v[u];
            *(f32x4_t*)((float*)out + o) = x;
          } else {
            f32x4_t x = {v[0], v[1], v[2], v[3]};
            *(f32x4_t*)((float*)out + o) = x;
          }
        } else {
#pragma unroll
          for (int u = 0; u < 4; ++u)
            if (nb + u < N) epilogue_store<EPI, half_t>(out, o + u, acc[j][i][4 * g + u], bv[u]);
        }
      }
    }
  }
}

// =================================================================================================
// fp32 check-mode kernel: 64x64 tile, 256 threads, 4x4 outputs per thread, K step 16.
// =================================================================================================
template <int EPI>
__global__ void __launch_bounds__(256)
    gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ W, const float* __restrict__ bias,
                    void* __restrict__ out, int M_max, const int* __restrict__ M_dev, int M_sub, int N, int K, int ldo) {
  __shared__ float As[16][64 + 4], Ws[16][64 + 4];
  const int M = M_dev ? min(M_max, *M_dev - M_sub) : M_max;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  if (m0 >= M) return;
  const int tid = threadIdx.x;
  const int lr = tid >> 2, lk = (tid & 3) * 4;
  const int ty = tid >> 4, tx = tid & 15;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    const int ar = min(m0 + lr, M - 1), wr = min(n0 + lr, N - 1);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int k = k0 + lk + e;
      As[lk + e][lr] = k < K ? A[(size_t)ar * K + k] : 0.f;
      Ws[lk + e][lr] = k < K ? W[(size_t)wr * K + k] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = As[k][ty * 4 + i];
        w[i] = Ws[k][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = m0 + ty * 4 + i;
    if (row >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = n0 + tx * 4 + j;
      if (col >= N) continue;
      const float bv = (EPI != EPI_F32 && bias) ? bias[col] : 0.f;
      epilogue_store<EPI, float>(out, (size_t)row * ldo + col, acc[i][j], bv);
    }
  }
}

// =================================================================================================
// Large-M kernel: 256x256 block tile, one block per CU, 8 waves of 128x64 (two per SIMD; a 4-wave
// form, 128x128 per wave, is kept as a template option).  Tiles go global -> LDS directly (global_load_lds, 16 bytes per lane: a wave
// instruction fills 1 KB; no staging registers, no ds_write) into TWO 64 KB stages of K depth 64.
// The depth is what matters: a tile row is then one full 128-byte line per stage.  With half
// lines (K depth 32, more and smaller stages) every line was requested twice from L2, one half per
// k-step, and the matrix cores waited on that request stream; fetching whole lines removed the
// stall, and a lookahead of one stage proved as good as three.  One raw s_barrier per stage with
// an explicit s_waitcnt; the tile loads and fragment reads of a stage are dealt out one at a time
// between the matrix instructions (scheduling fences
// keep the order), so each issues in the shadow of a matrix instruction.  Each lane picks its
// global chunk so that the linear LDS image is the XOR-swizzled layout the fragment reads expect
// (conflict-free ds_read_b128).
// =================================================================================================
#define RLHF_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define RLHF_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
constexpr int kDmaWaves = 8;                // waves per block of the large-M kernel (4 or 8)
constexpr int DK = 64;                      // K depth of one stage: 128 bytes per tile row
constexpr int DSTAGE = (256 + 256) * DK;    // halfs per stage (64 KB)

// KMAJ: both operands are given K-major -- A as [K, M] and W as [K, N], row-major, lda / ldw their row strides
// (the weight-gradient products of a backward pass: out = A^T W over the batch's rows, no transposed copies).  A stage
// then holds 64 k-rows of 512 bytes per operand, and a matrix-instruction operand slice (8 consecutive k of one
// column) comes from two transposing LDS reads (ds_read_b64_tr_b16: within a group of 16 lanes, lane i receives the
// (i mod 4)-th element of the 8-byte items addressed by lanes i/4, i/4+4, i/4+8, i/4+12; with lane r pointing at row
// k + r/4, columns 4(r mod 4).. of the tile, lane i gets column i of rows k .. k+3).  16-byte chunk c of k-row k sits at
// chunk c ^ 2(k mod 4) of the row, so that the four rows one group reads fall into four different 32-byte bank groups.
template <int EPI, int WAVES, bool KMAJ = false>
__global__ void __launch_bounds__(64 * WAVES, 1)
    gemm_f16_dma_kernel(const half_t* __restrict__ A, const half_t* __restrict__ W, const bf16_t* __restrict__ bias,
                        void* __restrict__ out, int M_max, const int* __restrict__ M_dev, int M_sub, int N, int K,
                        int ldo, int nb_m, int nb_n, int lda, int ldw, const bf16_t* __restrict__ bias2,
                        LseArgs lse, QkvArgs qk, int k_slice, size_t slab) {
  // WAVES = 4: one wave per SIMD, each 128 x 128 of the tile (256 accumulator registers).
  // WAVES = 8: two waves per SIMD, each 128 x 64 (128 accumulator registers): what one wave cannot
  // overlap (waits, epilogue arithmetic against stores) the SIMD's other wave fills.
  constexpr int TM = 256, TN = 256, MT = 4, NT = WAVES == 8 ? 2 : 4;
  constexpr int WN = 32 * NT;         // columns per wave
  constexpr int NWN = TN / WN;        // waves along N
  constexpr int NLD = 64 / WAVES;     // tile loads per wave per stage
  constexpr int NMF = MT * NT;        // matrix instructions per wave per sub-step
  __shared__ __attribute__((aligned(16))) uint16_t lds0[DSTAGE];
  __shared__ __attribute__((aligned(16))) uint16_t lds1[DSTAGE];
  const int M = M_dev ? min(M_max, *M_dev - M_sub) : M_max;
  nb_m = min(nb_m, (M + TM - 1) / TM);
  const int total = nb_m * nb_n;
  const int per_xcd = (total + 7) >> 3;
  if ((int)(blockIdx.x >> 3) >= per_xcd) return;
  const int lt = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (lt >= total) return;
  const int group_sz = GROUP_M * nb_n;
  const int grp = lt / group_sz, rem = lt - grp * group_sz;
  const int gm = min(GROUP_M, nb_m - grp * GROUP_M);
  const int tm = grp * GROUP_M + rem % gm, tn = rem / gm;
  const int m0 = tm * TM, n0 = tn * TN;

  // K split over blockIdx.y (weight-gradient products: few tiles, a very long K): slice z covers
  // [z * k_slice, min(K, (z + 1) * k_slice)) and writes its fp32 result to slab z of `out`
  if (k_slice > 0) {
    const int kb = blockIdx.y * k_slice;
    A += KMAJ ? (size_t)kb * lda : (size_t)kb;
    W += KMAJ ? (size_t)kb * ldw : (size_t)kb;
    K = min(k_slice, K - kb);
    out = (float*)out + (size_t)blockIdx.y * slab;
  }
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps LDS bases in SGPRs
  const int wm = (wave / NWN) * 128, wn = (wave % NWN) * WN;

  // ---- direct loads: a stage row is 128 B (8 chunks); wave-load j (= NLD*wave + i, i < NLD) fills
  //      rows 8j .. 8j+7 (rows < 256: A, else W); lane l lands at row 8j + l/8, physical chunk l%8,
  //      and therefore fetches logical chunk (l%8) ^ ((row>>1)&7)
  uint32_t goff[NLD];
  const int gld = wave < WAVES / 2 ? lda : ldw;  // row stride of the operand this wave loads
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    if (KMAJ) {
      // wave-load j covers k-rows 2j', 2j'+1 (j' = j mod 32) of its operand; lane l lands at k-row 2j' + l/32,
      // physical chunk l%32, and fetches logical chunk (l%32) ^ 2(k-row mod 4); columns past the operand's width
      // re-read its last chunk (those output columns are never stored)
      const int krow = 2 * ((NLD * wave + i) & 31) + (lane >> 5);
      const int c = (lane & 31) ^ (2 * (krow & 3));
      const int colb = wave < WAVES / 2 ? min(m0 + c * 8, M - 8) : min(n0 + c * 8, N - 8);
      goff[i] = (uint32_t)(krow * gld + colb);
    } else {
      const int row = 8 * (NLD * wave + i) + (lane >> 3);
      const int c = (lane & 7) ^ ((row >> 1) & 7);
      goff[i] = (uint32_t)((row < TM ? min(m0 + row, M - 1) * lda : min(n0 + row - TM, N - 1) * ldw) + c * 8);
    }
  }
  const half_t* gbase = wave < WAVES / 2 ? A : W;  // the first half of the waves loads A rows, the second W rows
  auto load_one = [&](uint16_t* stage, int k0, int i) {
    __builtin_amdgcn_global_load_lds(RLHF_GLOBAL_PTR(gbase + goff[i] + (KMAJ ? (size_t)k0 * gld : (size_t)k0)),
                                     RLHF_LDS_PTR(stage + (8 * (NLD * wave + i)) * DK), 16, 0, 0);
  };

  const int l32 = lane & 31, hf = lane >> 5;
  const int key = (l32 >> 1) & 7;
  const int a_off = (wm + l32) * DK, w_off = (TM + wn + l32) * DK;
  // sub-step s (16 of the 64 k of a stage) reads logical chunks 2s and 2s+1: one per half-wave
  // KMAJ: sub-step s reads k-rows 16s + 8hf .. +7 (256 halfs per row); the column part of a lane's address, with
  // the row swizzle, is fixed per fragment
  const int ch0 = KMAJ ? (0 + 8 * hf) * 256 : ((0 + hf) ^ key) << 3, ch1 = KMAJ ? (16 + 8 * hf) * 256 : ((2 + hf) ^ key) << 3,
            ch2 = KMAJ ? (32 + 8 * hf) * 256 : ((4 + hf) ^ key) << 3, ch3 = KMAJ ? (48 + 8 * hf) * 256 : ((6 + hf) ^ key) << 3;
  int koff[MT + NT];
  if (KMAJ) {
    const int r = lane & 15, gsel = (lane >> 4) & 1;
#pragma unroll
    for (int q = 0; q < MT + NT; ++q) {
      const int colb = (q < MT ? wm + 32 * q : wn + 32 * (q - MT)) + 16 * gsel;  // first column of the group's 16
      const int chunk = ((colb >> 3) + ((r & 3) >> 1)) ^ (2 * ((r >> 2) & 3));
      koff[q] = (q < MT ? 0 : 64 * 256) + (r >> 2) * 256 + chunk * 8 + (r & 1) * 4;
    }
  }

  f32x16_t acc[NT][MT];
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[j][i][e] = 0.f;

  // fragment buffers, used alternately by the four sub-steps of a stage.  Weights are the first
  // matrix operand: accumulator element e of a lane is then (n = 8*(e/4) + 4*(lane/32) + e%4,
  // m = lane%32), i.e. 4 consecutive output columns per lane
  f16x8_t fa0[MT], fw0[NT], fa1[MT], fw1[NT];
  auto frag_one = [&](const uint16_t* ls, int ch, int q, f16x8_t* fa, f16x8_t* fw) {
    if (KMAJ) {
      typedef __attribute__((ext_vector_type(4))) short s16x4_t;
      typedef __attribute__((ext_vector_type(8))) short s16x8_t;
      typedef __attribute__((address_space(3))) s16x4_t* lds4_t;
      const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4_t)(ls + koff[q] + ch));
      const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4_t)(ls + koff[q] + ch + 4 * 256));
      const s16x8_t b = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      const f16x8_t v = __builtin_bit_cast(f16x8_t, b);
      if (q < MT) fa[q] = v;
      else fw[q - MT] = v;
    } else if (q < MT) {
      fa[q] = *(const f16x8_t*)(ls + a_off + q * 32 * DK + ch);
    } else {
      fw[q - MT] = *(const f16x8_t*)(ls + w_off + (q - MT) * 32 * DK + ch);
    }
  };
  // NMF matrix instructions on (FA, FW); after the n-th, fragment read n (n < MT + NT) of the next
  // sub-step from (LS, CH) into (GA, GW) and, if LOAD, tile load n of the stage at K offset KL
#define RLHF_SUB(FA, FW, LS, CH, GA, GW, LOAD, LSTAGE, KL)                                        \
  _Pragma("unroll") for (int n = 0; n < NMF; ++n) {                                               \
    const int mi = ((n >> 2) & 1) ? 3 - (n & 3) : (n & 3); /* serpentine: one operand changes at a time */ \
    acc[n >> 2][mi] = __builtin_amdgcn_mfma_f32_32x32x16_f16(FW[n >> 2], FA[mi],                  \
                                                             acc[n >> 2][mi], 0, 0, 0);           \
    __builtin_amdgcn_sched_barrier(0);                                                            \
    if (n < MT + NT) frag_one(LS, CH, n, GA, GW);                                                 \
    if (LOAD && n < NLD) load_one(LSTAGE, KL, n);                                                 \
    __builtin_amdgcn_sched_barrier(0);                                                            \
  }
  // vmcnt(0) lgkmcnt(0) + barrier: every wave's tile loads have landed and every wave has finished
  // reading the current stage
#define RLHF_WAIT_BARRIER()                      \
  __builtin_amdgcn_sched_barrier(0);             \
  asm volatile("" ::: "memory");                 \
  __builtin_amdgcn_s_waitcnt(0x0070);            \
  __builtin_amdgcn_s_barrier();                  \
  asm volatile("" ::: "memory");                 \
  __builtin_amdgcn_sched_barrier(0);
  // One stage (K depth 64).  The first three sub-steps read their successors' fragments from CUR.
  // After the barrier CUR is free and OTHER holds the next stage: the last sub-step reads the next
  // stage's first fragments from OTHER and issues the loads of the stage after that into CUR, so a
  // load has a whole stage of matrix work to land.
#define RLHF_STAGE(CUR, OTHER, KT)                                                                \
  {                                                                                               \
    const int kload = min((KT) + 2, nk - 1) * DK;                                                 \
    RLHF_SUB(fa0, fw0, CUR, ch1, fa1, fw1, false, CUR, 0)                                         \
    RLHF_SUB(fa1, fw1, CUR, ch2, fa0, fw0, false, CUR, 0)                                         \
    RLHF_SUB(fa0, fw0, CUR, ch3, fa1, fw1, false, CUR, 0)                                         \
    RLHF_WAIT_BARRIER()                                                                           \
    RLHF_SUB(fa1, fw1, OTHER, ch0, fa0, fw0, true, CUR, kload)                                    \
  }

  // K is a multiple of 2*DK here (the launcher routes other shapes to the staged kernel), so the
  // loop is branch-free: past the end the final tile is re-issued into a stage nobody reads.
  const int nk = K / DK;
#pragma unroll
  for (int i = 0; i < NLD; ++i) load_one(lds0, 0, i);
#pragma unroll
  for (int i = 0; i < NLD; ++i) load_one(lds1, min(1, nk - 1) * DK, i);
  RLHF_WAIT_BARRIER()
#pragma unroll
  for (int q = 0; q < MT + NT; ++q) frag_one(lds0, ch0, q, fa0, fw0);
  for (int kt = 0; kt < nk; kt += 2) {
    RLHF_STAGE(lds0, lds1, kt)
    RLHF_STAGE(lds1, lds0, kt + 1)
  }
#undef RLHF_STAGE
#undef RLHF_SUB
#undef RLHF_WAIT_BARRIER
  __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0): the surplus loads have landed too
  __syncthreads();

  if (EPI == EPI_LSE) {
    // ---- scoring LM head: the logits stay in the accumulators.  A lane holds, for each of its 4
    //      rows (32*i + lane%32), half of the wave's WN columns (the other half is in lane ^ 32):
    //      running max and sum of exp over them, combined across the two half-waves, plus the
    //      target token's z if its column is among this lane's.
    const int part = NWN * tn + (wave % NWN);
    const int T = *lse.T_dev;
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int tr = M_sub + m0 + wm + 32 * i + l32;  // packed row
      const bool row_ok = m0 + wm + 32 * i + l32 < M;
      int tcol = -1;  // target column relative to this wave's first column, or out of range
      if (lse.tgt) {
        const int tg = row_ok && tr < T ? lse.tgt[tr] : -1;
        if (tg >= 0) tcol = tg - (n0 + wn);
      } else if (row_ok && tr + 1 < T && lse.pos[tr + 1] == lse.pos[tr] + 1) {
        tcol = lse.tok[tr + 1] - (n0 + wn);
      }
      float m = -INFINITY, zt = 0.f;
      bool has_t = false;
      float z[NT][16];
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int col = 32 * j + 8 * (e >> 2) + 4 * hf + (e & 3);
          float v = acc[j][i][e] * lse.inv_temperature;
          if (n0 + wn + col >= N) v = -INFINITY;
          if (col == tcol) { zt = v; has_t = true; }
          z[j][e] = v;
          m = fmaxf(m, v);
        }
      m = fmaxf(m, __shfl_xor(m, 32, 64));
      float sum = 0.f;
      if (m > -INFINITY) {
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) sum += __expf(z[j][e] - m);
      }
      sum += __shfl_xor(sum, 32, 64);
      if (row_ok) {
        if (hf == 0) {
          lse.pmax[(size_t)part * lse.stride + tr] = m;
          lse.psum[(size_t)part * lse.stride + tr] = sum;
        }
        if (has_t) lse.ztgt[tr] = zt;
      }
    }
    return;
  }
  // ---- epilogue.  In the accumulator layout a lane owns 4 consecutive columns of ONE row, so a
  //      direct store touches 32 rows with 8-16 bytes each -- partial-line writes that the memory
  //      system handles an order of magnitude slower than full lines.  Each wave therefore
  //      transposes its 128x128 tile through one of the four (now idle) 32 KB LDS stages and stores
  //      16 bytes per lane, 16 lanes per 256-byte row segment.  The LDS image is XOR-swizzled by
  //      row (chunk ^ (row & 15)); accumulator tiles are addressed through compile-time indices
  //      (a loop the compiler declines to unroll would spill all 256 accumulators to scratch).
  // The staging regions are private to a wave, so the waves need not wait for each other: a wave's
  // own LDS writes are complete, and visible to all its lanes, once its LDS counter has drained.
#define RLHF_WAVE_LDS_FENCE()                  \
  __builtin_amdgcn_sched_barrier(0);           \
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); \
  __builtin_amdgcn_wave_barrier();             \
  __builtin_amdgcn_sched_barrier(0);
  constexpr int EPW = 128 * WN;  // halfs of LDS per wave: its tile as fp16, or half of it as fp32
  uint16_t* ep = wave * EPW < DSTAGE ? lds0 + wave * EPW : lds1 + (wave * EPW - DSTAGE);
  constexpr int CH = WN / 8;     // 16-byte chunks per fp16 row of the wave's tile = lanes per row on the way out
  constexpr int RPI = 64 / CH;   // rows per store instruction
  const int rd_row = lane / CH, rd_c = lane % CH;
  // bias of this lane's 64 columns: 16 eight-byte loads issued together (N is a multiple of 8 here
  // and every column group starts at a multiple of 4, so a group is inside or outside as a whole)
  f32x4_t bias_v[NT][4];
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int nb = n0 + wn + 32 * j + 8 * g + 4 * hf;
      u32x2_t raw = {0, 0};
      if (EPI != EPI_F32 && bias && nb < N) raw = *(const u32x2_t*)(bias + nb);
      bias_v[j][g][0] = __uint_as_float(raw[0] << 16);
      bias_v[j][g][1] = __uint_as_float(raw[0] & 0xFFFF0000u);
      bias_v[j][g][2] = __uint_as_float(raw[1] << 16);
      bias_v[j][g][3] = __uint_as_float(raw[1] & 0xFFFF0000u);
      if (EPI != EPI_F32 && bias2 && nb < N) {
        raw = *(const u32x2_t*)(bias2 + nb);
        bias_v[j][g][0] += __uint_as_float(raw[0] << 16);
        bias_v[j][g][1] += __uint_as_float(raw[0] & 0xFFFF0000u);
        bias_v[j][g][2] += __uint_as_float(raw[1] << 16);
        bias_v[j][g][3] += __uint_as_float(raw[1] & 0xFFFF0000u);
      }
    }
  if (EPI == EPI_BIAS || EPI == EPI_BIAS_GELU || EPI == EPI_QKV) {
    // EPI_QKV: position of this lane's four rows, and for each of its eight 4-column groups the
    // index of its first rotary angle (-1: the group is not rotary).  A group is two whole pairs.
    const int qd = qk.H * qk.hd, qhalf = qk.r >> 1;
    int prow[MT], ang[NT][4];
    if (EPI == EPI_QKV) {
#pragma unroll
      for (int i = 0; i < MT; ++i) prow[i] = (qk.pos[M_sub + min(m0 + wm + 32 * i + l32, M - 1)] + qk.pos_add) * qhalf;
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int c = n0 + wn + 32 * j + 8 * g + 4 * hf;
          const int sec = c >= 2 * qd ? 2 : (c >= qd ? 1 : 0);
          const int e = (c - sec * qd) % qk.hd;
          ang[j][g] = (sec < 2 && e < qk.r && c < N) ? (e >> 1) : -1;
        }
    }
    auto put = [&](auto jc, auto ic) {
      constexpr int j = decltype(jc)::value, i = decltype(ic)::value;
      const int row = 32 * i + l32;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f16x4_t h;
        if (EPI == EPI_QKV) {
          float v[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) v[u] = acc[j][i][4 * g + u] + bias_v[j][g][u];
          if (ang[j][g] >= 0) {
            // the stand-alone kernel turns values already rounded to fp16: keep that order of roundings
            const f32x2_t co = *(const f32x2_t*)(qk.cos_t + prow[i] + ang[j][g]);
            const f32x2_t si = *(const f32x2_t*)(qk.sin_t + prow[i] + ang[j][g]);
#pragma unroll
            for (int u = 0; u < 2; ++u) {
              const float lo = (float)from_f32<half_t>(v[2 * u]), hi = (float)from_f32<half_t>(v[2 * u + 1]);
              v[2 * u] = lo * co[u] - hi * si[u];
              v[2 * u + 1] = hi * co[u] + lo * si[u];
            }
          }
#pragma unroll
          for (int u = 0; u < 4; ++u) h[u] = from_f32<half_t>(v[u]);
        } else {
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const float v = acc[j][i][4 * g + u] + bias_v[j][g][u];
            h[u] = from_f32<half_t>(EPI == EPI_BIAS_GELU ? gelu_f16out(v) : v);
          }
        }
        *(f16x4_t*)(ep + row * WN + (((4 * j + g) ^ (row & (CH - 1))) << 3) + 4 * hf) = h;
      }
    };
#define RLHF_ROW(J)                                                                        \
  put(std::integral_constant<int, J>{}, std::integral_constant<int, 0>{});                 \
  put(std::integral_constant<int, J>{}, std::integral_constant<int, 1>{});                 \
  put(std::integral_constant<int, J>{}, std::integral_constant<int, 2>{});                 \
  put(std::integral_constant<int, J>{}, std::integral_constant<int, 3>{});
    RLHF_ROW(0) RLHF_ROW(1)
    if constexpr (NT > 2) { RLHF_ROW(NT - 2) RLHF_ROW(NT - 1) }
#undef RLHF_ROW
    RLHF_WAVE_LDS_FENCE();
    const int gcol = n0 + wn + rd_c * 8;
    if (EPI == EPI_QKV) {
      // this lane's 16-byte chunk lies in one head of one section (head_dim is a multiple of 8)
      const int sec = gcol >= 2 * qd ? 2 : (gcol >= qd ? 1 : 0);
      const int hh = (gcol - sec * qd) / qk.hd, e = gcol - sec * qd - hh * qk.hd;
      half_t* cache = (half_t*)(sec == 1 ? qk.kc : qk.vc);
#pragma unroll 8
      for (int it = 0; it < 128 / RPI; ++it) {
        const int row = it * RPI + rd_row;
        const int grow = m0 + wm + row;
        const u32x4_t v = *(const u32x4_t*)(ep + row * WN + ((rd_c ^ (row & (CH - 1))) << 3));
        if (grow < M && gcol < N) {
          const int t = M_sub + grow;  // packed row: the row chunk of this launch starts at M_sub
          if (sec == 0) {
            *(u32x4_t*)((half_t*)qk.q + (size_t)t * qd + gcol) = v;
          } else {
            const int b = qk.rowid ? qk.rowid[t] : t;
            const long slot = (long)qk.kvoff[b] * qk.H + (qk.pos[t] + qk.pos_add) + (long)hh * (qk.len[b] + qk.kv_extra);
            *(u32x4_t*)(cache + (size_t)slot * qk.hd + e) = v;
          }
        }
      }
      return;
    }
#pragma unroll 8
    for (int it = 0; it < 128 / RPI; ++it) {
      const int row = it * RPI + rd_row;
      const int grow = m0 + wm + row;
      const u32x4_t v = *(const u32x4_t*)(ep + row * WN + ((rd_c ^ (row & (CH - 1))) << 3));
      if (grow < M && gcol < N) *(u32x4_t*)((half_t*)out + (size_t)grow * ldo + gcol) = v;
    }
  } else {
    float* epf = (float*)ep;   // 128 rows x PC floats per pass
    constexpr int PC = WN / 2;  // columns per pass; a row is PC/4 = CH 16-byte chunks, as in the fp16 case
    constexpr int JP = NT / 2;  // accumulator tiles along N per pass
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      const int gcol = n0 + wn + PC * hh + rd_c * 4;
      // residual rows of this pass: all loads are issued before the transpose, so their latency
      // hides behind the LDS traffic
      f32x4_t xv[128 / RPI];
      if (EPI == EPI_BIAS_RESADD) {
#pragma unroll
        for (int it = 0; it < 128 / RPI; ++it) {
          const int grow = m0 + wm + it * RPI + rd_row;
          if (grow < M && gcol < N) xv[it] = *(const f32x4_t*)((const float*)out + (size_t)grow * ldo + gcol);
        }
      }
      auto put = [&](auto jc, auto ic) {
        constexpr int j = decltype(jc)::value, i = decltype(ic)::value;
        const int row = 32 * i + l32;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4_t v = {acc[j][i][4 * g] + bias_v[j][g][0], acc[j][i][4 * g + 1] + bias_v[j][g][1],
                             acc[j][i][4 * g + 2] + bias_v[j][g][2], acc[j][i][4 * g + 3] + bias_v[j][g][3]};
          const int c = 8 * (j % JP) + 2 * g + hf;
          *(f32x4_t*)(epf + row * PC + ((c ^ (row & (CH - 1))) << 2)) = v;
        }
      };
#define RLHF_ROW(J)                                                                        \
  put(std::integral_constant<int, J>{}, std::integral_constant<int, 0>{});                 \
  put(std::integral_constant<int, J>{}, std::integral_constant<int, 1>{});                 \
  put(std::integral_constant<int, J>{}, std::integral_constant<int, 2>{});                 \
  put(std::integral_constant<int, J>{}, std::integral_constant<int, 3>{});
      if constexpr (NT > 2) {
        if (hh == 0) { RLHF_ROW(0) RLHF_ROW(1) } else { RLHF_ROW(NT - 2) RLHF_ROW(NT - 1) }
      } else {
        if (hh == 0) { RLHF_ROW(0) } else { RLHF_ROW(1) }
      }
#undef RLHF_ROW
      RLHF_WAVE_LDS_FENCE();
#pragma unroll
      for (int it = 0; it < 128 / RPI; ++it) {
        const int row = it * RPI + rd_row;
        const int grow = m0 + wm + row;
        f32x4_t v = *(const f32x4_t*)(epf + row * PC + ((rd_c ^ (row & (CH - 1))) << 2));
        if (grow < M && gcol < N) {
          if (EPI == EPI_BIAS_RESADD) v += xv[it];
          *(f32x4_t*)((float*)out + (size_t)grow * ldo + gcol) = v;
        }
      }
      RLHF_WAVE_LDS_FENCE();
    }
  }
#undef RLHF_WAVE_LDS_FENCE
}

template <int EPI>
static void launch_f16_dma(const GemmArgs& a, hipStream_t s, int k_slices = 1, int k_slice = 0) {
  const int nb_m = (a.M_max + 255) / 256, nb_n = (a.N + 255) / 256;
  const int per_xcd = (nb_m * nb_n + 7) / 8;
  // Eight waves measure 8-10 % faster than four on the layer shapes.
  constexpr int WV = kDmaWaves;
  const bool split = k_slices > 1;
  const dim3 grid(per_xcd * 8, split ? k_slices : 1), block(64 * WV);
  void* out = split ? a.splitk_ws : a.out;
  const int ldo = split ? a.N : a.ldo, ks = split ? k_slice : 0;
  const size_t slab = split ? (size_t)a.M_max * a.N : (size_t)0;
  if constexpr (EPI == EPI_F32) {
    if (a.k_major) {
      hipLaunchKernelGGL((gemm_f16_dma_kernel<EPI_F32, WV, true>), grid, block, 0, s, (const half_t*)a.A,
                         (const half_t*)a.W, (const bf16_t*)nullptr, out, a.M_max, (const int*)nullptr, 0, a.N, a.K, ldo,
                         nb_m, nb_n, a.lda ? a.lda : a.M_max, a.ldw ? a.ldw : a.N, (const bf16_t*)nullptr, LseArgs{},
                         QkvArgs{}, ks, slab);
      return;
    }
  }
  hipLaunchKernelGGL((gemm_f16_dma_kernel<EPI, WV>), grid, block, 0, s, (const half_t*)a.A, (const half_t*)a.W,
                     (const bf16_t*)a.bias, out, a.M_max, a.M_dev, a.M_sub, a.N, a.K, ldo, nb_m, nb_n,
                     a.lda ? a.lda : a.K, a.ldw ? a.ldw : a.K, (const bf16_t*)a.bias2, a.lse ? *a.lse : LseArgs{},
                     a.qkv ? *a.qkv : QkvArgs{}, ks, slab);
}

#ifndef RLHF_GEMM_DMA
#define RLHF_GEMM_DMA 1
#endif
#ifndef RLHF_GEMM_MT
#define RLHF_GEMM_MT 2
#define RLHF_GEMM_NT 4
#define RLHF_GEMM_PF 1
#define RLHF_GEMM_OCC 2
#endif
#ifndef RLHF_GEMM_SKINNY
#define RLHF_GEMM_SKINNY 1
#endif
#ifndef RLHF_DEC_PF
#define RLHF_DEC_PF 1
#define RLHF_DEC_OCC 4
#endif

template <int EPI, int MT, int NT, int PF, int OCC>
static void launch_f16(const GemmArgs& a, hipStream_t s, void* out, int ksplit) {
  const int nb_m = (a.M_max + 64 * MT - 1) / (64 * MT), nb_n = (a.N + 64 * NT - 1) / (64 * NT);
  const int per_xcd = (nb_m * nb_n + 7) / 8;
  hipLaunchKernelGGL((gemm_f16_kernel<EPI, MT, NT, PF, OCC>), dim3(per_xcd * 8, ksplit), dim3(256), 0, s,
                     (const half_t*)a.A, (const half_t*)a.W, (const bf16_t*)a.bias, out, a.M_max, a.M_dev, a.M_sub,
                     a.N, a.K, a.ldo, nb_m, nb_n, ksplit, a.lda ? a.lda : a.K, a.ldw ? a.ldw : a.K);
}

// out = epilogue(sum_z partial[z] + bias), slabs added in index order: deterministic.
template <int EPI>
__global__ void __launch_bounds__(256)
    splitk_reduce_kernel(const float* __restrict__ part, int ksplit, size_t slab, const bf16_t* __restrict__ bias,
                         void* __restrict__ out, int M, int N, int ldo) {
  const size_t i4 = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i4 >= (size_t)M * ldo) return;
  const int col = (int)(i4 % ldo);
  if (col >= N) return;
  f32x4_t v = *(const f32x4_t*)(part + i4);
  for (int z = 1; z < ksplit; ++z) v += *(const f32x4_t*)(part + z * slab + i4);
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (col + u < N) epilogue_store<EPI, half_t>(out, i4 + u, v[u], (EPI != EPI_F32 && bias) ? to_f32(bias[col + u]) : 0.f);
}

// Split factor of the few-rows path (1 = not split).  Few rows (decode): the chip is filled by small
// N tiles and by splitting K, so that every CU holds several short k-loops in flight; partial sums
// go through the caller's fp32 scratch.
int gemm_splitk_factor(int dtype, const GemmArgs& a) {
  if (RLHF_GEMM_SKINNY && gemm_skinny_takes(dtype, a)) return gemm_skinny_splitk(a);
  if (dtype != 1 || a.M_max > 512 || !a.splitk_ws || (a.ldo & 3) != 0) return 1;
  const int tiles = ((a.M_max + 127) / 128) * ((a.N + 63) / 64);
  const int nk = (a.K + TK - 1) / TK;
  // Measured on the decode layer of the 2.8B shape (batch 256, next to the attention kernel of the
  // same layer): a product whose tiles already cover the 256 CUs is fastest unsplit; otherwise K is
  // split while that leaves at least 16 k-steps per block and at most 640 blocks -- beyond that the
  // fp32 partial sums (written, then read by the reduction) outweigh the extra parallelism.
  if (tiles >= 256) return 1;
  int ksplit = 1;
  while (ksplit < 16 && tiles * ksplit * 2 <= 640 && nk / (ksplit * 2) >= 16) ksplit *= 2;
  if ((size_t)ksplit * a.M_max * a.ldo * sizeof(float) > a.splitk_ws_bytes) return 1;
  return ksplit;
}

// Shapes the large-M kernel takes: K a multiple of two stages, 16-byte aligned rows, 32-bit offsets.
static bool takes_dma(const GemmArgs& a) {
  if (a.k_major) {  // [K, M] and [K, N] operands, fp32 output: whole 16-byte chunks per operand row, 32-bit offsets
    const size_t lda = a.lda ? a.lda : a.M_max, ldw = a.ldw ? a.ldw : a.N;
    return RLHF_GEMM_DMA && a.epilogue == EPI_F32 && !a.M_dev && !a.bias && !a.bias2 && a.M_max > 512 && a.N >= 8 &&
           (a.M_max % 8) == 0 && (a.N % 8) == 0 && (a.K % (2 * DK)) == 0 && (a.ldo % 8) == 0 && (lda % 8) == 0 &&
           (ldw % 8) == 0 && (size_t)a.K * std::max(lda, ldw) < (1ull << 32);
  }
  const size_t lda = a.lda ? a.lda : a.K, ldw = a.ldw ? a.ldw : a.K;
  return RLHF_GEMM_DMA && a.M_max > 512 && (a.K % (2 * DK)) == 0 && (a.N % 8) == 0 && (a.ldo % 8) == 0 &&
         (lda % 8) == 0 && (ldw % 8) == 0 && std::max((size_t)a.M_max * lda, (size_t)a.N * ldw) < (1ull << 32);
}
// K slices of a large-M product with few output tiles and a long K (GemmArgs::long_k: the weight-gradient
// products of a backward pass, K = the batch's rows): the slice count (at most 8, each slice a whole number of
// stage pairs, the fp32 slabs fitting the caller's scratch) that minimises rounds of 256 tiles times slice length.
static int dma_k_slices(const GemmArgs& a, int* k_slice) {
  *k_slice = 0;
  if (!a.long_k || !a.splitk_ws || a.M_dev || a.bias || a.ldo != a.N ||
      (a.epilogue != EPI_F32 && a.epilogue != EPI_BIAS_RESADD))
    return 1;
  const int tiles = ((a.M_max + 255) / 256) * ((a.N + 255) / 256), pairs = a.K / (2 * DK);
  int best = 1, best_q = pairs;
  double best_t = (double)((tiles + 255) / 256) * pairs;
  for (int sp = 2; sp <= 8; ++sp) {
    const int q = (pairs + sp - 1) / sp, n = (pairs + q - 1) / q;  // n non-empty slices of q stage pairs
    if (q < 8 || (size_t)n * a.M_max * a.N * sizeof(float) > a.splitk_ws_bytes) continue;
    const double t = (double)((tiles * n + 255) / 256) * q;
    if (t < best_t * 0.97) { best_t = t; best = n; best_q = q; }
  }
  *k_slice = best_q * 2 * DK;
  return best;
}
bool gemm_takes_bias2(int dtype, const GemmArgs& a) { return dtype == 1 && takes_dma(a); }
bool gemm_takes_k_major(int dtype, const GemmArgs& a) { return dtype == 1 && a.k_major && takes_dma(a); }
bool gemm_takes_lse(int dtype, const GemmArgs& a) { return dtype == 1 && takes_dma(a); }
// EPI_QKV: 16-byte chunks must not straddle heads, a lane's 4-column group must be whole pairs, and the
// cos / sin pairs are read as aligned 8-byte words.
bool gemm_takes_qkv(int dtype, const GemmArgs& a, int H, int hd, int r) {
  return dtype == 1 && takes_dma(a) && H > 0 && hd > 0 && (hd % 8) == 0 && (r % 4) == 0 && r <= hd &&
         a.N == 3 * H * hd && a.bias != nullptr;
}
// Parts (column groups with their own max / sum-exp) the log-sum-exp epilogue leaves per row: one per wave
// column of every 256-column tile.
int gemm_lse_parts(int n_cols) { return (kDmaWaves == 8 ? 4 : 2) * ((n_cols + 255) / 256); }

template <int EPI>
static void launch_epi(int dtype, const GemmArgs& a, hipStream_t s) {
  if (dtype == 0) {
    dim3 grid((a.N + 63) / 64, (a.M_max + 63) / 64);
    hipLaunchKernelGGL(gemm_f32_kernel<EPI>, grid, dim3(256), 0, s, (const float*)a.A, (const float*)a.W,
                       (const float*)a.bias, a.out, a.M_max, a.M_dev, a.M_sub, a.N, a.K, a.ldo);
  } else {
    // Few rows (decode): the chip is filled by small N tiles and by splitting K, so that every CU
    // holds several short k-loops in flight; partial sums go through the caller's fp32 scratch.
    const int ksplit = gemm_splitk_factor(dtype, a);
    const bool skinny = RLHF_GEMM_SKINNY && gemm_skinny_takes(dtype, a);
    if (skinny && ksplit == 1) {
      launch_gemm_skinny(a, 1, s);
      return;
    }
    if (ksplit > 1) {
      if (a.phase != 2) {
        if (skinny) launch_gemm_skinny(a, ksplit, s);
        else launch_f16<EPI_F32, 2, 1, RLHF_DEC_PF, RLHF_DEC_OCC>(a, s, a.splitk_ws, ksplit);
      }
      if (a.phase != 1) {
        const size_t n4 = ((size_t)a.M_max * a.ldo + 3) / 4;
        hipLaunchKernelGGL(splitk_reduce_kernel<EPI>, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s,
                           (const float*)a.splitk_ws, ksplit, (size_t)a.M_max * a.ldo, (const bf16_t*)a.bias, a.out,
                           a.M_max, a.N, a.ldo);
      }
      return;
    }
    if (a.M_max <= 512)
      launch_f16<EPI, 2, 1, RLHF_DEC_PF, RLHF_DEC_OCC>(a, s, a.out, 1);
    else if (takes_dma(a)) {
      int k_slice = 0;
      const int n = dma_k_slices(a, &k_slice);
      if constexpr (EPI == EPI_F32 || EPI == EPI_BIAS_RESADD) {
        if (n > 1) {  // fp32 slabs, then their sum in slab order into (or, residual form, onto) the output
          launch_f16_dma<EPI_F32>(a, s, n, k_slice);
          const size_t quads = ((size_t)a.M_max * a.ldo + 3) / 4;
          hipLaunchKernelGGL((splitk_reduce_kernel<EPI>), dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s,
                             (const float*)a.splitk_ws, n, (size_t)a.M_max * a.N, (const bf16_t*)nullptr, a.out,
                             a.M_max, a.N, a.ldo);
          return;
        }
      }
      launch_f16_dma<EPI>(a, s);
    }
    else
      launch_f16<EPI, RLHF_GEMM_MT, RLHF_GEMM_NT, RLHF_GEMM_PF, RLHF_GEMM_OCC>(a, s, a.out, 1);
  }
}

hipError_t launch_gemm(int dtype, const GemmArgs& a, hipStream_t s) {
  if (a.M_max <= 0) return hipSuccess;
  if (dtype == 1 && (a.K % 8) != 0) return hipErrorInvalidValue;
  if (dtype != 1 && (a.lda || a.ldw || a.bias2)) return hipErrorInvalidValue;
  if (a.bias2 && !gemm_takes_bias2(dtype, a)) return hipErrorInvalidValue;
  if (a.k_major && !gemm_takes_k_major(dtype, a)) return hipErrorInvalidValue;
  switch (a.epilogue) {
    case EPI_BIAS: launch_epi<EPI_BIAS>(dtype, a, s); break;
    case EPI_BIAS_GELU: launch_epi<EPI_BIAS_GELU>(dtype, a, s); break;
    case EPI_BIAS_RESADD: launch_epi<EPI_BIAS_RESADD>(dtype, a, s); break;
    case EPI_F32: launch_epi<EPI_F32>(dtype, a, s); break;
    case EPI_LSE:
      if (!a.lse || !gemm_takes_lse(dtype, a)) return hipErrorInvalidValue;
      launch_f16_dma<EPI_LSE>(a, s);
      break;
    case EPI_QKV:
      if (!a.qkv || !gemm_takes_qkv(dtype, a, a.qkv->H, a.qkv->hd, a.qkv->r)) return hipErrorInvalidValue;
      launch_f16_dma<EPI_QKV>(a, s);
      break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace rlhf
