// C[M,N] = A[M,K] * W[N,K]^T (+ bias, + epilogue).  Both operands are K-contiguous, which is the
// natural operand order of the CDNA matrix cores: every lane loads 8 consecutive K elements of one
// row of A and of one row of W.
//
//  * bf16 mode (fp16 operands): v_mfma_f32_32x32x16_f16, 128x128 block tile, 4 waves (2x2) of 64x64, K step 64,
//          LDS double buffer with global->register->LDS staging, fp32 accumulation.
//  * fp32: plain FMA tile kernel (check mode only; not tuned).
#include "common.h"

namespace rlhf {

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

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
constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDS_ROW = BK + 8;  // 16-bit elements per LDS row: +16 bytes so that 16 consecutive rows
                                 // start in 16 different 16-byte bank groups

template <int EPI>
__global__ void __launch_bounds__(256)
    gemm_f16_kernel(const half_t* __restrict__ A, const half_t* __restrict__ W, const bf16_t* __restrict__ bias,
                     void* __restrict__ out, int M_max, const int* __restrict__ M_dev, int M_sub, int N, int K, int ldo) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[2][2][BM * LDS_ROW];  // [buffer][A|W]
  const int M = M_dev ? min(M_max, *M_dev - M_sub) : M_max;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  if (m0 >= M) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;

  // staging: tile = 128 rows x 8 chunks of 16 B; thread handles chunk ids tid + 256*i, i < 4
  const int ld_row = tid >> 3, ld_kc = tid & 7;  // rows ld_row + 32*i
  u32x4_t ra[4], rw[4];
  auto load_tiles = [&](int k0) {
    const int k = k0 + ld_kc * 8;
    const bool kok = k < K;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = ld_row + 32 * i;
      const int ar = min(m0 + r, M - 1), wr = min(n0 + r, N - 1);
      u32x4_t z = {0, 0, 0, 0};
      ra[i] = kok ? *(const u32x4_t*)(A + (size_t)ar * K + k) : z;
      rw[i] = kok ? *(const u32x4_t*)(W + (size_t)wr * K + k) : z;
    }
  };
  auto store_tiles = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = ld_row + 32 * i;
      *(u32x4_t*)(&lds[buf][0][r * LDS_ROW + ld_kc * 8]) = ra[i];
      *(u32x4_t*)(&lds[buf][1][r * LDS_ROW + ld_kc * 8]) = rw[i];
    }
  };

  f32x16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int nk = (K + BK - 1) / BK;
  load_tiles(0);
  store_tiles(0);
  __syncthreads();
  const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) load_tiles((kt + 1) * BK);
    const uint16_t* la = lds[buf][0];
    const uint16_t* lw = lds[buf][1];
#pragma unroll
    for (int ks = 0; ks < BK; ks += 16) {
      f16x8_t fa[2], fw[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        fa[i] = *(const f16x8_t*)(la + (wm + i * 32 + frag_row) * LDS_ROW + ks + frag_k);
        fw[i] = *(const f16x8_t*)(lw + (wn + i * 32 + frag_row) * LDS_ROW + ks + frag_k);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[i], fw[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store_tiles(buf ^ 1);
    __syncthreads();
  }

  // accumulator element e of lane l: row (e/4)*8 + (l/32)*4 + e%4, column l%32 of the 32x32 tile
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int col = n0 + wn + j * 32 + (lane & 31);
    if (col >= N) continue;
    const float bv = (EPI != EPI_F32 && bias) ? to_f32(bias[col]) : 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = m0 + wm + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        if (row < M) epilogue_store<EPI, half_t>(out, (size_t)row * ldo + col, acc[i][j][e], bv);
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

template <int EPI>
static void launch_epi(int dtype, const GemmArgs& a, hipStream_t s) {
  if (dtype == 0) {
    dim3 grid((a.N + 63) / 64, (a.M_max + 63) / 64);
    hipLaunchKernelGGL(gemm_f32_kernel<EPI>, grid, dim3(256), 0, s, (const float*)a.A, (const float*)a.W,
                       (const float*)a.bias, a.out, a.M_max, a.M_dev, a.M_sub, a.N, a.K, a.ldo);
  } else {
    dim3 grid((a.N + BN - 1) / BN, (a.M_max + BM - 1) / BM);
    hipLaunchKernelGGL(gemm_f16_kernel<EPI>, grid, dim3(256), 0, s, (const half_t*)a.A, (const half_t*)a.W,
                       (const bf16_t*)a.bias, a.out, a.M_max, a.M_dev, a.M_sub, a.N, a.K, a.ldo);
  }
}

hipError_t launch_gemm(int dtype, const GemmArgs& a, hipStream_t s) {
  if (a.M_max <= 0) return hipSuccess;
  if (dtype == 1 && (a.K % 8) != 0) return hipErrorInvalidValue;
  switch (a.epilogue) {
    case EPI_BIAS: launch_epi<EPI_BIAS>(dtype, a, s); break;
    case EPI_BIAS_GELU: launch_epi<EPI_BIAS_GELU>(dtype, a, s); break;
    case EPI_BIAS_RESADD: launch_epi<EPI_BIAS_RESADD>(dtype, a, s); break;
    case EPI_F32: launch_epi<EPI_F32>(dtype, a, s); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace rlhf
