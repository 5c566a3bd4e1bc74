// Few-rows product C[M,N] = A[M,K] * W[N,K]^T for the decode passes (M = batch, at most a few hundred rows).
//
// Such a product streams every weight once and multiplies it with all M rows: 2*M flop per weight byte
// pair, i.e. right at the ridge between HBM and the matrix cores for M = 256.  What the kernel is built
// around:
//   * Weights never touch LDS.  A wave owns 32 rows of W (32 output columns) for ALL rows of A: lane
//     (l32, hf) loads the 64 bytes W[n0 + l32][k0 + 32*hf .. +32) of a 64-deep k-step straight into
//     registers (4 x 16 B; a wave instruction group covers 32 full 128-byte lines) and uses each 16-byte
//     piece as the matrix instruction's second operand against MT = M/32 row tiles of A: every weight
//     register feeds MT matrix instructions.  The k order inside a step is permuted (hf = 0: k 0..31,
//     hf = 1: k 32..63); the A fragments are read with the same permutation, and a sum does not care.
//   * A (M x 64 per step, 32 KB at M = 256) goes global -> LDS directly (no registers) and is shared by
//     the block's four waves (128 output columns per block).  Per step a block pulls 32 KB of A and
//     16 KB of W through the vector memory path for 128 matrix instructions.
//   * Loads run three k-steps ahead of the arithmetic: four LDS stages, four register sets.  A wave's
//     loads complete in order, so the A stages must run as far ahead as the weights do, or waiting for
//     the next A stage would also wait for every weight load issued before it.
//   * K is split over blockIdx.y so that a product with few column blocks still covers the chip; the
//     fp32 partial slabs [split][M][ldo] are added in slab order by their consumer (deterministic).
//
// Accumulator layout (A fragment as the first operand): element e of lane (l32, hf) of row tile i is
//   row 32*i + 8*(e/4) + 4*hf + e%4, column n0 + l32
// so one store instruction writes two full 128-byte row segments.
#include <algorithm>

#include "common.h"

namespace rlhf {

typedef __attribute__((ext_vector_type(8))) _Float16 sk_f16x8_t;
typedef __attribute__((ext_vector_type(16))) float sk_f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t sk_u32x4_t;

#define SK_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define SK_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

__device__ __forceinline__ float sk_gelu_f16out(float x) {  // same fitted form as the large-M kernel's epilogue
  const float s = fminf(x * x, 64.0f);
  float p = fmaf(1.01426504e-3f, s, -1.06775735e-1f);
  p = fmaf(p, s, -2.30112140f);
  const float e = __builtin_amdgcn_exp2f(x * p);
  return x * __frcp_rn(1.0f + e);
}

constexpr int SK_BN = 128;  // output columns per block (4 waves x 32)

template <int MT, int EPI>
__global__ void __launch_bounds__(256, 1)
    gemm_skinny_f16_kernel(const half_t* __restrict__ A, const half_t* __restrict__ W, const bf16_t* __restrict__ bias,
                           void* __restrict__ out, int M, int N, int K, int ldo, int lda, int ldw, int per_split,
                           size_t slab) {
  constexpr int ROWS = 32 * MT;
  constexpr int STAGE = ROWS * 64;  // halfs per stage: ROWS rows of 128 bytes
  __shared__ __attribute__((aligned(16))) uint16_t lds[4 * STAGE];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hf = lane >> 5;
  const int n0 = blockIdx.x * SK_BN + wave * 32;
  const int m0 = blockIdx.z * ROWS;
  const int nk_all = K >> 6;
  const int kt0 = blockIdx.y * per_split;
  const int nks = min(per_split, nk_all - kt0);  // k-steps of this block (>= 1: the host sizes the grid so)

  // ---- A stage: wave-load j fills rows 8*(4j + wave) .. +7; lane l lands at row + l/8, physical chunk l%8,
  //      and therefore fetches logical chunk (l%8) ^ ((row >> 1) & 7) (conflict-free 16-byte fragment reads)
  uint32_t aoff[MT];
#pragma unroll
  for (int j = 0; j < MT; ++j) {
    const int row = 8 * (4 * j + wave) + (lane >> 3);
    const int c = (lane & 7) ^ ((row >> 1) & 7);
    aoff[j] = (uint32_t)(min(m0 + row, M - 1) * lda + c * 8);
  }
  const half_t* Ab = A + (size_t)kt0 * 64;
  const size_t woff = (size_t)min(n0 + l32, N - 1) * ldw + (size_t)kt0 * 64 + 32 * hf;  // this lane's 64 bytes of k-step 0

  // The loop below is scheduled by hand: the loads, the fragment reads and the waits are assembly statements
  // (kept in program order), so that "n loads still in flight" is exactly what the code says.  Left to the
  // compiler, the waits for direct-to-LDS loads come out as "wait for everything" at the loop header, and plain
  // loads from read-only memory get moved across hand-placed waits.
  sk_u32x4_t wr[4][4];  // [register set][16-byte piece of the lane's 64 bytes]
  // Loads of k-step k (relative to kt0): MT wave instructions for the A stage, 4 for the weights, always issued.
  // A step past the block's last one loads one 16-byte word per wave instruction (every lane the same address;
  // mask arithmetic, no branch) that nobody reads.
  auto issue_a = [&](int stage, int k) {
    const uint32_t m32 = k < nks ? 0xFFFFFFFFu : 0u;
#pragma unroll
    for (int j = 0; j < MT; ++j)
      __builtin_amdgcn_global_load_lds(SK_GLOBAL_PTR(Ab + ((aoff[j] + (uint32_t)k * 64u) & m32)),
                                       SK_LDS_PTR(lds + stage * STAGE + 8 * (4 * j + wave) * 64), 16, 0, 0);
  };
  auto issue_w = [&](int set, int k) {
    const size_t m64 = k < nks ? ~(size_t)0 : (size_t)0;
    const half_t* wp = W + ((woff + (size_t)k * 64) & m64);
    asm volatile("global_load_dwordx4 %0, %4, off\n\t"
                 "global_load_dwordx4 %1, %4, off offset:16\n\t"
                 "global_load_dwordx4 %2, %4, off offset:32\n\t"
                 "global_load_dwordx4 %3, %4, off offset:48"
                 : "=&v"(wr[set][0]), "=&v"(wr[set][1]), "=&v"(wr[set][2]), "=&v"(wr[set][3])
                 : "v"(wp)
                 : "memory");
  };

  sk_f32x16_t acc[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;

  // fragment addresses (LDS byte addresses): row l32 of a 32-row tile, logical chunk 4*hf + s of sub-step s
  // (the lane's k range of the step is 32*hf .. 32*hf + 31); tile i and the stage are added as offsets
  const int key = (l32 >> 1) & 7;
  const uint32_t lds0 = (uint32_t)(uintptr_t)SK_LDS_PTR(lds) + (uint32_t)l32 * 128u;
  uint32_t fad[4];
#pragma unroll
  for (int sb = 0; sb < 4; ++sb) fad[sb] = lds0 + (uint32_t)(((4 * hf + sb) ^ key) << 4);

  sk_f16x8_t fa[2][MT];
  // MT fragment reads of sub-step SB of stage STG into buffer BUF (tile i is 4 KB further on)
#define SK_RD(BUF, I, ADDR) \
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(fa[BUF][I]) : "v"(ADDR), "n"((I) * 4096) : "memory")
#define SK_FRAGS(BUF, STG, SB)                                                 \
  {                                                                            \
    const uint32_t ad_ = fad[SB] + (uint32_t)((STG) * STAGE * 2);              \
    SK_RD(BUF, 0, ad_); SK_RD(BUF, 1, ad_);                                    \
    if (MT > 2) { SK_RD(BUF, 2 % MT, ad_); SK_RD(BUF, 3 % MT, ad_); }          \
    if (MT > 4) { SK_RD(BUF, 4 % MT, ad_); SK_RD(BUF, 5 % MT, ad_); SK_RD(BUF, 6 % MT, ad_); SK_RD(BUF, 7 % MT, ad_); } \
  }
  // wait until at most N fragment reads are outstanding; the buffer's registers pass through the statement so
  // that the matrix instructions using them cannot be moved in front of it
#define SK_LGKM(N, BUF)                                                                        \
  {                                                                                            \
    if (MT == 2) asm volatile("s_waitcnt lgkmcnt(" #N ")" : "+v"(fa[BUF][0]), "+v"(fa[BUF][1])::"memory"); \
    else if (MT == 4)                                                                          \
      asm volatile("s_waitcnt lgkmcnt(" #N ")" : "+v"(fa[BUF][0]), "+v"(fa[BUF][1]), "+v"(fa[BUF][2 % MT]), "+v"(fa[BUF][3 % MT])::"memory"); \
    else                                                                                       \
      asm volatile("s_waitcnt lgkmcnt(" #N ")"                                                 \
                   : "+v"(fa[BUF][0]), "+v"(fa[BUF][1]), "+v"(fa[BUF][2 % MT]), "+v"(fa[BUF][3 % MT]), "+v"(fa[BUF][4 % MT]), \
                     "+v"(fa[BUF][5 % MT]), "+v"(fa[BUF][6 % MT]), "+v"(fa[BUF][7 % MT])::"memory"); \
  }
  auto mfmas = [&](int buf, const sk_u32x4_t& wv) {
    sk_f16x8_t wf;
    __builtin_memcpy(&wf, &wv, 16);
#pragma unroll
    for (int i = 0; i < MT; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[buf][i], wf, acc[i], 0, 0, 0);
  };
  // Wait until every load of the NEXT k-step has landed, then meet the other waves (their share of the next A
  // stage has landed too).  A wave's loads complete in order and are issued as A(k+2), W(k+3) at the start of
  // step k, so behind A(k+1) and W(k+1) there may still be W(k+2), A(k+2) and W(k+3) in flight: MT + 8 loads.
  // The next step's weight registers pass through the statement, so nothing that uses them can move above it.
#define SK_WAIT_BARRIER(NS)                                                                    \
  {                                                                                            \
    __builtin_amdgcn_sched_barrier(0);                                                         \
    asm volatile("s_waitcnt vmcnt(%4)"                                                         \
                 : "+v"(wr[NS][0]), "+v"(wr[NS][1]), "+v"(wr[NS][2]), "+v"(wr[NS][3])          \
                 : "n"(MT + 8)                                                                 \
                 : "memory");                                                                  \
    __builtin_amdgcn_s_barrier();                                                              \
    asm volatile("" ::: "memory");                                                             \
    __builtin_amdgcn_sched_barrier(0);                                                         \
  }
#define SK_FENCE() __builtin_amdgcn_sched_barrier(0)
#define SK_LGKM_MT(BUF) { if (MT == 8) SK_LGKM(8, BUF) else if (MT == 4) SK_LGKM(4, BUF) else SK_LGKM(2, BUF) }
  // One k-step on register set / stage S.  The MT fragments of a sub-step are read as one batch, two batches in
  // flight: while the matrix instructions of sub-steps 2 and 3 run, the first two batches of the NEXT step are
  // already being read -- which is why the wait-and-barrier sits in the middle of the step and not at its end
  // (all four waves start their reads right after a barrier: at the end of a step that burst, 64 KB through the
  // LDS port, would run with the matrix cores idle).  Loads: the A stage two steps ahead into stage (S+2)&3 --
  // last read two steps ago, and every wave has passed a barrier since -- and the weights three steps ahead
  // into register set (S+3)&3, last used by the previous step.  Steps past the block's last one only keep the
  // barrier and load counts equal; a fragment batch read ahead of a step that does not exist is never used.
#define SK_STEP(S)                                               \
  {                                                              \
    const int kk = kt + (S);                                     \
    issue_a(((S) + 2) & 3, kk + 2);                              \
    issue_w(((S) + 3) & 3, kk + 3);                              \
    SK_FENCE();                                                  \
    if (kk < nks) {                                              \
      SK_LGKM_MT(0)                                              \
      mfmas(0, wr[S][0]);                                        \
      SK_FENCE();                                                \
      SK_FRAGS(0, S, 2)                                          \
      SK_FENCE();                                                \
      SK_LGKM_MT(1)                                              \
      mfmas(1, wr[S][1]);                                        \
      SK_FENCE();                                                \
      SK_FRAGS(1, S, 3)                                          \
    }                                                            \
    SK_WAIT_BARRIER(((S) + 1) & 3)                               \
    if (kk < nks) {                                              \
      SK_LGKM_MT(0)                                              \
      mfmas(0, wr[S][2]);                                        \
      SK_FENCE();                                                \
      SK_FRAGS(0, ((S) + 1) & 3, 0)                              \
      SK_FENCE();                                                \
      SK_LGKM_MT(1)                                              \
      mfmas(1, wr[S][3]);                                        \
      SK_FENCE();                                                \
      SK_FRAGS(1, ((S) + 1) & 3, 1)                              \
      SK_FENCE();                                                \
    }                                                            \
  }

  issue_a(0, 0);
  issue_w(0, 0);
  issue_a(1, 1);
  issue_w(1, 1);
  issue_w(2, 2);
  SK_WAIT_BARRIER(0)
  SK_FRAGS(0, 0, 0)
  SK_FRAGS(1, 0, 1)
  SK_FENCE();
  for (int kt = 0; kt < nks; kt += 4) {
    SK_STEP(0)
    SK_STEP(1)
    SK_STEP(2)
    SK_STEP(3)
  }
#undef SK_STEP
#undef SK_LGKM_MT
#undef SK_FENCE
#undef SK_WAIT_BARRIER
#undef SK_LGKM
#undef SK_FRAGS
#undef SK_RD
  // Everything still in flight must land before the epilogue: the surplus loads of the last steps and the
  // fragment batches read ahead of a step that does not exist write registers that the compiler, which sees no
  // later use of those values, hands to the epilogue's addresses.
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the surplus loads of the last steps have landed too

  // ---- epilogue: one row tile at a time (fences keep the compiler from forming all 128 addresses at once)
  const int col = n0 + l32;
  if (col >= N) return;
  float bv = 0.f;
  if (EPI != EPI_F32 && bias) bv = to_f32(bias[col]);
  if (EPI == EPI_F32) out = (float*)out + (size_t)blockIdx.y * slab;  // split-K: this block's slab (0 when unsplit)
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    const int r0 = m0 + 32 * i + 4 * hf;
    char* p = (char*)out + ((size_t)r0 * ldo + col) * (EPI == EPI_BIAS || EPI == EPI_BIAS_GELU ? 2 : 4);
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int dr = 8 * (e >> 2) + (e & 3);  // row r0 + dr
      if (r0 + dr >= M) continue;
      const size_t o = (size_t)dr * ldo;
      const float v = acc[i][e] + bv;
      if (EPI == EPI_BIAS) ((half_t*)p)[o] = from_f32<half_t>(v);
      else if (EPI == EPI_BIAS_GELU) ((half_t*)p)[o] = from_f32<half_t>(sk_gelu_f16out(v));
      else if (EPI == EPI_BIAS_RESADD) ((float*)p)[o] += v;
      else ((float*)p)[o] = acc[i][e];
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Shapes the kernel takes: fp16 operands, a host-side row count of at most 512, whole 64-deep k-steps,
// 16-byte aligned rows.  (Everything else stays on the staged tile kernel.)
bool gemm_skinny_takes(int dtype, const GemmArgs& a) {
  const int lda = a.lda ? a.lda : a.K, ldw = a.ldw ? a.ldw : a.K;
  return dtype == 1 && !a.small_footprint && a.M_dev == nullptr && a.M_max > 0 && a.M_max <= 512 && a.K >= 64 && (a.K % 64) == 0 &&
         (lda % 8) == 0 && (ldw % 8) == 0 && a.epilogue != EPI_LSE && a.epilogue != EPI_QKV && !a.bias2 &&
         (size_t)a.M_max * lda < (1ull << 31);
}

static int sk_rows_per_block(int M) { return M <= 64 ? 64 : (M <= 128 ? 128 : 256); }

// K split: enough blocks to cover the chip (or `max_split`, if the caller caps it: a product that runs in the
// shadow of another kernel is better off with fewer, longer blocks and fewer partial sums), at least four
// k-steps per block, and what the partial-sum scratch holds.
int gemm_skinny_splitk(const GemmArgs& a) {
  if (!a.splitk_ws) return 1;
  const int rows = sk_rows_per_block(a.M_max);
  const int blocks = ((a.N + SK_BN - 1) / SK_BN) * ((a.M_max + rows - 1) / rows);
  const int nk = a.K / 64;
  int ks = std::max(1, std::min(240 / std::max(blocks, 1), nk / 4));
  if (a.max_split > 0) ks = std::min(ks, a.max_split);
  while (ks > 1 && (size_t)ks * a.M_max * a.ldo * sizeof(float) > a.splitk_ws_bytes) --ks;
  const int per_split = (nk + ks - 1) / ks;
  return (nk + per_split - 1) / per_split;
}

template <int MT, int EPI>
static void sk_launch(const GemmArgs& a, void* out, int ks, hipStream_t s) {
  const int nk = a.K / 64, per_split = (nk + ks - 1) / ks;
  const dim3 grid((a.N + SK_BN - 1) / SK_BN, ks, (a.M_max + 32 * MT - 1) / (32 * MT));
  hipLaunchKernelGGL((gemm_skinny_f16_kernel<MT, EPI>), grid, dim3(256), 0, s, (const half_t*)a.A, (const half_t*)a.W,
                     (const bf16_t*)a.bias, out, a.M_max, a.N, a.K, a.ldo, a.lda ? a.lda : a.K, a.ldw ? a.ldw : a.K,
                     per_split, (size_t)a.M_max * a.ldo);
}

template <int EPI>
static void sk_launch_rows(const GemmArgs& a, void* out, int ks, hipStream_t s) {
  const int rows = sk_rows_per_block(a.M_max);
  if (rows == 64) sk_launch<2, EPI>(a, out, ks, s);
  else if (rows == 128) sk_launch<4, EPI>(a, out, ks, s);
  else sk_launch<8, EPI>(a, out, ks, s);
}

// The product itself: with ks > 1 the fp32 partial slabs go to a.splitk_ws, else the epilogue runs in the kernel.
void launch_gemm_skinny(const GemmArgs& a, int ks, hipStream_t s) {
  if (ks > 1) {
    sk_launch_rows<EPI_F32>(a, a.splitk_ws, ks, s);
    return;
  }
  switch (a.epilogue) {
    case EPI_BIAS: sk_launch_rows<EPI_BIAS>(a, a.out, 1, s); break;
    case EPI_BIAS_GELU: sk_launch_rows<EPI_BIAS_GELU>(a, a.out, 1, s); break;
    case EPI_BIAS_RESADD: sk_launch_rows<EPI_BIAS_RESADD>(a, a.out, 1, s); break;
    default: sk_launch_rows<EPI_F32>(a, a.out, 1, s); break;
  }
}

}  // namespace rlhf
