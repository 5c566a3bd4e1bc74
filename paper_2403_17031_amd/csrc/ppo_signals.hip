// What PPO consumes after a rollout, computed on the device from the outputs of rollout_generate
// and score_sequences: per-token rewards (KL penalty per kept token, reward-model score on the last
// kept token, a constant in place of the score when the response has no EOS), generalised advantage
// estimates with returns, batch whitening, and the clipped objective with its gradient with respect
// to the model's outputs.  The arrays are tiny (batch x 53), so the kernels are
// latency-bound by construction: one wave per row, sums and recursions in double and in a fixed
// order (bit-reproducible; no atomics).
#include "common.h"

namespace rlhf {

__device__ __forceinline__ int wave_min_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o, 64));
  return v;
}

// One wave per row.  first = index of the first pad in the response (N if none); the row's kept
// tokens are t <= last = first - 1 (N - 1 if none), which is also where the reward model is read.
__global__ void __launch_bounds__(64)
    ppo_rewards_kernel(const float* __restrict__ lp, const float* __restrict__ ref_full,
                       const float* __restrict__ rm_full, const int* __restrict__ tokens, int Lq, int N, int eos_id,
                       int pad_id, float beta, float miss, float* __restrict__ rewards, float* __restrict__ scores,
                       float* __restrict__ kl_out, int* __restrict__ kept) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const size_t L = (size_t)Lq + N;
  const int* tok = tokens + b * L + Lq;
  const float* ref = ref_full + b * L + Lq;
  int first = N;
  for (int t = lane; t < N; t += 64)
    if (tok[t] == pad_id) first = min(first, t);
  first = wave_min_i(first);
  const int last = first - 1;  // -1: nothing was generated for this row
  float score = 0.f;
  if (last >= 0) score = tok[last] == eos_id ? rm_full[b * L + Lq + last] : miss;
  for (int t = lane; t < N; t += 64) {
    float r = 0.f;
    if (t <= last) {
      r = -beta * (lp[(size_t)b * N + t] - ref[t]);
      if (t == last) r += score;
    }
    rewards[(size_t)b * N + t] = r;
  }
  if (lane == 0) {
    double kl = 0.0;
    for (int t = 0; t <= last; ++t) kl += (double)lp[(size_t)b * N + t] - (double)ref[t];
    kl_out[b] = (float)kl;
    scores[b] = score;
    kept[b] = last + 1;
  }
}

// One thread per row: A_t = delta_t + gamma * lambda * A_{t+1}, delta_t = r_t + gamma * V_{t+1} - V_t,
// V = 0 beyond the last kept token; returns = A + V.
__global__ void __launch_bounds__(64)
    ppo_gae_kernel(const float* __restrict__ rewards, const float* __restrict__ values, long vstride,
                   const int* __restrict__ kept, int B, int N, float gamma, float lam, float* __restrict__ adv,
                   float* __restrict__ ret) {
  const int b = blockIdx.x * 64 + threadIdx.x;
  if (b >= B) return;
  const int L = min(max(kept[b], 0), N);
  const float* r = rewards + (size_t)b * N;
  const float* v = values + (size_t)b * vstride;
  for (int t = L; t < N; ++t) {
    adv[(size_t)b * N + t] = 0.f;
    ret[(size_t)b * N + t] = 0.f;
  }
  double running = 0.0, v_next = 0.0;
  for (int t = L - 1; t >= 0; --t) {
    const double vt = v[t];
    const double delta = (double)r[t] + (double)gamma * v_next - vt;
    running = delta + (double)gamma * (double)lam * running;
    adv[(size_t)b * N + t] = (float)running;
    ret[(size_t)b * N + t] = (float)(running + vt);
    v_next = vt;
  }
}

__device__ __forceinline__ double block_sum_1024_d(double v, double* sh) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  __syncthreads();  // sh may still be read from a previous call
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  double t = 0.0;
  for (int i = 0; i < 16; ++i) t += sh[i];
  return t;
}

// One block: (x - mean) * rsqrt(var + 1e-8) over the kept positions, biased variance; the mean is
// added back when shift_mean is 0.  Positions that are not kept get 0.
__global__ void __launch_bounds__(1024)
    ppo_whiten_kernel(const float* __restrict__ x, const int* __restrict__ kept, int B, int N, int shift_mean,
                      float* __restrict__ out) {
  __shared__ double sh[16];
  const size_t total = (size_t)B * N;
  auto is_kept = [&](size_t i) { return !kept || (int)(i % N) < kept[i / N]; };
  double s = 0.0, cnt = 0.0;
  for (size_t i = threadIdx.x; i < total; i += 1024)
    if (is_kept(i)) {
      s += x[i];
      cnt += 1.0;
    }
  const double n = block_sum_1024_d(cnt, sh);
  const double mean = n > 0 ? block_sum_1024_d(s, sh) / n : 0.0;
  double q = 0.0;
  for (size_t i = threadIdx.x; i < total; i += 1024)
    if (is_kept(i)) {
      const double dlt = x[i] - mean;
      q += dlt * dlt;
    }
  const double var = n > 0 ? block_sum_1024_d(q, sh) / n : 0.0;
  const double rstd = 1.0 / sqrt(var + 1e-8);
  for (size_t i = threadIdx.x; i < total; i += 1024) {
    float o = 0.f;
    if (is_kept(i)) {
      double w = (x[i] - mean) * rstd;
      if (!shift_mean) w += mean;
      o = (float)w;
    }
    out[i] = o;
  }
}

// One block: the clipped PPO objective over the kept response tokens and its gradient with respect
// to the new log-probs and the new values.  Branch choice and sums in double, fixed order.
// stats: loss, pg_loss, vf_loss, approx_kl, pg_clipfrac, vf_clipfrac, ratio_mean, n_tokens.
__global__ void __launch_bounds__(1024)
    ppo_loss_kernel(const float* __restrict__ lp, const float* __restrict__ lp0, const float* __restrict__ adv,
                    const float* __restrict__ v, const float* __restrict__ v0, const float* __restrict__ ret,
                    const int* __restrict__ kept, int B, int N, float eps, float eps_v, float c1,
                    float* __restrict__ d_lp, float* __restrict__ d_v, float* __restrict__ stats) {
  __shared__ double sh[16];
  const size_t total = (size_t)B * N;
  auto is_kept = [&](size_t i) { return (int)(i % N) < kept[i / N]; };
  double cnt = 0.0;
  for (size_t i = threadIdx.x; i < total; i += 1024)
    if (is_kept(i)) cnt += 1.0;
  const double n = block_sum_1024_d(cnt, sh);
  const double inv_n = n > 0 ? 1.0 / n : 0.0;
  double pg = 0.0, vf = 0.0, kl = 0.0, rs = 0.0, pgc = 0.0, vfc = 0.0;
  for (size_t i = threadIdx.x; i < total; i += 1024) {
    float g_lp = 0.f, g_v = 0.f;
    if (is_kept(i)) {
      const double diff = (double)lp[i] - (double)lp0[i];
      const double ratio = exp(diff);
      const double ratio_c = fmin(fmax(ratio, 1.0 - (double)eps), 1.0 + (double)eps);
      const double a = adv[i];
      const double pg1 = -a * ratio, pg2 = -a * ratio_c;
      pg += fmax(pg1, pg2);
      if (pg2 > pg1) pgc += 1.0;
      else g_lp = (float)(-a * ratio * inv_n);
      const double vv = v[i], vo = v0[i], r = ret[i];
      const double v_c = fmin(fmax(vv, vo - (double)eps_v), vo + (double)eps_v);
      const double vf1 = (vv - r) * (vv - r), vf2 = (v_c - r) * (v_c - r);
      vf += 0.5 * fmax(vf1, vf2);
      if (vf2 > vf1) vfc += 1.0;
      else g_v = (float)((double)c1 * (vv - r) * inv_n);
      kl += 0.5 * diff * diff;
      rs += ratio;
    }
    d_lp[i] = g_lp;
    d_v[i] = g_v;
  }
  pg = block_sum_1024_d(pg, sh) * inv_n;
  vf = block_sum_1024_d(vf, sh) * inv_n;
  kl = block_sum_1024_d(kl, sh) * inv_n;
  rs = block_sum_1024_d(rs, sh) * inv_n;
  pgc = block_sum_1024_d(pgc, sh) * inv_n;
  vfc = block_sum_1024_d(vfc, sh) * inv_n;
  if (threadIdx.x == 0) {
    stats[0] = (float)(pg + (double)c1 * vf);
    stats[1] = (float)pg;
    stats[2] = (float)vf;
    stats[3] = (float)kl;
    stats[4] = (float)pgc;
    stats[5] = (float)vfc;
    stats[6] = (float)rs;
    stats[7] = (float)n;
  }
}

hipError_t launch_ppo_loss(const float* lp, const float* lp0, const float* adv, const float* v, const float* v0,
                           const float* ret, const int* kept, int B, int N, float eps, float eps_v, float c1,
                           float* d_lp, float* d_v, float* stats, hipStream_t s) {
  hipLaunchKernelGGL(ppo_loss_kernel, dim3(1), dim3(1024), 0, s, lp, lp0, adv, v, v0, ret, kept, B, N, eps, eps_v, c1,
                     d_lp, d_v, stats);
  return hipGetLastError();
}

hipError_t launch_ppo_rewards(const float* lp, const float* ref_full, const float* rm_full, const int* tokens, int B,
                              int Lq, int N, int eos_id, int pad_id, float beta, float miss, float* rewards,
                              float* scores, float* kl, int* kept, hipStream_t s) {
  hipLaunchKernelGGL(ppo_rewards_kernel, dim3(B), dim3(64), 0, s, lp, ref_full, rm_full, tokens, Lq, N, eos_id,
                     pad_id, beta, miss, rewards, scores, kl, kept);
  return hipGetLastError();
}

hipError_t launch_ppo_gae(const float* rewards, const float* values, long vstride, const int* kept, int B, int N,
                          float gamma, float lam, float* adv, float* ret, hipStream_t s) {
  hipLaunchKernelGGL(ppo_gae_kernel, dim3((B + 63) / 64), dim3(64), 0, s, rewards, values, vstride, kept, B, N, gamma,
                     lam, adv, ret);
  return hipGetLastError();
}

hipError_t launch_ppo_whiten(const float* x, const int* kept, int B, int N, int shift_mean, float* out,
                             hipStream_t s) {
  hipLaunchKernelGGL(ppo_whiten_kernel, dim3(1), dim3(1024), 0, s, x, kept, B, N, shift_mean, out);
  return hipGetLastError();
}

// ---- glue of the update loop ------------------------------------------------------------------------------
__global__ void ppo_slice_kernel(const float* __restrict__ lp_full, const float* __restrict__ val_full, int L, int Lq,
                                 int N, float* __restrict__ new_lp, float* __restrict__ new_v) {
  const int b = blockIdx.x;
  for (int j = threadIdx.x; j < N; j += blockDim.x) {
    new_lp[(size_t)b * N + j] = lp_full[(size_t)b * L + Lq + j];
    new_v[(size_t)b * N + j] = (Lq - 1 + j >= 0) ? val_full[(size_t)b * L + Lq - 1 + j] : 0.f;
  }
}

hipError_t launch_ppo_slice(const float* lp_full, const float* val_full, int B, int L, int Lq, int N, float* new_lp,
                            float* new_v, hipStream_t s) {
  hipLaunchKernelGGL(ppo_slice_kernel, dim3(B), dim3(64), 0, s, lp_full, val_full, L, Lq, N, new_lp, new_v);
  return hipGetLastError();
}

__global__ void ppo_pack_grads_kernel(const int32_t* __restrict__ tokens, int L, int Lq, int N,
                                      const int* __restrict__ start, const int* __restrict__ len,
                                      const int* __restrict__ cu, const float* __restrict__ d_lp,
                                      const float* __restrict__ d_v, int32_t* __restrict__ targets,
                                      float* __restrict__ gl, float* __restrict__ gv) {
  const int b = blockIdx.x;
  const int st = start[b], n = len[b], base = cu[b];
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    const int c = st + i;
    const bool nxt = i + 1 < n;  // the next token of the row is real
    const int jr = c + 1 - Lq;   // response index of the token this row predicts
    const int jv = c - (Lq - 1); // response index whose value is read at this position
    targets[base + i] = nxt ? tokens[(size_t)b * L + c + 1] : -1;
    gl[base + i] = (nxt && jr >= 0 && jr < N) ? d_lp[(size_t)b * N + jr] : 0.f;
    gv[base + i] = (jv >= 0 && jv < N) ? d_v[(size_t)b * N + jv] : 0.f;
  }
}

hipError_t launch_ppo_pack_grads(const int32_t* tokens, int B, int L, int Lq, int N, const int* start, const int* len,
                                 const int* cu, const float* d_lp, const float* d_v, int32_t* targets, float* gl,
                                 float* gv, hipStream_t s) {
  hipLaunchKernelGGL(ppo_pack_grads_kernel, dim3(B), dim3(256), 0, s, tokens, L, Lq, N, start, len, cu, d_lp, d_v,
                     targets, gl, gv);
  return hipGetLastError();
}

}  // namespace rlhf
