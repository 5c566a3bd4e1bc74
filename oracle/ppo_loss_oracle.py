"""CPU oracle for the PPO objective on a rollout batch and its gradient with respect to the model's
outputs (new log-probs and new values).  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py may import this module.
It shares no code with the HIP library and never imports it.  Plain float64 numpy and Python
loops, one token at a time, in the order of the definitions.

What it computes.  The paper names the objective only through its hyperparameters [PPO
hyperparameter table: policy clipping coefficient 0.2, value clipping coefficient 0.2, value
function coefficient c1 = 0.1, value function loss clipping True] and its lineage; the readings
taken here are the standard ones of that lineage:

  * ratio_t = exp(logp_new_t - logp_old_t); policy term max(-A_t ratio_t, -A_t clip(ratio_t, 1-eps,
    1+eps)) (the pessimistic clipped surrogate of PPO), averaged over the kept response tokens of
    the batch;
  * value term 0.5 * max((V_t - R_t)^2, (clip(V_t, Vold_t - eps_v, Vold_t + eps_v) - R_t)^2), same
    average; loss = policy + c1 * value;
  * statistics: approx_kl = 0.5 * mean((logp_new - logp_old)^2), the fractions of tokens where the
    clipped branch is the strictly larger one, the mean ratio;
  * gradients of `loss` with respect to logp_new and V: where the unclipped branch is the larger
    one or the two are equal (inside the clip range they are the same function) the gradient is
    that of the unclipped branch, -A ratio / n and c1 (V - R) / n; where the clipped branch is
    strictly larger it is 0 (a clipped quantity does not move with its argument).  Positions that
    are not kept have zero gradient.  An empty batch (no kept token) gives zero loss and gradients.

Pins (tests/test_oracle_ppo_loss_pins.py): new == old gives ratio 1, loss -mean(A) + c1 * 0.5 *
mean((V-R)^2) and gradient -A/n; a four-token example worked by hand with both clips active in
both directions; central finite differences of `loss` against the returned gradients at random
points; invariance to what masked-out positions hold; batch duplication halves the gradients.
The paper prints no numbers for this step.
"""
from __future__ import annotations

import math

import numpy as np

F64 = np.float64


def ppo_loss(new_logprobs, old_logprobs, advantages, new_values, old_values, returns, kept,
             cliprange: float = 0.2, cliprange_value: float = 0.2, vf_coef: float = 0.1):
    """All arrays [B, N] over response positions; kept [B] = kept tokens per row.  Returns
    (stats dict, d_logprobs [B, N], d_values [B, N])."""
    lp = np.asarray(new_logprobs, F64)
    lp0 = np.asarray(old_logprobs, F64)
    adv = np.asarray(advantages, F64)
    v = np.asarray(new_values, F64)
    v0 = np.asarray(old_values, F64)
    ret = np.asarray(returns, F64)
    B, N = lp.shape
    n = int(sum(min(max(int(kept[b]), 0), N) for b in range(B)))
    d_lp = np.zeros((B, N), F64)
    d_v = np.zeros((B, N), F64)
    stats = dict(loss=0.0, pg_loss=0.0, vf_loss=0.0, approx_kl=0.0, pg_clipfrac=0.0, vf_clipfrac=0.0,
                 ratio_mean=0.0, n_tokens=float(n))
    if n == 0:
        return stats, d_lp, d_v
    pg_sum = vf_sum = kl_sum = ratio_sum = 0.0
    pg_clipped = vf_clipped = 0
    for b in range(B):
        for t in range(min(max(int(kept[b]), 0), N)):
            diff = lp[b, t] - lp0[b, t]
            ratio = math.exp(diff)
            ratio_c = min(max(ratio, 1.0 - cliprange), 1.0 + cliprange)
            pg1 = -adv[b, t] * ratio
            pg2 = -adv[b, t] * ratio_c
            pg_sum += max(pg1, pg2)
            if pg2 > pg1:
                pg_clipped += 1
            else:
                d_lp[b, t] = -adv[b, t] * ratio / n
            v_c = min(max(v[b, t], v0[b, t] - cliprange_value), v0[b, t] + cliprange_value)
            vf1 = (v[b, t] - ret[b, t]) ** 2
            vf2 = (v_c - ret[b, t]) ** 2
            vf_sum += 0.5 * max(vf1, vf2)
            if vf2 > vf1:
                vf_clipped += 1
            else:
                d_v[b, t] = vf_coef * (v[b, t] - ret[b, t]) / n
            kl_sum += 0.5 * diff * diff
            ratio_sum += ratio
    stats["pg_loss"] = pg_sum / n
    stats["vf_loss"] = vf_sum / n
    stats["loss"] = stats["pg_loss"] + vf_coef * stats["vf_loss"]
    stats["approx_kl"] = kl_sum / n
    stats["pg_clipfrac"] = pg_clipped / n
    stats["vf_clipfrac"] = vf_clipped / n
    stats["ratio_mean"] = ratio_sum / n
    return stats, d_lp, d_v
