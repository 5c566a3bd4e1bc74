"""CPU oracle for one PPO update of the policy (with its value head) on a rollout batch: the loop over
update iterations and mini-batches around the stage oracles.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py may import this module.
It shares no code with the HIP library and never imports it.  float64 numpy.

What it computes.  The paper gives the loop through its hyperparameters [PPO hyperparameter table:
K = 4 PPO update iterations per batch, N_mb = 1 mini-batch, AdamW (eps 1e-5, lr 3e-6), linear
scheduler, clipping coefficients 0.2, c1 = 0.1] and its lineage.  For iteration k = 0..K-1 and
mini-batch j = 0..N_mb-1, on the rows of that mini-batch:
    1. forward pass of the CURRENT weights over the (query + response) tokens: new log-probs of the
       response tokens and new values at the positions that emitted them (neox_oracle.score_sequences);
    2. the clipped objective against the rollout's log-probs / values, advantages and returns, averaged
       over the kept response tokens of the mini-batch (ppo_loss_oracle.ppo_loss), and its gradient
       with respect to the new log-probs and values;
    3. the gradient of every weight (policy_backward_oracle.policy_backward);
    4. one AdamW step on every weight (adamw_oracle.adamw_step), step counter first_step + (number of
       optimizer steps taken so far).

Readings where the paper is silent: a mini-batch is a contiguous slice of B / N_mb rows in row order
(a caller that wants shuffled mini-batches permutes the rows; with the paper's N_mb = 1 there is
nothing to shuffle); the learning rate is constant within one update (the linear schedule moves once
per rollout batch: the caller passes lr * (1 - k / K_total)); the old log-probs, values, advantages
and returns stay those of the rollout for all K iterations.

Pin (tests/test_oracle_ppo_update_pins.py): the same loop written with the `transformers` GPT-NeoX
class in float64, torch autograd and torch.optim.AdamW -- a forward, a differentiation and an
optimizer that share nothing with the stage oracles.
"""
from __future__ import annotations

import numpy as np

from . import adamw_oracle, ppo_loss_oracle
from .neox_oracle import OracleModel, score_sequences
from .policy_backward_oracle import policy_backward

F64 = np.float64


def ppo_update(weights: dict, cfg, tokens, mask, query_len: int, old_logprobs, advantages, old_values, returns,
               kept, temperature: float, epochs: int = 4, n_minibatches: int = 1, cliprange: float = 0.2,
               cliprange_value: float = 0.2, vf_coef: float = 0.1, lr: float = 3e-6, beta1: float = 0.9,
               beta2: float = 0.999, eps: float = 1e-5, weight_decay: float = 0.01, first_step: int = 1,
               state: dict | None = None, storage_round=None):
    """tokens, mask: [B, Lq + N]; old_logprobs, advantages, old_values, returns: [B, N]; kept: [B].
    storage_round: optional function array -> array.  Mixed-precision training as the paper runs it (bf16) keeps
    exact master weights for the optimizer while the forward and backward passes read the weights rounded to their
    storage type; with storage_round given, every pass reads storage_round(master) and the optimizer updates the
    masters.  None: the passes read the masters themselves.
    Returns (new weights: name -> float64 array, with 'value_b' a float; optimizer state: name ->
    (exp_avg, exp_avg_sq); list of the K * N_mb loss statistics in order)."""
    tokens, mask = np.asarray(tokens), np.asarray(mask)
    B, L = tokens.shape
    Lq = int(query_len)
    N = L - Lq
    if B % n_minibatches:
        raise ValueError("the batch must divide into the mini-batches")
    mb = B // n_minibatches
    w = {k: (np.array(v, F64) if k != "value_b" else float(v)) for k, v in weights.items()}
    state = {} if state is None else {k: (np.array(m, F64), np.array(v, F64)) for k, (m, v) in state.items()}
    stats_all = []
    step = int(first_step)
    for _ in range(epochs):
        for j in range(n_minibatches):
            r = slice(j * mb, (j + 1) * mb)
            if storage_round is None:
                wf = w
            else:  # value_b stays a plain scalar: it has no reduced-precision storage copy
                wf = {k: (np.asarray(storage_round(np.asarray(v, np.float32)), F64) if k != "value_b" else v)
                      for k, v in w.items()}
            lp, val = score_sequences(OracleModel(wf, cfg, cache_f64=False), tokens[r], mask[r], temperature)
            new_lp = lp[:, Lq:]
            new_v = val[:, Lq - 1:Lq - 1 + N]
            stats, d_lp, d_v = ppo_loss_oracle.ppo_loss(new_lp, old_logprobs[r], advantages[r], new_v, old_values[r],
                                                        returns[r], kept[r], cliprange, cliprange_value, vf_coef)
            stats_all.append(stats)
            GL, GV = np.zeros((mb, L), F64), np.zeros((mb, L), F64)
            GL[:, Lq:] = d_lp
            GV[:, Lq - 1:Lq - 1 + N] = d_v
            grads = policy_backward(wf, cfg, tokens[r], mask[r], GL, GV, temperature)
            for name, g in grads.items():
                p = np.asarray(w[name], F64)
                g = np.asarray(g, F64).reshape(p.shape)
                m0, v0 = state.get(name, (np.zeros(p.shape, F64), np.zeros(p.shape, F64)))
                p1, m1, v1 = adamw_oracle.adamw_step(p, g, m0, v0, step, lr=lr, beta1=beta1, beta2=beta2, eps=eps,
                                                     weight_decay=weight_decay)
                state[name] = (m1, v1)
                w[name] = float(p1) if name == "value_b" else p1
            step += 1
    return w, state, stats_all
