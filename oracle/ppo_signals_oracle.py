"""CPU oracle for what PPO consumes after a rollout: per-token rewards, advantages, returns,
whitening.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py may import this module.
It shares no code with the HIP library and never imports it.  Plain float64 numpy and Python
loops, written out in the order of the definitions.

What it computes (paper passages in brackets) and the readings taken where the paper is silent:

  * `rm_score_index`, `assemble_rewards` -- the reward of the RL problem, R = r - beta * KL
    [Preliminaries, Eq. (RL)], laid out per token as in the figure "Reward and values of a
    completion" [PPO Details, "Value model initializes from the reward model ..."]: every kept
    response token carries the KL penalty -beta * (log pi(y_t) - log pi_sft(y_t)) and the last kept
    token additionally carries the reward-model score.  The score is read at the index of the
    first padding token of the response minus one, i.e. at the EOS token, or at the last token if
    there is no padding [Reward Model Details, "Extract reward from the EOS token"]; a response
    without EOS gets the constant -1 in place of the score [PPO Details, "EOS trick", step 3].
    Readings: the KL term is the sampled-token estimate log pi - log pi_sft summed over the kept
    tokens (the paper gives the divergence only as a symbol; its figure shows one penalty per
    token); tokens after the first EOS carry reward 0; a row with no response (length 0) carries
    only zeros.  beta = 0.05 [PPO hyperparameter table].
  * `gae` -- generalised advantage estimation with discount gamma = 1 and lambda = 0.95 [PPO
    hyperparameter table]; the paper names the estimator but does not print it, so the standard
    definition is used: delta_t = r_t + gamma * V_{t+1} - V_t, A_t = sum_l (gamma*lambda)^l
    delta_{t+l}, with V = 0 beyond the last kept token; returns = A + V.  Positions after the
    last kept token hold 0.
  * `whiten` -- the normalisation the paper prints [PPO Details, "(Optional) Reward whitening",
    "Advantage whitening"]: biased variance, 1e-8 inside the square root, and the flag whose False
    value adds the mean back.  Reading: statistics run over the kept tokens of the batch when a
    mask is given (the printed function takes a dense tensor; with an all-ones mask the two
    agree), and masked-out positions stay 0.

Pins (tests/test_oracle_ppo_pins.py): the Eq. (RL) identity sum_t reward_t = score - beta * KL; the
-1 replacement; lambda = 1 and lambda = 0 closed forms of GAE, the defining double sum, a
geometric-series case; whitening against numpy's mean / var on dense input, scale and shift
invariance, mean restored when the flag is False.  The paper prints no numbers for these steps.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def rm_score_index(response_tokens, pad_id: int) -> int:
    """Index (within the response) where the reward model's scalar is read: first pad minus one,
    or the last token when the response holds no pad.  -1 for a response that starts with pad."""
    n = len(response_tokens)
    for t in range(n):
        if response_tokens[t] == pad_id:
            return t - 1
    return n - 1


def assemble_rewards(logprobs, ref_logprobs, rm_values, response_tokens, eos_id: int, pad_id: int,
                     beta: float, missing_eos_score: float = -1.0):
    """logprobs, ref_logprobs, rm_values, response_tokens: [B, N] over the response positions
    (rm_values[b, t] = reward-model scalar at response token t).  Returns rewards [B, N] float64,
    the per-row score that was used [B] and the per-row KL sum [B]."""
    lp = np.asarray(logprobs, F64)
    rlp = np.asarray(ref_logprobs, F64)
    rv = np.asarray(rm_values, F64)
    tok = np.asarray(response_tokens)
    B, N = tok.shape
    rewards = np.zeros((B, N), F64)
    scores = np.zeros(B, F64)
    kl_sum = np.zeros(B, F64)
    for b in range(B):
        last = rm_score_index(tok[b], pad_id)
        if last < 0:
            continue  # nothing was generated for this row
        for t in range(last + 1):
            kl = lp[b, t] - rlp[b, t]
            kl_sum[b] += kl
            rewards[b, t] = -beta * kl
        has_eos = tok[b, last] == eos_id
        scores[b] = rv[b, last] if has_eos else missing_eos_score
        rewards[b, last] += scores[b]
    return rewards, scores, kl_sum


def gae(rewards, values, lengths, gamma: float, lam: float):
    """rewards, values: [B, N]; lengths [B] = kept response tokens.  Returns (advantages, returns),
    both [B, N] float64, zero at t >= lengths[b]."""
    r = np.asarray(rewards, F64)
    v = np.asarray(values, F64)
    B, N = r.shape
    adv = np.zeros((B, N), F64)
    ret = np.zeros((B, N), F64)
    for b in range(B):
        L = int(lengths[b])
        running = 0.0
        for t in range(L - 1, -1, -1):
            v_next = v[b, t + 1] if t + 1 < L else 0.0
            delta = r[b, t] + gamma * v_next - v[b, t]
            running = delta + gamma * lam * running
            adv[b, t] = running
            ret[b, t] = running + v[b, t]
    return adv, ret


def whiten(values, mask=None, shift_mean: bool = True):
    """(values - mean) / sqrt(var + 1e-8) with the biased variance, mean added back when shift_mean
    is False.  With a mask, statistics are over mask == 1 and other positions return 0."""
    x = np.asarray(values, F64)
    if mask is None:
        sel = np.ones(x.shape, bool)
    else:
        sel = np.asarray(mask).astype(bool)
    n = int(sel.sum())
    out = np.zeros(x.shape, F64)
    if n == 0:
        return out
    mean = 0.0
    for val in x[sel]:
        mean += val
    mean /= n
    var = 0.0
    for val in x[sel]:
        var += (val - mean) * (val - mean)
    var /= n
    w = (x - mean) / np.sqrt(var + 1e-8)
    if not shift_mean:
        w = w + mean
    out[sel] = w[sel]
    return out
