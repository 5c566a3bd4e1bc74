"""CPU oracle for the backward pass through the model's output heads: from the gradients of the
PPO loss with respect to the new log-probs and values back to the residual stream after the last
decoder layer and to the head parameters.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py may import this module.
It shares no code with the HIP library and never imports it.  Plain float64 numpy, one row at a
time, each gradient the chain rule of the forward definition written out.

Forward (the paper's model, [Tech stack] GPT-NeoX through `transformers`; [Preliminaries] Step 2 /
[PPO Details] "Value model initializes from the reward model" for the scalar head; sampling
temperature of [General Details] / [PPO Details] applied to the logits before the softmax):

    h_t   = LN_f(x_t)            = (x_t - mean) / sqrt(var + eps) * g + b      (biased variance)
    z_t   = W h_t                  (untied LM head, no bias)
    lp_t  = log softmax(z_t / T)[y_t]        for rows with a target y_t >= 0
    v_t   = w_v . h_t + b_v

For a scalar loss L with dL/dlp_t = gl_t and dL/dv_t = gv_t (what the loss head returns) the
chain rule gives, with p_t = softmax(z_t / T), xh = (x - mean) / sqrt(var + eps):

    dL/dz_t   = gl_t / T * (onehot(y_t) - p_t)                 (0 where y_t < 0)
    dL/dW     = sum_t dL/dz_t  (outer)  h_t
    dL/dh_t   = W^T dL/dz_t + gv_t * w_v
    dL/dw_v   = sum_t gv_t h_t ,   dL/db_v = sum_t gv_t
    dL/dg     = sum_t dL/dh_t * xh_t ,   dL/db = sum_t dL/dh_t
    dL/dx_t   = rstd_t * (u - mean(u) - xh_t * mean(u * xh_t)),   u = dL/dh_t * g

The paper prints no numbers for this step (it trains through autograd).  Pins
(tests/test_oracle_head_backward_pins.py): central finite differences of L = sum gl*lp + sum gv*v
evaluated with `head_forward`; the same gradients from reverse-mode differentiation of an
independently written torch float64 forward; invariants (rows of dL/dz sum to zero, so the columns
of dL/dW sum to zero over the vocabulary; dL/dx_t has zero mean and is orthogonal to xh_t; rows
without a target and with gv = 0 get a zero gradient).
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def head_forward(x, lnf_g, lnf_b, embed_out, value_w, value_b, targets, temperature, ln_eps=1e-5):
    """x [T, d]; targets [T] int (-1: no log-prob for that row).  Returns (lp [T], v [T]); lp is 0
    where there is no target."""
    x = np.asarray(x, F64)
    g, b = np.asarray(lnf_g, F64), np.asarray(lnf_b, F64)
    W, wv = np.asarray(embed_out, F64), np.asarray(value_w, F64)
    T = x.shape[0]
    lp, v = np.zeros(T, F64), np.zeros(T, F64)
    for t in range(T):
        mu = x[t].mean()
        xc = x[t] - mu
        rstd = 1.0 / np.sqrt((xc * xc).mean() + ln_eps)
        h = xc * rstd * g + b
        v[t] = h @ wv + float(value_b)
        y = int(targets[t])
        if y >= 0:
            z = (W @ h) / float(temperature)
            mx = z.max()
            lp[t] = z[y] - (mx + np.log(np.exp(z - mx).sum()))
    return lp, v


def head_backward(x, lnf_g, lnf_b, embed_out, value_w, targets, d_logprobs, d_values, temperature,
                  ln_eps=1e-5):
    """Gradients of L (see the module text).  Returns a dict with d_x [T, d], d_lnf_g [d],
    d_lnf_b [d], d_embed_out [V, d], d_value_w [d], d_value_b (float)."""
    x = np.asarray(x, F64)
    g, b = np.asarray(lnf_g, F64), np.asarray(lnf_b, F64)
    W, wv = np.asarray(embed_out, F64), np.asarray(value_w, F64)
    gl, gv = np.asarray(d_logprobs, F64), np.asarray(d_values, F64)
    T, d = x.shape
    out = dict(d_x=np.zeros((T, d), F64), d_lnf_g=np.zeros(d, F64), d_lnf_b=np.zeros(d, F64),
               d_embed_out=np.zeros_like(W), d_value_w=np.zeros(d, F64), d_value_b=0.0)
    for t in range(T):
        mu = x[t].mean()
        xc = x[t] - mu
        rstd = 1.0 / np.sqrt((xc * xc).mean() + ln_eps)
        xh = xc * rstd
        h = xh * g + b
        dh = gv[t] * wv
        out["d_value_w"] += gv[t] * h
        out["d_value_b"] += gv[t]
        y = int(targets[t])
        if y >= 0:
            z = (W @ h) / float(temperature)
            p = np.exp(z - z.max())
            p /= p.sum()
            dz = -p
            dz[y] += 1.0
            dz *= gl[t] / float(temperature)
            out["d_embed_out"] += np.outer(dz, h)
            dh = dh + W.T @ dz
        out["d_lnf_g"] += dh * xh
        out["d_lnf_b"] += dh
        u = dh * g
        out["d_x"][t] = rstd * (u - u.mean() - xh * (u * xh).mean())
    return out
