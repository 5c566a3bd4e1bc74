"""CPU oracle for the backward pass through the attention branch of one decoder layer.  TEST
INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py may import this module.
It shares no code with the HIP library and never imports it.  Plain float64 numpy; the chain rule of
the forward definition, composed from the layer pieces of oracle/neox_oracle.py (LayerNorm, rotary)
and the attention core of oracle/attention_backward_oracle.py.

Forward ([Tech stack] GPT-NeoX through `transformers`; parallel residual, so this branch is a
function of the layer input alone): for packed rows of independent sequences,

    a = LN1(x);  [q | k | v] = a Wqkv^T + bqkv  (heads of hd inside each section);
    q, k <- rotary turn of the first r dims of every head by the row's position in its sequence
            (pair (i, i + r/2), angle pos * base^(-2i/r));
    o = causal softmax attention per (sequence, head);   y = o Wo^T + bo.

Backward for an upstream gradient G = dL/dx_out (the residual's identity term is not part of this
branch): dbo = sum_t G, dWo = G^T o, do = G Wo; (dq, dk, dv) by the attention core's backward; the
rotary turn is orthogonal, so its transpose is the turn by the negative angle; dbqkv = sum_t
[dq | dk | dv], dWqkv = [dq | dk | dv]^T a, da = [dq | dk | dv] Wqkv; LN1 backward as in the MLP
branch.

The paper prints no numbers for this step.  Pins (tests/test_oracle_attn_branch_backward_pins.py):
the forward against the decoder layer of oracle/neox_oracle.py with its MLP silenced; central finite
differences of <G, y>; linearity in G.
"""
from __future__ import annotations

import numpy as np

from .attention_backward_oracle import attention_backward, attention_forward
from .neox_oracle import layer_norm, rope

F64 = np.float64


def _positions(cu, T):
    pos = np.zeros(T, np.int64)
    for b in range(len(cu) - 1):
        pos[int(cu[b]):int(cu[b + 1])] = np.arange(int(cu[b + 1]) - int(cu[b]))
    return pos


def attn_branch_forward(x, g1, b1, wqkv, bqkv, wo, bo, cu, H, hd, r, base=10000.0, ln_eps=1e-5):
    x = np.asarray(x, F64)
    T, d = x.shape
    pos = _positions(cu, T)
    a = layer_norm(x, np.asarray(g1, F64), np.asarray(b1, F64), ln_eps)
    qkv = a @ np.asarray(wqkv, F64).T + np.asarray(bqkv, F64)
    q = rope(qkv[:, :d].reshape(T, H, hd), pos, r, base).reshape(T, d) if r else qkv[:, :d]
    k = rope(qkv[:, d:2 * d].reshape(T, H, hd), pos, r, base).reshape(T, d) if r else qkv[:, d:2 * d]
    v = qkv[:, 2 * d:]
    o = attention_forward(q, k, v, cu, H, hd)
    y = o @ np.asarray(wo, F64).T + np.asarray(bo, F64)
    return y, dict(a=a, q=q, k=k, v=v, o=o, pos=pos)


def attn_branch_backward(x, g1, b1, wqkv, bqkv, wo, bo, d_out, cu, H, hd, r, base=10000.0, ln_eps=1e-5):
    """Returns a dict: d_x (this branch's term), d_ln_g, d_ln_b [d], d_w_qkv [3d, d], d_b_qkv [3d],
    d_w_o [d, d], d_b_o [d]."""
    x, G = np.asarray(x, F64), np.asarray(d_out, F64)
    T, d = x.shape
    _, c = attn_branch_forward(x, g1, b1, wqkv, bqkv, wo, bo, cu, H, hd, r, base, ln_eps)
    wqkv, wo, g1 = np.asarray(wqkv, F64), np.asarray(wo, F64), np.asarray(g1, F64)
    do = G @ wo
    dq, dk, dv = attention_backward(c["q"], c["k"], c["v"], do, cu, H, hd)
    if r:  # transpose of the turn = the turn by the negative angle
        dq = rope(dq.reshape(T, H, hd), -c["pos"], r, base).reshape(T, d)
        dk = rope(dk.reshape(T, H, hd), -c["pos"], r, base).reshape(T, d)
    dqkv = np.concatenate([dq, dk, dv], axis=1)
    da = dqkv @ wqkv
    mu = x.mean(1, keepdims=True)
    xc = x - mu
    rstd = 1.0 / np.sqrt((xc * xc).mean(1, keepdims=True) + ln_eps)
    xh = xc * rstd
    u = da * g1
    dx = rstd * (u - u.mean(1, keepdims=True) - xh * (u * xh).mean(1, keepdims=True))
    return dict(d_x=dx, d_ln_g=(da * xh).sum(0), d_ln_b=da.sum(0), d_w_qkv=dqkv.T @ c["a"], d_b_qkv=dqkv.sum(0),
                d_w_o=G.T @ c["o"], d_b_o=G.sum(0))
