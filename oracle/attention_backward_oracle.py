"""CPU oracle for the backward pass through packed causal softmax attention (the core of a decoder
layer's attention branch: after the rotary turn, before the out-projection).  TEST INFRASTRUCTURE
ONLY.

Only tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py may import this module.
It shares no code with the HIP library and never imports it.  Plain float64 numpy, one (sequence,
head) pair at a time, the chain rule of the definition written out.

Forward ([Tech stack]: GPT-NeoX attention through `transformers`; sequences are independent, a
query attends to the keys of its own sequence at positions <= its own, scores scaled by
1/sqrt(head_dim)): for one sequence and head, with Q, K, V of shape [n, hd],

    S = Q K^T / sqrt(hd),  P = softmax over j <= i of S_ij,  O = P V.

For an upstream gradient dO the chain rule gives

    dV = P^T dO,   dP = dO V^T,   dS_ij = P_ij (dP_ij - sum_k P_ik dP_ik),
    dQ = dS K / sqrt(hd),   dK = dS^T Q / sqrt(hd).

The paper prints no numbers for this step (it trains through autograd).  Pins
(tests/test_oracle_attention_backward_pins.py): the forward against the attention of
oracle/neox_oracle.py; central finite differences of <dO, O>; reverse-mode differentiation of an
independently written torch float64 forward; invariants (rows of dS sum to zero, so shifting all of
a query's scores changes nothing: <dQ_i, c> = 0 for any c with K c constant is implied; the last
key of a sequence gets gradient from the last query only; sequences do not mix).
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def _split(x, H, hd):
    x = np.asarray(x, F64)
    return x.reshape(x.shape[0], H, hd)


def attention_forward(q, k, v, cu_seqlens, H, hd):
    """q, k, v [T, H*hd] packed rows; cu_seqlens [B+1].  Returns O [T, H*hd]."""
    q3, k3, v3 = _split(q, H, hd), _split(k, H, hd), _split(v, H, hd)
    out = np.zeros_like(q3)
    for b in range(len(cu_seqlens) - 1):
        s, e = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        n = e - s
        mask = np.tril(np.ones((n, n), bool))
        for h in range(H):
            S = q3[s:e, h] @ k3[s:e, h].T / np.sqrt(hd)
            S = np.where(mask, S, -np.inf)
            P = np.exp(S - S.max(1, keepdims=True))
            P /= P.sum(1, keepdims=True)
            out[s:e, h] = P @ v3[s:e, h]
    return out.reshape(out.shape[0], H * hd)


def attention_backward(q, k, v, d_out, cu_seqlens, H, hd):
    """Returns (dq, dk, dv), each [T, H*hd]."""
    q3, k3, v3, g3 = _split(q, H, hd), _split(k, H, hd), _split(v, H, hd), _split(d_out, H, hd)
    dq, dk, dv = np.zeros_like(q3), np.zeros_like(q3), np.zeros_like(q3)
    for b in range(len(cu_seqlens) - 1):
        s, e = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        n = e - s
        mask = np.tril(np.ones((n, n), bool))
        for h in range(H):
            Q, K, V, G = q3[s:e, h], k3[s:e, h], v3[s:e, h], g3[s:e, h]
            S = np.where(mask, Q @ K.T / np.sqrt(hd), -np.inf)
            P = np.exp(S - S.max(1, keepdims=True))
            P /= P.sum(1, keepdims=True)
            dP = G @ V.T
            dS = P * (dP - (P * dP).sum(1, keepdims=True))
            dv[s:e, h] = P.T @ G
            dq[s:e, h] = dS @ K / np.sqrt(hd)
            dk[s:e, h] = dS.T @ Q / np.sqrt(hd)
    T = q3.shape[0]
    return dq.reshape(T, H * hd), dk.reshape(T, H * hd), dv.reshape(T, H * hd)
