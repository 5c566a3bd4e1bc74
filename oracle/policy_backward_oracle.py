"""CPU oracle for the whole backward pass of the policy (with its value head): the chain of the
stage oracles over a packed batch.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py may import this module.
It shares no code with the HIP library and never imports it.  float64 numpy.

What it computes ([Tech stack] GPT-NeoX with parallel residual; [PPO Details] the update is
gradient descent on the PPO loss, whose gradient with respect to the model's outputs is the input
here): the forward pass of oracle/neox_oracle.py over every sequence, keeping the residual stream
at the input of each layer; then head_backward, and per layer from the last to the first
    dL/dx_in = dL/dx_out + (attention branch term) + (MLP branch term)
with the branch oracles; finally the input embedding's gradient, the sum of dL/dx_0 over the rows
that hold the same token.

Packing: the real tokens of row b of `tokens` (mask == 1, one contiguous run) become packed rows
cu[b] .. cu[b+1]-1 in order.  The packed row of token (b, t) predicts token (b, t+1): its target is
that token when it is real, else -1; `d_logprobs[b, t+1]` and `d_values[b, t]` are its gradients
(the index conventions of score_sequences' outputs).

Pin (tests/test_oracle_policy_backward_pins.py): central finite differences of
L = sum d_logprobs * logprobs + sum d_values * values evaluated with neox_oracle.score_sequences, a
forward pass that shares nothing with the stage oracles' own recomputation.
"""
from __future__ import annotations

import numpy as np

from .attn_branch_backward_oracle import attn_branch_backward
from .head_backward_oracle import head_backward
from .mlp_backward_oracle import mlp_backward
from .neox_oracle import OracleModel, decoder_layer

F64 = np.float64


def pack(tokens, mask, d_logprobs, d_values):
    """Returns (tok [T], cu [B+1], targets [T], gl [T], gv [T]) for the packed rows."""
    tokens, mask = np.asarray(tokens), np.asarray(mask).astype(bool)
    B, L = tokens.shape
    tok, tgt, gl, gv, cu = [], [], [], [], [0]
    for b in range(B):
        cols = np.flatnonzero(mask[b])
        for t in cols:
            tok.append(int(tokens[b, t]))
            nxt = t + 1 < L and mask[b, t + 1]
            tgt.append(int(tokens[b, t + 1]) if nxt else -1)
            gl.append(float(d_logprobs[b, t + 1]) if nxt else 0.0)
            gv.append(float(d_values[b, t]))
        cu.append(len(tok))
    return (np.asarray(tok, np.int64), np.asarray(cu, np.int64), np.asarray(tgt, np.int64), np.asarray(gl, F64),
            np.asarray(gv, F64))


def policy_backward(weights: dict, cfg, tokens, mask, d_logprobs, d_values, temperature):
    """Gradient of L with respect to every weight: dict with the names of `weights` (without 'value_b' -> also
    returned as 'value_b')."""
    m = OracleModel(weights, cfg)
    tok, cu, tgt, gl, gv = pack(tokens, mask, d_logprobs, d_values)
    T, d, nl = len(tok), cfg.d_model, cfg.n_layers
    xs = [m.get("embed_in")[tok].astype(F64)]
    for l in range(nl):
        nxt = np.empty_like(xs[-1])
        for b in range(len(cu) - 1):
            s, e = int(cu[b]), int(cu[b + 1])
            if e > s:
                res = decoder_layer(m, l, xs[-1][s:e], np.arange(e - s))
                nxt[s:e] = res[0] if isinstance(res, tuple) else res
        xs.append(nxt)
    g = {}
    hb = head_backward(xs[nl], m.get("lnf_g"), m.get("lnf_b"), m.get("embed_out"), m.get("value_w"), tgt, gl, gv,
                       temperature, ln_eps=cfg.ln_eps)
    g.update(lnf_g=hb["d_lnf_g"], lnf_b=hb["d_lnf_b"], embed_out=hb["d_embed_out"], value_w=hb["d_value_w"],
             value_b=hb["d_value_b"])
    dx = hb["d_x"]
    for l in range(nl - 1, -1, -1):
        W = lambda n: m.layer(l, n)
        mb = mlp_backward(xs[l], W("ln2_g"), W("ln2_b"), W("w_fc1"), W("b_fc1"), W("w_fc2"), W("b_fc2"), dx, cfg.ln_eps)
        ab = attn_branch_backward(xs[l], W("ln1_g"), W("ln1_b"), W("w_qkv"), W("b_qkv"), W("w_o"), W("b_o"), dx, cu,
                                  cfg.n_heads, cfg.head_dim, cfg.rotary_dims, cfg.rope_base, cfg.ln_eps)
        P = f"layers.{l}."
        g.update({P + "ln2_g": mb["d_ln_g"], P + "ln2_b": mb["d_ln_b"], P + "w_fc1": mb["d_w_fc1"],
                  P + "b_fc1": mb["d_b_fc1"], P + "w_fc2": mb["d_w_fc2"], P + "b_fc2": mb["d_b_fc2"],
                  P + "ln1_g": ab["d_ln_g"], P + "ln1_b": ab["d_ln_b"], P + "w_qkv": ab["d_w_qkv"],
                  P + "b_qkv": ab["d_b_qkv"], P + "w_o": ab["d_w_o"], P + "b_o": ab["d_b_o"]})
        dx = dx + ab["d_x"] + mb["d_x"]
    de = np.zeros_like(m.get("embed_in"), dtype=F64)
    np.add.at(de, tok, dx)
    g["embed_in"] = de
    return g
