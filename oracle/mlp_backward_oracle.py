"""CPU oracle for the backward pass through the MLP branch of one decoder layer.  TEST
INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py may import this module.
It shares no code with the HIP library and never imports it.  Plain float64 numpy; each gradient is
the chain rule of the forward definition written out.

Forward (the paper's model, [Tech stack] GPT-NeoX through `transformers`: parallel residual, so
the layer is x_out = x + attention(LN1(x)) + mlp(LN2(x)) and the two branches are independent
functions of the layer input):

    m = LN2(x) = (x - mean) / sqrt(var + eps) * g + b          (biased variance, per row)
    u = m W1^T + b1,   f = gelu(u) = u * Phi(u)  (exact erf form),   y = f W2^T + b2

For an upstream gradient G = dL/dx_out (the residual passes it on unchanged; that identity term is
not part of this branch) the chain rule gives, with phi the standard normal density:

    dL/db2 = sum_t G_t            dL/dW2 = G^T f            dL/df = G W2
    dL/du  = dL/df * (Phi(u) + u * phi(u))
    dL/db1 = sum_t dL/du_t        dL/dW1 = (dL/du)^T m      dL/dm = dL/du W1
    dL/dg  = sum_t dL/dm * xh     dL/db  = sum_t dL/dm
    branch term of dL/dx_t = rstd * (v - mean(v) - xh * mean(v * xh)),  v = dL/dm_t * g

The paper prints no numbers for this step (it trains through autograd).  Pins
(tests/test_oracle_mlp_backward_pins.py): central finite differences of <G, y> evaluated with
`mlp_forward`; reverse-mode differentiation of an independently written torch float64 forward;
the forward itself against the layer of oracle/neox_oracle.py; linearity in G.
"""
from __future__ import annotations

import math

import numpy as np

F64 = np.float64
_erf = np.vectorize(math.erf, otypes=[F64])


def mlp_forward(x, g, b, w1, b1, w2, b2, ln_eps=1e-5):
    """x [T, d] -> y [T, d] = mlp(LN2(x)); returns (y, cache of intermediates)."""
    x = np.asarray(x, F64)
    mu = x.mean(1, keepdims=True)
    xc = x - mu
    rstd = 1.0 / np.sqrt((xc * xc).mean(1, keepdims=True) + ln_eps)
    xh = xc * rstd
    m = xh * np.asarray(g, F64) + np.asarray(b, F64)
    u = m @ np.asarray(w1, F64).T + np.asarray(b1, F64)
    f = 0.5 * u * (1.0 + _erf(u / math.sqrt(2.0)))
    y = f @ np.asarray(w2, F64).T + np.asarray(b2, F64)
    return y, dict(xh=xh, rstd=rstd, m=m, u=u, f=f)


def mlp_backward(x, g, b, w1, b1, w2, b2, d_out, ln_eps=1e-5):
    """Gradients of L for dL/dx_out = d_out [T, d].  Returns a dict with d_x (this branch's term
    only), d_ln_g, d_ln_b [d], d_w_fc1 [F, d], d_b_fc1 [F], d_w_fc2 [d, F], d_b_fc2 [d]."""
    G = np.asarray(d_out, F64)
    _, c = mlp_forward(x, g, b, w1, b1, w2, b2, ln_eps)
    w1, w2, g = np.asarray(w1, F64), np.asarray(w2, F64), np.asarray(g, F64)
    u = c["u"]
    df = G @ w2
    Phi = 0.5 * (1.0 + _erf(u / math.sqrt(2.0)))
    phi = np.exp(-0.5 * u * u) / math.sqrt(2.0 * math.pi)
    du = df * (Phi + u * phi)
    dm = du @ w1
    v = dm * g
    xh = c["xh"]
    dx = c["rstd"] * (v - v.mean(1, keepdims=True) - xh * (v * xh).mean(1, keepdims=True))
    return dict(d_x=dx, d_ln_g=(dm * xh).sum(0), d_ln_b=dm.sum(0), d_w_fc1=du.T @ c["m"], d_b_fc1=du.sum(0),
                d_w_fc2=G.T @ c["f"], d_b_fc2=G.sum(0))
