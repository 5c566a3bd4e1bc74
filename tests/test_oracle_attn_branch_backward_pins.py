"""Pins of oracle/attn_branch_backward_oracle.py against things other than itself.  The paper prints no numbers for
this step."""
import numpy as np
import pytest

from oracle.attn_branch_backward_oracle import attn_branch_backward, attn_branch_forward

NAMES = ("g1", "b1", "wqkv", "bqkv", "wo", "bo")


def _case(seed, lens=(5, 2, 6), H=2, hd=6, r=4):
    g = np.random.default_rng(seed)
    d = H * hd
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    T = int(cu[-1])
    x = g.normal(0, 1.5, (T, d))
    p = dict(g1=g.normal(1, 0.2, d), b1=g.normal(0, 0.1, d), wqkv=g.normal(0, 0.5, (3 * d, d)),
             bqkv=g.normal(0, 0.2, 3 * d), wo=g.normal(0, 0.5, (d, d)), bo=g.normal(0, 0.2, d))
    G = g.normal(0, 1, (T, d))
    return x, p, G, cu, H, hd, r


def test_forward_is_the_attention_branch_of_the_decoder_layer():
    from oracle.neox_oracle import OracleModel, decoder_layer
    from synth import ModelConfig, make_weights
    cfg = ModelConfig(n_layers=1, d_model=16, n_heads=2, head_dim=8, rotary_dims=4, d_ff=24, vocab=32, dtype="fp32",
                      pad_id=0, eos_id=1)
    w = make_weights(cfg, 5, variant="test")
    w["layers.0.w_fc2"] = np.zeros_like(w["layers.0.w_fc2"])
    w["layers.0.b_fc2"] = np.zeros_like(w["layers.0.b_fc2"])
    m = OracleModel(w, cfg)
    lens = (5, 3)
    cu = np.array([0, 5, 8])
    x = np.random.default_rng(1).normal(0, 1, (8, cfg.d_model))
    L = lambda n: w[f"layers.0.{n}"]
    y, _ = attn_branch_forward(x, L("ln1_g"), L("ln1_b"), L("w_qkv"), L("b_qkv"), L("w_o"), L("b_o"), cu, 2, 8, 4,
                               cfg.rope_base, cfg.ln_eps)
    for b in range(2):
        s, e = int(cu[b]), int(cu[b + 1])
        res = decoder_layer(m, 0, x[s:e], np.arange(e - s))
        full = res[0] if isinstance(res, tuple) else res
        np.testing.assert_allclose(full, x[s:e] + y[s:e], rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("seed,r", [(0, 4), (1, 6), (2, 0)])
def test_gradients_match_central_differences_of_the_forward(seed, r):
    x, p, G, cu, H, hd, _ = _case(seed)
    args = lambda: [p[n] for n in NAMES]
    out = attn_branch_backward(x, *args(), G, cu, H, hd, r)
    L = lambda: float((attn_branch_forward(x, *args(), cu, H, hd, r)[0] * G).sum())
    g = np.random.default_rng(40 + seed)
    eps = 1e-6
    pairs = [(x, out["d_x"]), (p["g1"], out["d_ln_g"]), (p["b1"], out["d_ln_b"]), (p["wqkv"], out["d_w_qkv"]),
             (p["bqkv"], out["d_b_qkv"]), (p["wo"], out["d_w_o"]), (p["bo"], out["d_b_o"])]
    for arr, grad in pairs:
        for _ in range(6):
            idx = tuple(int(g.integers(0, n)) for n in arr.shape)
            old = arr[idx]
            arr[idx] = old + eps
            up = L()
            arr[idx] = old - eps
            dn = L()
            arr[idx] = old
            assert (up - dn) / (2 * eps) == pytest.approx(grad[idx], rel=5e-6, abs=1e-8)


def test_linear_in_the_upstream_gradient():
    x, p, G, cu, H, hd, r = _case(3)
    a = attn_branch_backward(x, *[p[n] for n in NAMES], G, cu, H, hd, r)
    b = attn_branch_backward(x, *[p[n] for n in NAMES], -3.0 * G, cu, H, hd, r)
    for k in a:
        np.testing.assert_allclose(b[k], -3.0 * a[k], rtol=1e-12, atol=1e-13)
