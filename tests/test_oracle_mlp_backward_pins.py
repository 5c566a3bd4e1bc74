"""Pins of oracle/mlp_backward_oracle.py against things other than itself: finite differences of the forward
definition, reverse-mode differentiation of an independently written torch float64 forward, the forward against the
decoder layer of oracle/neox_oracle.py, linearity.  The paper prints no numbers for this step."""
import numpy as np
import pytest
import torch

from oracle.mlp_backward_oracle import mlp_backward, mlp_forward

NAMES = ("g", "b", "w1", "b1", "w2", "b2")


def _case(seed, T=6, d=10, F=14):
    r = np.random.default_rng(seed)
    x = r.normal(0, 1.5, (T, d))
    p = dict(g=r.normal(1, 0.2, d), b=r.normal(0, 0.1, d), w1=r.normal(0, 0.5, (F, d)), b1=r.normal(0, 0.2, F),
             w2=r.normal(0, 0.5, (d, F)), b2=r.normal(0, 0.2, d))
    G = r.normal(0, 1, (T, d))
    return x, p, G


def _L(x, p, G):
    return float((mlp_forward(x, *[p[n] for n in NAMES])[0] * G).sum())


@pytest.mark.parametrize("seed", [0, 1])
def test_gradients_match_central_differences_of_the_forward(seed):
    x, p, G = _case(seed)
    out = mlp_backward(x, *[p[n] for n in NAMES], G)
    r = np.random.default_rng(20 + seed)
    eps = 1e-6
    pairs = [(x, out["d_x"]), (p["g"], out["d_ln_g"]), (p["b"], out["d_ln_b"]), (p["w1"], out["d_w_fc1"]),
             (p["b1"], out["d_b_fc1"]), (p["w2"], out["d_w_fc2"]), (p["b2"], out["d_b_fc2"])]
    for arr, grad in pairs:
        for _ in range(6):
            idx = tuple(int(r.integers(0, n)) for n in arr.shape)
            old = arr[idx]
            arr[idx] = old + eps
            up = _L(x, p, G)
            arr[idx] = old - eps
            dn = _L(x, p, G)
            arr[idx] = old
            assert (up - dn) / (2 * eps) == pytest.approx(grad[idx], rel=2e-6, abs=1e-8)


def test_gradients_match_torch_autograd():
    x, p, G = _case(3, T=8, d=12, F=20)
    out = mlp_backward(x, *[p[n] for n in NAMES], G)
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    tp = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()}
    m = torch.nn.functional.layer_norm(tx, (x.shape[1],), tp["g"], tp["b"], 1e-5)
    y = torch.nn.functional.gelu(m @ tp["w1"].T + tp["b1"]) @ tp["w2"].T + tp["b2"]
    (y * torch.tensor(G)).sum().backward()
    ref = dict(d_x=tx.grad, d_ln_g=tp["g"].grad, d_ln_b=tp["b"].grad, d_w_fc1=tp["w1"].grad, d_b_fc1=tp["b1"].grad,
               d_w_fc2=tp["w2"].grad, d_b_fc2=tp["b2"].grad)
    for k, v in ref.items():
        np.testing.assert_allclose(out[k], v.numpy(), rtol=1e-9, atol=1e-12, err_msg=k)


def test_forward_is_the_mlp_branch_of_the_decoder_layer():
    """The layer of the forward oracle with its attention branch silenced (zero out-projection) is x + mlp(LN2(x))."""
    from oracle.neox_oracle import OracleModel, decoder_layer
    from synth import ModelConfig, make_weights
    cfg = ModelConfig(n_layers=1, d_model=16, n_heads=2, head_dim=8, rotary_dims=4, d_ff=24, vocab=32, dtype="fp32",
                      pad_id=0, eos_id=1)
    w = make_weights(cfg, 3, variant="test")
    w["layers.0.w_o"] = np.zeros_like(w["layers.0.w_o"])
    w["layers.0.b_o"] = np.zeros_like(w["layers.0.b_o"])
    m = OracleModel(w, cfg)
    x = np.random.default_rng(0).normal(0, 1, (5, cfg.d_model))
    res = decoder_layer(m, 0, x, np.arange(5))
    full = res[0] if isinstance(res, tuple) else res
    L = lambda n: w[f"layers.0.{n}"]
    y, _ = mlp_forward(x, L("ln2_g"), L("ln2_b"), L("w_fc1"), L("b_fc1"), L("w_fc2"), L("b_fc2"), cfg.ln_eps)
    np.testing.assert_allclose(full, x + y, rtol=1e-12, atol=1e-12)


def test_linear_in_the_upstream_gradient_and_zero_rows_give_zero():
    x, p, G = _case(4)
    a = mlp_backward(x, *[p[n] for n in NAMES], G)
    b = mlp_backward(x, *[p[n] for n in NAMES], -2.5 * G)
    for k in a:
        np.testing.assert_allclose(b[k], -2.5 * a[k], rtol=1e-12, atol=1e-14)
    G2 = G.copy()
    G2[3] = 0.0
    c = mlp_backward(x, *[p[n] for n in NAMES], G2)
    assert np.all(c["d_x"][3] == 0.0)
