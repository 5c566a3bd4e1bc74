"""Pins of oracle/head_backward_oracle.py against things other than itself: finite differences of the forward
definition, reverse-mode differentiation of an independently written torch float64 forward, and invariants of the
softmax and LayerNorm gradients.  The paper prints no numbers for this step."""
import numpy as np
import pytest
import torch

from oracle.head_backward_oracle import head_backward, head_forward


def _case(seed, T=7, d=12, V=19):
    g = np.random.default_rng(seed)
    x = g.normal(0, 1.5, (T, d))
    p = dict(lnf_g=g.normal(1, 0.2, d), lnf_b=g.normal(0, 0.1, d), embed_out=g.normal(0, 0.4, (V, d)),
             value_w=g.normal(0, 0.3, d), value_b=0.17)
    y = g.integers(0, V, T)
    y[2] = -1                      # a row without a log-prob term
    gl, gv = g.normal(0, 1, T), g.normal(0, 1, T)
    gv[4] = 0.0
    return x, p, y, gl, gv


def _loss(x, p, y, gl, gv, T=0.7):
    lp, v = head_forward(x, p["lnf_g"], p["lnf_b"], p["embed_out"], p["value_w"], p["value_b"], y, T)
    return float((gl * lp).sum() + (gv * v).sum())


@pytest.mark.parametrize("seed", [0, 1])
def test_gradients_match_central_differences_of_the_forward(seed):
    x, p, y, gl, gv = _case(seed)
    out = head_backward(x, p["lnf_g"], p["lnf_b"], p["embed_out"], p["value_w"], y, gl, gv, 0.7)
    g = np.random.default_rng(10 + seed)
    eps = 1e-6

    def fd(arr, idx):
        old = arr[idx]
        arr[idx] = old + eps
        up = _loss(x, p, y, gl, gv)
        arr[idx] = old - eps
        dn = _loss(x, p, y, gl, gv)
        arr[idx] = old
        return (up - dn) / (2 * eps)

    for _ in range(12):
        i = (int(g.integers(0, x.shape[0])), int(g.integers(0, x.shape[1])))
        assert fd(x, i) == pytest.approx(out["d_x"][i], rel=1e-6, abs=1e-8)
        j = (int(g.integers(0, p["embed_out"].shape[0])), int(g.integers(0, x.shape[1])))
        assert fd(p["embed_out"], j) == pytest.approx(out["d_embed_out"][j], rel=1e-6, abs=1e-8)
        k = int(g.integers(0, x.shape[1]))
        assert fd(p["lnf_g"], k) == pytest.approx(out["d_lnf_g"][k], rel=1e-6, abs=1e-8)
        assert fd(p["lnf_b"], k) == pytest.approx(out["d_lnf_b"][k], rel=1e-6, abs=1e-8)
        assert fd(p["value_w"], k) == pytest.approx(out["d_value_w"][k], rel=1e-6, abs=1e-8)
    assert out["d_value_b"] == pytest.approx(gv.sum(), rel=1e-12)


def test_gradients_match_torch_autograd():
    x, p, y, gl, gv = _case(3, T=9, d=16, V=23)
    out = head_backward(x, p["lnf_g"], p["lnf_b"], p["embed_out"], p["value_w"], y, gl, gv, 0.7)
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    tp = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items() if k != "value_b"}
    tb = torch.tensor(p["value_b"], dtype=torch.float64, requires_grad=True)
    h = torch.nn.functional.layer_norm(tx, (x.shape[1],), tp["lnf_g"], tp["lnf_b"], 1e-5)
    lsm = torch.log_softmax(h @ tp["embed_out"].T / 0.7, dim=-1)
    keep = torch.tensor(y >= 0)
    lp = lsm[torch.arange(len(y)), torch.tensor(np.maximum(y, 0))] * keep
    v = h @ tp["value_w"] + tb
    (torch.tensor(gl) * lp + torch.tensor(gv) * v).sum().backward()
    np.testing.assert_allclose(out["d_x"], tx.grad.numpy(), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(out["d_embed_out"], tp["embed_out"].grad.numpy(), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(out["d_lnf_g"], tp["lnf_g"].grad.numpy(), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(out["d_lnf_b"], tp["lnf_b"].grad.numpy(), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(out["d_value_w"], tp["value_w"].grad.numpy(), rtol=1e-9, atol=1e-12)
    assert out["d_value_b"] == pytest.approx(float(tb.grad), rel=1e-12)


def test_invariants_of_the_softmax_and_layernorm_gradients():
    x, p, y, gl, gv = _case(5)
    out = head_backward(x, p["lnf_g"], p["lnf_b"], p["embed_out"], p["value_w"], y, gl, gv, 0.7)
    # rows of dL/dz sum to zero, so the gradient of the LM head sums to zero over the vocabulary
    np.testing.assert_allclose(out["d_embed_out"].sum(0), 0.0, atol=1e-12)
    # the LayerNorm input gradient has zero mean; with eps = 0 (the output is then invariant to a rescaling of
    # the row) it is also orthogonal to the centred row
    np.testing.assert_allclose(out["d_x"].mean(1), 0.0, atol=1e-12)
    o0 = head_backward(x, p["lnf_g"], p["lnf_b"], p["embed_out"], p["value_w"], y, gl, gv, 0.7, ln_eps=0.0)
    xc = x - x.mean(1, keepdims=True)
    np.testing.assert_allclose((o0["d_x"] * xc).sum(1), 0.0, atol=1e-10)
    # a row with neither a target nor a value gradient gets nothing, and adds nothing to the parameters
    y2, gv2 = y.copy(), gv.copy()
    gv2[2] = 0.0
    o2 = head_backward(x, p["lnf_g"], p["lnf_b"], p["embed_out"], p["value_w"], y2, gl, gv2, 0.7)
    assert np.all(o2["d_x"][2] == 0.0)
    x3 = x.copy()
    x3[2] = 100.0 * np.arange(x.shape[1])
    o3 = head_backward(x3, p["lnf_g"], p["lnf_b"], p["embed_out"], p["value_w"], y2, gl, gv2, 0.7)
    for k in ("d_embed_out", "d_lnf_g", "d_lnf_b", "d_value_w"):
        np.testing.assert_allclose(o3[k], o2[k], rtol=0, atol=1e-12)


def test_temperature_scales_the_logit_gradient():
    x, p, y, gl, gv = _case(6)
    gv[:] = 0.0
    a = head_backward(x, p["lnf_g"], p["lnf_b"], p["embed_out"], p["value_w"], y, gl, gv, 1.0)
    # doubling W and T together leaves the softmax unchanged: dL/dz halves, so dL/dW halves and dL/dh is unchanged
    b = head_backward(x, p["lnf_g"], p["lnf_b"], 2.0 * p["embed_out"], p["value_w"], y, gl, gv, 2.0)
    np.testing.assert_allclose(b["d_embed_out"], 0.5 * a["d_embed_out"], rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(b["d_x"], a["d_x"], rtol=1e-10, atol=1e-14)
