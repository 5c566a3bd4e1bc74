"""Pins of oracle/attention_backward_oracle.py against things other than itself.  The paper prints no numbers for
this step."""
import numpy as np
import pytest
import torch

from oracle.attention_backward_oracle import attention_backward, attention_forward


def _case(seed, lens=(5, 1, 7), H=2, hd=6):
    r = np.random.default_rng(seed)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    T = int(cu[-1])
    q, k, v, g = (r.normal(0, 1, (T, H * hd)) for _ in range(4))
    return q, k, v, g, cu, H, hd


def test_forward_is_the_attention_of_the_forward_oracle():
    from oracle.neox_oracle import attention
    q, k, v, g, cu, H, hd = _case(0)
    O = attention_forward(q, k, v, cu, H, hd)
    for b in range(len(cu) - 1):
        s, e = int(cu[b]), int(cu[b + 1])
        pos = np.arange(e - s)
        sl = lambda x: x[s:e].reshape(e - s, H, hd)
        ref = attention(sl(q), pos, sl(k), sl(v), pos, hd)
        np.testing.assert_allclose(O[s:e], np.asarray(ref).reshape(e - s, H * hd), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("seed", [1, 2])
def test_gradients_match_central_differences_of_the_forward(seed):
    q, k, v, g, cu, H, hd = _case(seed)
    dq, dk, dv = attention_backward(q, k, v, g, cu, H, hd)
    L = lambda: float((attention_forward(q, k, v, cu, H, hd) * g).sum())
    r = np.random.default_rng(30 + seed)
    eps = 1e-6
    for arr, grad in ((q, dq), (k, dk), (v, dv)):
        for _ in range(10):
            idx = (int(r.integers(0, arr.shape[0])), int(r.integers(0, arr.shape[1])))
            old = arr[idx]
            arr[idx] = old + eps
            up = L()
            arr[idx] = old - eps
            dn = L()
            arr[idx] = old
            assert (up - dn) / (2 * eps) == pytest.approx(grad[idx], rel=2e-6, abs=1e-8)


def test_gradients_match_torch_autograd():
    q, k, v, g, cu, H, hd = _case(3, lens=(9, 4), H=3, hd=8)
    dq, dk, dv = attention_backward(q, k, v, g, cu, H, hd)
    tq, tk, tv = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (q, k, v))
    outs = []
    for b in range(len(cu) - 1):
        s, e = int(cu[b]), int(cu[b + 1])
        sh = lambda t: t[s:e].reshape(e - s, H, hd).transpose(0, 1)          # [H, n, hd]
        outs.append(torch.nn.functional.scaled_dot_product_attention(sh(tq), sh(tk), sh(tv), is_causal=True)
                    .transpose(0, 1).reshape(e - s, H * hd))
    (torch.cat(outs) * torch.tensor(g)).sum().backward()
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=1e-9, atol=1e-12)


def test_structure_of_the_gradients():
    q, k, v, g, cu, H, hd = _case(4)
    dq, dk, dv = attention_backward(q, k, v, g, cu, H, hd)
    # the first query of a sequence sees one key: its output is v_0 whatever q is
    for b in range(len(cu) - 1):
        np.testing.assert_allclose(dq[int(cu[b])], 0.0, atol=1e-14)
    # the last key / value of a sequence is seen by the last query only
    s, e = int(cu[0]), int(cu[1])
    g2 = g.copy()
    g2[e - 1] = 0.0
    _, dk2, dv2 = attention_backward(q, k, v, g2, cu, H, hd)
    np.testing.assert_allclose(dk2[e - 1], 0.0, atol=1e-14)
    np.testing.assert_allclose(dv2[e - 1], 0.0, atol=1e-14)
    # sequences do not mix: an upstream gradient on sequence 0 only leaves the others without gradient
    g3 = np.zeros_like(g)
    g3[s:e] = g[s:e]
    dq3, dk3, dv3 = attention_backward(q, k, v, g3, cu, H, hd)
    assert np.all(dq3[e:] == 0) and np.all(dk3[e:] == 0) and np.all(dv3[e:] == 0)
    # sum over a sequence of dV equals the sum of the upstream gradients (softmax rows sum to one)
    np.testing.assert_allclose(dv[s:e].sum(0), g[s:e].sum(0), rtol=1e-12, atol=1e-12)
