"""GPU parity of the policy's whole backward pass (rlhf_forward_keep + rlhf_policy_backward) against
oracle/policy_backward_oracle.py, through the C ABI: every weight's gradient.

Bars: fp32 check mode 2e-4 of each tensor's largest magnitude (the chain is a few hundred fp32 operations deep);
bf16 mode the bars of a single stage -- a relative Frobenius error of 5e-3 per tensor and a largest element error of
2e-2 of the tensor's largest magnitude: the fp16 roundings of the stages are independent, so the error of the chain
grows like the square root of its depth (measured: 6e-4 relative on the worst tensor of these models)."""
import numpy as np
import pytest

import paper_2403_17031_amd as P
from synth import ModelConfig, make_weights

from bars import assert_signal_entries_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    P.load_library()  # fails loudly when the HIP library has not been built
    return P


def _batch(cfg, B, L, seed):
    g = np.random.default_rng(seed)
    tokens = g.integers(2, cfg.vocab - 2, (B, L)).astype(np.int32)
    mask = np.ones((B, L), np.uint8)
    for b in range(B):
        lp, rp = int(g.integers(0, L // 3)), int(g.integers(0, L // 3))
        mask[b, :lp] = 0
        if rp:
            mask[b, L - rp:] = 0
    tokens[mask == 0] = cfg.pad_id
    T = int(mask.sum())
    GL = (g.normal(0, 1, (B, L)) / T).astype(np.float32)
    GV = (g.normal(0, 0.3, (B, L)) / T).astype(np.float32)
    GL[:, : L // 2] = 0.0              # the loss only looks at the later ("response") positions
    GV[:, : L // 2] = 0.0
    return tokens, mask, GL, GV


def _check(P, cfg, B, L, seed, scale):
    from oracle.policy_backward_oracle import pack, policy_backward
    w = make_weights(cfg, 80 + seed, variant="test")
    tokens, mask, GL, GV = _batch(cfg, B, L, seed)
    tok, cu, tgt, gl, gv = pack(tokens, mask, GL, GV)
    pol = P.Policy(cfg, w)
    x_keep, cu_d, ptok = pol.forward_keep(tokens, mask)
    assert (cu_d.cpu().numpy() == cu).all()
    assert (ptok.cpu().numpy()[: len(tok)] == tok).all()
    got = pol.policy_backward(x_keep, cu_d, ptok, tgt.astype(np.int32), gl.astype(np.float32), gv.astype(np.float32),
                              0.7, grad_scale=scale)
    w64 = {k: (np.asarray(v, np.float64) if k != "value_b" else v) for k, v in w.items()}
    ref = policy_backward(w64, cfg, tokens, mask, GL, GV, 0.7)
    fp32 = cfg.dtype == "fp32"
    worst = {}
    for name, r in ref.items():
        a = got[name].cpu().numpy().astype(np.float64) / scale
        b = np.asarray(r, np.float64).reshape(a.shape)
        assert np.isfinite(a).all(), name
        top, err = np.abs(b).max(), np.abs(a - b).max()
        assert err <= (2e-4 if fp32 else 2e-2) * top, (name, err, top)
        if not fp32 and b.size > 1:
            rel = np.linalg.norm(a - b) / np.linalg.norm(b)
            assert rel <= 5e-3, (name, rel)
            worst[name] = rel
        assert_signal_entries_close(a, b, fp32, name)
    pol.close()
    return worst


def test_fp32_check_mode(gpu):
    cfg = ModelConfig(n_layers=2, d_model=32, n_heads=2, head_dim=16, rotary_dims=4, d_ff=64, vocab=96, dtype="fp32",
                      pad_id=95, eos_id=1)
    _check(gpu, cfg, B=3, L=20, seed=1, scale=1.0)


@pytest.mark.parametrize("layers,H,hd,r,F,B,L", [(2, 4, 16, 4, 128, 4, 24), (3, 2, 64, 16, 256, 6, 100),
                                                   (2, 8, 80, 20, 1280, 5, 200)])
def test_bf16_mode(gpu, layers, H, hd, r, F, B, L):
    d = H * hd
    cfg = ModelConfig(n_layers=layers, d_model=d, n_heads=H, head_dim=hd, rotary_dims=r, d_ff=F, vocab=520, dtype="bf16",
                      pad_id=519, eos_id=1)
    worst = _check(gpu, cfg, B=B, L=L, seed=layers + hd, scale=float(B * L) * 64.0)
    print("largest relative Frobenius errors:", sorted(worst.items(), key=lambda kv: -kv[1])[:4])
