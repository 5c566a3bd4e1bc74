"""Pin of oracle/policy_backward_oracle.py: central finite differences of the loss evaluated with the forward
oracle's score_sequences, which shares nothing with the stage oracles' own forward recomputation.  The paper prints
no numbers for this step."""
import numpy as np
import pytest

from oracle.neox_oracle import OracleModel, score_sequences
from oracle.policy_backward_oracle import policy_backward
from synth import ModelConfig, make_weights


def _setup():
    cfg = ModelConfig(n_layers=2, d_model=16, n_heads=2, head_dim=8, rotary_dims=4, d_ff=24, vocab=40, dtype="fp32",
                      pad_id=39, eos_id=1)
    w = {k: (np.asarray(v, np.float64) if k != "value_b" else v) for k, v in make_weights(cfg, 21, variant="test").items()}
    g = np.random.default_rng(0)
    B, L = 3, 9
    tokens = g.integers(2, 38, (B, L)).astype(np.int32)
    mask = np.ones((B, L), np.uint8)
    mask[0, :3] = 0                      # left padding
    mask[1, 7:] = 0                      # right padding
    mask[2, :1] = 0
    mask[2, 6:] = 0
    tokens[mask == 0] = cfg.pad_id
    tokens[0, 4] = tokens[0, 6]          # a repeated token: its embedding row collects two gradients
    GL = g.normal(0, 1, (B, L))
    GV = g.normal(0, 1, (B, L))
    return cfg, w, tokens, mask, GL, GV


def _loss(cfg, w, tokens, mask, GL, GV, T=0.7):
    lp, val = score_sequences(OracleModel(w, cfg, cache_f64=False), tokens, mask, T)
    return float((GL * lp).sum() + (GV * val * mask).sum())


def test_gradients_match_central_differences_of_the_scoring_forward():
    cfg, w, tokens, mask, GL, GV = _setup()
    grads = policy_backward(w, cfg, tokens, mask, GL, GV, 0.7)
    g = np.random.default_rng(1)
    eps = 1e-6
    names = ["embed_in", "embed_out", "lnf_g", "lnf_b", "value_w"] + [f"layers.{l}.{n}" for l in (0, 1) for n in (
        "ln1_g", "ln1_b", "ln2_g", "ln2_b", "w_qkv", "b_qkv", "w_o", "b_o", "w_fc1", "b_fc1", "w_fc2", "b_fc2")]
    for name in names:
        arr = w[name]
        for k in range(3):
            if name == "embed_in":
                idx = (int(tokens[0, 4 + k]), int(g.integers(0, arr.shape[1])))   # rows that are actually used
            else:
                idx = tuple(int(g.integers(0, n)) for n in arr.shape)
            old = arr[idx]
            arr[idx] = old + eps
            up = _loss(cfg, w, tokens, mask, GL, GV)
            arr[idx] = old - eps
            dn = _loss(cfg, w, tokens, mask, GL, GV)
            arr[idx] = old
            assert (up - dn) / (2 * eps) == pytest.approx(grads[name][idx], rel=2e-5, abs=2e-8), (name, idx)
    # value_b: dL/db_v = sum of the value gradients over real positions
    assert grads["value_b"] == pytest.approx(float((GV * mask).sum()), rel=1e-12)
    # unused embedding rows get no gradient
    unused = np.setdiff1d(np.arange(cfg.vocab), tokens[mask == 1])
    assert np.all(grads["embed_in"][unused] == 0.0)
