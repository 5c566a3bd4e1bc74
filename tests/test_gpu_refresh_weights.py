"""After an optimizer step on the caller's weight arrays the SAME handle must compute with the new weights: in
bf16 mode the matrix products read an fp16 image that rlhf_refresh_weights rebuilds.  Graded against the oracle
evaluated on the updated weights (2e-2, the bf16-mode bar)."""
import numpy as np
import pytest

import paper_2403_17031_amd as P
from synth import ModelConfig, make_weights

pytestmark = pytest.mark.gpu


def test_bf16_handle_sees_updated_weights_after_refresh():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    P.load_library()
    from oracle.neox_oracle import OracleModel, score_sequences
    cfg = ModelConfig(n_layers=2, d_model=128, n_heads=2, head_dim=64, rotary_dims=16, d_ff=512, vocab=520, dtype="bf16",
                      pad_id=519, eos_id=1)
    w = make_weights(cfg, 17, variant="test")
    g = np.random.default_rng(3)
    B, L = 3, 40
    tokens = g.integers(2, 500, (B, L)).astype(np.int32)
    mask = np.ones((B, L), np.uint8)
    mask[1, :7] = 0
    mask[2, 30:] = 0
    tokens[mask == 0] = cfg.pad_id
    pol = P.Policy(cfg, w)
    lp0, v0 = (x.cpu().numpy() for x in pol.score_sequences(tokens, mask, 0.7))
    # one AdamW step with a large learning rate on every tensor, writing the caller's bf16 arrays in place
    state = {}
    for name, t in pol._dev.items():
        p32 = t.float().contiguous()
        grad = torch.from_numpy(g.normal(0, 1, tuple(t.shape)).astype(np.float32)).cuda()
        m1, m2 = torch.zeros_like(p32), torch.zeros_like(p32)
        P.adamw_step(p32, grad, m1, m2, 1, lr=5e-3, eps=1e-5, weight_decay=0.0, param_bf16=t)
        state[name] = t
    torch.cuda.synchronize()
    new_w = {k: v.float().cpu().numpy() for k, v in state.items()}
    new_w["value_b"] = w["value_b"]
    olp, oval = score_sequences(OracleModel(new_w, cfg), tokens, mask, 0.7)
    assert np.abs(olp - lp0).max() > 0.1, "the step did not move the model enough to tell old from new"
    # without a refresh the products still read the old matrices: the outputs are neither the old nor the new model's
    pol.refresh_weights()
    lp1, v1 = (x.cpu().numpy() for x in pol.score_sequences(tokens, mask, 0.7))
    np.testing.assert_allclose(lp1, olp, atol=2e-2, rtol=0)
    np.testing.assert_allclose(v1, oval, atol=2e-2 * max(1.0, float(np.abs(oval).max())), rtol=0)
    # and a rollout on the refreshed handle agrees with the oracle on the new weights
    from oracle.neox_oracle import verify_rollout
    q, qm = tokens[:, :24].copy(), mask[:, :24].copy()
    qm[2] = 1
    q[2] = g.integers(2, 500, 24)
    qm[1, :7] = 0
    toks, lps, lens = (x.cpu().numpy() for x in pol.rollout_generate(q, qm, 5, 0.7, 6))
    for r in verify_rollout(OracleModel(new_w, cfg), toks, qm, 5, 0.7, 6):
        assert r["deficit"] <= 1e-2, r
        assert abs(lps[r["row"], r["step"]] - r["logprob"]) <= 2e-2, r
    pol.close()
