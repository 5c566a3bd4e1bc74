"""One whole PPO update through the C ABI against the chain of oracles: forward (score_sequences / rlhf_forward_keep),
loss head (rlhf_ppo_loss), backward pass (rlhf_policy_backward), optimizer (rlhf_adamw_step) on a small model in
fp32 check mode.  The gradients are held to 2e-4 of each tensor's largest magnitude, the updated weights to 5e-3 of
the learning rate (AdamW's first step is lr * g / (|g| + eps): with eps = 1e-3 here a gradient error of 1e-6 moves a
weight by at most 1e-3 lr), and the loss must go down."""
import numpy as np
import pytest

import paper_2403_17031_amd as P
from synth import ModelConfig, make_weights

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    P.load_library()  # fails loudly when the HIP library has not been built
    return P


def test_one_update_matches_the_oracles_and_lowers_the_loss(gpu):
    import torch
    from oracle import adamw_oracle, ppo_loss_oracle
    from oracle.neox_oracle import OracleModel, score_sequences
    from oracle.policy_backward_oracle import pack, policy_backward
    cfg = ModelConfig(n_layers=2, d_model=32, n_heads=2, head_dim=16, rotary_dims=4, d_ff=64, vocab=96, dtype="fp32",
                      pad_id=95, eos_id=1)
    w = make_weights(cfg, 91, variant="test")
    g = np.random.default_rng(5)
    B, Lq, N = 4, 10, 6
    L = Lq + N
    tokens = g.integers(2, 90, (B, L)).astype(np.int32)
    mask = np.ones((B, L), np.uint8)
    mask[0, :3] = 0                         # left-padded queries
    mask[2, :5] = 0
    kept = np.array([N, 4, N, 2], np.int32)  # response tokens kept per row; the rest is padding after EOS
    for b in range(B):
        mask[b, Lq + kept[b]:] = 0
    tokens[mask == 0] = cfg.pad_id
    T_, lr, eps = 0.7, 1e-3, 1e-3
    adv = g.normal(0, 1, (B, N)).astype(np.float32)
    ret = g.normal(0, 1, (B, N)).astype(np.float32)

    def gpu_losses(pol):
        lp, val = pol.score_sequences(tokens, mask, T_)
        return lp[:, Lq:].contiguous(), val[:, Lq - 1:Lq - 1 + N].contiguous()

    pol = gpu.Policy(cfg, w)
    new_lp, new_v = gpu_losses(pol)
    old_lp = (new_lp.cpu().numpy() + g.normal(0, 0.2, (B, N))).astype(np.float32)   # a policy that has moved
    old_v = (new_v.cpu().numpy() + g.normal(0, 0.2, (B, N))).astype(np.float32)
    stats, d_lp, d_v = gpu.ppo_loss(new_lp, old_lp, adv, new_v, old_v, ret, kept)
    loss0 = float(stats[0])
    # ---- the oracle chain on the same inputs
    w64 = {k: (np.asarray(v, np.float64) if k != "value_b" else v) for k, v in w.items()}
    o_lp, o_val = score_sequences(OracleModel(w64, cfg), tokens, mask, T_)
    o_stats, o_dlp, o_dv = ppo_loss_oracle.ppo_loss(o_lp[:, Lq:], old_lp, adv, o_val[:, Lq - 1:Lq - 1 + N], old_v, ret, kept)
    assert loss0 == pytest.approx(o_stats["loss"], rel=1e-4, abs=1e-6)
    GL, GV = np.zeros((B, L)), np.zeros((B, L))
    GL[:, Lq:] = o_dlp
    GV[:, Lq - 1:Lq - 1 + N] = o_dv
    o_grads = policy_backward(w64, cfg, tokens, mask, GL, GV, T_)
    # ---- the library: forward keeping the layer inputs, backward from its own loss gradients
    GLg, GVg = np.zeros((B, L), np.float32), np.zeros((B, L), np.float32)
    GLg[:, Lq:] = d_lp.cpu().numpy()
    GVg[:, Lq - 1:Lq - 1 + N] = d_v.cpu().numpy()
    _, cu, tgt, gl, gv = pack(tokens, mask, GLg, GVg)    # only index bookkeeping: which packed row gets which gradient
    x_keep, cu_d, ptok = pol.forward_keep(tokens, mask)
    scale = 256.0
    grads = pol.policy_backward(x_keep, cu_d, ptok, tgt.astype(np.int32), gl.astype(np.float32), gv.astype(np.float32),
                                T_, grad_scale=scale)
    new_w = {}
    for name, gt in grads.items():
        ref = np.asarray(o_grads[name], np.float64).reshape(tuple(gt.shape))
        a = gt.double().cpu().numpy() / scale
        assert np.abs(a - ref).max() <= 2e-4 * max(np.abs(ref).max(), 1e-12), name
        p0 = np.float64(w[name]) if name == "value_b" else np.asarray(w[name], np.float64).reshape(ref.shape)
        pt = torch.tensor(np.asarray(p0, np.float32).reshape(ref.shape), device="cuda")
        m1, m2 = torch.zeros_like(pt), torch.zeros_like(pt)
        gpu.adamw_step(pt, gt.contiguous(), m1, m2, 1, lr=lr, eps=eps, grad_scale=1.0 / scale)
        o_p, _, _ = adamw_oracle.adamw_step(np.asarray(p0, np.float32).reshape(ref.shape), ref, np.zeros_like(ref),
                                            np.zeros_like(ref), 1, lr=lr, eps=eps)
        assert np.abs(pt.double().cpu().numpy() - o_p).max() <= 5e-3 * lr, name
        new_w[name] = pt.cpu().numpy().reshape(np.shape(w[name])) if name != "value_b" else np.float32(pt.item())
    pol.close()
    # ---- the updated policy has a lower loss on the same batch
    pol2 = gpu.Policy(cfg, new_w)
    lp2, v2 = gpu_losses(pol2)
    stats2, _, _ = gpu.ppo_loss(lp2, old_lp, adv, v2, old_v, ret, kept)
    assert float(stats2[0]) < loss0
    pol2.close()
