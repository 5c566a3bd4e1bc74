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


def _loop_case(dtype):
    cfg = ModelConfig(n_layers=2, d_model=64, n_heads=2, head_dim=32, rotary_dims=8, d_ff=128, vocab=200, dtype=dtype,
                      pad_id=199, eos_id=1)
    w = make_weights(cfg, 92, variant="test")
    g = np.random.default_rng(6)
    B, Lq, N = 6, 12, 7
    L = Lq + N
    tokens = g.integers(2, 190, (B, L)).astype(np.int32)
    mask = np.ones((B, L), np.uint8)
    mask[0, :4] = 0
    mask[3, :9] = 0
    mask[5, :1] = 0
    kept = np.array([N, 3, N, 1, 5, N], np.int32)
    for b in range(B):
        mask[b, Lq + kept[b]:] = 0
    tokens[mask == 0] = cfg.pad_id
    adv = g.normal(0, 1, (B, N)).astype(np.float32)
    ret = g.normal(0, 1, (B, N)).astype(np.float32)
    return cfg, w, g, tokens, mask, kept, adv, ret, Lq, N


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_update_loop_matches_the_oracle_loop(gpu, dtype):
    """rlhf_ppo_update (K = 2 iterations over 2 mini-batches, optimizer steps 1..4) against
    oracle/ppo_update_oracle.py: the loss statistics of every step, every updated weight, and afterwards the same
    handle scores with the updated weights.  fp32 check mode: weights to 2 % of one step's size (lr).  bf16 mode:
    the oracle reads bf16-rounded copies of its exact masters in every pass, as the library does; what remains is
    the fp16 rounding of operands inside the passes: each tensor's movement to 5 % (Frobenius), losses to 2e-2."""
    import torch
    from oracle.neox_oracle import OracleModel, score_sequences
    from oracle.ppo_update_oracle import ppo_update
    from synth import round_to_bf16
    cfg, w, g, tokens, mask, kept, adv, ret, Lq, N = _loop_case(dtype)
    T_, K, NMB = 0.7, 2, 2
    hyp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-3, weight_decay=0.01)
    pol = gpu.Policy(cfg, w)
    lp0, v0 = (x.cpu().numpy() for x in pol.score_sequences(tokens, mask, T_))
    old_lp = (lp0[:, Lq:] + g.normal(0, 0.15, lp0[:, Lq:].shape)).astype(np.float32)
    old_v = (v0[:, Lq - 1:Lq - 1 + N] + g.normal(0, 0.15, (tokens.shape[0], N))).astype(np.float32)
    stats = pol.ppo_update(tokens, mask, Lq, old_lp, adv, old_v, ret, kept, T_, epochs=K, n_minibatches=NMB, **hyp)
    stats = stats.cpu().numpy()
    st = pol.train_state()
    assert st["steps"] == K * NMB
    fp32 = dtype == "fp32"
    o_w, _, o_stats = ppo_update(w, cfg, tokens, mask, Lq, old_lp, adv, old_v, ret, kept, T_, epochs=K, n_minibatches=NMB,
                                 storage_round=None if fp32 else round_to_bf16, **hyp)
    for i, s in enumerate(o_stats):
        assert stats[i, 0] == pytest.approx(s["loss"], rel=1e-4, abs=1e-5 if fp32 else 2e-2), (i, stats[i], s)
        assert stats[i, 7] == s["n_tokens"]
    for name, want in o_w.items():
        got = (st["master"][name] if (not fp32 or name == "value_b") else pol._dev[name]).double().cpu().numpy()
        want = np.asarray(want, np.float64).reshape(got.shape)
        start = np.asarray(w[name], np.float64).reshape(got.shape)
        if fp32:
            assert np.abs(got - want).max() <= 2e-2 * hyp["lr"], (name, np.abs(got - want).max())
        else:
            moved = np.linalg.norm(want - start)
            assert np.linalg.norm(got - want) <= 5e-2 * moved + 1e-7, (name, np.linalg.norm(got - want), moved)
            # the storage copy the forward passes read is the rounded master
            if name != "value_b":
                assert bool((pol._dev[name].float() == st["master"][name].bfloat16().float()).all()), name
    # the handle now computes with the updated weights (value bias included: it lives on the device)
    new_w = {k: (np.asarray(v, np.float64) if fp32 else round_to_bf16(np.asarray(v, np.float32))) for k, v in o_w.items()
             if k != "value_b"}
    new_w["value_b"] = np.float32(o_w["value_b"])
    olp, oval = score_sequences(OracleModel(new_w, cfg), tokens, mask, T_)
    lp1, v1 = (x.cpu().numpy() for x in pol.score_sequences(tokens, mask, T_))
    tol = 1e-3 if fp32 else 2e-2
    np.testing.assert_allclose(lp1, olp, atol=tol, rtol=0)
    np.testing.assert_allclose(v1, oval, atol=tol * max(1.0, float(np.abs(oval).max())), rtol=0)
    assert abs(float(st["master"]["value_b"][0]) - float(w["value_b"])) > 1e-4   # the bias moved, and v1 saw it
    pol.close()


@pytest.mark.parametrize("keep", [True, False])
def test_update_loop_with_the_heads_on_the_response_rows_only(gpu, keep):
    """A batch with enough response rows (40 sequences x 14 columns) for the loop to run the LM head, and the output
    heads' backward pass, on the rows from the last query column on only (the log-probs and values of the other rows
    are never read), at a head size for which the loop keeps every layer's rotated q rows and K / V cache from the
    forward pass instead of recomputing the QKV product in the backward pass: one iteration over the whole batch
    against the oracle loop, every tensor; with workspace for the kept FC1 pre-activations and with the minimum
    (FC1 recomputed in the backward pass)."""
    from oracle.ppo_update_oracle import ppo_update
    from synth import round_to_bf16
    cfg = ModelConfig(n_layers=2, d_model=128, n_heads=2, head_dim=64, rotary_dims=16, d_ff=256, vocab=200, dtype="bf16",
                      pad_id=199, eos_id=1)   # head size 64: the loop also keeps q and the K / V cache of every layer
    w = make_weights(cfg, 93, variant="test")
    g = np.random.default_rng(16)
    B, Lq, N = 40, 24, 13
    L = Lq + N
    tokens = g.integers(2, 190, (B, L)).astype(np.int32)
    qlen = g.integers(5, Lq + 1, B)
    kept = g.integers(1, N + 1, B).astype(np.int32)
    kept[:4] = N
    col = np.arange(L)[None, :]
    mask = ((col >= (Lq - qlen)[:, None]) & (col < (Lq + kept)[:, None])).astype(np.uint8)
    tokens[mask == 0] = cfg.pad_id
    adv = g.normal(0, 1, (B, N)).astype(np.float32)
    ret = g.normal(0, 1, (B, N)).astype(np.float32)
    T_ = 0.7
    hyp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-3, weight_decay=0.01)
    pol = gpu.Policy(cfg, w)
    lp0, v0 = (x.cpu().numpy() for x in pol.score_sequences(tokens, mask, T_))
    old_lp = (lp0[:, Lq:] + g.normal(0, 0.15, (B, N))).astype(np.float32)
    old_v = (v0[:, Lq - 1:Lq - 1 + N] + g.normal(0, 0.15, (B, N))).astype(np.float32)
    stats = pol.ppo_update(tokens, mask, Lq, old_lp, adv, old_v, ret, kept, T_, epochs=1, n_minibatches=1,
                           keep_preactivations=keep, **hyp)
    stats = stats.cpu().numpy()
    st = pol.train_state()
    o_w, _, o_stats = ppo_update(w, cfg, tokens, mask, Lq, old_lp, adv, old_v, ret, kept, T_, epochs=1, n_minibatches=1,
                                 storage_round=round_to_bf16, **hyp)
    assert stats[0, 0] == pytest.approx(o_stats[0]["loss"], abs=2e-2)
    assert stats[0, 7] == o_stats[0]["n_tokens"] == int(kept.sum())
    for name, want in o_w.items():
        got = st["master"][name].double().cpu().numpy()
        want = np.asarray(want, np.float64).reshape(got.shape)
        start = np.asarray(w[name], np.float64).reshape(got.shape)
        moved = np.linalg.norm(want - start)
        assert np.linalg.norm(got - want) <= 5e-2 * moved + 1e-7, (name, np.linalg.norm(got - want), moved)
    pol.close()


def test_update_loop_rejects_bad_arguments(gpu):
    cfg, w, g, tokens, mask, kept, adv, ret, Lq, N = _loop_case("fp32")
    pol = gpu.Policy(cfg, w)
    z = np.zeros((tokens.shape[0], N), np.float32)
    with pytest.raises(gpu.RlhfError):
        pol.ppo_update(tokens, mask, Lq, z, adv, z, ret, kept, 0.7, n_minibatches=4)      # 4 does not divide 6
    with pytest.raises(gpu.RlhfError):
        pol.ppo_update(tokens, mask, Lq, z, adv, z, ret, kept, 0.0)                       # temperature
    with pytest.raises(gpu.RlhfError):
        pol.ppo_update(tokens, mask, Lq, z, adv, z, ret, kept, 0.7, epochs=0)
    pol.close()
