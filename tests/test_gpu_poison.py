"""Every entry point on a workspace and output buffers filled with 0xFF bytes (NaN as fp32 and fp16, -1 as an
integer) before each call: a kernel that reads a region its own call has not written -- which on a reused workspace
would see plausible values left by the previous call -- turns its results into NaN or wrong indices here, and the
ordinary parity checks against the oracle catch it.  Also: what happens at fp16's range limit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from synth import ModelConfig, WORKLOADS, make_weights
from test_gpu_parity import _check_rollout_and_scores, _queries


@pytest.fixture()
def poisoned(monkeypatch):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2403_17031_amd as P
    P.load_library()
    monkeypatch.setattr(P.binding, "POISON", True)
    return P


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_rollout_scoring_and_logits_on_poisoned_buffers_small(poisoned, tiny_cfg, dtype):
    """Ragged tiny model (generic kernels), two calls in a row on the same handle (the second on a workspace the
    first has used)."""
    cfg = tiny_cfg.with_(dtype=dtype)
    w = make_weights(cfg, 7, variant="test")
    for seed in (3, 4):
        queries, mask = _queries(cfg, B=5, Lq=40, lo=1, hi=40, seed=seed)
        queries[2], mask[2] = cfg.pad_id, 0          # an all-pad row
        _check_rollout_and_scores(poisoned, cfg, w, queries, mask, seed=11, T=0.7, N=9)


@pytest.mark.parametrize("shape", ["2.8b", "1b"])
def test_rollout_and_scoring_on_poisoned_buffers_large_row_kernels(poisoned, shape):
    """The benchmark layer shapes at 2 layers with more than 2048 packed rows: direct-to-LDS products with their
    QKV / log-sum-exp epilogues, the matrix-core attention, the few-rows decode products and their folded
    reductions."""
    idx = {"1b": 3, "2.8b": 4}[shape]
    cfg = WORKLOADS[idx].model.with_(n_layers=2)
    w = make_weights(cfg, 200 + idx)
    queries, mask = _queries(cfg, B=16, Lq=150, lo=100, hi=150, seed=10 + idx)
    _check_rollout_and_scores(poisoned, cfg, w, queries, mask, seed=10 + idx, T=0.7, N=4, rows=[0, 7, 15])


def test_backward_and_update_on_poisoned_buffers(poisoned):
    """rlhf_forward_keep + rlhf_policy_backward (which runs the head, MLP-branch, attention-branch and attention
    backward entry points) and rlhf_ppo_update, bf16 mode, against their oracles."""
    from oracle.policy_backward_oracle import pack, policy_backward
    from oracle.ppo_update_oracle import ppo_update
    from synth import round_to_bf16
    P = poisoned
    cfg = ModelConfig(n_layers=2, d_model=128, n_heads=2, head_dim=64, rotary_dims=16, d_ff=256, vocab=520, dtype="bf16",
                      pad_id=519, eos_id=1)
    w = make_weights(cfg, 81, variant="test")
    g = np.random.default_rng(2)
    B, Lq, N = 4, 30, 10
    L = Lq + N
    tokens = g.integers(2, 500, (B, L)).astype(np.int32)
    mask = np.ones((B, L), np.uint8)
    mask[1, :11] = 0
    kept = np.array([N, 4, 7, N], np.int32)
    for b in range(B):
        mask[b, Lq + kept[b]:] = 0
    tokens[mask == 0] = cfg.pad_id
    T = int(mask.sum())
    GL = np.zeros((B, L), np.float32)
    GV = np.zeros((B, L), np.float32)
    GL[:, Lq:] = g.normal(0, 1, (B, N)) / T
    GV[:, Lq - 1:Lq - 1 + N] = g.normal(0, 0.3, (B, N)) / T
    GL[mask == 0] = 0
    _, cu, tgt, gl, gv = pack(tokens, mask, GL, GV)
    pol = P.Policy(cfg, w)
    scale = 64.0 * T
    for _ in range(2):   # the second pass runs on buffers the first has used (and that were poisoned again)
        x_keep, cu_d, ptok = pol.forward_keep(tokens, mask)
        got = pol.policy_backward(x_keep, cu_d, ptok, tgt.astype(np.int32), gl.astype(np.float32), gv.astype(np.float32),
                                  0.7, grad_scale=scale)
    w64 = {k: (np.asarray(v, np.float64) if k != "value_b" else v) for k, v in w.items()}
    ref = policy_backward(w64, cfg, tokens, mask, GL, GV, 0.7)
    for name, r in ref.items():
        a = got[name].cpu().numpy().astype(np.float64) / scale
        b = np.asarray(r, np.float64).reshape(a.shape)
        assert np.isfinite(a).all(), name
        assert np.abs(a - b).max() <= 2e-2 * np.abs(b).max(), name
        if b.size > 1:
            assert np.linalg.norm(a - b) <= 5e-3 * np.linalg.norm(b), name
    adv = g.normal(0, 1, (B, N)).astype(np.float32)
    ret = g.normal(0, 1, (B, N)).astype(np.float32)
    lp0, v0 = (x.cpu().numpy() for x in pol.score_sequences(tokens, mask, 0.7))
    old_lp, old_v = lp0[:, Lq:].copy(), v0[:, Lq - 1:Lq - 1 + N].copy()
    hyp = dict(lr=1e-3, eps=1e-3)
    stats = pol.ppo_update(tokens, mask, Lq, old_lp, adv, old_v, ret, kept, 0.7, epochs=2, n_minibatches=2, **hyp).cpu().numpy()
    o_w, _, o_stats = ppo_update(w, cfg, tokens, mask, Lq, old_lp, adv, old_v, ret, kept, 0.7, epochs=2, n_minibatches=2,
                                 storage_round=round_to_bf16, **hyp)
    assert np.isfinite(stats).all()
    for i, s in enumerate(o_stats):
        assert stats[i, 0] == pytest.approx(s["loss"], abs=2e-2), (i, stats[i], s)
    st = pol.train_state()
    for name, want in o_w.items():
        got_w = st["master"][name].double().cpu().numpy()
        want = np.asarray(want, np.float64).reshape(got_w.shape)
        start = np.asarray(w[name], np.float64).reshape(got_w.shape)
        assert np.isfinite(got_w).all(), name
        assert np.linalg.norm(got_w - want) <= 5e-2 * np.linalg.norm(want - start) + 1e-7, name
    pol.close()


def test_fp16_operands_saturate_instead_of_overflowing(poisoned):
    """The documented failure mode of the fp16 operand type: an activation beyond fp16's range (|x| > 65504) is
    clamped to the largest finite fp16 value, silently, and never becomes infinite -- here the FC1 bias of one layer
    pushes two hidden units to 99840 and 66560.  The bf16-mode outputs stay finite, but both units arrive at FC2 as
    65504, so the residual stream points along the sum of their FC2 columns instead of 1.5 : 1 (one huge unit alone
    would not show: the final LayerNorm removes a common scale), and the outputs differ from the oracle's on the same
    weights by far more than the parity bar; the fp32 check mode carries the values unclamped and matches the oracle."""
    from oracle import neox_oracle as O
    P = poisoned
    base = ModelConfig(n_layers=1, d_model=64, n_heads=2, head_dim=32, rotary_dims=8, d_ff=128, vocab=300, dtype="bf16",
                       pad_id=299, eos_id=1)
    g = np.random.default_rng(0)
    tokens = g.integers(2, 290, (2, 12)).astype(np.int32)
    mask = np.ones((2, 12), np.uint8)
    out = {}
    for dtype in ("bf16", "fp32"):
        cfg = base.with_(dtype=dtype)
        w = make_weights(cfg, 5, variant="test")
        w["layers.0.b_fc1"] = w["layers.0.b_fc1"].copy()
        w["layers.0.b_fc1"][7] = np.float32(99840.0)      # bf16 values beyond fp16's largest (65504)
        w["layers.0.b_fc1"][9] = np.float32(66560.0)
        pol = P.Policy(cfg, w)
        lp, val = (x.cpu().numpy() for x in pol.score_sequences(tokens, mask, 1.0))
        pol.close()
        olp, oval = O.score_sequences(O.OracleModel(w, cfg), tokens, mask, 1.0)
        assert np.isfinite(lp).all() and np.isfinite(val).all(), dtype
        out[dtype] = (np.abs(lp - olp).max(), np.abs(val - oval).max())
    assert out["fp32"][0] <= 1e-3 and out["fp32"][1] <= 1e-3, out     # check mode: no clamp, matches the oracle
    assert out["bf16"][0] > 2e-2 or out["bf16"][1] > 2e-2, out         # fp16 operands: finite, but clamped
