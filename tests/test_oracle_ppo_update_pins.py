"""Pin of oracle/ppo_update_oracle.py (K update iterations over mini-batches: forward, clipped objective, backward,
AdamW) against the same loop built from parts that share nothing with the oracles: the `transformers` GPT-NeoX class
in float64 as the forward pass (the paper's own: General Details, Tech stack), torch autograd as the differentiation,
torch.optim.AdamW as the optimizer.  The paper prints no numbers for this step."""
import numpy as np
import pytest

from oracle.ppo_update_oracle import ppo_update
from synth import ModelConfig, make_weights

torch = pytest.importorskip("torch")
tr = pytest.importorskip("transformers")


def _hf_model(cfg, w):
    hc = tr.GPTNeoXConfig(vocab_size=cfg.vocab, hidden_size=cfg.d_model, num_hidden_layers=cfg.n_layers,
                          num_attention_heads=cfg.n_heads, intermediate_size=cfg.d_ff, hidden_act="gelu",
                          rotary_pct=cfg.rotary_dims / cfg.head_dim, rotary_emb_base=cfg.rope_base,
                          max_position_embeddings=64, layer_norm_eps=cfg.ln_eps, use_parallel_residual=True,
                          tie_word_embeddings=False, attention_dropout=0.0, hidden_dropout=0.0, attention_bias=True)
    hf = tr.GPTNeoXForCausalLM(hc).double().train()   # dropout is 0: train mode only enables gradients
    H, hd, d = cfg.n_heads, cfg.head_dim, cfg.d_model
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    sd = {"gpt_neox.embed_in.weight": t(w["embed_in"]), "lm_head.weight": t(w["embed_out"]),
          "gpt_neox.final_layer_norm.weight": t(w["lnf_g"]), "gpt_neox.final_layer_norm.bias": t(w["lnf_b"])}
    names = {"attention.dense.weight": "w_o", "attention.dense.bias": "b_o", "input_layernorm.weight": "ln1_g",
             "input_layernorm.bias": "ln1_b", "post_attention_layernorm.weight": "ln2_g",
             "post_attention_layernorm.bias": "ln2_b", "mlp.dense_h_to_4h.weight": "w_fc1",
             "mlp.dense_h_to_4h.bias": "b_fc1", "mlp.dense_4h_to_h.weight": "w_fc2", "mlp.dense_4h_to_h.bias": "b_fc2"}
    for l in range(cfg.n_layers):
        p = f"gpt_neox.layers.{l}."
        g = lambda n: w[f"layers.{l}.{n}"]
        # that class orders the fused projection's rows [head][q|k|v]; this repository [q all heads | k | v]
        sd[p + "attention.query_key_value.weight"] = t(g("w_qkv").reshape(3, H, hd, d).transpose(1, 0, 2, 3).reshape(3 * d, d))
        sd[p + "attention.query_key_value.bias"] = t(g("b_qkv").reshape(3, H, hd).transpose(1, 0, 2).reshape(3 * d))
        for hn, mine in names.items():
            sd[p + hn] = t(g(mine))
    missing, unexpected = hf.load_state_dict(sd, strict=False)
    assert not [k for k in missing if "inv_freq" not in k and "rotary" not in k] and not unexpected
    return hf


def _back_to_names(cfg, hf, vw, vb):
    H, hd, d = cfg.n_heads, cfg.head_dim, cfg.d_model
    sd = {k: v.detach().numpy() for k, v in hf.state_dict().items()}
    out = {"embed_in": sd["gpt_neox.embed_in.weight"], "embed_out": sd["lm_head.weight"],
           "lnf_g": sd["gpt_neox.final_layer_norm.weight"], "lnf_b": sd["gpt_neox.final_layer_norm.bias"],
           "value_w": vw.detach().numpy(), "value_b": float(vb.detach())}
    names = {"attention.dense.weight": "w_o", "attention.dense.bias": "b_o", "input_layernorm.weight": "ln1_g",
             "input_layernorm.bias": "ln1_b", "post_attention_layernorm.weight": "ln2_g",
             "post_attention_layernorm.bias": "ln2_b", "mlp.dense_h_to_4h.weight": "w_fc1",
             "mlp.dense_h_to_4h.bias": "b_fc1", "mlp.dense_4h_to_h.weight": "w_fc2", "mlp.dense_4h_to_h.bias": "b_fc2"}
    for l in range(cfg.n_layers):
        p = f"gpt_neox.layers.{l}."
        out[f"layers.{l}.w_qkv"] = sd[p + "attention.query_key_value.weight"].reshape(H, 3, hd, d).transpose(1, 0, 2, 3).reshape(3 * d, d)
        out[f"layers.{l}.b_qkv"] = sd[p + "attention.query_key_value.bias"].reshape(H, 3, hd).transpose(1, 0, 2).reshape(3 * d)
        for hn, mine in names.items():
            out[f"layers.{l}.{mine}"] = sd[p + hn]
    return out


def test_k_iterations_over_minibatches_match_library_forward_autograd_and_adamw():
    cfg = ModelConfig(n_layers=2, d_model=16, n_heads=2, head_dim=8, rotary_dims=4, d_ff=24, vocab=40, dtype="fp32",
                      pad_id=39, eos_id=1)
    w = make_weights(cfg, 33, variant="test")
    g = np.random.default_rng(4)
    B, Lq, N = 4, 6, 5
    L = Lq + N
    tokens = g.integers(2, 38, (B, L)).astype(np.int32)
    mask = np.ones((B, L), np.uint8)
    mask[0, :2] = 0
    mask[3, :4] = 0
    kept = np.array([5, 3, 1, 4], np.int32)
    for b in range(B):
        mask[b, Lq + kept[b]:] = 0
    tokens[mask == 0] = cfg.pad_id
    T_, K, NMB = 0.7, 2, 2
    hyp = dict(lr=2e-3, beta1=0.9, beta2=0.999, eps=1e-3, weight_decay=0.01)
    old_lp = -np.abs(g.normal(3, 0.5, (B, N)))
    old_v = g.normal(0, 1, (B, N))
    adv = g.normal(0, 1, (B, N))
    ret = g.normal(0, 1, (B, N))
    # first find the policy's own outputs so that the "old" ones sit close enough for both clip branches to occur
    from oracle.neox_oracle import OracleModel, score_sequences
    lp0, v0 = score_sequences(OracleModel(w, cfg), tokens, mask, T_)
    old_lp = lp0[:, Lq:] + g.normal(0, 0.15, (B, N))
    old_v = v0[:, Lq - 1:Lq - 1 + N] + g.normal(0, 0.15, (B, N))
    new_w, state, stats = ppo_update(w, cfg, tokens, mask, Lq, old_lp, adv, old_v, ret, kept, T_, epochs=K,
                                     n_minibatches=NMB, first_step=3, **hyp)
    assert len(stats) == K * NMB and any(s["pg_clipfrac"] > 0 or s["vf_clipfrac"] > 0 for s in stats)

    # ---- the same loop with library parts
    hf = _hf_model(cfg, w)
    vw = torch.tensor(np.asarray(w["value_w"], np.float64), requires_grad=True)
    vb = torch.tensor(float(w["value_b"]), dtype=torch.float64, requires_grad=True)
    params = list(hf.parameters()) + [vw, vb]
    opt = torch.optim.AdamW(params, lr=hyp["lr"], betas=(hyp["beta1"], hyp["beta2"]), eps=hyp["eps"],
                            weight_decay=hyp["weight_decay"])
    # optimizer steps 1 and 2 happened "before": start the step counter at 3 with zero moments, as the oracle was told
    for p in params:
        opt.state[p] = {"step": torch.tensor(2.0), "exp_avg": torch.zeros_like(p), "exp_avg_sq": torch.zeros_like(p)}
    mb = B // NMB
    tt = lambda a: torch.tensor(np.asarray(a, np.float64))
    losses = []
    for _ in range(K):
        for j in range(NMB):
            r = slice(j * mb, (j + 1) * mb)
            am = torch.tensor(mask[r].astype(np.int64))
            pos = torch.clamp(am.cumsum(-1) - 1, min=0)
            o = hf(input_ids=torch.tensor(tokens[r].astype(np.int64)), attention_mask=am, position_ids=pos,
                   output_hidden_states=True)
            lsm = torch.log_softmax(o.logits / T_, dim=-1)
            nxt = torch.tensor(tokens[r, 1:].astype(np.int64))
            lp_full = torch.gather(lsm[:, :-1], 2, nxt[:, :, None])[:, :, 0]          # log-prob of token t+1 at position t
            new_lp = lp_full[:, Lq - 1:]
            new_v = (o.hidden_states[-1] @ vw + vb)[:, Lq - 1:Lq - 1 + N]
            keep = torch.tensor(np.arange(N)[None, :] < kept[r][:, None])
            n = keep.sum()
            ratio = torch.exp(new_lp - tt(old_lp[r]))
            pg = torch.maximum(-tt(adv[r]) * ratio, -tt(adv[r]) * torch.clamp(ratio, 0.8, 1.2))
            vc = torch.maximum(torch.minimum(new_v, tt(old_v[r]) + 0.2), tt(old_v[r]) - 0.2)
            vf = 0.5 * torch.maximum((new_v - tt(ret[r])) ** 2, (vc - tt(ret[r])) ** 2)
            loss = (pg * keep).sum() / n + 0.1 * (vf * keep).sum() / n
            losses.append(float(loss.detach()))
            opt.zero_grad()
            loss.backward()
            opt.step()
    for s, l in zip(stats, losses):
        assert s["loss"] == pytest.approx(l, rel=1e-6, abs=1e-8)
    ref = _back_to_names(cfg, hf, vw, vb)
    for name, want in ref.items():
        got = np.asarray(new_w[name], np.float64)
        moved = np.abs(np.asarray(w[name], np.float64) - want).max()
        assert np.abs(got - want).max() <= 1e-5 * max(moved, 1e-4) + 1e-9, (name, np.abs(got - want).max(), moved)
    assert any(np.abs(np.asarray(w[n], np.float64) - ref[n]).max() > 1e-3 for n in ref if n != "value_b")
