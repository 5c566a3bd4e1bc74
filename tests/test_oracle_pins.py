"""Pins of the CPU oracle against things other than itself: a library implementation of the
same decoder, brute force, closed forms, invariants and a frequency test of the sampler."""
import math

import numpy as np
import pytest

from oracle import neox_oracle as O
from synth import ModelConfig, Workload, make_weights, make_queries, boost_eos


def _wl(cfg, B=3, Lq=12, N=6, lo=5, hi=12):
    return Workload("t", cfg, B, Lq, N, lo, hi, 0.7, 11, 22, 33)


def _queries(cfg, B=3, Lq=12, lo=5, hi=12, seed=5):
    g = np.random.default_rng(seed)
    lens = g.integers(lo, hi + 1, size=B)
    q = g.integers(1, cfg.pad_id, size=(B, Lq)).astype(np.int32)
    mask = (np.arange(Lq)[None, :] >= (Lq - lens)[:, None]).astype(np.uint8)
    return np.where(mask == 1, q, cfg.pad_id).astype(np.int32), mask


@pytest.fixture(scope="module")
def model(tiny_cfg):
    w = make_weights(tiny_cfg, 7, variant="test")
    for k in w:  # larger weights so that attention and MLP matter numerically
        if k.endswith(("w_qkv", "w_o", "w_fc1", "w_fc2")) or k in ("embed_in", "embed_out"):
            w[k] = (w[k] * 8).astype(np.float32)
    return O.OracleModel(w, tiny_cfg)


# ------------------------------------------------------------------ library implementation pin
def test_forward_matches_transformers_gpt_neox(model, tiny_cfg):
    """The paper's forward IS transformers' GPT-NeoX (General Details, Tech stack): load the same
    weights into that class (float64, CPU) and compare logits on a left-padded batch."""
    torch = pytest.importorskip("torch")
    tr = pytest.importorskip("transformers")
    cfg = tiny_cfg
    hc = tr.GPTNeoXConfig(vocab_size=cfg.vocab, hidden_size=cfg.d_model, num_hidden_layers=cfg.n_layers,
                          num_attention_heads=cfg.n_heads, intermediate_size=cfg.d_ff, hidden_act="gelu",
                          rotary_pct=cfg.rotary_dims / cfg.head_dim, rotary_emb_base=cfg.rope_base,
                          max_position_embeddings=64, layer_norm_eps=cfg.ln_eps, use_parallel_residual=True,
                          tie_word_embeddings=False, attention_dropout=0.0, hidden_dropout=0.0,
                          attention_bias=True)
    hf = tr.GPTNeoXForCausalLM(hc).double().eval()
    w = model.w
    H, hd, d = cfg.n_heads, cfg.head_dim, cfg.d_model
    sd = {}
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    sd["gpt_neox.embed_in.weight"] = t(w["embed_in"])
    sd["lm_head.weight"] = t(w["embed_out"])
    sd["gpt_neox.final_layer_norm.weight"] = t(w["lnf_g"])
    sd["gpt_neox.final_layer_norm.bias"] = t(w["lnf_b"])
    for l in range(cfg.n_layers):
        p = f"gpt_neox.layers.{l}."
        g = lambda n: w[f"layers.{l}.{n}"]
        # that class views the fused projection output as [H, 3*hd] (q|k|v inside each head); this
        # repo orders rows [q all heads | k all heads | v all heads] -> permute rows
        wq = g("w_qkv").reshape(3, H, hd, d).transpose(1, 0, 2, 3).reshape(3 * d, d)
        bq = g("b_qkv").reshape(3, H, hd).transpose(1, 0, 2).reshape(3 * d)
        sd[p + "attention.query_key_value.weight"] = t(wq)
        sd[p + "attention.query_key_value.bias"] = t(bq)
        sd[p + "attention.dense.weight"] = t(g("w_o"))
        sd[p + "attention.dense.bias"] = t(g("b_o"))
        sd[p + "input_layernorm.weight"] = t(g("ln1_g"))
        sd[p + "input_layernorm.bias"] = t(g("ln1_b"))
        sd[p + "post_attention_layernorm.weight"] = t(g("ln2_g"))
        sd[p + "post_attention_layernorm.bias"] = t(g("ln2_b"))
        sd[p + "mlp.dense_h_to_4h.weight"] = t(g("w_fc1"))
        sd[p + "mlp.dense_h_to_4h.bias"] = t(g("b_fc1"))
        sd[p + "mlp.dense_4h_to_h.weight"] = t(g("w_fc2"))
        sd[p + "mlp.dense_4h_to_h.bias"] = t(g("b_fc2"))
    missing, unexpected = hf.load_state_dict(sd, strict=False)
    assert not [k for k in missing if "inv_freq" not in k and "rotary" not in k], missing
    assert not unexpected
    tokens, mask = _queries(cfg, B=3, Lq=12)
    am = torch.tensor(mask.astype(np.int64))
    pos = torch.clamp(am.cumsum(-1) - 1, min=0)
    with torch.no_grad():
        ref = hf(input_ids=torch.tensor(tokens.astype(np.int64)), attention_mask=am, position_ids=pos).logits.numpy()
    rows = [(b, t) for b in range(3) for t in range(12) if mask[b, t]]
    mine = O.logits_rows(model, tokens, mask, rows)
    want = np.stack([ref[b, t] for b, t in rows])
    assert np.abs(want).max() > 0.5  # the comparison is not vacuous
    np.testing.assert_allclose(mine, want, atol=1e-6, rtol=0)  # that class builds its rotary tables in float32


# ------------------------------------------------------------------ brute force: no KV cache
def test_cached_decode_equals_full_recompute(model, tiny_cfg):
    cfg = tiny_cfg
    queries, mask = _queries(cfg, B=2, Lq=10, lo=4, hi=10, seed=9)
    seed, T, N = 1234, 0.7, 7
    toks, lps, lens = O.rollout_generate(model, queries, mask, seed, T, N)
    for b in range(2):
        seq = list(queries[b][mask[b] == 1])
        for t in range(N):
            x, _ = O.forward_sequence(model, np.array(seq), np.arange(len(seq)))  # whole prefix, no cache
            logits, _ = O.heads(model, x[-1:])
            g = O.gumbel_from_bits(O.noise_bits(seed, b, t, cfg.vocab))
            tok, lp, _ = O.sample_token(logits[0], T, g)
            if t < lens[b]:
                assert tok == toks[b, 10 + t]
                assert abs(lp - lps[b, t]) < 1e-10
            seq.append(tok)


def test_rescoring_reproduces_rollout_logprobs(model, tiny_cfg):
    """Dropout is off, so the rescored log-probs equal the behaviour policy's (General Details,
    "Disable dropout": PPO ratios are 1 in the first epoch)."""
    cfg = tiny_cfg
    queries, mask = _queries(cfg, B=3, Lq=12)
    toks, lps, lens = O.rollout_generate(model, queries, mask, 77, 0.7, 6)
    full_mask = np.concatenate([mask, (np.arange(6)[None, :] < lens[:, None]).astype(np.uint8)], axis=1)
    slp, _ = O.score_sequences(model, toks, full_mask, 0.7)
    np.testing.assert_allclose(slp[:, 12:], lps, atol=1e-10)
    assert (lps <= 0).all() and (lps[:, 0] < 0).all()


# ------------------------------------------------------------------ invariants
def test_left_padding_does_not_change_outputs(model, tiny_cfg):
    cfg = tiny_cfg
    g = np.random.default_rng(3)
    body = g.integers(1, cfg.pad_id, size=7).astype(np.int32)
    outs = []
    for pad in (0, 5):
        q = np.concatenate([np.full(pad, cfg.pad_id, np.int32), body])[None, :]
        m = np.concatenate([np.zeros(pad, np.uint8), np.ones(7, np.uint8)])[None, :]
        outs.append(O.rollout_generate(model, q, m, 5, 0.7, 5))
    assert (outs[0][0][0, 7:] == outs[1][0][0, 12:]).all()
    assert (outs[0][1] == outs[1][1]).all()  # bit-identical: masked keys are skipped, not added


def test_causality_and_batch_independence(model, tiny_cfg):
    cfg = tiny_cfg
    tokens, mask = _queries(cfg, B=2, Lq=12, lo=12, hi=12)
    lp0, v0 = O.score_sequences(model, tokens, mask, 1.0)
    t2 = tokens.copy()
    t2[0, 8] = (t2[0, 8] + 1) % cfg.pad_id
    lp1, v1 = O.score_sequences(model, t2, mask, 1.0)
    assert (v0[0, :8] == v1[0, :8]).all() and (lp0[0, :8] == lp1[0, :8]).all()
    assert (v0[0, 8:] != v1[0, 8:]).all()
    assert (lp0[1] == lp1[1]).all()
    lp_single, _ = O.score_sequences(model, tokens[1:], mask[1:], 1.0)
    assert (lp_single[0] == lp0[1]).all()


def test_softmax_rows_sum_to_one(model, tiny_cfg):
    tokens, mask = _queries(tiny_cfg, B=1, Lq=6, lo=6, hi=6)
    logits = O.logits_rows(model, tokens, mask, [(0, 3)])[0]
    lps = np.array([O.log_softmax_at(logits, 0.7, v) for v in range(tiny_cfg.vocab)])
    assert (lps <= 0).all()
    assert abs(np.exp(lps).sum() - 1.0) < 1e-12
    # against the textbook definition written directly
    z = logits / float(np.float32(0.7))
    np.testing.assert_allclose(lps, z - np.log(np.exp(z).sum()), atol=1e-12)


# ------------------------------------------------------------------ closed forms
def test_zero_output_embedding_gives_uniform_logprobs(tiny_cfg):
    cfg = tiny_cfg.with_(vocab=50304, pad_id=50277)
    w = make_weights(cfg, 3, variant="test")
    w["embed_out"] = np.zeros_like(w["embed_out"])
    m = O.OracleModel(w, cfg)
    tokens, mask = _queries(cfg, B=1, Lq=5, lo=4, hi=4)
    lp, val = O.score_sequences(m, tokens, mask, 0.7)
    np.testing.assert_allclose(lp[0, 2:], -math.log(50304), atol=1e-12)
    assert abs(-math.log(50304) - (-10.825840)) < 1e-6
    assert lp[0, 0] == 0 and lp[0, 1] == 0  # pad, and the first real token has no predecessor


def test_zero_layer_model_is_layernorm_times_embedding(tiny_cfg):
    cfg = tiny_cfg.with_(n_layers=0)
    w = make_weights(cfg, 4, variant="test")
    m = O.OracleModel(w, cfg)
    tokens, mask = _queries(cfg, B=1, Lq=4, lo=4, hi=4)
    got = O.logits_rows(m, tokens, mask, [(0, 2)])[0]
    e = w["embed_in"][tokens[0, 2]].astype(np.float64)
    h = (e - e.mean()) / np.sqrt(e.var() + cfg.ln_eps) * w["lnf_g"] + w["lnf_b"]
    np.testing.assert_allclose(got, w["embed_out"].astype(np.float64) @ h, atol=1e-12)
    _, val = O.score_sequences(m, tokens, mask, 1.0)
    assert abs(val[0, 2] - (h @ w["value_w"].astype(np.float64) + float(np.float32(0.3)))) < 1e-12


def test_single_token_attention_returns_value(tiny_cfg):
    g = np.random.default_rng(0)
    q, k, v = (g.standard_normal((1, 3, 16)) for _ in range(3))
    np.testing.assert_allclose(O.attention(q, [0], k, v, [0], 16), v, atol=1e-15)


def test_attention_against_explicit_loops(tiny_cfg):
    g = np.random.default_rng(1)
    n, H, hd = 5, 2, 8
    q, k, v = (g.standard_normal((n, H, hd)) for _ in range(3))
    got = O.attention(q, np.arange(n), k, v, np.arange(n), hd)
    for i in range(n):
        for h in range(H):
            s = np.array([q[i, h] @ k[j, h] / math.sqrt(hd) for j in range(i + 1)])
            p = np.exp(s) / np.exp(s).sum()
            want = sum(p[j] * v[j, h] for j in range(i + 1))
            np.testing.assert_allclose(got[i, h], want, atol=1e-13)


def test_layer_norm_and_gelu_against_library():
    torch = pytest.importorskip("torch")
    g = np.random.default_rng(2)
    x = g.standard_normal((4, 32)) * 3 + 1
    y = O.layer_norm(x, 1.0, 0.0, 1e-5)
    assert np.abs(y.mean(-1)).max() < 1e-12 and np.abs(y.var(-1) - 1).max() < 1e-4
    gam, bet = g.standard_normal(32), g.standard_normal(32)
    want = torch.nn.functional.layer_norm(torch.tensor(x), (32,), torch.tensor(gam), torch.tensor(bet), 1e-5)
    np.testing.assert_allclose(O.layer_norm(x, gam, bet, 1e-5), want.numpy(), atol=1e-12)
    np.testing.assert_allclose(O.gelu_erf(x), torch.nn.functional.gelu(torch.tensor(x)).numpy(), atol=1e-12)
    assert abs(O.gelu_erf(np.array([1.0]))[0] - 0.8413447460685429) < 1e-12  # Phi(1)


def test_rope_identities():
    g = np.random.default_rng(4)
    r, base = 8, 10000.0
    q = g.standard_normal((1, 2, 16))
    k = g.standard_normal((1, 2, 16))
    np.testing.assert_array_equal(O.rope(q, [0], r, base), q)  # position 0 is the identity
    for p in (1, 17):
        rq = O.rope(q, [p], r, base)
        np.testing.assert_array_equal(rq[..., r:], q[..., r:])  # dims >= r untouched
        np.testing.assert_allclose((rq ** 2).sum(-1), (q ** 2).sum(-1), atol=1e-12)  # norm kept
    d1 = (O.rope(q, [9], r, base) * O.rope(k, [4], r, base)).sum(-1)
    d2 = (O.rope(q, [25], r, base) * O.rope(k, [20], r, base)).sum(-1)
    np.testing.assert_allclose(d1, d2, atol=1e-10)  # depends on the offset only
    # pair (i, i + r/2) turns by pos * base^(-2i/r): check one pair by hand
    u = np.zeros((1, 1, 16)); u[0, 0, 1] = 1.0
    out = O.rope(u, [3], r, base)
    th = 3 * base ** (-2 * 1 / r)
    assert abs(out[0, 0, 1] - math.cos(th)) < 1e-15 and abs(out[0, 0, 1 + r // 2] - math.sin(th)) < 1e-15


# ------------------------------------------------------------------ sampler
def test_noise_is_a_pure_function_of_its_four_keys():
    a = O.noise_bits(1, 2, 3, 64)
    assert (a == O.noise_bits(1, 2, 3, 64)).all()
    assert (a[:32] == O.noise_bits(1, 2, 3, 32)).all()  # entry v does not depend on the vocab size
    for other in (O.noise_bits(2, 2, 3, 64), O.noise_bits(1, 3, 3, 64), O.noise_bits(1, 2, 4, 64)):
        assert (a != other).mean() > 0.9
    # golden values: fix the integer arithmetic the GPU must reproduce bit for bit
    assert O.noise_bits(0, 0, 0, 4).tolist() == _scalar_hash_reference(0, 0, 0, 4)
    assert O.noise_bits(2**64 - 1, 511, 52, 3).tolist() == _scalar_hash_reference(2**64 - 1, 511, 52, 3)


def _scalar_hash_reference(seed, b, t, n):
    """The same hash in plain Python integers (unbounded, reduced mod 2^64 by hand)."""
    M = (1 << 64) - 1
    G, M1, M2 = 0x9E3779B97F4A7C15, 0xBF58476D1CE4E5B9, 0x94D049BB133111EB

    def f(x):
        x ^= x >> 30; x = (x * M1) & M
        x ^= x >> 27; x = (x * M2) & M
        return x ^ (x >> 31)
    kr = f((seed + G * (b + 1)) & M)
    ks = f((kr + G * (t + 1)) & M)
    return [f((ks + G * (v + 1)) & M) >> 32 for v in range(n)]


def test_hash_avalanche():
    a = O.noise_bits(5, 0, 0, 4096)
    flips = []
    for other in (O.noise_bits(5 ^ 1, 0, 0, 4096), O.noise_bits(5, 1, 0, 4096), O.noise_bits(5, 0, 1, 4096)):
        x = a ^ other
        flips.append(np.unpackbits(x.view(np.uint8)).mean())
    assert all(0.47 < f < 0.53 for f in flips), flips
    # consecutive token ids: neighbouring outputs differ in about half their bits
    x = a[1:] ^ a[:-1]
    assert 0.47 < np.unpackbits(x.view(np.uint8)).mean() < 0.53
    u = (a.astype(np.float64) + 0.5) / 2**32
    assert abs(u.mean() - 0.5) < 0.02 and abs(u.var() - 1 / 12) < 0.01


def test_gumbel_extremes_are_finite():
    g = O.gumbel_from_bits(np.array([0, 1, 2**31 - 1, 2**31, 2**32 - 2, 2**32 - 1], dtype=np.uint32))
    assert np.isfinite(g).all()
    assert (np.diff(g) >= 0).all() and g[0] < g[2] < g[-1]
    assert abs(float(g[0]) - (-math.log(-math.log(0.5 / 2**32)))) < 1e-6
    assert abs(float(g[-1]) - (-math.log(-math.log1p(-0.5 / 2**32)))) < 1e-5


def test_gumbel_max_samples_from_softmax():
    """Gumbel-max is an exact sampler: over many independent draws the token frequencies follow
    softmax(logits / T).  Chi-square on a vocabulary of 8."""
    V, T, n = 8, 0.7, 40000
    logits = np.array([0.3, -1.0, 1.2, 0.0, 2.0, -0.5, 0.9, 0.1])
    z = logits / float(np.float32(T))
    p = np.exp(z) / np.exp(z).sum()
    counts = np.zeros(V)
    for i in range(n):
        tok, lp, score = O.sample_token(logits, T, O.gumbel_from_bits(O.noise_bits(99, i % 200, i // 200, V)))
        counts[tok] += 1
        assert tok == int(np.argmax(score))
        if i < 50:
            assert abs(lp - math.log(p[tok])) < 1e-12
    chi2 = ((counts - n * p) ** 2 / (n * p)).sum()
    assert chi2 < 24.3, chi2  # 99.9th percentile of chi-square with 7 degrees of freedom


def test_argmax_ties_go_to_the_lowest_id():
    logits = np.zeros(6)
    g = np.array([0.5, 1.5, 1.5, -1.0, 1.5, 0.0], dtype=np.float32)
    assert O.sample_token(logits, 0.7, g)[0] == 1


# ------------------------------------------------------------------ EOS stop mask
def test_eos_truncation(tiny_cfg):
    cfg = tiny_cfg
    w = make_weights(cfg, 7, variant="test")
    wb = boost_eos(cfg, w, alpha=3.0)
    m0, m1 = O.OracleModel(w, cfg), O.OracleModel(wb, cfg)
    queries, mask = _queries(cfg, B=6, Lq=8, lo=3, hi=8, seed=1)
    N = 10
    toks, lps, lens = O.rollout_generate(m1, queries, mask, 4321, 0.7, N)
    assert (lens < N).any() and (lens > 1).any()
    for b in range(6):
        r = toks[b, 8:]
        L = lens[b]
        if L < N:
            assert r[L - 1] == cfg.eos_id and (r[:L - 1] != cfg.eos_id).all()
            assert (r[L:] == cfg.pad_id).all() and (lps[b, L:] == 0).all()
        assert (lps[b, :L] < 0).all()
    assert (toks[:, :8] == queries).all()
    # verify_rollout accepts the oracle's own rollout with zero deficit everywhere
    rep = O.verify_rollout(m1, toks, mask, 4321, 0.7, N)
    assert len(rep) == int(lens.sum())
    assert all(r["deficit"] == 0.0 and r["token"] == r["argmax"] for r in rep)
    for r in rep:
        assert abs(r["logprob"] - lps[r["row"], r["step"]]) < 1e-10
    # and it flags a wrong token
    bad = toks.copy()
    bad[0, 8] = (bad[0, 8] + 1) % cfg.pad_id
    rep = O.verify_rollout(m1, bad, mask, 4321, 0.7, N, rows=[0])
    assert rep[0]["deficit"] > 0


def test_all_pad_row_and_mask_validation(model, tiny_cfg):
    cfg = tiny_cfg
    q = np.full((1, 4), cfg.pad_id, np.int32)
    toks, lps, lens = O.rollout_generate(model, q, np.zeros((1, 4), np.uint8), 1, 0.7, 3)
    assert lens[0] == 0 and (toks == cfg.pad_id).all() and (lps == 0).all()
    with pytest.raises(ValueError):
        O.score_sequences(model, np.ones((1, 4), np.int32), np.array([[1, 0, 1, 1]], np.uint8), 1.0)
