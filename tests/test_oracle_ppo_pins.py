"""Pins of oracle/ppo_signals_oracle.py against what the paper and the mathematics fix (CPU only)."""
import numpy as np
import pytest

from oracle import ppo_signals_oracle as O

EOS, PAD = 0, 50277


def _batch(seed, B=7, N=11):
    g = np.random.default_rng(seed)
    lp = -np.abs(g.normal(2.0, 1.0, (B, N)))
    rlp = -np.abs(g.normal(2.0, 1.0, (B, N)))
    rv = g.normal(0.0, 2.0, (B, N))
    tok = g.integers(1, 50000, (B, N))
    lengths = g.integers(1, N + 1, B)
    lengths[0] = N            # full length, no EOS
    tok[1, N - 1] = EOS       # EOS exactly at the last slot
    lengths[1] = N
    for b in range(2, B):
        tok[b, lengths[b] - 1] = EOS
        tok[b, lengths[b]:] = PAD
    return lp, rlp, rv, tok, lengths


def test_score_index_is_first_pad_minus_one_or_last_token():
    """Reward Model Details, "Extract reward from the EOS token"."""
    assert O.rm_score_index([5, 6, EOS, PAD, PAD], PAD) == 2
    assert O.rm_score_index([5, 6, 7, 8, 9], PAD) == 4
    assert O.rm_score_index([5, 6, 7, 8, EOS], PAD) == 4
    assert O.rm_score_index([EOS, PAD, PAD], PAD) == 0
    assert O.rm_score_index([PAD, PAD], PAD) == -1


def test_total_reward_is_score_minus_beta_kl():
    """Preliminaries, Eq. (RL): the per-token rewards of a row sum to r - beta * KL."""
    lp, rlp, rv, tok, lengths = _batch(1)
    beta = 0.05
    rew, scores, kl = O.assemble_rewards(lp, rlp, rv, tok, EOS, PAD, beta)
    for b in range(len(lengths)):
        L = lengths[b]
        kl_direct = float(np.sum(lp[b, :L] - rlp[b, :L]))
        assert kl[b] == pytest.approx(kl_direct, abs=1e-12)
        assert rew[b].sum() == pytest.approx(scores[b] - beta * kl_direct, abs=1e-12)
        assert (rew[b, L:] == 0).all()
        # all tokens but the last carry the penalty only (figure "Reward and values of a completion")
        np.testing.assert_allclose(rew[b, :L - 1], -beta * (lp[b, :L - 1] - rlp[b, :L - 1]), atol=1e-15)


def test_missing_eos_gets_minus_one_and_eos_rows_get_the_rm_value_at_eos():
    """PPO Details, "EOS trick", step 3."""
    lp, rlp, rv, tok, lengths = _batch(2)
    _, scores, _ = O.assemble_rewards(lp, rlp, rv, tok, EOS, PAD, 0.05)
    assert scores[0] == -1.0                       # 11 tokens, none of them EOS
    assert scores[1] == rv[1, -1]                  # EOS in the last slot: a valid score
    for b in range(2, len(lengths)):
        assert scores[b] == rv[b, lengths[b] - 1]


def test_beta_zero_leaves_only_the_score_and_identical_policies_have_no_penalty():
    lp, rlp, rv, tok, lengths = _batch(3)
    rew, scores, _ = O.assemble_rewards(lp, rlp, rv, tok, EOS, PAD, 0.0)
    for b in range(len(lengths)):
        assert np.count_nonzero(rew[b]) <= 1 and rew[b, lengths[b] - 1] == scores[b]
    rew2, scores2, kl2 = O.assemble_rewards(lp, lp, rv, tok, EOS, PAD, 0.05)
    assert (kl2 == 0).all()
    np.testing.assert_array_equal(rew2, rew)


def test_row_without_response_is_all_zero():
    lp, rlp, rv, tok, _ = _batch(4)
    tok[3, :] = PAD
    rew, scores, kl = O.assemble_rewards(lp, rlp, rv, tok, EOS, PAD, 0.05)
    assert (rew[3] == 0).all() and scores[3] == 0 and kl[3] == 0


def _gae_double_sum(r, v, L, gamma, lam):
    """The definition written out: A_t = sum_{l>=0} (gamma*lam)^l delta_{t+l}."""
    delta = [r[t] + gamma * (v[t + 1] if t + 1 < L else 0.0) - v[t] for t in range(L)]
    return [sum((gamma * lam) ** (s - t) * delta[s] for s in range(t, L)) for t in range(L)]


@pytest.mark.parametrize("gamma,lam", [(1.0, 0.95), (0.99, 0.9), (1.0, 1.0), (0.9, 0.0)])
def test_gae_matches_the_defining_double_sum(gamma, lam):
    g = np.random.default_rng(5)
    B, N = 6, 13
    r, v = g.normal(0, 1, (B, N)), g.normal(0, 1, (B, N))
    lengths = np.array([13, 1, 0, 7, 12, 2])
    adv, ret = O.gae(r, v, lengths, gamma, lam)
    for b in range(B):
        L = lengths[b]
        np.testing.assert_allclose(adv[b, :L], _gae_double_sum(r[b], v[b], L, gamma, lam), atol=1e-12)
        np.testing.assert_allclose(ret[b, :L], adv[b, :L] + v[b, :L], atol=1e-15)
        assert (adv[b, L:] == 0).all() and (ret[b, L:] == 0).all()


def test_gae_lambda_one_is_reward_to_go_minus_value_and_lambda_zero_is_td_residual():
    """With gamma = 1 (PPO hyperparameter table): lambda = 1 telescopes to sum_{s>=t} r_s - V_t, so the
    return is the plain reward-to-go; lambda = 0 leaves the one-step residual."""
    g = np.random.default_rng(6)
    r, v = g.normal(0, 1, (3, 9)), g.normal(0, 1, (3, 9))
    lengths = np.array([9, 4, 6])
    adv1, ret1 = O.gae(r, v, lengths, 1.0, 1.0)
    adv0, _ = O.gae(r, v, lengths, 1.0, 0.0)
    for b in range(3):
        L = lengths[b]
        togo = np.cumsum(r[b, :L][::-1])[::-1]
        np.testing.assert_allclose(ret1[b, :L], togo, atol=1e-12)
        np.testing.assert_allclose(adv1[b, :L], togo - v[b, :L], atol=1e-12)
        vn = np.append(v[b, 1:L], 0.0)
        np.testing.assert_allclose(adv0[b, :L], r[b, :L] + vn - v[b, :L], atol=1e-15)


def test_gae_constant_residual_is_a_geometric_series():
    """Zero values and reward c at every step: delta = c, so A_t = c * (1 - x^(L-t)) / (1 - x) with
    x = gamma * lambda."""
    L, c, gamma, lam = 20, 0.3, 1.0, 0.95
    r = np.full((1, L), c)
    adv, _ = O.gae(r, np.zeros((1, L)), np.array([L]), gamma, lam)
    x = gamma * lam
    want = c * (1 - x ** (L - np.arange(L))) / (1 - x)
    np.testing.assert_allclose(adv[0], want, rtol=1e-12)


def test_whiten_dense_matches_mean_and_biased_variance():
    """PPO Details, "(Optional) Reward whitening": the printed function on a dense tensor."""
    g = np.random.default_rng(7)
    x = g.normal(3.0, 2.5, (8, 53))
    w = O.whiten(x)
    want = (x - x.mean()) / np.sqrt(x.var() + 1e-8)   # numpy's var is the biased one
    np.testing.assert_allclose(w, want, atol=1e-12)
    assert abs(w.mean()) < 1e-12 and w.var() == pytest.approx(1.0, abs=1e-7)
    # the flag set to False adds the mean back: unit variance around the old mean
    w2 = O.whiten(x, shift_mean=False)
    np.testing.assert_allclose(w2, want + x.mean(), atol=1e-12)
    assert w2.mean() == pytest.approx(x.mean(), abs=1e-12)


def test_whiten_is_invariant_to_scale_and_shift_and_respects_the_mask():
    g = np.random.default_rng(8)
    x = g.normal(0.0, 1.0, (5, 17))
    mask = (np.arange(17)[None, :] < np.array([17, 3, 0, 9, 1])[:, None])
    w = O.whiten(x, mask)
    np.testing.assert_allclose(O.whiten(4.0 * x + 11.0, mask), w, atol=1e-6)   # 1e-8 inside the root
    assert (w[~mask] == 0).all()
    sel = x[mask]
    np.testing.assert_allclose(w[mask], (sel - sel.mean()) / np.sqrt(sel.var() + 1e-8), atol=1e-12)
    # garbage outside the mask does not matter
    y = x.copy()
    y[~mask] = 1e9
    np.testing.assert_array_equal(O.whiten(y, mask), w)
    assert (O.whiten(x, np.zeros_like(mask)) == 0).all()


def test_whiten_of_a_constant_is_zero_not_nan():
    w = O.whiten(np.full((2, 3), 5.0))
    assert np.isfinite(w).all() and (w == 0).all()
