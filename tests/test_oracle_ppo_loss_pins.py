"""Pins of oracle/ppo_loss_oracle.py against closed forms, a hand-worked example and finite differences
(CPU only)."""
import numpy as np
import pytest

from oracle import ppo_loss_oracle as O


def _batch(seed, B=6, N=9):
    g = np.random.default_rng(seed)
    lp0 = -np.abs(g.normal(2.0, 1.0, (B, N)))
    lp = lp0 + g.normal(0.0, 0.25, (B, N))        # ratios from ~0.5 to ~2: both clips occur
    adv = g.normal(0.0, 1.0, (B, N))
    v0 = g.normal(0.0, 1.0, (B, N))
    v = v0 + g.normal(0.0, 0.3, (B, N))           # beyond +-0.2 often
    ret = v0 + g.normal(0.0, 0.5, (B, N))
    kept = g.integers(0, N + 1, B)
    kept[0], kept[1] = N, 0
    return lp, lp0, adv, v, v0, ret, kept


def test_identical_policies_and_values_reduce_to_plain_means():
    """ratio = 1 everywhere and V = V_old: nothing clips, loss = -mean(A) + c1 * 0.5 * mean((V-R)^2),
    gradients -A/n and c1 (V-R)/n (PPO hyperparameter table: c1 = 0.1)."""
    lp, lp0, adv, v, v0, ret, kept = _batch(1)
    st, dlp, dv = O.ppo_loss(lp0, lp0, adv, v0, v0, ret, kept)
    mask = np.arange(adv.shape[1])[None, :] < kept[:, None]
    n = mask.sum()
    assert st["n_tokens"] == n
    assert st["pg_loss"] == pytest.approx(-adv[mask].mean(), abs=1e-14)
    assert st["vf_loss"] == pytest.approx(0.5 * ((v0 - ret)[mask] ** 2).mean(), abs=1e-14)
    assert st["loss"] == pytest.approx(st["pg_loss"] + 0.1 * st["vf_loss"], abs=1e-15)
    assert st["approx_kl"] == 0 and st["pg_clipfrac"] == 0 and st["vf_clipfrac"] == 0 and st["ratio_mean"] == 1
    np.testing.assert_allclose(dlp[mask], -adv[mask] / n, atol=1e-15)
    np.testing.assert_allclose(dv[mask], 0.1 * (v0 - ret)[mask] / n, atol=1e-15)
    assert (dlp[~mask] == 0).all() and (dv[~mask] == 0).all()


def test_hand_worked_example_with_both_clips_in_both_directions():
    """Four tokens, eps = eps_v = 0.2, c1 = 0.1, worked on paper:
    t0: A=+1, ratio=1.5 -> surrogates -1.5 / -1.2, max -1.2 (clipped, no gradient)
    t1: A=-1, ratio=1.5 -> +1.5 / +1.2, max 1.5 (unclipped, gradient -A*ratio/n = 1.5/4)
    t2: A=+2, ratio=0.5 -> -1.0 / -1.6, max -1.0 (unclipped, gradient -2*0.5/4)
    t3: A=-2, ratio=0.5 -> +1.0 / +1.6, max 1.6 (clipped)
    values (V, Vold, R): (1.0, 0.5, 0.0): clip to 0.7 -> 1.0 vs 0.49, max 1.0 (unclipped, grad 0.1*1/4)
                         (0.0, 0.5, 1.0): clip to 0.3 -> 1.0 vs 0.49, unclipped, grad 0.1*(-1)/4
                         (1.0, 0.5, 2.0): clip to 0.7 -> 1.0 vs 1.69, clipped
                         (0.6, 0.5, 0.0): inside -> 0.36 both, unclipped, grad 0.1*0.6/4"""
    lp0 = np.zeros((1, 4))
    lp = np.log(np.array([[1.5, 1.5, 0.5, 0.5]]))
    adv = np.array([[1.0, -1.0, 2.0, -2.0]])
    v = np.array([[1.0, 0.0, 1.0, 0.6]])
    v0 = np.full((1, 4), 0.5)
    ret = np.array([[0.0, 1.0, 2.0, 0.0]])
    st, dlp, dv = O.ppo_loss(lp, lp0, adv, v, v0, ret, [4])
    assert st["pg_loss"] == pytest.approx((-1.2 + 1.5 - 1.0 + 1.6) / 4, abs=1e-12)
    assert st["vf_loss"] == pytest.approx(0.5 * (1.0 + 1.0 + 1.69 + 0.36) / 4, abs=1e-12)
    assert st["loss"] == pytest.approx(st["pg_loss"] + 0.1 * st["vf_loss"], abs=1e-15)
    assert st["pg_clipfrac"] == 0.5 and st["vf_clipfrac"] == 0.25
    assert st["ratio_mean"] == pytest.approx(1.0, abs=1e-12)
    assert st["approx_kl"] == pytest.approx(0.5 * (2 * np.log(1.5) ** 2 + 2 * np.log(0.5) ** 2) / 4, abs=1e-12)
    np.testing.assert_allclose(dlp[0], [0.0, 1.5 / 4, -1.0 / 4, 0.0], atol=1e-12)
    np.testing.assert_allclose(dv[0], [0.1 / 4, -0.1 / 4, 0.0, 0.06 / 4], atol=1e-12)


def test_gradients_match_central_finite_differences():
    lp, lp0, adv, v, v0, ret, kept = _batch(2)
    st, dlp, dv = O.ppo_loss(lp, lp0, adv, v, v0, ret, kept)
    h = 1e-6
    g = np.random.default_rng(3)
    checked = 0
    for _ in range(60):
        b, t = int(g.integers(0, lp.shape[0])), int(g.integers(0, lp.shape[1]))
        # stay away from the kinks of clip and max, where the one-sided derivatives differ
        ratio = np.exp(lp[b, t] - lp0[b, t])
        if min(abs(ratio - 0.8), abs(ratio - 1.2)) < 1e-3:
            continue
        if min(abs(v[b, t] - v0[b, t] - 0.2), abs(v[b, t] - v0[b, t] + 0.2)) < 1e-3:
            continue
        vc = min(max(v[b, t], v0[b, t] - 0.2), v0[b, t] + 0.2)
        if abs((v[b, t] - ret[b, t]) ** 2 - (vc - ret[b, t]) ** 2) < 1e-3 and vc != v[b, t]:
            continue
        for arr, grad in ((lp, dlp), (v, dv)):
            up, dn = arr.copy(), arr.copy()
            up[b, t] += h
            dn[b, t] -= h
            args_up = (up, lp0, adv, v, v0, ret, kept) if arr is lp else (lp, lp0, adv, up, v0, ret, kept)
            args_dn = (dn, lp0, adv, v, v0, ret, kept) if arr is lp else (lp, lp0, adv, dn, v0, ret, kept)
            fd = (O.ppo_loss(*args_up)[0]["loss"] - O.ppo_loss(*args_dn)[0]["loss"]) / (2 * h)
            assert fd == pytest.approx(grad[b, t], abs=2e-8)
        checked += 1
    assert checked > 30


def test_masked_positions_do_not_matter_and_empty_batch_is_zero():
    lp, lp0, adv, v, v0, ret, kept = _batch(4)
    st, dlp, dv = O.ppo_loss(lp, lp0, adv, v, v0, ret, kept)
    mask = np.arange(adv.shape[1])[None, :] < kept[:, None]
    junk = [a.copy() for a in (lp, lp0, adv, v, v0, ret)]
    for a in junk:
        a[~mask] = 1e6
    st2, dlp2, dv2 = O.ppo_loss(*junk, kept)
    assert st2 == st
    np.testing.assert_array_equal(dlp2, dlp)
    np.testing.assert_array_equal(dv2, dv)
    st0, dlp0, dv0 = O.ppo_loss(lp, lp0, adv, v, v0, ret, np.zeros(len(kept), int))
    assert st0["loss"] == 0 and st0["n_tokens"] == 0 and not dlp0.any() and not dv0.any()


def test_duplicating_the_batch_keeps_the_loss_and_halves_the_gradients():
    lp, lp0, adv, v, v0, ret, kept = _batch(5)
    st, dlp, dv = O.ppo_loss(lp, lp0, adv, v, v0, ret, kept)
    two = [np.concatenate([a, a]) for a in (lp, lp0, adv, v, v0, ret)]
    st2, dlp2, dv2 = O.ppo_loss(*two, np.concatenate([kept, kept]))
    for k in ("loss", "pg_loss", "vf_loss", "approx_kl", "pg_clipfrac", "vf_clipfrac", "ratio_mean"):
        assert st2[k] == pytest.approx(st[k], rel=1e-13, abs=1e-15)
    np.testing.assert_allclose(dlp2[: len(kept)], dlp / 2, atol=1e-15)
    np.testing.assert_allclose(dv2[len(kept):], dv / 2, atol=1e-15)


def test_clip_ranges_and_coefficient_are_the_papers_defaults():
    """PPO hyperparameter table: eps = 0.2, value clip 0.2, c1 = 0.1."""
    import inspect
    sig = inspect.signature(O.ppo_loss)
    assert sig.parameters["cliprange"].default == 0.2
    assert sig.parameters["cliprange_value"].default == 0.2
    assert sig.parameters["vf_coef"].default == 0.1
