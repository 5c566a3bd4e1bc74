"""GPU parity of the PPO objective and its output gradients against oracle/ppo_loss_oracle.py, through
the C ABI.  Both sides take the clip decisions in double on the same fp32 inputs; outputs are fp32
roundings of double results: the bar is 2e-6 relative (plus 1e-9 absolute for values near zero)."""
import numpy as np
import pytest

import paper_2403_17031_amd as P

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    P.load_library()  # fails loudly when the HIP library has not been built
    return P


def _batch(seed, B, N):
    g = np.random.default_rng(seed)
    f = np.float32
    lp0 = (-np.abs(g.normal(2.0, 1.0, (B, N)))).astype(f)
    lp = (lp0 + g.normal(0.0, 0.25, (B, N))).astype(f)
    adv = g.normal(0.0, 1.0, (B, N)).astype(f)
    v0 = g.normal(0.0, 1.0, (B, N)).astype(f)
    v = (v0 + g.normal(0.0, 0.3, (B, N))).astype(f)
    ret = (v0 + g.normal(0.0, 0.5, (B, N))).astype(f)
    kept = g.integers(0, N + 1, B).astype(np.int32)
    kept[0] = N
    if B > 1:
        kept[1] = 0
    # some tokens exactly on the old policy / old value (ratio exactly 1, no value move)
    lp[0, : min(3, N)] = lp0[0, : min(3, N)]
    v[0, : min(3, N)] = v0[0, : min(3, N)]
    return lp, lp0, adv, v, v0, ret, kept


def _compare(P, args, **kw):
    from oracle import ppo_loss_oracle as O
    stats, d_lp, d_v = P.ppo_loss(*args, **kw)
    o_stats, o_dlp, o_dv = O.ppo_loss(*args, **kw)
    stats = stats.cpu().numpy()
    for i, name in enumerate(P.PPO_LOSS_STATS):
        assert stats[i] == pytest.approx(o_stats[name], rel=2e-6, abs=1e-9), name
    np.testing.assert_allclose(d_lp.cpu().numpy(), o_dlp, rtol=2e-6, atol=1e-12)
    np.testing.assert_allclose(d_v.cpu().numpy(), o_dv, rtol=2e-6, atol=1e-12)
    # the clip decision itself is exact: the same positions carry a gradient
    assert ((d_lp.cpu().numpy() != 0) == (o_dlp != 0)).all()
    assert ((d_v.cpu().numpy() != 0) == (o_dv != 0)).all()
    return o_stats


@pytest.mark.parametrize("B,N", [(1, 1), (7, 9), (64, 53), (256, 53), (512, 53), (3, 1300)])
def test_loss_and_gradients_match_the_oracle(gpu, B, N):
    st = _compare(gpu, _batch(100 + B + N, B, N))
    if B >= 7:
        assert 0 < st["pg_clipfrac"] < 1 and 0 < st["vf_clipfrac"] < 1  # both branches were exercised


def test_other_coefficients(gpu):
    _compare(gpu, _batch(7, 33, 21), cliprange=0.1, cliprange_value=0.35, vf_coef=0.5)
    _compare(gpu, _batch(8, 33, 21), cliprange=0.0, cliprange_value=0.0, vf_coef=1.0)


def test_empty_batch_and_first_epoch(gpu):
    lp, lp0, adv, v, v0, ret, kept = _batch(9, 12, 17)
    stats, d_lp, d_v = gpu.ppo_loss(lp, lp0, adv, v, v0, ret, np.zeros(12, np.int32))
    assert not stats.cpu().numpy().any() and not d_lp.cpu().numpy().any() and not d_v.cpu().numpy().any()
    # first PPO epoch: the model has not moved, so ratio = 1 on every token and nothing clips
    st = _compare(gpu, (lp0, lp0, adv, v0, v0, ret, kept))
    assert st["ratio_mean"] == 1.0 and st["pg_clipfrac"] == 0 and st["approx_kl"] == 0


def test_rejects_bad_arguments(gpu):
    lp, lp0, adv, v, v0, ret, kept = _batch(10, 4, 5)
    with pytest.raises(gpu.RlhfError):
        gpu.ppo_loss(lp, lp0, adv, v, v0, ret, kept, cliprange=-0.1)
    with pytest.raises(gpu.RlhfError):
        gpu.ppo_loss(lp, lp0, adv, v, v0, ret, kept[:3])
    with pytest.raises(gpu.RlhfError):
        gpu.ppo_loss(lp, lp0[:, :4], adv, v, v0, ret, kept)
