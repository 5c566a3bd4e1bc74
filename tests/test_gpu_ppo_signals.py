"""GPU parity of reward assembly, GAE and whitening against oracle/ppo_signals_oracle.py, through the
C ABI.  fp32 outputs of double-precision recursions: the bar is 1e-5 absolute on O(1) values
(relative where values are large)."""
import numpy as np
import pytest

import paper_2403_17031_amd as P
from synth import WORKLOADS, make_weights

pytestmark = pytest.mark.gpu

EOS, PAD = 0, 50277


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    P.load_library()  # fails loudly when the HIP library has not been built
    return P


def _oracle():
    from oracle import ppo_signals_oracle as O
    return O


def _synthetic(seed, B, Lq, N):
    """Response-shaped inputs with every edge case: no EOS, EOS in the last slot, EOS first, an empty
    response, a pad id drawn in the middle of a response."""
    g = np.random.default_rng(seed)
    L = Lq + N
    tok = g.integers(1, 50000, (B, L)).astype(np.int32)
    lengths = g.integers(1, N + 1, B)
    lengths[0] = N
    lengths[1] = N
    tok[1, L - 1] = EOS
    lengths[2] = 1
    for b in range(2, B):
        tok[b, Lq + lengths[b] - 1] = EOS
        tok[b, Lq + lengths[b]:] = PAD
    if B > 4:
        tok[3, Lq:] = PAD                       # nothing generated
        tok[4, Lq + min(2, N - 1)] = PAD        # a stray pad id inside the response
    lp = -np.abs(g.normal(2.0, 1.0, (B, N))).astype(np.float32)
    ref = -np.abs(g.normal(2.0, 1.0, (B, L))).astype(np.float32)
    rm = g.normal(0.0, 2.0, (B, L)).astype(np.float32)
    val = g.normal(0.0, 1.0, (B, L)).astype(np.float32)
    return tok, lp, ref, rm, val


@pytest.mark.parametrize("B,Lq,N", [(9, 5, 7), (64, 16, 53), (256, 512, 53), (3, 0, 130)])
def test_rewards_gae_whiten_match_the_oracle(gpu, B, Lq, N):
    O = _oracle()
    tok, lp, ref, rm, val = _synthetic(B + N, B, Lq, N)
    beta = 0.05
    rew, sc, kl, kept = (x.cpu().numpy() for x in P.ppo_assemble_rewards(lp, ref, rm, tok, Lq, EOS, PAD, beta))
    o_rew, o_sc, o_kl = O.assemble_rewards(lp, ref[:, Lq:], rm[:, Lq:], tok[:, Lq:], EOS, PAD, beta)
    o_kept = np.array([O.rm_score_index(tok[b, Lq:], PAD) + 1 for b in range(B)])
    assert (kept == o_kept).all()
    np.testing.assert_allclose(rew, o_rew, atol=1e-6, rtol=1e-6)
    np.testing.assert_allclose(sc, o_sc, atol=0, rtol=0)
    np.testing.assert_allclose(kl, o_kl, atol=1e-5, rtol=1e-6)

    # state values of the response tokens are read one position earlier (the state that emitted them)
    off = max(Lq - 1, 0)
    adv, ret = (x.cpu().numpy() for x in P.ppo_gae(rew, val, kept, 1.0, 0.95, value_offset=off))
    o_adv, o_ret = O.gae(rew, val[:, off:off + N], kept, 1.0, 0.95)
    np.testing.assert_allclose(adv, o_adv, atol=1e-5, rtol=1e-6)
    np.testing.assert_allclose(ret, o_ret, atol=1e-5, rtol=1e-6)

    mask = np.arange(N)[None, :] < kept[:, None]
    for shift in (True, False):
        w = P.ppo_whiten(adv, kept, shift_mean=shift).cpu().numpy()
        np.testing.assert_allclose(w, O.whiten(adv, mask, shift), atol=2e-5, rtol=1e-5)
        assert (w[~mask] == 0).all()
    wd = P.ppo_whiten(rew, None, shift_mean=False).cpu().numpy()
    np.testing.assert_allclose(wd, O.whiten(rew, None, False), atol=2e-5, rtol=1e-5)


def test_degenerate_inputs(gpu):
    O = _oracle()
    x = np.full((4, 6), 2.5, np.float32)
    assert (P.ppo_whiten(x).cpu().numpy() == 0).all()                       # constant: zero, not NaN
    kept0 = np.zeros(4, np.int32)
    assert (P.ppo_whiten(x, kept0).cpu().numpy() == 0).all()                # nothing kept
    adv, ret = (t.cpu().numpy() for t in P.ppo_gae(x, x, kept0))
    assert (adv == 0).all() and (ret == 0).all()
    with pytest.raises(P.RlhfError):
        P.ppo_gae(x, x[:, :3], kept0)                                        # values shorter than N
    with pytest.raises(P.RlhfError):
        P.ppo_assemble_rewards(x, x, x, np.zeros((4, 6), np.int32), 1, EOS, PAD)  # [B, Lq+N] shapes wrong


def test_end_to_end_signals_from_a_gpu_rollout(gpu, tiny_cfg):
    """Rollout with one weight set, reference log-probs and reward-model values from two others, all
    on the GPU; the oracle recomputes the two scoring passes and the signals from the GPU's tokens."""
    from oracle import neox_oracle as NO
    O = _oracle()
    from synth.inputs import boost_eos
    cfg = tiny_cfg.with_(dtype="fp32")
    w_pol = boost_eos(cfg, make_weights(cfg, 11, variant="test"), 6.0)
    w_ref = make_weights(cfg, 12, variant="test")
    w_rm = make_weights(cfg, 13, variant="test")
    g = np.random.default_rng(5)
    B, Lq, N, T = 6, 12, 9, 0.7
    lens = g.integers(3, Lq + 1, B)
    q = g.integers(1, cfg.pad_id, (B, Lq)).astype(np.int32)
    mask = (np.arange(Lq)[None, :] >= (Lq - lens)[:, None]).astype(np.uint8)
    q[mask == 0] = cfg.pad_id
    pol, ref, rm = P.Policy(cfg, w_pol), P.Policy(cfg, w_ref), P.Policy(cfg, w_rm)
    toks, lps, lengths, omask = pol.rollout_generate(q, mask, 3, T, N, return_mask=True)
    ref_lp, _ = ref.score_sequences(toks, omask, T)
    _, rm_val = rm.score_sequences(toks, omask, T)
    _, pol_val = pol.score_sequences(toks, omask, T)
    rew, sc, kl, kept = P.ppo_assemble_rewards(lps, ref_lp, rm_val, toks, Lq, cfg.eos_id, cfg.pad_id, 0.05)
    adv, ret = P.ppo_gae(rew, pol_val, kept, 1.0, 0.95, value_offset=Lq - 1)
    wadv = P.ppo_whiten(adv, kept)
    toks_h, om_h = toks.cpu().numpy(), omask.cpu().numpy()
    assert (kept.cpu().numpy() == lengths.cpu().numpy()).all()
    o_ref_lp, _ = NO.score_sequences(NO.OracleModel(w_ref, cfg), toks_h, om_h, T)
    _, o_rm_val = NO.score_sequences(NO.OracleModel(w_rm, cfg), toks_h, om_h, T)
    _, o_pol_val = NO.score_sequences(NO.OracleModel(w_pol, cfg), toks_h, om_h, T)
    o_rew, o_sc, o_kl = O.assemble_rewards(lps.cpu().numpy(), o_ref_lp[:, Lq:], o_rm_val[:, Lq:], toks_h[:, Lq:],
                                           cfg.eos_id, cfg.pad_id, 0.05)
    np.testing.assert_allclose(rew.cpu().numpy(), o_rew, atol=1e-4)
    np.testing.assert_allclose(sc.cpu().numpy(), o_sc, atol=1e-4)
    o_adv, o_ret = O.gae(o_rew, o_pol_val[:, Lq - 1:Lq - 1 + N], lengths.cpu().numpy(), 1.0, 0.95)
    np.testing.assert_allclose(adv.cpu().numpy(), o_adv, atol=5e-4)
    np.testing.assert_allclose(ret.cpu().numpy(), o_ret, atol=5e-4)
    km = np.arange(N)[None, :] < lengths.cpu().numpy()[:, None]
    np.testing.assert_allclose(wadv.cpu().numpy(), O.whiten(o_adv, km), atol=5e-3)
    assert (sc.cpu().numpy() == -1.0).any() or (lengths.cpu().numpy() < N).all()
    for p_ in (pol, ref, rm):
        p_.close()
