"""score_responses (rescoring restricted to the response columns; PPO Details: the log-probabilities and values
PPO uses are those of the response positions) against the oracle's rescoring and against score_sequences: equal bit
for bit where the same kernels run (small shapes, fp32 check mode), and within a tenth of the parity bar where the
smaller row count of the restricted path selects other kernel variants (LayerNorm summation order)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from synth import ModelConfig, Workload, WORKLOADS, make_weights, make_random_responses

TOL = {"fp32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2403_17031_amd as P
    P.load_library()
    return P


def _batch(cfg, B, Lq, N, lo, hi, seed):
    g = np.random.default_rng(seed)
    lens = g.integers(lo, hi + 1, size=B)
    q = g.integers(1, min(cfg.pad_id, cfg.vocab), size=(B, Lq)).astype(np.int32)
    mask = (np.arange(Lq)[None, :] >= (Lq - lens)[:, None]).astype(np.uint8)
    q = np.where(mask == 1, q, cfg.pad_id).astype(np.int32)
    wl = Workload("t", cfg, B, Lq, N, lo, hi)
    tokens, fmask = make_random_responses(wl, q, mask, seed=seed + 1)
    return np.minimum(tokens, cfg.vocab - 1).astype(np.int32), fmask


def _expected(lp, val, first_col):
    elp, eval_ = lp.copy(), val.copy()
    elp[:, :first_col] = 0
    eval_[:, :max(first_col - 1, 0)] = 0
    return elp, eval_


def _check(pol, tokens, fmask, first_col, T, atol=0.0):
    lp, val = (x.cpu().numpy() for x in pol.score_sequences(tokens, fmask, T))
    rlp, rval = (x.cpu().numpy() for x in pol.score_responses(tokens, fmask, first_col, T))
    elp, eval_ = _expected(lp, val, first_col)
    assert ((rlp == 0) == (elp == 0)).all() and ((rval == 0) == (eval_ == 0)).all()
    assert np.abs(rlp - elp).max() <= atol, np.abs(rlp - elp).max()
    assert np.abs(rval - eval_).max() <= atol * max(1.0, float(np.abs(eval_).max())), np.abs(rval - eval_).max()
    return rlp, rval


@pytest.mark.parametrize("shape", ["160m", "2.8b"])
def test_selected_rows_path_equals_full_scoring_and_the_oracle(gpu, shape):
    """Enough response rows (24 sequences x 54 columns) for the restricted path to be taken: the LM head and the
    final layer's out-projection and MLP then run on the selected rows only.  Ragged queries (some shorter than the
    query window, one all-pad row, one sequence with a single response token), random right-padded responses."""
    from oracle import neox_oracle as O
    idx = {"160m": 2, "2.8b": 4}[shape]
    cfg = WORKLOADS[idx].model.with_(n_layers=2)
    w = make_weights(cfg, 500 + idx)
    B, Lq, N = 24, 120, 53
    tokens, fmask = _batch(cfg, B, Lq, N, 40, 120, seed=idx)
    fmask[3] = 0
    tokens[3] = cfg.pad_id
    fmask[5, Lq + 1:] = 0
    tokens[5, Lq + 1:] = cfg.pad_id
    pol = gpu.Policy(cfg, w)
    rlp, rval = _check(pol, tokens, fmask, Lq, 0.7, atol=2e-3)
    assert (rlp[:, :Lq] == 0).all() and (rval[:, :Lq - 1] == 0).all()
    rows = [0, 5, B - 1]
    olp, oval = O.score_sequences(O.OracleModel(w, cfg), tokens[rows], fmask[rows], 0.7)
    np.testing.assert_allclose(rlp[rows][:, Lq:], olp[:, Lq:], atol=TOL["bf16"], rtol=0)
    np.testing.assert_allclose(rval[rows][:, Lq - 1:], oval[:, Lq - 1:],
                               atol=TOL["bf16"] * max(1.0, float(np.abs(oval).max())), rtol=0)
    # other first columns: inside the queries (sequences that start after it), the last column, none
    for fc in (60, Lq + N - 1, Lq + N, 1, 0):
        _check(pol, tokens, fmask, fc, 0.7, atol=2e-3)
    # a second call with another batch size reuses nothing stale
    _check(pol, tokens[:11], fmask[:11], Lq, 1.0, atol=2e-3)
    pol.close()


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_small_shapes_take_the_full_path_with_the_same_outputs(gpu, dtype):
    """Few rows (the restricted path needs more than the few-rows kernels' limit) and the fp32 check mode: every row
    is computed and the columns before first_col are written as zeros."""
    cfg = ModelConfig(n_layers=2, d_model=64, n_heads=4, head_dim=16, rotary_dims=4, d_ff=256, vocab=96, eos_id=1,
                      pad_id=95, dtype=dtype)
    w = make_weights(cfg, 77, variant="test")
    tokens, fmask = _batch(cfg, 5, 20, 7, 3, 20, seed=70)
    pol = gpu.Policy(cfg, w)
    for fc in (20, 5, 0, 27):
        _check(pol, tokens, fmask, fc, 0.7)
    pol.close()


def test_score_responses_rejects_bad_arguments(gpu):
    cfg = ModelConfig(n_layers=1, d_model=64, n_heads=4, head_dim=16, rotary_dims=4, d_ff=256, vocab=96, eos_id=1,
                      pad_id=95, dtype="bf16")
    w = make_weights(cfg, 78, variant="test")
    tokens, fmask = _batch(cfg, 2, 8, 3, 2, 8, seed=71)
    pol = gpu.Policy(cfg, w)
    with pytest.raises(gpu.RlhfError):
        pol.score_responses(tokens, fmask, -1, 0.7)
    with pytest.raises(gpu.RlhfError):
        pol.score_responses(tokens, fmask, tokens.shape[1] + 1, 0.7)
    with pytest.raises(gpu.RlhfError):
        pol.score_responses(tokens, fmask, 8, 0.0)
    pol.close()
