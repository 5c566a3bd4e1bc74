"""GPU parity of the backward pass through the output heads (final LayerNorm, LM head with temperature,
value head) against oracle/head_backward_oracle.py, through the C ABI.

Bars.  fp32 check mode: every product accumulates in fp32 over at most a few thousand terms, so each output
agrees to 1e-4 of its tensor's largest magnitude.  bf16 mode: h and dL/dz enter the two gradient products rounded
to fp16 (relative error 2^-11 each), the logits come from fp16 h; over n accumulated terms the roundings are
independent, which puts the error of a sum at about 2^-11 * sqrt(2) of the norm of its terms: the bar is a relative
Frobenius error of 5e-3 per tensor and a largest element error of 2e-2 of the tensor's largest magnitude (the
bf16-mode bar of the forward pass, applied relative to scale since gradients have no natural unit)."""
import numpy as np
import pytest

import paper_2403_17031_amd as P
from synth import ModelConfig, make_weights

from bars import assert_signal_entries_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    P.load_library()  # fails loudly when the HIP library has not been built
    return P


def _inputs(cfg, T, seed, frac_no_target=0.2):
    g = np.random.default_rng(seed)
    x = (g.normal(0.0, 2.0, (T, cfg.d_model)) + g.normal(0.0, 0.5, (T, 1))).astype(np.float32)
    y = g.integers(0, cfg.vocab, T).astype(np.int32)
    y[g.random(T) < frac_no_target] = -1
    gl = (g.normal(0.0, 1.0, T) / T).astype(np.float32)      # the scale of a mean over T tokens
    gv = (g.normal(0.0, 0.1, T) / T).astype(np.float32)
    return x, y, gl, gv


def _check(P, cfg, w, T, seed, scale, value_head=True, frac_no_target=0.2):
    from oracle.head_backward_oracle import head_backward
    if not value_head:
        w = {k: v for k, v in w.items() if k not in ("value_w", "value_b")}
    x, y, gl, gv = _inputs(cfg, T, seed, frac_no_target)
    pol = P.Policy(cfg, w)
    got = pol.head_backward(x, y, gl, gv if value_head else None, 0.7, grad_scale=scale)
    zero_w = np.zeros(cfg.d_model)
    ref = head_backward(x, w["lnf_g"], w["lnf_b"], w["embed_out"], w["value_w"] if value_head else zero_w, y, gl,
                        gv if value_head else np.zeros(T), 0.7, ln_eps=cfg.ln_eps)
    names = ["d_x", "d_lnf_g", "d_lnf_b", "d_embed_out"] + (["d_value_w", "d_value_b"] if value_head else [])
    fp32 = cfg.dtype == "fp32"
    for n in names:
        a = got[n].cpu().numpy().astype(np.float64) / scale
        b = np.asarray(ref[n], np.float64).reshape(a.shape)
        top = np.abs(b).max()
        err = np.abs(a - b).max()
        assert np.isfinite(a).all(), n
        if top == 0.0:
            assert err == 0.0, n
            continue
        assert err <= (1e-4 if fp32 else 2e-2) * top, (n, err, top)
        if not fp32:
            assert np.linalg.norm(a - b) <= 5e-3 * np.linalg.norm(b), (n, np.linalg.norm(a - b) / np.linalg.norm(b))
        assert_signal_entries_close(a, b, fp32, n)
    pol.close()
    return got, ref


@pytest.mark.parametrize("T,d,V", [(1, 16, 24), (37, 64, 517), (700, 48, 131)])
def test_fp32_check_mode(gpu, T, d, V):
    cfg = ModelConfig(n_layers=0, d_model=d, n_heads=1, head_dim=d, rotary_dims=0, d_ff=d, vocab=V, dtype="fp32",
                      pad_id=0, eos_id=1)
    _check(gpu, cfg, make_weights(cfg, 11, variant="test"), T, seed=T, scale=1.0)


@pytest.mark.parametrize("T,d,V", [(5, 64, 520), (300, 128, 1000), (700, 128, 517), (1500, 256, 2048)])
def test_bf16_mode(gpu, T, d, V):
    """Few rows and many (the weight-gradient product's K is the row count, padded to 128), a vocabulary that is
    not a multiple of 8 (padded columns of the input-gradient product), widths the large-tile GEMM takes."""
    cfg = ModelConfig(n_layers=0, d_model=d, n_heads=1, head_dim=d, rotary_dims=0, d_ff=d, vocab=V, dtype="bf16",
                      pad_id=0, eos_id=1)
    _check(gpu, cfg, make_weights(cfg, 12, variant="test"), T, seed=T, scale=float(T) * 64.0)


def test_more_rows_than_one_chunk(gpu):
    """16,384 rows of logits exist at a time: the LM-head gradient accumulates over chunks, the last one ragged."""
    cfg = ModelConfig(n_layers=0, d_model=64, n_heads=1, head_dim=64, rotary_dims=0, d_ff=64, vocab=520,
                      dtype="bf16", pad_id=0, eos_id=1)
    T = 16384 + 333
    _check(gpu, cfg, make_weights(cfg, 13, variant="test"), T, seed=5, scale=T * 64.0)


def test_without_value_head_and_without_targets(gpu):
    cfg = ModelConfig(n_layers=0, d_model=64, n_heads=1, head_dim=64, rotary_dims=0, d_ff=64, vocab=520,
                      dtype="bf16", pad_id=0, eos_id=1)
    w = make_weights(cfg, 14, variant="test")
    _check(gpu, cfg, w, 90, seed=6, scale=90.0 * 64.0, value_head=False)
    got, _ = _check(gpu, cfg, w, 90, seed=7, scale=90.0 * 64.0, frac_no_target=1.1)   # no row has a target
    assert float(got["d_embed_out"].abs().max()) == 0.0


def test_grad_scale_is_linear_and_results_are_deterministic(gpu):
    cfg = ModelConfig(n_layers=0, d_model=128, n_heads=1, head_dim=128, rotary_dims=0, d_ff=128, vocab=1000,
                      dtype="fp32", pad_id=0, eos_id=1)
    w = make_weights(cfg, 15, variant="test")
    x, y, gl, gv = _inputs(cfg, 200, 8)
    pol = gpu.Policy(cfg, w)
    a = pol.head_backward(x, y, gl, gv, 0.7, grad_scale=1.0)
    a = {k: v.clone() for k, v in a.items()}
    b = pol.head_backward(x, y, gl, gv, 0.7, grad_scale=4.0)     # a power of two: exact in binary arithmetic
    c = pol.head_backward(x, y, gl, gv, 0.7, grad_scale=1.0)
    for k in a:
        assert bool((b[k] == 4.0 * a[k]).all()), k
        assert bool((c[k] == a[k]).all()), k
    pol.close()


def test_bad_arguments_are_rejected(gpu):
    cfg = ModelConfig(n_layers=0, d_model=64, n_heads=1, head_dim=64, rotary_dims=0, d_ff=64, vocab=520,
                      dtype="bf16", pad_id=0, eos_id=1)
    pol = gpu.Policy(cfg, make_weights(cfg, 16, variant="test"))
    x, y, gl, gv = _inputs(cfg, 10, 9)
    with pytest.raises(gpu.RlhfError):
        pol.head_backward(x, y, gl, gv, 0.0)
    with pytest.raises(gpu.RlhfError):
        pol.head_backward(x, y, gl, gv, 0.7, grad_scale=float("inf"))
    with pytest.raises(gpu.RlhfError):
        pol.head_backward(x[:, :32], y, gl, gv, 0.7)
    pol.close()
