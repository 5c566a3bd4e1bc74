"""GPU parity of the backward pass through a decoder layer's MLP branch against oracle/mlp_backward_oracle.py,
through the C ABI.

Bars as for the output heads: fp32 check mode 1e-4 of each tensor's largest magnitude; bf16 mode (the upstream
gradient, gelu(u) and dL/du are fp16 operands of the gradient products, each rounded to 2^-11 relative, and the
recomputed forward has the forward pass's own fp16 roundings) a relative Frobenius error of 5e-3 per tensor and a
largest element error of 2e-2 of the tensor's largest magnitude."""
import numpy as np
import pytest

import paper_2403_17031_amd as P
from synth import ModelConfig, make_weights

from bars import assert_signal_entries_close

pytestmark = pytest.mark.gpu

NAMES = ("d_x", "d_ln2_g", "d_ln2_b", "d_w_fc1", "d_b_fc1", "d_w_fc2", "d_b_fc2")


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    P.load_library()  # fails loudly when the HIP library has not been built
    return P


def _check(P, cfg, T, seed, layer=0, scale=1.0):
    from oracle.mlp_backward_oracle import mlp_backward
    w = make_weights(cfg, 40 + seed, variant="test")
    g = np.random.default_rng(seed)
    x = (g.normal(0.0, 2.0, (T, cfg.d_model)) + g.normal(0.0, 0.5, (T, 1))).astype(np.float32)
    G = (g.normal(0.0, 1.0, (T, cfg.d_model)) * scale).astype(np.float32)
    G[T // 2] = 0.0
    pol = P.Policy(cfg, w)
    got = pol.mlp_backward(layer, x, G)
    L = lambda n: w[f"layers.{layer}.{n}"]
    ref = mlp_backward(x, L("ln2_g"), L("ln2_b"), L("w_fc1"), L("b_fc1"), L("w_fc2"), L("b_fc2"), G, cfg.ln_eps)
    ref = dict(d_x=ref["d_x"], d_ln2_g=ref["d_ln_g"], d_ln2_b=ref["d_ln_b"], d_w_fc1=ref["d_w_fc1"],
               d_b_fc1=ref["d_b_fc1"], d_w_fc2=ref["d_w_fc2"], d_b_fc2=ref["d_b_fc2"])
    fp32 = cfg.dtype == "fp32"
    for n in NAMES:
        a = got[n].cpu().numpy().astype(np.float64)
        b = np.asarray(ref[n], np.float64)
        assert a.shape == b.shape and np.isfinite(a).all(), n
        top, err = np.abs(b).max(), np.abs(a - b).max()
        assert err <= (1e-4 if fp32 else 2e-2) * top, (n, err, top)
        if not fp32:
            assert np.linalg.norm(a - b) <= 5e-3 * np.linalg.norm(b), (n, np.linalg.norm(a - b) / np.linalg.norm(b))
        assert_signal_entries_close(a, b, fp32, n)
    pol.close()
    return got


def _cfg(d, F, dtype, layers=2):
    hd = d if d <= 128 else 64
    return ModelConfig(n_layers=layers, d_model=d, n_heads=d // hd, head_dim=hd, rotary_dims=0, d_ff=F, vocab=64,
                       dtype=dtype, pad_id=0, eos_id=1)


@pytest.mark.parametrize("T,d,F", [(1, 16, 24), (37, 64, 160), (700, 48, 96)])
def test_fp32_check_mode(gpu, T, d, F):
    _check(gpu, _cfg(d, F, "fp32"), T, seed=T, layer=1)


@pytest.mark.parametrize("T,d,F", [(5, 64, 256), (300, 128, 512), (700, 128, 328), (1500, 256, 1024), (2100, 384, 768), (1333, 640, 1544)])
def test_bf16_mode(gpu, T, d, F):
    """Few rows and many (the weight-gradient products' K is the row count, padded to 128), widths the large-tile
    GEMM takes and widths it does not, a row count that is not a multiple of 4 (scalar transposes), widths beyond 512
    that are no multiple of the 256-wide tile (the weight-gradient products then read K-major operands)."""
    _check(gpu, _cfg(d, F, "bf16"), T, seed=T, layer=0, scale=8.0)


def test_linear_in_the_upstream_gradient_and_deterministic(gpu):
    cfg = _cfg(128, 512, "fp32")
    w = make_weights(cfg, 44, variant="test")
    g = np.random.default_rng(2)
    x = g.normal(0, 2, (200, 128)).astype(np.float32)
    G = g.normal(0, 1, (200, 128)).astype(np.float32)
    pol = gpu.Policy(cfg, w)
    a = {k: v.clone() for k, v in pol.mlp_backward(0, x, G).items()}
    b = pol.mlp_backward(0, x, 4.0 * G)
    for k in a:
        assert bool((b[k] == 4.0 * a[k]).all()), k
    c = pol.mlp_backward(0, x, G)
    for k in a:
        assert bool((c[k] == a[k]).all()), k
    pol.close()


def test_bad_arguments_are_rejected(gpu):
    cfg = _cfg(64, 128, "bf16")
    pol = gpu.Policy(cfg, make_weights(cfg, 45, variant="test"))
    x = np.zeros((4, 64), np.float32)
    with pytest.raises(gpu.RlhfError):
        pol.mlp_backward(2, x, x)          # layer out of range
    with pytest.raises(gpu.RlhfError):
        pol.mlp_backward(0, x, x[:, :32])
    pol.close()
