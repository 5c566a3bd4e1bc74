"""GPU parity of the backward pass through a decoder layer's attention branch against
oracle/attn_branch_backward_oracle.py, through the C ABI.

Bars as for the MLP branch: fp32 check mode 1e-4 of each tensor's largest magnitude; bf16 mode (q, k, v, the
attention output, the upstream gradient and the attention gradients are fp16, each rounded to 2^-11 relative, and
the recomputed forward has the forward pass's own fp16 roundings) a relative Frobenius error of 5e-3 per tensor and a
largest element error of 2e-2 of the tensor's largest magnitude."""
import numpy as np
import pytest

import paper_2403_17031_amd as P
from synth import ModelConfig, make_weights

from bars import assert_signal_entries_close

pytestmark = pytest.mark.gpu

PAIRS = dict(d_x="d_x", d_ln1_g="d_ln_g", d_ln1_b="d_ln_b", d_w_qkv="d_w_qkv", d_b_qkv="d_b_qkv", d_w_o="d_w_o",
             d_b_o="d_b_o")


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    P.load_library()  # fails loudly when the HIP library has not been built
    return P


def _check(P, cfg, lens, seed, layer=0, scale=1.0):
    from oracle.attn_branch_backward_oracle import attn_branch_backward
    w = make_weights(cfg, 60 + seed, variant="test")
    g = np.random.default_rng(seed)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    x = (g.normal(0.0, 2.0, (T, cfg.d_model)) + g.normal(0.0, 0.5, (T, 1))).astype(np.float32)
    G = (g.normal(0.0, 1.0, (T, cfg.d_model)) * scale).astype(np.float32)
    pol = P.Policy(cfg, w)
    got = pol.attention_branch_backward(layer, x, G, cu)
    L = lambda n: w[f"layers.{layer}.{n}"]
    ref = attn_branch_backward(x, L("ln1_g"), L("ln1_b"), L("w_qkv"), L("b_qkv"), L("w_o"), L("b_o"), G, cu,
                               cfg.n_heads, cfg.head_dim, cfg.rotary_dims, cfg.rope_base, cfg.ln_eps)
    fp32 = cfg.dtype == "fp32"
    for n, rn in PAIRS.items():
        a = got[n].cpu().numpy().astype(np.float64)
        b = np.asarray(ref[rn], np.float64)
        assert a.shape == b.shape and np.isfinite(a).all(), n
        top, err = np.abs(b).max(), np.abs(a - b).max()
        assert err <= (1e-4 if fp32 else 2e-2) * top, (n, err, top)
        if not fp32:
            assert np.linalg.norm(a - b) <= 5e-3 * np.linalg.norm(b), (n, np.linalg.norm(a - b) / np.linalg.norm(b))
        assert_signal_entries_close(a, b, fp32, n)
    pol.close()


def _cfg(H, hd, r, dtype, layers=2):
    d = H * hd
    return ModelConfig(n_layers=layers, d_model=d, n_heads=H, head_dim=hd, rotary_dims=r, d_ff=2 * d, vocab=64,
                       dtype=dtype, pad_id=0, eos_id=1)


@pytest.mark.parametrize("lens,H,hd,r", [((1,), 1, 8, 4), ((5, 1, 7), 2, 8, 4), ((64, 65, 130), 3, 16, 8),
                                          ((200, 77), 2, 32, 0)])
def test_fp32_check_mode(gpu, lens, H, hd, r):
    _check(gpu, _cfg(H, hd, r, "fp32"), lens, seed=sum(lens), layer=1)


@pytest.mark.parametrize("lens,H,hd,r", [((3,), 1, 16, 4), ((5, 1, 7, 2), 2, 16, 8), ((64, 65, 1, 130, 63), 4, 32, 8),
                                          ((352, 565, 96), 8, 80, 20), ((129, 40, 700), 2, 64, 64), ((90,), 2, 128, 32)])
def test_bf16_mode(gpu, lens, H, hd, r):
    """Sequence lengths around the wave width and the benchmark's range, the head shapes of the model family (rotary
    on a quarter of the head), full rotary, row counts on both sides of the few-rows GEMM limit."""
    _check(gpu, _cfg(H, hd, r, "bf16"), lens, seed=sum(lens) + hd, layer=0, scale=8.0)


def test_bad_arguments_are_rejected(gpu):
    cfg = _cfg(2, 16, 4, "bf16")
    pol = gpu.Policy(cfg, make_weights(cfg, 65, variant="test"))
    x = np.zeros((8, 32), np.float32)
    with pytest.raises(gpu.RlhfError):
        pol.attention_branch_backward(2, x, x, [0, 8])          # layer out of range
    with pytest.raises(gpu.RlhfError):
        pol.attention_branch_backward(0, x, x, [0, 8], max_len=100000)
    pol.close()
