"""GPU parity of the packed causal attention backward against oracle/attention_backward_oracle.py, through the
C ABI.

Both sides start from the same stored inputs (float32, or float16 in the bf16 mode's activation type) and the kernels
compute in fp32, so what separates them is fp32 rounding of sums over at most a few thousand terms and, in fp16 mode,
the rounding of the outputs to fp16 (2^-11 relative): the bar is 1e-4 (fp32) and 2e-3 (fp16) of each tensor's largest
magnitude, with a relative Frobenius error of 1e-5 and 1e-3."""
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


def _run(P, lens, H, hd, dtype, seed, max_len=None):
    import torch
    from oracle.attention_backward_oracle import attention_backward
    r = np.random.default_rng(seed)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    tdt = torch.float32 if dtype == "fp32" else torch.float16
    host = [torch.from_numpy(r.normal(0, 1, (T, H * hd)).astype(np.float32)).to(tdt) for _ in range(4)]
    dev = [t.cuda() for t in host]
    got = P.attention_backward(*dev, cu, H, max_len=max_len)
    ref = attention_backward(*[t.double().numpy() for t in host], cu, H, hd)
    top_bar, fro_bar = (1e-4, 1e-5) if dtype == "fp32" else (2e-3, 1e-3)
    for name, a, b in zip(("dq", "dk", "dv"), got, ref):
        a = a.double().cpu().numpy()
        assert np.isfinite(a).all(), name
        assert np.abs(a - b).max() <= top_bar * np.abs(b).max(), (name, np.abs(a - b).max(), np.abs(b).max())
        assert np.linalg.norm(a - b) <= fro_bar * np.linalg.norm(b), (name, np.linalg.norm(a - b) / np.linalg.norm(b))
    return got


@pytest.mark.parametrize("lens,H,hd", [((1,), 1, 4), ((5, 1, 7), 2, 8), ((64, 65, 1, 130), 3, 16), ((300, 77), 2, 80)])
def test_fp32(gpu, lens, H, hd):
    _run(gpu, lens, H, hd, "fp32", seed=sum(lens))


@pytest.mark.parametrize("lens,H,hd", [((3,), 1, 8), ((5, 1, 7, 2), 2, 16), ((64, 65, 1, 130, 63), 3, 64),
                                        ((352, 565, 96, 211), 4, 80), ((129, 40), 2, 128), ((70,), 1, 256), ((300, 70, 129, 565), 2, 256)])
def test_fp16(gpu, lens, H, hd):
    """Sequence lengths around the 64-lane wave width and the benchmark's range, every head size of the model
    family."""
    _run(gpu, lens, H, hd, "fp16", seed=sum(lens) + hd)


def test_long_sequences_need_the_large_scratch(gpu):
    _run(gpu, (2021, 638), 1, 80, "fp16", seed=9)


def test_deterministic_and_max_len_is_only_an_upper_bound(gpu):
    a = _run(gpu, (100, 33), 2, 16, "fp16", seed=3)
    b = _run(gpu, (100, 33), 2, 16, "fp16", seed=3, max_len=500)
    for x, y in zip(a, b):
        assert bool((x == y).all())


def test_bad_arguments_are_rejected(gpu):
    import torch
    q = torch.zeros(8, 24, device="cuda", dtype=torch.float16)
    with pytest.raises(gpu.RlhfError):
        gpu.attention_backward(q, q, q, q, [0, 8], 2)             # head_dim 12 is not a multiple of 8
    q = torch.zeros(8, 32, device="cuda", dtype=torch.float16)
    with pytest.raises(gpu.RlhfError):
        gpu.attention_backward(q, q, q, q, [0, 8], 2, max_len=100000)
    with pytest.raises(gpu.RlhfError):
        gpu.attention_backward(q, q, q[:4], q, [0, 8], 2)
