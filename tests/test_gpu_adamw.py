"""GPU parity of the AdamW step against oracle/adamw_oracle.py, through the C ABI.  The kernel works in
fp32 on fp32 state; the oracle in float64 on the same fp32 inputs.  Bars: moments 2e-6 relative (the first moment relative to its two terms, which may cancel); the
parameters within 2 fp32 ulps of the oracle's plus the first-order effect of the moments' fp32 error on the update (a 3e-6 learning rate moves a weight of size 1 by 25 ulps,
so the update itself is resolved to a few per cent -- the price of fp32 master weights, not of the
kernel); the bf16 copy is exactly the nearest-even rounding of the kernel's own fp32 result."""
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


def _state(seed, n):
    g = np.random.default_rng(seed)
    f = np.float32
    p = g.normal(0, 0.5, n).astype(f)
    grad = (g.normal(0, 1, n) * 10.0 ** g.integers(-4, 1, n)).astype(f)
    m = (g.normal(0, 0.1, n)).astype(f)
    v = (g.random(n) * 0.01).astype(f)
    return p, grad, m, v


def _ulp(x):
    return np.spacing(np.abs(x).astype(np.float32)).astype(np.float64)


def _check(P, n, step, seed, **kw):
    import torch
    from oracle import adamw_oracle as O
    p, grad, m, v = _state(seed, n)
    if step == 1:
        m[:], v[:] = 0, 0
    tp, tg, tm, tv = (torch.from_numpy(a.copy()).cuda() for a in (p, grad, m, v))
    tb = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    P.adamw_step(tp, tg, tm, tv, step, param_bf16=tb, **kw)
    op, om, ov = O.adamw_step(p, grad, m, v, step, **kw)
    gp, gm, gv = tp.cpu().numpy(), tm.cpu().numpy(), tv.cpu().numpy()
    # m is a signed sum (its two terms may cancel): error relative to the terms, not to the result
    scale = float(kw.get("grad_scale", 1.0))
    assert (np.abs(gm - om) <= 2e-6 * np.abs(om) + 3e-7 * (np.abs(m) + np.abs(grad * scale))).all()
    np.testing.assert_allclose(gv, ov, rtol=2e-6, atol=1e-30)
    # 2 ulps of the result plus what the fp32 error of the moments does to the update term
    # step_size * m / denom (first order: err(m) / denom + |m| * err(denom) / denom^2)
    lr, b1, b2 = kw.get("lr", 3e-6), kw.get("beta1", 0.9), kw.get("beta2", 0.999)
    denom = np.sqrt(ov) / np.sqrt(1 - b2 ** step) + kw.get("eps", 1e-5)
    err_m = 2e-6 * np.abs(om) + 3e-7 * (np.abs(m) + np.abs(grad * scale))
    tol = 2 * _ulp(op) + lr / (1 - b1 ** step) * (err_m + 2e-6 * np.abs(om)) / denom + 1e-30
    assert (np.abs(gp.astype(np.float64) - op) <= tol).all()
    assert (tg.cpu().numpy() == grad).all()                       # gradients are read-only
    assert torch.equal(tb, tp.to(torch.bfloat16))                 # nearest-even rounding of the fp32 result
    return gp, op


@pytest.mark.parametrize("n", [1, 3, 4, 1023, 4096, (1 << 20) + 3, 5_000_001])
def test_one_step_matches_the_oracle(gpu, n):
    _check(gpu, n, 1, n)
    _check(gpu, n, 7, n + 1)
    _check(gpu, n, 4000, n + 2, lr=1e-2, weight_decay=0.0)
    _check(gpu, n, 2, n + 3, lr=1e-3, beta1=0.8, beta2=0.95, eps=1e-8, weight_decay=0.1, grad_scale=0.125)


def test_trajectory_of_several_updates_with_the_linear_schedule(gpu):
    """Ten updates at a learning rate large enough to move the weights visibly; state carried on the GPU
    in fp32 and in the oracle in float64."""
    import torch
    from oracle import adamw_oracle as O
    n, K, base = 10007, 10, 1e-2
    p, _, _, _ = _state(5, n)
    tp = torch.from_numpy(p.copy()).cuda()
    tm, tv = torch.zeros_like(tp), torch.zeros_like(tp)
    op, om, ov = p.astype(np.float64), np.zeros(n), np.zeros(n)
    g = np.random.default_rng(6)
    for k in range(K):
        grad = g.normal(0, 1, n).astype(np.float32)
        lr = gpu.linear_lr(base, k, K)
        assert lr == O.linear_lr(base, k, K)
        gpu.adamw_step(tp, torch.from_numpy(grad).cuda(), tm, tv, k + 1, lr=lr)
        op, om, ov = O.adamw_step(op, grad, om, ov, k + 1, lr=lr)
    np.testing.assert_allclose(tp.cpu().numpy(), op, rtol=0, atol=2e-6)
    np.testing.assert_allclose(tm.cpu().numpy(), om, rtol=1e-5, atol=5e-7)   # a sum of ten signed O(0.1) terms
    assert np.abs(tp.cpu().numpy() - p).max() > 1e-2   # the weights did move


def test_empty_and_bad_arguments(gpu):
    import torch
    z = torch.zeros(0, dtype=torch.float32, device="cuda")
    gpu.adamw_step(z, z.clone(), z.clone(), z.clone(), 1)   # nothing to do, no error
    a = torch.zeros(8, dtype=torch.float32, device="cuda")
    with pytest.raises(gpu.RlhfError):
        gpu.adamw_step(a, a.clone(), a.clone(), a.clone(), 0)
    with pytest.raises(gpu.RlhfError):
        gpu.adamw_step(a, a.clone(), a.clone(), a.clone(), 1, beta1=1.0)
    with pytest.raises(gpu.RlhfError):
        gpu.adamw_step(a, a.clone()[:4], a.clone(), a.clone(), 1)
    with pytest.raises(gpu.RlhfError):
        gpu.adamw_step(a, a.clone(), a.clone(), a.clone(), 1, eps=0.0)
