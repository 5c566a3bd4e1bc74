"""The allocation-free entry point rlhf_attention_backward_noalloc against rlhf_attention_backward (caller
scratch), through the C ABI: same kernels, so the outputs must be bit-identical.  Two calls in a row on the
library's fixed scratch array, the second with a smaller input, then a size beyond the array's limit."""
import numpy as np
import pytest

import paper_2403_17031_amd as P

pytestmark = pytest.mark.gpu


def _inputs(lens, H, hd, dtype, seed):
    import torch
    r = np.random.default_rng(seed)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    ts = [torch.from_numpy(r.normal(0, 1, (T, H * hd)).astype(np.float32)).to(dtype).cuda() for _ in range(4)]
    return ts, cu


@pytest.mark.parametrize("dtype_name,hd", [("float16", 80), ("float32", 16)])
def test_noalloc_matches_caller_scratch_twice_in_a_row(dtype_name, hd):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    P.load_library()
    dtype = getattr(torch, dtype_name)
    H = 4
    for call, lens in enumerate([(352, 565, 96, 211, 1), (130, 7)]):  # the second call is smaller
        ts, cu = _inputs(lens, H, hd, dtype, seed=11 + call)
        ref = P.attention_backward(*ts, cu, H)
        torch.cuda.synchronize()
        # outputs allocated by the test beforehand: the call itself allocates nothing
        out = tuple(torch.full_like(ts[0], float("nan")) for _ in range(3))
        cu_dev = torch.from_numpy(cu).cuda()
        torch.cuda.synchronize()
        # free device memory as the driver reports it (this sees any hipMalloc, the library's included); the
        # first call on a device may still load code, so the comparison is made on the second
        free_before = torch.cuda.mem_get_info()[0]
        got = P.attention_backward(*ts, cu_dev, H, max_len=max(lens), noalloc=True, out=out)
        torch.cuda.synchronize()
        if call == 1:
            assert torch.cuda.mem_get_info()[0] >= free_before
        for name, a, b in zip(("dq", "dk", "dv"), got, ref):
            assert bool(torch.isfinite(a).all()), (call, name)
            assert bool((a == b).all()), (call, name, float((a.float() - b.float()).abs().max()))


def test_noalloc_rejects_sizes_beyond_its_scratch():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    P.load_library()
    H, hd, T = 64, 8, 16385  # T * H = 1,048,640 > 1,048,576
    q = torch.zeros(T, H * hd, device="cuda", dtype=torch.float16)
    with pytest.raises(P.RlhfError, match="static scratch"):
        P.attention_backward(q, q, q, q, [0, T], H, noalloc=True, out=(q, q, q))
