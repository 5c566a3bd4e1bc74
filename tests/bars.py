"""Shared bars of the backward-pass parity tests (helpers only; collected by no test run)."""
import numpy as np

# Element-wise relative bar over the entries that carry signal: every entry whose reference magnitude is at least
# 1 % of the tensor's largest must itself be right to REL (worst entry) and REL_P99 (99th percentile).  The
# max-relative-to-the-tensor and Frobenius bars beside it bound the small entries in absolute terms only.
# fp32 check mode: fp32 summation over at most a few thousand terms.  bf16 mode: operands rounded to fp16
# (2^-11 relative each) enter sums with cancellation, so an entry at 1 % of the maximum sees the absolute error of
# the large ones: measured worst entries are a few per cent.
REL = {True: 2e-3, False: 0.25}
REL_P99 = {True: 5e-4, False: 0.05}


def assert_signal_entries_close(a, b, fp32, name=""):
    a, b = np.asarray(a, np.float64).ravel(), np.asarray(b, np.float64).ravel()
    top = np.abs(b).max() if b.size else 0.0
    if top == 0.0:
        return 0.0
    sel = np.abs(b) >= 1e-2 * top
    rel = np.abs(a[sel] - b[sel]) / np.abs(b[sel])
    worst, p99 = float(rel.max()), float(np.quantile(rel, 0.99))
    assert worst <= REL[fp32], (name, "worst relative error of an entry above 1% of the maximum", worst)
    assert p99 <= REL_P99[fp32], (name, "99th percentile of the relative error", p99)
    return worst
