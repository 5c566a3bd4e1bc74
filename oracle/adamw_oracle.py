"""CPU oracle for the optimizer step of the PPO update: AdamW with a linear learning-rate schedule.
TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py may import this module.
It shares no code with the HIP library and never imports it.  Plain float64 numpy, one statement per
line of the algorithm.

What it computes.  The paper fixes the optimizer by name and two numbers [PPO hyperparameter table:
"AdamW (eps = 1e-5, lr = 3e-6)", "Scheduler: Linear"]; the algorithm itself is the published one
(Adam with decoupled weight decay), written out here in its usual order for update number t >= 1:

    p <- p * (1 - lr * weight_decay)
    m <- beta1 * m + (1 - beta1) * g
    v <- beta2 * v + (1 - beta2) * g * g
    p <- p - (lr / (1 - beta1^t)) * m / (sqrt(v) / sqrt(1 - beta2^t) + eps)

Readings where the paper is silent: beta1 = 0.9, beta2 = 0.999 and weight_decay = 0.01 (the defaults
of the library optimizer of that name); the linear schedule decays from the base rate at the first
update to zero after the last one with no warm-up, lr_k = lr * (1 - k / K) for update index
k = 0 .. K-1; gradients may carry a common scale factor (accumulation, clipping) applied before
everything else.

Pins (tests/test_oracle_adamw_pins.py): the library's own AdamW on the CPU in float64 over several
steps; the closed form of the first step (p - lr * g / (|g| + eps) without decay); zero gradients
leave pure decay; scale invariance of the first step; the schedule's end points.
"""
from __future__ import annotations

import math

import numpy as np

F64 = np.float64


def linear_lr(base_lr: float, update_index: int, total_updates: int) -> float:
    """Learning rate of update `update_index` (0-based) out of `total_updates`."""
    if total_updates <= 0:
        raise ValueError("total_updates must be positive")
    k = min(max(update_index, 0), total_updates)
    return base_lr * (1.0 - k / total_updates)


def adamw_step(param, grad, exp_avg, exp_avg_sq, step: int, lr: float = 3e-6, beta1: float = 0.9,
               beta2: float = 0.999, eps: float = 1e-5, weight_decay: float = 0.01, grad_scale: float = 1.0):
    """One update; `step` is 1 for the first.  Returns new (param, exp_avg, exp_avg_sq) as float64."""
    if step < 1:
        raise ValueError("step counts from 1")
    p = np.asarray(param, F64).copy()
    g = np.asarray(grad, F64) * grad_scale
    m = np.asarray(exp_avg, F64).copy()
    v = np.asarray(exp_avg_sq, F64).copy()
    p = p * (1.0 - lr * weight_decay)
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    bias1 = 1.0 - beta1 ** step
    bias2 = 1.0 - beta2 ** step
    denom = np.sqrt(v) / math.sqrt(bias2) + eps
    p = p - (lr / bias1) * m / denom
    return p, m, v
