"""Host-side per-step scalars of the paper's set-up (they cross the C ABI as plain arguments).

The EMA coefficient: 0.5 for the first 1k iterations, then a cosine decay to 0.01 (end of the
theory section).  The learning rate: linear warm-up over 3k iterations from 1e-7 to 3e-4, then
cosine decay to 3e-5 (experimental-setup appendix).  The paper does not say where the EMA cosine
ends; here it ends with training (`total_steps`).
"""
from __future__ import annotations

import math


def ema_lambda(t: int, total_steps: int, hold: int = 1000, start: float = 0.5, end: float = 0.01) -> float:
    """lambda_t for step t = 1, 2, ...: `start` up to step `hold`, cosine from there to `end` at `total_steps`."""
    if t <= hold or total_steps <= hold:
        return start
    x = min(1.0, (t - hold) / (total_steps - hold))
    return end + 0.5 * (start - end) * (1.0 + math.cos(math.pi * x))


def learning_rate(t: int, total_steps: int, warmup: int = 3000, lr_start: float = 1e-7,
                  lr_peak: float = 3e-4, lr_end: float = 3e-5) -> float:
    """eta_t: linear warm-up from lr_start (t = 0) to lr_peak (t = warmup), cosine to lr_end at total_steps."""
    if t <= warmup:
        return lr_start + (lr_peak - lr_start) * (t / warmup if warmup else 1.0)
    if total_steps <= warmup:
        return lr_peak
    x = min(1.0, (t - warmup) / (total_steps - warmup))
    return lr_end + 0.5 * (lr_peak - lr_end) * (1.0 + math.cos(math.pi * x))
