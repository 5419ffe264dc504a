"""Host-side per-step scalars of the paper's set-up (they cross the C ABI as plain arguments).

The EMA coefficient: 0.5 for the first 1k iterations, then a cosine decay to 0.01 (end of the
theory section).  The learning rate: linear warm-up over 3k iterations from 1e-7 to 3e-4, then
cosine decay to 3e-5 (experimental-setup appendix).  The paper does not say where the EMA cosine
ends; here it ends with training (`total_steps`).  The heterogeneous set-up: relative device
speeds such as [2, 1, 2, 3] (appendix), the averaging interval proportional to the device speed.
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


def active_mask(t: int, speeds) -> int:
    """Which replicas make a local step in tick t = 1, 2, ... when replica i has relative device
    speed speeds[i] (positive integers).  A round lasts K = max(speeds) ticks and ends with an
    averaging step (use avg_interval = K); replica i makes speeds[i] steps per round, spread evenly
    over it, so the fastest replica steps in every tick.  Bit i of the result = replica i steps."""
    K = max(speeds)
    pos = (t - 1) % K
    mask = 0
    for i, s in enumerate(speeds):
        if not 1 <= s <= K:
            raise ValueError("speeds must be positive integers")
        if ((pos + 1) * s) // K > (pos * s) // K:
            mask |= 1 << i
    return mask
