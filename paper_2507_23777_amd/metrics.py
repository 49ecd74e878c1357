"""Accounting of the paper's speed metrics (Sec. 5.1 "Metrics")."""
from __future__ import annotations


def step_compression_ratio(n_accepted_per_step) -> float:
    """SCR = generated-and-accepted tokens / decoding steps."""
    steps = len(n_accepted_per_step)
    if steps == 0:
        raise ValueError("no decoding steps")
    return float(sum(int(a) for a in n_accepted_per_step)) / steps


def speedup(scr: float, step_latency: float, plain_step_latency: float) -> float:
    """Speedup over next-token decoding: tokens per unit time of the speculative
    loop (SCR / step latency) over that of the plain loop (1 / plain latency)."""
    if step_latency <= 0 or plain_step_latency <= 0:
        raise ValueError("latencies must be positive")
    return scr * plain_step_latency / step_latency
