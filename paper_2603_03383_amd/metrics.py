"""The paper's evaluation metrics (Section 4.1, "Evaluation Metrics").

  AC        average number of tokens verified and accepted per decoding step
  Overhead  Time_spec / Time_AR: one speculative step (heads + tree verification + acceptance + compaction)
            relative to one ordinary autoregressive step
  Speedup   AC / Overhead: the end-to-end gain over autoregressive decoding

Pure arithmetic on measured times; nothing here touches the GPU.
"""
from __future__ import annotations


def overhead(time_spec: float, time_ar: float) -> float:
    if time_spec <= 0 or time_ar <= 0:
        raise ValueError("times must be positive")
    return time_spec / time_ar


def speedup(ac: float, overhead_ratio: float) -> float:
    if ac < 1 or overhead_ratio <= 0:
        raise ValueError("AC counts the root, so it is at least 1; overhead must be positive")
    return ac / overhead_ratio


def break_even_ac(overhead_ratio: float) -> float:
    """The AC above which speculative decoding is faster than autoregressive decoding."""
    return overhead_ratio
