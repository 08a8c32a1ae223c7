"""Choosing where a long-lived KV cache sits in device memory.

The time of the compression pass depends on where the driver places its buffers physically: the same
kernel on the same bytes runs at one of a few distinct, individually stable speeds from one allocation
of the working set to the next (on a 128K-token, batch-4 cache: 14.1 to 16.4 ms).  A server allocates
its cache once and keeps it, so it can afford to try a few allocations when it starts and keep the
fastest.  `pick` does that for any caller: it knows nothing about the pass, only how to ask for a
working set, how to time it and how to give memory back.
"""
from __future__ import annotations

from typing import Callable, List, Tuple, TypeVar

T = TypeVar("T")


def pick(build: Callable[[], T], time_ms: Callable[[T], float], trials: int = 6,
         release: Callable[[], None] = lambda: None) -> Tuple[T, List[float]]:
    """Builds the working set `trials` times (at least once), times each with `time_ms` and returns the
    fastest one together with every trial's time, first allocation first.  At most two sets exist at a
    time: the best so far and the candidate; `release` is called after a set has been dropped (for
    torch: torch.cuda.empty_cache, so that the next candidate is a fresh allocation)."""
    times: List[float] = []
    best = None
    for _ in range(max(1, trials)):
        cand = build()
        ms = float(time_ms(cand))
        times.append(ms)
        if best is None or ms < best[0]:
            best = (ms, cand)
        del cand
        release()
    kept = best[1]
    del best
    release()
    return kept, times
