"""CPU oracle for the per-table reuse profile.  TEST INFRASTRUCTURE ONLY.

Definition (the device-side stand-in for the offline hot-index profiling of paper Sec. 4.3): for
table t take the first `window` lookups of the batch that go to t; `dup_count` is how many of
them name a row that an earlier one of them already named, i.e. (lookups examined) - (distinct
row ids).  With w lookups examined, d repeats among them and n_t lookups sent to the table by
the whole batch, the hint is "streaming" (1) when
  - nothing was examined, or
  - w^2 * row_bytes * min(row_bytes, 128) > d * 2^36: the birthday estimate puts the rows in use
    at w^2 / (2 d); for rows of 128 bytes or more the condition says that these exceed 256 MiB
    (the memory-side cache), for narrower rows, 128 / row_bytes of which share a cache line, that
    they exceed 256 MiB times that number, or
  - n_t * d * 1000 * 128 < threshold_permille * w^2 * min(row_bytes, 128): the share of the
    table's lookups expected to find their 128-byte cache line already fetched is below the
    threshold (n_t * d / w^2 of them repeat a row, which for n_t <= window is d / n_t itself, and
    a line holds 128 / row_bytes rows); threshold_permille is capped at 1,000,000,
else "default" (0).  Integer work: parity is bit-exact.

Pins (tests/test_oracle_pins.py): hand-worked cases typed in, the all-distinct and all-equal
closed forms, and the birthday-problem expectation for uniform draws.
"""
from __future__ import annotations

from typing import Tuple

import numpy as np


MAX_WINDOW = 16384   # the largest window the interface examines


def profile_reuse(indices: np.ndarray, offsets: np.ndarray, T: int, B: int, window: int,
                  threshold_permille: int = 75, *, row_bytes: int
                  ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    window = int(window)
    if not 1 <= window <= MAX_WINDOW:
        raise ValueError(f"window must be in [1, {MAX_WINDOW}] (the interface clamps; this definition does not)")
    dup = np.zeros(T, dtype=np.int32)
    used = np.zeros(T, dtype=np.int32)
    hints = np.zeros(T, dtype=np.uint8)
    for t in range(T):
        s, e = int(offsets[t * B]), int(offsets[(t + 1) * B])
        seg = [int(x) for x in indices[s:e][:window]]
        w, n_t = len(seg), e - s
        d = w - len(set(seg))
        used[t], dup[t] = w, d
        beyond_cache = w * w * int(row_bytes) * min(int(row_bytes), 128) > d * (1 << 36)
        thr = min(int(threshold_permille), 1_000_000)
        few_repeats = n_t * d * 1000 * 128 < thr * w * w * min(int(row_bytes), 128)
        hints[t] = 1 if (w == 0 or beyond_cache or few_repeats) else 0
    return dup, used, hints
