"""CPU oracle for the per-table reuse profile.  TEST INFRASTRUCTURE ONLY.

Definition (the device-side stand-in for the offline hot-index profiling of paper Sec. 4.3): for
table t take the first `window` lookups of the batch that go to t; `dup_count` is how many of
them name a row that an earlier one of them already named, i.e. (lookups examined) - (distinct
row ids); the hint is "streaming" (1) when none was examined, or when fewer than
threshold_permille/1000 of them are repeats AND the share of repeats expected over all n_t
lookups the batch sends to the table, n_t * dup / examined^2 (the birthday estimate: dup repeats
among w draws put the rows in use at w^2 / (2 dup)), is below a quarter; else "default" (0).
Integer work: parity is bit-exact.

Pins (tests/test_oracle_pins.py): hand-worked cases typed in, the all-distinct and all-equal
closed forms, and the birthday-problem expectation for uniform draws.
"""
from __future__ import annotations

from typing import Tuple

import numpy as np


def profile_reuse(indices: np.ndarray, offsets: np.ndarray, T: int, B: int, window: int,
                  threshold_permille: int = 20) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    window = min(max(int(window), 1), 4096)
    dup = np.zeros(T, dtype=np.int32)
    used = np.zeros(T, dtype=np.int32)
    hints = np.zeros(T, dtype=np.uint8)
    for t in range(T):
        s, e = int(offsets[t * B]), int(offsets[(t + 1) * B])
        seg = [int(x) for x in indices[s:e][:window]]
        used[t] = len(seg)
        dup[t] = len(seg) - len(set(seg))
        few_in_window = int(dup[t]) * 1000 < threshold_permille * len(seg)
        few_in_batch = (e - s) * int(dup[t]) * 4 < len(seg) * len(seg)
        hints[t] = 1 if (not seg or (few_in_window and few_in_batch)) else 0
    return dup, used, hints
