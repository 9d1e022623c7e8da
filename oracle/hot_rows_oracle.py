"""CPU oracle for the hot-row profile.  TEST INFRASTRUCTURE ONLY: nothing outside tests/,
__graft_entry__.smoke() and bench.py's cpu_baseline leg may import it.

Definition (the profiling step of paper Sec. 4.3, which finds "the top 60K hot indices" of every
table offline; the paper does not say how ties are ordered or which sample is profiled, so: the
sample is the table's first `window` lookups of one batch, and ties go to the smaller row id).
For table t take the first `window` lookups of the batch that go to t, drop ids outside
[0, 2^40 - 1), count how often each distinct row id occurs, and order the distinct ids by
(count descending, id ascending).  The first k of that order are the table's hot rows:
num_hot[t] = min(k, distinct ids), hot_ids[t, r] / hot_counts[t, r] the r-th id and its count for
r < num_hot[t], and -1 / 0 beyond.  Integer work: parity with the device is bit-exact.

Pins (tests/test_oracle_pins.py): hand-worked cases typed in, closed forms (all distinct, one
item, id i occurring i + 1 times), ties, the window, and collections.Counter as a second route.
"""
from __future__ import annotations

from typing import Tuple

import numpy as np

ID_LIMIT = (1 << 40) - 1


def profile_hot_rows(indices: np.ndarray, offsets: np.ndarray, T: int, B: int, window: int,
                     k: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    hot_ids = np.full((T, k), -1, dtype=np.int64)
    hot_counts = np.zeros((T, k), dtype=np.int32)
    num_hot = np.zeros(T, dtype=np.int32)
    for t in range(T):
        s, e = int(offsets[t * B]), int(offsets[(t + 1) * B])
        seg = np.asarray(indices[s:e][:window], dtype=np.int64)
        seg = seg[(seg >= 0) & (seg < ID_LIMIT)]
        ids, counts = np.unique(seg, return_counts=True)
        order = sorted(range(len(ids)), key=lambda i: (-int(counts[i]), int(ids[i])))[:k]
        num_hot[t] = len(order)
        for r, i in enumerate(order):
            hot_ids[t, r] = ids[i]
            hot_counts[t, r] = counts[i]
    return hot_ids, hot_counts, num_hot
