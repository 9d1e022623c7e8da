"""Byte and throughput accounting for the embedding stage.

The paper counts the data an embedding table processes as BS x (average lookups per sample) x
ED x precision (Sec. 3.1: 2048 x 150 x 128 x 4 B per table).  `gathered_bytes` is that figure
for a whole multi-table batch; `algorithmic_bytes` adds the index, offset and output traffic the
operation cannot avoid.
"""
from __future__ import annotations

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth, GB/s (decimal)


def gathered_bytes(num_lookups: int, dim: int, elem_bytes: int, row_bytes: int = 0) -> int:
    """Bytes of table rows gathered: one row of dim*elem_bytes per lookup (`row_bytes`, when given,
    overrides the product: quantised rows carry 8 bytes of scale and bias)."""
    return int(num_lookups) * (int(row_bytes) if row_bytes else int(dim) * int(elem_bytes))


def algorithmic_bytes(num_lookups: int, num_tables: int, batch: int, dim: int, elem_bytes: int,
                      weighted: bool = False, row_bytes: int = 0) -> int:
    """Gathered rows + int64 indices + int64 CSR offsets + fp32 output (+ fp32 weights)."""
    total = gathered_bytes(num_lookups, dim, elem_bytes, row_bytes)
    total += 8 * int(num_lookups)
    total += 8 * (int(num_tables) * int(batch) + 1)
    total += 4 * int(batch) * int(num_tables) * int(dim)
    if weighted:
        total += 4 * int(num_lookups)
    return total


def lookups_per_second(num_lookups: int, seconds: float) -> float:
    return num_lookups / seconds


def effective_gbps(nbytes: int, seconds: float) -> float:
    return nbytes / seconds / 1e9
