"""Exact integer definition of the adaptive resource manager's choice (TEST INFRASTRUCTURE ONLY).

Section 4.5.3 of the paper: when the decode load is light both phases are given every
compute unit (over-allocation); under heavier load an offline profile gives, per decode
load, the smallest number of compute units with which decode still meets its inter-token
latency objective, decode is given exactly that many and prefill the remainder.  When no
prefill is in flight decode may take all compute units.

Readings where the paper is silent:
  * the profile is keyed by (decode batch size, total cached tokens), each rounded UP to the
    next profiled bucket (loads beyond the last bucket use the last bucket);
  * "light" means: the profiled latency under over-allocation meets the objective;
  * when no profiled split meets the objective decode gets the split with the lowest profiled
    latency (fewest compute units on ties);
  * no hysteresis.
"""
from __future__ import annotations

import dataclasses
from typing import List, Sequence, Tuple

TOTAL_CUS = 256


@dataclasses.dataclass
class Profile:
    batch_edges: Sequence[int]        # ascending decode batch sizes that were profiled
    ctx_edges: Sequence[int]          # ascending totals of cached tokens that were profiled
    decode_cus: Sequence[int]         # ascending decode CU counts of the distinct splits
    lat_distinct_us: List[List[List[int]]]  # [batch][ctx][split] decode step latency, co-run
    lat_over_us: List[List[int]]      # [batch][ctx] decode step latency under 256/256


def _bucket(edges: Sequence[int], value: int) -> int:
    for i, e in enumerate(edges):
        if value <= e:
            return i
    return len(edges) - 1


def choose_split(batch: int, sum_ctx: int, prefill_pending: bool, prof: Profile,
                 slo_us: int) -> Tuple[int, int]:
    """Returns (prefill_cus, decode_cus)."""
    if not prefill_pending:
        return 0, TOTAL_CUS
    if batch <= 0:
        return TOTAL_CUS, 0
    b = _bucket(prof.batch_edges, batch)
    c = _bucket(prof.ctx_edges, sum_ctx)
    if prof.lat_over_us[b][c] <= slo_us:
        return TOTAL_CUS, TOTAL_CUS
    row = prof.lat_distinct_us[b][c]
    for s, cus in enumerate(prof.decode_cus):
        if row[s] <= slo_us:
            return TOTAL_CUS - cus, cus
    best = 0
    for s in range(1, len(row)):
        if row[s] < row[best]:
            best = s
    cus = prof.decode_cus[best]
    return TOTAL_CUS - cus, cus
