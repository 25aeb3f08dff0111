"""CPU model of per-kernel right-sizing (LithOS Section 4.5, Section 7.2).

TEST INFRASTRUCTURE ONLY.  Plain Python floats (fp64).

Two selection rules:

* the sweep rule: from measured latencies t(c) at a list of CU counts, take
  the smallest c whose latency is within (1+delta) of the full-GPU latency;
* the paper's two-point model: fit l = m/t + b through the latencies at one
  unit and at all T units, then take the smallest t with l(t) <= k*l(T).

plus the occupancy bound of 'Filtering Outliers' and the capacity-saving
statistic of Section 7.2 (time-weighted mean units before vs after).
"""
from __future__ import annotations

import math
from typing import Dict, List, Sequence, Tuple


def select_from_sweep(cus: Sequence[int], lat: Sequence[float], delta: float) -> int:
    """Smallest CU count whose latency is <= (1+delta) * latency at max(cus).

    The curve need not be monotone: the smallest qualifying point wins.
    """
    if len(cus) != len(lat) or not cus:
        raise ValueError("cus and lat must be same-length, non-empty")
    full = lat[max(range(len(cus)), key=lambda i: cus[i])]
    ok = [c for c, t in zip(cus, lat) if t <= (1.0 + delta) * full]
    return min(ok)


def fit_two_point(l1: float, lT: float, T: int) -> Tuple[float, float]:
    """(m, b) of l = m/t + b passing through (1, l1) and (T, lT)."""
    if T <= 1:
        raise ValueError("need T > 1")
    m = (l1 - lT) * T / (T - 1)
    b = l1 - m
    return m, b


def model_latency(m: float, b: float, t: float) -> float:
    return m / t + b


def min_units_for_slip(m: float, b: float, T: int, k: float) -> int:
    """Smallest integer t in [1,T] with m/t + b <= k * (m/T + b).

    Found by direct search over t (the definition), not by a closed form.
    """
    target = k * model_latency(m, b, T)
    for t in range(1, T + 1):
        if model_latency(m, b, t) <= target * (1 + 1e-12):
            return t
    return T


def occupancy_bound(total_blocks: int, blocks_per_unit: int) -> int:
    """Units a kernel can fill: ceil(total blocks / resident blocks per unit)."""
    if blocks_per_unit <= 0:
        raise ValueError("blocks_per_unit must be positive")
    return max(1, -(-total_blocks // blocks_per_unit))


def capacity_saving(full_units: int, chosen: Sequence[int], lat_at_chosen: Sequence[float]) -> float:
    """1 - (time-weighted mean of chosen units) / full_units  (Section 7.2)."""
    tw = sum(c * t for c, t in zip(chosen, lat_at_chosen))
    tt = sum(lat_at_chosen)
    return 1.0 - (tw / tt) / full_units


def unit_seconds_saved(full_units: int, lat_full: Sequence[float], chosen: Sequence[int],
                       lat_at_chosen: Sequence[float]) -> float:
    """sum_k [ full*t_k(full) - c_k*t_k(c_k) ]"""
    return sum(full_units * tf - c * tc for tf, c, tc in zip(lat_full, chosen, lat_at_chosen))


def predicted_slowdown(lat_full: Sequence[float], lat_at_chosen: Sequence[float]) -> float:
    return sum(lat_at_chosen) / sum(lat_full) - 1.0


def r_squared(y: Sequence[float], yhat: Sequence[float]) -> float:
    mean = sum(y) / len(y)
    ss_tot = sum((v - mean) ** 2 for v in y)
    ss_res = sum((v - w) ** 2 for v, w in zip(y, yhat))
    return 1.0 - ss_res / ss_tot if ss_tot > 0 else 1.0
