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


def fit_through(t1: float, l1: float, t2: float, l2: float) -> Tuple[float, float]:
    """(m, b) of l = m/t + b passing through (t1, l1) and (t2, l2), t1 != t2.

    Section 4.5 'Modeling Kernel Scaling' takes one unit and all units as the two points; on a
    device where the smallest maskable set has more than one unit, the two points are whatever
    two allocations have been measured."""
    if t1 <= 0 or t2 <= 0 or t1 == t2:
        raise ValueError("need two distinct positive unit counts")
    m = (l1 - l2) / (1.0 / t1 - 1.0 / t2)
    b = l2 - m / t2
    return m, b


def online_choice(total_blocks: int, blocks_per_unit: int, allocated: int, candidates: Sequence[int],
                  measured: Dict[int, float], k: float) -> int:
    """Section 4.5 'Operation' for one kernel, on a device that offers only the unit counts in
    ``candidates`` (the CU sets a tenant has queues for), the largest being what the job holds.

    1. Occupancy filter: if the kernel cannot fill the allocation (bound < allocated), it is
       launched on the smallest candidate that still holds the bound (the largest candidate if
       none does).
    2. Otherwise the scaling model: with latencies measured at two of the candidates (``measured``
       maps unit count -> latency of the whole kernel), fit l = m/t + b through the smallest and
       the largest measured count, take the minimum t with l(t) <= k * l(allocated), and launch
       on the smallest candidate >= that t.  The model needs the kernel's latency on two
       allocations, which only running it there can give: while the allocation itself has not
       been measured the kernel keeps it; once it has, and the smallest candidate has not, the
       kernel runs there once.
    """
    cands = sorted(set(candidates))
    if not cands or allocated != cands[-1]:
        raise ValueError("the allocation must be the largest candidate")
    if k < 1.0:
        raise ValueError("latency slip k must be >= 1")
    bound = occupancy_bound(total_blocks, blocks_per_unit)
    if bound < allocated:
        fits = [c for c in cands if c >= bound]
        return fits[0] if fits else cands[-1]
    known = sorted(c for c in measured if c in cands)
    if allocated not in known:
        return allocated
    if len(known) < 2:
        return cands[0] if len(cands) > 1 else allocated
    t1, t2 = known[0], known[-1]
    m, b = fit_through(t1, measured[t1], t2, measured[t2])
    need = min_units_for_slip(m, b, allocated, k)
    return min(c for c in cands if c >= need)
