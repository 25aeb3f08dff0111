"""The request planning of bench.py (no GPU): every leg of a stacking run gets at least one timed
request and never indexes past its own arrivals, whatever --steps / --warmup are."""
import numpy as np
import pytest

import bench
from paper_2504_15465_amd import inputs


@pytest.mark.parametrize("steps,warmup", [(1, 0), (20, 5), (100, 100), (3000, 200), (0, 0), (5, 1000)])
def test_every_leg_has_timed_requests_inside_its_arrivals(steps, warmup):
    legs = bench.plan_legs(steps, warmup)
    assert legs["main"] == (max(0, warmup), max(1, steps))          # exactly --steps timed after --warmup
    for name, (warm, timed) in legs.items():
        assert warm >= 0 and timed >= 1, name
        arr = inputs.poisson_arrivals(200.0, warm + timed, seed=3)   # each leg draws its own arrivals
        warm_arr, timed_arr = bench.split_arrivals(arr, warm)
        assert len(warm_arr) == warm and len(timed_arr) == timed
        assert np.all(np.diff(timed_arr) >= 0) and timed_arr[0] > 0  # re-based: gaps of the same process
        if warm:
            assert timed_arr[0] == pytest.approx(arr[warm] - arr[warm - 1])
    w_c, n_c = legs["comparator"]
    assert n_c <= max(1, steps) and n_c <= 1000 and w_c <= min(max(0, warmup), 100)


def test_split_clamps_a_warmup_longer_than_the_leg():
    arr = inputs.poisson_arrivals(200.0, 25, seed=3)
    warm_arr, timed = bench.split_arrivals(arr, 100)                 # the failure of the first driver run
    assert len(warm_arr) == 24 and len(timed) == 1
    with pytest.raises(ValueError):
        bench.split_arrivals(arr[:0], 0)


def test_nearest_rank_percentile():
    x = list(range(1, 101))
    assert bench.nearest_rank(x, 0.99) == 99 and bench.nearest_rank(x, 0.5) == 50
    assert bench.nearest_rank([7.0], 0.99) == 7.0
    assert bench.nearest_rank(list(range(20)), 0.99) == 19          # under 100 samples p99 is the maximum
