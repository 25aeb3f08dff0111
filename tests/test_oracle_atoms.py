"""Pins for the atom-decomposition model and the right-sizing rules."""
import math
import os
import random

import pytest

from oracle import atoms, rightsize

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    out = {"range": []}
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        if key == "range":
            out["range"].append(tuple(int(v) for v in vals))
        else:
            out[key] = [float(v) if "." in v else int(v) for v in vals]
    return out


def test_paper_worked_example():
    g = _golden("atomizer_worked_example.txt")
    grid = tuple(g["grid"])
    total = atoms.total_blocks(grid)
    assert total == g["total_blocks"][0]
    n = g["atoms"][0]
    assert atoms.decompose(grid, total // n) == g["range"]
    assert len(atoms.decompose(grid, 1)) == g["max_atoms"][0]
    # block_idx of Algorithm 1 runs 0..63 over the grid, x fastest
    assert atoms.linearize((0, 0, 0), grid) == 0
    assert atoms.linearize((7, 7, 0), grid) == 63
    assert atoms.linearize((3, 2, 0), grid) == 19
    assert atoms.delinearize(19, grid) == (3, 2, 0)


def test_config1_eight_atoms_of_eight():
    ranges = atoms.decompose((8, 8, 1), 8)
    assert ranges == [(8 * i, 8 * i + 8) for i in range(8)]


def test_linearize_delinearize_are_inverse_and_ordered():
    grid = (5, 3, 4)
    seen = []
    for z in range(4):
        for y in range(3):
            for x in range(5):
                idx = atoms.linearize((x, y, z), grid)
                assert atoms.delinearize(idx, grid) == (x, y, z)
                seen.append(idx)
    assert seen == list(range(60))          # z-major, then y, then x


@pytest.mark.parametrize("pi", [atoms.identity_pi, atoms.xcd_interleave_pi])
def test_every_block_exactly_once_random_grids(pi):
    rnd = random.Random(11)
    grids = [(1, 1, 1), (1, 7, 1), (13, 1, 1), (7, 11, 3), (64, 1, 2), (31, 2, 1)]
    grids += [(rnd.randint(1, 12), rnd.randint(1, 9), rnd.randint(1, 4)) for _ in range(30)]
    for grid in grids:
        total = atoms.total_blocks(grid)
        for B in {0, 1, 2, 3, 7, 8, total - 1, total, total + 5, rnd.randint(1, total)}:
            if B < 0:
                continue
            ranges = atoms.decompose(grid, B)
            # ordered, contiguous, disjoint cover of [0,total)
            assert ranges[0][0] == 0 and ranges[-1][1] == total
            for (a, b), (c, d) in zip(ranges, ranges[1:]):
                assert b == c and a < b
            if 0 < B < total:
                assert len(ranges) == math.ceil(total / B)
                assert ranges[-1][1] - ranges[-1][0] == total - (len(ranges) - 1) * B
            else:
                assert ranges == [(0, total)]
            assert atoms.visit_counts(grid, ranges, pi) == [1] * total


def test_prelude_and_remap_visit_the_same_blocks():
    grid = (6, 5, 3)
    for lo, hi in atoms.decompose(grid, 17):
        a = sorted(atoms.run_atom_prelude(lo, hi, grid))
        b = sorted(atoms.run_atom_remap(lo, hi, grid))
        c = sorted(atoms.run_atom_remap(lo, hi, grid, atoms.xcd_interleave_pi))
        assert a == b == c
        assert len(a) == hi - lo


def test_xcd_interleave_is_a_bijection_for_every_length():
    for n in list(range(1, 70)) + [255, 256, 257, 1000, 1023]:
        image = sorted(atoms.xcd_interleave_pi(h, n) for h in range(n))
        assert image == list(range(n))
    # workgroups that land on one die (h % 8 equal) get consecutive logical slots
    n = 20
    die3 = [atoms.xcd_interleave_pi(h, n) for h in range(3, n, 8)]
    assert die3 == list(range(die3[0], die3[0] + len(die3)))


def test_overlapping_or_gapped_ranges_are_detected():
    grid = (4, 4, 1)
    assert atoms.visit_counts(grid, [(0, 8), (7, 16)])[7] == 2       # overlap shows as a double visit
    assert atoms.visit_counts(grid, [(0, 8), (9, 16)])[8] == 0       # gap shows as a miss


def test_atom_count_and_size():
    assert atoms.atom_count(1000.0, 250.0, 64) == 4
    assert atoms.atom_count(1001.0, 250.0, 64) == 5          # rounded up
    assert atoms.atom_count(100.0, 250.0, 64) == 1           # short kernels stay whole
    assert atoms.atom_count(1e9, 250.0, 64) == 64            # at most one block per atom
    assert atoms.atom_size(1024, 4) == 256
    assert atoms.atom_size(1000, 3, 192) == 384              # 334 -> next multiple of 192
    assert atoms.atom_size(1000, 1, 192) == 1000
    assert atoms.atom_size(100, 2, 192) == 100               # never beyond the kernel


# ------------------------------------------------------------ right-sizing --

def test_two_point_fit_reproduces_both_points_and_limits():
    g = _golden("rightsize_eval_constants.txt")
    k = g["latency_slip"][0]
    T = 256
    m, b = rightsize.fit_two_point(1000.0, 10.0, T)
    assert abs(rightsize.model_latency(m, b, 1) - 1000.0) < 1e-9
    assert abs(rightsize.model_latency(m, b, T) - 10.0) < 1e-9
    # k = 1: nothing may slow down -> all units
    assert rightsize.min_units_for_slip(m, b, T, 1.0) == T
    # perfectly parallel kernel (b = 0): l = m/t, so t_min = ceil(T/k)
    m0, b0 = rightsize.fit_two_point(256.0, 1.0, T)
    assert abs(b0) < 1e-12
    assert rightsize.min_units_for_slip(m0, b0, T, k) == math.ceil(T / k)
    # closed form m / (k (m/T + b) - b), rounded up, equals the direct search
    for l1, lT in [(1000.0, 10.0), (500.0, 100.0), (90.0, 3.0)]:
        m, b = rightsize.fit_two_point(l1, lT, T)
        closed = math.ceil(m / (k * (m / T + b) - b) - 1e-9)
        assert rightsize.min_units_for_slip(m, b, T, k) == closed
    # monotone in k
    m, b = rightsize.fit_two_point(1000.0, 10.0, T)
    picks = [rightsize.min_units_for_slip(m, b, T, kk) for kk in (1.0, 1.05, 1.1, 1.5, 3.0)]
    assert picks == sorted(picks, reverse=True)
    # a kernel that does not scale (l1 == lT) needs one unit
    m, b = rightsize.fit_two_point(50.0, 50.0, T)
    assert rightsize.min_units_for_slip(m, b, T, k) == 1


def test_sweep_selection_rule():
    cus = list(range(8, 257, 8))
    lat = [1000.0 / c + 5.0 for c in cus]
    pick = rightsize.select_from_sweep(cus, lat, 0.04)
    full = lat[-1]
    assert 1000.0 / pick + 5.0 <= 1.04 * full
    assert 1000.0 / (pick - 8) + 5.0 > 1.04 * full
    # non-monotone curve: the smallest qualifying point wins
    lat2 = list(lat)
    lat2[3] = full                      # cus = 32 happens to be as fast as 256
    assert rightsize.select_from_sweep(cus, lat2, 0.04) == 32
    assert rightsize.select_from_sweep(cus, lat, 0.0) == 256
    assert rightsize.select_from_sweep([256, 8], [1.0, 1.0], 0.04) == 8    # order-independent


def test_capacity_statistics():
    # two kernels, 256 units: one keeps 256 for 1 ms, one drops to 64 for 3 ms
    sav = rightsize.capacity_saving(256, [256, 64], [1.0, 3.0])
    assert abs(sav - (1 - ((256 * 1 + 64 * 3) / 4) / 256)) < 1e-15
    assert rightsize.capacity_saving(256, [256, 256], [1.0, 3.0]) == 0.0
    assert abs(rightsize.unit_seconds_saved(256, [1.0, 2.9], [256, 64], [1.0, 3.0]) - (256 * 2.9 - 64 * 3.0)) < 1e-12
    assert abs(rightsize.predicted_slowdown([1.0, 2.9], [1.0, 3.0]) - (4.0 / 3.9 - 1)) < 1e-15
    assert rightsize.occupancy_bound(64, 2) == 32
    assert rightsize.occupancy_bound(65, 2) == 33
    assert rightsize.occupancy_bound(1, 8) == 1
    y = [3.0, 2.0, 1.0]
    assert rightsize.r_squared(y, y) == 1.0
    assert abs(rightsize.r_squared(y, [2.0, 2.0, 2.0])) < 1e-15


def test_general_two_point_fit_and_the_online_rule():
    """Section 4.5: the fit through any two allocations reduces to the (1, T) fit, passes through its
    points, and recovers a known Amdahl curve; 'Operation' = occupancy filter first, model second."""
    T = 108
    m1, b1 = rightsize.fit_two_point(1000.0, 10.0, T)
    m2, b2 = rightsize.fit_through(1, 1000.0, T, 10.0)
    assert abs(m1 - m2) < 1e-9 and abs(b1 - b2) < 1e-9
    m, b = 4000.0, 7.5                                    # l = 4000/t + 7.5 sampled at 64 and 256 units
    mm, bb = rightsize.fit_through(64, m / 64 + b, 256, m / 256 + b)
    assert abs(mm - m) < 1e-9 and abs(bb - b) < 1e-9
    mm, bb = rightsize.fit_through(256, m / 256 + b, 64, m / 64 + b)          # order of the points is free
    assert abs(mm - m) < 1e-9 and abs(bb - b) < 1e-9
    with pytest.raises(ValueError):
        rightsize.fit_through(64, 1.0, 64, 2.0)

    cands = [64, 256]
    lat = lambda t: m / t + b
    # occupancy filter: 128 blocks, 2 per unit -> 64 units are all the kernel can fill
    assert rightsize.online_choice(128, 2, 256, cands, {}, 1.1) == 64
    assert rightsize.online_choice(130, 2, 256, cands, {}, 1.1) == 256        # bound 65 > 64: next set up
    assert rightsize.online_choice(10 ** 6, 2, 256, cands, {}, 1.1) == 256    # model unknown: keep the allocation
    assert rightsize.online_choice(10 ** 6, 2, 256, cands, {256: lat(256)}, 1.1) == 64    # second point: run there once
    assert rightsize.online_choice(10 ** 6, 2, 256, cands, {64: lat(64)}, 1.1) == 256     # the allocation first
    assert rightsize.online_choice(10 ** 6, 2, 256, [256], {256: lat(256)}, 1.1) == 256   # nothing narrower on offer
    # model: l(256) = 23.125; k = 1.1 needs 4000/t + 7.5 <= 25.44 -> t >= 223 -> 256;
    # k = 3.0 needs 4000/t <= 61.9 -> t >= 65 -> 256; k = 3.1 -> t >= 63 -> 64
    known = {64: lat(64), 256: lat(256)}
    assert rightsize.online_choice(10 ** 6, 2, 256, cands, known, 1.1) == 256
    assert rightsize.online_choice(10 ** 6, 2, 256, cands, known, 3.0) == 256
    assert rightsize.online_choice(10 ** 6, 2, 256, cands, known, 3.1) == 64
    # a kernel that does not scale (constant latency): one unit would do, the smallest set wins at any k
    assert rightsize.online_choice(10 ** 6, 2, 256, cands, {64: 50.0, 256: 50.0}, 1.0) == 64
    # brute force: the choice is the smallest candidate whose model latency is within the slip
    for k in (1.0, 1.05, 1.1, 1.5, 2.0, 4.0):
        for mb in ((100.0, 1.0), (5000.0, 0.0), (10.0, 40.0)):
            f = lambda t: mb[0] / t + mb[1]
            c3 = [64, 128, 192, 256]
            got = rightsize.online_choice(10 ** 6, 1, 256, c3, {64: f(64), 256: f(256)}, k)
            want = min(c for c in c3 if min(t for t in range(1, 257) if f(t) <= k * f(256) * (1 + 1e-12)) <= c)
            assert got == want, (k, mb, got, want)
    with pytest.raises(ValueError):
        rightsize.online_choice(10, 1, 128, cands, {}, 1.1)                    # allocation is not a candidate
