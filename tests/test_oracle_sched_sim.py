"""Invariants of the scheduler model (it is a heuristic: no reference numbers)."""
import random

import pytest

from oracle.sched_sim import Kernel, SimConfig, Simulator

HP_Q = frozenset(range(0, 8))        # 8 groups = 64 CUs
BE_Q = frozenset(range(8, 32))       # 24 groups = 192 CUs


def lat(op, cus, blocks):
    """Device truth: perfectly parallel per block-wave plus a fixed launch cost."""
    per_block = {"be_gemm": 250.0 * 256 / 1024, "hp_gemm": 20.0 * 64 / 64, "hp_ln": 3.0 * 64 / 8}[op]
    return 2.0 + per_block * blocks / cus


def build(cfg, be_kernels=8, hp_times=(), hp_chain=("hp_gemm", "hp_ln")):
    sim = Simulator(cfg, lat)
    hp = sim.add_tenant(HP_Q, hp=True)
    be = sim.add_tenant(BE_Q, hp=False)
    for i in range(be_kernels):
        sim.submit_at(0.0, be, Kernel("be_gemm", 1024, 1))
        sim.sync_at(0.0, be)              # one kernel per batch: ordinal 0 every time
    hp_kids = []
    for t in hp_times:
        kids = []
        for op in hp_chain:
            kids.append(sim.submit_at(t, hp, Kernel(op, 64 if op == "hp_gemm" else 8, 1)))
        sim.sync_at(t, hp)
        hp_kids.append((t, kids))
    return sim, hp, be, hp_kids


def test_every_block_of_every_kernel_runs_exactly_once():
    cfg = SimConfig(atom_duration_us=100.0)
    sim, hp, be, _ = build(cfg, be_kernels=6, hp_times=[500.0, 2100.0, 2150.0, 9000.0])
    sim.run()
    assert len(sim.kernel_done) == len(sim.kernel_submit)
    for kid, seen in sim.kernel_blocks_seen.items():
        assert seen == [1] * len(seen)
    # atoms of one kernel are consecutive ranges in launch order
    by_kernel = {}
    for a in sim.trace:
        by_kernel.setdefault(a.kid, []).append((a.lo, a.hi))
    for ranges in by_kernel.values():
        assert ranges[0][0] == 0
        for (a, b), (c, d) in zip(ranges, ranges[1:]):
            assert b == c


def test_masks_stay_inside_quota_plus_stolen_and_revocation():
    cfg = SimConfig(atom_duration_us=100.0)
    hp_times = [1000.0, 1030.0, 5000.0]
    sim, hp, be, hp_kids = build(cfg, be_kernels=10, hp_times=hp_times)
    sim.run()
    for a in sim.trace:
        own = HP_Q if a.tenant == hp else BE_Q
        other = BE_Q if a.tenant == hp else HP_Q
        assert own <= a.mask
        assert a.mask <= own | other
        assert a.stolen == bool(a.mask - own)
        if a.mask - own:
            assert a.mask == own | other          # whole quota or nothing
    # while HP has work (from submit until its last kernel completes) no BE atom
    # *launched* in that window may include HP groups
    for t_sub, kids in hp_kids:
        t_done = max(sim.kernel_done[k] for k in kids)
        for a in sim.trace:
            if a.tenant == be and t_sub <= a.t_launch < t_done:
                assert not (a.mask & HP_Q), (a, t_sub, t_done)
    # BE does steal when HP is idle (work conservation)
    assert any(a.tenant == be and a.stolen for a in sim.trace)


def test_no_stealing_means_independent_timelines():
    cfg = SimConfig(steal=False, atom_duration_us=100.0)
    sim_a, hp, be, _ = build(cfg, be_kernels=5, hp_times=[100.0, 400.0])
    sim_a.run()
    sim_b, _, _, _ = build(cfg, be_kernels=5, hp_times=[])
    sim_b.run()
    be_a = [(a.lo, a.hi, a.t_start, a.t_end) for a in sim_a.trace if a.tenant == be]
    be_b = [(a.lo, a.hi, a.t_start, a.t_end) for a in sim_b.trace if a.tenant == be]
    assert be_a == be_b
    assert all(not a.stolen for a in sim_a.trace)


def test_hp_wait_is_bounded_by_outstanding_stolen_atoms():
    for atom_us, max_out in [(100.0, 2), (200.0, 1), (50.0, 3)]:
        cfg = SimConfig(atom_duration_us=atom_us, max_outstanding=max_out)
        rnd = random.Random(3)
        hp_times = sorted(rnd.uniform(3000, 60000) for _ in range(40))
        sim, hp, be, hp_kids = build(cfg, be_kernels=60, hp_times=hp_times, hp_chain=("hp_gemm",))
        sim.run()
        # once the predictor is warm a stolen atom holds HP's CUs for about one
        # atom_duration; the quantised atom may be longer by one wave of blocks
        wave = lat("be_gemm", 256, 256)
        bound = max_out * (atom_us + wave) + 1e-6
        first = {a.kid: a for a in reversed(sim.trace)}
        solo = lat("hp_gemm", 64, 64)
        waits = []
        for t_sub, kids in hp_kids:
            a = first[kids[0]]
            waits.append(a.t_start - max(t_sub, a.t_launch))
        assert max(waits) <= bound, (atom_us, max_out, max(waits), bound)


def test_atomization_off_gives_longer_hp_waits_than_on():
    def p_max(atomize):
        cfg = SimConfig(atom_duration_us=100.0, atomize=atomize)
        rnd = random.Random(5)
        hp_times = sorted(rnd.uniform(3000, 60000) for _ in range(60))
        sim, hp, be, hp_kids = build(cfg, be_kernels=80, hp_times=hp_times, hp_chain=("hp_gemm",))
        sim.run()
        return max(sim.kernel_done[k[0]] - t for t, k in hp_kids)
    assert p_max(True) < p_max(False)


def test_work_conservation_and_outstanding_limit():
    cfg = SimConfig(atom_duration_us=100.0, max_outstanding=2)
    sim, hp, be, _ = build(cfg, be_kernels=6, hp_times=[700.0])
    sim.run()
    # at no time more than max_outstanding atoms of one tenant are on the device
    for tid in (hp, be):
        spans = sorted((a.t_launch, a.t_end) for a in sim.trace if a.tenant == tid)
        for i, (tl, _) in enumerate(spans):
            inflight = sum(1 for (l, e) in spans[:i] if e > tl)
            assert inflight < cfg.max_outstanding
    # BE's device timeline has no gaps while it has work queued (closed loop at t=0)
    be_atoms = [a for a in sim.trace if a.tenant == be]
    for a, b in zip(be_atoms, be_atoms[1:]):
        assert b.t_start - a.t_end < 1e-9 or b.t_launch <= a.t_end + 1e-9


def test_ordinal_resets_at_sync_and_predictor_learns():
    cfg = SimConfig(atom_duration_us=100.0)
    sim, hp, be, hp_kids = build(cfg, be_kernels=0, hp_times=[0.0, 1000.0, 2000.0])
    sim.run()
    ords = [a.ordinal for a in sim.trace if a.tenant == hp]
    assert ords == [0, 1, 0, 1, 0, 1]
    # first request is cold (no prediction), later ones are predicted exactly
    preds = [a.predicted_us for a in sim.trace if a.tenant == hp]
    assert preds[0] is None and preds[1] is None
    for a in sim.trace[2:]:
        assert abs(a.predicted_us - (a.t_end - a.t_start)) < 1e-9
    assert sim.stats["mispredicts"] == 0


def test_unseen_cu_count_scales_linearly():
    from oracle.sched_sim import Predictor
    p = Predictor(0.25)
    assert p.us_per_block(0, 256) is None
    p.update(0, 256, 100, 50.0)                 # 0.5 us per block on 256 CUs
    assert p.us_per_block(0, 256) == 0.5
    assert p.us_per_block(0, 128) == 1.0        # half the CUs: twice as long
    p.update(0, 256, 100, 90.0)                 # EMA: 0.75*0.5 + 0.25*0.9
    assert abs(p.us_per_block(0, 256) - 0.6) < 1e-12


def _revocations_from_trace(sim, tenant):
    """Recount from the atom trace: boundaries inside one kernel where the mask lost groups."""
    by_kernel = {}
    for a in sim.trace:
        if a.tenant == tenant:
            by_kernel.setdefault(a.kid, []).append(a.mask)
    return sum(1 for masks in by_kernel.values() for m0, m1 in zip(masks, masks[1:]) if m0 - m1)


def test_revocations_count_atom_boundaries_where_lent_groups_go_back():
    """One long best-effort kernel per batch, cut in atoms; a high-priority request that arrives in the
    middle of a kernel takes its groups back at the next atom boundary: exactly one revocation per such
    arrival, none without arrivals, none when kernels stay whole or nothing is lent."""
    cfg = SimConfig(atom_duration_us=50.0, max_outstanding=1)
    # warm the predictor with two kernels, then one arrival inside the fourth kernel
    sim, hp, be, _ = build(cfg, be_kernels=6, hp_times=[])
    sim.run()
    assert sim.stats["revocations"] == 0 and sim.stats["steals"] > 0
    sim, hp, be, _ = build(cfg, be_kernels=6, hp_times=[700.0])
    sim.run()
    cut = [a for a in sim.trace if a.tenant == be and a.t_launch <= 700.0 < a.t_end]
    assert cut and cut[0].stolen and cut[0].hi < 1024         # the arrival falls inside a stolen, inner atom
    assert sim.per_tenant[be]["revocations"] == 1
    assert sim.per_tenant[hp]["revocations"] == 0
    assert sim.stats["revocations"] == _revocations_from_trace(sim, be) == 1
    # many arrivals: the count equals the recount from the trace
    rnd = random.Random(5)
    times = sorted(rnd.uniform(300.0, 6000.0) for _ in range(12))
    sim, hp, be, _ = build(cfg, be_kernels=30, hp_times=times)
    sim.run()
    assert sim.per_tenant[be]["revocations"] == _revocations_from_trace(sim, be) > 0
    assert sim.per_tenant[be]["revocations"] <= len(times)
    for off in (dict(atomize=False), dict(steal=False)):
        sim, hp, be, _ = build(SimConfig(atom_duration_us=50.0, max_outstanding=1, **off), be_kernels=30, hp_times=times)
        sim.run()
        assert sim.stats["revocations"] == 0
