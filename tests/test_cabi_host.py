"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and its scheduler policy core takes the same decisions as the
oracle's scheduler model on the same scenario (no compute calls, no GPU)."""
import os
import random
import re

import pytest

from oracle.sched_sim import Kernel, SimConfig, Simulator
from paper_2504_15465_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_gemm_split_hint_fills_the_partition():
    """Host-only entry point: output tiles x K slices is about one workgroup per CU."""
    def hint(m, n, k, cus):
        return B.lithos_gemm_split_hint(B.make_op(B.OP_GEMM, (m, n, k)), cus)
    assert hint(1024, 3072, 16384, 256) == (256, 5)       # 48 tiles x 5 = 240 workgroups
    assert hint(1024, 1024, 16384, 256) == (256, 16)
    assert hint(1024, 4096, 16384, 192) == (256, 3)
    assert hint(8192, 8192, 8192, 256) == (0, 1)          # 1024 tiles fill the chip: leave it whole
    assert hint(1024, 1024, 1024, 256) == (256, 2)        # at least 8 k-tiles per slice
    assert hint(1024, 1024, 512, 256) == (0, 1)           # K too short to cut
    assert hint(8, 4096, 4096, 64) == (0, 1)              # weight-streaming shapes are not cut
    with pytest.raises(B.LithosError):
        B.lithos_gemm_split_hint(B.make_op(B.OP_SPIN, (4, 10)), 64)


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "lithos.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lithos_[a-z0-9_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = B.lib()
    names = _declared_symbols()
    assert len(names) >= 30
    for n in names:
        assert hasattr(lib, n), "liblithos.so does not export %s" % n
    assert sorted(B.EXPORTS) == names, "binding and header disagree"


def test_binding_struct_sizes_match_the_header_layout():
    import ctypes as C
    assert C.sizeof(B.Op) == 4 * 4 + 8 * 8 + 4 * 8 + 4 * 4 + 6 * 8 + 2 * 8
    assert C.sizeof(B.Dim3) == 12
    assert C.sizeof(B.Config) == 48
    assert C.sizeof(B.CoreAtom) == 56
    assert C.sizeof(B.Stats) == 64


def test_core_rejects_bad_arguments():
    with pytest.raises(B.LithosError) as e:
        B.lithos_core_create(None, 0, 8)
    assert e.value.code == B.EINVAL
    c = B.lithos_core_create(None, 32, 8)
    t0 = B.lithos_core_add_tenant(c, B.CLASS_HP, 0xFF)
    with pytest.raises(B.LithosError) as e:
        B.lithos_core_add_tenant(c, B.CLASS_BE, 0x80)          # overlaps tenant 0
    assert e.value.code == B.EMASK
    with pytest.raises(B.LithosError):
        B.lithos_core_add_tenant(c, B.CLASS_BE, 0)             # empty quota
    with pytest.raises(B.LithosError):
        B.lithos_core_submit(c, 5, 10)                         # unknown tenant
    with pytest.raises(B.LithosError):
        B.lithos_core_submit(c, t0, 0)                         # empty kernel
    with pytest.raises(B.LithosError) as e:
        B.lithos_core_complete(c, 12345, 0.0, 1.0)             # not in flight
    assert e.value.code == B.ESTATE
    assert B.lithos_core_next_atom(c, t0, 0.0) is None
    B.lithos_core_destroy(c)


# ---- lock-step comparison with the oracle's scheduler model -------------------

HP_Q = frozenset(range(0, 8))
BE_Q = frozenset(range(8, 32))


def _lat(op, cus, blocks):
    if op == "be_flat":                        # a kernel that does not scale with CUs (per-block serial work)
        return 2.0 + 0.4 * blocks
    per_block = {"be": 62.5, "hp_a": 20.0, "hp_b": 24.0, "be_small": 300.0}[op]
    return 2.0 + per_block * blocks / cus


def _bits(groups):
    m = 0
    for g in groups:
        m |= 1 << g
    return m


class CoreHarness:
    """Plays clock and device for the C policy core exactly as the oracle's
    simulator plays them for its own policy (exclusive CU groups, stream order)."""

    def __init__(self, cfg: B.Config, ops_by_kernel, tenants=None):
        self.c = B.lithos_core_create(cfg, 32, 8)
        tenants = tenants or [(B.CLASS_HP, HP_Q), (B.CLASS_BE, BE_Q)]
        self.ids = [B.lithos_core_add_tenant(self.c, cls, _bits(q)) for cls, q in tenants]
        self.hp, self.be = self.ids[0], self.ids[-1]
        self.group_free = [0.0] * 32
        self.last_end = {t: 0.0 for t in self.ids}
        self.events = []
        self.seq = 0
        self.trace = []
        self.op_of = ops_by_kernel

    def push(self, time, kind, payload):
        import heapq
        heapq.heappush(self.events, (time, self.seq, kind, payload))
        self.seq += 1

    def dispatch_all(self, now):
        progressed = True
        while progressed:
            progressed = False
            for t in self.ids:
                a = B.lithos_core_next_atom(self.c, t, now)
                if a is None:
                    continue
                progressed = True
                groups = [g for g in range(32) if a.group_mask >> g & 1]
                cus = 8 * len(groups)
                start = max(now, self.last_end[t], max(self.group_free[g] for g in groups))
                dur = _lat(self.op_of[a.kernel_id], cus, a.hi - a.lo)
                end = start + dur
                self.last_end[t] = end
                for g in groups:
                    self.group_free[g] = end
                self.trace.append((t, a.ordinal, a.lo, a.hi, a.group_mask, bool(a.stolen),
                                   a.predicted_us if a.has_prediction else None, start, end))
                self.push(end, "complete", (a.atom_id, dur))

    def run(self):
        import heapq
        while self.events:
            time, _, kind, payload = heapq.heappop(self.events)
            if kind == "submit":
                t, total, op = payload
                kid = B.lithos_core_submit(self.c, t, total, 1)
                self.op_of[kid] = op
            elif kind == "sync":
                B.lithos_core_sync_mark(self.c, payload)
            else:
                atom_id, dur = payload
                B.lithos_core_complete(self.c, atom_id, time, dur)
            self.dispatch_all(time)


@pytest.mark.parametrize("atomize,steal,atom_us,max_out,max_out_hp", [
    (True, True, 100.0, 2, 0), (False, True, 100.0, 2, 0), (True, False, 100.0, 2, 0),
    (True, True, 40.0, 3, 8), (True, True, 400.0, 1, 4)])
def test_policy_core_matches_oracle_model_step_by_step(atomize, steal, atom_us, max_out, max_out_hp):
    rnd = random.Random(42)
    hp_times = sorted(rnd.uniform(100, 30000) for _ in range(40))
    scenario = []                      # (time, kind, tenant, total, op)
    for i in range(50):
        scenario.append((0.0, "submit", "be", 1024, "be"))
        scenario.append((0.0, "sync", "be", 0, ""))
    for t in hp_times:
        scenario.append((t, "submit", "hp", 64, "hp_a"))
        scenario.append((t, "submit", "hp", 48, "hp_b"))
        scenario.append((t, "sync", "hp", 0, ""))

    # oracle model
    sim = Simulator(SimConfig(atom_duration_us=atom_us, max_outstanding=max_out, max_outstanding_hp=max_out_hp,
                              steal=steal, atomize=atomize), _lat)
    hp = sim.add_tenant(HP_Q, hp=True)
    be = sim.add_tenant(BE_Q, hp=False)
    for time, kind, who, total, op in scenario:
        tid = hp if who == "hp" else be
        if kind == "submit":
            sim.submit_at(time, tid, Kernel(op, total, 1))
        else:
            sim.sync_at(time, tid)
    sim.run()
    want = [(a.tenant, a.ordinal, a.lo, a.hi, _bits(a.mask), a.stolen, a.predicted_us, a.t_start, a.t_end)
            for a in sim.trace]

    # C core under the same clock and device
    cfg = B.Config.default(atom_duration_us=atom_us, max_outstanding=max_out, max_outstanding_hp=max_out_hp,
                           steal=int(steal), atomize=int(atomize))
    h = CoreHarness(cfg, {})
    for time, kind, who, total, op in scenario:
        tid = h.hp if who == "hp" else h.be
        if kind == "submit":
            h.push(time, "submit", (tid, total, op))
        else:
            h.push(time, "sync", tid)
    h.run()

    assert len(h.trace) == len(want)
    for got, exp in zip(h.trace, want):
        assert got[:6] == exp[:6], (got, exp)
        if exp[6] is None:
            assert got[6] is None
        else:
            assert abs(got[6] - exp[6]) < 1e-9
        assert abs(got[7] - exp[7]) < 1e-9 and abs(got[8] - exp[8]) < 1e-9
    s_hp, s_be = B.lithos_core_stats(h.c, h.hp), B.lithos_core_stats(h.c, h.be)
    assert s_hp.atoms + s_be.atoms == sim.stats["atoms"]
    assert s_hp.stolen_atoms + s_be.stolen_atoms == sim.stats["steals"]
    assert (s_hp.revocations, s_be.revocations) == (sim.per_tenant[hp]["revocations"], sim.per_tenant[be]["revocations"])
    assert (s_hp.stolen_atoms, s_be.stolen_atoms) == (sim.per_tenant[hp]["steals"], sim.per_tenant[be]["steals"])
    if atomize and steal and atom_us <= 100.0:
        assert s_be.revocations > 0          # the scenario does hand CUs back at atom boundaries
    elif atomize and steal:
        pass                                 # 400 us atoms: these kernels are predicted shorter and stay whole
    else:
        assert s_be.revocations == 0         # whole kernels have no inner boundary; no lending, nothing to revoke
    assert s_hp.revocations == 0             # the best-effort tenant never idles, so nothing is lent to the other
    assert s_hp.mispredicts + s_be.mispredicts == sim.stats["mispredicts"]
    assert s_hp.predictions + s_be.predictions == sim.stats["predictions"]
    B.lithos_core_destroy(h.c)


@pytest.mark.parametrize("atomize,steal", [(True, True), (False, True), (True, False)])
def test_policy_core_matches_oracle_model_with_three_tenants(atomize, steal):
    """Two high-priority tenants (quotas of 128 and 64 CUs) and a best-effort tenant with a small
    quota (64 CUs) that lives on what the other two leave idle (paper Section 7.1, inference-only
    stacking): the C core and the oracle's model take the same decisions, and a high-priority
    tenant may also borrow the other one's idle CUs."""
    quotas = [frozenset(range(0, 16)), frozenset(range(16, 24)), frozenset(range(24, 32))]
    rnd = random.Random(7)
    scenario = []
    for i in range(40):
        scenario.append((0.0, "submit", 2, 1024, "be"))
        scenario.append((0.0, "sync", 2, 0, ""))
    for t in sorted(rnd.uniform(100, 40000) for _ in range(30)):
        scenario.append((t, "submit", 0, 256, "hp_a"))
        scenario.append((t, "submit", 0, 64, "hp_b"))
        scenario.append((t, "sync", 0, 0, ""))
    for t in sorted(rnd.uniform(100, 40000) for _ in range(25)):
        scenario.append((t, "submit", 1, 96, "hp_b"))
        scenario.append((t, "sync", 1, 0, ""))
    scenario.sort(key=lambda e: e[0])           # stable: same-time events keep their order

    sim = Simulator(SimConfig(atom_duration_us=100.0, max_outstanding=2, max_outstanding_hp=4, steal=steal, atomize=atomize), _lat)
    sim_ids = [sim.add_tenant(quotas[0], hp=True), sim.add_tenant(quotas[1], hp=True), sim.add_tenant(quotas[2], hp=False)]
    for time, kind, who, total, op in scenario:
        if kind == "submit":
            sim.submit_at(time, sim_ids[who], Kernel(op, total, 1))
        else:
            sim.sync_at(time, sim_ids[who])
    sim.run()
    want = [(a.tenant, a.ordinal, a.lo, a.hi, _bits(a.mask), a.stolen, a.t_start, a.t_end) for a in sim.trace]

    cfg = B.Config.default(atom_duration_us=100.0, max_outstanding=2, max_outstanding_hp=4, steal=int(steal), atomize=int(atomize))
    h = CoreHarness(cfg, {}, [(B.CLASS_HP, quotas[0]), (B.CLASS_HP, quotas[1]), (B.CLASS_BE, quotas[2])])
    for time, kind, who, total, op in scenario:
        if kind == "submit":
            h.push(time, "submit", (h.ids[who], total, op))
        else:
            h.push(time, "sync", h.ids[who])
    h.run()
    got = [(sim_ids[h.ids.index(t)], o, lo, hi, m, st, s, e) for t, o, lo, hi, m, st, _, s, e in h.trace]
    assert len(got) == len(want)
    for g, w in zip(got, want):
        assert g[:6] == w[:6], (g, w)
        assert abs(g[6] - w[6]) < 1e-9 and abs(g[7] - w[7]) < 1e-9
    # no atom ever ran on CUs outside its tenant's quota plus quotas lent by an idle owner
    for t, o, lo, hi, m, st, s, e in got:
        own = _bits(quotas[sim_ids.index(t)])
        assert m & own == own
        assert st == (m != own)
        if not steal:
            assert m == own
    for who in range(3):
        st = B.lithos_core_stats(h.c, h.ids[who])
        book = sim.per_tenant[sim_ids[who]]
        assert (st.atoms, st.stolen_atoms, st.revocations) == (book["atoms"], book["steals"], book["revocations"])
    if steal:
        stolen_by = {t for t, *_rest in [(g[0], g[5]) for g in got if g[5]]}
        assert sim_ids[2] in stolen_by                      # best effort lives on lent CUs
        assert any(g[5] and g[0] in sim_ids[:2] for g in got)   # a high-priority tenant borrowed too
    B.lithos_core_destroy(h.c)


@pytest.mark.parametrize("slip", [1.1, 1.5])
def test_policy_core_right_sizes_online_like_the_oracle_model(slip):
    """Section 4.5 'Operation' in the dispatcher: a best-effort tenant whose kernels could borrow the idle
    high-priority CUs borrows them only when the occupancy filter and the two-point model say the wider
    set pays.  Three kinds of best-effort kernel per batch: one that scales (1024 blocks), one that does
    not (constant latency per block count), one too small to fill more than the quota (96 blocks)."""
    rnd = random.Random(11)
    scenario = []
    for i in range(60):
        for total, op in ((1024, "be"), (512, "be_flat"), (96, "be_small")):
            scenario.append((0.0, "submit", "be", total, op))
        scenario.append((0.0, "sync", "be", 0, ""))
    for t in sorted(rnd.uniform(100, 60000) for _ in range(25)):
        scenario.append((t, "submit", "hp", 64, "hp_a"))
        scenario.append((t, "sync", "hp", 0, ""))

    sim = Simulator(SimConfig(atom_duration_us=100.0, max_outstanding=2, rightsize_slip=slip), _lat)
    hp, be = sim.add_tenant(HP_Q, hp=True), sim.add_tenant(BE_Q, hp=False)
    for time, kind, who, total, op in scenario:
        tid = hp if who == "hp" else be
        if kind == "submit":
            sim.submit_at(time, tid, Kernel(op, total, 1))
        else:
            sim.sync_at(time, tid)
    sim.run()
    want = [(a.tenant, a.ordinal, a.lo, a.hi, _bits(a.mask), a.stolen, a.t_start, a.t_end) for a in sim.trace]

    h = CoreHarness(B.Config.default(atom_duration_us=100.0, max_outstanding=2, rightsize_slip=slip), {})
    for time, kind, who, total, op in scenario:
        tid = h.hp if who == "hp" else h.be
        if kind == "submit":
            h.push(time, "submit", (tid, total, op))
        else:
            h.push(time, "sync", tid)
    h.run()
    got = [(t, o, lo, hi, m, st, s, e) for t, o, lo, hi, m, st, _, s, e in h.trace]
    assert len(got) == len(want)
    for g, w in zip(got, want):
        assert g[:6] == w[:6], (g, w)
        assert abs(g[6] - w[6]) < 1e-9 and abs(g[7] - w[7]) < 1e-9
    st = B.lithos_core_stats(h.c, h.be)
    book = sim.per_tenant[be]
    assert (st.atoms, st.stolen_atoms, st.revocations, st.rightsized_kernels) == \
        (book["atoms"], book["steals"], book["revocations"], book["rightsized"])
    # once the best-effort queue has drained, the high-priority kernels (64 blocks = its 64 CUs) could
    # borrow and the occupancy filter keeps them at home: the same count on both sides
    assert B.lithos_core_stats(h.c, h.hp).rightsized_kernels == sim.per_tenant[hp]["rightsized"]
    assert all(g[4] == _bits(HP_Q) for g in got if g[0] == h.hp)
    own = _bits(BE_Q)
    small = [g for g in got if g[0] == h.be and g[1] == 2]
    assert small and all(g[4] == own for g in small)                  # 96 blocks cannot fill more than 192 CUs: never borrows
    flat = [g for g in got if g[0] == h.be and g[1] == 1]
    assert any(g[4] != own for g in flat[:6])                          # borrows until both CU sets have been measured ...
    assert all(g[4] == own for g in flat[-20:])                        # ... then the model says the wider set gains nothing
    scal = [g for g in got if g[0] == h.be and g[1] == 0]
    if slip == 1.1:
        assert any(g[4] != own for g in scal[-20:])                    # 256 vs 192 CUs is a 1.33x gain: worth borrowing at k = 1.1
    else:
        assert all(g[4] == own for g in scal[-20:])                    # but inside a slip of 1.5
    B.lithos_core_destroy(h.c)


@pytest.mark.parametrize("seed", range(48))
def test_policy_core_matches_oracle_model_on_random_scenarios(seed):
    """Seeded random tenants, quotas, kernels, arrival times and scheduler settings (atom length,
    outstanding limits, stealing, atomization, right-sizing slip): the C policy core and the oracle's
    model emit the same atoms on the same CU groups at the same times, and keep the same books."""
    rnd = random.Random(1000 + seed)
    n_hp = rnd.choice([1, 1, 2])
    cuts = sorted(rnd.sample(range(1, 32), n_hp))                     # group boundaries of the quotas
    bounds = [0] + cuts + [32]
    quotas = [frozenset(range(bounds[i], bounds[i + 1])) for i in range(n_hp + 1)]
    classes = [True] * n_hp + [False]
    scfg = dict(atom_duration_us=rnd.choice([30.0, 80.0, 150.0, 300.0]), max_outstanding=rnd.randint(1, 3),
                max_outstanding_hp=rnd.choice([0, 2, 8]), steal=rnd.random() < 0.8, atomize=rnd.random() < 0.8,
                rightsize_slip=rnd.choice([0.0, 0.0, 1.1, 1.5]))
    scenario = []
    be = n_hp
    for i in range(rnd.randint(10, 40)):                              # best effort: batches of 1-3 kernels, all queued at once
        for _ in range(rnd.randint(1, 3)):
            scenario.append((0.0, "submit", be, rnd.choice([96, 512, 1024, 1500]), rnd.choice(["be", "be", "be_flat", "be_small"])))
        scenario.append((0.0, "sync", be, 0, ""))
    horizon = rnd.uniform(5000, 50000)
    for who in range(n_hp):
        for t in sorted(rnd.uniform(50, horizon) for _ in range(rnd.randint(5, 40))):
            for _ in range(rnd.randint(1, 3)):
                scenario.append((t, "submit", who, rnd.choice([16, 48, 64, 200, 256]), rnd.choice(["hp_a", "hp_b"])))
            scenario.append((t, "sync", who, 0, ""))
    scenario.sort(key=lambda e: e[0])                                 # stable: same-time events keep their order

    sim = Simulator(SimConfig(**scfg), _lat)
    sim_ids = [sim.add_tenant(q, hp=c) for q, c in zip(quotas, classes)]
    for time, kind, who, total, op in scenario:
        if kind == "submit":
            sim.submit_at(time, sim_ids[who], Kernel(op, total, 1))
        else:
            sim.sync_at(time, sim_ids[who])
    sim.run()
    want = [(a.tenant, a.ordinal, a.lo, a.hi, _bits(a.mask), a.stolen, a.predicted_us, a.t_start, a.t_end) for a in sim.trace]

    cfg = B.Config.default(**{k: (int(v) if isinstance(v, bool) else v) for k, v in scfg.items()})
    h = CoreHarness(cfg, {}, [(B.CLASS_HP if c else B.CLASS_BE, q) for q, c in zip(quotas, classes)])
    for time, kind, who, total, op in scenario:
        if kind == "submit":
            h.push(time, "submit", (h.ids[who], total, op))
        else:
            h.push(time, "sync", h.ids[who])
    h.run()
    got = [(sim_ids[h.ids.index(t)],) + tuple(rest) for t, *rest in h.trace]
    assert len(got) == len(want), (scfg, len(got), len(want))
    for g, w in zip(got, want):
        assert g[:6] == w[:6], (scfg, g, w)
        assert (g[6] is None) == (w[6] is None) and (w[6] is None or abs(g[6] - w[6]) < 1e-9)
        assert abs(g[7] - w[7]) < 1e-9 and abs(g[8] - w[8]) < 1e-9
    for who in range(n_hp + 1):
        st = B.lithos_core_stats(h.c, h.ids[who])
        book = sim.per_tenant[sim_ids[who]]
        assert (st.atoms, st.stolen_atoms, st.revocations, st.rightsized_kernels) == \
            (book["atoms"], book["steals"], book["revocations"], book["rightsized"]), (scfg, who)
        own = _bits(quotas[who])
        for g in got:
            if g[0] == sim_ids[who]:
                assert g[4] & own == own and (g[5] == (g[4] != own))
                if not scfg["steal"]:
                    assert g[4] == own
    B.lithos_core_destroy(h.c)


def test_core_refuses_a_slip_below_one():
    with pytest.raises(B.LithosError) as e:
        B.lithos_core_create(B.Config.default(rightsize_slip=0.5), 32, 8)
    assert e.value.code == B.EINVAL
