"""Discrete-event model of the spatial scheduler (LithOS Sections 4.2-4.4, 4.7).

TEST INFRASTRUCTURE ONLY.  Pure Python, fake clock, fake device.

What is modelled, in the paper's order:

* launch queues: one FIFO of submitted kernels per tenant; submission
  returns at once and dispatch is deferred (Section 4.2).
* compute quotas: each tenant owns a set of CU groups it is guaranteed
  (Section 4.2).
* dispatch: a tenant may have at most ``max_outstanding`` atoms on the device
  (the sync-queue backlog threshold, Section 4.3 'Operation').
* atomization: the kernel's predicted duration on the chosen CUs divided by
  ``atom_duration`` gives the number of atoms (Section 4.4 'Operation');
  kernels predicted shorter than one atom stay whole (Section 4.4
  'Performance Optimizations').
* stealing: a tenant may add to its quota the groups of a tenant that is
  idle (nothing queued, nothing in flight) and whose per-group timers have
  expired; once the owner submits, later atoms of the thief use only its own
  quota, atoms already in flight run to completion (Section 4.3 'TPC
  Stealing', Section 4.4 second paragraph of 'Operation').  Such an atom
  boundary, where a kernel's next atom runs on fewer groups than its previous
  one, is counted as a revocation.
* right-sizing (optional): when a kernel could borrow CUs, the occupancy
  filter and the two-point scaling model decide whether the wider set is
  worth taking; if not, the kernel and all its atoms stay on the quota
  (Section 4.5 'Operation').
* prediction: per launch queue, keyed by the ordinal of the kernel since the
  last synchronisation and by the CU count; unseen CU counts scale the
  nearest known one linearly (Section 4.7).

The device is a timeline of exclusive CU groups: an atom starts when it has
been launched, the previous atom of the same tenant has finished, and every
group in its mask is free; it then holds all groups of its mask for its true
latency (given by the scenario's latency function).

The simulator is checked by invariants, not by reference numbers.
"""
from __future__ import annotations

import heapq
from collections import deque
from dataclasses import dataclass, field
from typing import Callable, Dict, FrozenSet, List, Optional, Tuple

from . import atoms as atom_model
from . import rightsize as rightsize_model

MISPREDICT_US = 50.0   # Section 7.4: absolute error above 50 us is a misprediction


@dataclass
class SimConfig:
    n_groups: int = 32
    cus_per_group: int = 8
    atom_duration_us: float = 250.0
    max_outstanding: int = 2
    max_outstanding_hp: int = 0      # 0: high-priority tenants use max_outstanding too
    steal: bool = True
    atomize: bool = True
    ema_alpha: float = 0.25
    rightsize_slip: float = 0.0      # Section 4.5 latency slip k (>= 1); 0: no online right-sizing


@dataclass
class Kernel:
    op: str                 # name looked up by the scenario's latency function
    total_blocks: int
    wg_per_cu: int = 1
    kid: int = -1           # filled at submit
    ordinal: int = -1       # filled at dispatch of its first atom


@dataclass
class Atom:
    aid: int
    tenant: int
    kid: int
    op: str
    ordinal: int
    lo: int
    hi: int
    mask: FrozenSet[int]
    stolen: bool
    t_launch: float
    predicted_us: Optional[float]
    t_start: float = 0.0
    t_end: float = 0.0


class Predictor:
    """EMA of microseconds per block, keyed (ordinal, CU count)."""

    def __init__(self, alpha: float):
        self.alpha = alpha
        self.table: Dict[int, Dict[int, float]] = {}

    def us_per_block(self, ordinal: int, cus: int) -> Optional[float]:
        row = self.table.get(ordinal)
        if not row:
            return None
        if cus in row:
            return row[cus]
        c0 = min(row, key=lambda c: (abs(c - cus), -c))
        return row[c0] * c0 / cus          # linear scaling in CUs

    def update(self, ordinal: int, cus: int, blocks: int, actual_us: float) -> None:
        row = self.table.setdefault(ordinal, {})
        v = actual_us / blocks
        row[cus] = v if cus not in row else (1 - self.alpha) * row[cus] + self.alpha * v


@dataclass
class Tenant:
    tid: int
    hp: bool
    quota: FrozenSet[int]
    queue: deque = field(default_factory=deque)      # Kernel or the string "sync"
    cur: Optional[Kernel] = None
    next_block: int = 0
    next_ordinal: int = 0
    outstanding: int = 0
    last_end: float = 0.0                            # device-side stream order
    cur_mask: Optional[FrozenSet[int]] = None        # CU groups of the current kernel's latest atom
    cur_narrow: bool = False                         # right-sizing keeps the current kernel on the quota
    predictor: Predictor = None

    def idle(self) -> bool:
        return self.cur is None and self.outstanding == 0 and not any(
            isinstance(k, Kernel) for k in self.queue)


class Simulator:
    def __init__(self, cfg: SimConfig, latency_us: Callable[[str, int, int], float]):
        """``latency_us(op, cus, blocks)`` is the device's true atom latency."""
        self.cfg = cfg
        self.latency_us = latency_us
        self.tenants: List[Tenant] = []
        self.now = 0.0
        self._events: List[Tuple[float, int, str, object]] = []
        self._seq = 0
        self._kid = 0
        self._aid = 0
        # policy-side timers (predicted) and who set them
        self.busy_until = [0.0] * cfg.n_groups
        self.busy_by = [-1] * cfg.n_groups
        # device-side truth
        self.group_free_at = [0.0] * cfg.n_groups
        self.trace: List[Atom] = []
        self.kernel_done: Dict[int, float] = {}
        self.kernel_submit: Dict[int, float] = {}
        self.kernel_blocks_seen: Dict[int, List[int]] = {}
        self.stats = dict(atoms=0, steals=0, revocations=0, mispredicts=0, predictions=0)
        self.per_tenant: List[Dict[str, int]] = []

    # ---- set-up ----------------------------------------------------------
    def add_tenant(self, quota, hp: bool) -> int:
        t = Tenant(tid=len(self.tenants), hp=hp, quota=frozenset(quota),
                   predictor=Predictor(self.cfg.ema_alpha))
        self.tenants.append(t)
        self.per_tenant.append(dict(atoms=0, steals=0, revocations=0, rightsized=0))
        return t.tid

    def submit_at(self, time: float, tid: int, kernel: Kernel) -> int:
        kernel.kid = self._kid
        self._kid += 1
        self._push(time, "submit", (tid, kernel))
        return kernel.kid

    def sync_at(self, time: float, tid: int) -> None:
        self._push(time, "sync", tid)

    def _push(self, time, kind, payload):
        heapq.heappush(self._events, (time, self._seq, kind, payload))
        self._seq += 1

    # ---- policy ----------------------------------------------------------
    def _choose_mask(self, t: Tenant) -> Tuple[FrozenSet[int], bool]:
        mask = set(t.quota)
        stolen = False
        if self.cfg.steal:
            for o in self.tenants:
                if o.tid == t.tid or not o.idle():
                    continue
                free = [g for g in o.quota
                        if self.busy_until[g] <= self.now or self.busy_by[g] == t.tid]
                if len(free) == len(o.quota):      # whole quota or nothing
                    mask |= o.quota
                    stolen = True
        return frozenset(mask), stolen

    def _choose_blocks(self, t: Tenant, k: Kernel, cus: int) -> Tuple[int, Optional[float]]:
        remaining = k.total_blocks - t.next_block
        upb = t.predictor.us_per_block(k.ordinal, cus)
        if upb is None:
            return remaining, None                  # cold: run whole, learn
        if not self.cfg.atomize:
            return remaining, upb * remaining
        pred_kernel = upb * k.total_blocks
        n = atom_model.atom_count(pred_kernel, self.cfg.atom_duration_us, k.total_blocks)
        b = atom_model.atom_size(k.total_blocks, n, cus * k.wg_per_cu)
        if b >= k.total_blocks and pred_kernel > 2 * self.cfg.atom_duration_us:
            b = atom_model.atom_size(k.total_blocks, n, 1)   # quantum too coarse
        b = min(b, remaining)
        return b, upb * b

    def _dispatch(self, t: Tenant) -> bool:
        limit = self.cfg.max_outstanding
        if t.hp and self.cfg.max_outstanding_hp > 0:
            limit = self.cfg.max_outstanding_hp
        if t.outstanding >= limit:
            return False
        while t.cur is None:
            if not t.queue:
                return False
            head = t.queue.popleft()
            if head == "sync":
                t.next_ordinal = 0                  # batch boundary (Section 4.7)
                continue
            t.cur = head
            t.cur.ordinal = t.next_ordinal
            t.next_ordinal += 1
            t.next_block = 0
            t.cur_mask = None
        k = t.cur
        mask, stolen = self._choose_mask(t)
        if t.next_block == 0:
            # Section 4.5 'Operation', once per kernel (its atoms inherit the allocation): the CU
            # sets on offer are the quota and the quota plus what can be borrowed right now
            t.cur_narrow = False
            if stolen and self.cfg.rightsize_slip >= 1.0:
                own = len(t.quota) * self.cfg.cus_per_group
                wide = len(mask) * self.cfg.cus_per_group
                row = t.predictor.table.get(k.ordinal, {})
                measured = {c: row[c] * k.total_blocks for c in (own, wide) if c in row}
                pick = rightsize_model.online_choice(k.total_blocks, k.wg_per_cu, wide, [own, wide],
                                                     measured, self.cfg.rightsize_slip)
                t.cur_narrow = pick == own
                self.per_tenant[t.tid]["rightsized"] += int(t.cur_narrow)
        if t.cur_narrow:
            mask, stolen = frozenset(t.quota), False
        cus = len(mask) * self.cfg.cus_per_group
        blocks, pred = self._choose_blocks(t, k, cus)
        atom = Atom(aid=self._aid, tenant=t.tid, kid=k.kid, op=k.op, ordinal=k.ordinal,
                    lo=t.next_block, hi=t.next_block + blocks, mask=mask, stolen=stolen,
                    t_launch=self.now, predicted_us=pred)
        self._aid += 1
        t.next_block += blocks
        if t.next_block >= k.total_blocks:
            t.cur = None
        t.outstanding += 1
        # policy timers use the prediction (unknown -> treat as one atom_duration)
        hold = pred if pred is not None else self.cfg.atom_duration_us
        for g in mask:
            self.busy_until[g] = max(self.busy_until[g], self.now) + hold
            self.busy_by[g] = t.tid
        # device truth
        start = max(self.now, t.last_end, max(self.group_free_at[g] for g in mask))
        dur = self.latency_us(k.op, cus, blocks)
        atom.t_start, atom.t_end = start, start + dur
        t.last_end = atom.t_end
        for g in mask:
            self.group_free_at[g] = atom.t_end
        self.trace.append(atom)
        # revocation (Section 4.4 'Operation', second paragraph): the kernel's previous atom ran on
        # groups that this one no longer gets - lent CUs went back at the atom boundary
        revoked = t.cur_mask is not None and len(t.cur_mask - mask) > 0
        t.cur_mask = mask
        for book in (self.stats, self.per_tenant[t.tid]):
            book["atoms"] += 1
            book["steals"] += int(stolen)
            book["revocations"] += int(revoked)
        self._push(atom.t_end, "complete", atom)
        return True

    def _dispatch_all(self) -> None:
        progressed = True
        while progressed:
            progressed = False
            for t in sorted(self.tenants, key=lambda t: (not t.hp, t.tid)):
                if self._dispatch(t):
                    progressed = True

    # ---- event loop ------------------------------------------------------
    def run(self, until: float = float("inf")) -> None:
        while self._events and self._events[0][0] <= until:
            time, _, kind, payload = heapq.heappop(self._events)
            self.now = time
            if kind == "submit":
                tid, k = payload
                self.tenants[tid].queue.append(k)
                self.kernel_submit[k.kid] = time
                self.kernel_blocks_seen[k.kid] = [0] * k.total_blocks
            elif kind == "sync":
                self.tenants[payload].queue.append("sync")
            elif kind == "complete":
                a: Atom = payload
                t = self.tenants[a.tenant]
                t.outstanding -= 1
                actual = a.t_end - a.t_start
                cus = len(a.mask) * self.cfg.cus_per_group
                if a.predicted_us is not None:
                    self.stats["predictions"] += 1
                    if abs(a.predicted_us - actual) > MISPREDICT_US:
                        self.stats["mispredicts"] += 1
                t.predictor.update(a.ordinal, cus, a.hi - a.lo, actual)
                seen = self.kernel_blocks_seen[a.kid]
                for b in range(a.lo, a.hi):
                    seen[b] += 1
                if a.hi == len(seen):
                    self.kernel_done[a.kid] = a.t_end
                for g in a.mask:
                    if self.busy_by[g] == a.tenant and t.outstanding == 0:
                        self.busy_until[g] = min(self.busy_until[g], self.now)
            self._dispatch_all()
