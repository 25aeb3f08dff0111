"""CPU model of kernel atomization (LithOS Section 4.4, Algorithm 1).

TEST INFRASTRUCTURE ONLY.  Pure Python, integer arithmetic, written for
reading, not for speed.

A launch with logical grid (gx, gy, gz) has ``total = gx*gy*gz`` thread
blocks.  Algorithm 1 numbers them ``idx = z*gy*gx + y*gx + x`` and an atom is
a half-open range ``[lo, hi)`` of those numbers; non-overlapping ranges that
cover ``[0, total)`` run every block exactly once.

Two ways of executing an atom are modelled:

* ``run_atom_prelude`` - the paper's: launch the full grid, each block
  computes its linear index and exits unless it falls in ``[lo, hi)``.
* ``run_atom_remap`` - the build's: launch only ``hi - lo`` workgroups; the
  hardware workgroup number ``h`` is turned into the logical index
  ``lo + pi(h)`` for a bijection ``pi`` of ``[0, hi-lo)``, and the logical
  index is un-flattened with the same formula read backwards.

Both must visit the same blocks.
"""
from __future__ import annotations

import math
from typing import Callable, Iterable, List, Sequence, Tuple

Grid = Tuple[int, int, int]
Block = Tuple[int, int, int]


def total_blocks(grid: Grid) -> int:
    gx, gy, gz = grid
    if gx <= 0 or gy <= 0 or gz <= 0:
        raise ValueError("grid dimensions must be positive")
    return gx * gy * gz


def linearize(block: Block, grid: Grid) -> int:
    """Algorithm 1: idx = z*gy*gx + y*gx + x."""
    x, y, z = block
    gx, gy, _ = grid
    return z * gy * gx + y * gx + x


def delinearize(idx: int, grid: Grid) -> Block:
    """Inverse of :func:`linearize` (x fastest)."""
    gx, gy, _ = grid
    return (idx % gx, (idx // gx) % gy, idx // (gx * gy))


def decompose(grid: Grid, atom_blocks: int) -> List[Tuple[int, int]]:
    """Cut [0,total) into consecutive atoms of ``atom_blocks`` blocks.

    ``atom_blocks`` of 0 or >= total means "do not atomize": one atom.
    The last atom holds the remainder.
    """
    total = total_blocks(grid)
    if atom_blocks < 0:
        raise ValueError("atom_blocks must be >= 0")
    if atom_blocks == 0 or atom_blocks >= total:
        return [(0, total)]
    n = -(-total // atom_blocks)
    return [(i * atom_blocks, min((i + 1) * atom_blocks, total)) for i in range(n)]


def identity_pi(h: int, n: int) -> int:
    return h


def xcd_interleave_pi(h: int, n: int, n_xcd: int = 8) -> int:
    """Bijection of [0,n) that undoes round-robin placement over ``n_xcd`` dies.

    Hardware workgroup ``h`` lands on die ``h % n_xcd`` as its ``h // n_xcd``-th
    workgroup.  Die ``x`` is given a contiguous run of logical slots: the first
    ``r = n % n_xcd`` dies get ``q+1 = n//n_xcd + 1`` slots, the rest ``q``.
    """
    q, r = divmod(n, n_xcd)
    x, s = h % n_xcd, h // n_xcd
    return x * q + min(x, r) + s


def run_atom_remap(lo: int, hi: int, grid: Grid,
                   pi: Callable[[int, int], int] = identity_pi) -> List[Block]:
    """Blocks visited by a launch of hi-lo workgroups with index remapping."""
    n = hi - lo
    return [delinearize(lo + pi(h, n), grid) for h in range(n)]


def run_atom_prelude(lo: int, hi: int, grid: Grid) -> List[Block]:
    """Blocks that survive the range test of Algorithm 1 in a full-grid launch."""
    gx, gy, gz = grid
    out = []
    for z in range(gz):
        for y in range(gy):
            for x in range(gx):
                idx = z * gy * gx + y * gx + x
                if lo <= idx < hi:
                    out.append((x, y, z))
    return out


def visit_counts(grid: Grid, atoms: Iterable[Tuple[int, int]],
                 pi: Callable[[int, int], int] = identity_pi) -> List[int]:
    """How many times each logical block is executed over a set of atoms."""
    counts = [0] * total_blocks(grid)
    for lo, hi in atoms:
        for blk in run_atom_remap(lo, hi, grid, pi):
            counts[linearize(blk, grid)] += 1
    return counts


def atom_count(predicted_us: float, atom_duration_us: float, total: int) -> int:
    """Section 4.4 'Operation': predicted duration / atom_duration.

    The quotient is rounded up and clamped to [1, total] (a kernel cannot be
    cut finer than one block per atom; "up to 64 atoms" for 64 blocks).
    """
    if atom_duration_us <= 0:
        raise ValueError("atom_duration must be positive")
    n = math.ceil(predicted_us / atom_duration_us) if predicted_us > 0 else 1
    return max(1, min(n, total))


def atom_size(total: int, n_atoms: int, quantum: int = 1) -> int:
    """Blocks per atom for ``n_atoms`` atoms, rounded up to a launch quantum.

    ``quantum`` is the number of workgroups the assigned CUs hold at once
    (CUs x resident workgroups per CU); whole multiples keep the tail of each
    atom from idling CUs.
    """
    if n_atoms <= 1:
        return total
    b = -(-total // n_atoms)
    if quantum > 1:
        b = -(-b // quantum) * quantum
    return min(b, total)
