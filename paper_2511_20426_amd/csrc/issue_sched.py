"""Issue-slot model of a gfx950 wave and a list scheduler over it, shared by the generators of
the hand-scheduled kernels (attention core, GEMM core).

Measured on gfx950 with one wave per SIMD (cycle counter around loops of MFMAs with fillers): the
wave issues one instruction per 4 cycles whatever its kind; an MFMA 32x32x16 holds the issue port
for 8 cycles and the matrix pipe for 32, so the 32 cycles from one MFMA to the next have room for
6 more issue quanta of 4 cycles.  v_exp_f32 takes 2 quanta, ds_read_b128 2.2, v_readlane 2, a
global->LDS load 2.7, a branch that is not taken 2.5 (5 if it directly follows the instruction
that sets its condition), everything else (VALU, SALU, s_waitcnt, s_nop) 1.  Whatever exceeds
8 quanta between two MFMAs delays the second one by the full excess; there is no carry-over of
slack between slots.
"""
from __future__ import annotations


def quanta(line):
    op = line.split()[0]
    if op.endswith(":") or op.startswith(";"):
        return 0.0
    if op.startswith("v_mfma"):
        return 2.0
    if op.startswith("v_exp"):
        return 2.0
    if op.startswith(("ds_read_b128", "ds_write_b128")):
        return 2.2
    if op.startswith("v_readlane"):
        return 2.0
    if op.startswith("global_load"):
        return 2.7
    if op.startswith("s_cbranch"):
        return 2.5
    return 1.0


class Atom:
    """Instructions that stay together, with the earliest slot they may issue in (`ready`, or
    `gap` slots after the latest of the atoms in `after`), the slot they should issue by
    (`deadline`, the scheduling priority) and the slot they must issue by (`hard`)."""
    def __init__(self, lines, ready=0, deadline=31, after=(), gap=0, tag=None, hard=31):
        self.lines = list(lines)
        self.cost = sum(quanta(l) for l in self.lines)
        self.ready, self.deadline, self.tag, self.hard = ready, deadline, tag, hard
        self.after = [(a, gap) for a in after]            # (atom, slots that must lie between)
        self.slot = None

    def ready_slot(self):
        r = self.ready
        for a, gap in self.after:
            if a.slot is None:
                return None
            r = max(r, a.slot + gap)
        return r


def schedule(fixed_load, atoms, cap):
    """Earliest-deadline-first list scheduling of `atoms` into len(fixed_load) slots of `cap`
    quanta each.  fixed_load[i]: quanta already spoken for in slot i (the MFMA and whatever is
    pinned to it).  Returns per-slot lists of atoms, in issue order."""
    n = len(fixed_load)
    placed = [[] for _ in range(n)]
    pending = list(atoms)
    widest = cap - min(fixed_load)                       # an atom larger than this fits no slot:
    for i in range(n):                                    # it takes one that holds nothing else yet
        room = cap - fixed_load[i]
        while True:
            cands = [a for a in pending if a.ready_slot() is not None and a.ready_slot() <= i]
            cands.sort(key=lambda a: a.deadline)
            pick = None
            for a in cands:
                oversize = a.cost > widest + 1e-9 and not placed[i] and room >= widest - 1e-9
                if a.cost <= room + 1e-9 or a.hard <= i or oversize:
                    pick = a
                    break
            if pick is None:
                break
            pick.slot = i
            placed[i].append(pick)
            pending.remove(pick)
            room -= pick.cost
    assert not pending, [a.lines for a in pending]
    return placed
