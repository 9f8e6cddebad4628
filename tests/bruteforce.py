"""Pure-Python brute force used to pin the C oracle on tiny programs.

Written straight from the definitions, with no fixed point and no interval
lists: liveness by graph search over instructions, safety by enumerating every
point and every pair.  Only usable for a few dozen instructions.
"""
from __future__ import annotations

import numpy as np

DEF, USE = 1, 2


def instr_block(m):
    blk = np.zeros(m.n_instr, np.int64)
    for b in range(m.n_block):
        blk[m.blk_start[b]:m.blk_start[b + 1]] = b
    return blk


def first_instr_of(m, b, seen=None):
    """Entry points of block b: its first instruction, or (empty block) those of
    its successors."""
    seen = set() if seen is None else seen
    if b in seen:
        return []
    seen.add(b)
    if m.blk_start[b] < m.blk_start[b + 1]:
        return [int(m.blk_start[b])]
    out = []
    for e in range(m.succ_off[b], m.succ_off[b + 1]):
        out += first_instr_of(m, int(m.succ[e]), seen)
    return out


def instr_succ(m):
    blk = instr_block(m)
    succ = []
    for i in range(m.n_instr):
        b = blk[i]
        if i + 1 < m.blk_start[b + 1]:
            succ.append([i + 1])
        else:
            s = []
            for e in range(m.succ_off[b], m.succ_off[b + 1]):
                s += first_instr_of(m, int(m.succ[e]))
            succ.append(sorted(set(s)))
    return succ


def uses_defs(m):
    uses, defs = [], []
    for i in range(m.n_instr):
        u, d = set(), set()
        for o in range(m.instr_occ_off[i], m.instr_occ_off[i + 1]):
            if m.occ_flags[o] & USE:
                u.add(int(m.occ_vreg[o]))
            if m.occ_flags[o] & DEF:
                d.add(int(m.occ_vreg[o]))
        uses.append(u)
        defs.append(d)
    return uses, defs


def live_after_by_search(m):
    """v is live after i iff some path leaves i, reaches an instruction that
    reads v, and no instruction strictly in between writes v."""
    succ = instr_succ(m)
    uses, defs = uses_defs(m)
    res = []
    for i in range(m.n_instr):
        live = set()
        for v in range(m.n_vreg):
            seen, stack, hit = set(), list(succ[i]), False
            while stack and not hit:
                j = stack.pop()
                if j in seen:
                    continue
                seen.add(j)
                if v in uses[j]:
                    hit = True
                elif v not in defs[j]:
                    stack.extend(succ[j])
            if hit:
                live.add(v)
        res.append(live)
    return res


def has_early_clobber(m, i):
    return any(m.occ_flags[o] & 4 for o in range(m.instr_occ_off[i], m.instr_occ_off[i + 1]))


def occupancy(m, live_after):
    """P(i): live after i, or written at i, or (an early-clobber definition at i is written
    before the operands are read) read at i."""
    uses, defs = uses_defs(m)
    return [live_after[i] | defs[i] | (uses[i] if has_early_clobber(m, i) else set()) for i in range(m.n_instr)]


def first_occ(m):
    first = {}
    for o in range(m.n_occ):
        first.setdefault(int(m.occ_vreg[o]), o)
    return first


def realizability_bits(m, v, p):
    c, w, al = int(m.vreg_class[v]), int(m.vreg_width[v]), int(m.vreg_align[v])
    bad = 0
    if p + w > int(m.class_size[c]):
        bad |= 1
    if p % al:
        bad |= 2
    if m.class_reserved is not None:
        for r in range(p, p + w):
            if r < 512 and (int(m.class_reserved[c][r >> 5]) >> (r & 31)) & 1:
                bad |= 4
    return bad


def verify(m, P, row, def_points_only=False):
    """(status, where, a, b) by the definition.  With def_points_only, a pair is
    only examined at instructions that define one of its members (the claim
    that this finds the same first violation is what the GPU walk relies on)."""
    first = first_occ(m)
    for o in range(m.n_occ):
        v = int(m.occ_vreg[o])
        if row[o] != row[first[v]]:
            return (1, o, v, first[v])
    bad = [(first[v], v, realizability_bits(m, v, int(row[first[v]]))) for v in first]
    bad = [t for t in bad if t[2]]
    if bad:
        return (2,) + min(bad)
    _, defs = uses_defs(m)
    for i in range(m.n_instr):
        hits = []
        for a in sorted(P[i]):
            for b in sorted(P[i]):
                if a >= b or m.vreg_class[a] != m.vreg_class[b]:
                    continue
                if def_points_only and a not in defs[i] and b not in defs[i]:
                    continue
                pa, pb = int(row[first[a]]), int(row[first[b]])
                if pa < pb + int(m.vreg_width[b]) and pb < pa + int(m.vreg_width[a]):
                    hits.append((a, b))
        if hits:
            return (3, i) + min(hits)
    return (0, 0, 0, 0)


def verify_rows_by_marking(m, member, rows):
    """(status, where, a, b) per row, again from the definition but usable at thousands of
    instructions: at every instruction the registers of the tuples of P(i)'s members are
    marked, class by class, and a register marked twice is a clash (two members of one class
    whose ranges meet).  `member`: [N, V] 0/1 membership of P(i), every v at most once per i.
    Consistency and realizability as in verify(); the pair of a clash by enumeration at the
    first clashing instruction only."""
    rows = np.asarray(rows).astype(np.int64)
    K = rows.shape[0]
    occ_vreg = np.asarray(m.occ_vreg).astype(np.int64)
    first = np.full(m.n_vreg, -1, np.int64)
    for o in range(m.n_occ - 1, -1, -1):
        first[occ_vreg[o]] = o
    width = np.asarray(m.vreg_width).astype(np.int64)
    align = np.asarray(m.vreg_align).astype(np.int64)
    cls = np.asarray(m.vreg_class).astype(np.int64)
    size = np.asarray(m.class_size).astype(np.int64)
    C = len(size)
    mentioned = np.nonzero(first >= 0)[0]
    pi, pv = np.nonzero(member)          # every (instruction, member of P) once
    # one entry per register of every member's tuple: where register 0 of the class file of
    # that instruction sits in the array of marks, plus the offset inside the tuple
    sel = [np.nonzero(width[pv] > j)[0] for j in range(int(width.max()) if len(pv) else 0)]
    slot0 = np.concatenate([(pi[x] * C + cls[pv[x]]) * 512 + j for j, x in enumerate(sel)] or [np.zeros(0, np.int64)])
    who = np.concatenate([pv[x] for x in sel] or [np.zeros(0, np.int64)])
    out = []
    for k in range(K):
        row = rows[k]
        stray = np.nonzero(row != row[first[occ_vreg]])[0]
        if len(stray):
            o = int(stray[0])
            out.append((1, o, int(occ_vreg[o]), int(first[occ_vreg[o]])))
            continue
        base = np.zeros(m.n_vreg, np.int64)
        base[mentioned] = row[first[mentioned]]
        bad = [(int(first[v]), int(v), realizability_bits(m, int(v), int(base[v]))) for v in mentioned
               if base[v] + width[v] > size[cls[v]] or base[v] % align[v] or m.class_reserved is not None]
        bad = [t for t in bad if t[2]]
        if bad:
            out.append((2,) + min(bad))
            continue
        marks = np.bincount(slot0 + base[who], minlength=m.n_instr * C * 512)
        twice = np.nonzero(marks > 1)[0]
        if len(twice) == 0:
            out.append((0, 0, 0, 0))
            continue
        i = int(twice[0]) // (C * 512)
        here = [int(v) for v in np.nonzero(member[i])[0]]
        hits = [(a, b) for a in here for b in here
                if a < b and cls[a] == cls[b] and base[a] < base[b] + width[b] and base[b] < base[a] + width[a]]
        out.append((3, i) + min(hits))
    return out


# ---- with lane masks: every (vreg, lane) pair is a value of its own ----

def lane_touch(m, occ_lanes, o, j):
    return occ_lanes is None or int(occ_lanes[o]) == 0 or (int(occ_lanes[o]) >> j) & 1


def uses_defs_lanes(m, occ_lanes):
    """per instruction the sets of (vreg, lane) read and written"""
    uses, defs = [], []
    for i in range(m.n_instr):
        u, d = set(), set()
        for o in range(m.instr_occ_off[i], m.instr_occ_off[i + 1]):
            v = int(m.occ_vreg[o])
            for j in range(int(m.vreg_width[v])):
                if not lane_touch(m, occ_lanes, o, j):
                    continue
                if m.occ_flags[o] & USE:
                    u.add((v, j))
                if m.occ_flags[o] & DEF:
                    d.add((v, j))
        uses.append(u)
        defs.append(d)
    return uses, defs


def live_after_lanes_by_search(m, occ_lanes):
    """(v, j) is live after i iff some path leaves i, reaches an instruction that reads lane j
    of v, and no instruction strictly in between writes that lane."""
    succ = instr_succ(m)
    uses, defs = uses_defs_lanes(m, occ_lanes)
    lanes = [(v, j) for v in range(m.n_vreg) for j in range(int(m.vreg_width[v]))]
    res = []
    for i in range(m.n_instr):
        live = set()
        for x in lanes:
            seen, stack, hit = set(), list(succ[i]), False
            while stack and not hit:
                k = stack.pop()
                if k in seen:
                    continue
                seen.add(k)
                if x in uses[k]:
                    hit = True
                elif x not in defs[k]:
                    stack.extend(succ[k])
            if hit:
                live.add(x)
        res.append(live)
    return res


def occupancy_lanes(m, occ_lanes, live_after):
    uses, defs = uses_defs_lanes(m, occ_lanes)
    return [live_after[i] | defs[i] | (uses[i] if has_early_clobber(m, i) else set()) for i in range(m.n_instr)]


def verify_lanes(m, P, row):
    """(status, where, a, b): consistency and realizability per vreg as in verify(); safety by
    enumerating, at every instruction, every pair of lanes of different vregs of one class."""
    first = first_occ(m)
    for o in range(m.n_occ):
        v = int(m.occ_vreg[o])
        if row[o] != row[first[v]]:
            return (1, o, v, first[v])
    bad = [(first[v], v, realizability_bits(m, v, int(row[first[v]]))) for v in first]
    bad = [t for t in bad if t[2]]
    if bad:
        return (2,) + min(bad)
    for i in range(m.n_instr):
        hits = []
        for (a, ja) in P[i]:
            for (b, jb) in P[i]:
                if a < b and m.vreg_class[a] == m.vreg_class[b] and int(row[first[a]]) + ja == int(row[first[b]]) + jb:
                    hits.append((a, b))
        if hits:
            return (3, i) + min(hits)
    return (0, 0, 0, 0)
