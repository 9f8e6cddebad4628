"""Pins for the CPU oracle: everything here checks the C oracle against
something other than itself (hand-worked examples, cases the paper states,
pure-Python brute force from the definitions, algebraic invariants)."""
import json
import os

import numpy as np
import pytest

import bruteforce as bf
from oracle import vlo
from vlgen.mir import Mir
from vlgen.tiny import tiny_mir, tiny_rows

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def sets_of(rows, V):
    return [set(np.nonzero(r)[0].tolist()) for r in vlo.unpack_bits(rows, V)]


def load_examples():
    with open(os.path.join(GOLD, "worked_examples.json")) as f:
        return json.load(f)["examples"]


def example_mir(ex):
    blocks = [[(tuple(i[0]), tuple(i[1])) for i in blk] for blk in ex["blocks"]]
    return Mir.build(blocks, ex["succ"], ex["n_vreg"], ex["class_size"], name=ex["name"])


@pytest.mark.parametrize("ex", load_examples(), ids=lambda e: e["name"])
def test_worked_examples(ex):
    m = example_mir(ex)
    an = vlo.analyze(m)
    V = m.n_vreg
    assert [set(np.nonzero(r)[0].tolist()) for r in an.live_in] == [set(s) for s in ex["live_in"]]
    assert [set(np.nonzero(r)[0].tolist()) for r in an.live_out] == [set(s) for s in ex["live_out"]]
    assert sets_of(an.live_after, V) == [set(s) for s in ex["live_after"]]
    for v in range(V):
        got = an.seg[an.seg_off[v]:an.seg_off[v + 1]].tolist()
        assert got == ex["segments"].get(str(v), []), v
        if got:
            assert an.hull[v].tolist() == [got[0][0], got[-1][1]]
    assert np.nonzero(an.occ_kill)[0].tolist() == ex["kills"]
    for c in ex["candidates"]:
        row = np.array([c["row"]], np.uint16)
        r = vlo.verify(m, an, row)[0]
        assert [int(x) for x in r] == c["result"], c
        r2 = vlo.verify_points(m, an, row)[0]
        assert [int(x) for x in r2] == c["result"], c


def test_paper_tuple_and_sequential_cases():
    with open(os.path.join(GOLD, "paper_cases.json")) as f:
        g = json.load(f)
    t = g["tuple"]
    # one 64-bit value: def then use
    m = Mir.build([[((0,), ()), ((), (0,))]], [[]], 1, [t["file"]], vreg_width=[t["width"]],
                  vreg_align=[t["align"]])
    an = vlo.analyze(m)
    ok = vlo.verify(m, an, np.full((1, 2), t["ok_base"], np.uint16))[0]
    assert int(ok["status"]) == vlo.OK
    bad = vlo.verify(m, an, np.full((1, 2), t["bad_base"], np.uint16))[0]
    assert [int(x) for x in bad] == [vlo.REALIZABILITY, 0, 0, t["bad_bits"]]
    # the last pair of the file is fine, one further is out of bounds
    edge = vlo.verify(m, an, np.full((1, 2), t["file"] - 2, np.uint16))[0]
    assert int(edge["status"]) == vlo.OK
    over = vlo.verify(m, an, np.full((1, 2), t["file"], np.uint16))[0]
    assert [int(x) for x in over] == [vlo.REALIZABILITY, 0, 0, vlo.BAD_BOUNDS]
    # sequential no-reuse assignment on arbitrary programs with 15 vregs
    s = g["sequential"]
    n = s["last"] - s["first"] + 1
    for seed in range(40):
        mm = tiny_mir(seed, max_vreg=n, max_blocks=4, max_instr=6, two_classes=False, wide=False)
        mm.class_size[:] = 256
        a = vlo.analyze(mm)
        row = (np.arange(mm.n_vreg) + s["first"]).astype(np.uint16)[mm.occ_vreg][None, :]
        assert int(vlo.verify(mm, a, row)[0]["status"]) == vlo.OK


@pytest.mark.parametrize("strict", [True, False])
def test_liveness_against_path_search(strict):
    for seed in range(250):
        m = tiny_mir(seed, strict=strict)
        an = vlo.analyze(m, interference=False)
        want = bf.live_after_by_search(m)
        assert sets_of(an.live_after, m.n_vreg) == want, seed
        # block sets agree with the per-point ones
        uses, defs = bf.uses_defs(m)
        for b in range(m.n_block):
            s, e = int(m.blk_start[b]), int(m.blk_start[b + 1])
            lb_first = uses[s] | (want[s] - defs[s])
            assert set(np.nonzero(an.live_in[b])[0].tolist()) == lb_first, (seed, b)
            assert set(np.nonzero(an.live_out[b])[0].tolist()) == want[e - 1], (seed, b)
        if strict:
            assert an.contract == 0


def test_fixed_point_is_least_on_a_dead_loop():
    # a loop that only passes a value around never makes it live
    m = Mir.build([[((0,), ())], [((1,), ())], [((), ())]], [[1], [1, 2], []], 2)
    an = vlo.analyze(m)
    assert not an.live_in.any() and not an.live_out.any()
    assert an.seg.tolist() == [[0, 1], [1, 2]]


def test_occupancy_kills_segments_against_definitions():
    for seed in range(200):
        m = tiny_mir(1000 + seed)
        an = vlo.analyze(m, interference=False)
        la = bf.live_after_by_search(m)
        P = bf.occupancy(m, la)
        assert sets_of(an.P, m.n_vreg) == P
        blk = np.repeat(np.arange(m.n_instr), np.diff(m.instr_occ_off))
        for o in range(m.n_occ):
            want = bool(m.occ_flags[o] & 2) and int(m.occ_vreg[o]) not in P[blk[o]]
            assert bool(an.occ_kill[o]) == want
        # segments are the maximal runs of membership, and their total length is
        # the total occupancy
        total = 0
        for v in range(m.n_vreg):
            member = [v in P[i] for i in range(m.n_instr)]
            runs, i = [], 0
            while i < m.n_instr:
                if member[i]:
                    j = i
                    while j < m.n_instr and member[j]:
                        j += 1
                    runs.append([i, j])
                    i = j
                else:
                    i += 1
            assert an.seg[an.seg_off[v]:an.seg_off[v + 1]].tolist() == runs
            total += sum(e - s for s, e in runs)
        assert total == sum(len(p) for p in P)


def test_interference_is_cooccupancy():
    for seed in range(150):
        m = tiny_mir(2000 + seed)
        an = vlo.analyze(m)
        P = bf.occupancy(m, bf.live_after_by_search(m))
        want = {}
        for i, p in enumerate(P):
            for a in p:
                for b in p:
                    if a < b and m.vreg_class[a] == m.vreg_class[b]:
                        want.setdefault((a, b), i)
        got = {(int(e["a"]), int(e["b"])): int(e["first"]) for e in an.edges}
        assert got == want, seed


@pytest.mark.parametrize("reserved", [False, True])
def test_verify_against_bruteforce(reserved):
    n_status = [0, 0, 0, 0]
    for seed in range(300):
        m = tiny_mir(3000 + seed, reserved=reserved)
        an = vlo.analyze(m)
        P = bf.occupancy(m, bf.live_after_by_search(m))
        rows = tiny_rows(m, seed, K=6)
        got = vlo.verify(m, an, rows)
        got2 = vlo.verify_points(m, an, rows)
        for k in range(len(rows)):
            want = bf.verify(m, P, rows[k])
            assert tuple(int(x) for x in got[k]) == want, (seed, k)
            assert tuple(int(x) for x in got2[k]) == want, (seed, k)
            n_status[want[0]] += 1
    assert all(n > 20 for n in n_status), n_status


def test_first_violation_is_at_a_defining_instruction():
    """Under the input contract (nothing live into the entry, every block has
    an earlier predecessor) the first co-occupancy point of any pair is an
    instruction defining one of them, so looking only at definitions finds the
    same first violation."""
    checked = 0
    for seed in range(400):
        m = tiny_mir(4000 + seed, strict=True)
        an = vlo.analyze(m)
        if an.contract != 0:
            continue
        P = bf.occupancy(m, bf.live_after_by_search(m))
        _, defs = bf.uses_defs(m)
        for e in an.edges:
            assert int(e["a"]) in defs[int(e["first"])] or int(e["b"]) in defs[int(e["first"])]
        rows = tiny_rows(m, seed, K=4)
        for k in range(len(rows)):
            assert bf.verify(m, P, rows[k]) == bf.verify(m, P, rows[k], def_points_only=True)
            checked += 1
    assert checked > 1000


def test_contract_codes():
    # value live into the entry
    m = Mir.build([[((), (0,))]], [[]], 1)
    assert vlo.analyze(m).contract == 1
    # block 1 only reachable from a later block
    m = Mir.build([[((0,), ())], [((), ())], [((), ())]], [[2], [], [1]], 1)
    assert vlo.analyze(m).contract == 2


def test_shift_invariance_and_use_deletion():
    rng = np.random.default_rng(7)
    for seed in range(120):
        m = tiny_mir(5000 + seed, wide=True)
        m.class_size[:] = 64
        an = vlo.analyze(m)
        rows = tiny_rows(m, seed, K=4)
        base = vlo.verify(m, an, rows)
        # adding a multiple of the largest alignment to every register of every
        # class keeps the verdict (all values stay in bounds: file is 64 wide)
        shifted = rows.copy()
        small = rows < 16
        shifted[small] += 8
        keep = small.all(axis=1)
        got = vlo.verify(m, an, shifted)
        for k in np.nonzero(keep)[0]:
            if base[k]["status"] in (vlo.OK, vlo.SAFETY, vlo.CONSISTENCY):
                assert got[k] == base[k], (seed, k)
        # deleting a USE occurrence never turns OK into SAFETY
        uses = np.nonzero((m.occ_flags & 2) != 0)[0]
        if len(uses) == 0:
            continue
        o = int(rng.choice(uses))
        i = int(np.searchsorted(m.instr_occ_off, o, side="right") - 1)
        off = m.instr_occ_off.copy()
        off[i + 1:] -= 1
        m2 = Mir(m.blk_start, m.succ_off, m.succ, off, np.delete(m.occ_vreg, o),
                 np.delete(m.occ_flags, o), m.vreg_class, m.vreg_width, m.vreg_align, m.class_size)
        an2 = vlo.analyze(m2)
        got2 = vlo.verify(m2, an2, np.delete(rows, o, axis=1))
        for k in range(len(rows)):
            if base[k]["status"] == vlo.OK:
                assert got2[k]["status"] != vlo.SAFETY, (seed, k)
