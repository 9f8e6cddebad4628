"""Pins for early-clobber definitions in the oracle.  A definition flagged early-clobber is
written before its instruction has read the operands, so it cannot take the register of an
operand even if that operand dies there (the paper's Safety condition, Section 3.4, applied
to the earlier write; Section 2: values with overlapping life cycles need disjoint
registers).  Expected values are hand-written or come from the pure-Python brute force
(path-search liveness, all pairs at every point), which knows the flag on its own."""
import numpy as np
import pytest

import bruteforce as bf
from oracle import vlo
from vlgen.mir import Mir
from vlgen.tiny import tiny_mir, tiny_rows


def two_instructions(early):
    d = ("ec", 1) if early else 1
    return Mir.build([[((0,), ()), ((d,), (0,))], [((), (1,))]], [[1], []], 2, [8])


def test_hand_written_case():
    # i0: def v0; i1: def v1, reads v0 (its last use); i2: reads v1
    plain, early = two_instructions(False), two_instructions(True)
    a_plain, a_early = vlo.analyze(plain), vlo.analyze(early)
    same = np.array([[3, 3, 3, 3]], np.uint16)       # v1 takes over the register of v0
    apart = np.array([[3, 4, 3, 4]], np.uint16)
    assert vlo.verify(plain, a_plain, same)["status"][0] == 0
    r = vlo.verify(early, a_early, same)[0]
    assert (int(r["status"]), int(r["where"]), int(r["a"]), int(r["b"])) == (3, 1, 0, 1)
    assert vlo.verify(early, a_early, apart)["status"][0] == 0
    # occupancy at i1, intervals and kill flags
    assert list(vlo.unpack_bits(a_plain.P, 2)[1]) == [0, 1] and list(vlo.unpack_bits(a_early.P, 2)[1]) == [1, 1]
    assert a_plain.seg[a_plain.seg_off[0]:a_plain.seg_off[1]].tolist() == [[0, 1]]
    assert a_early.seg[a_early.seg_off[0]:a_early.seg_off[1]].tolist() == [[0, 2]]
    assert list(a_plain.occ_kill) == list(a_early.occ_kill) == [0, 0, 1, 1]   # the reads are last uses either way
    assert len(a_plain.edges) == 0 and [(int(e["a"]), int(e["b"]), int(e["first"])) for e in a_early.edges] == [(0, 1, 1)]
    # the decoding mask withholds the operand's register, the all-violations mode counts the pair
    assert not (int(vlo.free_bases(early, a_early, same[0], 1)[0]) >> 3) & 1
    assert (int(vlo.free_bases(plain, a_plain, same[0], 1)[0]) >> 3) & 1
    assert int(vlo.count_violations(early, a_early, same)["n_safe"][0]) == 1


@pytest.mark.parametrize("reserved", [False, True])
def test_tiny_programs_against_bruteforce(reserved):
    checked, with_flag, differs = 0, 0, 0
    for seed in range(300):
        m = tiny_mir(seed, reserved=reserved, early=0.4)
        an = vlo.analyze(m)
        if an.contract != 0:
            continue
        la = bf.live_after_by_search(m)
        P = bf.occupancy(m, la)
        assert [set(np.nonzero(r)[0]) for r in vlo.unpack_bits(an.P, m.n_vreg)] == P
        with_flag += any(m.occ_flags & 4)
        rows = tiny_rows(m, seed, K=6)
        # one more row, aimed at the flag: consistent, and an early-clobber definition sits on
        # the register of an operand that dies at its instruction
        first = {}
        for o, v in enumerate(m.occ_vreg):
            first.setdefault(int(v), o)
        aimed = np.array([rows[0][first[int(v)]] for v in m.occ_vreg], np.uint16)
        for i in range(m.n_instr):
            ops = range(int(m.instr_occ_off[i]), int(m.instr_occ_off[i + 1]))
            ds = [int(m.occ_vreg[o]) for o in ops if m.occ_flags[o] & 4]
            us = [int(m.occ_vreg[o]) for o in ops if an.occ_kill[o]]
            if ds and us and ds[0] != us[0] and m.vreg_class[ds[0]] == m.vreg_class[us[0]]:
                aimed[m.occ_vreg == ds[0]] = aimed[first[us[0]]]
                break
        rows = np.vstack([rows, aimed[None, :]])
        got = vlo.verify(m, an, rows)
        pts = vlo.verify_points(m, an, rows)
        plain = Mir(m.blk_start, m.succ_off, m.succ, m.instr_occ_off, m.occ_vreg, m.occ_flags & 3, m.vreg_class,
                    m.vreg_width, m.vreg_align, m.class_size, m.class_reserved, "plain")
        other = vlo.verify(plain, vlo.analyze(plain), rows)
        for k in range(len(rows)):
            want = bf.verify(m, P, rows[k])
            assert (int(got["status"][k]), int(got["where"][k]), int(got["a"][k]), int(got["b"][k])) == want
            assert (int(pts["status"][k]), int(pts["where"][k]), int(pts["a"][k]), int(pts["b"][k])) == want
            differs += int(other["status"][k]) != want[0] or int(other["where"][k]) != want[1]
            checked += 1
    assert checked > 1000 and with_flag > 100
    assert differs >= 4          # the flag matters in these cases: some verdicts change without it
