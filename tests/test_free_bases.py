"""Pins for the oracle's constrained-decoding mask (Section 4.5, last sentence of the
error analysis: mask out the registers that are occupied during generation).  None
of the expected values comes from the function under test: hand-written cases, closed
forms, and the verifier itself as referee: where no value is written twice an allocation
decoded under the mask must verify (two values then overlap exactly when one is live
where the other is written), the registers of an accepted allocation must be offered,
and putting a value on a base the mask withholds must make the verifier reject the
allocation."""
import numpy as np

from oracle import vlo
from vlgen.mir import Mir
from vlgen.mixed import mixed_mir
from vlgen.tiny import tiny_mir


def bits(mask):
    return [p for p in range(512) if (int(mask[p >> 5]) >> (p & 31)) & 1]


def test_hand_written_case():
    # one file of 8 registers.  i0: def v0 (width 1); i1: def v1 (width 2, aligned 2);
    # i2: def v2 (width 1), reads v0; i3: reads v1, v2
    blocks = [[((0,), ()), ((1,), ()), ((2,), (0,)), ((), (1, 2))]]
    m = Mir.build(blocks, [[]], 3, [8], np.zeros(3, np.uint8), np.array([1, 2, 1], np.uint8), np.array([1, 2, 1], np.uint8))
    an = vlo.analyze(m)
    row = np.zeros(m.n_occ, np.uint16)
    # occurrences: 0 = v0 def, 1 = v1 def, 2 = v2 def, 3 = v0 use, 4 = v1 use, 5 = v2 use
    assert list(m.occ_vreg) == [0, 1, 2, 0, 1, 2]
    assert bits(vlo.free_bases(m, an, row, 0)) == list(range(8))          # nothing is live yet
    row[0] = 2
    assert bits(vlo.free_bases(m, an, row, 1)) == [0, 4, 6]               # pairs, not the one holding register 2
    row[1] = 4
    # v0 dies at i2, where v2 is written: its register is free again; v1 holds 4 and 5
    assert bits(vlo.free_bases(m, an, row, 2)) == [0, 1, 2, 3, 6, 7]
    row[2] = 2
    assert bits(vlo.free_bases(m, an, row, 3)) == [2]                     # v0 again: only its own register
    assert bits(vlo.free_bases(m, an, row, 4)) == [4]
    row[3], row[4], row[5] = 2, 4, 2
    assert vlo.verify(m, an, row[None, :])["status"][0] == 0


def test_first_definition_sees_only_the_hardware_rules():
    """Nothing is live at the program's first definition: every aligned base that fits and
    touches no reserved register is offered."""
    for seed in range(4):
        m = mixed_mir(0xD000 + seed, n_instr=300, reserved=seed % 2 == 1)
        an = vlo.analyze(m, interference=False)
        row = np.zeros(m.n_occ, np.uint16)
        v = int(m.occ_vreg[0])
        c, w, al = int(m.vreg_class[v]), int(m.vreg_width[v]), int(m.vreg_align[v])
        F = int(m.class_size[c])
        res = m.class_reserved
        want = []
        for p in range(0, 512):
            free = all(r < 512 and not (res is not None and (int(res[c, r >> 5]) >> (r & 31)) & 1) for r in range(p, p + w))
            if p % al == 0 and p + w <= F and free:
                want.append(p)
        assert bits(vlo.free_bases(m, an, row, 0)) == want


def decode(m, an, rng=None):
    """Emits the occurrences in order, each time taking a base the mask offers (the lowest,
    or a random one).  Returns the row, or None when some mask was empty."""
    row = np.zeros(m.n_occ, np.uint16)
    for q in range(m.n_occ):
        offered = bits(vlo.free_bases(m, an, row, q))
        if not offered:
            return None
        row[q] = offered[0] if rng is None else offered[int(rng.integers(0, len(offered)))]
    return row


def programs():
    out = [mixed_mir(0xE000 + s, n_instr=260, wide_instr=1, reserved=s % 2 == 0) for s in range(3)]
    out += [tiny_mir(s, max_blocks=5, max_instr=6, max_vreg=7) for s in range(60)]
    return out


def written_once(m):
    defs = np.bincount(m.occ_vreg[(m.occ_flags & 1) != 0], minlength=m.n_vreg)
    return bool((defs <= 1).all())


def test_decoding_under_the_mask_gives_allocations_that_verify():
    """The mask looks at what is occupied where the value is written (the paper's wording),
    which settles every overlap when each value is written once; a value written again
    later, while something newer is live, is beyond it."""
    rng = np.random.default_rng(3)
    progs = [mixed_mir(0xF000 + s, n_instr=300, wide_instr=1, reserved=s % 2 == 0, redefine=False) for s in range(5)]
    progs += [m for m in (tiny_mir(s, max_blocks=5, max_instr=6, max_vreg=7) for s in range(1500)) if written_once(m)]
    done = 0
    for m in progs:
        assert written_once(m)
        an = vlo.analyze(m)
        if an.contract != 0:
            continue
        for chooser in (None, rng):
            row = decode(m, an, chooser)
            if row is None:          # the files of the tiny programs are small: the decoder may run out
                continue
            assert vlo.verify(m, an, row[None, :])["status"][0] == 0, m.name
            assert vlo.verify_points(m, an, row[None, :])["status"][0] == 0, m.name
            done += 1
    assert done >= 20, done


def test_accepted_registers_are_offered_and_withheld_bases_are_rejected():
    rng = np.random.default_rng(4)
    checked_in, checked_out = 0, 0
    for m in programs():
        an = vlo.analyze(m)
        if an.contract != 0:
            continue
        row = decode(m, an, rng)
        if row is None or vlo.verify(m, an, row[None, :])["status"][0] != 0:
            continue
        first = np.full(m.n_vreg, -1, np.int64)
        for o in range(m.n_occ - 1, -1, -1):
            first[m.occ_vreg[o]] = o
        step = max(1, m.n_occ // 60)
        for q in range(0, m.n_occ, step):
            v = int(m.occ_vreg[q])
            mask = vlo.free_bases(m, an, row, q)
            offered = bits(mask)
            assert int(row[q]) in offered                      # what the accepted allocation chose
            checked_in += 1
            if first[v] != q:
                assert offered == [int(row[first[v]])]         # a later mention: only its own register
                continue
            F = int(m.class_size[m.vreg_class[v]])
            withheld = [p for p in range(min(F + 2, 512)) if p not in offered]
            for p in withheld[:: max(1, len(withheld) // 6)]:
                bad = row.copy()
                bad[m.occ_vreg == v] = p                       # the whole value moves to a withheld base
                assert vlo.verify_points(m, an, bad[None, :])["status"][0] != 0, (m.name, q, p)
                checked_out += 1
    assert checked_in >= 300 and checked_out >= 300
