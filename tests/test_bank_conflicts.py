"""Pins for the oracle's register-bank conflict score (Section 2: registers come in banks,
four on NVIDIA GPUs; reading several values from one bank costs a cycle per extra value;
the FFMA of the overview figure reads R4, R6 and R9 because they lie in different banks).  Expected
values: the paper's example, hand-written cases, closed forms, and a plain Python count."""
import json
import os

import numpy as np

from oracle import vlo
from vlgen.mir import Mir
from vlgen.mixed import mixed_mir


def ffma(widths=(1, 1, 1, 1)):
    """one instruction: v3 = f(v0, v1, v2), preceded by the three definitions"""
    w = np.array(widths, np.uint8)
    blocks = [[((0,), ()), ((1,), ()), ((2,), ()), ((3,), (0, 1, 2))]]
    return Mir.build(blocks, [[]], 4, [256], np.zeros(4, np.uint8), w, np.ones(4, np.uint8))


def row_for(m, regs):
    return np.array([[regs[v] for v in m.occ_vreg]], np.uint16)


def test_the_example_of_the_paper():
    m = ffma()
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_cases.json")) as f:
        case = json.load(f)["ffma_banks"]
    # R4, R6, R9: banks 0, 2, 1 of four: no stall.  (The destination is not read.)
    assert vlo.bank_conflicts(m, row_for(m, case["reads"] + [4]), case["n_banks"])[0] == case["stalls"] == 0
    # R4, R8, R9: two values from bank 0: one extra cycle
    assert vlo.bank_conflicts(m, row_for(m, [4, 8, 9, 5]), 4)[0] == 1
    # R4, R8, R12: all three from bank 0: two extra cycles
    assert vlo.bank_conflicts(m, row_for(m, [4, 8, 12, 5]), 4)[0] == 2


def test_hand_written_cases():
    # a pair at base 2 reads registers 2 and 3; with a single at 6 (bank 2) the worst bank delivers two
    m = ffma((2, 1, 1, 1))
    assert vlo.bank_conflicts(m, row_for(m, [2, 6, 9, 0]), 4)[0] == 1
    assert vlo.bank_conflicts(m, row_for(m, [2, 4, 9, 0]), 4)[0] == 0      # banks 2, 3 | 0 | 1
    # a tuple of eight covers every one of four banks twice by itself
    m = ffma((8, 1, 1, 1))
    assert vlo.bank_conflicts(m, row_for(m, [8, 16, 17, 0]), 4)[0] == 2    # banks 0 and 1 deliver three each
    # the same value read by two operands is read once
    blocks = [[((0,), ()), ((1,), (0, 0, 0))]]
    m2 = Mir.build(blocks, [[]], 2, [256], np.zeros(2, np.uint8), np.ones(2, np.uint8), np.ones(2, np.uint8))
    assert vlo.bank_conflicts(m2, row_for(m2, [4, 8]), 4)[0] == 0
    # one bank: everything queues up; as many banks as registers in use: nothing does
    m = ffma()
    assert vlo.bank_conflicts(m, row_for(m, [4, 6, 9, 4]), 1)[0] == 2
    assert vlo.bank_conflicts(m, row_for(m, [4, 6, 9, 4]), 32)[0] == 0


def python_score(m, row, n_banks):
    total = 0
    for i in range(m.n_instr):
        seen, banks = set(), {}
        for o in range(int(m.instr_occ_off[i]), int(m.instr_occ_off[i + 1])):
            v = int(m.occ_vreg[o])
            if not (m.occ_flags[o] & 2) or v in seen:
                continue
            seen.add(v)
            for j in range(int(m.vreg_width[v])):
                b = (int(row[o]) + j) % n_banks
                banks[b] = banks.get(b, 0) + 1
        if banks:
            total += max(banks.values()) - 1
    return total


def test_mixed_programs_against_plain_python():
    rng = np.random.default_rng(12)
    for seed in range(3):
        m = mixed_mir(0xBA00 + seed, n_instr=300, wide_instr=2)
        rows = rng.integers(0, 500, (5, m.n_occ)).astype(np.uint16)
        rows[4] = 65535                                    # sums past 16 bits must not wrap
        for n_banks in (1, 3, 4, 8, 32):
            got = vlo.bank_conflicts(m, rows, n_banks)
            assert [int(x) for x in got] == [python_score(m, rows[k], n_banks) for k in range(5)]


def test_closed_form_every_read_from_one_bank():
    """All registers multiples of the bank count and all values single: an instruction that
    reads n distinct values stalls n - 1 cycles."""
    m = mixed_mir(0xBA10, n_instr=200, wide_instr=1)
    ones = Mir(m.blk_start, m.succ_off, m.succ, m.instr_occ_off, m.occ_vreg, m.occ_flags, m.vreg_class,
               np.ones_like(m.vreg_width), np.ones_like(m.vreg_align), m.class_size, None, "ones")
    row = (ones.occ_vreg.astype(np.uint32) * 4 % 65536).astype(np.uint16)[None, :]
    want = 0
    for i in range(ones.n_instr):
        o0, o1 = int(ones.instr_occ_off[i]), int(ones.instr_occ_off[i + 1])
        # distinct (vreg, register) reads; two vregs whose registers coincide modulo 65536 still count twice
        n = len({int(ones.occ_vreg[o]) for o in range(o0, o1) if ones.occ_flags[o] & 2})
        want += max(0, n - 1)
    assert vlo.bank_conflicts(ones, row, 4)[0] == want
