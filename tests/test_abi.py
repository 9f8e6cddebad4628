"""The C-ABI library without a GPU: it loads, exports every symbol the header
declares, maps error codes to text, and rejects malformed programs before any
device call."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2506_17506_amd as vl
from paper_2506_17506_amd import binding
from vlgen.mir import Mir

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "vl.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vl_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = vl.load()
    names = declared_symbols()
    assert {"vl_mir_create", "vl_liveness", "vl_liveness_multi", "vl_verify_batch", "vl_verify_multi",
            "vl_live_get", "vl_strerror", "vl_summarize_multi", "vl_free_bases_multi", "vl_count_violations_multi", "vl_bank_conflicts", "vl_verify_multi_occ_major"} <= set(names)
    for n in names:
        assert getattr(lib, n) is not None, n


def test_error_strings():
    for code in range(0, -9, -1):
        assert vl.vl_strerror(code) and "unknown" not in vl.vl_strerror(code)
    assert "unknown" in vl.vl_strerror(-99)


def ok_mir():
    return Mir.build([[((0,), ()), ((1,), (0,))], [((), (1,))]], [[1], []], 2, [8])


def create_code(m):
    try:
        h = vl.vl_mir_create(m)
    except vl.VlError as e:
        return e.code
    vl.vl_mir_destroy(h)
    return 0


def test_validation_rejects_malformed_programs_before_touching_the_device():
    cases = []
    m = ok_mir(); m.occ_vreg[0] = 7; cases.append((m, -3))                 # vreg id out of range
    m = ok_mir(); m.vreg_width[0] = 0; cases.append((m, -3))               # width 0
    m = ok_mir(); m.vreg_width[0] = 33; cases.append((m, -3))              # width > 32
    m = ok_mir(); m.vreg_align[1] = 0; cases.append((m, -3))               # align 0
    m = ok_mir(); m.class_size[0] = 513; cases.append((m, -3))             # file > 512
    m = ok_mir(); m.vreg_class[0] = 1; cases.append((m, -3))               # class out of range
    m = ok_mir(); m.occ_flags[0] = 4; cases.append((m, -3))                # unknown flag bit
    m = ok_mir(); m.succ[0] = 5; cases.append((m, -3))                     # successor out of range
    m = ok_mir(); m.blk_start[1] = 0; cases.append((m, -4))                # empty block
    m = ok_mir(); m.blk_start[2] = 2; cases.append((m, -4))                # blocks do not cover N
    m = ok_mir(); m.succ_off[1] = 0; m.succ_off[2] = 1; m.succ[0] = 0; cases.append((m, -4))  # no earlier pred
    m = ok_mir(); m.instr_occ_off[1] = 3; m.instr_occ_off[2] = 2; cases.append((m, -2))       # offsets decrease
    m = Mir.build([[(tuple(range(40)), tuple(range(40)))]], [[]], 40, [64]); cases.append((m, -3))  # 80 operands
    for m, want in cases:
        assert create_code(m) == want, (want, m)
    # more vregs than a bitset row in LDS has room for: refused here, so that no launch can
    # fail for want of LDS later
    big = 491520 + 1
    m = ok_mir()
    m.vreg_class, m.vreg_width, m.vreg_align = np.zeros(big, np.uint8), np.ones(big, np.uint8), np.ones(big, np.uint8)
    assert create_code(m) == -3
    # a well-formed program passes validation; without a GPU the device copy then fails
    assert create_code(ok_mir()) in (0, -6)


def test_lane_masks_are_validated_before_touching_the_device():
    lib = vl.load()

    def code(m, lanes):
        d, keep = binding.make_desc(m)
        out = C.c_void_p()
        a = np.ascontiguousarray(lanes, np.uint32)
        rc = lib.vl_mir_create_lanes(C.byref(d), a.ctypes.data_as(C.c_void_p), C.byref(out))
        if rc == 0:
            lib.vl_mir_destroy(out)
        return rc
    m = Mir.build([[((0,), ()), ((1,), (0,))], [((), (1,))]], [[1], []], 2, [8], vreg_width=[2, 1], vreg_align=[2, 1])
    assert code(m, [0, 0, 1, 0]) in (0, -6)          # lane 0 of the two-register vreg: fine (no GPU: the copy fails)
    assert code(m, [0, 0, 4, 0]) == -3               # lane 2 of a vreg of width 2
    assert code(m, [0, 2, 0, 0]) == -3               # lane 1 of a vreg of width 1
    # five operands of width 16, one of them accessed in part: 5 x 17 occurrences after rewriting
    wide = Mir.build([[((0, 1, 2, 3, 4), ()), ((), (0, 1, 2, 3, 4))]], [[]], 5, [512], vreg_width=[16] * 5, vreg_align=[16] * 5)
    lanes = np.zeros(10, np.uint32)
    assert code(wide, lanes) in (0, -6)
    for o in range(5, 10):
        lanes[o] = 1
    assert code(wide, lanes) == -3


def test_null_arguments():
    lib = vl.load()
    assert lib.vl_mir_create(None, None) == -1
    assert lib.vl_verify_multi(None, 1, None) == -1
    assert lib.vl_mir_create_lanes(None, None, None) == -1
    assert lib.vl_mir_lanes_get(None, None) == -1
    assert lib.vl_lanes_expand(None, None, 1, 1, None, 1, None) == -1
    assert lib.vl_verify_batch_static(None, None, None, 1, 1, None, None) in (-1, -6)
    assert lib.vl_verify_batch_static(None, None, None, 65537, 1, None, None) == -8
    assert lib.vl_verify_multi_occ_major(None, 1, None) == -1
    assert lib.vl_summarize_multi(None, 1, None, None, None) == -1
    assert lib.vl_free_bases_multi(None, 1, None, None) == -1
    assert lib.vl_count_violations_multi(None, 1, None) == -1
    assert lib.vl_bank_conflicts(None, None, 1, 1, 4, None, None) == -1
    assert lib.vl_liveness_multi(None, 1, 0, 0, None, None) == -1
    assert lib.vl_live_get(None, None) == -1
    lib.vl_mir_destroy(None)
    lib.vl_live_destroy(None)
