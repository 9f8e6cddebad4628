"""Container for a machine-IR kernel as flat arrays (inputs only, no analysis).

This module belongs to the seeded input generators.  It holds none of the
method's arithmetic: it only stores and checks the shape of a program
description, so that the CPU oracle and the GPU binding can both be fed from
the same inputs without importing each other.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Iterable, Sequence

import numpy as np

OCC_DEF = 1
OCC_USE = 2
OCC_EARLY = 4   # on a DEF: written before the instruction has read its operands


@dataclass
class Mir:
    """Instructions 0..N-1 in one linear order; block b is the contiguous range
    [blk_start[b], blk_start[b+1]); occurrences (operand slots) are numbered in
    instruction order, then operand order."""
    blk_start: np.ndarray      # uint32 [n_block+1]
    succ_off: np.ndarray       # uint32 [n_block+1]
    succ: np.ndarray           # uint32 [n_edge]
    instr_occ_off: np.ndarray  # uint32 [n_instr+1]
    occ_vreg: np.ndarray       # uint32 [n_occ]
    occ_flags: np.ndarray      # uint8  [n_occ]  OCC_DEF | OCC_USE
    vreg_class: np.ndarray     # uint8  [n_vreg]
    vreg_width: np.ndarray     # uint8  [n_vreg]  in 32-bit registers
    vreg_align: np.ndarray     # uint8  [n_vreg]
    class_size: np.ndarray     # uint16 [n_class]
    class_reserved: np.ndarray | None = None  # uint32 [n_class,16] or None
    name: str = ""
    occ_lanes: np.ndarray | None = None       # uint32 [n_occ]: lanes of the vreg's tuple the occurrence accesses
                                              # (bit j = lane j; 0 = all), or None: every occurrence accesses all
    meta: dict = field(default_factory=dict)

    def __post_init__(self):
        c = np.ascontiguousarray
        self.blk_start = c(self.blk_start, dtype=np.uint32)
        self.succ_off = c(self.succ_off, dtype=np.uint32)
        self.succ = c(self.succ, dtype=np.uint32)
        self.instr_occ_off = c(self.instr_occ_off, dtype=np.uint32)
        self.occ_vreg = c(self.occ_vreg, dtype=np.uint32)
        self.occ_flags = c(self.occ_flags, dtype=np.uint8)
        self.vreg_class = c(self.vreg_class, dtype=np.uint8)
        self.vreg_width = c(self.vreg_width, dtype=np.uint8)
        self.vreg_align = c(self.vreg_align, dtype=np.uint8)
        self.class_size = c(self.class_size, dtype=np.uint16)
        if self.class_reserved is not None:
            self.class_reserved = c(self.class_reserved, dtype=np.uint32).reshape(-1, 16)
        if self.occ_lanes is not None:
            self.occ_lanes = c(self.occ_lanes, dtype=np.uint32)

    @property
    def n_instr(self) -> int:
        return len(self.instr_occ_off) - 1

    @property
    def n_vreg(self) -> int:
        return len(self.vreg_class)

    @property
    def n_block(self) -> int:
        return len(self.blk_start) - 1

    @property
    def n_occ(self) -> int:
        return len(self.occ_vreg)

    @property
    def n_class(self) -> int:
        return len(self.class_size)

    @property
    def n_edge(self) -> int:
        return len(self.succ)

    @property
    def words(self) -> int:
        return (self.n_vreg + 31) // 32

    @staticmethod
    def build(blocks: Sequence[Sequence[tuple]], succ: Sequence[Iterable[int]],
              n_vreg: int, class_size: Sequence[int] = (4,),
              vreg_class=None, vreg_width=None, vreg_align=None,
              class_reserved=None, name: str = "") -> "Mir":
        """Readable constructor for small hand-written programs.

        blocks[b] is a list of instructions; an instruction is a tuple
        (defs, uses) of vreg-id sequences, operands listed defs first.
        A vreg id may be given as ('du', v) inside defs to make a single
        occurrence that is both DEF and USE, or as ('ec', v) to make an
        early-clobber DEF."""
        blk_start = [0]
        occ_off = [0]
        occ_v, occ_f = [], []
        for blk in blocks:
            for defs, uses in blk:
                for d in defs:
                    if isinstance(d, tuple):
                        occ_v.append(d[1])
                        occ_f.append(OCC_DEF | (OCC_EARLY if d[0] == "ec" else OCC_USE))
                    else:
                        occ_v.append(d)
                        occ_f.append(OCC_DEF)
                for u in uses:
                    occ_v.append(u)
                    occ_f.append(OCC_USE)
                occ_off.append(len(occ_v))
            blk_start.append(len(occ_off) - 1)
        s_off, s = [0], []
        for ss in succ:
            s.extend(ss)
            s_off.append(len(s))
        z = lambda x, d: np.full(n_vreg, d, np.uint8) if x is None else np.asarray(x, np.uint8)
        return Mir(blk_start, s_off, s, occ_off, occ_v, occ_f, z(vreg_class, 0),
                   z(vreg_width, 1), z(vreg_align, 1), np.asarray(class_size, np.uint16),
                   class_reserved, name)
