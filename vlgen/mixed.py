"""Seeded programs of mixed operand shapes, for parity tests away from the
benchmark's regular kernels.

Input generation only (none of the method's arithmetic): tuples of every width
from 1 to 32 with alignments that are not always a power of two and not always
the width (so that a correctly placed tuple may cross a 32-register word),
three register files of 40 / 300 / 512 registers, values that are not mentioned
for hundreds or thousands of operand slots, instructions with dozens of
operands, loops and a diamond.  Every value is written before it is read on
every path: globals in the entry block, locals inside the block that uses them.
"""
from __future__ import annotations

import numpy as np

from .mir import Mir

WIDTHS = [1] * 8 + [2] * 4 + [3, 4, 4, 5, 8, 16, 32]


def _attrs(rng, V: int):
    vclass = rng.choice([0, 1, 1, 2, 2, 2], V).astype(np.uint8)
    width = rng.choice(WIDTHS, V).astype(np.uint8)
    width[vclass == 0] = np.minimum(width[vclass == 0], 4)      # the small file
    kind = rng.random(V)
    align = np.where(kind < 0.6, width, np.where(kind < 0.8, 1, np.where(kind < 0.9, 2, 3))).astype(np.uint8)
    return vclass, width, align


def mixed_mir(seed: int, n_instr: int = 2500, n_global: int = 24, reserved: bool = False,
              wide_instr: int = 4, stretch: int = 0, redefine: bool = True, early: float = 0.0) -> Mir:
    """n_instr instructions (about) in 7 blocks: entry, a loop of two blocks, a
    diamond, a second loop, exit.  `wide_instr` instructions carry 40-60
    operands.  `stretch` > 0 appends that many filler instructions before the
    exit block, which reads the globals once more (a gap of many operand slots
    between two mentions of one value).  With redefine=False no value is written
    twice (no redefinitions, no read-modify-write operands).  `early`: share of the
    defining instructions whose first plain definition is early-clobber."""
    rng = np.random.default_rng(seed)
    n_blocks = 7
    per = max(8, n_instr // n_blocks)
    n_local = per // 2
    V = n_global + n_local * n_blocks
    vclass, width, align = _attrs(rng, V)
    # globals stay narrow so that they all fit next to the locals
    width[:n_global] = np.minimum(width[:n_global], 2)
    align[:n_global] = np.where(align[:n_global] > width[:n_global], 1, align[:n_global])
    succ = [[1], [2], [1, 3], [4, 5], [5], [5, 6], []]
    blocks = []
    wide_at = set(int(x) for x in rng.integers(0, n_blocks * per, wide_instr))
    for b in range(n_blocks):
        blk = []
        lo = n_global + b * n_local
        born = []          # locals written so far in this block
        if b == 0:
            for g in range(0, n_global, 3):
                blk.append((list(range(g, min(n_global, g + 3))), []))
        if b == n_blocks - 1 and stretch:
            filler = lo
            blk.append(([filler], []))
            born.append(filler)
            for _ in range(stretch):
                blk.append(([], [filler, filler, filler]))
        for i in range(per):
            wide = (b * per + i) in wide_at
            nd = int(rng.integers(12, 20)) if wide else int(rng.choice([0, 1, 1, 1, 2]))
            nu = int(rng.integers(25, 40)) if wide else int(rng.choice([1, 2, 2, 3]))
            defs, uses = [], []
            n_before = len(born)    # only values written by earlier instructions may be read
            for _ in range(nu):
                r = rng.random()
                if n_before and r < 0.85:
                    back = min(n_before, 1 + int(rng.geometric(0.15)))       # recent
                    uses.append(born[n_before - back])
                elif n_before and r < 0.90:
                    back = min(n_before, int(rng.integers(1, 120)))           # a long gap
                    uses.append(born[n_before - back])
                else:
                    uses.append(int(rng.integers(0, n_global)))
            for _ in range(nd):
                r = rng.random()
                if r < 0.8 and len(born) < n_local:
                    v = lo + len(born)
                    born.append(v)
                    defs.append(v)
                elif not redefine:
                    pass
                elif n_before and r < 0.9:
                    defs.append(born[n_before - min(n_before, int(rng.integers(1, 40)))])        # redefinition
                elif n_before:
                    defs.append(("du", born[n_before - min(n_before, int(rng.integers(1, 40)))]))  # read-modify-write
                else:
                    defs.append(int(rng.integers(0, n_global)))
            blk.append((defs, uses))
        if b == n_blocks - 1:
            blk.append(([], list(range(n_global))))
        blocks.append(blk)
    if early > 0:   # marks drawn from a stream of their own: the programs stay what they were
        rng_e = np.random.default_rng([seed, 0xEC])
        for blk in blocks:
            for k, (defs, uses) in enumerate(blk):
                plain = [j for j, d in enumerate(defs) if not isinstance(d, tuple)]
                if plain and uses and rng_e.random() < early:
                    defs = list(defs)
                    defs[plain[0]] = ("ec", defs[plain[0]])
                    blk[k] = (defs, uses)
    res = None
    if reserved:
        res = np.zeros((3, 16), np.uint32)
        for c, F in enumerate((40, 300, 512)):
            for r in rng.integers(0, F, 3):
                res[c, int(r) >> 5] |= np.uint32(1 << (int(r) & 31))
    return Mir.build(blocks, succ, V, (40, 300, 512), vclass, width, align, res, name=f"mixed{seed}")


def many_blocks_mir(seed: int, n_blocks: int = 150, per: int = 40, n_global: int = 12, gap: int = 8) -> Mir:
    """A long chain of small blocks with extra forward and backward edges: many
    blocks times many bitset words.  Each block writes its own locals before it
    reads them and reads the globals (written in the entry block); `gap` vreg
    numbers after each block's locals are never mentioned at all."""
    rng = np.random.default_rng(seed)
    n_local = per // 2
    stride = n_local + gap
    V = n_global + n_blocks * stride
    vclass, width, align = _attrs(rng, V)
    width[:] = np.minimum(width, 4)
    align[:] = np.where(align > width, 1, align)
    width[:n_global] = 1
    align[:n_global] = 1
    succ, blocks = [], []
    for b in range(n_blocks):
        s = [b + 1] if b + 1 < n_blocks else []
        if s and rng.random() < 0.3:
            t = int(rng.integers(1, n_blocks))
            if t not in s:
                s.append(t)
        succ.append(s)
        blk = []
        lo = n_global + b * stride
        born = []
        if b == 0:
            for g in range(0, n_global, 3):
                blk.append((list(range(g, min(n_global, g + 3))), []))
        for _ in range(per):
            uses = []
            for _ in range(int(rng.choice([1, 2, 2, 3]))):
                if born and rng.random() < 0.85:
                    uses.append(born[-min(len(born), 1 + int(rng.geometric(0.3)))])
                else:
                    uses.append(int(rng.integers(0, n_global)))
            defs = []
            if len(born) < n_local and rng.random() < 0.7:
                defs.append(lo + len(born))
            blk.append((defs, uses))
            born.extend(defs)
        blocks.append(blk)
    return Mir.build(blocks, succ, V, (40, 300, 512), vclass, width, align, None, name=f"chain{seed}")
