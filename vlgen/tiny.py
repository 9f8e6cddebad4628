"""Seeded random tiny programs and candidate rows for brute-force testing.

Input generation only: draws shapes and operands from a numpy Generator and
holds none of the method's arithmetic.
"""
from __future__ import annotations

import numpy as np

from .mir import Mir, OCC_DEF, OCC_USE


def tiny_mir(seed: int, strict: bool = True, max_blocks: int = 4, max_instr: int = 4,
             max_vreg: int = 6, two_classes: bool = True, wide: bool = True,
             reserved: bool = False, early: float = 0.0, min_vreg: int = 1) -> Mir:
    """A random CFG of up to max_blocks blocks in which every non-entry block
    has a predecessor placed before it.  With strict, the entry block first
    defines every vreg, so nothing is live into the program.  `early`: share of
    the defining instructions whose first plain definition is early-clobber.
    `min_vreg` above 32 gives bitset rows of several words."""
    rng = np.random.default_rng(seed)
    nb = int(rng.integers(1, max_blocks + 1))
    V = int(rng.integers(min_vreg, max_vreg + 1))
    n_class = 2 if (two_classes and V >= 2 and rng.random() < 0.5) else 1
    vclass = rng.integers(0, n_class, V).astype(np.uint8)
    width = np.ones(V, np.uint8)
    if wide:
        width = rng.choice([1, 1, 1, 2, 4], V).astype(np.uint8)
    align = np.where(rng.random(V) < 0.7, width, 1).astype(np.uint8)
    class_size = rng.integers(4, 9, n_class).astype(np.uint16)
    succ = [set() for _ in range(nb)]
    for b in range(1, nb):
        succ[int(rng.integers(0, b))].add(b)
    for b in range(nb):
        for t in range(nb):
            if rng.random() < 0.25:
                succ[b].add(t)
    blocks = []
    for b in range(nb):
        blk = []
        if b == 0 and strict:
            order = rng.permutation(V)
            i = 0
            while i < V:
                k = int(rng.integers(1, 3))
                blk.append(([int(x) for x in order[i:i + k]], []))
                i += k
        for _ in range(int(rng.integers(1, max_instr + 1))):
            nd = int(rng.choice([0, 1, 1, 1, 2]))
            nu = int(rng.choice([0, 1, 2, 2, 3]))
            defs = [int(x) for x in rng.integers(0, V, nd)]
            if defs and rng.random() < 0.15:
                defs[0] = ("du", defs[0])
            uses = [int(x) for x in rng.integers(0, V, nu)]
            blk.append((defs, uses))
        blocks.append(blk)
    if early > 0:   # marks drawn from a stream of their own: the programs stay what they were
        rng_e = np.random.default_rng([seed, 0xEC])
        for blk in blocks:
            for k, (defs, uses) in enumerate(blk):
                plain = [j for j, d in enumerate(defs) if not isinstance(d, tuple)]
                if plain and rng_e.random() < early:
                    defs = list(defs)
                    defs[plain[0]] = ("ec", defs[plain[0]])
                    blk[k] = (defs, uses)
    res = None
    if reserved:
        res = np.zeros((n_class, 16), np.uint32)
        for c in range(n_class):
            if rng.random() < 0.7:
                r = int(rng.integers(0, class_size[c]))
                res[c, r >> 5] |= np.uint32(1 << (r & 31))
    return Mir.build(blocks, [sorted(s) for s in succ], V, class_size, vclass, width, align,
                     res, name=f"tiny{seed}")


def tiny_rows(m: Mir, seed: int, K: int = 8) -> np.ndarray:
    """K candidate rows: a random table per row, expanded to occurrences, with
    occasional single-occurrence disturbances and out-of-range values."""
    rng = np.random.default_rng(seed)
    rows = np.zeros((K, m.n_occ), np.uint16)
    for k in range(K):
        table = np.zeros(m.n_vreg, np.int64)
        for v in range(m.n_vreg):
            F = int(m.class_size[m.vreg_class[v]])
            a = int(m.vreg_align[v])
            if rng.random() < 0.8:
                table[v] = int(rng.integers(0, max(1, (F - int(m.vreg_width[v])) // a + 1))) * a
            else:
                table[v] = int(rng.integers(0, F + 2))
        rows[k] = table[m.occ_vreg]
        if m.n_occ and rng.random() < 0.25:
            rows[k, int(rng.integers(0, m.n_occ))] = int(rng.integers(0, 8))
        if m.n_occ and rng.random() < 0.05:
            rows[k, int(rng.integers(0, m.n_occ))] = 0xFFFF
    return rows


__all__ = ["tiny_mir", "tiny_rows", "OCC_DEF", "OCC_USE"]


def tiny_lanes(m: Mir, seed: int, share: float = 0.5, keep_first_block: bool = True) -> np.ndarray:
    """Random lane masks for the occurrences of a program: with probability `share` an
    occurrence of a vreg wider than one register accesses a random non-empty subset of its
    lanes, otherwise all of them (mask 0).  With keep_first_block the entry block is left
    alone, so that a program whose entry block writes every vreg whole stays strict."""
    rng = np.random.default_rng([seed, 0x1A])
    lanes = np.zeros(m.n_occ, np.uint32)
    first_block_end = int(m.instr_occ_off[m.blk_start[1]]) if keep_first_block else 0
    for o in range(first_block_end, m.n_occ):
        w = int(m.vreg_width[m.occ_vreg[o]])
        if w > 1 and rng.random() < share:
            lanes[o] = int(rng.integers(1, 1 << w))
    return lanes


__all__ += ["tiny_lanes"]
