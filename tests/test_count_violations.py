"""Pins for the oracle's all-violations mode (Section 4.5: failures sorted into dataflow and
hardware-constraint violations; Section 6: the verifier as feedback or reward).  Expected
values are hand-written, closed forms of planted damage, the first-violation verifier as
referee for the set of kinds, and for the safety count a brute force over the per-point
sets P(i) that uses neither the live intervals nor the interference edges."""
import numpy as np

from oracle import vlo
from vlgen import gen
from vlgen.mir import Mir
from vlgen.mixed import mixed_mir
from vlgen.tiny import tiny_mir, tiny_rows


def test_hand_written_case():
    # one file of 8 registers; v0 (width 1), v1 (width 2, aligned 2), v2 (width 1)
    # i0: def v0; i1: def v1; i2: def v2, reads v0; i3: reads v1, v2
    # P(i0) = {v0}, P(i1) = {v0, v1}, P(i2) = {v1, v2}, P(i3) = {}: v0-v1 and v1-v2 interfere, v0-v2 do not
    blocks = [[((0,), ()), ((1,), ()), ((2,), (0,)), ((), (1, 2))]]
    m = Mir.build(blocks, [[]], 3, [8], np.zeros(3, np.uint8), np.array([1, 2, 1], np.uint8), np.array([1, 2, 1], np.uint8))
    an = vlo.analyze(m)
    assert list(m.occ_vreg) == [0, 1, 2, 0, 1, 2]

    def counts(row):
        c = vlo.count_violations(m, an, np.array([row], np.uint16))[0]
        return int(c["kinds"]), int(c["n_cons"]), int(c["n_real"]), int(c["n_safe"]), int(c["real_bits"])

    assert counts([2, 4, 2, 2, 4, 2]) == (0, 0, 0, 0, 0)           # v2 reuses the register of v0, which dies at i2
    assert counts([4, 4, 5, 4, 4, 5]) == (4, 0, 0, 2, 0)           # v1 = {4, 5} meets v0 = {4} and v2 = {5}
    assert counts([2, 4, 2, 3, 4, 2]) == (1, 1, 0, 0, 0)           # one stray occurrence of v0
    assert counts([2, 4, 2, 3, 5, 6]) == (1, 3, 0, 0, 0)           # three stray occurrences; the table is still fine
    assert counts([2, 3, 2, 2, 3, 2]) == (2, 0, 1, 0, vlo.BAD_ALIGN)              # v1 = {3, 4}: misaligned, meets nothing
    assert counts([3, 3, 2, 3, 3, 2]) == (2 | 4, 0, 1, 1, vlo.BAD_ALIGN)          # v1 = {3, 4}: misaligned, and on top of v0
    assert counts([0, 7, 1, 0, 7, 1]) == (2, 0, 1, 0, vlo.BAD_BOUNDS | vlo.BAD_ALIGN)   # v1 = {7, 8}: out of the file, odd


def brute_force_safe(m, an, row):
    """pairs a < b of one class that are in some P(i) together and whose tuples overlap"""
    member = vlo.unpack_bits(an.P, m.n_vreg).astype(np.int32)       # [N, V]
    together = (member.T @ member) > 0
    first = np.full(m.n_vreg, -1, np.int64)
    for o in range(m.n_occ - 1, -1, -1):
        first[m.occ_vreg[o]] = o
    n = 0
    for a in range(m.n_vreg):
        for b in range(a + 1, m.n_vreg):
            if not together[a, b] or m.vreg_class[a] != m.vreg_class[b]:
                continue
            pa, pb = int(row[first[a]]), int(row[first[b]])
            if pa < pb + int(m.vreg_width[b]) and pb < pa + int(m.vreg_width[a]):
                n += 1
    return n


def python_counts(m, row):
    first = {}
    for o, v in enumerate(m.occ_vreg):
        first.setdefault(int(v), o)
    n_cons = sum(1 for o, v in enumerate(m.occ_vreg) if row[o] != row[first[int(v)]])
    n_real, bits = 0, 0
    for v, o in first.items():
        p, w, al, c = int(row[o]), int(m.vreg_width[v]), int(m.vreg_align[v]), int(m.vreg_class[v])
        b = 0
        if p + w > int(m.class_size[c]):
            b |= vlo.BAD_BOUNDS
        if p % al:
            b |= vlo.BAD_ALIGN
        if m.class_reserved is not None:
            for r in range(p, p + w):
                if r < 512 and (int(m.class_reserved[c, r >> 5]) >> (r & 31)) & 1:
                    b |= vlo.BAD_RESERVED
        n_real += b != 0
        bits |= b
    return n_cons, n_real, bits


def test_tiny_programs_against_plain_python():
    checked = 0
    for seed in range(120):
        m = tiny_mir(seed, reserved=seed % 3 == 0)
        an = vlo.analyze(m)
        if an.contract != 0:
            continue
        rows = tiny_rows(m, seed, K=6)
        got = vlo.count_violations(m, an, rows)
        ref = vlo.verify(m, an, rows)
        for k in range(len(rows)):
            n_cons, n_real, bits = python_counts(m, rows[k])
            assert (int(got["n_cons"][k]), int(got["n_real"][k]), int(got["real_bits"][k])) == (n_cons, n_real, bits)
            assert int(got["n_safe"][k]) == brute_force_safe(m, an, rows[k])
            kinds = int(got["kinds"][k])
            assert kinds == (n_cons > 0) | ((n_real > 0) << 1) | ((int(got["n_safe"][k]) > 0) << 2)
            # the first-violation verifier reports the lowest kind present
            lowest = 0 if kinds == 0 else 1 + [kinds >> t & 1 for t in range(3)].index(1)
            assert int(ref["status"][k]) == lowest
            checked += 1
    assert checked > 400


def test_planted_damage_on_a_benchmark_kernel():
    k = gen.Kernel(gen.MHA, 0x77, 1500, 1100)
    m = k.mir
    an = vlo.analyze(m, threads=8)
    rows, _ = k.candidates(3, 8, 0, 0)            # undamaged
    base = vlo.count_violations(m, an, rows, threads=8)
    assert (base["kinds"] == 0).all() and (base["n_cons"] == 0).all() and (base["n_safe"] == 0).all()
    rng = np.random.default_rng(9)
    counts_of = np.bincount(m.occ_vreg, minlength=m.n_vreg)
    # j stray occurrences (not first ones) of distinct vregs: n_cons = j, nothing else changes
    for j in (1, 5, 40):
        row = rows[0].copy()
        vs = rng.choice(np.nonzero(counts_of >= 2)[0], j, replace=False)
        for v in vs:
            occ = np.nonzero(m.occ_vreg == v)[0]
            row[occ[int(rng.integers(1, len(occ)))]] += 1
        c = vlo.count_violations(m, an, row[None, :])[0]
        assert (int(c["kinds"]), int(c["n_cons"]), int(c["n_real"]), int(c["n_safe"])) == (1, j, 0, 0)
    # a value moved wholly beyond its file: one realizability violation, and no overlap there
    v = int(rng.integers(0, m.n_vreg))
    row = rows[0].copy()
    row[m.occ_vreg == v] = 600
    c = vlo.count_violations(m, an, row[None, :])[0]
    assert (int(c["kinds"]), int(c["n_cons"]), int(c["n_real"]), int(c["n_safe"])) == (2, 0, 1, 0)
    assert int(c["real_bits"]) & vlo.BAD_BOUNDS
    # a value moved wholly onto the register of one it interferes with: n_safe counts the pairs
    e = an.edges[int(rng.integers(0, len(an.edges)))]
    a, b = int(e["a"]), int(e["b"])
    first = {}
    for o, vv in enumerate(m.occ_vreg):
        first.setdefault(int(vv), o)
    row = rows[0].copy()
    row[m.occ_vreg == a] = row[first[b]]
    c = vlo.count_violations(m, an, row[None, :])[0]
    assert int(c["n_cons"]) == 0 and int(c["n_safe"]) >= 1 and int(c["kinds"]) & 4
    assert int(c["n_safe"]) == brute_force_safe(m, an, row)


def test_mixed_shapes_safety_count_against_brute_force():
    m = mixed_mir(0xD100, n_instr=400, wide_instr=1, reserved=True)
    an = vlo.analyze(m)
    rng = np.random.default_rng(3)
    rows = rng.integers(0, 60, (4, m.n_occ)).astype(np.uint16)
    first = {}
    for o, v in enumerate(m.occ_vreg):
        first.setdefault(int(v), o)
    rows[2] = np.array([rows[2][first[int(v)]] for v in m.occ_vreg], np.uint16)    # a consistent row
    got = vlo.count_violations(m, an, rows)
    for k in range(4):
        assert int(got["n_safe"][k]) == brute_force_safe(m, an, rows[k])
        assert (int(got["n_cons"][k]), int(got["n_real"][k]), int(got["real_bits"][k])) == python_counts(m, rows[k])
    assert got["n_cons"][2] == 0 and got["n_safe"][2] > 0
