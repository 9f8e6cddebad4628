"""Pins for the oracle where a bitset row has several 32-bit words (more than 32 vregs):
path search, the definitions of occupancy / kill flags / maximal runs, interference and the
verdict by enumeration on programs with 65-100 vregs; and, at thousands of instructions, both
oracle verifiers against a register-marking check written from the definition in Python."""
import numpy as np
import pytest

import bruteforce as bf
from oracle import vlo
from vlgen import gen
from vlgen.tiny import tiny_mir, tiny_rows


def sets_of(rows, V):
    return [set(np.nonzero(r)[0].tolist()) for r in vlo.unpack_bits(rows, V)]


def wide_mir(seed, **kw):
    m = tiny_mir(seed, min_vreg=65, max_vreg=100, max_blocks=4, max_instr=12, **kw)
    assert (m.n_vreg + 31) // 32 >= 3
    return m


def rows_from_colouring(m, P, seed, K=8):
    """Rows for programs with many vregs (random tables would nearly all fail the hardware
    rules): a first-fit colouring of the co-occupancy graph read off the brute-force P(i),
    then per row nothing, a stray occurrence, a base outside the file or off its alignment, or
    one value moved onto a neighbour's register."""
    rng = np.random.default_rng([seed, 0xC0])
    V = m.n_vreg
    nb = [set() for _ in range(V)]
    for p in P:
        for a in p:
            for b in p:
                if a != b and m.vreg_class[a] == m.vreg_class[b]:
                    nb[a].add(b)
    rows = np.zeros((K, m.n_occ), np.uint16)
    for k in range(K):
        base = np.full(V, -1, np.int64)
        for v in rng.permutation(V):
            w, al, F = int(m.vreg_width[v]), int(m.vreg_align[v]), int(m.class_size[m.vreg_class[v]])
            res = 0 if m.class_reserved is None else int(sum(int(x) << (32 * t) for t, x in enumerate(m.class_reserved[m.vreg_class[v]])))
            taken = [(int(base[u]), int(m.vreg_width[u])) for u in nb[v] if base[u] >= 0]
            for p in range(0, F - w + 1, al):
                if any(p < q + wq and q < p + w for q, wq in taken) or (res >> p) & ((1 << w) - 1):
                    continue
                base[v] = p
                break
            assert base[v] >= 0, "file too small for a first fit"
        rows[k] = base[m.occ_vreg]
        what = k % 4
        if what == 1:
            o = int(rng.integers(0, m.n_occ))
            rows[k, o] += 1 + int(rng.integers(0, 3))
        elif what == 2:
            v = int(m.occ_vreg[int(rng.integers(0, m.n_occ))])
            bad = int(m.class_size[m.vreg_class[v]]) - int(m.vreg_width[v]) + 1
            if m.vreg_align[v] > 1 and rng.random() < 0.5:
                bad = int(base[v]) + 1
            rows[k, m.occ_vreg == v] = bad
        elif what == 3:
            pairs = [(a, b) for a in range(V) for b in nb[a]]
            if pairs:
                a, b = pairs[int(rng.integers(0, len(pairs)))]
                rows[k, m.occ_vreg == a] = (int(base[b]) // int(m.vreg_align[a])) * int(m.vreg_align[a])
    return rows


def test_points_occupancy_kills_runs_with_several_words():
    members_high = 0
    for seed in range(30):
        m = wide_mir(8000 + seed, early=0.2 if seed % 3 == 0 else 0.0)
        an = vlo.analyze(m, interference=False)
        la = bf.live_after_by_search(m)
        assert sets_of(an.live_after, m.n_vreg) == la, seed
        P = bf.occupancy(m, la)
        assert sets_of(an.P, m.n_vreg) == P, seed
        members_high += sum(1 for p in P for v in p if v >= 32)
        instr = np.repeat(np.arange(m.n_instr), np.diff(m.instr_occ_off))
        _, defs = bf.uses_defs(m)
        for o in range(m.n_occ):
            v, i = int(m.occ_vreg[o]), int(instr[o])
            want = bool(m.occ_flags[o] & 2) and v not in la[i] and v not in defs[i]
            assert bool(an.occ_kill[o]) == want, (seed, o)
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
            assert an.seg[an.seg_off[v]:an.seg_off[v + 1]].tolist() == runs, (seed, v)
            assert an.hull[v].tolist() == ([runs[0][0], runs[-1][1]] if runs else [0, 0]), (seed, v)
            total += sum(e - s for s, e in runs)
        assert total == sum(len(p) for p in P)
    assert members_high > 2000   # the words beyond the first are really exercised


def test_interference_and_verdicts_with_several_words():
    n_status = [0, 0, 0, 0]
    for seed in range(30):
        m = wide_mir(8100 + seed, reserved=seed % 2 == 1)
        m.class_size[:] = 96 if seed % 2 else 200   # room enough for some rows to pass
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
        rows = np.concatenate([rows_from_colouring(m, P, seed), tiny_rows(m, seed, K=2)])
        r1 = vlo.verify(m, an, rows)
        r2 = vlo.verify_points(m, an, rows)
        marked = bf.verify_rows_by_marking(m, vlo.unpack_bits(an.P, m.n_vreg), rows)
        for k in range(len(rows)):
            ref = bf.verify(m, P, rows[k])
            assert tuple(int(x) for x in r1[k]) == ref, (seed, k)
            assert tuple(int(x) for x in r2[k]) == ref, (seed, k)
            assert marked[k] == ref, (seed, k)
            n_status[ref[0]] += 1
    assert all(n >= 30 for n in n_status), n_status


def test_marking_check_agrees_with_enumeration_on_tiny_programs():
    """the Python marking check itself, against the enumeration it stands in for"""
    for seed in range(150):
        m = tiny_mir(8300 + seed, reserved=seed % 2 == 0)
        P = bf.occupancy(m, bf.live_after_by_search(m))
        member = np.zeros((m.n_instr, m.n_vreg), np.uint8)
        for i, p in enumerate(P):
            member[i, sorted(p)] = 1
        rows = tiny_rows(m, seed, K=5)
        got = bf.verify_rows_by_marking(m, member, rows)
        assert got == [bf.verify(m, P, r) for r in rows], seed


@pytest.mark.parametrize("cfg", [2, 3])
def test_every_row_of_configs_2_and_3(cfg):
    """vlo.verify (interference list) on every row of the loop and GEMM-shaped workloads
    against the marking check; on the loop workload also against the literal per-point
    verifier."""
    w = gen.config(cfg)
    m, rows = w.kernels[0].mir, w.rows[0]
    an = vlo.analyze(m, threads=8)
    got = vlo.verify(m, an, rows, threads=8)
    want = bf.verify_rows_by_marking(m, vlo.unpack_bits(an.P, m.n_vreg), rows)
    assert [tuple(int(x) for x in r) for r in got] == want
    assert set(np.unique(got["status"])) >= {0, 3}
    if cfg == 2:
        assert (vlo.verify_points(m, an, rows) == got).all()
