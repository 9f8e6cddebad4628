"""GPU library against the CPU oracle on programs of mixed operand shapes:
tuples of width 1..32 whose alignment is not always the width or a power of two
(word-crossing tuples, the general realizability test), three register files,
reserved registers, instructions with dozens of operands, values not mentioned
for thousands of operand slots (links far beyond the verifier's window, one of
them beyond the 16-bit distance field), and candidate values far outside any
file.  Candidate rows start from a colouring of the oracle's interference graph
and are then disturbed, so that first violations lie deep inside the program.
Every comparison is exact."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2506_17506_amd as vl  # noqa: E402
from oracle import vlo  # noqa: E402
from vlgen.mixed import mixed_mir  # noqa: E402
from test_gpu_parity import (assert_liveness_equal, assert_results_equal, free, gpu_analyze,  # noqa: E402
                             gpu_verify)


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    vl.load()


def coloured_table(m, an, rng):
    """One base register per vreg such that interfering vregs are disjoint, as far as
    a randomized first fit over the oracle's interference edges manages (a vreg that
    finds no room gets register 0 and makes the row fail, which is fine)."""
    V = m.n_vreg
    adj = [[] for _ in range(V)]
    for a, b in zip(an.edges["a"], an.edges["b"]):
        adj[a].append(b)
        adj[b].append(a)
    res = m.class_reserved
    table = np.full(V, -1, np.int64)
    order = np.argsort(an.first + rng.integers(0, 3, V))
    for v in order:
        c, w, al = int(m.vreg_class[v]), int(m.vreg_width[v]), int(m.vreg_align[v])
        F = int(m.class_size[c])
        taken = np.zeros(F + 64, bool)
        if res is not None:
            for r in range(F):
                taken[r] = (res[c, r >> 5] >> (r & 31)) & 1
        for u in adj[v]:
            if table[u] >= 0 and m.vreg_class[u] == c:
                taken[table[u]:table[u] + int(m.vreg_width[u])] = True
        starts = list(range(0, F - w + 1, al))
        if len(starts) > 1 and rng.random() < 0.5:
            k = int(rng.integers(0, len(starts)))
            starts = starts[k:] + starts[:k]
        table[v] = 0
        for p in starts:
            if not taken[p:p + w].any():
                table[v] = p
                break
    return table


def disturbed_rows(m, an, seed, K):
    rng = np.random.default_rng(seed)
    rows = np.zeros((K, m.n_occ), np.uint16)
    counts = np.bincount(m.occ_vreg, minlength=m.n_vreg)
    mentioned = np.nonzero(counts > 0)[0]
    for k in range(K):
        table = coloured_table(m, an, rng)
        row = table[m.occ_vreg].astype(np.int64)
        kind = k % 8
        if kind == 1:      # one occurrence of a much-mentioned value differs
            v = int(rng.choice(np.nonzero(counts >= 3)[0]))
            occ = np.nonzero(m.occ_vreg == v)[0]
            row[occ[int(rng.integers(1, len(occ)))]] += 1
        elif kind == 2:    # the last occurrence of a value differs (longest link)
            v = int(rng.choice(mentioned))
            occ = np.nonzero(m.occ_vreg == v)[0]
            row[occ[-1]] ^= 1
        elif kind == 3:    # a whole value moved onto its neighbour's register
            v = int(rng.choice(mentioned))
            row[m.occ_vreg == v] = (table[v] + int(m.vreg_width[v]) - 1) % int(m.class_size[m.vreg_class[v]])
        elif kind == 4:    # values outside any file
            v = int(rng.choice(mentioned))
            row[m.occ_vreg == v] = int(rng.choice([511, 512, 600, 4095, 65535]))
        elif kind == 5:    # one occurrence outside any file
            row[int(rng.integers(0, m.n_occ))] = int(rng.choice([513, 1023, 65535]))
        elif kind == 6:    # two values swapped
            a, b = rng.choice(mentioned, 2)
            row[m.occ_vreg == a], row[m.occ_vreg == b] = table[b], table[a]
        rows[k] = row.astype(np.uint16)
    return rows


def run_case(m, K, seed, tile_lens):
    an = vlo.analyze(m, threads=8)
    assert an.contract == 0
    rows = disturbed_rows(m, an, seed, K)
    want = vlo.verify(m, an, rows, threads=8)
    assert (want["status"] == 0).sum() >= 1, "no candidate of this case is accepted: the case tests less than it should"
    assert len(np.unique(want["status"])) >= 3
    for tile_len in tile_lens:
        hm, hl, got, views = gpu_analyze([m], tile_len=tile_len, dense=False)
        try:
            assert_liveness_equal(m, an, got[0], f"{m.name} tile {tile_len}")
            for aligned in (True, False):
                res = gpu_verify(hm, hl, [rows], aligned=aligned)[0]
                assert_results_equal(want, res, f"{m.name} tile {tile_len} aligned {aligned}")
        finally:
            free(hm, hl)
    return want


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_mixed_shapes(seed):
    m = mixed_mir(0xA000 + seed, n_instr=2500)
    run_case(m, K=72, seed=seed, tile_lens=[0, 300])


def test_mixed_shapes_with_reserved_registers():
    m = mixed_mir(0xB001, n_instr=1500, reserved=True)
    run_case(m, K=40, seed=11, tile_lens=[0, 64])


def test_gap_beyond_the_distance_field():
    """The globals are read at the very end, more than 65,535 operand slots after their
    previous mention."""
    m = mixed_mir(0xC001, n_instr=700, stretch=23000)
    assert m.n_occ > 70000
    run_case(m, K=16, seed=21, tile_lens=[0])


def test_many_blocks_times_many_words():
    """150 blocks and over 200 bitset words, with vreg numbers that are never mentioned: the
    block summaries of most slices of the sorted entries do not fit the on-chip table and
    take the other path, the last slice fits."""
    from vlgen.mixed import many_blocks_mir
    m = many_blocks_mir(7, gap=96)
    assert m.n_block == 150 and (m.n_vreg + 31) // 32 > 500 and m.n_occ > 12 * 1024
    run_case(m, K=24, seed=31, tile_lens=[0, 100])


def test_thousands_of_clashes_in_one_call():
    """Two programs with 5,000 candidates each, nearly all of which fail on safety (one value
    moved onto the register of a value it interferes with): the pairs of far more failing
    candidates than there are workgroups to look for them."""
    mirs = [mixed_mir(0xD001, n_instr=500), mixed_mir(0xD002, n_instr=700)]
    rows_list, wants = [], []
    for j, m in enumerate(mirs):
        an = vlo.analyze(m, threads=8)
        assert an.contract == 0
        rng = np.random.default_rng(100 + j)
        table = coloured_table(m, an, rng)
        a, b = np.asarray(an.edges["a"]), np.asarray(an.edges["b"])
        same = ((m.vreg_class[a] == m.vreg_class[b]) & (m.vreg_width[a] == m.vreg_width[b]) &
                (m.vreg_align[a] == m.vreg_align[b]))
        a, b = a[same], b[same]
        assert len(a) > 100
        K = 5000
        rows = np.tile(table[m.occ_vreg].astype(np.uint16), (K, 1))
        for k in range(1, K):   # row 0 stays as coloured
            e = int(rng.integers(0, len(a)))
            rows[k, m.occ_vreg == a[e]] = table[b[e]]
        rows_list.append(rows)
        wants.append(vlo.verify(m, an, rows, threads=8))
    assert sum(int((w["status"] == 3).sum()) for w in wants) > 8000
    hm, hl, _, _ = gpu_analyze(mirs, dense=False)
    try:
        for res, want, m in zip(gpu_verify(hm, hl, rows_list), wants, mirs):
            assert_results_equal(want, res, m.name)
    finally:
        free(hm, hl)


def test_more_candidates_than_the_list_of_clashes_holds_at_first():
    """Calls with 70,000 and then 120,000 candidates on one stream, most of them failing on
    safety: the library's list of candidates whose pair has to be found grows twice (it
    starts with room for 65,536), each time after the stream has drained."""
    from vlgen.tiny import tiny_mir
    m = None
    for seed in range(500, 600):
        c = tiny_mir(seed, max_blocks=4, max_instr=8, max_vreg=10)
        an = vlo.analyze(c)
        if an.contract == 0 and len(an.edges["a"]) >= 6 and c.n_occ >= 30:
            m = c
            break
    assert m is not None
    rng = np.random.default_rng(9)
    table = coloured_table(m, an, rng)
    a, b = np.asarray(an.edges["a"]), np.asarray(an.edges["b"])
    same = ((m.vreg_class[a] == m.vreg_class[b]) & (m.vreg_width[a] == m.vreg_width[b]) &
            (m.vreg_align[a] == m.vreg_align[b]))
    a, b = a[same], b[same]
    assert len(a) >= 2
    hm, hl, _, _ = gpu_analyze([m], dense=False)
    try:
        for K in (70000, 120000, 300):
            rows = np.tile(table[m.occ_vreg].astype(np.uint16), (K, 1))
            pick = rng.integers(0, len(a), K)
            for e in range(len(a)):   # row k: value a[pick] moved onto the register of b[pick]
                sel = np.nonzero(pick == e)[0]
                sel = sel[sel % 5 != 0]   # every fifth row stays as coloured
                cols = np.nonzero(m.occ_vreg == a[e])[0]
                rows[np.ix_(sel, cols)] = table[b[e]]
            want = vlo.verify(m, an, rows, threads=8)
            assert (want["status"] == 3).sum() > K // 2
            assert_results_equal(want, gpu_verify(hm, hl, [rows])[0], f"K {K}")
    finally:
        free(hm, hl)
