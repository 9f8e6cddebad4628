"""Early-clobber definitions through the GPU library, against the oracle, exactly: the
hand-written case, tiny random programs with many flagged definitions over several tile
lengths, and programs of mixed shapes large enough for several tiles, with rows coloured
from the oracle's interference graph (which knows the flag) and then disturbed.  Liveness
views, first violations, all-violations counts and decoding masks."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2506_17506_amd as vl  # noqa: E402
from oracle import vlo  # noqa: E402
from vlgen.mir import Mir  # noqa: E402
from vlgen.mixed import mixed_mir  # noqa: E402
from vlgen.tiny import tiny_mir, tiny_rows  # noqa: E402
from test_gpu_parity import assert_liveness_equal, assert_results_equal, free, gpu_analyze, gpu_verify  # noqa: E402
from test_gpu_count_violations import assert_counts_equal, gpu_counts  # noqa: E402
from test_gpu_mixed_shapes import disturbed_rows  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    vl.load()


def check_masks(m, an, hm, hl, rows, queries):
    dev, ld = vl.rows_to_device(rows)
    masks = torch.zeros((len(queries), 16), dtype=torch.int32, device="cuda")
    vl.vl_free_bases_multi([(hm, hl, dev[k], q) for k, q in queries], masks)
    torch.cuda.synchronize()
    got = masks.cpu().numpy().view(np.uint32)
    for j, (k, q) in enumerate(queries):
        assert (got[j] == vlo.free_bases(m, an, rows[k], q)).all(), (m.name, k, q)


def test_hand_written_case():
    # i0: def v0; i1: early-clobber def v1, reads v0 (its last use); i2: reads v1
    m = Mir.build([[((0,), ()), ((("ec", 1),), (0,))], [((), (1,))]], [[1], []], 2, [8])
    an = vlo.analyze(m)
    rows = np.array([[3, 3, 3, 3], [3, 4, 3, 4]], np.uint16)
    want = vlo.verify(m, an, rows)
    assert list(want["status"]) == [3, 0]
    for tile_len in (0, 1):
        hm, hl, got, _ = gpu_analyze([m], tile_len=tile_len, dense=True)
        try:
            assert_liveness_equal(m, an, got[0], "hand-written")
            assert_results_equal(want, gpu_verify(hm, hl, [rows])[0], "hand-written")
            check_masks(m, an, hm[0], hl[0], rows, [(0, q) for q in range(m.n_occ)])
        finally:
            free(hm, hl)


@pytest.mark.parametrize("tile_len", [0, 1, 3])
def test_tiny_programs(tile_len):
    ms, ans, rows = [], [], []
    for seed in range(400):
        m = tiny_mir(seed, reserved=seed % 2 == 1, early=0.5)
        an = vlo.analyze(m)
        if an.contract == 0:
            ms.append(m); ans.append(an); rows.append(tiny_rows(m, seed, K=6))
    assert sum(bool((m.occ_flags & 4).any()) for m in ms) > 150
    hm, hl, got, _ = gpu_analyze(ms, tile_len=tile_len, dense=True)
    try:
        res = gpu_verify(hm, hl, rows)
        cnt = gpu_counts(hm, hl, rows)
        for j, m in enumerate(ms):
            assert_liveness_equal(m, ans[j], got[j], f"{m.name} tile {tile_len}")
            assert_results_equal(vlo.verify(m, ans[j], rows[j]), res[j], f"{m.name} tile {tile_len}")
            assert_counts_equal(vlo.count_violations(m, ans[j], rows[j]), cnt[j], m.name)
    finally:
        free(hm, hl)


def aimed_rows(m, an, accepted, limit=12):
    """Copies of an accepted row in which one early-clobber definition is moved onto the
    register of an operand that dies at its instruction (where alignment and file allow)."""
    first = np.zeros(m.n_vreg, np.int64)
    for o in range(m.n_occ - 1, -1, -1):
        first[m.occ_vreg[o]] = o
    out = []
    for i in range(m.n_instr):
        ops = range(int(m.instr_occ_off[i]), int(m.instr_occ_off[i + 1]))
        ds = [int(m.occ_vreg[o]) for o in ops if m.occ_flags[o] & 4]
        us = [int(m.occ_vreg[o]) for o in ops if an.occ_kill[o]]
        for d in ds:
            for u in us:
                p = int(accepted[first[u]])
                if (u != d and m.vreg_class[u] == m.vreg_class[d] and p % int(m.vreg_align[d]) == 0
                        and p + int(m.vreg_width[d]) <= int(m.class_size[m.vreg_class[d]])):
                    row = accepted.copy()
                    row[m.occ_vreg == d] = p
                    out.append(row)
        if len(out) >= limit:
            break
    return np.array(out[:limit], np.uint16)


@pytest.mark.parametrize("base,n_instr,reserved", [(0xA002, 2500, False), (0xB001, 1500, True)])
def test_mixed_shapes(base, n_instr, reserved):
    m = mixed_mir(base, n_instr=n_instr, reserved=reserved, early=0.3)
    assert ((m.occ_flags & 4) != 0).sum() > 100
    an = vlo.analyze(m, threads=8)
    assert an.contract == 0
    rows = disturbed_rows(m, an, 5, 60)
    want = vlo.verify(m, an, rows, threads=8)
    assert (want["status"] == 0).sum() >= 1 and (want["status"] == 3).sum() >= 1
    extra = aimed_rows(m, an, rows[int(np.nonzero(want["status"] == 0)[0][0])])
    assert len(extra) >= 6
    rows = np.vstack([rows, extra])
    want = vlo.verify(m, an, rows, threads=8)
    # the flag decides these: without it the aimed rows are accepted or fail elsewhere
    plain = Mir(m.blk_start, m.succ_off, m.succ, m.instr_occ_off, m.occ_vreg, m.occ_flags & 3, m.vreg_class,
                m.vreg_width, m.vreg_align, m.class_size, m.class_reserved, "plain")
    other = vlo.verify(plain, vlo.analyze(plain, threads=8), rows, threads=8)
    assert (want["status"][60:] == 3).sum() >= 4 and (other["status"][60:] == 0).sum() >= 4
    rng = np.random.default_rng(base)
    for tile_len in (0, 150):
        hm, hl, got, _ = gpu_analyze([m], tile_len=tile_len, dense=False)
        try:
            assert_liveness_equal(m, an, got[0], f"{m.name} tile {tile_len}")
            assert_results_equal(want, gpu_verify(hm, hl, [rows])[0], f"{m.name} tile {tile_len}")
            assert_counts_equal(vlo.count_violations(m, an, rows, threads=8), gpu_counts(hm, hl, [rows])[0], m.name)
            flagged = np.nonzero(m.occ_flags & 4)[0]
            queries = [(int(rng.integers(0, len(rows))), int(q)) for q in rng.choice(flagged, 80)]
            check_masks(m, an, hm[0], hl[0], rows, queries)
        finally:
            free(hm, hl)


def test_flag_on_a_use_is_rejected():
    m = Mir.build([[((0,), ()), ((), (0,))]], [[]], 1, [8])
    m.occ_flags = m.occ_flags.copy()
    m.occ_flags[1] |= 4
    with pytest.raises(vl.VlError) as e:
        vl.vl_mir_create(m)
    assert e.value.code == -3
