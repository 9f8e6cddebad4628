"""Degenerate and extreme shapes through every entry point, against the oracle: a program
without operands or vregs, vregs that are never mentioned, instructions with the maximum of
64 operands over eight register files with tuples of every power-of-two width."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2506_17506_amd as vl  # noqa: E402
from oracle import vlo  # noqa: E402
from vlgen.mir import Mir  # noqa: E402
from test_gpu_parity import assert_liveness_equal, assert_results_equal, free, gpu_analyze, gpu_verify  # noqa: E402
from test_gpu_count_violations import assert_counts_equal, gpu_counts  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    vl.load()


def no_operands(n_vreg):
    z = np.zeros(n_vreg, np.uint8)
    return Mir.build([[((), ()), ((), ())], [((), ())]], [[1], []], n_vreg, [8], z, z + 1, z + 1)


@pytest.mark.parametrize("n_vreg", [0, 3])
def test_program_without_operands(n_vreg):
    m = no_operands(n_vreg)
    an = vlo.analyze(m)
    rows = np.zeros((3, 1), np.uint16)          # a pitch of one element: there is nothing to read
    hm, hl, got, _ = gpu_analyze([m], dense=False)
    try:
        assert_liveness_equal(m, an, got[0], "no operands")
        assert_results_equal(vlo.verify(m, an, rows), gpu_verify(hm, hl, [rows])[0], "no operands")
        assert_counts_equal(vlo.count_violations(m, an, rows), gpu_counts(hm, hl, [rows], calls=2)[0], "no operands")
        masks = torch.zeros((1, 16), dtype=torch.int32, device="cuda")
        with pytest.raises(vl.VlError) as e:
            vl.vl_free_bases_multi([(hm[0], hl[0], masks, 0)], masks)    # no occurrence to ask about
        assert e.value.code == -2
    finally:
        free(hm, hl)


def test_widest_instructions_over_eight_files():
    V = 64
    vclass = (np.arange(V) % 8).astype(np.uint8)
    width = np.array([1, 2, 4, 8, 16, 32, 3, 5] * 8, np.uint8)
    align = np.array([1, 2, 4, 8, 16, 32, 1, 3] * 8, np.uint8)
    blocks = [[(tuple(range(32)), ()), (tuple(range(32, 64)), tuple(range(32)))], [((), tuple(range(64)))]]
    m = Mir.build(blocks, [[1], []], V, [512] * 8, vclass, width, align)
    assert np.diff(m.instr_occ_off).max() == 64
    an = vlo.analyze(m)
    rng = np.random.default_rng(8)
    # per class the eight values side by side (accepted), then disturbed copies and garbage
    base = np.zeros(V, np.int64)
    for c in range(8):
        at = 0
        for v in range(c, V, 8):
            at = (at + int(align[v]) - 1) // int(align[v]) * int(align[v])
            base[v] = at
            at += int(width[v])
    K = 40
    rows = np.tile(base[m.occ_vreg].astype(np.uint16), (K, 1))
    for k in range(1, K):
        kind = k % 4
        if kind == 1:
            rows[k, rng.integers(0, m.n_occ)] += 1
        elif kind == 2:
            v = int(rng.integers(0, V))
            rows[k, m.occ_vreg == v] = rng.integers(0, 520)
        elif kind == 3:
            rows[k] = rng.integers(0, 512, m.n_occ)
    want = vlo.verify(m, an, rows)
    assert want["status"][0] == 0 and len(np.unique(want["status"])) == 4
    for tile_len in (0, 1):
        hm, hl, got, _ = gpu_analyze([m], tile_len=tile_len, dense=True)
        try:
            assert_liveness_equal(m, an, got[0], "wide")
            assert_results_equal(want, gpu_verify(hm, hl, [rows])[0], f"wide tile {tile_len}")
            assert_counts_equal(vlo.count_violations(m, an, rows), gpu_counts(hm, hl, [rows])[0], "wide")
            dev, ld = vl.rows_to_device(rows)
            queries = [(k, q) for k in (0, 2, 3) for q in range(0, m.n_occ, 3)]
            masks = torch.zeros((len(queries), 16), dtype=torch.int32, device="cuda")
            vl.vl_free_bases_multi([(hm[0], hl[0], dev[k], q) for k, q in queries], masks)
            torch.cuda.synchronize()
            got_m = masks.cpu().numpy().view(np.uint32)
            for j, (k, q) in enumerate(queries):
                assert (got_m[j] == vlo.free_bases(m, an, rows[k], q)).all(), (tile_len, k, q)
        finally:
            free(hm, hl)
