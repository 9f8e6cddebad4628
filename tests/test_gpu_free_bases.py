"""Constrained-decoding masks from the GPU library against the oracle's, bit for bit:
first mentions (the occupied set matters) and later mentions (only the own register
remains), on accepted and on damaged rows, benchmark kernels of full size and programs of
mixed shapes with reserved registers, several tile lengths, and a decode driven by the
GPU's own masks that must end in an allocation the oracle accepts."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2506_17506_amd as vl  # noqa: E402
from oracle import vlo  # noqa: E402
from vlgen import gen  # noqa: E402
from vlgen.mixed import mixed_mir  # noqa: E402
from test_gpu_parity import free, gpu_analyze  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    vl.load()


def gpu_masks(hm, hl, dev_rows, queries):
    """queries: list of (row index, occurrence) -> uint32 [n, 16]"""
    masks = torch.full((len(queries), 16), -1, dtype=torch.int32, device="cuda")
    vl.vl_free_bases_multi([(hm, hl, dev_rows[k], q) for k, q in queries], masks)
    torch.cuda.synchronize()
    return masks.cpu().numpy().view(np.uint32)


def compare(m, rows, queries, tile_lens=(0,)):
    an = vlo.analyze(m, interference=False, threads=8)
    want = np.stack([vlo.free_bases(m, an, rows[k], q) for k, q in queries])
    for tile_len in tile_lens:
        hm, hl, _, _ = gpu_analyze([m], tile_len=tile_len, dense=False)
        try:
            dev, ld = vl.rows_to_device(rows)
            got = gpu_masks(hm[0], hl[0], dev, queries)
            bad = np.nonzero((got != want).any(axis=1))[0]
            assert len(bad) == 0, (m.name, tile_len, [queries[j] for j in bad[:5]])
        finally:
            free(hm, hl)
    return want


def sample_queries(m, n_rows, rng, n):
    first = np.full(m.n_vreg, m.n_occ, np.int64)
    for o in range(m.n_occ - 1, -1, -1):
        first[m.occ_vreg[o]] = o
    firsts = np.unique(first[first < m.n_occ])
    qs = [(int(rng.integers(0, n_rows)), int(q)) for q in rng.choice(firsts, min(n, len(firsts)), replace=False)]
    qs += [(int(rng.integers(0, n_rows)), int(q)) for q in rng.integers(0, m.n_occ, n // 2)]
    qs += [(0, 0), (n_rows - 1, m.n_occ - 1)]
    return qs


def test_benchmark_kernels_full_size():
    rng = np.random.default_rng(1)
    w = gen.config(5, n_kernels=8)
    some = 0
    for k, rows in list(zip(w.kernels, w.rows))[:3]:
        want = compare(k.mir, rows[:24], sample_queries(k.mir, 24, rng, 150), tile_lens=(0, 200))
        some += int((want != 0).any())
    assert some == 3


def test_mixed_shapes_and_reserved_registers():
    rng = np.random.default_rng(2)
    for seed, reserved in ((1, False), (2, True)):
        m = mixed_mir(0xA100 + seed, n_instr=1500, reserved=reserved)
        rows = rng.integers(0, 48, (6, m.n_occ)).astype(np.uint16)   # dense garbage: every mask is busy
        rows[3] = rng.integers(0, 600, m.n_occ)                       # registers outside every file too
        want = compare(m, rows, sample_queries(m, 6, rng, 200), tile_lens=(0, 64))
        pop = np.array([sum(bin(int(x)).count("1") for x in r) for r in want])
        assert (pop == 0).any() and (pop > 1).any()


def test_decoding_with_the_library_masks_gives_an_accepted_allocation():
    """Occurrence by occurrence: ask the library for the mask, take the lowest base it offers,
    write it into the row on the device.  No value is written twice in this program, so
    the finished row must verify (oracle and library)."""
    m = mixed_mir(0xF001, n_instr=300, wide_instr=1, redefine=False)
    an = vlo.analyze(m, threads=8)
    hm, hl, _, _ = gpu_analyze([m], dense=False)
    try:
        row = np.zeros((1, m.n_occ), np.uint16)
        dev, ld = vl.rows_to_device(row)
        masks = torch.zeros((1, 16), dtype=torch.int32, device="cuda")
        for q in range(m.n_occ):
            vl.vl_free_bases_multi([(hm[0], hl[0], dev[0], q)], masks)
            bits = masks.cpu().numpy().view(np.uint32)[0]
            offered = [32 * t + b for t in range(16) for b in range(32) if (int(bits[t]) >> b) & 1]
            assert offered, q
            assert (bits == vlo.free_bases(m, an, row[0], q)).all(), q
            row[0, q] = offered[0]
            dev[0, q] = int(offered[0])
        assert vlo.verify(m, an, row)["status"][0] == 0
        out = torch.zeros((1, 4), dtype=torch.int32, device="cuda")
        vl.vl_verify_batch(hm[0], hl[0], dev, 1, ld, out)
        torch.cuda.synchronize()
        assert out.cpu().numpy()[0, 0] == 0
    finally:
        free(hm, hl)


def test_argument_errors():
    m = mixed_mir(0xF002, n_instr=100, wide_instr=0)
    hm, hl, _, _ = gpu_analyze([m], dense=False)
    try:
        dev, ld = vl.rows_to_device(np.zeros((1, m.n_occ), np.uint16))
        masks = torch.full((1, 16), 5, dtype=torch.int32, device="cuda")
        with pytest.raises(vl.VlError) as e:
            vl.vl_free_bases_multi([(hm[0], hl[0], dev[0], m.n_occ)], masks)
        assert e.value.code == -2
        with pytest.raises(vl.VlError) as e:
            vl.vl_free_bases_multi([], masks)
        assert e.value.code == -2
        torch.cuda.synchronize()
        assert (masks.cpu().numpy() == 5).all()
    finally:
        free(hm, hl)
