"""All-violations mode on the GPU against the oracle's counts, exactly: benchmark kernels of
full size with their damaged candidates, programs of mixed shapes (wide tuples, reserved
registers, three files) with dense garbage rows, row counts around the 64-candidate groups,
tiny programs, and the tie between the set of kinds and the first-violation status."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2506_17506_amd as vl  # noqa: E402
from oracle import vlo  # noqa: E402
from vlgen import gen  # noqa: E402
from vlgen.mixed import many_blocks_mir, mixed_mir  # noqa: E402
from vlgen.tiny import tiny_mir, tiny_rows  # noqa: E402
from test_gpu_parity import free, gpu_analyze, gpu_verify  # noqa: E402

FIELDS = ("kinds", "n_cons", "n_real", "n_safe", "real_bits")


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    vl.load()


def gpu_counts(hm, hl, rows_list, calls=1):
    jobs, outs, keep = [], [], []
    for m, l, rows in zip(hm, hl, rows_list):
        dev, ld = vl.rows_to_device(rows)
        out = torch.full((rows.shape[0], 8), -1, dtype=torch.int32, device="cuda")
        keep.append(dev)
        outs.append(out)
        jobs.append((m, l, dev, rows.shape[0], ld, out))
    for _ in range(calls):     # the second call finds the pairs cached with the program
        vl.vl_count_violations_multi(jobs)
    torch.cuda.synchronize()
    return [o.cpu().numpy().view(np.uint32).reshape(-1).view(vl.COUNTS_DTYPE) for o in outs]


def assert_counts_equal(want, got, tag):
    for f in FIELDS:
        bad = np.nonzero(want[f] != got[f])[0]
        assert len(bad) == 0, (tag, f, bad[:5], want[f][bad[:5]], got[f][bad[:5]])


def test_benchmark_kernels_full_size():
    w = gen.config(5, n_kernels=10)
    mirs = [k.mir for k in w.kernels]
    hm, hl, _, _ = gpu_analyze(mirs, dense=False)
    try:
        got = gpu_counts(hm, hl, w.rows, calls=2)
        res = gpu_verify(hm, hl, w.rows)
        seen = set()
        for k, m in enumerate(mirs):
            an = vlo.analyze(m, threads=16)
            want = vlo.count_violations(m, an, w.rows[k], threads=16)
            assert_counts_equal(want, got[k], m.name)
            # the first-violation status is the lowest kind present
            kinds = got[k]["kinds"]
            lowest = np.where(kinds == 0, 0, np.where(kinds & 1, 1, np.where(kinds & 2, 2, 3)))
            assert (lowest == res[k]["status"]).all(), m.name
            seen |= set(int(x) for x in kinds)
        assert len(seen) >= 4
    finally:
        free(hm, hl)


def test_mixed_shapes_with_garbage_rows():
    rng = np.random.default_rng(6)
    mirs = [mixed_mir(0xA200, n_instr=1200, reserved=True), mixed_mir(0xA201, n_instr=800),
            many_blocks_mir(5, n_blocks=40, gap=3)]
    rows_list = []
    for j, m in enumerate(mirs):
        K = (70, 64, 129)[j]
        rows = rng.integers(0, 64, (K, m.n_occ)).astype(np.uint16)
        rows[1] = rng.integers(0, 700, m.n_occ)              # far outside every file
        first = np.zeros(m.n_vreg, np.int64)
        for o in range(m.n_occ - 1, -1, -1):
            first[m.occ_vreg[o]] = o
        for k in range(2, K, 3):                              # consistent rows: only table violations
            rows[k] = rows[k][first[m.occ_vreg]]
        rows_list.append(rows)
    hm, hl, _, _ = gpu_analyze(mirs, dense=False)
    try:
        got = gpu_counts(hm, hl, rows_list)
        for k, m in enumerate(mirs):
            an = vlo.analyze(m, threads=16)
            want = vlo.count_violations(m, an, rows_list[k], threads=16)
            assert_counts_equal(want, got[k], m.name)
            assert (want["n_cons"][2::3] == 0).all() and (want["n_safe"] > 0).any()
    finally:
        free(hm, hl)


def test_tiny_programs():
    done = 0
    for seed in range(40):
        m = tiny_mir(seed, reserved=seed % 3 == 0)
        an = vlo.analyze(m)
        if an.contract != 0:
            continue
        rows = tiny_rows(m, seed, K=5)
        hm, hl, _, _ = gpu_analyze([m], dense=False)
        try:
            got = gpu_counts(hm, hl, [rows])[0]
        finally:
            free(hm, hl)
        assert_counts_equal(vlo.count_violations(m, an, rows), got, m.name)
        done += 1
    assert done >= 25


def test_argument_errors():
    m = mixed_mir(0xF003, n_instr=100, wide_instr=0)
    hm, hl, _, _ = gpu_analyze([m], dense=False)
    try:
        dev, ld = vl.rows_to_device(np.zeros((2, m.n_occ), np.uint16))
        out = torch.full((2, 8), 5, dtype=torch.int32, device="cuda")
        for K, pitch in ((0, ld), (2, m.n_occ - 1)):
            with pytest.raises(vl.VlError) as e:
                vl.vl_count_violations_multi([(hm[0], hl[0], dev, K, pitch, out)])
            assert e.value.code == -2
        torch.cuda.synchronize()
        assert (out.cpu().numpy() == 5).all()
    finally:
        free(hm, hl)
