"""Verification of occurrence-major candidates (cand[occurrence][candidate]) against the
oracle, which reads the same candidates row by row: the verdicts must be those of the
row-major path, for every group shape the split by 8 produces."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2506_17506_amd as vl  # noqa: E402
from oracle import vlo  # noqa: E402
from vlgen import gen  # noqa: E402
from vlgen.mixed import mixed_mir  # noqa: E402
from vlgen.tiny import tiny_mir, tiny_rows  # noqa: E402
from test_gpu_parity import assert_results_equal, free, gpu_analyze  # noqa: E402
from test_gpu_mixed_shapes import disturbed_rows  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    vl.load()


def verify_occ_major(hm, hl, rows_list, pad=0):
    jobs, outs, keep = [], [], []
    for m, l, rows in zip(hm, hl, rows_list):
        K, O = rows.shape
        ld = (K + 7) // 8 * 8 + pad
        host = np.full((max(O, 1), ld), 0xABCD, np.uint16)    # the padding holds junk on purpose
        host[:O, :K] = rows.T
        dev = torch.from_numpy(host.view(np.int16)).cuda()
        out = torch.full((K, 4), -1, dtype=torch.int32, device="cuda")
        keep.append(dev)
        outs.append(out)
        jobs.append((m, l, dev, K, ld, out))
    vl.vl_verify_multi_occ_major(jobs)
    torch.cuda.synchronize()
    return [o.cpu().numpy().view(np.uint32).reshape(-1, 4).copy().view(vl.RESULT_DTYPE).reshape(-1) for o in outs]


@pytest.mark.parametrize("K", [1, 7, 8, 50, 52, 53, 64, 65, 100, 130, 200])
def test_group_shapes(K):
    k = gen.Kernel(gen.LOOP3, 0xABD, 600, 450)
    rows, _ = k.candidates(5, K, K // 2, 2)
    an = vlo.analyze(k.mir)
    want = vlo.verify(k.mir, an, rows)
    for tile_len in (0, 100):
        hm, hl, _, _ = gpu_analyze([k.mir], tile_len, dense=False)
        try:
            assert_results_equal(want, verify_occ_major(hm, hl, [rows])[0], f"K {K} tile {tile_len}")
            assert_results_equal(want, verify_occ_major(hm, hl, [rows], pad=24)[0], f"K {K} padded")
        finally:
            free(hm, hl)


def test_benchmark_kernels_full_size():
    w = gen.config(5, n_kernels=12)
    mirs = [k.mir for k in w.kernels]
    hm, hl, _, _ = gpu_analyze(mirs, tile_len=512, dense=False)   # the tile length of the benchmark's batch of 256
    try:
        res = verify_occ_major(hm, hl, w.rows)
        for k, m in enumerate(mirs):
            an = vlo.analyze(m, threads=16)
            assert_results_equal(vlo.verify(m, an, w.rows[k], threads=16), res[k], m.name)
    finally:
        free(hm, hl)


def test_config3_many_groups():
    w = gen.config(3)
    k, rows = w.kernels[0], w.rows[0]          # K = 1,000: sixteen groups
    an = vlo.analyze(k.mir, threads=16)
    hm, hl, _, _ = gpu_analyze([k.mir], dense=False)
    try:
        assert_results_equal(vlo.verify(k.mir, an, rows, threads=16), verify_occ_major(hm, hl, [rows])[0], "config 3")
    finally:
        free(hm, hl)


def test_mixed_shapes_and_tiny_programs():
    m = mixed_mir(0xA001, n_instr=2500)
    an = vlo.analyze(m, threads=8)
    rows = disturbed_rows(m, an, 1, 72)
    ms, ans, rl = [m], [an], [rows]
    for seed in range(60):
        t = tiny_mir(seed, reserved=seed % 2 == 0, early=0.3)
        a = vlo.analyze(t)
        if a.contract == 0:
            ms.append(t); ans.append(a); rl.append(tiny_rows(t, seed, K=int(1 + seed % 11)))
    for tile_len in (0, 3):
        hm, hl, _, _ = gpu_analyze(ms, tile_len, dense=False)
        try:
            res = verify_occ_major(hm, hl, rl)
            for j, mm in enumerate(ms):
                assert_results_equal(vlo.verify(mm, ans[j], rl[j]), res[j], f"{mm.name} tile {tile_len}")
        finally:
            free(hm, hl)


def test_argument_errors():
    k = gen.Kernel(gen.LOOP3, 0xABD, 200, 150)
    rows, _ = k.candidates(5, 10, 0, 0)
    hm, hl, _, _ = gpu_analyze([k.mir], dense=False)
    try:
        O = k.mir.n_occ
        dev = torch.zeros((O, 16), dtype=torch.int16, device="cuda")
        out = torch.full((10, 4), 7, dtype=torch.int32, device="cuda")
        for ld, K, cand in ((12, 10, dev), (8, 10, dev), (16, 10, dev.view(-1)[1:])):   # pitch not a multiple of 8; pitch below K; misaligned
            with pytest.raises(vl.VlError) as e:
                vl.vl_verify_multi_occ_major([(hm[0], hl[0], cand, K, ld, out)])
            assert e.value.code == -2
        torch.cuda.synchronize()
        assert (out.cpu().numpy() == 7).all()
    finally:
        free(hm, hl)


def test_loop_reductions_follow_occurrence_major_verification():
    """the regeneration-loop reductions read only the results, so the same jobs serve them
    after either entry point (here: pitch K rounded up to 8, far below the occurrence count)"""
    ks = [gen.Kernel(gen.LOOP3, 0xAC0 + j, 400 + 100 * j, 300 + 75 * j) for j in range(3)]
    rl = [k.candidates(5 + j, 40 + 30 * j, 25, 2)[0] for j, k in enumerate(ks)]
    hm, hl, _, _ = gpu_analyze([k.mir for k in ks], dense=False)
    try:
        jobs, keep = [], []
        for m, l, rows in zip(hm, hl, rl):
            K, O = rows.shape
            ld = (K + 7) // 8 * 8
            host = np.zeros((O, ld), np.uint16)
            host[:, :K] = rows.T
            dev = torch.from_numpy(host.view(np.int16)).cuda()
            out = torch.full((K, 4), -1, dtype=torch.int32, device="cuda")
            keep.append((dev, out))
            jobs.append((m, l, dev, K, ld, out))
        jobs = vl.make_jobs(jobs)
        summaries = torch.full((3, 6), -1, dtype=torch.int32, device="cuda")
        stats = torch.full((6,), -1, dtype=torch.int64, device="cuda")
        for _ in range(2):
            vl.vl_verify_multi_occ_major(jobs)
            vl.vl_summarize_multi(jobs, summaries, stats)
        torch.cuda.synchronize()
        got_s = summaries.cpu().numpy().view(np.uint32).reshape(-1).view(vl.SUMMARY_DTYPE)
        got_l = stats.cpu().numpy().view(np.uint8).view(vl.LOOP_DTYPE)[0]
    finally:
        free(hm, hl)
    want_s = np.array([vlo.summarize(vlo.verify(k.mir, vlo.analyze(k.mir), rows))[0] for k, rows in zip(ks, rl)],
                      vlo.SUMMARY_DTYPE)
    want_l = vlo.loop_stats(want_s, [r.shape[0] for r in rl])[0]
    for f in ("first_ok", "passed", "hist"):
        assert (got_s[f] == want_s[f]).all(), f
    for f in ("n_passed", "max_tries", "sum_tries", "hist"):
        assert (got_l[f] == want_l[f]).all(), f
