"""Regeneration-loop reductions on the GPU (first accepted candidate, pass flag,
status histogram per kernel; attempts over the suite) against the oracle's,
computed from the oracle's own verdicts.  Exact."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2506_17506_amd as vl  # noqa: E402
from oracle import vlo  # noqa: E402
from vlgen import gen  # noqa: E402
from test_gpu_parity import free, gpu_analyze  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    vl.load()


def run(kernels, rows_list):
    mirs = [k.mir for k in kernels]
    hm, hl, _, _ = gpu_analyze(mirs, dense=False)
    try:
        keep, jobs = [], []
        for m, l, rows in zip(hm, hl, rows_list):
            dev, ld = vl.rows_to_device(rows)
            out = torch.full((rows.shape[0], 4), -1, dtype=torch.int32, device="cuda")
            keep.append((dev, out))
            jobs.append((m, l, dev, rows.shape[0], ld, out))
        jobs = vl.make_jobs(jobs)
        n = len(kernels)
        summaries = torch.full((n, 6), -1, dtype=torch.int32, device="cuda")
        stats = torch.full((6,), -1, dtype=torch.int64, device="cuda")
        for _ in range(2):   # the totals are cleared by the call itself
            vl.vl_verify_multi(jobs)
            vl.vl_summarize_multi(jobs, summaries, stats)
        torch.cuda.synchronize()
        got_s = summaries.cpu().numpy().view(np.uint32).reshape(-1).view(vl.SUMMARY_DTYPE)
        got_l = stats.cpu().numpy().view(np.uint8).view(vl.LOOP_DTYPE)[0]
        # per-kernel call without totals
        only = torch.zeros((n, 6), dtype=torch.int32, device="cuda")
        vl.vl_summarize_multi(jobs, only, None)
        torch.cuda.synchronize()
        assert (only.cpu().numpy() == summaries.cpu().numpy()).all()
    finally:
        free(hm, hl)
    want_s = []
    for k, rows in zip(kernels, rows_list):
        an = vlo.analyze(k.mir, threads=8)
        want_s.append(vlo.summarize(vlo.verify(k.mir, an, rows, threads=8))[0])
    want_s = np.array(want_s, vlo.SUMMARY_DTYPE)
    want_l = vlo.loop_stats(want_s, [r.shape[0] for r in rows_list])[0]
    for f in ("first_ok", "passed", "hist"):
        assert (got_s[f] == want_s[f]).all(), f
    for f in ("n_passed", "max_tries", "sum_tries", "hist"):
        assert (got_l[f] == want_l[f]).all(), f
    return want_s, want_l


def test_reductions_on_benchmark_kernels():
    w = gen.config(5, n_kernels=12)
    # put the undamaged rows at different depths so that first_ok varies
    rows_list = []
    for j, rows in enumerate(w.rows):
        rows_list.append(np.ascontiguousarray(np.roll(rows, j * 7, axis=0)))
    want_s, want_l = run(w.kernels, rows_list)
    assert want_l["n_passed"] == len(w.kernels)
    assert len(set(int(x) for x in want_s["first_ok"])) > 1


def test_exhausted_attempts_are_reported():
    """A kernel whose every candidate is damaged exhausts its attempts: first_ok = K,
    passed = 0, and it costs K attempts in the totals."""
    w = gen.config(5, n_kernels=3)
    rows_list = [r.copy() for r in w.rows]
    bad = rows_list[1]
    bad[:, 0] = 65535            # no register file holds this base
    want_s, want_l = run(w.kernels, rows_list)
    assert want_s["passed"][1] == 0 and want_s["first_ok"][1] == bad.shape[0]
    assert want_l["n_passed"] == 2 and want_l["max_tries"] == bad.shape[0]
