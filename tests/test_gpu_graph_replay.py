"""The steady-state pass (analysis into recycled handles, verification, the loop's
reductions) recorded once into a HIP graph and replayed: every replay, with fresh
candidates in the same device buffers and eager calls and synchronisations between
the replays, must give exactly the eager results and the oracle's."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2506_17506_amd as vl  # noqa: E402
from oracle import vlo  # noqa: E402
from vlgen import gen  # noqa: E402
from test_gpu_parity import assert_liveness_equal, assert_results_equal, free  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    vl.load()


def results(outs):
    return [o.cpu().numpy().view(np.uint32).reshape(-1, 4).copy().view(vl.RESULT_DTYPE).reshape(-1) for o in outs]


def test_graph_replays_match_eager_and_oracle():
    w = gen.config(5, n_kernels=8)
    mirs = [k.mir for k in w.kernels]
    n = len(mirs)
    # three candidate sets for the same kernels: the generator's rows rolled and damaged
    rng = np.random.default_rng(99)
    sets = []
    for r in range(3):
        rows_list = []
        for j, rows in enumerate(w.rows):
            x = np.ascontiguousarray(np.roll(rows, 3 * r + j, axis=0))
            for k in rng.integers(0, x.shape[0], 4 * r):
                x[int(k), int(rng.integers(0, x.shape[1]))] ^= 1
            rows_list.append(x)
        sets.append(rows_list)
    ans = [vlo.analyze(m, threads=16) for m in mirs]
    want = [[vlo.verify(m, an, rows, threads=16) for m, an, rows in zip(mirs, ans, rows_list)] for rows_list in sets]

    hm = [vl.vl_mir_create(m) for m in mirs]
    side = torch.cuda.Stream()
    devs, outs, jobs = [], [], []
    hl = None
    try:
        with torch.cuda.stream(side):
            hl = vl.vl_liveness_multi(hm, 0, 0)
            for m, l, rows in zip(hm, hl, sets[0]):
                dev, ld = vl.rows_to_device(rows)
                out = torch.full((rows.shape[0], 4), -1, dtype=torch.int32, device="cuda")
                devs.append(dev)
                outs.append(out)
                jobs.append((m, l, dev, rows.shape[0], ld, out))
            jobs = vl.make_jobs(jobs)
            summaries = torch.full((n, 6), -1, dtype=torch.int32, device="cuda")
            stats = torch.full((6,), -1, dtype=torch.int64, device="cuda")

            def one_pass():
                again = vl.vl_liveness_multi(hm, 0, 0, live=hl)
                assert [a.value for a in again] == [a.value for a in hl]
                vl.vl_verify_multi(jobs)
                vl.vl_summarize_multi(jobs, summaries, stats)

            # eager passes: the second and third run with known sizes and current tables,
            # which is the state the recording needs (no read-back, no upload, no allocation)
            for _ in range(3):
                one_pass()
            side.synchronize()
            assert [(a == b).all() for a, b in zip(results(outs), want[0])] == [True] * n

            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                one_pass()

        def load(rows_list):
            for dev, rows in zip(devs, rows_list):
                dev[:, :rows.shape[1]].copy_(torch.from_numpy(rows.view(np.int16)))

        for r in (1, 2, 0, 1):
            load(sets[r])
            for o in outs:
                o.fill_(-1)
            summaries.fill_(-1)
            stats.fill_(-1)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            got = results(outs)
            got_s = summaries.cpu().numpy().copy()
            got_l = stats.cpu().numpy().copy()
            for k in range(n):
                assert_results_equal(want[r][k], got[k], f"replay of set {r}, kernel {k}")
            views = [vl.view_to_numpy(vl.vl_live_get(l)) for l in hl]
            for k in (0, n - 1):
                assert_liveness_equal(mirs[k], ans[k], views[k], f"replay of set {r}")
            # the program's own eager work between replays: the same pass, eagerly
            one_pass()
            torch.cuda.synchronize()
            for a, b in zip(results(outs), got):
                assert (a == b).all()
            assert (summaries.cpu().numpy() == got_s).all()
            assert (stats.cpu().numpy() == got_l).all()
            want_s = np.array([vlo.summarize(x)[0] for x in want[r]], vlo.SUMMARY_DTYPE)
            got_sv = got_s.view(np.uint32).reshape(-1).view(vl.SUMMARY_DTYPE)
            for f in ("first_ok", "passed", "hist"):
                assert (got_sv[f] == want_s[f]).all(), f
    finally:
        torch.cuda.synchronize()
        if hl is not None:
            free(hm, hl)
        else:
            for m in hm:
                vl.vl_mir_destroy(m)
