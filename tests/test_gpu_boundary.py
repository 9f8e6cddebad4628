"""Behaviour of the C ABI on the GPU beyond plain parity: a stream that is not
the default one, error codes for arguments that do not fit, and handles that
outlive a failed call."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2506_17506_amd as vl  # noqa: E402
from oracle import vlo  # noqa: E402
from vlgen import gen  # noqa: E402
from vlgen.mir import Mir  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    vl.load()


def results(out):
    return out.cpu().numpy().view(np.uint32).reshape(-1, 4).copy().view(vl.RESULT_DTYPE).reshape(-1)


def test_work_on_a_side_stream():
    """Everything is enqueued on the stream passed in; nothing relies on the default stream."""
    w = gen.config(2)
    k, rows = w.kernels[0], w.rows[0]
    an = vlo.analyze(k.mir, threads=8)
    want = vlo.verify(k.mir, an, rows, threads=8)
    side = torch.cuda.Stream()
    hm = vl.vl_mir_create(k.mir)
    dev, ld = vl.rows_to_device(rows)
    out = torch.full((rows.shape[0], 4), -1, dtype=torch.int32, device="cuda")
    summaries = torch.zeros((1, 6), dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    hl = vl.vl_liveness(hm, 0, stream=side)
    jobs = vl.make_jobs([(hm, hl, dev, rows.shape[0], ld, out)])
    vl.vl_verify_multi(jobs, stream=side)
    vl.vl_summarize_multi(jobs, summaries, None, stream=side)
    side.synchronize()
    got = results(out)
    assert (got == want).all()
    s = summaries.cpu().numpy().view(np.uint32).reshape(-1).view(vl.SUMMARY_DTYPE)[0]
    assert s["hist"].sum() == rows.shape[0] and s["hist"][0] == (want["status"] == 0).sum()
    vl.vl_live_destroy(hl)
    vl.vl_mir_destroy(hm)


def test_argument_errors_are_codes_not_faults():
    w = gen.config(1)
    k, rows = w.kernels[0], w.rows[0]
    other = Mir.build([[((0,), ()), ((1,), (0,))], [((), (1,))]], [[1], []], 2, [8])
    hm, ho = vl.vl_mir_create(k.mir), vl.vl_mir_create(other)
    hl, hlo = vl.vl_liveness(hm), vl.vl_liveness(ho)
    dev, ld = vl.rows_to_device(rows)
    K = rows.shape[0]
    out = torch.full((K, 4), 7, dtype=torch.int32, device="cuda")

    def code(job):
        try:
            vl.vl_verify_multi(vl.make_jobs([job]))
        except vl.VlError as e:
            return e.code
        return 0

    assert code((hm, hl, dev, 0, ld, out)) == -2                    # K == 0
    assert code((hm, hl, dev, K, k.mir.n_occ - 1, out)) == -2      # pitch shorter than a row
    assert code((hm, hlo, dev, K, ld, out)) == -7                   # analysis of another program
    assert code((ho, hl, dev, K, ld, out)) == -7
    torch.cuda.synchronize()
    assert (out.cpu().numpy() == 7).all()                           # nothing was launched
    # the handles are still good
    assert code((hm, hl, dev, K, ld, out)) == 0
    torch.cuda.synchronize()
    want = vlo.verify(k.mir, vlo.analyze(k.mir), rows)
    assert (results(out) == want).all()
    # recycling with handles of another batch is refused and leaves them usable
    lib = vl.load()
    import ctypes as C
    arr_m = (C.c_void_p * 1)(hm.value)
    arr_l = (C.c_void_p * 1)(hlo.value)
    assert lib.vl_liveness_multi(arr_m, 1, 0, 0, None, arr_l) == -7
    for h in (hl, hlo):
        vl.vl_live_destroy(h)
    for h in (hm, ho):
        vl.vl_mir_destroy(h)


def test_calls_alternating_over_streams():
    """Each stream has its own job table on the device: calls with different tables that
    alternate over streams without waiting for one another give every stream its own
    answers, also with more streams than the library keeps tables for."""
    w = gen.config(5, n_kernels=6)
    want = []
    for k, rows in zip(w.kernels, w.rows):
        want.append(vlo.verify(k.mir, vlo.analyze(k.mir, threads=8), rows, threads=8))
    hm = [vl.vl_mir_create(k.mir) for k in w.kernels]
    hl = vl.vl_liveness_multi(hm)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in range(6)]
    devs = [vl.rows_to_device(rows) for rows in w.rows]
    outs = [torch.full((rows.shape[0], 4), -1, dtype=torch.int32, device="cuda") for rows in w.rows]
    torch.cuda.synchronize()
    # stream j verifies kernel j only (six different one-job tables); three rounds, no waits
    jobs = [vl.make_jobs([(hm[j], hl[j], devs[j][0], w.rows[j].shape[0], devs[j][1], outs[j])]) for j in range(6)]
    for _ in range(3):
        for j, st in enumerate(streams):
            vl.vl_verify_multi(jobs[j], stream=st)
    torch.cuda.synchronize()
    for j in range(6):
        assert (results(outs[j]) == want[j]).all(), j
    for l in hl:
        vl.vl_live_destroy(l)
    for m in hm:
        vl.vl_mir_destroy(m)


def test_stream_read_probe_arguments():
    """the benchmark's streaming-read hook (a library of its own, include/vl_bench.h)"""
    from paper_2506_17506_amd import measure
    buf = torch.ones(1 << 20, dtype=torch.int32, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    assert measure.vl_stream_read_probe(buf, buf.numel() * 4, sink) == 0
    assert measure.vl_stream_read_probe(buf, 16 * 1000 + 16, sink) == 0   # a length that leaves a tail for the last loop
    torch.cuda.synchronize()
    assert int(sink.cpu()[0]) == 0
    assert measure.vl_stream_read_probe(buf[1:], 64, sink) == -2          # not 16-byte aligned
    assert measure.vl_stream_read_probe(buf, 8, sink) == -2
