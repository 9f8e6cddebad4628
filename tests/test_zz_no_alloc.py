"""The entry point that allocates nothing (vl_verify_batch_static) against vl_verify_batch,
through the C ABI: same results on two calls in a row, the second with a smaller program and
fewer candidates, so that what the first call left in the library's fixed device array (job
table, list of clashes to resolve) must not leak into the second."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2506_17506_amd as vl  # noqa: E402
from oracle import vlo  # noqa: E402
from vlgen import gen  # noqa: E402


def results(out):
    return out.cpu().numpy().view(np.uint32).reshape(-1, 4).copy().view(vl.RESULT_DTYPE).reshape(-1)


def test_static_entry_point_matches_the_allocating_one():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    vl.load()
    big = gen.Kernel(gen.MHA, 0x5A1, 3000, 2250)
    small = gen.Kernel(gen.LOOP3, 0x5A2, 500, 380)
    cases = [(big, big.candidates(7, 130, 90, 2)[0]), (small, small.candidates(8, 37, 20, 2)[0])]
    handles = []
    for k, rows in cases:
        hm = vl.vl_mir_create(k.mir)
        hl = vl.vl_liveness(hm)
        dev, ld = vl.rows_to_device(rows)
        handles.append((hm, hl, dev, ld))
    torch.cuda.synchronize()
    seen = set()
    for (k, rows), (hm, hl, dev, ld) in zip(cases, handles):   # two calls in a row, the second smaller
        K = rows.shape[0]
        out_s = torch.full((K, 4), -1, dtype=torch.int32, device="cuda")
        vl.vl_verify_batch_static(hm, hl, dev, K, ld, out_s)
        torch.cuda.synchronize()
        out_a = torch.full((K, 4), -1, dtype=torch.int32, device="cuda")
        vl.vl_verify_batch(hm, hl, dev, K, ld, out_a)
        torch.cuda.synchronize()
        got_s, got_a = results(out_s), results(out_a)
        assert (got_s == got_a).all(), k.mir.name
        want = vlo.verify(k.mir, vlo.analyze(k.mir), rows)
        assert (got_s == want).all(), k.mir.name
        seen |= set(np.unique(want["status"]).tolist())
    assert seen >= {0, 3}
    # beyond the fixed capacity: refused, nothing launched
    hm, hl, dev, ld = handles[0]
    with pytest.raises(vl.VlError) as e:
        vl.vl_verify_batch_static(hm, hl, dev, 65537, ld, out_s)
    assert e.value.code == -8
    for hm, hl, _, _ in handles:
        vl.vl_live_destroy(hl)
        vl.vl_mir_destroy(hm)
