"""GPU library against the CPU oracle, bit for bit, through the C ABI.

Every comparison is exact: live sets, kill flags, intervals, and per candidate
the status and the first violation."""
import json
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2506_17506_amd as vl  # noqa: E402
from oracle import vlo  # noqa: E402
from vlgen import gen  # noqa: E402
from vlgen.mir import Mir  # noqa: E402
from vlgen.tiny import tiny_mir, tiny_rows  # noqa: E402

GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    vl.load()


def gpu_analyze(mirs, tile_len=0, dense=True):
    """-> (mir handles, live handles, [numpy dict per kernel])"""
    hm = [vl.vl_mir_create(m) for m in mirs]
    hl = vl.vl_liveness_multi(hm, vl.VL_DENSE_POINTS if dense else 0, tile_len)
    torch.cuda.synchronize()
    views = [vl.vl_live_get(l) for l in hl]
    return hm, hl, [vl.view_to_numpy(v) for v in views], views


def gpu_verify(hm, hl, rows_list, aligned=True):
    """aligned: True = rows padded to whole 128-byte lines (staged without bounds), "pitch8" =
    16-byte aligned rows whose pitch is the next multiple of 8 (16-byte reads with bounds),
    False = odd pitch from a 2-byte aligned start (element by element)"""
    jobs, outs, keep = [], [], []
    for m, l, rows in zip(hm, hl, rows_list):
        K, O = rows.shape
        if aligned == "pitch8":
            ld = (O + 7) // 8 * 8
            host = np.zeros((K, ld), np.uint16)
            host[:, :O] = rows
            dev = torch.from_numpy(host.view(np.int16)).cuda()
        elif aligned:
            dev, ld = vl.rows_to_device(rows)
        else:  # odd pitch, 2-byte aligned start: the element-wise staging path
            ld = O + 1 if (O + 1) % 2 else O + 2
            host = np.zeros(K * ld + 1, np.uint16)
            host[1:].reshape(K, ld)[:, :O] = rows
            flat = torch.from_numpy(host.view(np.int16)).cuda()
            dev = flat[1:]
        out = torch.full((K, 4), -1, dtype=torch.int32, device="cuda")
        keep.append((dev, out))
        jobs.append((m, l, dev, K, ld, out))
        outs.append(out)
    vl.vl_verify_multi(jobs)
    torch.cuda.synchronize()
    return [o.cpu().numpy().view(np.uint32).reshape(-1, 4).copy().view(vl.RESULT_DTYPE).reshape(-1) for o in outs]


def free(hm, hl):
    for l in hl:
        vl.vl_live_destroy(l)
    for m in hm:
        vl.vl_mir_destroy(m)


def assert_liveness_equal(m, an, got, tag=""):
    V = m.n_vreg
    assert (got["live_in"] == vlo.pack_bits(an.live_in)).all(), tag
    assert (got["live_out"] == vlo.pack_bits(an.live_out)).all(), tag
    if got["live_after"] is not None:
        assert (got["live_after"] == an.live_after).all(), tag
    assert (got["occ_kill"] == an.occ_kill).all(), tag
    assert (got["seg_off"] == an.seg_off).all(), tag
    assert (got["seg"] == an.seg).all(), tag
    assert (got["hull"] == an.hull).all(), tag


def assert_results_equal(want, got, tag=""):
    bad = np.nonzero(want != got)[0]
    assert len(bad) == 0, f"{tag}: first mismatch row {bad[0]}: oracle {want[bad[0]]} gpu {got[bad[0]]}"


def test_worked_examples():
    with open(os.path.join(GOLD, "worked_examples.json")) as f:
        exs = json.load(f)["examples"]
    mirs = [Mir.build([[(tuple(i[0]), tuple(i[1])) for i in blk] for blk in ex["blocks"]], ex["succ"],
                      ex["n_vreg"], ex["class_size"]) for ex in exs]
    for tile_len in (0, 1, 2):
        hm, hl, got, _ = gpu_analyze(mirs, tile_len)
        rows = [np.array([c["row"] for c in ex["candidates"]], np.uint16) for ex in exs]
        res = gpu_verify(hm, hl, rows)
        for ex, m, g, r in zip(exs, mirs, got, res):
            an = vlo.analyze(m)
            assert_liveness_equal(m, an, g, ex["name"])
            assert [[int(x) for x in rr] for rr in r] == [c["result"] for c in ex["candidates"]], ex["name"]
        free(hm, hl)


@pytest.mark.parametrize("tile_len", [1, 2, 3, 5, 0])
@pytest.mark.parametrize("reserved", [False, True])
def test_tiny_random_programs(tile_len, reserved):
    mirs, ans = [], []
    seed = 0
    while len(mirs) < 150:
        m = tiny_mir(7000 + seed, strict=True, reserved=reserved, max_instr=6)
        seed += 1
        an = vlo.analyze(m)
        if an.contract == 0:
            mirs.append(m)
            ans.append(an)
    hm, hl, got, _ = gpu_analyze(mirs, tile_len)
    rows = [tiny_rows(m, 100 + k, K=9) for k, m in enumerate(mirs)]
    res = gpu_verify(hm, hl, rows, aligned=(tile_len != 3))
    hist = np.zeros(4, int)
    for k, (m, an, g, r) in enumerate(zip(mirs, ans, got, res)):
        assert_liveness_equal(m, an, g, f"tiny {k}")
        want = vlo.verify(m, an, rows[k])
        assert_results_equal(want, r, f"tiny {k} tile {tile_len}")
        hist += np.bincount(want["status"], minlength=4)
    assert (hist > 30).all(), hist
    free(hm, hl)


def test_not_strict_is_reported():
    m = Mir.build([[((), (0,))], [((0,), ())]], [[1], []], 1)
    h = vl.vl_mir_create(m)
    with pytest.raises(vl.VlError) as e:
        vl.vl_liveness(h)
    assert e.value.code == -5
    vl.vl_mir_destroy(h)


@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_configs_full_size(cfg):
    w = gen.config(cfg)
    k, rows = w.kernels[0], w.rows[0]
    an = vlo.analyze(k.mir, threads=16)
    want = vlo.verify(k.mir, an, rows, threads=16)
    for tile_len in (0, 97, 512):   # the default (which follows the size of the batch), an odd one, the benchmark's
        hm, hl, got, views = gpu_analyze([k.mir], tile_len)
        assert_liveness_equal(k.mir, an, got[0], f"config {cfg}")
        for aligned in (True, "pitch8", False):
            res = gpu_verify(hm, hl, [rows], aligned)
            assert_results_equal(want, res[0], f"config {cfg} tile {tile_len} aligned {aligned}")
        free(hm, hl)
    assert set(np.unique(want["status"])) >= ({0, 1, 3} if cfg == 1 else {0, 3})


@pytest.mark.parametrize("K", [1, 63, 64, 65, 130])
def test_row_counts(K):
    k = gen.Kernel(gen.LOOP3, 0xABC, 600, 450)
    rows, log = k.candidates(5, K, K // 2, 2)
    an = vlo.analyze(k.mir)
    want = vlo.verify(k.mir, an, rows)
    hm, hl, got, _ = gpu_analyze([k.mir], 128, dense=False)
    res = gpu_verify(hm, hl, [rows])
    assert_results_equal(want, res[0], f"K {K}")
    # single-kernel entry point
    dev, ld = vl.rows_to_device(rows)
    out = torch.zeros((K, 4), dtype=torch.int32, device="cuda")
    vl.vl_verify_batch(hm[0], hl[0], dev, K, ld, out)
    torch.cuda.synchronize()
    got1 = out.cpu().numpy().view(np.uint32).copy().view(vl.RESULT_DTYPE).reshape(-1)
    assert_results_equal(want, got1, f"K {K} single")
    free(hm, hl)


def test_config4_and_5_kernels_full_size():
    w4 = gen.config(4, n_kernels=3)
    w5 = gen.config(5, n_kernels=24)
    kernels = w4.kernels + w5.kernels
    rows = w4.rows + w5.rows
    mirs = [k.mir for k in kernels]
    hm, hl, got, views = gpu_analyze(mirs, 512, dense=False)   # the tile length of the benchmark's batch of 256
    res = gpu_verify(hm, hl, rows)
    for k, (m, r) in enumerate(zip(mirs, res)):
        an = vlo.analyze(m, threads=16)
        assert_liveness_equal(m, an, got[k], m.name)
        want = vlo.verify(m, an, rows[k], threads=16)
        assert_results_equal(want, r, m.name)
    # recycle the handles: same storage, same answers.  The first recycling call with the
    # same options reuses the known sizes without waiting, the second also the device tables;
    # then other options (dense points, another tile length) size everything afresh.
    for flags, tile_len, dense in ((0, 512, False), (0, 512, False), (vl.VL_DENSE_POINTS, 512, True), (0, 300, False),
                                   (0, 300, False), (0, 0, False)):
        hl2 = vl.vl_liveness_multi(hm, flags, tile_len, live=hl)
        assert [a.value for a in hl2] == [a.value for a in hl]
        torch.cuda.synchronize()
        got2 = [vl.view_to_numpy(vl.vl_live_get(l)) for l in hl2]
        for k, m in enumerate(mirs[:6]):
            an = vlo.analyze(m, interference=False, threads=16)
            assert_liveness_equal(m, an, got2[k], f"{m.name} recycled {flags} {tile_len}")
            assert (got2[k]["live_after"] is not None) == dense
        res2 = gpu_verify(hm, hl2, rows)
        for a, b in zip(res, res2):
            assert (a == b).all()
    free(hm, hl)


def oracle_light(m, rows):
    """the oracle's results for one kernel without the per-point rows (which take 75 MB at
    20,000 instructions): what assert_liveness_equal compares when no dense rows are asked
    for, and the verdicts"""
    an = vlo.analyze(m, threads=1)
    want = vlo.verify(m, an, rows, threads=1)
    an.live_after = an.P = None
    return an, want


def test_config4_every_kernel():
    """All 64 attention-shaped kernels of 20,000 instructions with their 100 candidates each,
    in one batch as the library is meant to take them: liveness results and every verdict."""
    from concurrent.futures import ThreadPoolExecutor
    w = gen.config(4)
    assert len(w.kernels) == 64 and all(r.shape[0] == 100 for r in w.rows)
    mirs = [k.mir for k in w.kernels]
    hm, hl, got, views = gpu_analyze(mirs, 0, dense=False)
    assert views[0].tile_len == 512
    res = gpu_verify(hm, hl, w.rows)
    with ThreadPoolExecutor(16) as pool:   # the oracle releases the interpreter lock while it runs
        ref = list(pool.map(oracle_light, mirs, w.rows))
    hist = np.zeros(4, int)
    for k, (m, (an, want)) in enumerate(zip(mirs, ref)):
        got[k]["live_after"] = None
        assert_liveness_equal(m, an, got[k], m.name)
        assert_results_equal(want, res[k], m.name)
        hist += np.bincount(want["status"], minlength=4)
    assert hist.sum() == 6400 and (hist > 0).all(), hist
    free(hm, hl)


def test_dense_points_on_a_large_kernel():
    k = gen.Kernel(gen.MHA, 77, 6000, 4500)
    an = vlo.analyze(k.mir, interference=False)
    hm, hl, got, _ = gpu_analyze([k.mir], 0, dense=True)
    assert_liveness_equal(k.mir, an, got[0], "dense")
    free(hm, hl)
