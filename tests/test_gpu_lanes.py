"""Liveness of parts of a tuple on the GPU (vl_mir_create_lanes) against the oracle's
per-lane analysis, through the C ABI and exactly: live sets, kill flags and live intervals of
every (vreg, lane) through the maps the library gives, and every verdict in the caller's
numbering."""
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
from vlgen.tiny import tiny_lanes, tiny_mir, tiny_rows  # noqa: E402

GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    vl.load()


def run(mirs, lanes_list, rows_list, tile_len=0):
    """-> per program (maps, liveness arrays of the rewritten program, results)"""
    hm = [vl.vl_mir_create_lanes(m, l) for m, l in zip(mirs, lanes_list)]
    hl = vl.vl_liveness_multi(hm, vl.VL_DENSE_POINTS, tile_len)
    torch.cuda.synchronize()
    maps = [vl.vl_mir_lanes_get(h) for h in hm]
    live = [vl.view_to_numpy(vl.vl_live_get(l)) for l in hl]
    jobs, outs, keep = [], [], []
    for h, l, mp, rows in zip(hm, hl, maps, rows_list):
        K = rows.shape[0]
        dev, ld = vl.rows_to_device(rows)
        ld_low = vl.pad_ld(mp["n_occ_low"])
        low = torch.zeros((K, ld_low), dtype=torch.int16, device="cuda")
        vl.vl_lanes_expand(h, dev, K, ld, low, ld_low)
        out = torch.full((K, 4), -1, dtype=torch.int32, device="cuda")
        keep.append((dev, low, out))
        outs.append(out)
        jobs.append((h, l, low, K, ld_low, out))
    vl.vl_verify_multi(jobs)
    torch.cuda.synchronize()
    res = [o.cpu().numpy().view(np.uint32).reshape(-1, 4).copy().view(vl.RESULT_DTYPE).reshape(-1) for o in outs]
    for l in hl:
        vl.vl_live_destroy(l)
    for h in hm:
        vl.vl_mir_destroy(h)
    return maps, live, res


def assert_lane_liveness(m, lanes, mp, got, tag):
    an = vlo.analyze_lanes(m, lanes)
    vv, vl_ = mp["val_vreg"].astype(np.int64), mp["val_lane"].astype(np.int64)
    split = np.zeros(m.n_vreg, bool)
    split[vv[vl_ != 0xFF]] = True
    whole_of_split = (vl_ == 0xFF) & split[vv]
    # the oracle's lane of every value: its own lane, lane 0 for a vreg that was never split (all its lanes
    # behave alike); the whole-vreg value of a split vreg takes part in nothing
    lane_idx = an.lane_base[vv].astype(np.int64) + np.where(vl_ == 0xFF, 0, vl_)
    Vl = mp["n_vreg_low"]
    for name, want in (("live_in", an.live_in), ("live_out", an.live_out), ("live_after", an.live_after)):
        g = vlo.unpack_bits(got[name], Vl)
        assert (g[:, ~whole_of_split] == want[:, lane_idx[~whole_of_split]]).all(), (tag, name)
        assert not g[:, whole_of_split].any(), (tag, name)
    src, add = mp["occ_src"].astype(np.int64), mp["occ_add"].astype(np.int64)
    occ_val = np.zeros(mp["n_occ_low"], np.int64)   # the value of every rewritten occurrence, from the maps alone
    k = 0
    for o in range(m.n_occ):
        v = int(m.occ_vreg[o])
        first_id = int(np.nonzero((vv == v) & (vl_ == 0xFF))[0][0])
        assert src[k] == o and add[k] == 0
        occ_val[k] = first_id
        k += 1
        if split[v]:
            mask = int(lanes[o]) if lanes is not None and int(lanes[o]) else (1 << int(m.vreg_width[v])) - 1
            for j in range(int(m.vreg_width[v])):
                if (mask >> j) & 1:
                    assert src[k] == o and add[k] == j
                    occ_val[k] = first_id + 1 + j
                    k += 1
    assert k == mp["n_occ_low"]
    whole_occ = whole_of_split[occ_val]
    want_kill = np.where(split[vv[occ_val]], (an.occ_kill[src] >> add) & 1, an.occ_kill[src] != 0)
    assert (got["occ_kill"][~whole_occ] == want_kill[~whole_occ]).all(), (tag, "kill")
    assert not got["occ_kill"][whole_occ].any()
    for x in range(Vl):
        runs = got["seg"][got["seg_off"][x]:got["seg_off"][x + 1]]
        if whole_of_split[x]:
            assert len(runs) == 0
            continue
        y = int(lane_idx[x])
        assert (runs == an.seg[an.seg_off[y]:an.seg_off[y + 1]]).all(), (tag, "seg", x)
        assert (got["hull"][x] == an.hull[y]).all()
    return an


def test_hand_derived_examples():
    with open(os.path.join(GOLD, "lane_examples.json")) as f:
        exs = json.load(f)["examples"]
    mirs, lanes, rows = [], [], []
    for ex in exs:
        occ_v = [op[0] for ins in ex["instrs"] for op in ins]
        occ_f = [op[1] for ins in ex["instrs"] for op in ins]
        off = np.cumsum([0] + [len(ins) for ins in ex["instrs"]])
        V = len(ex["width"])
        mirs.append(Mir([0, len(ex["instrs"])], [0, 0], [], off, occ_v, occ_f, np.zeros(V, np.uint8), ex["width"], ex["align"],
                        ex["class_size"], None, ex["name"]))
        lanes.append(np.array([op[2] for ins in ex["instrs"] for op in ins], np.uint32))
        rows.append(np.array([c["row"] for c in ex["candidates"]], np.uint16))
    for tile_len in (0, 1, 2):
        maps, live, res = run(mirs, lanes, rows, tile_len)
        for ex, m, l, mp, g, r in zip(exs, mirs, lanes, maps, live, res):
            assert_lane_liveness(m, l, mp, g, ex["name"])
            assert [[int(x) for x in rr] for rr in r] == [c["result"] for c in ex["candidates"]], (ex["name"], tile_len)


@pytest.mark.parametrize("tile_len", [0, 1, 3])
def test_tiny_programs_with_lane_masks(tile_len):
    mirs, lanes, rows = [], [], []
    seed = 0
    while len(mirs) < 120:
        m = tiny_mir(9700 + seed, strict=True, reserved=seed % 2 == 0, early=0.25 if seed % 3 == 0 else 0.0, max_instr=6)
        l = tiny_lanes(m, seed)
        seed += 1
        if vlo.analyze(m, interference=False).contract != 0 or vlo.analyze_lanes(m, l).live_in[0].any():
            continue
        mirs.append(m); lanes.append(l); rows.append(tiny_rows(m, seed, K=9))
    maps, live, res = run(mirs, lanes, rows, tile_len)
    hist, n_split = np.zeros(4, int), 0
    for j, (m, l, mp, g, r) in enumerate(zip(mirs, lanes, maps, live, res)):
        an = assert_lane_liveness(m, l, mp, g, f"tiny {j}")
        want = vlo.verify_lanes(m, an, rows[j])
        bad = np.nonzero(want != r)[0]
        assert len(bad) == 0, f"tiny {j} tile {tile_len}: row {bad[0]}: oracle {want[bad[0]]} gpu {r[bad[0]]}"
        hist += np.bincount(want["status"], minlength=4)
        n_split += int((mp["val_lane"] != 0xFF).sum())
    assert (hist > 20).all() and n_split > 100, (hist, n_split)


def test_generated_kernels_with_lane_masks():
    """programs of a few thousand instructions (tuples up to 16 wide, loops, two files) whose
    occurrences outside the entry block access random parts of their tuples"""
    ks = [gen.Kernel(gen.LOOP3, 0x1A0, 900, 700), gen.Kernel(gen.MHA, 0x1A1, 1500, 1100), gen.Kernel(gen.GEMM, 0x1A2, 1200, 900)]
    mirs, lanes, rows = [], [], []
    for j, k in enumerate(ks):
        l = tiny_lanes(k.mir, 77 + j, share=0.3)
        an = vlo.analyze_lanes(k.mir, l)
        if an.live_in[0].any():     # a lane read before the entry block wrote it: leave that vreg whole
            owner = np.repeat(np.arange(k.mir.n_vreg), k.mir.vreg_width)
            l[np.isin(k.mir.occ_vreg, owner[np.nonzero(an.live_in[0])[0]])] = 0
            assert not vlo.analyze_lanes(k.mir, l).live_in[0].any()
        mirs.append(k.mir); lanes.append(l); rows.append(k.candidates(5 + j, 60, 30, 2)[0])
    for tile_len in (0, 100):
        maps, live, res = run(mirs, lanes, rows, tile_len)
        for j, (m, l, mp, g, r) in enumerate(zip(mirs, lanes, maps, live, res)):
            an = assert_lane_liveness(m, l, mp, g, m.name)
            want = vlo.verify_lanes(m, an, rows[j])
            bad = np.nonzero(want != r)[0]
            assert len(bad) == 0, f"{m.name} tile {tile_len}: row {bad[0]}: oracle {want[bad[0]]} gpu {r[bad[0]]}"
            assert (mp["val_lane"] != 0xFF).sum() > 50
            assert set(np.unique(want["status"])) >= {0, 3}


def test_arguments():
    m = tiny_mir(9700, strict=True)
    h = vl.vl_mir_create(m)            # not a handle with lanes
    with pytest.raises(vl.VlError) as e:
        vl.vl_mir_lanes_get(h)
    assert e.value.code == -7
    vl.vl_mir_destroy(h)
    bad = np.zeros(m.n_occ, np.uint32)
    bad[0] = 1 << int(m.vreg_width[m.occ_vreg[0]])      # a lane the vreg does not have
    with pytest.raises(vl.VlError) as e:
        vl.vl_mir_create_lanes(m, bad)
    assert e.value.code == -3
    h = vl.vl_mir_create_lanes(m, tiny_lanes(m, 1))
    hl = vl.vl_liveness(h)
    out = torch.zeros((1, 8), dtype=torch.int32, device="cuda")
    row = torch.zeros((1, 64), dtype=torch.int16, device="cuda")
    with pytest.raises(vl.VlError) as e:
        vl.vl_count_violations_multi([(h, hl, row, 1, 64, out)])
    assert e.value.code == -7
    vl.vl_live_destroy(hl)
    vl.vl_mir_destroy(h)
