"""The synthetic workloads against the oracle: allocations made from the
generator's own occupancy ranges always verify, every guaranteed damage is
caught with the predicted status, and what the generator claims to know about
its programs holds."""
import numpy as np
import pytest

from oracle import vlo
from vlgen import gen


def check_kernel(k, rows, log):
    m = k.mir
    an = vlo.analyze(m, threads=8)
    assert an.contract == 0
    # recorded ranges contain the real intervals; certain ranges lie inside one
    for v in range(m.n_vreg):
        s = an.seg[an.seg_off[v]:an.seg_off[v + 1]]
        if len(s):
            assert k.range[v, 0] <= s[0, 0] and s[-1, 1] <= k.range[v, 1], v
        if k.sure[v, 1] > k.sure[v, 0]:
            assert any(a <= k.sure[v, 0] and k.sure[v, 1] <= b for a, b in s), v
    res = vlo.verify(m, an, rows, threads=8)
    clean = log["kind"] == 0
    assert (res["status"][clean] == vlo.OK).all()
    known = log["expect"] != 255
    assert (res["status"][known] == log["expect"][known]).all()
    return an, res


def test_config1_shape_and_results():
    w = gen.config(1)
    m = w.kernels[0].mir
    assert (m.n_instr, m.n_vreg, m.n_block, m.n_occ) == (200, 200, 1, 598)
    assert w.rows[0].shape == (64, 598)
    log = w.logs[0]
    assert (log["kind"] == 0).sum() == 32 and (log["kind"] == 5).sum() == 16 and (log["kind"] == 1).sum() == 16
    an, res = check_kernel(w.kernels[0], w.rows[0], log)
    assert (res["status"] == vlo.CONSISTENCY).sum() == 16
    # the literal per-point checker agrees on every row
    assert (vlo.verify_points(m, an, w.rows[0]) == res).all()


def test_config2_shape_and_results():
    w = gen.config(2)
    m = w.kernels[0].mir
    assert (m.n_instr, m.n_vreg, m.n_block) == (2000, 1500, 3)
    assert m.blk_start.tolist() == [0, 300, 1700, 2000]
    assert m.class_size.tolist() == [256, 102]
    assert (w.logs[0]["kind"] != 0).sum() == 50
    an, res = check_kernel(w.kernels[0], w.rows[0], w.logs[0])
    # some values are live around the back edge
    assert an.live_out[1].sum() >= 37 and (an.live_in[1] & an.live_out[1]).sum() >= 37
    assert (vlo.verify_points(m, an, w.rows[0][:10]) == res[:10]).all()
    assert set(np.unique(res["status"])) == {0, 1, 2, 3}


def test_config3_gemm_shape():
    w = gen.config(3, scale=0.25)
    m = w.kernels[0].mir
    assert m.n_block == 22 and m.class_size.tolist() == [512, 102]
    assert (m.vreg_width == 16).sum() == 64
    an, res = check_kernel(w.kernels[0], w.rows[0], w.logs[0])
    assert (res["status"] == vlo.SAFETY).sum() == (w.logs[0]["kind"] == 4).sum()


@pytest.mark.parametrize("cfg,nk", [(4, 1), (5, 6)])
def test_config45_kernels(cfg, nk):
    w = gen.config(cfg, n_kernels=nk)
    for k, rows, log in zip(w.kernels, w.rows, w.logs):
        assert rows.shape[0] == 100 and (log["kind"] != 0).sum() == 20
        check_kernel(k, rows, log)
    if cfg == 4:
        m = w.kernels[0].mir
        assert (m.n_instr, m.n_vreg) == (20000, 15000)
        assert set(np.unique(m.vreg_width)) == {1, 2, 4, 8, 16}


def test_generator_is_deterministic():
    a, b = gen.config(2), gen.config(2)
    assert (a.rows[0] == b.rows[0]).all() and (a.logs[0] == b.logs[0]).all()
    assert (a.kernels[0].mir.occ_vreg == b.kernels[0].mir.occ_vreg).all()
    assert gen.sweep_sizes(4) == gen.sweep_sizes(4)
    s = gen.sweep_sizes(256)
    assert min(s) >= 1000 and max(s) <= 20000


def test_mixed_shape_programs_meet_the_input_contract():
    """The mixed-shape generator writes every value before it is read on every path
    (nothing live into the entry) and covers the shapes it is there for."""
    from vlgen.mixed import mixed_mir
    for seed in range(6):
        m = mixed_mir(0xA000 + seed, n_instr=700, reserved=seed % 2 == 1)
        an = vlo.analyze(m, interference=False)
        assert an.contract == 0, seed
        assert not an.live_in[0].any()
        assert m.vreg_width.max() == 32 and (m.vreg_align == 3).any() and len(m.class_size) == 3
        assert np.diff(m.instr_occ_off).max() >= 30
    m = mixed_mir(0xC001, n_instr=700, stretch=23000)
    last, worst = {}, 0
    for o, v in enumerate(m.occ_vreg):
        if v in last:
            worst = max(worst, o - last[v])
        last[v] = o
    assert worst > 65535


def test_many_block_programs_meet_the_input_contract():
    from vlgen.mixed import many_blocks_mir
    for seed in range(3):
        m = many_blocks_mir(seed, n_blocks=60, gap=5)
        an = vlo.analyze(m, interference=False)
        assert an.contract == 0, seed
        assert not an.live_in[0].any()
        assert m.n_block == 60
        # extra edges exist, some of them backwards, and some vreg numbers are never mentioned
        succ = [list(m.succ[m.succ_off[b]:m.succ_off[b + 1]]) for b in range(m.n_block)]
        assert any(len(s) == 2 for s in succ) and any(t <= b for b, s in enumerate(succ) for t in s)
        assert (np.bincount(m.occ_vreg, minlength=m.n_vreg) == 0).sum() >= 60 * 5
