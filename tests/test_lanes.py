"""Pins for the oracle's liveness of parts of a tuple (lane masks on occurrences): with all
masks full it is the plain oracle; hand-derived examples; path search and pair enumeration
per (vreg, lane) in Python; and a program rewritten by hand with one vreg per lane, run
through the plain oracle."""
import json
import os

import numpy as np
import pytest

import bruteforce as bf
from oracle import vlo
from vlgen import gen
from vlgen.mir import Mir
from vlgen.tiny import tiny_lanes, tiny_mir, tiny_rows

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def lane_sets(rows, an, m):
    """[N, Lt] bytes -> per instruction the set of (vreg, lane)"""
    owner = np.repeat(np.arange(m.n_vreg), m.vreg_width)
    lane = np.arange(len(owner)) - an.lane_base[owner]
    return [set((int(owner[x]), int(lane[x])) for x in np.nonzero(r)[0]) for r in rows]


def test_hand_derived_examples():
    with open(os.path.join(GOLD, "lane_examples.json")) as f:
        exs = json.load(f)["examples"]
    for ex in exs:
        occ_v = [op[0] for ins in ex["instrs"] for op in ins]
        occ_f = [op[1] for ins in ex["instrs"] for op in ins]
        lanes = [op[2] for ins in ex["instrs"] for op in ins]
        off = np.cumsum([0] + [len(ins) for ins in ex["instrs"]])
        V = len(ex["width"])
        m = Mir([0, len(ex["instrs"])], [0, 0], [], off, occ_v, occ_f, np.zeros(V, np.uint8), ex["width"], ex["align"],
                ex["class_size"], None, ex["name"], np.array(lanes, np.uint32))
        an = vlo.analyze_lanes(m, m.occ_lanes)
        assert lane_sets(an.live_after, an, m) == [set(tuple(x) for x in s) for s in ex["live_after"]], ex["name"]
        assert an.occ_kill.tolist() == ex["kills"], ex["name"]
        for key, runs in ex["segments"].items():
            v, j = (int(t) for t in key.split(","))
            x = int(an.lane_base[v]) + j
            assert an.seg[an.seg_off[x]:an.seg_off[x + 1]].tolist() == runs, (ex["name"], key)
        for c in ex["candidates"]:
            r = vlo.verify_lanes(m, an, np.array([c["row"]], np.uint16))[0]
            assert [int(x) for x in r] == c["result"], (ex["name"], c)


def test_full_masks_reduce_to_the_plain_oracle():
    def check(m, rows):
        plain = vlo.analyze(m)
        for lanes in (None, np.zeros(m.n_occ, np.uint32),
                      ((1 << m.vreg_width[m.occ_vreg].astype(np.uint64)) - 1).astype(np.uint32)):
            an = vlo.analyze_lanes(m, lanes)
            per_lane = np.repeat(np.arange(m.n_vreg), m.vreg_width)   # every lane behaves as its vreg
            assert (an.live_in == plain.live_in[:, per_lane]).all() and (an.live_out == plain.live_out[:, per_lane]).all()
            assert (an.live_after == vlo.unpack_bits(plain.live_after, m.n_vreg)[:, per_lane]).all()
            assert (an.P == vlo.unpack_bits(plain.P, m.n_vreg)[:, per_lane]).all()
            assert ((an.occ_kill != 0) == (plain.occ_kill != 0)).all()
            for v in range(m.n_vreg):
                for j in range(int(m.vreg_width[v])):
                    x = int(an.lane_base[v]) + j
                    assert (an.seg[an.seg_off[x]:an.seg_off[x + 1]] == plain.seg[plain.seg_off[v]:plain.seg_off[v + 1]]).all()
            assert (vlo.verify_lanes(m, an, rows) == vlo.verify(m, plain, rows)).all()
    for seed in range(120):
        m = tiny_mir(9000 + seed, reserved=seed % 3 == 0, early=0.3 if seed % 2 else 0.0)
        check(m, tiny_rows(m, seed, K=6))
    w = gen.config(2, scale=0.3)
    check(w.kernels[0].mir, w.rows[0][:40])


def test_lanes_against_path_search_and_enumeration():
    n_status, n_partial = [0, 0, 0, 0], 0
    for seed in range(220):
        m = tiny_mir(9200 + seed, strict=seed % 2 == 0, early=0.25 if seed % 3 == 0 else 0.0)
        lanes = tiny_lanes(m, seed, keep_first_block=seed % 4 != 3)
        n_partial += int((lanes != 0).sum())
        an = vlo.analyze_lanes(m, lanes)
        la = bf.live_after_lanes_by_search(m, lanes)
        assert lane_sets(an.live_after, an, m) == la, seed
        P = bf.occupancy_lanes(m, lanes, la)
        assert lane_sets(an.P, an, m) == P, seed
        uses, defs = bf.uses_defs_lanes(m, lanes)
        instr = np.repeat(np.arange(m.n_instr), np.diff(m.instr_occ_off))
        for o in range(m.n_occ):
            v, i = int(m.occ_vreg[o]), int(instr[o])
            want = 0
            for j in range(int(m.vreg_width[v])):
                if (m.occ_flags[o] & 2) and bf.lane_touch(m, lanes, o, j) and (v, j) not in la[i] and (v, j) not in defs[i]:
                    want |= 1 << j
            assert int(an.occ_kill[o]) == want, (seed, o)
        for v in range(m.n_vreg):
            for j in range(int(m.vreg_width[v])):
                member = [(v, j) in P[i] for i in range(m.n_instr)]
                runs, i = [], 0
                while i < m.n_instr:
                    if member[i]:
                        k = i
                        while k < m.n_instr and member[k]:
                            k += 1
                        runs.append([i, k])
                        i = k
                    else:
                        i += 1
                x = int(an.lane_base[v]) + j
                assert an.seg[an.seg_off[x]:an.seg_off[x + 1]].tolist() == runs, (seed, v, j)
                assert an.hull[x].tolist() == ([runs[0][0], runs[-1][1]] if runs else [0, 0])
        rows = tiny_rows(m, seed, K=6)
        got = vlo.verify_lanes(m, an, rows)
        for k in range(len(rows)):
            want = bf.verify_lanes(m, P, rows[k])
            assert tuple(int(x) for x in got[k]) == want, (seed, k)
            n_status[want[0]] += 1
    assert n_partial > 300 and all(n > 25 for n in n_status), (n_partial, n_status)


def test_one_vreg_per_lane_by_hand_gives_the_same_safety():
    """Rewriting a program so that every lane is a vreg of its own (width 1), each occurrence
    becoming one occurrence per lane it accesses, and giving the lanes the registers base + j:
    the plain oracle then finds a register clash exactly where the lane oracle does."""
    checked = 0
    for seed in range(150):
        m = tiny_mir(9500 + seed, early=0.0)
        lanes = tiny_lanes(m, seed)
        an = vlo.analyze_lanes(m, lanes)
        base = an.lane_base
        occ_v, occ_f, off, src, add = [], [], [0], [], []
        for i in range(m.n_instr):
            for o in range(m.instr_occ_off[i], m.instr_occ_off[i + 1]):
                v = int(m.occ_vreg[o])
                for j in range(int(m.vreg_width[v])):
                    if bf.lane_touch(m, lanes, o, j):
                        occ_v.append(int(base[v]) + j); occ_f.append(int(m.occ_flags[o])); src.append(o); add.append(j)
            off.append(len(occ_v))
        Lt = int(base[m.n_vreg])
        owner = np.repeat(np.arange(m.n_vreg), m.vreg_width)
        if max(np.diff(off)) > 64:
            continue
        m2 = Mir(m.blk_start, m.succ_off, m.succ, off, occ_v, occ_f, m.vreg_class[owner], np.ones(Lt, np.uint8),
                 np.ones(Lt, np.uint8), m.class_size)
        an2 = vlo.analyze(m2)
        rows = tiny_rows(m, seed, K=6)
        got = vlo.verify_lanes(m, an, rows)
        for k in range(len(rows)):
            if got[k]["status"] in (1, 2):
                continue   # decided per vreg and whole tuple: nothing the rewritten program knows of
            row2 = (rows[k][src].astype(np.int64) + np.array(add)).astype(np.uint16)[None, :]
            r2 = vlo.verify_points(m2, an2, row2)[0]
            assert int(r2["status"]) in (0, 3)
            assert int(r2["status"]) == int(got[k]["status"]), (seed, k)
            if r2["status"] == 3:
                # the same instruction; the pair reported is the smallest pair of vregs, which need not be
                # the vregs of the smallest pair of lanes: take the smallest over all clashing lanes there
                i = int(r2["where"])
                assert i == int(got[k]["where"])
                here = np.nonzero(vlo.unpack_bits(an2.P[i:i + 1], Lt)[0])[0]
                pairs = [(int(owner[x]), int(owner[y])) for x in here for y in here
                         if x < y and owner[x] != owner[y] and m2.vreg_class[x] == m2.vreg_class[y] and row2[0, an2.first[x]] == row2[0, an2.first[y]]]
                assert min(pairs) == (int(got[k]["a"]), int(got[k]["b"])), (seed, k)
            checked += 1
    assert checked > 300
