"""ctypes wrapper around the C oracle (oracle/vlo.c).  TEST INFRASTRUCTURE ONLY.

Marshals a program description (any object with the array attributes of
vlgen.mir.Mir) into the oracle's own structures and returns numpy arrays.
It imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

from . import build as _build

RESULT_DTYPE = np.dtype([("status", "<u4"), ("where", "<u4"), ("a", "<u4"), ("b", "<u4")])
EDGE_DTYPE = np.dtype([("a", "<u4"), ("b", "<u4"), ("first", "<u4")])
OK, CONSISTENCY, REALIZABILITY, SAFETY = 0, 1, 2, 3
BAD_BOUNDS, BAD_ALIGN, BAD_RESERVED = 1, 2, 4


class _Mir(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in
                ("n_instr", "n_vreg", "n_block", "n_occ", "n_class", "n_edge")] + \
               [(n, C.c_void_p) for n in
                ("blk_start", "succ_off", "succ", "instr_occ_off", "occ_vreg", "occ_flags",
                 "vreg_class", "vreg_width", "vreg_align", "class_size", "class_reserved")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        _lib.vlo_block_liveness.restype = C.c_int
        _lib.vlo_segments.restype = C.c_uint64
        _lib.vlo_interference.restype = C.c_uint64
        _lib.vlo_contract.restype = C.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _marshal(m):
    keep = dict(
        blk_start=np.ascontiguousarray(m.blk_start, np.uint32),
        succ_off=np.ascontiguousarray(m.succ_off, np.uint32),
        succ=np.ascontiguousarray(m.succ, np.uint32),
        instr_occ_off=np.ascontiguousarray(m.instr_occ_off, np.uint32),
        occ_vreg=np.ascontiguousarray(m.occ_vreg, np.uint32),
        occ_flags=np.ascontiguousarray(m.occ_flags, np.uint8),
        vreg_class=np.ascontiguousarray(m.vreg_class, np.uint8),
        vreg_width=np.ascontiguousarray(m.vreg_width, np.uint8),
        vreg_align=np.ascontiguousarray(m.vreg_align, np.uint8),
        class_size=np.ascontiguousarray(m.class_size, np.uint16),
        class_reserved=None if m.class_reserved is None else
        np.ascontiguousarray(m.class_reserved, np.uint32),
    )
    s = _Mir(len(keep["instr_occ_off"]) - 1, len(keep["vreg_class"]), len(keep["blk_start"]) - 1,
             len(keep["occ_vreg"]), len(keep["class_size"]), len(keep["succ"]),
             *[_p(keep[k]) for k in ("blk_start", "succ_off", "succ", "instr_occ_off", "occ_vreg",
                                     "occ_flags", "vreg_class", "vreg_width", "vreg_align",
                                     "class_size", "class_reserved")])
    return s, keep


@dataclass
class Analysis:
    """Everything the oracle derives from a program alone."""
    live_in: np.ndarray      # uint8 [n_block, V]
    live_out: np.ndarray     # uint8 [n_block, V]
    live_after: np.ndarray   # uint32 [N, W] bit-packed
    P: np.ndarray            # uint32 [N, W] occupancy rows
    occ_kill: np.ndarray     # uint8 [O]
    seg_off: np.ndarray      # uint32 [V+1]
    seg: np.ndarray          # uint32 [S, 2]
    hull: np.ndarray         # uint32 [V, 2]
    first: np.ndarray        # uint32 [V]
    sweeps: int
    contract: int
    edges: np.ndarray | None = None  # EDGE_DTYPE [E]


def unpack_bits(rows: np.ndarray, n_vreg: int) -> np.ndarray:
    """[.., W] uint32 -> [.., V] uint8 membership."""
    b = np.unpackbits(np.ascontiguousarray(rows).view(np.uint8), axis=-1, bitorder="little")
    return b[..., :n_vreg]


def pack_bits(member: np.ndarray) -> np.ndarray:
    """[.., V] 0/1 -> [.., W] uint32."""
    V = member.shape[-1]
    W = (V + 31) // 32
    pad = np.zeros(member.shape[:-1] + (W * 32,), np.uint8)
    pad[..., :V] = member
    return np.packbits(pad, axis=-1, bitorder="little").view(np.uint32).reshape(member.shape[:-1] + (W,))


def analyze(m, interference: bool = True, threads: int = 1) -> Analysis:
    s, keep = _marshal(m)
    L = lib()
    N, V, B, O = s.n_instr, s.n_vreg, s.n_block, s.n_occ
    W = (V + 31) // 32
    live_in = np.zeros((B, V), np.uint8)
    live_out = np.zeros((B, V), np.uint8)
    sweeps = L.vlo_block_liveness(C.byref(s), _p(live_in), _p(live_out))
    live_after = np.zeros((N, W), np.uint32)
    L.vlo_points(C.byref(s), _p(live_out), _p(live_after))
    P = np.zeros((N, W), np.uint32)
    L.vlo_occupancy(C.byref(s), _p(live_after), _p(P))
    kill = np.zeros(O, np.uint8)
    L.vlo_kill_flags(C.byref(s), _p(live_after), _p(kill))
    seg_off = np.zeros(V + 1, np.uint32)
    hull = np.zeros((V, 2), np.uint32)
    n = L.vlo_segments(C.byref(s), _p(P), _p(seg_off), None, C.c_uint64(0), _p(hull))
    seg = np.zeros((max(n, 1), 2), np.uint32)
    L.vlo_segments(C.byref(s), _p(P), _p(seg_off), _p(seg), C.c_uint64(n), _p(hull))
    seg = seg[:n]
    first = np.zeros(V, np.uint32)
    L.vlo_first_occurrence(C.byref(s), _p(first))
    contract = L.vlo_contract(C.byref(s), _p(live_in))
    an = Analysis(live_in, live_out, live_after, P, kill, seg_off, seg, hull, first, sweeps, contract)
    if interference:
        an.edges = interference_edges(m, an, threads)
    return an


def interference_edges(m, an: Analysis, threads: int = 1) -> np.ndarray:
    s, keep = _marshal(m)
    L = lib()
    seg = np.ascontiguousarray(an.seg if len(an.seg) else np.zeros((1, 2), np.uint32))
    n = L.vlo_interference(C.byref(s), _p(an.seg_off), _p(seg), None, C.c_uint64(0), C.c_int(threads))
    edges = np.zeros(max(n, 1), EDGE_DTYPE)
    L.vlo_interference(C.byref(s), _p(an.seg_off), _p(seg), _p(edges), C.c_uint64(n), C.c_int(threads))
    return edges[:n]


def verify(m, an: Analysis, cand: np.ndarray, threads: int = 1) -> np.ndarray:
    """cand: uint16 [K, ld] with ld >= n_occ.  Returns RESULT_DTYPE [K]."""
    s, keep = _marshal(m)
    cand = np.asarray(cand)
    assert cand.dtype == np.uint16 and cand.ndim == 2 and cand.shape[1] >= s.n_occ
    assert cand.strides[1] == 2
    K, ld = cand.shape[0], cand.strides[0] // 2
    out = np.zeros(K, RESULT_DTYPE)
    edges = an.edges if an.edges is not None else interference_edges(m, an, threads)
    e = np.ascontiguousarray(edges if len(edges) else np.zeros(1, EDGE_DTYPE))
    lib().vlo_verify(C.byref(s), _p(e), C.c_uint64(len(edges)), _p(cand), C.c_uint32(K),
                     C.c_uint64(ld), _p(out), C.c_int(threads))
    return out


def verify_points(m, an: Analysis, cand: np.ndarray) -> np.ndarray:
    """The literal per-point all-pairs definition, one row at a time."""
    s, keep = _marshal(m)
    cand = np.ascontiguousarray(np.atleast_2d(cand), np.uint16)
    out = np.zeros(cand.shape[0], RESULT_DTYPE)
    P = np.ascontiguousarray(an.P)
    for k in range(cand.shape[0]):
        lib().vlo_verify_points(C.byref(s), _p(P), _p(cand[k]), C.c_void_p(out[k:k + 1].ctypes.data))
    return out


SUMMARY_DTYPE = np.dtype([("first_ok", "<u4"), ("passed", "<u4"), ("hist", "<u4", (4,))])
LOOP_DTYPE = np.dtype([("n_passed", "<u4"), ("max_tries", "<u4"), ("sum_tries", "<u8"), ("hist", "<u8", (4,))])


def summarize(results: np.ndarray) -> np.ndarray:
    """Regeneration-loop reduction over one kernel's verdicts, in sampling order
    (Section 3.4; metrics of Section 4.2).  Returns SUMMARY_DTYPE [1]."""
    res = np.ascontiguousarray(results, RESULT_DTYPE)
    out = np.zeros(1, SUMMARY_DTYPE)
    lib().vlo_summarize(C.c_void_p(res.ctypes.data), C.c_uint32(len(res)), C.c_void_p(out.ctypes.data))
    return out


def loop_stats(summaries: np.ndarray, Ks) -> np.ndarray:
    """Over n kernels: passed kernels, maximum and summed attempts, histogram."""
    s = np.ascontiguousarray(summaries, SUMMARY_DTYPE)
    K = np.ascontiguousarray(Ks, np.uint32)
    assert len(s) == len(K)
    out = np.zeros(1, LOOP_DTYPE)
    lib().vlo_loop(C.c_void_p(s.ctypes.data), C.c_void_p(K.ctypes.data), C.c_uint32(len(s)), C.c_void_p(out.ctypes.data))
    return out


def free_bases(m, an: Analysis, row: np.ndarray, q: int) -> np.ndarray:
    """Bases a decoder may still give occurrence q of `row` (whose occurrences before q
    are fixed) without breaking consistency, realizability or safety against them
    (Section 4.5, error analysis: masking occupied registers).  uint32 [16]."""
    s, keep = _marshal(m)
    row = np.ascontiguousarray(row, np.uint16)
    P = np.ascontiguousarray(an.P)
    out = np.zeros(16, np.uint32)
    lib().vlo_free_bases(C.byref(s), _p(P), _p(row), C.c_uint32(q), _p(out))
    return out


COUNTS_DTYPE = np.dtype([("kinds", "<u4"), ("n_cons", "<u4"), ("n_real", "<u4"), ("n_safe", "<u4"), ("real_bits", "<u4"),
                         ("pad", "<u4", (3,))])


def count_violations(m, an: Analysis, cand: np.ndarray, threads: int = 1) -> np.ndarray:
    """Every violation of each candidate row, by kind (Section 4.5 error taxonomy;
    Section 6: the verifier as feedback or reward).  Returns COUNTS_DTYPE [K]."""
    s, keep = _marshal(m)
    cand = np.ascontiguousarray(np.atleast_2d(cand), np.uint16)
    out = np.zeros(cand.shape[0], COUNTS_DTYPE)
    edges = an.edges if an.edges is not None else interference_edges(m, an, threads)
    e = np.ascontiguousarray(edges if len(edges) else np.zeros(1, EDGE_DTYPE))
    lib().vlo_count_violations(C.byref(s), _p(e), C.c_uint64(len(edges)), _p(cand),
                               C.c_uint32(cand.shape[0]), C.c_uint64(cand.shape[1]), C.c_void_p(out.ctypes.data),
                               C.c_int(threads))
    return out


def bank_conflicts(m, cand: np.ndarray, n_banks: int = 4) -> np.ndarray:
    """Stall cycles from register-bank conflicts per candidate row (Section 2: banks and
    the FFMA example).  uint32 [K]."""
    s, keep = _marshal(m)
    cand = np.ascontiguousarray(np.atleast_2d(cand), np.uint16)
    out = np.zeros(cand.shape[0], np.uint32)
    lib().vlo_bank_conflicts(C.byref(s), _p(cand), C.c_uint32(cand.shape[0]), C.c_uint64(cand.shape[1]),
                             C.c_uint32(n_banks), _p(out))
    return out


# ---- liveness of parts of a tuple (sub-register liveness) ----

@dataclass
class LaneAnalysis:
    """Per (vreg, lane); lane (v, j) has the index lane_base[v] + j."""
    lane_base: np.ndarray    # uint32 [V+1]
    live_in: np.ndarray      # uint8 [n_block, Lt]
    live_out: np.ndarray     # uint8 [n_block, Lt]
    live_after: np.ndarray   # uint8 [N, Lt]
    P: np.ndarray            # uint8 [N, Lt]
    occ_kill: np.ndarray     # uint32 [O]: lanes read for the last time
    seg_off: np.ndarray      # uint32 [Lt+1]
    seg: np.ndarray          # uint32 [S, 2]
    hull: np.ndarray         # uint32 [Lt, 2]
    sweeps: int


def _lanes(m, occ_lanes):
    if occ_lanes is None:
        return None
    a = np.ascontiguousarray(occ_lanes, np.uint32)
    assert a.shape == (len(m.occ_vreg),)
    return a


def analyze_lanes(m, occ_lanes=None) -> LaneAnalysis:
    """occ_lanes: uint32 [n_occ], bit j = the occurrence accesses lane j of its vreg; None
    or 0 = all lanes."""
    s, keep = _marshal(m)
    L = lib()
    L.vlo_block_liveness_lanes.restype = C.c_int
    L.vlo_segments_lanes.restype = C.c_uint64
    lanes = _lanes(m, occ_lanes)
    N, V, B, O = s.n_instr, s.n_vreg, s.n_block, s.n_occ
    base = np.zeros(V + 1, np.uint32)
    L.vlo_lane_base(C.byref(s), _p(base))
    Lt = int(base[V])
    live_in = np.zeros((B, Lt), np.uint8)
    live_out = np.zeros((B, Lt), np.uint8)
    sweeps = L.vlo_block_liveness_lanes(C.byref(s), _p(lanes), _p(live_in), _p(live_out))
    live_after = np.zeros((N, Lt), np.uint8)
    L.vlo_points_lanes(C.byref(s), _p(lanes), _p(live_out), _p(live_after))
    P = np.zeros((N, Lt), np.uint8)
    L.vlo_occupancy_lanes(C.byref(s), _p(lanes), _p(live_after), _p(P))
    kill = np.zeros(O, np.uint32)
    L.vlo_kill_lanes(C.byref(s), _p(lanes), _p(live_after), _p(kill))
    seg_off = np.zeros(Lt + 1, np.uint32)
    hull = np.zeros((max(Lt, 1), 2), np.uint32)
    n = L.vlo_segments_lanes(C.byref(s), _p(P), _p(seg_off), None, C.c_uint64(0), _p(hull))
    seg = np.zeros((max(n, 1), 2), np.uint32)
    L.vlo_segments_lanes(C.byref(s), _p(P), _p(seg_off), _p(seg), C.c_uint64(n), _p(hull))
    return LaneAnalysis(base, live_in, live_out, live_after, P, kill, seg_off, seg[:n], hull[:Lt], sweeps)


def verify_lanes(m, an: LaneAnalysis, cand: np.ndarray) -> np.ndarray:
    """Consistency and realizability per vreg, safety on the lanes in use.  RESULT_DTYPE [K]."""
    s, keep = _marshal(m)
    cand = np.ascontiguousarray(np.atleast_2d(cand), np.uint16)
    out = np.zeros(cand.shape[0], RESULT_DTYPE)
    P = np.ascontiguousarray(an.P)
    for k in range(cand.shape[0]):
        lib().vlo_verify_lanes(C.byref(s), _p(P), _p(cand[k]), C.c_void_p(out[k:k + 1].ctypes.data))
    return out
