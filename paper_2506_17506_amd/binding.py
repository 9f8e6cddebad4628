"""ctypes binding of libvl.so.  Argument marshalling only: every step of the
path runs in the library's kernels.  torch supplies device memory and streams.

The functions carry the names of the C entry points (include/vl.h).  Handles
are returned as opaque ctypes pointers; the caller destroys them.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libvl.so")

VL_DENSE_POINTS = 1
RESULT_DTYPE = np.dtype([("status", "<u4"), ("where", "<u4"), ("a", "<u4"), ("b", "<u4")])
SUMMARY_DTYPE = np.dtype([("first_ok", "<u4"), ("passed", "<u4"), ("hist", "<u4", (4,))])                       # vl_summary
LOOP_DTYPE = np.dtype([("n_passed", "<u4"), ("max_tries", "<u4"), ("sum_tries", "<u8"), ("hist", "<u8", (4,))])  # vl_loop_stats


class VlError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {vl_strerror(code)} (code {code}, hip {vl_last_hip_error()})")
        self.code = code


class _Desc(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in
                ("n_instr", "n_vreg", "n_block", "n_occ", "n_class", "n_edge")] + \
               [(n, C.c_void_p) for n in
                ("blk_start", "succ_off", "succ", "instr_occ_off", "occ_vreg", "occ_flags",
                 "vreg_class", "vreg_width", "vreg_align", "class_size", "class_reserved")]


class _View(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in
                ("n_instr", "n_vreg", "n_block", "n_occ", "words", "n_seg", "n_tile", "tile_len",
                 "plan_len", "sweeps")] + \
               [(n, C.c_void_p) for n in
                ("live_in", "live_out", "live_after", "occ_kill", "seg_off", "seg", "hull")]


class _LanesView(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("n_occ", "n_vreg", "n_occ_low", "n_vreg_low")] + \
               [(n, C.c_void_p) for n in ("occ_src", "occ_add", "val_vreg", "val_lane")]


class _CountJob(C.Structure):
    _fields_ = [("mir", C.c_void_p), ("live", C.c_void_p), ("cand", C.c_void_p), ("K", C.c_uint32),
                ("ld", C.c_uint64), ("out", C.c_void_p)]


class _MaskQuery(C.Structure):
    _fields_ = [("mir", C.c_void_p), ("live", C.c_void_p), ("cand", C.c_void_p), ("occ", C.c_uint32),
                ("reserved0", C.c_uint32)]


class _Job(C.Structure):
    _fields_ = [("mir", C.c_void_p), ("live", C.c_void_p), ("cand", C.c_void_p), ("K", C.c_uint32),
                ("ld", C.c_uint64), ("out", C.c_void_p)]


_lib = None


def load():
    """Loads the built library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2506_17506_amd.build` (hipcc, gfx950)")
        # torch first: the library must bind to the HIP runtime torch has loaded, so that
        # both see the same device context and allocations
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        L.vl_mir_create.restype = C.c_int32
        L.vl_mir_create.argtypes = [C.c_void_p, C.POINTER(C.c_void_p)]
        L.vl_mir_create_lanes.restype = C.c_int32
        L.vl_mir_create_lanes.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]
        L.vl_mir_lanes_get.restype = C.c_int32
        L.vl_mir_lanes_get.argtypes = [C.c_void_p, C.c_void_p]
        L.vl_lanes_expand.restype = C.c_int32
        L.vl_lanes_expand.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint64, C.c_void_p, C.c_uint64, C.c_void_p]
        L.vl_mir_destroy.restype = None
        L.vl_mir_destroy.argtypes = [C.c_void_p]
        L.vl_liveness_multi.restype = C.c_int32
        L.vl_liveness_multi.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p]
        L.vl_liveness.restype = C.c_int32
        L.vl_liveness.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p, C.POINTER(C.c_void_p)]
        L.vl_live_destroy.restype = None
        L.vl_live_destroy.argtypes = [C.c_void_p]
        L.vl_live_get.restype = C.c_int32
        L.vl_live_get.argtypes = [C.c_void_p, C.c_void_p]
        L.vl_verify_batch.restype = C.c_int32
        L.vl_verify_batch.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint64, C.c_void_p, C.c_void_p]
        L.vl_verify_batch_static.restype = C.c_int32
        L.vl_verify_batch_static.argtypes = L.vl_verify_batch.argtypes
        L.vl_verify_multi.restype = C.c_int32
        L.vl_verify_multi.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p]
        L.vl_verify_multi_occ_major.restype = C.c_int32
        L.vl_verify_multi_occ_major.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p]
        L.vl_summarize_multi.restype = C.c_int32
        L.vl_summarize_multi.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.vl_count_violations_multi.restype = C.c_int32
        L.vl_count_violations_multi.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p]
        L.vl_bank_conflicts.restype = C.c_int32
        L.vl_bank_conflicts.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint64, C.c_uint32, C.c_void_p, C.c_void_p]
        L.vl_free_bases_multi.restype = C.c_int32
        L.vl_free_bases_multi.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p]
        L.vl_strerror.restype = C.c_char_p
        L.vl_strerror.argtypes = [C.c_int32]
        L.vl_last_hip_error.restype = C.c_int32
        _lib = L
    return _lib


def vl_strerror(code: int) -> str:
    return load().vl_strerror(code).decode()


def vl_last_hip_error() -> int:
    return int(load().vl_last_hip_error())


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(int(getattr(stream, "cuda_stream", stream)))


def make_desc(m):
    """(desc, keepalive) for any object with the array attributes of a program
    description (blk_start, succ_off, succ, instr_occ_off, occ_vreg, occ_flags,
    vreg_class, vreg_width, vreg_align, class_size, class_reserved)."""
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
        class_reserved=None if getattr(m, "class_reserved", None) is None else
        np.ascontiguousarray(m.class_reserved, np.uint32),
    )
    d = _Desc(len(keep["instr_occ_off"]) - 1, len(keep["vreg_class"]), len(keep["blk_start"]) - 1,
              len(keep["occ_vreg"]), len(keep["class_size"]), len(keep["succ"]),
              *[_p(keep[k]) for k in ("blk_start", "succ_off", "succ", "instr_occ_off", "occ_vreg",
                                      "occ_flags", "vreg_class", "vreg_width", "vreg_align",
                                      "class_size", "class_reserved")])
    return d, keep


def vl_mir_create(m) -> C.c_void_p:
    d, keep = m if isinstance(m, tuple) else make_desc(m)
    out = C.c_void_p()
    rc = load().vl_mir_create(C.byref(d), C.byref(out))
    if rc != 0:
        raise VlError(rc, "vl_mir_create")
    return out


def vl_mir_create_lanes(m, occ_lanes=None) -> C.c_void_p:
    """occ_lanes: uint32 [n_occ] (bit j = lane j, 0 = all) or None; defaults to m.occ_lanes."""
    d, keep = m if isinstance(m, tuple) else make_desc(m)
    if occ_lanes is None and not isinstance(m, tuple):
        occ_lanes = getattr(m, "occ_lanes", None)
    lanes = None if occ_lanes is None else np.ascontiguousarray(occ_lanes, np.uint32)
    out = C.c_void_p()
    rc = load().vl_mir_create_lanes(C.byref(d), _p(lanes), C.byref(out))
    if rc != 0:
        raise VlError(rc, "vl_mir_create_lanes")
    return out


def vl_mir_lanes_get(mir) -> dict:
    """The maps of a handle made by vl_mir_create_lanes, copied to numpy (synchronises)."""
    v = _LanesView()
    rc = load().vl_mir_lanes_get(mir, C.byref(v))
    if rc != 0:
        raise VlError(rc, "vl_mir_lanes_get")
    import torch
    torch.cuda.synchronize()
    hip = hip_runtime()

    def grab(ptr, n, dtype):
        a = np.zeros(n, dtype)
        if ptr and a.nbytes:
            assert hip.hipMemcpy(_p(a), C.c_void_p(ptr), a.nbytes, 2) == 0
        return a
    return dict(n_occ=v.n_occ, n_vreg=v.n_vreg, n_occ_low=v.n_occ_low, n_vreg_low=v.n_vreg_low,
                occ_src=grab(v.occ_src, v.n_occ_low, np.uint32), occ_add=grab(v.occ_add, v.n_occ_low, np.uint8),
                val_vreg=grab(v.val_vreg, v.n_vreg_low, np.uint32), val_lane=grab(v.val_lane, v.n_vreg_low, np.uint8))


def vl_lanes_expand(mir, cand, K: int, ld: int, cand_low, ld_low: int, stream=None) -> None:
    """cand, cand_low: device pointers or tensors of uint16 rows."""
    rc = load().vl_lanes_expand(mir, C.c_void_p(_dev_ptr(cand)), K, ld, C.c_void_p(_dev_ptr(cand_low)), ld_low,
                                _stream_ptr(stream))
    if rc != 0:
        raise VlError(rc, "vl_lanes_expand")


def vl_mir_destroy(mir) -> None:
    load().vl_mir_destroy(mir)


def vl_liveness_multi(mirs, flags: int = 0, tile_len: int = 0, stream=None, live=None):
    """Returns the list of live handles; pass the previous list as `live` to
    reuse its device storage."""
    n = len(mirs)
    arr_m = (C.c_void_p * n)(*[m.value for m in mirs])
    arr_l = (C.c_void_p * n)(*([None] * n if live is None else [l.value for l in live]))
    rc = load().vl_liveness_multi(arr_m, n, flags, tile_len, _stream_ptr(stream), arr_l)
    if rc != 0:
        raise VlError(rc, "vl_liveness_multi")
    return [C.c_void_p(arr_l[k]) for k in range(n)]


def vl_liveness(mir, flags: int = 0, stream=None) -> C.c_void_p:
    out = C.c_void_p()
    rc = load().vl_liveness(mir, flags, _stream_ptr(stream), C.byref(out))
    if rc != 0:
        raise VlError(rc, "vl_liveness")
    return out


def vl_live_destroy(live) -> None:
    load().vl_live_destroy(live)


def vl_live_get(live) -> _View:
    v = _View()
    rc = load().vl_live_get(live, C.byref(v))
    if rc != 0:
        raise VlError(rc, "vl_live_get")
    return v


def vl_verify_batch(mir, live, cand, K: int, ld: int, out, stream=None) -> None:
    """cand, out: device pointers (int) or torch tensors."""
    rc = load().vl_verify_batch(mir, live, C.c_void_p(_dev_ptr(cand)), K, ld, C.c_void_p(_dev_ptr(out)),
                                _stream_ptr(stream))
    if rc != 0:
        raise VlError(rc, "vl_verify_batch")


def vl_verify_batch_static(mir, live, cand, K: int, ld: int, out, stream=None) -> None:
    """vl_verify_batch without any allocation inside the library."""
    rc = load().vl_verify_batch_static(mir, live, C.c_void_p(_dev_ptr(cand)), K, ld, C.c_void_p(_dev_ptr(out)),
                                       _stream_ptr(stream))
    if rc != 0:
        raise VlError(rc, "vl_verify_batch_static")


def make_jobs(jobs):
    """jobs: sequence of (mir, live, cand, K, ld, out) -> ctypes array (reusable)."""
    arr = (_Job * len(jobs))()
    for i, (mir, live, cand, K, ld, out) in enumerate(jobs):
        arr[i].mir, arr[i].live = mir.value, live.value
        arr[i].cand, arr[i].K, arr[i].ld, arr[i].out = _dev_ptr(cand), K, ld, _dev_ptr(out)
    return arr


def vl_verify_multi(jobs, stream=None) -> None:
    arr = jobs if isinstance(jobs, C.Array) else make_jobs(jobs)
    rc = load().vl_verify_multi(arr, len(arr), _stream_ptr(stream))
    if rc != 0:
        raise VlError(rc, "vl_verify_multi")


def vl_verify_multi_occ_major(jobs, stream=None) -> None:
    """jobs as for vl_verify_multi, but cand is [n_occ][ld] (occurrence-major), ld >= K."""
    arr = jobs if isinstance(jobs, C.Array) else make_jobs(jobs)
    rc = load().vl_verify_multi_occ_major(arr, len(arr), _stream_ptr(stream))
    if rc != 0:
        raise VlError(rc, "vl_verify_multi_occ_major")


def vl_summarize_multi(jobs, summaries, stats=None, stream=None) -> None:
    """summaries: device buffer of len(jobs) vl_summary records (24 bytes each); stats:
    device buffer of one vl_loop_stats record (48 bytes) or None."""
    arr = jobs if isinstance(jobs, C.Array) else make_jobs(jobs)
    rc = load().vl_summarize_multi(arr, len(arr), C.c_void_p(_dev_ptr(summaries)),
                                   C.c_void_p(_dev_ptr(stats)) if stats is not None else None, _stream_ptr(stream))
    if rc != 0:
        raise VlError(rc, "vl_summarize_multi")


COUNTS_DTYPE = np.dtype([("kinds", "<u4"), ("n_cons", "<u4"), ("n_real", "<u4"), ("n_safe", "<u4"), ("real_bits", "<u4"),
                         ("reserved", "<u4", (3,))])


def vl_count_violations_multi(jobs, stream=None) -> None:
    """jobs: sequence of (mir, live, cand, K, ld, out) with out a device buffer of K records
    of 32 bytes (COUNTS_DTYPE)."""
    arr = (_CountJob * len(jobs))()
    for i, (mir, live, cand, K, ld, out) in enumerate(jobs):
        arr[i].mir, arr[i].live = mir.value, live.value
        arr[i].cand, arr[i].K, arr[i].ld, arr[i].out = _dev_ptr(cand), K, ld, _dev_ptr(out)
    rc = load().vl_count_violations_multi(arr, len(arr), _stream_ptr(stream))
    if rc != 0:
        raise VlError(rc, "vl_count_violations_multi")


def vl_bank_conflicts(mir, cand, K: int, ld: int, n_banks: int, out, stream=None) -> None:
    """out: device buffer of K uint32."""
    rc = load().vl_bank_conflicts(mir, C.c_void_p(_dev_ptr(cand)), K, ld, n_banks, C.c_void_p(_dev_ptr(out)),
                                  _stream_ptr(stream))
    if rc != 0:
        raise VlError(rc, "vl_bank_conflicts")


def make_mask_queries(queries):
    """queries: sequence of (mir, live, row, occ), row a device pointer or tensor holding one
    candidate row -> ctypes array (reusable)."""
    arr = (_MaskQuery * len(queries))()
    for j, (mir, live, row, occ) in enumerate(queries):
        arr[j].mir, arr[j].live, arr[j].cand, arr[j].occ, arr[j].reserved0 = mir.value, live.value, _dev_ptr(row), occ, 0
    return arr


def vl_free_bases_multi(queries, masks, stream=None) -> None:
    """masks: device buffer of 16 uint32 per query."""
    arr = queries if isinstance(queries, C.Array) else make_mask_queries(queries)
    rc = load().vl_free_bases_multi(arr, len(arr), C.c_void_p(_dev_ptr(masks)), _stream_ptr(stream))
    if rc != 0:
        raise VlError(rc, "vl_free_bases_multi")


def _dev_ptr(x) -> int:
    return int(x.data_ptr()) if hasattr(x, "data_ptr") else int(x)


# ---- helpers around torch device memory (no arithmetic of the method) ----

def pad_ld(n_occ: int) -> int:
    """Row pitch in elements: rows start on 128-byte lines."""
    return max(64, (n_occ + 63) // 64 * 64)


def rows_to_device(rows: np.ndarray, device="cuda"):
    """uint16 [K, O] host rows -> (int16 device tensor [K, ld], ld)."""
    import torch
    K, O = rows.shape
    ld = pad_ld(O)
    host = np.zeros((K, ld), np.uint16)
    host[:, :O] = rows
    return torch.from_numpy(host.view(np.int16)).to(device), ld


_hip = None


def hip_runtime():
    """The HIP runtime library already mapped into this process (torch's)."""
    global _hip
    if _hip is None:
        import torch  # noqa: F401
        path = "libamdhip64.so"
        with open("/proc/self/maps") as f:
            for line in f:
                if "libamdhip64" in line:
                    path = line.split()[-1]
                    break
        _hip = C.CDLL(path)
        _hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
        _hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        _hip.hipEventDestroy.argtypes = [C.c_void_p]
        _hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
    return _hip


def view_to_numpy(v: _View) -> dict:
    """Copies the device arrays of a live view to numpy (synchronises)."""
    import torch
    torch.cuda.synchronize()
    hip = hip_runtime()

    def grab(ptr, shape, dtype):
        a = np.zeros(shape, dtype)
        if ptr and a.nbytes:
            rc = hip.hipMemcpy(_p(a), C.c_void_p(ptr), a.nbytes, 2)
            if rc != 0:
                raise RuntimeError(f"hipMemcpy failed: {rc}")
        return a
    W = v.words
    out = dict(
        live_in=grab(v.live_in, (v.n_block, W), np.uint32),
        live_out=grab(v.live_out, (v.n_block, W), np.uint32),
        occ_kill=grab(v.occ_kill, (v.n_occ,), np.uint8),
        seg_off=grab(v.seg_off, (v.n_vreg + 1,), np.uint32),
        seg=grab(v.seg, (v.n_seg, 2), np.uint32),
        hull=grab(v.hull, (v.n_vreg, 2), np.uint32),
    )
    out["live_after"] = grab(v.live_after, (v.n_instr, W), np.uint32) if v.live_after else None
    return out
