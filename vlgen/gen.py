"""Seeded synthetic workloads: kernels, candidate rows and the damage log.

Thin ctypes wrapper over vlgen/gen.cpp plus the recipes of the five benchmark
configurations.  Input generation only; no analysis or checking happens here.
"""
from __future__ import annotations

import ctypes as C
import math
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

from .mir import Mir

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "gen.cpp")
LIB = os.path.join(HERE, "libvlgen.so")

MUT_DTYPE = np.dtype([("kind", "<u4"), ("vreg", "<u4"), ("other", "<u4"), ("expect", "<u4")])
STRAIGHT, LOOP3, GEMM, MHA = 1, 2, 3, 4
SEED0 = 0x5EED0000


def build(force: bool = False) -> str:
    if force or not os.path.exists(LIB) or os.path.getmtime(SRC) > os.path.getmtime(LIB):
        subprocess.run(["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-o", LIB, SRC], check=True)
    return LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.vlgen_make.restype = C.c_void_p
        _lib.vlgen_make.argtypes = [C.c_int, C.c_uint64, C.c_uint32, C.c_uint32]
        _lib.vlgen_free.argtypes = [C.c_void_p]
        _lib.vlgen_sizes.argtypes = [C.c_void_p, C.c_void_p]
        _lib.vlgen_copy.argtypes = [C.c_void_p] * 13
        _lib.vlgen_candidates.restype = C.c_int
        _lib.vlgen_candidates.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32, C.c_uint32, C.c_int,
                                          C.c_void_p, C.c_uint64, C.c_void_p]
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


class Kernel:
    """One synthetic kernel: the program (self.mir) and what the generator knows
    about it by construction (self.range: conservative occupancy range per vreg,
    self.sure: range where occupancy is certain, possibly empty)."""

    def __init__(self, kind: int, seed: int, n_instr: int, n_vreg: int = 0, name: str = ""):
        L = lib()
        self.kind, self.seed = kind, seed
        self._h = L.vlgen_make(kind, seed, n_instr, n_vreg)
        if not self._h:
            raise ValueError("unknown kernel kind")
        sz = np.zeros(8, np.uint32)
        L.vlgen_sizes(self._h, _p(sz))
        N, V, B, O, Cn, E = (int(x) for x in sz[:6])
        a = dict(blk_start=np.zeros(B + 1, np.uint32), succ_off=np.zeros(B + 1, np.uint32),
                 succ=np.zeros(max(E, 1), np.uint32), occ_off=np.zeros(N + 1, np.uint32),
                 occ_vreg=np.zeros(max(O, 1), np.uint32), occ_flags=np.zeros(max(O, 1), np.uint8),
                 vclass=np.zeros(V, np.uint8), vwidth=np.zeros(V, np.uint8), valign=np.zeros(V, np.uint8),
                 class_size=np.zeros(Cn, np.uint16), range=np.zeros((V, 2), np.uint32),
                 sure=np.zeros((V, 2), np.uint32))
        L.vlgen_copy(self._h, *[_p(a[k]) for k in ("blk_start", "succ_off", "succ", "occ_off", "occ_vreg",
                                                    "occ_flags", "vclass", "vwidth", "valign", "class_size",
                                                    "range", "sure")])
        self.mir = Mir(a["blk_start"], a["succ_off"], a["succ"][:E], a["occ_off"], a["occ_vreg"][:O],
                       a["occ_flags"][:O], a["vclass"], a["vwidth"], a["valign"], a["class_size"],
                       None, name or f"k{kind}_{seed:x}")
        self.range, self.sure = a["range"], a["sure"]

    def __del__(self):
        # at interpreter shutdown the module's globals may already be gone: then the
        # process is ending and the handle goes with it
        if getattr(self, "_h", None) and lib is not None:
            lib().vlgen_free(self._h)
            self._h = None

    def candidates(self, seed: int, K: int, n_mut: int, mode: int, out: np.ndarray | None = None):
        """K rows [K, n_occ] uint16 and the damage log [K].  mode 0: plain first
        fit, undamaged; 1: plain first fit, damage = random reassignments and
        single-occurrence remaps; 2: randomized first fit, damage in the paper's
        error proportions; 3: randomized first fit, 1-3 injected conflicts."""
        O = self.mir.n_occ
        rows = np.zeros((K, O), np.uint16) if out is None else out
        assert rows.dtype == np.uint16 and rows.shape == (K, O) and rows.strides[1] == 2
        log = np.zeros(K, MUT_DTYPE)
        rc = lib().vlgen_candidates(self._h, seed, K, n_mut, mode, _p(rows), rows.strides[0] // 2, _p(log))
        if rc != 0:
            raise RuntimeError(f"no allocation found for {self.mir.name} (seed {seed:#x})")
        return rows, log


@dataclass
class Workload:
    name: str
    kernels: list          # [Kernel]
    rows: list             # [np.ndarray uint16 [K, O]] per kernel
    logs: list             # [np.ndarray MUT_DTYPE [K]] per kernel

    @property
    def n_candidates(self) -> int:
        return sum(r.shape[0] for r in self.rows)

    @property
    def n_checks(self) -> int:
        """instruction x candidate checks"""
        return sum(k.mir.n_instr * r.shape[0] for k, r in zip(self.kernels, self.rows))


def _kernel_seed(config: int, index: int) -> int:
    return SEED0 + 0x100 * config + index


def _with_retry(kind, config, index, N, V, K, n_mut, mode, name):
    """A kernel whose allocator fails takes the next seed (recorded in meta)."""
    base = _kernel_seed(config, index)
    for bump in range(16):
        seed = base + (bump << 20)
        k = Kernel(kind, seed, N, V, name)
        try:
            rows, log = k.candidates(seed ^ 0xC0FFEE, K, n_mut, mode)
        except RuntimeError:
            continue
        k.mir.meta["seed"] = seed
        k.mir.meta["seed_bumps"] = bump
        return k, rows, log
    raise RuntimeError(f"config {config} kernel {index}: no seed gives an allocation")


def sweep_sizes(n_kernels: int, lo: int = 1000, hi: int = 20000, seed: int = SEED0 + 0x500):
    """Instruction counts log-uniform in [lo, hi] from a SplitMix64 stream."""
    out, s = [], seed & 0xFFFFFFFFFFFFFFFF
    for _ in range(n_kernels):
        s = (s + 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF
        z = s
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
        z ^= z >> 31
        u = (z >> 11) / float(1 << 53)
        out.append(int(math.floor(math.exp(math.log(lo) + u * (math.log(hi) - math.log(lo))))))
    return out


def config(n: int, scale: float = 1.0, threads: int = 8, n_kernels: int | None = None) -> Workload:
    """The five benchmark configurations.  scale < 1 shrinks instruction counts
    and (for 4 and 5) the number of kernels, for quick tests."""
    if n == 1:
        k, rows, log = _with_retry(STRAIGHT, 1, 0, 200, 200, 64, 32, 1, "straight200")
        return Workload("config1", [k], [rows], [log])
    if n == 2:
        N = max(200, int(2000 * scale))
        k, rows, log = _with_retry(LOOP3, 2, 0, N, N * 3 // 4, 100, 50, 2, "loop3")
        return Workload("config2", [k], [rows], [log])
    if n == 3:
        N = max(1000, int(8000 * scale))
        K = max(64, int(1000 * scale))
        k, rows, log = _with_retry(GEMM, 3, 0, N, N * 3 // 4, K, K * 3 // 10, 3, "gemm")
        return Workload("config3", [k], [rows], [log])
    if n == 4:
        N = max(1000, int(20000 * scale))
        nk = n_kernels if n_kernels is not None else max(2, int(64 * scale))
        jobs = [(MHA, 4, i, N, N * 3 // 4, 100, 20, 2, f"mha{i}") for i in range(nk)]
        name = "config4"
    elif n == 5:
        nk = n_kernels if n_kernels is not None else max(4, int(256 * scale))
        sizes = sweep_sizes(nk)
        jobs = [((GEMM if i % 2 == 0 else MHA), 5, i, sizes[i], sizes[i] * 3 // 4, 100, 20, 2,
                 f"{'gemm' if i % 2 == 0 else 'mha'}{i}_{sizes[i]}") for i in range(nk)]
        name = "config5"
    else:
        raise ValueError("config 1..5")
    with ThreadPoolExecutor(max_workers=threads) as ex:
        res = list(ex.map(lambda j: _with_retry(*j), jobs))
    return Workload(name, [r[0] for r in res], [r[1] for r in res], [r[2] for r in res])
