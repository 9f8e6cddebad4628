"""Compile the HIP sources into paper_2506_17506_amd/libvl.so for gfx950."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
SOURCES = ["vl_mir.hip", "vl_liveness.hip", "vl_verify.hip", "vl_mask.hip", "vl_count.hip", "vl_score.hip"]
BENCH_SOURCES = ["vl_probe.hip"]   # measurement hooks of the benchmark (include/vl_bench.h), a library of their own
LIB = os.path.join(HERE, "libvl.so")
BENCH_LIB = os.path.join(HERE, "libvlbench.so")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def stale() -> bool:
    if not os.path.exists(LIB) or not os.path.exists(BENCH_LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    deps.append(os.path.join(os.path.dirname(HERE), "include", "vl.h"))
    deps.append(os.path.join(os.path.dirname(HERE), "include", "vl_bench.h"))
    return any(os.path.getmtime(p) > t for p in deps)


def build(force: bool = True) -> str:
    if force or stale():
        cmd = ["hipcc"] + FLAGS + ["-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
        subprocess.run(cmd, check=True)
        cmd = ["hipcc"] + FLAGS + ["-o", BENCH_LIB] + [os.path.join(CSRC, s) for s in BENCH_SOURCES]
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
