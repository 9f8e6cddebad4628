"""Throughput of the hot path on one MI355X.

One step = liveness analysis of every kernel of the workload plus verification
of every candidate row, inputs resident in device memory.  Prints one JSON
line: candidates verified per second, the roofline figures of the candidate
walk kernel (measured with HIP events around that kernel inside the timed
region) and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import ctypes as C
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published
ALU_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12  # plain (unpacked, non-FMA) vector operations: 39.3 T lane-operations/s


def from_profile(kernel_source: str, key: str):
    """A per-launch figure of the walk kernel from the committed counter runs (HBM bytes,
    vector instructions), or None when there is none for the kernel as it is now."""
    path = os.path.join(ROOT, "profiles", "k_walk_config5_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        rec = json.load(f)
    with open(kernel_source, "rb") as f:
        sha = hashlib.sha256(f.read()).hexdigest()
    if rec.get("source_sha256") != sha:
        return None
    return rec.get(key)


def cpu_baseline(workload, min_seconds=10.0, max_seconds=30.0):
    """The oracle, as it stands, on whole passes over the same workload: per kernel
    liveness, intervals and interference, then every candidate row; all host
    cores.  Passes are repeated until min_seconds have gone by; a pass is cut
    short after the kernel that crosses max_seconds."""
    from oracle import vlo
    cores = min(os.cpu_count() or 1, 16)
    n_rows, n_checks, n_kernels, t0 = 0, 0, 0, time.perf_counter()
    while time.perf_counter() - t0 < min_seconds:
        for k, rows in zip(workload.kernels, workload.rows):
            an = vlo.analyze(k.mir, threads=cores)
            vlo.verify(k.mir, an, rows, threads=cores)
            n_rows += rows.shape[0]
            n_checks += rows.shape[0] * k.mir.n_instr
            n_kernels += 1
            if time.perf_counter() - t0 > max_seconds:
                break
    dt = time.perf_counter() - t0
    return {"value": n_rows / dt, "unit": "candidates/s", "cores": cores, "kind": "oracle",
            "sample": f"{n_kernels / len(workload.kernels):.2f} passes over the {len(workload.kernels)} kernels of the "
                      f"workload, every candidate row, liveness included ({n_rows} candidates, {n_checks} "
                      f"instruction x candidate checks in {dt:.2f} s)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--kernels", type=int, default=256, help="kernels in the sweep (256 = the benchmark)")
    ap.add_argument("--tile", type=int, default=0, help="instructions per verification tile (0 = default)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step as replays of a recorded HIP graph (reported beside the eager figure)")
    ap.add_argument("--no-two-stream", action="store_true",
                    help="skip the extra leg that alternates the steps over two streams (it lengthens the "
                         "candidate walk's launches, which a kernel trace of the run would average in)")
    ap.add_argument("--streams", type=int, default=1,
                    help="steps alternate over this many streams, each with its own analysis handles and result "
                         "buffers (steps on different streams may overlap on the device)")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MIB",
                    help="before the warm-up, run one plain elementwise kernel that reads MIB MiB and writes "
                         "MIB MiB: a dispatch of known traffic to scale hardware byte counters by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2506_17506_amd as vl
    from vlgen import gen

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    vl.load()
    hip = vl.hip_runtime()

    t0 = time.perf_counter()
    w = gen.config(5, n_kernels=args.kernels, threads=min(os.cpu_count() or 1, 16))
    t_gen = time.perf_counter() - t0
    print(f"[bench] generated {len(w.kernels)} kernels, {w.n_candidates} candidates in {t_gen:.1f} s",
          file=sys.stderr, flush=True)

    mirs = [vl.vl_mir_create(k.mir) for k in w.kernels]
    dev_rows, outs, lds = [], [], []
    alg_bytes = 0
    for k, rows in zip(w.kernels, w.rows):
        d, ld = vl.rows_to_device(rows)
        dev_rows.append(d)
        lds.append(ld)
        outs.append(torch.zeros((rows.shape[0], 4), dtype=torch.int32, device="cuda"))
        # algorithmic traffic of the walk: each candidate row once, its result once, and the
        # kernel's event stream once (it stays in cache for the other candidates)
        alg_bytes += rows.shape[0] * (2 * k.mir.n_occ + 16)
    torch.cuda.synchronize()
    print("[bench] inputs resident on the device", file=sys.stderr, flush=True)

    stream = torch.cuda.current_stream()
    lives = vl.vl_liveness_multi(mirs, 0, args.tile, stream)
    for k, l in zip(w.kernels, lives):
        alg_bytes += 8 * vl.vl_live_get(l).plan_len
    jobs = vl.make_jobs([(m, l, d, r.shape[0], ld, o)
                         for m, l, d, r, ld, o in zip(mirs, lives, dev_rows, w.rows, lds, outs)])
    # further streams: the same kernels and candidates, analysis handles and results of their own
    lanes = [(stream, lives, jobs)]
    keep = []
    for _ in range(1, max(2, args.streams)):
        st = torch.cuda.Stream()
        lv = vl.vl_liveness_multi(mirs, 0, args.tile, st)
        oo = [torch.zeros_like(o) for o in outs]
        keep.append(oo)
        lanes.append((st, lv, vl.make_jobs([(m, l, d, r.shape[0], ld, o)
                                            for m, l, d, r, ld, o in zip(mirs, lv, dev_rows, w.rows, lds, oo)])))
    torch.cuda.synchronize()
    turn, n_lanes = 0, args.streams

    def step(ev=None):
        nonlocal turn
        st, lv, jb = lanes[turn % n_lanes]
        turn += 1
        vl.vl_liveness_multi(mirs, 0, args.tile, st, live=lv)
        if ev is not None:
            vl.vl_verify_time_next(ev[0].value, ev[1].value)
        vl.vl_verify_multi(jb, st)

    events = []
    for _ in range(args.steps):
        a, b = C.c_void_p(), C.c_void_p()
        assert hip.hipEventCreate(C.byref(a)) == 0 and hip.hipEventCreate(C.byref(b)) == 0
        events.append((a, b))
    if args.copy_probe:
        src_probe = torch.zeros(args.copy_probe * (1 << 18), dtype=torch.int32, device="cuda")
        dst_probe = torch.empty_like(src_probe)
        torch.cuda.synchronize()
        torch.add(src_probe, 1, out=dst_probe)   # the probe: one launch, 4 bytes in and 4 bytes out per element
        torch.cuda.synchronize()
        del src_probe, dst_probe
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    dt_enqueue = time.perf_counter() - t0   # host time to enqueue the steps (they run asynchronously)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    walk_ms = []
    for a, b in events:
        ms = C.c_float()
        assert hip.hipEventElapsedTime(C.byref(ms), a, b) == 0
        walk_ms.append(ms.value)
    walk_avg_s = sum(walk_ms) / len(walk_ms) / 1e3

    # separate timings of the two stages (outside the timed region, for the record)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(5):
        lives = vl.vl_liveness_multi(mirs, 0, args.tile, stream, live=lives)
    torch.cuda.synchronize()
    live_ms = (time.perf_counter() - t1) / 5 * 1e3
    t1 = time.perf_counter()
    for _ in range(5):
        vl.vl_verify_multi(jobs, stream)
    torch.cuda.synchronize()
    verify_ms = (time.perf_counter() - t1) / 5 * 1e3

    # the same steps alternating over two streams (for the record): the analysis of one step
    # then overlaps the candidate walk of the step before it
    two_stream_ms = None
    if not args.no_two_stream:
        n_lanes = 2
        for _ in range(max(2, args.warmup)):
            step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        two_stream_ms = (time.perf_counter() - t1) / args.steps * 1e3

    # the same step recorded once into a HIP graph and replayed (for the record)
    graph_ms = None
    if args.graph:
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            for _ in range(2):   # known sizes and current tables on this stream's first calls too
                vl.vl_liveness_multi(mirs, 0, args.tile, side, live=lives)
                vl.vl_verify_multi(jobs, side)
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                cap = torch.cuda.current_stream()
                vl.vl_liveness_multi(mirs, 0, args.tile, cap, live=lives)
                vl.vl_verify_multi(jobs, cap)
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t1) / args.steps * 1e3

    # the regeneration-loop reductions over the results (not part of the timed step)
    summaries = torch.zeros((len(mirs), 6), dtype=torch.int32, device="cuda")
    loop_dev = torch.zeros((6,), dtype=torch.int64, device="cuda")
    vl.vl_summarize_multi(jobs, summaries, loop_dev, stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(5):
        vl.vl_summarize_multi(jobs, summaries, loop_dev, stream)
    torch.cuda.synchronize()
    summarize_us = (time.perf_counter() - t1) / 5 * 1e6
    loop = loop_dev.cpu().numpy().view(np.uint8).view(vl.LOOP_DTYPE)[0]

    # constrained-decoding masks (not part of the timed step): one query per candidate, at the
    # first mention of a vreg halfway through its kernel
    mask_queries = []
    for k, m, l, d in zip(w.kernels, mirs, lives, dev_rows):
        _, firsts = np.unique(k.mir.occ_vreg, return_index=True)
        q = int(firsts[np.argmin(np.abs(firsts.astype(np.int64) - k.mir.n_occ // 2))])
        mask_queries += [(m, l, d[r], q) for r in range(d.shape[0])]
    mask_queries = vl.make_mask_queries(mask_queries)
    masks = torch.zeros((len(mask_queries), 16), dtype=torch.int32, device="cuda")
    vl.vl_free_bases_multi(mask_queries, masks, stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(5):
        vl.vl_free_bases_multi(mask_queries, masks, stream)
    torch.cuda.synchronize()
    mask_us = (time.perf_counter() - t1) / 5 * 1e6

    # all-violations mode over the same candidates (not part of the timed step); the first
    # call also enumerates every kernel's interfering pairs
    count_outs = [torch.zeros((r.shape[0], 8), dtype=torch.int32, device="cuda") for r in w.rows]
    count_jobs = [(m, l, d, r.shape[0], ld, o) for m, l, d, r, ld, o in zip(mirs, lives, dev_rows, w.rows, lds, count_outs)]
    t1 = time.perf_counter()
    vl.vl_count_violations_multi(count_jobs, stream)
    torch.cuda.synchronize()
    count_first_ms = (time.perf_counter() - t1) * 1e3
    t1 = time.perf_counter()
    for _ in range(3):
        vl.vl_count_violations_multi(count_jobs, stream)
    torch.cuda.synchronize()
    count_ms = (time.perf_counter() - t1) / 3 * 1e3
    kinds = np.concatenate([o.cpu().numpy()[:, 0] for o in count_outs])

    # the same candidates stored occurrence-major (how a batched decoder leaves them), not part
    # of the timed step: verification only, results compared with the row-major ones
    t_jobs, t_keep, t_outs = [], [], []
    for m, l, d, r in zip(mirs, lives, dev_rows, w.rows):
        K, O = r.shape
        ld_t = (K + 7) // 8 * 8
        t = torch.zeros((max(O, 1), ld_t), dtype=torch.int16, device="cuda")
        t[:O, :K] = d[:, :O].t()
        o = torch.zeros((K, 4), dtype=torch.int32, device="cuda")
        t_keep.append(t)
        t_outs.append(o)
        t_jobs.append((m, l, t, K, ld_t, o))
    t_jobs = vl.make_jobs(t_jobs)
    vl.vl_verify_multi(jobs, stream)                 # fresh row-major results to compare with
    vl.vl_verify_multi_occ_major(t_jobs, stream)
    torch.cuda.synchronize()
    assert all(bool((a == b).all()) for a, b in zip(t_outs, outs)), "occurrence-major results differ"
    ev_a, ev_b = C.c_void_p(), C.c_void_p()
    assert hip.hipEventCreate(C.byref(ev_a)) == 0 and hip.hipEventCreate(C.byref(ev_b)) == 0
    t1 = time.perf_counter()
    for _ in range(5):
        vl.vl_verify_time_next(ev_a.value, ev_b.value)
        vl.vl_verify_multi_occ_major(t_jobs, stream)
    torch.cuda.synchronize()
    occ_major_ms = (time.perf_counter() - t1) / 5 * 1e3
    ms = C.c_float()
    assert hip.hipEventElapsedTime(C.byref(ms), ev_a, ev_b) == 0
    occ_major_walk_ms = ms.value
    del t_keep, t_jobs

    # what a plain streaming read reaches on this device (context for the roofline figure):
    # the library's read-only probe over 1 GiB, best of five
    probe = torch.ones(1 << 28, dtype=torch.int32, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    stream_read = 0.0
    for _ in range(6):
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        vl.vl_stream_read_probe(probe, probe.numel() * 4, sink, stream)
        torch.cuda.synchronize()
        stream_read = max(stream_read, probe.numel() * 4 / (time.perf_counter() - t1) / 1e9)
    del probe

    status = np.concatenate([o.cpu().numpy()[:, 0] for o in outs])
    for oo in keep[:max(args.streams, 1 if args.no_two_stream else 2) - 1]:   # every stream used gave the first stream's results
        assert all(bool((a == b).all()) for a, b in zip(oo, outs)), "results differ between streams"
    achieved = alg_bytes / walk_avg_s / 1e9
    src = os.path.join(ROOT, "paper_2506_17506_amd", "csrc", "vl_verify.hip")
    # the other bound: vector instructions of the launch (counted once with the profiler,
    # 64 lane-operations each) against 256 compute units x 64 lanes x 2.4 GHz
    valu = from_profile(src, "valu_insts_per_launch")
    alu = None
    if valu:
        alu = {"achieved": valu * 64 / walk_avg_s / 1e12, "peak": ALU_PEAK_TOPS, "unit": "T lane-op/s",
               "frac": valu * 64 / walk_avg_s / 1e12 / ALU_PEAK_TOPS, "vector_instructions_per_launch": valu}
    rec = {
        "metric": "candidate allocations verified/sec at K=100",
        "value": w.n_candidates * args.steps / dt,
        "unit": "candidates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u16", "data": "synthetic",
        "config": {"workload": f"config5: {len(w.kernels)} synthetic GEMM/attention-shaped kernels, "
                               "1,000-20,000 instructions log-uniform, K=100 candidates each, 20% damaged; "
                               "liveness of every kernel + verification of every candidate per step",
                   "kernels": len(w.kernels), "candidates": w.n_candidates,
                   "instr_x_candidate_checks": w.n_checks, "tile_len": int(vl.vl_live_get(lives[0]).tile_len)},
        "checks_per_s": w.n_checks * args.steps / dt,
        "liveness_ms": live_ms, "verify_ms": verify_ms, "host_enqueue_ms_per_step": dt_enqueue / args.steps * 1e3,
        "graph_replay_ms_per_step": graph_ms, "streams": args.streams,
        "two_stream_ms_per_step": two_stream_ms, "two_stream_value": w.n_candidates / two_stream_ms * 1e3 if two_stream_ms else None,
        "status_histogram": np.bincount(status, minlength=4).tolist(),
        "regeneration_loop": {"kernels_passed": int(loop["n_passed"]), "avg_tries": float(loop["sum_tries"]) / len(mirs),
                              "max_tries": int(loop["max_tries"]), "summarize_us": summarize_us},
        "all_violations": {"ms_per_pass": count_ms, "first_pass_ms": count_first_ms,
                           "candidates_per_s": w.n_candidates / count_ms * 1e3,
                           "kinds_histogram": np.bincount(kinds, minlength=8).tolist()},
        "occurrence_major": {"verify_ms": occ_major_ms, "walk_ms": occ_major_walk_ms},
        "decoding_mask": {"queries": len(mask_queries), "us_per_call": mask_us,
                          "masks_per_s": len(mask_queries) / mask_us * 1e6},
        "roofline": {"bound": "hbm", "kernel": "k_walk", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": from_profile(src, "hbm_bytes_per_launch"),
                     "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_ms": walk_avg_s * 1e3,
                     "measured_stream_read": stream_read, "frac_of_measured_stream_read": achieved / stream_read,
                     "alu": alu},
    }
    if not args.no_cpu:
        rec["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
