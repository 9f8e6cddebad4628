"""Throughput of the hot path on one MI355X.

One step = liveness analysis of every kernel of the workload plus verification
of every candidate row, inputs resident in device memory.  Prints one JSON
line: candidates verified per second over the timed steps, the spread of the
per-step times (HIP events around every step and around its two stages), the
roofline figures of the candidate walk kernel (HIP events around that kernel
inside the timed region) and of the liveness stage, the comparison of every
GPU verdict with the CPU oracle's, and the oracle's own rate on the host cores.
Exits non-zero when a verdict differs.
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
PROFILE = os.path.join("profiles", "k_walk_config5_traffic.json")


def from_profile(kernel_source: str, key: str):
    """A per-launch figure of the walk kernel from the committed counter runs (HBM bytes,
    vector instructions), or None when there is none for the kernel as it is now."""
    path = os.path.join(ROOT, PROFILE)
    if not os.path.exists(path):
        return None
    with open(path) as f:
        rec = json.load(f)
    with open(kernel_source, "rb") as f:
        sha = hashlib.sha256(f.read()).hexdigest()
    if rec.get("source_sha256") != sha:
        return None
    return rec.get(key)


def oracle_pass(kernels, rows_list, workers):
    """The oracle, as it stands, on every kernel given: liveness, intervals, interference,
    then every candidate row; one kernel per worker thread (the C code releases the
    interpreter lock).  Returns (verdicts per kernel, seconds)."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import vlo

    def one(job):
        k, rows = job
        an = vlo.analyze(k.mir, threads=1)
        return vlo.verify(k.mir, an, rows, threads=1)
    t0 = time.perf_counter()
    if workers <= 1:
        res = [one(j) for j in zip(kernels, rows_list)]
    else:
        with ThreadPoolExecutor(workers) as pool:
            res = list(pool.map(one, zip(kernels, rows_list)))
    return res, time.perf_counter() - t0


def spread(ms):
    import numpy as np
    a = np.asarray(ms, dtype=np.float64)
    return {"median": float(np.median(a)), "min": float(a.min()), "max": float(a.max()), "mean": float(a.mean())}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--kernels", type=int, default=256, help="kernels in the sweep (256 = the benchmark)")
    ap.add_argument("--tile", type=int, default=0, help="instructions per verification tile (0 = default)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg (no parity check, no baseline)")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the timed steps: none of the legs reported beside the headline (other streams, graph "
                         "replay, reductions, masks, all-violations mode, occurrence-major layout, streaming probe)")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step as replays of a recorded HIP graph (reported beside the eager figure)")
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
    from paper_2506_17506_amd import measure
    from vlgen import gen

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    vl.load()
    hip = vl.hip_runtime()
    hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
    host_cpus = os.cpu_count() or 1
    workers = min(host_cpus, 16)   # the share of the host a one-GPU job may use

    t0 = time.perf_counter()
    w = gen.config(5, n_kernels=args.kernels, threads=workers)
    print(f"[bench] generated {len(w.kernels)} kernels, {w.n_candidates} candidates in {time.perf_counter() - t0:.1f} s",
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
        # kernel's stream of checks and events once (it stays in cache for the other candidates)
        alg_bytes += rows.shape[0] * (2 * k.mir.n_occ + 16)
    torch.cuda.synchronize()
    print("[bench] inputs resident on the device", file=sys.stderr, flush=True)

    stream = torch.cuda.current_stream()
    sp = C.c_void_p(stream.cuda_stream)
    lives = vl.vl_liveness_multi(mirs, 0, args.tile, stream)
    live_bytes = 0
    for k, l in zip(w.kernels, lives):
        v = vl.vl_live_get(l)
        alg_bytes += 8 * v.plan_len
        # algorithmic traffic of the analysis: the occurrences read (vreg 4 B + flags 1 B), and
        # written: kill flags, the block sets in and out, interval segments and their offsets
        live_bytes += 5 * v.n_occ + v.n_occ + 8 * v.n_block * v.words + 8 * v.n_seg + 4 * v.n_vreg
    jobs = vl.make_jobs([(m, l, d, r.shape[0], ld, o)
                         for m, l, d, r, ld, o in zip(mirs, lives, dev_rows, w.rows, lds, outs)])
    torch.cuda.synchronize()

    def new_event():
        e = C.c_void_p()
        assert hip.hipEventCreate(C.byref(e)) == 0
        return e

    def elapsed(a, b):
        ms = C.c_float()
        assert hip.hipEventElapsedTime(C.byref(ms), a, b) == 0
        return ms.value

    def step(ev=None):
        if ev is not None:
            assert hip.hipEventRecord(ev[0], sp) == 0
        vl.vl_liveness_multi(mirs, 0, args.tile, stream, live=lives)
        if ev is not None:
            assert hip.hipEventRecord(ev[1], sp) == 0
            measure.vl_verify_time_next(ev[3].value, ev[4].value)
        vl.vl_verify_multi(jobs, stream)
        if ev is not None:
            assert hip.hipEventRecord(ev[2], sp) == 0

    # per step: start, between the stages, end, and the two around the walk kernel
    events = [[new_event() for _ in range(5)] for _ in range(args.steps)]
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

    step_ms = [elapsed(e[0], e[2]) for e in events]
    live_ms = [elapsed(e[0], e[1]) for e in events]
    verify_ms = [elapsed(e[1], e[2]) for e in events]
    walk_ms = [elapsed(e[3], e[4]) for e in events]
    walk_avg_s = sum(walk_ms) / len(walk_ms) / 1e3
    live_avg_s = sum(live_ms) / len(live_ms) / 1e3
    status = np.concatenate([o.cpu().numpy()[:, 0] for o in outs])
    gpu_results = [o.cpu().numpy().view(np.uint32).reshape(-1, 4).copy().view(vl.RESULT_DTYPE).reshape(-1) for o in outs]

    achieved = alg_bytes / walk_avg_s / 1e9
    src = os.path.join(ROOT, "paper_2506_17506_amd", "csrc", "vl_verify.hip")
    # the other bound: vector instructions of the launch (counted once with the profiler,
    # 64 lane-operations each) against 256 compute units x 64 lanes x 2.4 GHz
    valu = from_profile(src, "valu_insts_per_launch")
    traffic = from_profile(src, "hbm_bytes_per_launch")
    alu = None
    if valu:
        alu = {"achieved": valu * 64 / walk_avg_s / 1e12, "peak": ALU_PEAK_TOPS, "unit": "T lane-op/s",
               "frac": valu * 64 / walk_avg_s / 1e12 / ALU_PEAK_TOPS, "vector_instructions_per_launch": valu,
               "source": PROFILE + " (counter run of the same command, this kernel source)"}
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
        "step_ms": spread(step_ms), "liveness_ms": spread(live_ms), "verify_ms": spread(verify_ms),
        "walk_ms": spread(walk_ms),
        "timing": "HIP events on the library's stream around every step, its two stages and the walk kernel; "
                  "value and ms_per_step from the host clock around all steps",
        "host_enqueue_ms_per_step": dt_enqueue / args.steps * 1e3,
        "status_histogram": np.bincount(status, minlength=4).tolist(),
        "roofline": {"bound": "hbm", "kernel": "k_walk", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic,
                     "traffic_source": (PROFILE + " (two counter runs of the same command, this kernel source; not "
                                        "measured in this run)") if traffic else None,
                     "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_ms": walk_avg_s * 1e3,
                     "alu": alu},
        "roofline_liveness": {"bound": "hbm", "kernels": "the analysis stage (all its launches)",
                              "achieved": live_bytes / live_avg_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": live_bytes / live_avg_s / 1e9 / HBM_PEAK_GBS,
                              "algorithmic_bytes_per_step": live_bytes, "avg_stage_ms": live_avg_s * 1e3},
    }

    if not args.no_extras:
        rec.update(extras(args, vl, measure, hip, torch, np, w, mirs, lives, jobs, dev_rows, lds, outs, stream,
                          achieved))

    rc = 0
    if not args.no_cpu:
        # every verdict against the oracle's, and the oracle's rate on this pass
        want, secs = oracle_pass(w.kernels, w.rows, workers)
        bad = [(j, int(np.nonzero(a != b)[0][0])) for j, (a, b) in enumerate(zip(want, gpu_results)) if (a != b).any()]
        mismatches = int(sum(int((a != b).sum()) for a, b in zip(want, gpu_results)))
        rec["parity"] = {"rows": int(sum(len(a) for a in want)), "mismatches": mismatches,
                         "compared": "status, where, a, b of every candidate of every kernel, GPU against oracle"}
        if bad:
            j, r = bad[0]
            rec["parity"]["first"] = {"kernel": j, "row": r, "oracle": [int(x) for x in want[j][r]],
                                      "gpu": [int(x) for x in gpu_results[j][r]]}
            rc = 1
        n_single = min(8, len(w.kernels))
        _, secs1 = oracle_pass(w.kernels[:n_single], w.rows[:n_single], 1)
        rows1 = sum(r.shape[0] for r in w.rows[:n_single])
        rec["cpu_baseline"] = {
            "value": w.n_candidates / secs, "unit": "candidates/s", "cores": workers, "kind": "oracle",
            "host_cpu_count": host_cpus,
            "single_thread_value": rows1 / secs1,
            "sample": f"one pass over the {len(w.kernels)} kernels of the workload, every candidate row, liveness "
                      f"included ({w.n_candidates} candidates in {secs:.2f} s on {workers} threads, one kernel per "
                      f"thread); single thread: the first {n_single} kernels ({rows1} candidates in {secs1:.2f} s)"}
    print(json.dumps(rec), flush=True)
    sys.exit(rc)


def extras(args, vl, measure, hip, torch, np, w, mirs, lives, jobs, dev_rows, lds, outs, stream, achieved):
    """Figures reported beside the headline, all outside the timed region."""
    out = {}
    n = len(mirs)

    # the same steps alternating over two streams, each with analysis handles and results of
    # its own: the analysis of one step then overlaps the candidate walk of the step before it
    st2 = torch.cuda.Stream()
    lives2 = vl.vl_liveness_multi(mirs, 0, args.tile, st2)
    outs2 = [torch.zeros_like(o) for o in outs]
    jobs2 = vl.make_jobs([(m, l, d, r.shape[0], ld, o)
                          for m, l, d, r, ld, o in zip(mirs, lives2, dev_rows, w.rows, lds, outs2)])
    lanes = [(stream, lives, jobs), (st2, lives2, jobs2)]

    def step2(i):
        st, lv, jb = lanes[i % 2]
        vl.vl_liveness_multi(mirs, 0, args.tile, st, live=lv)
        vl.vl_verify_multi(jb, st)
    for i in range(4):
        step2(i)
    torch.cuda.synchronize()
    reps = min(args.steps, 40)
    t1 = time.perf_counter()
    for i in range(reps):
        step2(i)
    torch.cuda.synchronize()
    two_ms = (time.perf_counter() - t1) / reps * 1e3
    assert all(bool((a == b).all()) for a, b in zip(outs2, outs)), "results differ between streams"
    out["two_stream_ms_per_step"] = two_ms
    out["two_stream_value"] = w.n_candidates / two_ms * 1e3

    # the same step recorded once into a HIP graph and replayed
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
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        out["graph_replay_ms_per_step"] = (time.perf_counter() - t1) / reps * 1e3

    # the regeneration-loop reductions over the results
    summaries = torch.zeros((n, 6), dtype=torch.int32, device="cuda")
    loop_dev = torch.zeros((6,), dtype=torch.int64, device="cuda")
    vl.vl_summarize_multi(jobs, summaries, loop_dev, stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(5):
        vl.vl_summarize_multi(jobs, summaries, loop_dev, stream)
    torch.cuda.synchronize()
    loop = loop_dev.cpu().numpy().view(np.uint8).view(vl.LOOP_DTYPE)[0]
    out["regeneration_loop"] = {"kernels_passed": int(loop["n_passed"]), "avg_tries": float(loop["sum_tries"]) / n,
                                "max_tries": int(loop["max_tries"]),
                                "summarize_us": (time.perf_counter() - t1) / 5 * 1e6}

    # constrained-decoding masks: one query per candidate, at the first mention of a vreg
    # halfway through its kernel
    queries = []
    for k, m, l, d in zip(w.kernels, mirs, lives, dev_rows):
        _, firsts = np.unique(k.mir.occ_vreg, return_index=True)
        q = int(firsts[np.argmin(np.abs(firsts.astype(np.int64) - k.mir.n_occ // 2))])
        queries += [(m, l, d[r], q) for r in range(d.shape[0])]
    queries = vl.make_mask_queries(queries)
    masks = torch.zeros((len(queries), 16), dtype=torch.int32, device="cuda")
    vl.vl_free_bases_multi(queries, masks, stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(5):
        vl.vl_free_bases_multi(queries, masks, stream)
    torch.cuda.synchronize()
    mask_us = (time.perf_counter() - t1) / 5 * 1e6
    out["decoding_mask"] = {"queries": len(queries), "us_per_call": mask_us, "masks_per_s": len(queries) / mask_us * 1e6}

    # all-violations mode over the same candidates; the first call also enumerates every
    # kernel's interfering pairs
    count_outs = [torch.zeros((r.shape[0], 8), dtype=torch.int32, device="cuda") for r in w.rows]
    count_jobs = [(m, l, d, r.shape[0], ld, o) for m, l, d, r, ld, o in zip(mirs, lives, dev_rows, w.rows, lds, count_outs)]
    t1 = time.perf_counter()
    vl.vl_count_violations_multi(count_jobs, stream)
    torch.cuda.synchronize()
    first_ms = (time.perf_counter() - t1) * 1e3
    t1 = time.perf_counter()
    for _ in range(3):
        vl.vl_count_violations_multi(count_jobs, stream)
    torch.cuda.synchronize()
    count_ms = (time.perf_counter() - t1) / 3 * 1e3
    kinds = np.concatenate([o.cpu().numpy()[:, 0] for o in count_outs])
    out["all_violations"] = {"ms_per_pass": count_ms, "first_pass_ms": first_ms,
                             "candidates_per_s": w.n_candidates / count_ms * 1e3,
                             "kinds_histogram": np.bincount(kinds, minlength=8).tolist()}

    # register-bank conflict score of every candidate (four banks, as in the paper's example):
    # one call per kernel
    score_outs = [torch.zeros(r.shape[0], dtype=torch.int32, device="cuda") for r in w.rows]
    def score_pass():
        for m, d, r, ld, o in zip(mirs, dev_rows, w.rows, lds, score_outs):
            vl.vl_bank_conflicts(m, d, r.shape[0], ld, 4, o, stream)
    score_pass()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(3):
        score_pass()
    torch.cuda.synchronize()
    score_ms = (time.perf_counter() - t1) / 3 * 1e3
    stalls = np.concatenate([o.cpu().numpy() for o in score_outs]).astype(np.int64)
    out["bank_score"] = {"ms_per_pass": score_ms, "candidates_per_s": w.n_candidates / score_ms * 1e3,
                         "banks": 4, "mean_stall_cycles_per_instruction": float(stalls.sum()) / w.n_checks}

    # the same candidates stored occurrence-major (how a batched decoder leaves them):
    # verification only, results compared with the row-major ones
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
        measure.vl_verify_time_next(ev_a.value, ev_b.value)
        vl.vl_verify_multi_occ_major(t_jobs, stream)
    torch.cuda.synchronize()
    occ_ms = (time.perf_counter() - t1) / 5 * 1e3
    ms = C.c_float()
    assert hip.hipEventElapsedTime(C.byref(ms), ev_a, ev_b) == 0
    out["occurrence_major"] = {"verify_ms": occ_ms, "walk_ms": ms.value}
    del t_keep, t_jobs

    # what a plain streaming read reaches on this device (context for the roofline figure):
    # the read-only probe over 1 GiB, best of six
    probe = torch.ones(1 << 28, dtype=torch.int32, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    best = 0.0
    for _ in range(6):
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        assert measure.vl_stream_read_probe(probe, probe.numel() * 4, sink, stream) == 0
        torch.cuda.synchronize()
        best = max(best, probe.numel() * 4 / (time.perf_counter() - t1) / 1e9)
    del probe
    out["measured_stream_read_gbs"] = best
    out["walk_frac_of_measured_stream_read"] = achieved / best
    return out


if __name__ == "__main__":
    main()
