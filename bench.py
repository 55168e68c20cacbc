#!/usr/bin/env python3
"""Benchmark of the PAG search hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--cfg 2] [--n N] [--nq NQ] [--efc EFC]

A "step" is one pag_search call over the whole query batch of the workload (query rotation,
projection tables and the fused best-first search), queries and results resident in HBM.
The workload is configuration 2 of the synthetic set (n = 1,000,000, d = 768, inner product on
unit vectors, degree 32, 32 subspaces, K = 10): the index is built on the GPU by pag_build, the
efS grid is swept against brute-force ground truth, and the timed steps run at the smallest efS
whose recall@10 reaches 0.95.  One JSON line is printed:
  value        whole-batch queries per second over the timed steps
  roofline     algorithmic HBM bytes of the search kernel / its HIP-event duration, against 8 TB/s
  cpu_baseline the CPU oracle searching the same exported index with the same efS on a bounded
               sample of the queries, on the host cores of this machine
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
TARGET_RECALL = 0.95


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(c, d, K, vec_bytes=4):
    """Bytes the method itself must move (Sec. 4.2's terms): per query the query vector and the
    results, per expanded node its adjacency record, per exact distance one base vector."""
    return (c["queries"] * (4 * d + 8 * K) + c["hops"] * c["adj_record_bytes"] + c["exact"] * vec_bytes * d)


def read_traffic(tag, efS):
    """HBM bytes per search-kernel launch from the committed rocprofv3 counter summary, if it covers this run
    (same workload, same efS); otherwise None."""
    path = os.path.join(ROOT, "profiles", "search_kernel_%s_hbm_traffic.txt" % tag)
    vals = {}
    try:
        with open(path) as f:
            for line in f:
                if line.startswith(("traffic_bytes_per_launch:", "efS:")):
                    k, v = line.split(":")
                    vals[k] = float(v)
    except OSError:
        return None
    if vals.get("efS") != float(efS):
        return None
    return vals.get("traffic_bytes_per_launch")


def online_insertion(args, w, wl, torch, np, PagIndex):
    """Workload 5 (the paper's online-insertion experiment, Sec. 5.2 D6, at synthetic scale): build on the
    initial vectors, then rounds of pag_insert followed by a query batch; reports insertion throughput and
    the recall after every round against brute force over the vectors inserted so far."""
    rounds = args.rounds
    per_round = args.insert_batch
    t0 = time.time()
    base = wl.make(w, "base")
    q = wl.make(w, "query")
    log("generated %s: base %s, queries %s in %.1f s" % (w.name, base.shape, q.shape, time.time() - t0))
    cap = w.n + (rounds + 1) * per_round      # one more batch for the concurrent phase
    all_d = torch.empty((cap, w.d), dtype=torch.float32, device="cuda")
    all_d[:w.n] = torch.from_numpy(base)
    del base
    q_d = torch.from_numpy(q).cuda()
    t0 = time.time()
    ix = PagIndex.build(all_d[:w.n], metric="ip", max_degree=w.deg, num_subspaces=w.P, ef_construction=args.efc,
                        seed=2603, capacity=cap)
    build_s = time.time() - t0
    log("pag_build of the initial %d vectors: %.2f s" % (w.n, build_s))
    # efS: the smallest of a grid that reaches the recall target on the initial index, then kept
    efS = args.efs
    if not efS:
        gt0, _ = wl.brute_force_torch(all_d[:w.n], q_d, w.K, w.metric)
        for efS in (128, 256, 512, 768, 1024, 1536, 2048, 3072, 4096):
            ids, _ = ix.search(q_d, w.K, efS)
            rec0 = wl.recall_at_k(ids.cpu().numpy(), gt0)
            log("initial index: efS %4d recall@%d %.4f" % (efS, w.K, rec0))
            if rec0 >= TARGET_RECALL:
                break
    n = w.n
    rows = []
    ins_time = 0.0
    for r in range(rounds):
        x = wl.make(w, "insert%d" % r, n=per_round)
        all_d[n:n + per_round] = torch.from_numpy(x)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ix.insert(all_d[n:n + per_round])
        dt = time.perf_counter() - t1
        ins_time += dt
        n += per_round
        t1 = time.perf_counter()
        ids, _ = ix.search(q_d, w.K, efS)
        ts = time.perf_counter() - t1
        gt, _ = wl.brute_force_torch(all_d[:n], q_d, w.K, w.metric)
        rec = wl.recall_at_k(ids.cpu().numpy(), gt)
        rows.append({"round": r + 1, "n": n, "insert_vectors_per_s": round(per_round / dt, 1),
                     "search_qps": round(w.nq / ts, 1), "recall": round(rec, 4)})
        log("round %2d: n = %d, insert %.0f vectors/s, search %.0f QPS at efS %d, recall@%d %.4f" %
            (r + 1, n, per_round / dt, w.nq / ts, efS, w.K, rec))
    # ---- one more batch, inserted while a searcher answers query batches from this thread ----
    import threading
    x = wl.make(w, "insert%d" % rounds, n=per_round)
    all_d[n:n + per_round] = torch.from_numpy(x)
    srch = ix.searcher()
    srch.search(q_d, w.K, efS)
    torch.cuda.synchronize()
    timing = {}

    def grow():
        t = time.perf_counter()
        ix.insert(all_d[n:n + per_round])
        timing["insert_s"] = time.perf_counter() - t

    th = threading.Thread(target=grow)
    t1 = time.perf_counter()
    th.start()
    batches = 0
    while th.is_alive():
        ids, _ = srch.search(q_d, w.K, efS)
        batches += 1
    t_search = time.perf_counter() - t1
    th.join()
    gt, _ = wl.brute_force_torch(all_d[:n], q_d, w.K, w.metric)           # the last answer saw n or n + batch nodes
    rec_c = wl.recall_at_k(ids.cpu().numpy(), gt)
    concurrent = {"insert_vectors_per_s": round(per_round / timing["insert_s"], 1),
                  "search_qps_meanwhile": round(batches * w.nq / t_search, 1), "query_batches": batches,
                  "recall_of_last_batch_vs_index_before": round(rec_c, 4)}
    log("concurrent: insert %.0f vectors/s while a searcher answered %d batches at %.0f QPS (recall %.4f)" %
        (per_round / timing["insert_s"], batches, batches * w.nq / t_search, rec_c))
    srch.close()
    out = {"metric": "online insertion throughput (1 GPU)", "value": round(rounds * per_round / ins_time, 1),
           "unit": "vectors/s", "n_gpus": 1, "steps": rounds, "warmup": 0,
           "ms_per_step": round(1e3 * ins_time / rounds, 3), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": "cfg5 %s: start n=%d d=%d, %d rounds x (insert %d, search %d queries) K=%d deg=%d "
                                  "P=%d efC=%d efS=%d" % (w.name, w.n, w.d, rounds, per_round, w.nq, w.K, w.deg, w.P,
                                                           args.efc, efS),
                      "initial_build_seconds": round(build_s, 2), "rounds": rows,
                      "insert_and_search_at_once": concurrent},
           "roofline": None, "cpu_baseline": None}
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--cfg", type=int, default=2)
    ap.add_argument("--n", type=int, default=None)
    ap.add_argument("--nq", type=int, default=None)
    ap.add_argument("--efc", type=int, default=2000)
    ap.add_argument("--efs", type=int, default=0, help="skip the sweep and time this efS")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--fp16-vectors", action="store_true",
                    help="keep the base vectors as 16-bit floats (the paper's payload); NOT the headline configuration")
    ap.add_argument("--rounds", type=int, default=10, help="cfg 5: insertion rounds")
    ap.add_argument("--insert-batch", type=int, default=50000, help="cfg 5: vectors per insertion round")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="also launch one elementwise kernel of known size (1 GiB read, 1 GiB written) so that "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no sharding, no collectives); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import pag_workloads as wl
    from paper_2603_06660_amd import PagIndex, load_library

    load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = wl.workload(args.cfg, n=args.n, nq=args.nq)
    metric = {0: "l2", 1: "ip", 2: "cos"}[w.metric]

    if w.cfg == 5:
        return online_insertion(args, w, wl, torch, np, PagIndex)

    t0 = time.time()
    base = wl.make(w, "base")
    q = wl.make(w, "query")
    log("generated %s: base %s, queries %s in %.1f s" % (w.name, base.shape, q.shape, time.time() - t0))
    base_d = torch.from_numpy(base).cuda()
    q_d = torch.from_numpy(q).cuda()
    del base

    t0 = time.time()
    from paper_2603_06660_amd import FLAG_FP16_VECTORS
    vec_bytes = 2 if args.fp16_vectors else 4
    ix = PagIndex.build(base_d, metric=metric, max_degree=w.deg, num_subspaces=w.P, ef_construction=args.efc,
                        seed=2603, flags=FLAG_FP16_VECTORS if args.fp16_vectors else 0)
    build_s = time.time() - t0
    log("pag_build: %.2f s (%.0f vectors/s)" % (build_s, w.n / build_s))

    t0 = time.time()
    gt, _ = wl.brute_force_torch(base_d, q_d, w.K, w.metric)
    log("ground truth: %.1f s" % (time.time() - t0))
    del base_d
    torch.cuda.empty_cache()

    # ---- efS sweep: smallest efS of the grid with recall@K >= 0.95 ----
    curve = []
    chosen = None
    # the configuration's grid, continued upwards: this synthetic set needs more than efS = 512
    grid = (args.efs,) if args.efs else tuple(w.efs_grid) + tuple(
        e for e in (640, 768, 896, 1024, 1152, 1280, 1408, 1536, 1664, 1792, 1920, 2048, 2560, 3072, 4096)
        if e > max(w.efs_grid))
    for efS in grid:
        ix.reset_counters()
        t1 = time.time()
        ids, dists = ix.search(q_d, w.K, efS)
        dt = time.time() - t1
        rec = wl.recall_at_k(ids.cpu().numpy(), gt)
        c = ix.counters()
        curve.append({"efS": efS, "recall": round(rec, 4), "qps_single_call": round(w.nq / dt, 1),
                      "hops_per_query": round(c["hops"] / w.nq, 1), "exact_per_query": round(c["exact"] / w.nq, 1),
                      "gamma": round(c["passes"] / max(1, c["tests"]), 4)})
        log("efS %4d: recall@%d %.4f, %.0f QPS (one call), hops/q %.1f, exact/q %.1f, pass ratio %.3f" %
            (efS, w.K, rec, w.nq / dt, c["hops"] / w.nq, c["exact"] / w.nq, c["passes"] / max(1, c["tests"])))
        if chosen is None and rec >= TARGET_RECALL:
            chosen = (efS, rec)
            if not args.efs:
                break
    reached = chosen is not None
    if chosen is None:
        chosen = (curve[-1]["efS"], curve[-1]["recall"])
        log("recall %.2f not reached on the grid; timing the largest efS" % TARGET_RECALL)
    efS, recall = chosen
    # linear interpolation between the two grid points that bracket the target (single-call rates)
    interp = None
    for lo, hi in zip(curve, curve[1:]):
        if lo["recall"] < TARGET_RECALL <= hi["recall"] and hi["efS"] == efS:
            t = (TARGET_RECALL - lo["recall"]) / (hi["recall"] - lo["recall"])
            interp = round(lo["qps_single_call"] + t * (hi["qps_single_call"] - lo["qps_single_call"]), 1)

    if args.pmc_probe:
        x = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        y = torch.empty_like(x)
        torch.add(x, 1.0, out=y)
        torch.cuda.synchronize()
        del x, y

    # ---- timed region ----
    ids = torch.empty((w.nq, w.K), dtype=torch.int64, device="cuda")
    dists = torch.empty((w.nq, w.K), dtype=torch.float32, device="cuda")
    for _ in range(args.warmup):
        ix.search(q_d, w.K, efS, out=(ids, dists))
    ix.reset_counters()
    kernel_ms = []
    prep_ms = []
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        ix.search(q_d, w.K, efS, out=(ids, dists))
        # HIP-event durations recorded by the library on its own stream around the kernels of this call
        c = ix.counters()
        kernel_ms.append(c["last_search_kernel_ms"])
        prep_ms.append(c["last_prepare_ms"])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    c = ix.counters()
    ms_per_step = 1e3 * elapsed / args.steps
    qps = w.nq * args.steps / elapsed
    bytes_per_launch = algorithmic_bytes(c, w.d, w.K, vec_bytes) / args.steps
    k_ms = float(np.mean(kernel_ms))
    achieved = bytes_per_launch / (k_ms * 1e-3) / 1e9
    tag = "cfg%d" % w.cfg if (args.n is None and args.nq is None and not args.fp16_vectors) else "custom"
    # what this machine delivers when a kernel does nothing but fetch rows of the same vector store
    rows_probe = min(8 * w.n, 4_000_000)
    stream_gbs = ix.measure_row_reads(rows_probe, False)
    gather_gbs = ix.measure_row_reads(rows_probe, True)
    hop_gbs = ix.measure_row_reads(rows_probe, 2)
    log("row reads on this box: in order %.0f GB/s, scattered %.0f GB/s; with a hop's side traffic %.0f GB/s" %
        (stream_gbs, gather_gbs, hop_gbs))
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": read_traffic(tag, efS),
                "kernel": "pagk::k_search", "kernel_ms": round(k_ms, 4), "kernel_ms_median": round(float(np.median(kernel_ms)), 4),
                "prepare_ms": round(float(np.mean(prep_ms)), 4),
                "algorithmic_bytes_per_launch": int(bytes_per_launch),
                "measured_row_read_GBps": {"in_order": round(stream_gbs, 1), "scattered": round(gather_gbs, 1),
                                           "scattered_with_hop_side_traffic": round(hop_gbs, 1)},
                "frac_of_measured_scattered_reads": round(achieved / gather_gbs, 4),
                "frac_of_measured_hop_traffic": round(achieved / hop_gbs, 4)}

    # ---- CPU oracle on the same index, same efS, bounded sample ----
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import pag_oracle as orc
        ex = ix.export()
        oix = orc.OracleIndex(ex["vectors"], ex["adj"], ex["a"], ex["c"], ex["e2"], ex["codes"], ex["rotation"],
                              ex["codebooks"], ex["entry"], metric=ex["metric"])
        cores = min(16, os.cpu_count() or 1)
        probe = min(w.nq, 2 * cores)
        t2 = time.perf_counter()
        oix.search(q[:probe], w.K, efS, threads=cores)
        per_q = (time.perf_counter() - t2) / probe
        sample = int(max(probe, min(w.nq, args.cpu_seconds / max(per_q, 1e-9))))
        t2 = time.perf_counter()
        oi, od, oc = oix.search(q[:sample], w.K, efS, threads=cores)
        dt = time.perf_counter() - t2
        agree = float((oi == ids[:sample].cpu().numpy()).mean())
        # the paper's own convention is one thread: a few seconds of that as well
        n1 = int(max(4, min(sample, 4.0 / max(per_q * cores, 1e-9))))
        t2 = time.perf_counter()
        oix.search(q[:n1], w.K, efS, threads=1)
        dt1 = time.perf_counter() - t2
        oracle_skipped = round(1.0 - oc["passes"] / max(1, oc["tests"]), 4)
        cpu = {"value": round(sample / dt, 1), "unit": "queries/s", "cores": cores, "kind": "oracle",
               "sample": "first %d of %d queries, same exported index, efS=%d; id-slot agreement with the GPU %.5f"
                         % (sample, w.nq, efS, agree),
               "single_thread": {"value": round(n1 / dt1, 1), "unit": "queries/s", "sample": "first %d queries" % n1},
               "skipped_fraction_of_unseen_neighbours": oracle_skipped}
        log("cpu oracle: %.1f QPS on %d threads over %d queries; GPU/oracle id agreement %.5f" %
            (sample / dt, cores, sample, agree))

    out = {
        "metric": "batched QPS at recall@%d>=0.95 (1 GPU)" % w.K, "value": round(qps, 1), "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic" + (" (base vectors stored as 16-bit floats)" if args.fp16_vectors else ""),
        "config": {"workload": "cfg%d %s: n=%d d=%d nq=%d K=%d deg=%d P=%d efC=%d" %
                               (w.cfg, w.name, w.n, w.d, w.nq, w.K, w.deg, w.P, args.efc),
                   "efS": efS, "efS_within_configured_grid": bool(efS <= max(w.efs_grid)),
                   "recall_at_K": round(recall, 4), "recall_target_reached": reached,
                   "qps_interpolated_at_recall_%.2f" % TARGET_RECALL: interp,
                   "skipped_fraction_of_evaluated_neighbours": round(1.0 - c["passes"] / max(1, c["tests"]), 4),
                   "hops_per_query": round(c["hops"] / max(1, c["queries"]), 1),
                   "exact_per_query": round(c["exact"] / max(1, c["queries"]), 1),
                   "build_seconds": round(build_s, 2), "sweep": curve},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
