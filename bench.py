#!/usr/bin/env python3
"""Benchmark of the PAG search hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--cfg 2] [--n N] [--nq NQ] [--efc EFC] [--K K]

A "step" is one pag_search call over the whole query batch of the workload (query rotation,
projection tables and the fused best-first search), queries and results resident in HBM.
The headline workload is configuration 2 of the synthetic set (n = 1,000,000, d = 768, inner product
on unit vectors, degree 32, 32 subspaces, K = 10): the index is built on the GPU by pag_build, the
efS grid is swept against brute-force ground truth, and the timed steps run at the smallest efS
whose recall@10 reaches 0.95, with the paper's working-set size b = max(10, K).  One JSON line is printed:
  value        whole-batch queries per second over the timed steps
  roofline     algorithmic HBM bytes of the search kernel / its HIP-event duration, against 8 TB/s
  cpu_baseline the CPU oracle searching the same exported index with the same efS on a bounded
               sample of the queries, on the host cores of this machine
  config.tuned           the same search with the working-set size the method leaves free (search_b)
  config.build           what index construction cost, against its own byte model
  config.other_workloads configurations 3, 5 and 4, as far as the time budget allows
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
T_START = time.time()

# what the secondary workloads took on an MI355X machine (generation on the host, build, ground truth, sweep, timing),
# with some margin: a workload only starts if it fits what is left of the budget
SECONDARY_SECONDS = {3: 45.0, 5: 130.0, 4: 130.0}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(c, d, K, vec_bytes=4):
    """Bytes the method itself must move (Sec. 4.2's terms): per query the query vector and the
    results, per expanded node its adjacency record, per exact distance one base vector."""
    return (c["queries"] * (4 * d + 8 * K) + c["hops"] * c["adj_record_bytes"] + c["exact"] * vec_bytes * d)


def read_traffic(tag, efS):
    """HBM bytes per search-kernel launch from the committed rocprofv3 counter summary, if it covers this run
    (same workload, same efS); otherwise None.  The figure is a recording of an earlier run of this same
    command under rocprofv3 --pmc, not something this process measured."""
    path = os.path.join(ROOT, "profiles", "search_kernel_%s_hbm_traffic.txt" % tag)
    vals = {}
    try:
        with open(path) as f:
            for line in f:
                if line.startswith(("traffic_bytes_per_launch:", "efS:")):
                    k, v = line.split(":")
                    vals[k] = float(v)
    except OSError:
        return None, None
    if vals.get("efS") != float(efS):
        return None, None
    return vals.get("traffic_bytes_per_launch"), os.path.relpath(path, ROOT)


def build_report(c, w, n_vectors, build_s, efc, vec_bytes=4):
    """Index construction against its byte model.  Per inserted vector (Sec. 4.2, insertion cost): the search
    moves one adjacency record per expanded node and one base vector per exact distance; RobustPrune reads each
    of the <= efC candidates once and, for every candidate, the kept neighbours until one occludes it (counted
    here at its upper bound efC + efC * deg / 2 rows); the reverse-edge pass reads deg rows per kept neighbour."""
    q = max(1, c["queries"])
    search_bytes = c["hops"] * c["adj_record_bytes"] + c["exact"] * vec_bytes * w.d
    ph = c["last_build_phase_ms"]
    out = {"seconds": round(build_s, 2), "vectors_per_s": round(n_vectors / build_s, 1), "efC": efc,
           "insertion_searches": int(c["queries"]),
           "hops_per_vector": round(c["hops"] / q, 1), "exact_per_vector": round(c["exact"] / q, 1),
           "gamma": round(c["passes"] / max(1, c["tests"]), 4),
           "search_algorithmic_bytes_per_vector": int(search_bytes / q),
           "phase_ms": {"search_kernel": round(ph[0], 1), "sort_and_robust_prune": round(ph[1], 1),
                        "pair_sort_and_reverse_edges": round(ph[2], 1), "inference_information": round(ph[3], 1)},
           "relinked_batches": int(c["relinked_batches"])}
    if ph[0] > 0:
        gbs = search_bytes / (ph[0] * 1e-3) / 1e9
        out["search_kernel_roofline"] = {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                         "frac": round(gbs / HBM_PEAK_GBS, 4)}
    return out


def search_workload(args, w, wl, torch, np, PagIndex, *, steps, warmup, efs_fixed=0, fp16=False, K=None, extra_K=()):
    """Generate the workload, build its index, sweep efS up to the recall target, time `steps` searches there.
    Returns the measurements and what the caller may want to go on with (index, queries, ids)."""
    from paper_2603_06660_amd import FLAG_FP16_VECTORS, FLAG_EXACT_TEST_COUNT
    K = K or w.K
    metric = {0: "l2", 1: "ip", 2: "cos"}[w.metric]
    t0 = time.time()
    base = wl.make(w, "base")
    q = wl.make(w, "query")
    log("generated %s: base %s, queries %s in %.1f s" % (w.name, base.shape, q.shape, time.time() - t0))
    base_d = torch.from_numpy(base).cuda()
    q_d = torch.from_numpy(q).cuda()
    del base

    t0 = time.time()
    vec_bytes = 2 if fp16 else 4
    ix = PagIndex.build(base_d, metric=metric, max_degree=w.deg, num_subspaces=w.P, ef_construction=args.efc,
                        seed=2603, flags=FLAG_FP16_VECTORS if fp16 else 0)
    build_s = time.time() - t0
    build = build_report(ix.counters(), w, w.n, build_s, args.efc, vec_bytes)
    log("pag_build: %.2f s (%.0f vectors/s); phases %s" % (build_s, w.n / build_s, build["phase_ms"]))

    t0 = time.time()
    Ks = (K,) + tuple(k for k in extra_K if k != K)
    gts = {}
    gt_big, _ = wl.brute_force_torch(base_d, q_d, max(Ks), w.metric)
    for k in Ks:
        gts[k] = gt_big[:, :k]
    gt_s = time.time() - t0
    log("ground truth: %.1f s" % gt_s)
    del base_d
    torch.cuda.empty_cache()

    def one_search(k, efS, counting):
        """one untimed call; counting: the seen set is resolved before the test, so tests = unseen neighbours"""
        ix.set_search_options(args.search_b, FLAG_EXACT_TEST_COUNT if counting else 0)
        ix.reset_counters()
        t1 = time.time()
        ids, _ = ix.search(q_d, k, efS)
        dt = time.time() - t1
        c = ix.counters()
        ix.set_search_options(args.search_b, 0)
        return ids, dt, c

    def sweep(k, fixed):
        curve, chosen = [], None
        grid = (fixed,) if fixed else tuple(w.efs_grid) + tuple(
            e for e in (640, 768, 896, 1024, 1152, 1280, 1408, 1536, 1664, 1792, 1920, 2048, 2560, 3072, 4096)
            if e > max(w.efs_grid))
        grid = tuple(e for e in grid if e >= k) or (k,)
        for efS in grid:
            ids, dt, c = one_search(k, efS, False)
            rec = wl.recall_at_k(ids.cpu().numpy(), gts[k])
            _, _, cx = one_search(k, efS, True)
            gamma = cx["passes"] / max(1, cx["tests"])
            curve.append({"efS": efS, "recall": round(rec, 4), "qps_single_call": round(w.nq / dt, 1),
                          "hops_per_query": round(c["hops"] / w.nq, 1), "exact_per_query": round(c["exact"] / w.nq, 1),
                          "gamma": round(gamma, 4)})
            log("K %d efS %4d: recall@%d %.4f, %.0f QPS (one call), hops/q %.1f, exact/q %.1f, pass ratio %.3f" %
                (k, efS, k, rec, w.nq / dt, c["hops"] / w.nq, c["exact"] / w.nq, gamma))
            if chosen is None and rec >= TARGET_RECALL:
                chosen = (efS, rec)
                if not fixed:
                    break
        reached = chosen is not None
        if chosen is None:
            chosen = (curve[-1]["efS"], curve[-1]["recall"])
            log("recall %.2f not reached on the grid; timing the largest efS" % TARGET_RECALL)
        return curve, chosen, reached

    # ---- efS sweep: smallest efS of the grid (the configuration's, continued upwards) with recall@K >= 0.95 ----
    curve, (efS, recall), reached = sweep(K, efs_fixed)
    interp = None      # linear interpolation between the two grid points that bracket the target (single-call rates)
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

    def timed(k, efS, search_b):
        ix.set_search_options(search_b, 0)
        ids = torch.empty((w.nq, k), dtype=torch.int64, device="cuda")
        dists = torch.empty((w.nq, k), dtype=torch.float32, device="cuda")
        for _ in range(warmup):
            ix.search(q_d, k, efS, out=(ids, dists))
        ix.reset_counters()
        kernel_ms, prep_ms = [], []
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(steps):
            ix.search(q_d, k, efS, out=(ids, dists))
            # HIP-event durations recorded by the library on its own stream around the kernels of this call
            c = ix.counters()
            kernel_ms.append(c["last_search_kernel_ms"])
            prep_ms.append(c["last_prepare_ms"])
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t1
        c = ix.counters()
        bytes_per_launch = algorithmic_bytes(c, w.d, k, vec_bytes) / steps
        k_ms = float(np.mean(kernel_ms))
        achieved = bytes_per_launch / (k_ms * 1e-3) / 1e9
        ix.set_search_options(args.search_b, 0)
        return {"ids": ids, "qps": w.nq * steps / elapsed, "ms_per_step": 1e3 * elapsed / steps, "counters": c,
                "kernel_ms": k_ms, "kernel_ms_median": float(np.median(kernel_ms)), "prepare_ms": float(np.mean(prep_ms)),
                "bytes_per_launch": bytes_per_launch, "achieved": achieved,
                "recall": wl.recall_at_k(ids.cpu().numpy(), gts[k])}

    # ---- timed region ----
    t = timed(K, efS, args.search_b)
    c = t["counters"]
    # for scale: the same batch taken as numbered instead of in the library's own order (not in the runs that
    # a profiler summarises: every launch of those is the timed configuration)
    numbered_ms = []
    if not args.no_tuned:
        from paper_2603_06660_amd import FLAG_KEEP_QUERY_ORDER
        ix.set_search_options(args.search_b, FLAG_KEEP_QUERY_ORDER)
        for i in range(4):
            ix.search(q_d, K, efS)
            if i:
                numbered_ms.append(ix.counters()["last_search_kernel_ms"])
        ix.set_search_options(args.search_b, 0)
    _, _, cx = one_search(K, efS, True)
    skipped = 1.0 - cx["passes"] / max(1, cx["tests"])
    tag = "cfg%d" % w.cfg if (args.n is None and args.nq is None and not fp16 and K == w.K and not args.search_b) else "custom"
    # what this machine delivers when a kernel does nothing but fetch rows of the same vector store
    rows_probe = min(8 * w.n, 4_000_000)
    stream_gbs = ix.measure_row_reads(rows_probe, False)
    gather_gbs = ix.measure_row_reads(rows_probe, True)
    hop_gbs = ix.measure_row_reads(rows_probe, 2)
    log("row reads on this box: in order %.0f GB/s, scattered %.0f GB/s; with a hop's side traffic %.0f GB/s" %
        (stream_gbs, gather_gbs, hop_gbs))
    traffic, traffic_src = read_traffic(tag, efS)
    roofline = {"bound": "hbm", "achieved": round(t["achieved"], 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(t["achieved"] / HBM_PEAK_GBS, 4), "traffic": traffic,
                "traffic_source": ("recorded earlier by rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on this command: %s" % traffic_src)
                if traffic else None,
                "kernel": "pagk::k_search", "kernel_ms": round(t["kernel_ms"], 4),
                "kernel_ms_median": round(t["kernel_ms_median"], 4), "prepare_ms": round(t["prepare_ms"], 4),
                "algorithmic_bytes_per_launch": int(t["bytes_per_launch"]),
                "kernel_ms_queries_as_numbered": round(float(np.mean(numbered_ms)), 4) if numbered_ms else None,
                # secondary: table additions of the screen (hops x neighbours x subspaces) + 3 d per exact distance
                "alu_TFLOPs": round((c["hops"] * w.deg * w.P + c["exact"] * 3 * w.d) / steps / (t["kernel_ms"] * 1e-3) / 1e12, 2),
                "measured_row_read_GBps": {"in_order": round(stream_gbs, 1), "scattered": round(gather_gbs, 1),
                                           "scattered_with_hop_side_traffic": round(hop_gbs, 1)},
                "frac_of_measured_scattered_reads": round(t["achieved"] / gather_gbs, 4),
                "frac_of_measured_hop_traffic": round(t["achieved"] / hop_gbs, 4)}
    res = {"w": w, "K": K, "ix": ix, "q": q, "q_d": q_d, "ids": t["ids"], "efS": efS, "recall": recall, "reached": reached,
           "interp": interp, "curve": curve, "qps": t["qps"], "ms_per_step": t["ms_per_step"], "counters": c,
           "skipped": skipped, "roofline": roofline, "build": build, "build_s": build_s, "vec_bytes": vec_bytes, "gt_s": gt_s,
           "timed": timed, "gts": gts, "hop_gbs": hop_gbs}
    # further retrieval sizes on the same index (cfg 4: K = 10 and K = 50)
    res["extra_K"] = {}
    for k in extra_K:
        if k == K:
            continue
        cv, (e2, r2), ok = sweep(k, 0)
        t2 = timed(k, e2, args.search_b)
        res["extra_K"]["K=%d" % k] = {"efS": e2, "recall": round(r2, 4), "recall_target_reached": ok,
                                      "queries_per_s": round(t2["qps"], 1), "kernel_ms": round(t2["kernel_ms"], 3),
                                      "roofline_frac": round(t2["achieved"] / HBM_PEAK_GBS, 4),
                                      "frac_of_measured_hop_traffic": round(t2["achieved"] / hop_gbs, 4)}
    return res


def tuned_working_set(res, np, log_=log):
    """The working-set size b is a free parameter of the method (Alg. 2 takes it as input; max(10, K) is the paper's
    default).  At the headline's efS, the fastest b of a small grid that still reaches the recall target."""
    w, K, efS = res["w"], res["K"], res["efS"]
    best = None
    rows = []
    for b in (16, 24, 32, 48, 64):
        if b < K:
            continue
        t = res["timed"](K, efS, b)
        rows.append({"search_b": b, "recall": round(t["recall"], 4), "queries_per_s": round(t["qps"], 1),
                     "kernel_ms": round(t["kernel_ms"], 3)})
        log_("search_b %3d at efS %d: recall %.4f, %.0f QPS, kernel %.2f ms" % (b, efS, t["recall"], t["qps"], t["kernel_ms"]))
        if t["recall"] >= TARGET_RECALL and (best is None or t["qps"] > best[1]["qps"]):
            best = (b, t)
    if best is None:
        return {"grid": rows, "search_b": None}
    b, t = best
    return {"search_b": b, "efS": efS, "recall_at_K": round(t["recall"], 4), "value": round(t["qps"], 1), "unit": "queries/s",
            "ms_per_step": round(t["ms_per_step"], 4),
            "roofline": {"bound": "hbm", "achieved": round(t["achieved"], 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": round(t["achieved"] / HBM_PEAK_GBS, 4), "kernel_ms": round(t["kernel_ms"], 4),
                         "algorithmic_bytes_per_launch": int(t["bytes_per_launch"])},
            "grid": rows, "ids": t["ids"]}


def cpu_baseline(args, res, np, tuned):
    """The oracle as it stands on the host cores of this machine: all cores on a bounded sample, one thread (the paper's
    own convention) on the first 1,000 queries; the same exported index, the same efS."""
    from oracle import pag_oracle as orc
    w, K, efS, ix, q = res["w"], res["K"], res["efS"], res["ix"], res["q"]
    ex = ix.export()
    oix = orc.OracleIndex(ex["vectors"], ex["adj"], ex["a"], ex["c"], ex["e2"], ex["codes"], ex["rotation"],
                          ex["codebooks"], ex["entry"], metric=ex["metric"])
    nproc = os.cpu_count() or 1
    try:
        cores = len(os.sched_getaffinity(0))      # the cores this process may actually run on
    except AttributeError:
        cores = nproc
    probe = min(w.nq, 2 * cores)
    t2 = time.perf_counter()
    oix.search(q[:probe], K, efS, threads=cores)
    per_q = (time.perf_counter() - t2) / probe
    sample = int(max(probe, min(w.nq, args.cpu_seconds / max(per_q, 1e-9))))
    t2 = time.perf_counter()
    oi, od, oc = oix.search(q[:sample], K, efS, threads=cores)
    dt = time.perf_counter() - t2
    agree = float((oi == res["ids"][:sample].cpu().numpy()).mean())
    n1 = min(w.nq, 1000)
    if per_q * cores * n1 > 2.0 * args.cpu_seconds:          # keep the default run within minutes on a slow host
        n1 = int(max(16, 2.0 * args.cpu_seconds / (per_q * cores)))
    t2 = time.perf_counter()
    oix.search(q[:n1], K, efS, threads=1)
    dt1 = time.perf_counter() - t2
    oracle_skipped = round(1.0 - oc["passes"] / max(1, oc["tests"]), 4)
    cpu = {"value": round(sample / dt, 1), "unit": "queries/s", "cores": cores, "nproc": nproc, "kind": "oracle",
           "sample": "first %d of %d queries, same exported index, efS=%d; id-slot agreement with the GPU %.5f"
                     % (sample, w.nq, efS, agree),
           "single_thread": {"value": round(n1 / dt1, 1), "unit": "queries/s", "sample": "first %d queries" % n1},
           "skipped_fraction_of_unseen_neighbours": oracle_skipped}
    log("cpu oracle: %.1f QPS on %d threads (nproc %d) over %d queries; one thread %.1f QPS over %d; GPU/oracle id agreement %.5f" %
        (sample / dt, cores, nproc, sample, n1 / dt1, n1, agree))
    if tuned and tuned.get("search_b"):
        ns = max(2 * cores, sample // 4)
        oi, _, _ = oix.search(q[:ns], K, efS, b=tuned["search_b"], threads=cores)
        tuned["oracle_id_agreement"] = round(float((oi == tuned["ids"][:ns].cpu().numpy()).mean()), 5)
        tuned["oracle_sample"] = "first %d queries at search_b=%d" % (ns, tuned["search_b"])
    return cpu


def online_insertion(args, w, wl, torch, np, PagIndex):
    """Workload 5 (the paper's online-insertion experiment, Sec. 5.2 D6, at synthetic scale): build on the
    initial vectors, then rounds of pag_insert followed by a query batch; reports insertion throughput, the
    recall after every round against brute force over the vectors inserted so far, and the search kernel's
    rate against the HBM roofline."""
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
    build = build_report(ix.counters(), w, w.n, build_s, args.efc)
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
    ins_phase = np.zeros(4)
    ins_counters = {"queries": 0, "hops": 0, "exact": 0}
    fracs = []
    for r in range(rounds):
        x = wl.make(w, "insert%d" % r, n=per_round)
        all_d[n:n + per_round] = torch.from_numpy(x)
        torch.cuda.synchronize()
        ix.reset_counters()
        t1 = time.perf_counter()
        ix.insert(all_d[n:n + per_round])
        dt = time.perf_counter() - t1
        ci = ix.counters()
        ins_time += dt
        ins_phase += np.array(ci["last_build_phase_ms"])
        for k in ins_counters:
            ins_counters[k] += ci[k]
        n += per_round
        ix.search(q_d, w.K, efS)                                   # warm-up: workspaces sized, caches filled
        ix.reset_counters()
        t1 = time.perf_counter()
        ids, _ = ix.search(q_d, w.K, efS)
        ts = time.perf_counter() - t1
        c = ix.counters()
        gbs = algorithmic_bytes(c, w.d, w.K) / (c["last_search_kernel_ms"] * 1e-3) / 1e9
        fracs.append(gbs / HBM_PEAK_GBS)
        gt, _ = wl.brute_force_torch(all_d[:n], q_d, w.K, w.metric)
        rec = wl.recall_at_k(ids.cpu().numpy(), gt)
        rows.append({"round": r + 1, "n": n, "insert_vectors_per_s": round(per_round / dt, 1),
                     "search_qps": round(w.nq / ts, 1), "recall": round(rec, 4),
                     "search_kernel_ms": round(c["last_search_kernel_ms"], 3), "search_roofline_frac": round(gbs / HBM_PEAK_GBS, 4)})
        log("round %2d: n = %d, insert %.0f vectors/s, search %.0f QPS at efS %d (kernel %.2f ms, %.0f GB/s), recall@%d %.4f" %
            (r + 1, n, per_round / dt, w.nq / ts, efS, c["last_search_kernel_ms"], gbs, w.K, rec))
    hop_gbs = ix.measure_row_reads(2_000_000, 2)
    out = {"workload": "cfg5 %s: start n=%d d=%d, %d rounds x (insert %d, search %d queries) K=%d deg=%d P=%d efC=%d efS=%d" %
                       (w.name, w.n, w.d, rounds, per_round, w.nq, w.K, w.deg, w.P, args.efc, efS),
           "insert_vectors_per_s": round(rounds * per_round / ins_time, 1),
           "ms_per_round_insert": round(1e3 * ins_time / max(1, rounds), 3),
           "recall_first_round": rows[0]["recall"] if rows else None, "recall_last_round": rows[-1]["recall"] if rows else None,
           "search_qps_last_round": rows[-1]["search_qps"] if rows else None,
           "search_roofline": {"bound": "hbm", "peak": HBM_PEAK_GBS, "unit": "GB/s",
                               "achieved": round(float(np.mean(fracs)) * HBM_PEAK_GBS, 1) if fracs else None,
                               "frac": round(float(np.mean(fracs)), 4) if fracs else None,
                               "frac_of_measured_hop_traffic": round(float(np.mean(fracs)) * HBM_PEAK_GBS / hop_gbs, 4) if fracs else None},
           "insert_phase_ms_per_round": {k: round(v / max(1, rounds), 1) for k, v in
                                         zip(("search_kernel", "sort_and_robust_prune", "pair_sort_and_reverse_edges",
                                              "inference_information"), ins_phase)},
           "insert_hops_per_vector": round(ins_counters["hops"] / max(1, ins_counters["queries"]), 1),
           "insert_exact_per_vector": round(ins_counters["exact"] / max(1, ins_counters["queries"]), 1),
           "initial_build": build, "rounds": rows}
    if args.concurrent:
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
        out["insert_and_search_at_once"] = {
            "insert_vectors_per_s": round(per_round / timing["insert_s"], 1),
            "search_qps_meanwhile": round(batches * w.nq / t_search, 1), "query_batches": batches,
            "recall_of_last_batch_vs_index_before": round(rec_c, 4)}
        log("concurrent: insert %.0f vectors/s while a searcher answered %d batches at %.0f QPS (recall %.4f)" %
            (per_round / timing["insert_s"], batches, batches * w.nq / t_search, rec_c))
        srch.close()
    ix.close()
    del all_d
    torch.cuda.empty_cache()
    return out


def compact(res):
    """What a secondary workload reports under config.other_workloads."""
    w, c = res["w"], res["counters"]
    r = res["roofline"]
    out = {"workload": "cfg%d %s: n=%d d=%d nq=%d K=%d deg=%d P=%d" % (w.cfg, w.name, w.n, w.d, w.nq, res["K"], w.deg, w.P),
           "efS": res["efS"], "recall_at_K": round(res["recall"], 4), "recall_target_reached": res["reached"],
           "queries_per_s": round(res["qps"], 1), "ms_per_step": round(res["ms_per_step"], 3),
           "gamma": round(1.0 - res["skipped"], 4),
           "hops_per_query": round(c["hops"] / max(1, c["queries"]), 1), "exact_per_query": round(c["exact"] / max(1, c["queries"]), 1),
           "roofline": {k: r[k] for k in ("bound", "achieved", "peak", "unit", "frac", "kernel_ms", "kernel_ms_queries_as_numbered",
                                          "algorithmic_bytes_per_launch", "frac_of_measured_hop_traffic")},
           "build": res["build"], "sweep": [{k: p[k] for k in ("efS", "recall", "gamma")} for p in res["curve"]]}
    if res["extra_K"]:
        out["other_retrieval_sizes"] = res["extra_K"]
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--cfg", type=int, default=2)
    ap.add_argument("--n", type=int, default=None)
    ap.add_argument("--nq", type=int, default=None)
    ap.add_argument("--K", type=int, default=None, help="retrieval size, if not the configuration's")
    ap.add_argument("--efc", type=int, default=2000)
    ap.add_argument("--efs", type=int, default=0, help="skip the sweep and time this efS")
    ap.add_argument("--search-b", type=int, default=0, help="working-set size b; 0 = the paper's max(10, K)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--fp16-vectors", action="store_true",
                    help="keep the base vectors as 16-bit floats (the paper's payload); NOT the headline configuration")
    ap.add_argument("--rounds", type=int, default=10, help="cfg 5: insertion rounds")
    ap.add_argument("--insert-batch", type=int, default=50000, help="cfg 5: vectors per insertion round")
    ap.add_argument("--concurrent", action="store_true", help="cfg 5: one more batch inserted while a searcher answers queries")
    ap.add_argument("--no-other-workloads", action="store_true", help="headline workload only")
    ap.add_argument("--no-tuned", action="store_true", help="skip the working-set size grid and the as-numbered query order timing")
    ap.add_argument("--budget-seconds", type=float, default=420.0,
                    help="wall-clock budget of the whole run: a secondary workload is left out if it would not fit")
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

    if w.cfg == 5:
        r = online_insertion(args, w, wl, torch, np, PagIndex)
        out = {"metric": "online insertion throughput (1 GPU)", "value": r["insert_vectors_per_s"],
               "unit": "vectors/s", "n_gpus": 1, "steps": args.rounds, "warmup": 0,
               "ms_per_step": r["ms_per_round_insert"], "higher_is_better": True, "scaling": "weak",
               "vs_baseline": None, "dtype": "f32", "data": "synthetic", "config": r,
               "roofline": r["search_roofline"], "cpu_baseline": None}
        print(json.dumps(out), flush=True)
        return

    headline = w.cfg == 2 and args.n is None and args.nq is None and not args.fp16_vectors and not args.K and not args.search_b
    res = search_workload(args, w, wl, torch, np, PagIndex, steps=args.steps, warmup=args.warmup, efs_fixed=args.efs,
                          fp16=args.fp16_vectors, K=args.K, extra_K=(10, 50) if w.cfg == 4 and not args.K else ())
    tuned = None
    if not args.no_tuned and not args.search_b:
        tuned = tuned_working_set(res, np)
    cpu = None if args.no_cpu_baseline else cpu_baseline(args, res, np, tuned)
    if tuned:
        tuned.pop("ids", None)
    c = res["counters"]
    K = res["K"]
    config = {"workload": "cfg%d %s: n=%d d=%d nq=%d K=%d deg=%d P=%d efC=%d" %
                          (w.cfg, w.name, w.n, w.d, w.nq, K, w.deg, w.P, args.efc),
              "efS": res["efS"], "efS_within_configured_grid": bool(res["efS"] <= max(w.efs_grid)),
              "search_b": args.search_b or max(10, K),
              "recall_at_K": round(res["recall"], 4), "recall_target_reached": res["reached"],
              "qps_interpolated_at_recall_%.2f" % TARGET_RECALL: res["interp"],
              "gamma": round(1.0 - res["skipped"], 4),
              "skipped_fraction_of_unseen_neighbours": round(res["skipped"], 4),
              "hops_per_query": round(c["hops"] / max(1, c["queries"]), 1),
              "exact_per_query": round(c["exact"] / max(1, c["queries"]), 1),
              "build_seconds": round(res["build_s"], 2), "build": res["build"], "sweep": res["curve"], "tuned": tuned,
              # for scale: exhaustive search of the same batch (torch matmul + top-k on the GPU, re-ranked in fp64), the ground truth
              "brute_force_queries_per_s": round(w.nq / res["gt_s"], 1)}
    if res["extra_K"]:
        config["other_retrieval_sizes"] = res["extra_K"]
    head = {"qps": res["qps"], "ms_per_step": res["ms_per_step"], "roofline": res["roofline"]}
    # ---- the other configurations, as far as the time budget allows (headline run only) ----
    if headline and not args.no_other_workloads:
        res["ix"].close()
        res = None
        torch.cuda.empty_cache()
        others, left_out = {}, []
        for cfg in (3, 5, 4):
            spent = time.time() - T_START
            if spent + SECONDARY_SECONDS[cfg] > args.budget_seconds:
                left_out.append("cfg%d (%.0f s spent, needs about %.0f s, budget %.0f s)" %
                                (cfg, spent, SECONDARY_SECONDS[cfg], args.budget_seconds))
                continue
            t0 = time.time()
            w2 = wl.workload(cfg)
            try:
                if cfg == 5:
                    others["cfg5"] = online_insertion(args, w2, wl, torch, np, PagIndex)
                else:
                    r2 = search_workload(args, w2, wl, torch, np, PagIndex, steps=5, warmup=2,
                                         extra_K=(10, 50) if cfg == 4 else ())
                    others["cfg%d" % cfg] = compact(r2)
                    r2["ix"].close()
                    del r2
            except Exception as ex:          # a secondary workload must not cost the run its headline line
                log("cfg%d failed: %r" % (cfg, ex))
                others["cfg%d" % cfg] = {"error": repr(ex)}
            torch.cuda.empty_cache()
            others["cfg%d" % cfg]["wall_seconds"] = round(time.time() - t0, 1)
        others["left_out"] = left_out
        config["other_workloads"] = others
    out = {
        "metric": "batched QPS at recall@%d>=0.95 (1 GPU)" % K, "value": round(head["qps"], 1), "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(head["ms_per_step"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic" + (" (base vectors stored as 16-bit floats)" if args.fp16_vectors else ""),
        "config": config, "roofline": head["roofline"], "cpu_baseline": cpu,
        "wall_seconds": round(time.time() - T_START, 1),
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
