"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Bars (stated by the benchmark spec): result ids equal on >= 99.9 % of (query, rank) slots, distances within
1e-5 relative, recall@K within 0.002; integer / index work (codes) bit-exact.  Because both sides
take every decision in the same precision, the observed agreement is normally 100 %.
"""
import numpy as np
import pytest

import pag_workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_06660_amd import PagIndex, load_library
    load_library()          # raises if the HIP library is not built: there is no fallback
    return PagIndex


def _import(PagIndex, oix, **kw):
    metric = {0: "l2", 1: "ip", 2: "cos"}[oix.metric]
    return PagIndex.from_arrays(oix.vec, oix.adj, oix.a, oix.c, oix.e2, oix.codes, oix.rot, oix.cb, oix.entry,
                                metric=metric, **kw)


def _assert_search_parity(gix, oix, q, K, efS, gt=None, b=0):
    qd = torch.from_numpy(q).cuda()
    gi, gd = gix.search(qd, K, efS)
    gi, gd = gi.cpu().numpy(), gd.cpu().numpy()
    oi, od, oc = oix.search(q, K, efS, b=b)
    agree = (gi == oi).mean()
    assert agree >= 0.999, "id slots agreeing: %.5f" % agree
    same = gi == oi
    fin = same & np.isfinite(od)
    assert np.all(np.abs(gd[fin] - od[fin]) <= 1e-5 * np.abs(od[fin]))
    assert np.array_equal(np.isinf(gd), gi < 0)
    if gt is not None:
        assert abs(wl.recall_at_k(gi, gt) - wl.recall_at_k(oi, gt)) <= 0.002
    # per query: ascending by (dist, id)
    assert np.all(np.diff(gd, axis=1) >= 0)
    return gi, gd, oc


def _check_tests_counter(gix, q, K, efS, gc, oc, search_b=0):
    """`tests` counts the neighbours the projection test was evaluated for.  Short searches (exact LDS seen
    set) evaluate it for unseen neighbours only, like the oracle.  Long searches consult the second level of
    the seen set only for neighbours that pass, so their count also holds the seen neighbours that the first
    level did not recognise and that failed the test: at most one per exact distance computed and expanded
    node (a seen node is met again through one of its in-edges).  In counting mode
    (PAG_FLAG_EXACT_TEST_COUNT) the second level is consulted first and the count is the oracle's."""
    from paper_2603_06660_amd import FLAG_EXACT_TEST_COUNT
    b = search_b if search_b else max(10, K)
    if b + 8 * max(efS, b) <= 1024:
        assert gc["tests"] == oc["tests"], (gc["tests"], oc["tests"])
        return
    assert oc["tests"] <= gc["tests"], (gc["tests"], oc["tests"])
    qd = torch.from_numpy(q).cuda()
    ref = gix.search(qd, K, efS)
    try:
        gix.set_search_options(search_b, FLAG_EXACT_TEST_COUNT)
        gix.reset_counters()
        got = gix.search(qd, K, efS)
        gx = gix.counters()
    finally:
        gix.set_search_options(search_b, 0)
    assert torch.equal(ref[0], got[0]) and torch.equal(ref[1], got[1])
    assert gx["tests"] == oc["tests"], (gx["tests"], oc["tests"])
    for k_g, k_o in (("hops", "hops"), ("passes", "passes"), ("exact", "exact"), ("rounds", "rounds")):
        assert gx[k_g] == oc[k_o], (k_g, gx[k_g], oc[k_o])


@pytest.fixture(scope="module")
def imported(orc, cfg1_small, cfg1_oracle_index):
    PagIndex = _gpu()
    return _import(PagIndex, cfg1_oracle_index)


def test_prepare_queries(orc, cfg1_small, cfg1_oracle_index, imported):
    """Rotation (fp64 MFMA) and projection tables against the oracle's fp64 loops."""
    w, base, q, gt, gtk = cfg1_small
    qr, T = imported.prepare_queries(torch.from_numpy(q).cuda())
    oqr, oT = cfg1_oracle_index.prepare(q)
    qr, T = qr.cpu().numpy(), T.cpu().numpy()
    assert (qr == oqr).mean() >= 0.9999
    assert np.allclose(qr, oqr, rtol=1e-6, atol=1e-6)
    assert (T == oT).mean() >= 0.9999
    assert np.allclose(T, oT, rtol=1e-6, atol=1e-7)


def test_exact_distances(orc, cfg1_small, cfg1_oracle_index, imported):
    w, base, q, gt, gtk = cfg1_small
    oix = cfg1_oracle_index
    oqr, _ = oix.prepare(q)
    rng = np.random.default_rng(3)
    ids = rng.integers(0, oix.n, size=(len(q), 9)).astype(np.int32)
    keys = imported.exact_distances(torch.from_numpy(oqr).cuda(), torch.from_numpy(ids).cuda()).cpu().numpy()
    ref = np.array([[orc.key(oqr[i], oix.vec[j]) for j in ids[i]] for i in range(len(q))], np.float32)
    assert np.all(np.abs(keys - ref) <= 1e-5 * ref)
    assert (keys == ref).mean() >= 0.999


def test_projection_screen(orc, cfg1_small, cfg1_oracle_index, imported):
    """est = D_u + c - 2 a S for every neighbour slot of an expanded node: fp32, fixed order -> bit-exact."""
    w, base, q, gt, gtk = cfg1_small
    oix = cfg1_oracle_index
    oqr, oT = oix.prepare(q)
    rng = np.random.default_rng(4)
    u = rng.integers(0, oix.n, size=len(q)).astype(np.int32)
    Du = np.array([orc.key(oqr[i], oix.vec[u[i]]) for i in range(len(q))], np.float32)
    est = imported.screen(torch.from_numpy(oT).cuda(), torch.from_numpy(u).cuda(), torch.from_numpy(Du).cuda())
    est = est.cpu().numpy()
    for i in range(len(q)):
        for s in range(oix.deg):
            if oix.adj[u[i], s] == orc.EMPTY:
                assert np.isnan(est[i, s])
                continue
            S = orc.S32(oT[i], oix.codes[u[i], s])
            ref = np.float32(orc.est32(Du[i], oix.a[u[i], s], oix.c[u[i], s], S))
            assert est[i, s] == ref


def test_edge_inference_information(orc, cfg1_oracle_index, imported):
    """codes (argmax per subspace) bit-exact; a, c, e2 equal up to one rounding of an fp64 value."""
    oix = cfg1_oracle_index
    codes, a, c, e2 = imported.edge_info(100, 400)
    assert np.array_equal(codes, oix.codes[100:400])
    for got, ref in ((a, oix.a[100:400]), (c, oix.c[100:400]), (e2, oix.e2[100:400])):
        assert np.allclose(got, ref, rtol=2e-7, atol=0)
        assert (got == ref).mean() >= 0.999


@pytest.mark.parametrize("efS", [10, 32, 64, 200])
def test_search_parity_config1(orc, cfg1_small, cfg1_oracle_index, imported, efS):
    w, base, q, gt, gtk = cfg1_small
    imported.reset_counters()
    gi, gd, oc = _assert_search_parity(imported, cfg1_oracle_index, q, w.K, efS, gt)
    gc = imported.counters()
    # the traversal itself agrees: same numbers of expanded nodes, tests, passes, exact distances
    for k_g, k_o in (("hops", "hops"), ("passes", "passes"), ("exact", "exact"),
                     ("rounds", "rounds"), ("rf_overflow", "rf_over"), ("rt_overflow", "rt_over")):
        assert abs(gc[k_g] - oc[k_o]) <= 0.002 * max(1, oc[k_o]), (k_g, gc[k_g], oc[k_o])
    _check_tests_counter(imported, q, w.K, efS, gc, oc)


def test_search_is_deterministic(cfg1_small, imported):
    w, base, q, gt, gtk = cfg1_small
    qd = torch.from_numpy(q).cuda()
    a = imported.search(qd, w.K, 64)
    b = imported.search(qd, w.K, 64)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_more_queries_than_resident_waves(orc, cfg1_small, cfg1_oracle_index, imported):
    """A batch larger than the number of resident waves is taken in the library's own order (projections onto the
    batch's direction of largest spread): the answers are those of the batch taken as numbered, bit for bit, and the
    oracle's; the counters do not change either."""
    from paper_2603_06660_amd import FLAG_KEEP_QUERY_ORDER
    w, base, q, gt, gtk = cfg1_small
    rng = np.random.default_rng(17)
    many = wl.make(wl.workload(1, n=3000, nq=9000), "query")
    many = many[rng.permutation(len(many))]
    qd = torch.from_numpy(many).cuda()
    imported.reset_counters()
    a = imported.search(qd, w.K, 48)
    ca = imported.counters()
    imported.set_search_options(0, FLAG_KEEP_QUERY_ORDER)
    try:
        imported.reset_counters()
        b = imported.search(qd, w.K, 48)
        cb = imported.counters()
    finally:
        imported.set_search_options(0, 0)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    for k in ("queries", "hops", "tests", "passes", "exact", "rounds"):
        assert ca[k] == cb[k], k
    oi, od, _ = cfg1_oracle_index.search(many[:300], w.K, 48)
    assert (a[0][:300].cpu().numpy() == oi).mean() >= 0.999


def test_seen_set_spill_path(orc, cfg1_small, cfg1_oracle_index, imported):
    """A 64-slot LDS seen set overflows at once: the HBM bitmap must keep the search exact."""
    w, base, q, gt, gtk = cfg1_small
    imported.set_seen_capacity_log2(6)
    try:
        imported.reset_counters()
        _assert_search_parity(imported, cfg1_oracle_index, q, w.K, 64, gt)
        assert imported.counters()["seen_spills"] > 0
        # and a second batch on the same waves starts from clean bitmaps
        _assert_search_parity(imported, cfg1_oracle_index, q[::-1].copy(), w.K, 64)
    finally:
        imported.set_seen_capacity_log2(0)


def test_large_k_two_entries_per_lane(orc, cfg1_small, cfg1_oracle_index, imported):
    """K = 100 -> b = 100: W and R_L span two register slots per lane."""
    w, base, q, gt, gtk = cfg1_small
    gt100, _ = wl.brute_force(base, q, 100)
    _assert_search_parity(imported, cfg1_oracle_index, q[:80], 100, 256, gt100[:80])
    _assert_search_parity(imported, cfg1_oracle_index, q[:40], 50, 128)


@pytest.mark.parametrize("K,efS,b", [(200, 400, 0), (129, 129, 0), (500, 700, 0), (1000, 1000, 0), (1000, 2500, 0),
                                     (10, 512, 512), (10, 900, 300), (64, 1024, 1024)])
def test_large_working_sets(orc, cfg1_small, cfg1_oracle_index, imported, K, efS, b):
    """Retrieval sizes up to K = 1000 (Sec. 5, demand D5): W and R_L take 4, 8 or 16 register slots per
    lane and round ends sort up to 2b keys with the bitonic network; b = efS is the single-pool mode."""
    w, base, q, gt, gtk = cfg1_small
    gtK, _ = wl.brute_force(base, q[:48], K, w.metric)
    try:
        imported.set_search_options(search_b=b, flags=0)
        imported.reset_counters()
        gi, gd, oc = _assert_search_parity(imported, cfg1_oracle_index, q[:48], K, efS, gtK, b=b)
        gc = imported.counters()
        for k_g, k_o in (("hops", "hops"), ("passes", "passes"), ("exact", "exact"),
                         ("rounds", "rounds"), ("rf_overflow", "rf_over"), ("rt_overflow", "rt_over")):
            assert gc[k_g] == oc[k_o], (k_g, gc[k_g], oc[k_o])
        _check_tests_counter(imported, q[:48], K, efS, gc, oc, search_b=b)
    finally:
        imported.set_search_options(0, 0)


def test_working_set_override_and_no_prt(orc, cfg1_small, cfg1_oracle_index, imported):
    """search_b = efS (one pool, one round) and the test switched off: textbook best-first search."""
    w, base, q, gt, gtk = cfg1_small
    from paper_2603_06660_amd import FLAG_NO_PRT
    try:
        imported.set_search_options(search_b=48, flags=0)
        _assert_search_parity(imported, cfg1_oracle_index, q, 10, 48, gt, b=48)
        imported.set_search_options(search_b=48, flags=FLAG_NO_PRT)
        qd = torch.from_numpy(q).cuda()
        gi, gd = imported.search(qd, 10, 48)
        oi, od, _ = cfg1_oracle_index.search(q, 10, 48, b=48, flags=orc.NO_PRT)
        assert (gi.cpu().numpy() == oi).mean() >= 0.999
    finally:
        imported.set_search_options(0, 0)


def test_edge_cases(orc):
    PagIndex = _gpu()
    from paper_2603_06660_amd import PagError
    rng = np.random.default_rng(12)
    # tiny index: fewer nodes than the working set; K slots beyond the reachable nodes are (-1, inf)
    base = rng.standard_normal((7, 16)).astype(np.float32)
    oix = orc.OracleIndex.build(base, wl.L2, deg=4, P=2, efC=20, seed=2)
    gix = _import(PagIndex, oix)
    q = rng.standard_normal((5, 16)).astype(np.float32)
    gi, gd, _ = _assert_search_parity(gix, oix, q, 7, 30)
    assert (gi >= 0).all()          # 7 nodes, all reachable from the entry list
    with pytest.raises(PagError):
        gix.search(torch.from_numpy(q).cuda(), 8, 30)            # K > n
    with pytest.raises(PagError):
        gix.search(torch.from_numpy(q).cuda(), 0, 30)            # K == 0
    ids, dists = gix.search(torch.empty((0, 16), device="cuda"), 3, 10)   # empty batch
    assert ids.shape == (0, 3)
    # efS below b -> one round; ragged d (not a multiple of 256), odd degree
    base = rng.standard_normal((500, 72)).astype(np.float32)
    oix = orc.OracleIndex.build(base, wl.L2, deg=11, P=9, efC=40, seed=3)
    gix = _import(PagIndex, oix)
    q = rng.standard_normal((33, 72)).astype(np.float32)
    _assert_search_parity(gix, oix, q, 10, 3)
    _assert_search_parity(gix, oix, q, 10, 57)
    with pytest.raises(PagError):
        PagIndex.build(torch.zeros((10, 30), device="cuda"), num_subspaces=4)      # d % P != 0
    # imported graphs are validated: ids in range, no neighbour listed twice, distinct entry ids
    for breakage in ("range", "twice", "entry"):
        adj, entry = oix.adj.copy(), oix.entry.copy()
        if breakage == "range":
            adj[3, 0] = 500
        elif breakage == "twice":
            adj[3, 1] = adj[3, 0]
        else:
            entry[1] = entry[0]
        with pytest.raises(PagError):
            PagIndex.from_arrays(oix.vec, adj, oix.a, oix.c, oix.e2, oix.codes, oix.rot, oix.cb, entry, metric="l2")


def test_unreachable_nodes_and_duplicate_vectors(orc):
    """Degenerate inputs.  (a) A graph of two components with every entry node in the first: the second
    component is never reached and the result slots beyond the first component hold (-1, +inf).
    (b) A base set whose last quarter repeats its first quarter (zero-length edges: a = c = 0, Sec. 3.1's
    angles are undefined there; equal keys are ordered by id): GPU build, export, oracle-validated
    inference information, search parity."""
    PagIndex = _gpu()
    from paper_2603_06660_amd import FLAG_NO_PRT
    rng = np.random.default_rng(77)
    n, d, deg, P = 40, 16, 4, 2
    vec = rng.standard_normal((n, d)).astype(np.float32)
    adj = np.full((n, deg), orc.EMPTY, np.uint32)
    for i in range(n):
        comp, k = divmod(i, 20)
        adj[i] = [comp * 20 + (k + s) % 20 for s in (1, 2, 19, 18)]
    z = lambda *shape: np.zeros(shape, np.float32)
    oix = orc.OracleIndex(vec, adj, z(n, deg), z(n, deg), z(n, deg), np.zeros((n, deg, P), np.uint8),
                          np.eye(d, dtype=np.float32), orc.make_codebooks(d, P, 5), np.arange(10, dtype=np.uint32))
    codes, a, c, e2 = oix.recompute_edge_info()
    oix.codes[:], oix.a[:], oix.c[:], oix.e2[:] = codes, a, c, e2
    gix = _import(PagIndex, oix)
    q = rng.standard_normal((9, d)).astype(np.float32)
    for flags in (0, FLAG_NO_PRT):
        gix.set_search_options(0, flags)
        qd = torch.from_numpy(q).cuda()
        gi, gd = gix.search(qd, 30, 90)
        gi, gd = gi.cpu().numpy(), gd.cpu().numpy()
        oi, od, _ = oix.search(q, 30, 90, flags=orc.NO_PRT if flags else 0)
        assert np.array_equal(gi, oi)
        assert np.all(gi[:, 20:] == -1) and np.all(np.isinf(gd[:, 20:])) and np.all(gi < 20)
        if flags:
            assert np.all(gi[:, :20] >= 0)                  # without the test the whole component is visited
            assert np.array_equal(np.sort(gi[:, :20], axis=1), np.tile(np.arange(20), (9, 1)))
    # (b) duplicates
    base = rng.standard_normal((2000, 32)).astype(np.float32)
    base[1500:] = base[:500]                               # far apart in id: a twin is in the graph when its pair is inserted
    gix = PagIndex.build(torch.from_numpy(base).cuda(), metric="l2", max_degree=8, num_subspaces=4,
                         ef_construction=60, seed=4)
    ex = gix.export()
    oix = orc.OracleIndex(ex["vectors"], ex["adj"], ex["a"], ex["c"], ex["e2"], ex["codes"], ex["rotation"],
                          ex["codebooks"], ex["entry"], metric=ex["metric"])
    codes, a, c, e2 = oix.recompute_edge_info()
    zero = (ex["e2"] == 0) & (ex["adj"] != orc.EMPTY)
    assert zero.sum() > 100                                 # duplicates do link to each other
    assert np.array_equal(codes, ex["codes"])
    assert np.allclose(a, ex["a"], rtol=2e-7, atol=0) and np.allclose(c, ex["c"], rtol=2e-7, atol=0)
    assert np.all(ex["a"][zero] == 0) and np.all(ex["c"][zero] == 0)
    q = (base[0:400:5] + 0.01 * rng.standard_normal((80, 32))).astype(np.float32)   # near duplicated points
    gi, gd, _ = _assert_search_parity(gix, oix, q, 10, 64)
    pair = gd[:, 0] == gd[:, 1]
    assert pair.mean() >= 0.3 and np.array_equal(gi[pair, 0] + 1500, gi[pair, 1])    # a duplicated pair: smaller id first


def test_cosine_and_ip(orc):
    PagIndex = _gpu()
    w = wl.workload(2, n=4000, nq=100)
    w = w.__class__(**{**w.__dict__, "d": 256, "P": 16})
    base, q = wl.make(w, "base"), wl.make(w, "query")
    oix = orc.OracleIndex.build(base, wl.IP, deg=16, P=16, efC=64, seed=5)
    gix = _import(PagIndex, oix)
    gt, _ = wl.brute_force(base, q, 10, wl.IP)
    _assert_search_parity(gix, oix, q, 10, 64, gt)
    oixc = orc.OracleIndex(oix.vec, oix.adj, oix.a, oix.c, oix.e2, oix.codes, oix.rot, oix.cb, oix.entry, metric=wl.COS)
    gixc = _import(PagIndex, oixc)
    _assert_search_parity(gixc, oixc, (2.5 * q).astype(np.float32), 10, 64, gt)


def test_traffic_diagnostics_leave_the_index_usable(orc, cfg1_small, cfg1_oracle_index, imported):
    """The roofline diagnostics (row reads in order / scattered, whole-hop traffic with seen-set writes) return
    rates and leave the per-wave seen-set workspaces clean: searches afterwards still match the oracle."""
    w, base, q, gt, gtk = cfg1_small
    for mode in (0, 1, 2):
        assert imported.measure_row_reads(20000, mode) > 0.0
    imported.set_seen_capacity_log2(6)           # force the bitmap level so that leftovers would show
    try:
        _assert_search_parity(imported, cfg1_oracle_index, q, w.K, 64, gt)
    finally:
        imported.set_seen_capacity_log2(0)
