"""Index construction and online insertion on the GPU against the oracle, element by element (Alg. 1;
Eq. 1; Eq. 5; Sec. 4.1), through the C ABI.

Both sides are given the same vectors, the same transform and codebooks and the same insertion order, and
must produce the same graph slot by slot: out-neighbour ids in the same slots, the same 4-bit codes, and
per-edge scalars equal up to one rounding of an fp64 sum.  Three settings:
  * one node after another (insert_subbatch = 1): Alg. 1 as printed; the oracle side is its sequential
    construction with the PES buffer of a node verified right after its insertion;
  * the library's default batches: the oracle side is its batch-synchronous construction with the same
    batch schedule;
  * pag_insert into an existing index, against the oracle continuing its own index.
What this compares, kernel by kernel: the indexing-mode search (R_L of capacity efC, b = min(efC, 100), PES
screening into H(v)), RobustPrune, the reverse-edge pass, PES verification, the inference information.
The lists R_L and H(v) themselves are compared through pag_insertion_candidates.

Where two keys are exactly equal the order is by node id; the library's ids are the caller's row numbers and
the oracle's are insertion positions, so data with exact ties (duplicates) is kept out of these cases.
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
    load_library()
    return PagIndex


def _data(cfg, n, d=None, P=None, deg=None):
    w = wl.workload(cfg, n=n, nq=64)
    over = {k: v for k, v in (("d", d), ("P", P), ("deg", deg)) if v is not None}
    w = w.__class__(**{**w.__dict__, **over})
    return w, wl.make(w, "base"), wl.make(w, "query")


def _relabel(ex, order, empty):
    """The exported index with nodes renamed to their insertion positions: node order[i] becomes i."""
    n = len(order)
    pos = np.empty(n, np.int64)
    pos[order] = np.arange(n)
    adj = ex["adj"][order].astype(np.int64)
    used = adj != empty
    adj[used] = pos[adj[used]]
    out = {k: ex[k][order] for k in ("vectors", "a", "c", "e2", "codes")}
    out["adj"] = adj.astype(np.uint32)
    return out


def _assert_same_index(got, oix, what):
    """got: arrays of the GPU-built index in the oracle's labelling."""
    n = oix.n
    same_rows = (got["adj"][:n] == oix.adj).all(axis=1)
    assert same_rows.all(), "%s: %d of %d adjacency rows differ, first at node %d" % (
        what, (~same_rows).sum(), n, int(np.argmin(same_rows)))
    assert np.array_equal(got["codes"][:n], oix.codes)
    for k in ("a", "c", "e2"):
        assert np.allclose(got[k][:n], getattr(oix, k), rtol=2e-7, atol=0), k
        assert (got[k][:n] == getattr(oix, k)).mean() >= 0.999, k


def _oracle_on(orc, ex, order, base, check_rotation=True, **kw):
    """The oracle's construction over the index's rotated vectors taken in insertion order.  The vectors are
    the exported ones, checked first against the oracle's own rotation of the raw data (the two agree in all
    but a few last bits; construction is chaotic in those, so both sides must start from the same values)."""
    vec = ex["vectors"][order]
    if check_rotation:
        raw = base[order[:200]]
        if ex["metric"] == wl.COS:
            r64 = raw.astype(np.float64)      # x / ||x|| in fp64, rounded once: the oracle's normalisation
            raw = (r64 / np.sqrt((r64 * r64).sum(axis=1, keepdims=True))).astype(np.float32)
        ref = np.stack([orc.rotate(ex["rotation"], x) for x in raw])
        assert (ref == vec[:200]).mean() >= 0.999 and np.allclose(ref, vec[:200], rtol=1e-5, atol=1e-6)
    return orc.OracleIndex.build(vec, wl.L2, rot=np.eye(vec.shape[1], dtype=np.float32), cb=ex["codebooks"], **kw)


def _signed_permutation(d, seed):
    """An orthogonal transform whose products are exact in floating point: both sides then hold bit-identical
    rotated vectors without exchanging them."""
    rng = np.random.default_rng(seed)
    rot = np.zeros((d, d), np.float32)
    rot[np.arange(d), rng.permutation(d)] = rng.choice(np.array([-1.0, 1.0], np.float32), d)
    return rot


SHAPES = [
    # cfg, n, d, P, deg, metric, efC
    (1, 900, 128, 16, 32, "l2", 64),
    (2, 700, 192, 64, 48, "ip", 250),       # three rounds of b = 100 per insertion
]


@pytest.mark.parametrize("cfg,n,d,P,deg,metric,efC", SHAPES)
@pytest.mark.parametrize("pes", [False, True])
def test_one_node_after_another(orc, cfg, n, d, P, deg, metric, efC, pes):
    """insert_subbatch = 1 in the given order: the paper's sequential construction."""
    PagIndex = _gpu()
    from paper_2603_06660_amd import FLAG_KEEP_ORDER, FLAG_NO_PES
    w, base, q = _data(cfg, n, d, P, deg)
    gix = PagIndex.build(torch.from_numpy(base).cuda(), metric=metric, max_degree=deg, num_subspaces=P,
                         ef_construction=efC, insert_subbatch=1, seed=41,
                         flags=FLAG_KEEP_ORDER | (0 if pes else FLAG_NO_PES))
    ex = gix.export()
    assert ex["entry"].tolist() == list(range(min(n, 1024)))
    assert gix.counters()["relinked_batches"] == 0
    order = np.arange(n)
    oix = _oracle_on(orc, ex, order, base, deg=deg, P=P, efC=efC, pes=pes, pes_every=1)
    _assert_same_index(ex, oix, "sequential")
    if pes:
        assert oix.pes_edges_added > 0


def test_one_node_after_another_in_shuffled_order(orc):
    """The default seeded shuffle with insert_subbatch = 1: the exported entry list is the insertion order
    (n <= 1024), the oracle inserts in that order, and the graphs agree after renaming."""
    PagIndex = _gpu()
    n, deg, P, efC = 800, 32, 16, 100
    w, base, q = _data(1, n)
    gix = PagIndex.build(torch.from_numpy(base).cuda(), metric="l2", max_degree=deg, num_subspaces=P,
                         ef_construction=efC, insert_subbatch=1, seed=43)
    ex = gix.export()
    order = ex["entry"].astype(np.int64)
    assert sorted(order.tolist()) == list(range(n)) and order.tolist() != list(range(n))
    oix = _oracle_on(orc, ex, order, base, deg=deg, P=P, efC=efC, pes=True, pes_every=1)
    _assert_same_index(_relabel(ex, order, orc.EMPTY), oix, "shuffled sequential")


@pytest.mark.parametrize("cfg,n,d,P,deg,metric,efC,subbatch", [
    (1, 3000, 128, 16, 32, "l2", 100, 0),        # the library's own schedule: batches of up to half the graph, at most 1024
    (1, 2500, 128, 16, 32, "l2", 64, 160),
    (3, 1500, 256, 32, 48, "ip", 220, 0),
    (1, 30000, 128, 16, 32, "l2", 100, 0),       # 35 batches, the last ones of 1024 nodes
    (2, 12000, 256, 32, 32, "ip", 300, 0),       # three rounds per insertion, long-search seen set
])
def test_default_batches(orc, cfg, n, d, P, deg, metric, efC, subbatch):
    """The batch-synchronous construction, batch schedule and all, against the oracle's."""
    PagIndex = _gpu()
    from paper_2603_06660_amd import FLAG_KEEP_ORDER
    w, base, q = _data(cfg, n, d, P, deg)
    gix = PagIndex.build(torch.from_numpy(base).cuda(), metric=metric, max_degree=deg, num_subspaces=P,
                         ef_construction=efC, insert_subbatch=subbatch, seed=47, flags=FLAG_KEEP_ORDER)
    ex = gix.export()
    assert gix.counters()["relinked_batches"] == 0
    max_batch = subbatch if subbatch else min(16384, max(1024, n // 50))
    oix = _oracle_on(orc, ex, np.arange(n), base, deg=deg, P=P, efC=efC, pes=True, max_batch=min(max_batch, n))
    assert oix.batches >= 5
    _assert_same_index(ex, oix, "batched")
    # and both answer queries alike
    gi, gd = gix.search(torch.from_numpy(q).cuda(), 10, 64)
    view = orc.OracleIndex(ex["vectors"], oix.adj, oix.a, oix.c, oix.e2, oix.codes, ex["rotation"], ex["codebooks"],
                           ex["entry"], metric=ex["metric"])
    oi, od, _ = view.search(q, 10, 64)
    assert (gi.cpu().numpy() == oi).mean() >= 0.999


@pytest.mark.parametrize("subbatch,metric", [(1, "l2"), (0, "l2"), (0, "cos")])
def test_insert_continues_the_oracle_index(orc, subbatch, metric):
    """Online insertion (Sec. 4.1) with nothing flowing from the library to the oracle: the oracle builds an
    index on the first block of raw vectors and inserts two more blocks; the library imports the oracle's
    first index and gets the same two blocks through pag_insert (normalising and rotating them itself).  The
    transform is a signed permutation, so both sides hold bit-identical vectors."""
    PagIndex = _gpu()
    from paper_2603_06660_amd import FLAG_KEEP_ORDER
    n0, n1, n2, deg, P, efC = 600, 900, 1400, 32, 16, 80
    w, base, q = _data(1, n2)
    m = wl.COS if metric == "cos" else wl.L2
    rot = _signed_permutation(w.d, 3)
    kw = dict(pes=True, pes_every=1) if subbatch else dict(pes=True)
    # the library sizes the batches of a call from the size the index will have after the call
    mb = (lambda lo, hi: {}) if subbatch else (lambda lo, hi: dict(max_batch=min(hi - lo, min(16384, max(1024, hi // 50)))))
    oix = orc.OracleIndex.build(base[:n0], m, deg=deg, P=P, efC=efC, rot=rot, seed=7, **kw, **mb(0, n0))
    gix = PagIndex.from_arrays(oix.vec, oix.adj, oix.a, oix.c, oix.e2, oix.codes, oix.rot, oix.cb, oix.entry,
                               metric=metric, ef_construction=efC, capacity=n2, flags=FLAG_KEEP_ORDER,
                               insert_subbatch=subbatch)
    bd = torch.from_numpy(base).cuda()
    gix.insert(bd[n0:n1].contiguous())
    gix.insert(bd[n1:].contiguous())
    oix.insert(base[n0:n1], efC=efC, **kw, **mb(n0, n1))
    oix.insert(base[n1:], efC=efC, **kw, **mb(n1, n2))
    ex = gix.export()
    assert gix.counters()["relinked_batches"] == 0
    assert np.array_equal(ex["entry"], oix.entry) and len(oix.entry) == 1024
    assert np.array_equal(ex["vectors"], oix.vec)
    _assert_same_index(ex, oix, "insert")
    assert oix.pes_edges_added > 0


def test_insertion_candidates(orc, cfg1_small, cfg1_oracle_index):
    """The search of one insertion on an oracle-built index: R_L (capacity efC, several rounds of b = 100)
    and the PES buffer H(v), element by element, for vectors that are not in the index."""
    PagIndex = _gpu()
    w, base, q, gt, gtk = cfg1_small
    oix = cfg1_oracle_index
    for efC in (40, 100, 250):
        gix = PagIndex.from_arrays(oix.vec, oix.adj, oix.a, oix.c, oix.e2, oix.codes, oix.rot, oix.cb, oix.entry,
                                   metric="l2", ef_construction=efC)
        ci, ck, cn, hi, hk, hn = gix.insertion_candidates(torch.from_numpy(q[:60]).cuda(), efC)
        qr, _ = oix.prepare(q[:60])
        n_pes = 0
        for i in range(60):
            oi, ok, ohi, ohk, _ = oix.index_search(qr[i], efC)
            assert cn[i] == len(oi) and ci[i, :cn[i]].tolist() == oi.tolist(), (efC, i)
            assert np.all(np.abs(ck[i, :cn[i]] - ok) <= 1e-5 * ok)
            assert hn[i] == len(ohi) and hi[i, :hn[i]].tolist() == ohi.tolist(), (efC, i)
            assert np.all(np.abs(hk[i, :hn[i]] - ohk) <= 1e-5 * ohk)
            assert np.all(ci[i, cn[i]:] == orc.EMPTY) and np.all(hi[i, hn[i]:] == orc.EMPTY)
            n_pes += len(ohi)
        assert n_pes > 0
        gix.close()


def test_crowded_insert(orc):
    """pag_insert of vectors that all lie where the index has none yet (the points farthest along one
    direction, held out of the build and inserted in order along it): the batch is found to crowd a region
    of its own and is linked a second time, in eight parts.  Density rule, second pass and all, the graph
    must be the oracle's."""
    PagIndex = _gpu()
    from paper_2603_06660_amd import FLAG_KEEP_ORDER
    w = wl.workload(1, n=6000, nq=64)
    base = wl.make(w, "base")
    u = base[0] - base.mean(0)
    proj = base @ (u / np.linalg.norm(u))
    new = proj > np.quantile(proj, 0.88)
    old_rows, new_rows = base[~new], base[new][np.argsort(proj[new], kind="stable")]
    deg, P, efC = 32, 16, 64
    rot = _signed_permutation(w.d, 5)
    n_all = len(base)
    oix = orc.OracleIndex.build(old_rows, wl.L2, deg=deg, P=P, efC=efC, rot=rot, seed=7, pes=True,
                                max_batch=min(len(old_rows), 1024))
    assert oix.relinked_batches == 0
    gix = PagIndex.from_arrays(oix.vec, oix.adj, oix.a, oix.c, oix.e2, oix.codes, oix.rot, oix.cb, oix.entry,
                               metric="l2", ef_construction=efC, capacity=n_all, flags=FLAG_KEEP_ORDER)
    gix.insert(torch.from_numpy(new_rows).cuda())
    oix.insert(new_rows, efC=efC, pes=True, max_batch=min(len(new_rows), 1024))
    assert oix.relinked_batches == 1 and gix.counters()["relinked_batches"] == 1
    ex = gix.export()
    assert np.array_equal(ex["vectors"], oix.vec)
    _assert_same_index(ex, oix, "crowded insert")


@pytest.mark.parametrize("n,d,P,deg,efC,subbatch", [
    (1, 32, 4, 8, 20, 0),          # a single node
    (2, 32, 4, 8, 20, 1),
    (7, 32, 4, 8, 20, 0),          # fewer nodes than the degree and than the initial set
    (21, 32, 4, 8, 20, 1),         # one node more than the initial set
    (150, 64, 8, 64, 120, 0),      # the largest degree; the initial set (100 nodes) is most of the index
    (260, 3072, 64, 16, 60, 0),    # the longest rows and most subspaces this build takes
    (300, 72, 9, 11, 40, 0),       # ragged: 72 = 9 x 8, odd degree
])
def test_small_and_extreme_shapes(orc, n, d, P, deg, efC, subbatch):
    """Construction at the edges of what the library accepts, against the oracle (sequential or in the
    default batches, PES on)."""
    PagIndex = _gpu()
    from paper_2603_06660_amd import FLAG_KEEP_ORDER
    rng = np.random.default_rng(1000 * n + d)
    base = rng.standard_normal((n, d)).astype(np.float32)
    gix = PagIndex.build(torch.from_numpy(base).cuda(), metric="l2", max_degree=deg, num_subspaces=P,
                         ef_construction=efC, insert_subbatch=subbatch, seed=61, flags=FLAG_KEEP_ORDER)
    ex = gix.export()
    kw = dict(pes_every=1) if subbatch else dict(max_batch=min(n, 1024))
    oix = _oracle_on(orc, ex, np.arange(n), base, deg=deg, P=P, efC=efC, pes=True, **kw)
    _assert_same_index(ex, oix, "shape n=%d d=%d" % (n, d))
    assert ex["entry"].tolist() == list(range(n))


@pytest.mark.parametrize("d,P,deg,efC,metric,half", [
    (96, 12, 40, 90, "l2", False),       # one 16-byte chunk per lane, half the lanes idle; more neighbours kept than LDS rows
    (384, 16, 32, 80, "ip", False),      # two chunks per lane
    (640, 20, 24, 70, "l2", False),      # three, ragged
    (1024, 32, 48, 110, "cos", False),   # four
    (1280, 40, 36, 60, "l2", False),     # five of six
    (2048, 64, 32, 60, "ip", False),     # eight
    (2560, 40, 20, 50, "l2", False),     # ten of twelve
    (768, 32, 32, 100, "l2", True),      # the 16-bit vector store
])
def test_every_row_length_class(orc, d, P, deg, efC, metric, half):
    """Construction in the default batches at one row length per instantiation of the pruning kernel (16-byte
    chunks per lane: 1, 2, 3, 4, 6, 8, 12), on isotropic data, where RobustPrune keeps more neighbours than the
    kernel holds in LDS: both of its paths (kept rows in LDS, kept rows from memory) decide as the oracle does."""
    PagIndex = _gpu()
    from paper_2603_06660_amd import FLAG_FP16_VECTORS, FLAG_KEEP_ORDER
    n = 520
    rng = np.random.default_rng(7000 + d)
    base = rng.standard_normal((n, d)).astype(np.float32)
    if metric == "ip":
        base /= np.linalg.norm(base, axis=1, keepdims=True)
    gix = PagIndex.build(torch.from_numpy(base).cuda(), metric=metric, max_degree=deg, num_subspaces=P,
                         ef_construction=efC, seed=73, flags=FLAG_KEEP_ORDER | (FLAG_FP16_VECTORS if half else 0))
    ex = gix.export()
    # with the 16-bit store the index is the rounded data: the oracle starts from the exported values as they are
    oix = _oracle_on(orc, ex, np.arange(n), base, check_rotation=not half, deg=deg, P=P, efC=efC, pes=True,
                     max_batch=min(n, 1024))
    _assert_same_index(ex, oix, "row length d=%d" % d)
    kept = (ex["adj"] != orc.EMPTY).sum(axis=1)
    assert kept.max() > 16 or deg <= 16        # beyond the rows held in LDS at every length


def test_duplicated_vectors(orc):
    """Every vector of the second half repeats one of the first: zero-length edges, exact ties between
    distances everywhere (ordered by id on both sides, the ids being the same: rows are linked in the order
    given), RobustPrune's `<=` deciding between equals.  Sequential and batched."""
    PagIndex = _gpu()
    from paper_2603_06660_amd import FLAG_KEEP_ORDER
    rng = np.random.default_rng(99)
    half = rng.standard_normal((400, 64)).astype(np.float32)
    base = np.concatenate([half, half[rng.permutation(400)]])
    for subbatch in (1, 0):
        gix = PagIndex.build(torch.from_numpy(base).cuda(), metric="l2", max_degree=16, num_subspaces=8,
                             ef_construction=64, insert_subbatch=subbatch, seed=67, flags=FLAG_KEEP_ORDER)
        ex = gix.export()
        kw = dict(pes_every=1) if subbatch else dict(max_batch=800)
        oix = _oracle_on(orc, ex, np.arange(800), base, deg=16, P=8, efC=64, pes=True, **kw)
        _assert_same_index(ex, oix, "duplicates")
        assert ((ex["e2"] == 0) & (ex["adj"] != orc.EMPTY)).sum() > 100


@pytest.mark.parametrize("subbatch,metric", [(1, "l2"), (0, "l2"), (0, "cos")])
def test_build_from_raw_vectors(orc, subbatch, metric):
    """pag_build with nothing computed by the library reaching the oracle: the transform is a signed permutation
    (PAG_FLAG_PERMUTATION_TRANSFORM), so the oracle, given the raw vectors and the library's random draws (Q and the
    codebooks), holds bit-identical rotated vectors of its own making; initial nodes, entry list, every batch and the
    PES verification must then give the same index."""
    PagIndex = _gpu()
    from paper_2603_06660_amd import FLAG_KEEP_ORDER, FLAG_PERMUTATION_TRANSFORM
    n, deg, P, efC = 2200, 32, 16, 90
    w, base, q = _data(1, n)
    gix = PagIndex.build(torch.from_numpy(base).cuda(), metric=metric, max_degree=deg, num_subspaces=P, ef_construction=efC,
                         insert_subbatch=subbatch, seed=71, flags=FLAG_KEEP_ORDER | FLAG_PERMUTATION_TRANSFORM)
    ex = gix.export()
    rot = ex["rotation"]
    assert np.array_equal(np.abs(rot).sum(0), np.ones(w.d)) and np.array_equal(np.abs(rot).sum(1), np.ones(w.d))
    kw = dict(pes_every=1) if subbatch else dict(max_batch=min(n, 1024))
    oix = orc.OracleIndex.build(base, wl.COS if metric == "cos" else wl.L2, deg=deg, P=P, efC=efC, rot=rot,
                                cb=ex["codebooks"], pes=True, **kw)
    assert np.array_equal(ex["vectors"], oix.vec)
    assert ex["entry"].tolist() == list(range(1024))
    _assert_same_index(ex, oix, "build from raw vectors")
