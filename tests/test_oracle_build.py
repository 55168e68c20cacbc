"""Pins for the oracle's index construction (Alg. 1): the initial nodes, the reverse-edge rule
(Sec. 2.1, Eq. 1), the PES screening inside the insertion search and the trimming of H(v)
(Sec. 3.4, Eq. 5), the verification of buffered candidates, whole insertions, and the
batch-synchronous construction.

The expected values of the planar cases live in tests/golden/alg1_hand_cases.txt, where each is
derived by hand from the rule it exercises.  The batch-synchronous construction is pinned to the
sequential one: with batches of one node it must give the same graph.
"""
import os

import numpy as np
import pytest

import pag_workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))


def _cases():
    cases, cur = {}, None
    for line in open(os.path.join(HERE, "golden", "alg1_hand_cases.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        if line.startswith("["):
            cur = {}
            cases[line.strip("[]")] = cur
            continue
        key, val = line.split(":", 1)
        cur[key.strip()] = val.strip()
    return cases


CASES = _cases()


def _axis_codebook(P, ds):
    cb = np.zeros((P, 16, ds), np.float32)
    for l in range(P):
        for k in range(ds):
            cb[l, 2 * k, k], cb[l, 2 * k + 1, k] = 1.0, -1.0
        cb[l, 2 * ds:] = cb[l, 0]
    return (cb / np.float32(np.sqrt(P))).astype(np.float32)


def _points(text):
    return np.array([[float(x) for x in p.split(",")] for p in text.split()], np.float32)


def _adjacency(text, n, deg, orc):
    adj = np.full((n, deg), orc.EMPTY, np.uint32)
    for item in (text or "").split():
        u, nb = item.split(":")
        for s, w in enumerate(nb.split(",")):
            if w != "-":
                adj[int(u), s] = int(w)
    return adj


def _index(orc, pts, adj, entry=None, cb=None):
    n, d = pts.shape
    deg = adj.shape[1]
    cb = _axis_codebook(1, d) if cb is None else cb
    P = cb.shape[0]
    ix = orc.OracleIndex(pts, adj, np.zeros((n, deg), np.float32), np.zeros((n, deg), np.float32),
                         np.zeros((n, deg), np.float32), np.zeros((n, deg, P), np.uint8), np.eye(d, dtype=np.float32),
                         cb, np.arange(n, dtype=np.uint32) if entry is None else np.array(entry, np.uint32))
    codes, a, c, e2 = ix.recompute_edge_info()
    ix.codes[:], ix.a[:], ix.c[:], ix.e2[:] = codes, a, c, e2
    return ix


def _assert_graph(orc, ix, text):
    want = _adjacency(text, ix.n, ix.deg, orc)
    assert ix.adj.tolist() == want.tolist()
    # whatever was written carries the inference information of its edge
    codes, a, c, e2 = ix.recompute_edge_info()
    assert np.array_equal(codes, ix.codes) and np.array_equal(a, ix.a)
    assert np.array_equal(c, ix.c) and np.array_equal(e2, ix.e2)


@pytest.mark.parametrize("name", [k for k in CASES if k.startswith(("reverse", "pes "))])
def test_reverse_edge_and_pes_verification(orc, name):
    case = CASES[name]
    pts = _points(case["points"])
    deg = int(case["deg"])
    ix = _index(orc, pts, _adjacency(case["adjacency"], len(pts), deg, orc))
    kind, u, v, duv = case["call"].split()
    assert orc.key(pts[int(u)], pts[int(v)]) == float(duv)
    if kind == "reverse":
        ix.reverse_edge(int(u), int(v), float(duv))
    else:
        assert ix.pes_edge(int(u), int(v), float(duv)) == int(case["returns"])
    _assert_graph(orc, ix, case["expect"])


@pytest.mark.parametrize("name", ["initial nodes", "initial nodes tie"])
def test_initial_nodes(orc, name):
    case = CASES[name]
    pts = _points(case["points"])
    ix = orc.OracleIndex.build(pts[:int(case["build"])], wl.L2, deg=int(case["deg"]), P=1, efC=int(case["efC"]),
                               rot=np.eye(2, dtype=np.float32), cb=_axis_codebook(1, 2), pes=False)
    _assert_graph(orc, ix, case["expect"])


@pytest.mark.parametrize("mode", ["sequential", "sequential, buffers verified per node", "batches of one", "insert"])
def test_two_insertions_traced_by_hand(orc, mode):
    case = CASES["two insertions"]
    pts = _points(case["points"])
    kw = dict(deg=int(case["deg"]), P=1, efC=int(case["efC"]), rot=np.eye(2, dtype=np.float32), cb=_axis_codebook(1, 2))
    first = orc.OracleIndex.build(pts[:5], wl.L2, pes=True, **kw)
    _assert_graph(orc, first, case["expect_after_first"])
    ci, ck, hi, hk, ctr = first.index_search(pts[5], kw["efC"])
    assert ci.tolist() == [int(x) for x in case["cand_ids"].split()]
    assert ck.tolist() == [float(x) for x in case["cand_keys"].split()]
    assert hi.tolist() == [int(x) for x in case["pes_ids"].split()]
    assert hk.tolist() == [float(x) for x in case["pes_keys"].split()]
    for k in ("hops", "tests", "passes", "exact"):
        assert ctr[k] == int(case[k]), k
    for pes in (False, True):
        if mode == "sequential":
            ix = orc.OracleIndex.build(pts, wl.L2, pes=pes, **kw)
        elif mode == "sequential, buffers verified per node":
            ix = orc.OracleIndex.build(pts, wl.L2, pes=pes, pes_every=1, **kw)
        elif mode == "batches of one":
            ix = orc.OracleIndex.build(pts, wl.L2, pes=pes, max_batch=1, **kw)
        else:
            ix = orc.OracleIndex.build(pts[:4], wl.L2, pes=pes, **kw)
            ix.insert(pts[4:5], efC=kw["efC"], pes=pes)
            ix.insert(pts[5:6], efC=kw["efC"], pes=pes)
        _assert_graph(orc, ix, case["expect" if pes else "expect_without_pes"])
        assert ix.pes_edges_added == (int(case["pes_added"]) if pes else 0)


@pytest.mark.parametrize("name", ["screening and trimming", "screening tie"])
def test_pes_screening_and_trimming_inside_the_search(orc, name):
    case = CASES[name]
    pts = _points(case["points"])
    deg = int(case["deg"])
    ix = _index(orc, pts, _adjacency(case["adjacency"], len(pts), deg, orc), entry=[int(x) for x in case["entries"].split()])
    ci, ck, hi, hk, ctr = ix.index_search(_points(case["search_point"])[0], int(case["efC"]))
    assert ci.tolist() == [int(x) for x in case["cand_ids"].split()]
    assert ck.tolist() == [float(x) for x in case["cand_keys"].split()]
    assert hi.tolist() == [int(x) for x in case["pes_ids"].split()]
    assert hk.tolist() == [float(x) for x in case["pes_keys"].split()]
    for k in ("hops", "tests", "passes", "exact"):
        assert ctr[k] == int(case[k]), k


@pytest.mark.parametrize("witness", [True, False])
def test_pes_screening_on_the_worked_example(orc, witness):
    """Eq. 5 on the hand-computed geometry of worked_example.txt: the neighbour whose estimate (7.2) lies
    below D_u = 10 is a witness against the edge u -> v; without it (estimate 40.8 only) u survives."""
    case = CASES["worked example with witness" if witness else "worked example without witness"]
    vec = np.array([[0, 0, 0, 0], [3, 1, 0, -2], [-3, -1, 0, 2]], np.float32)
    adj = np.full((3, 2), orc.EMPTY, np.uint32)
    adj[0] = [1, 2] if witness else [2, orc.EMPTY]
    ix = _index(orc, vec, adj, entry=[0], cb=_axis_codebook(2, 2))
    v = np.array([2, 2, 1, -1], np.float32)
    # the two statistics, from the printed definition (fp64): w is a witness (positive term), w' is not
    assert orc.stats(ix.cb, vec[0], vec[1], v, 0.0)["pes_term"] > 0 > orc.stats(ix.cb, vec[0], vec[2], v, 0.0)["pes_term"]
    ci, ck, hi, hk, _ = ix.index_search(v, 1)
    assert hi.tolist() == [int(x) for x in case["pes_ids"].split()]
    assert hk.tolist() == [float(x) for x in case["pes_keys"].split()]
    assert ci.tolist() == [int(x) for x in case["cand_ids"].split()]
    assert ck.tolist() == [float(x) for x in case["cand_keys"].split()]


def test_pes_screen_in_estimate_form_is_eq5(orc):
    """The screening inside the search uses min_i est_i > D_u.  Against Eq. 5 as printed (fp64, with
    square roots and divisions): over random triples the sign of cos(theta)/cos(beta) - delta is
    the sign of D_u - est, so "the maximum is negative" is "every estimate exceeds D_u"."""
    rng = np.random.default_rng(7)
    cb = orc.make_codebooks(16, 4, 3)
    agree = 0
    for _ in range(400):
        u, w, v = (rng.standard_normal(16).astype(np.float32) for _ in range(3))
        s = orc.stats(cb, u, w, v, 1.0)
        du = orc.sqdist64(u, v)
        if abs(s["pes_term"]) > 1e-9:
            assert (s["pes_term"] < 0) == (s["est"] > du)
            agree += 1
    assert agree >= 390


def test_batches_of_one_are_the_sequential_build(orc, cfg1_small):
    """The batch-synchronous construction with batches of one node is Alg. 1 as printed (one node after
    another), with and without the PES steps; larger batches give a different but equally good graph."""
    w, base, q, gt, gtk = cfg1_small
    kw = dict(deg=w.deg, P=w.P, efC=48, seed=17)
    n = 1200
    gt12, _ = wl.brute_force(base[:n], q, w.K)
    seq = orc.OracleIndex.build(base[:n], w.metric, pes=False, **kw)
    one = orc.OracleIndex.build(base[:n], w.metric, pes=False, max_batch=1, **kw)
    assert np.array_equal(seq.adj, one.adj) and np.array_equal(seq.codes, one.codes)
    assert np.array_equal(seq.a, one.a) and np.array_equal(seq.c, one.c) and np.array_equal(seq.e2, one.e2)
    seq = orc.OracleIndex.build(base[:n], w.metric, pes=True, pes_every=1, **kw)
    one = orc.OracleIndex.build(base[:n], w.metric, pes=True, max_batch=1, **kw)
    assert np.array_equal(seq.adj, one.adj) and seq.pes_edges_added == one.pes_edges_added > 0
    # insertion in two calls continues the same sequence
    two = orc.OracleIndex.build(base[:700], w.metric, pes=True, pes_every=1, **kw)
    two.insert(base[700:n], efC=48, pes=True, pes_every=1)
    assert np.array_equal(two.adj, seq.adj) and np.array_equal(two.entry, seq.entry)
    big = orc.OracleIndex.build(base[:n], w.metric, pes=True, max_batch=256, **kw)
    assert big.batches < 20 and not np.array_equal(big.adj, seq.adj)
    r_seq = wl.recall_at_k(seq.search(q, w.K, 32)[0], gt12)
    r_big = wl.recall_at_k(big.search(q, w.K, 32)[0], gt12)
    assert r_big >= r_seq - 0.04 and r_seq >= 0.9      # batches up to half the graph, on 1200 nodes
    # verifying the buffers only at the very end (Alg. 1's last loop) differs in a few slots, not in quality
    end = orc.OracleIndex.build(base[:n], w.metric, pes=True, **kw)
    assert 0 < (end.adj != seq.adj).mean() < 0.1
    assert abs(wl.recall_at_k(end.search(q, w.K, 32)[0], gt12) - r_seq) <= 0.02


def _held_out_region(n, frac=0.12):
    """cfg 1's mixture with the points farthest along one direction held out: (old rows, new rows sorted along
    that direction).  Inserting the new rows puts them where the index built on the old rows has no node."""
    w = wl.workload(1, n=n, nq=400)
    base, q = wl.make(w, "base"), wl.make(w, "query")
    u = base[0] - base.mean(0)
    proj = base @ (u / np.linalg.norm(u))
    cut = np.quantile(proj, 1.0 - frac)
    new = proj > cut
    return w, base[~new], base[new][np.argsort(proj[new], kind="stable")], q


def test_crowded_batch_is_linked_twice(orc):
    """Batch-synchronous insertion of vectors that all lie where the index has none yet: the batch's nodes do
    not see each other in the first pass; the density rule notices and links them a second time, after which
    queries that land in the new region are answered as well as by the sequential construction.  Ordinary
    builds never trigger the rule."""
    w, old, new, q = _held_out_region(4000)
    kw = dict(deg=w.deg, P=w.P, efC=64, seed=19)
    allv = np.concatenate([old, new])
    gt, _ = wl.brute_force(allv, q, w.K)
    near = gt[:, 0] >= len(old)
    assert near.sum() >= 20 and 300 <= len(new) <= 600
    seq = orc.OracleIndex.build(old, w.metric, pes=True, pes_every=1, **kw)
    seq.insert(new, efC=64, pes=True, pes_every=1)
    bat = orc.OracleIndex.build(old, w.metric, pes=True, max_batch=1024, **kw)
    assert bat.relinked_batches == 0                       # a mixed build: batch-mates are as dense as older nodes
    bat.insert(new, efC=64, pes=True, max_batch=len(new))
    assert bat.batches == 1 and bat.relinked_batches == 1
    once = orc.OracleIndex.build(old, w.metric, pes=True, max_batch=1024, **kw)
    once.insert(new, efC=64, pes=True, max_batch=len(new), relink=False)        # what the rule is worth
    r_seq = wl.recall_at_k(seq.search(q, w.K, 32)[0][near], gt[near])
    r_bat = wl.recall_at_k(bat.search(q, w.K, 32)[0][near], gt[near])
    r_once = wl.recall_at_k(once.search(q, w.K, 32)[0][near], gt[near])
    assert r_bat >= r_seq - 0.05 and r_seq >= 0.9 and r_once <= r_bat - 0.2, (r_seq, r_bat, r_once)
    # the relinked nodes link to each other: most of their out-neighbours are batch-mates
    adj_new = bat.adj[len(old):]
    used = adj_new != orc.EMPTY
    assert (adj_new[used] >= len(old)).mean() > 0.5
    # no node lists itself or a neighbour twice
    for v in range(len(old), bat.n):
        nb = bat.adj[v][bat.adj[v] != orc.EMPTY]
        assert v not in nb and len(set(nb.tolist())) == len(nb)
