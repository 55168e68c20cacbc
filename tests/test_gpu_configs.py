"""Search parity at the true shapes of the other workloads (d, K, degree, subspaces, metric, OOD
queries, online insertion) on reduced n with every query checked, and at the full size of every
workload (n, d, query-batch size as configured) on a sample of the queries.  Index: built by the GPU
library, exported, validated by the oracle, then searched by both sides."""
import dataclasses

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


def _oracle_view(orc, ex):
    return orc.OracleIndex(ex["vectors"], ex["adj"], ex["a"], ex["c"], ex["e2"], ex["codes"], ex["rotation"],
                           ex["codebooks"], ex["entry"], metric=ex["metric"])


def _parity(orc, gix, oix, q, K, efS, sample=None):
    gi, gd = gix.search(torch.from_numpy(q).cuda(), K, efS)
    gi, gd = gi.cpu().numpy(), gd.cpu().numpy()
    sel = slice(None) if sample is None else sample
    oi, od, oc = oix.search(q[sel], K, efS, threads=8)
    gi_s, gd_s = gi[sel], gd[sel]
    agree = (gi_s == oi).mean()
    assert agree >= 0.999, agree
    m = (gi_s == oi) & np.isfinite(od)
    assert np.all(np.abs(gd_s[m] - od[m]) <= 1e-5 * np.abs(od[m]))
    return gi, gd, oi


def _check_edge_info(orc, oix, ex, nodes):
    for lo in nodes:
        codes, a, c, e2 = oix.recompute_edge_info(lo, lo + 64)
        assert np.array_equal(codes, ex["codes"][lo:lo + 64])
        assert np.allclose(a, ex["a"][lo:lo + 64], rtol=2e-7, atol=0)
        assert np.allclose(c, ex["c"][lo:lo + 64], rtol=2e-7, atol=0)


@pytest.mark.parametrize("cfg,n,nq,efC,efS", [(3, 20000, 200, 128, 256), (4, 20000, 200, 100, 128),
                                              (5, 8000, 100, 100, 96)])
def test_other_workload_shapes(orc, cfg, n, nq, efC, efS):
    PagIndex = _gpu()
    w = wl.workload(cfg, n=n, nq=nq)
    base, q = wl.make(w, "base"), wl.make(w, "query")
    metric = {0: "l2", 1: "ip", 2: "cos"}[w.metric]
    gix = PagIndex.build(torch.from_numpy(base).cuda(), metric=metric, max_degree=w.deg, num_subspaces=w.P,
                         ef_construction=efC, seed=cfg)
    ex = gix.export()
    oix = _oracle_view(orc, ex)
    _check_edge_info(orc, oix, ex, (0, n // 2, n - 64))
    gt, _ = wl.brute_force(base, q, w.K, w.metric)
    gi, gd, oi = _parity(orc, gix, oix, q, w.K, efS)
    rg, ro = wl.recall_at_k(gi, gt), wl.recall_at_k(oi, gt)
    assert abs(rg - ro) <= 0.002
    assert rg >= 0.8, rg
    if cfg == 4:                       # second retrieval size of that workload
        _parity(orc, gix, oix, q, 50, 200)
    # reported keys: 1 - <q, x> on unit vectors
    qn = q / np.linalg.norm(q, axis=1, keepdims=True)
    bn = base / np.linalg.norm(base, axis=1, keepdims=True)
    ip = np.einsum("qkd,qd->qk", bn[gi].astype(np.float64), qn.astype(np.float64))
    assert np.allclose(gd, 1.0 - ip, atol=5e-6)


@pytest.mark.parametrize("cfg,n,K,efS,fp16", [(3, 20000, 300, 600, False), (4, 12000, 200, 400, True),
                                               (5, 8000, 1000, 1000, False)])
def test_large_retrieval_sizes_at_workload_shapes(orc, cfg, n, K, efS, fp16):
    """K = 200 .. 1000 (4, 8, 16 register slots per lane, rings in HBM) at the other workloads' row
    lengths, degrees and code widths, on an fp32 and on a 16-bit store."""
    PagIndex = _gpu()
    from paper_2603_06660_amd import FLAG_FP16_VECTORS
    w = wl.workload(cfg, n=n, nq=64)
    base, q = wl.make(w, "base"), wl.make(w, "query")
    metric = {0: "l2", 1: "ip", 2: "cos"}[w.metric]
    gix = PagIndex.build(torch.from_numpy(base).cuda(), metric=metric, max_degree=w.deg, num_subspaces=w.P,
                         ef_construction=100, seed=cfg, flags=FLAG_FP16_VECTORS if fp16 else 0)
    ex = gix.export()
    oix = _oracle_view(orc, ex)
    gt, _ = wl.brute_force(base, q, K, w.metric)
    gix.reset_counters()
    gi, gd, oi = _parity(orc, gix, oix, q, K, efS)
    assert abs(wl.recall_at_k(gi, gt) - wl.recall_at_k(oi, gt)) <= 0.002
    assert wl.recall_at_k(gi, gt) >= 0.8
    assert np.all(np.diff(gd, axis=1) >= 0)


@pytest.mark.parametrize("d", [1152, 1280, 1792, 2304, 2560, 2816])
@pytest.mark.parametrize("fp16", [False, True])
def test_row_lengths_between_instantiated_kernels(orc, d, fp16):
    """Row lengths whose number of per-lane chunks is not itself instantiated (5, 7, 9, 11 chunk rows) or
    whose last chunk row is only partly filled: the kernel for one more chunk row masks its last two."""
    PagIndex = _gpu()
    from paper_2603_06660_amd import FLAG_FP16_VECTORS
    rng = np.random.default_rng(d + int(fp16))
    n = 400
    base = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((40, d)).astype(np.float32)
    gix = PagIndex.build(torch.from_numpy(base).cuda(), metric="l2", max_degree=16, num_subspaces=16,
                         ef_construction=60, seed=5, flags=FLAG_FP16_VECTORS if fp16 else 0)
    ex = gix.export()
    oix = _oracle_view(orc, ex)
    for K, efS in ((10, 40), (100, 150)):
        _parity(orc, gix, oix, q, K, efS)
    # the last node's row is the last of the store: its distances are right as well
    ids, dists = gix.search(torch.from_numpy(base[-1:].copy()).cuda(), 1, 400)
    assert int(ids[0, 0]) == n - 1


def test_seeded_random_shapes(orc):
    """A seeded sweep over shapes nobody would pick by hand (subspace sizes 4..96, degrees 4..64, odd K,
    efS from 1 to 2000, both metrics, both stores, working-set overrides): build, export, oracle parity."""
    PagIndex = _gpu()
    from paper_2603_06660_amd import FLAG_FP16_VECTORS
    rng = np.random.default_rng(2603)
    done = 0
    while done < 14:
        P = int(rng.choice([1, 2, 4, 8, 12, 16, 32, 48, 64]))
        d = P * int(rng.choice([4, 8, 12, 20, 24, 40, 48, 96]))
        if d > 3072 or d % 8:
            continue
        deg = int(rng.choice([4, 8, 16, 31, 32, 48, 64]))
        n = min(int(rng.choice([50, 300, 1500])), max(50, 2_000_000 // d))
        K = min(n, int(rng.choice([1, 5, 10, 37, 100, 200, 600])))
        efS = int(rng.choice([1, 10, 50, 200, 700, 2000]))
        metric = str(rng.choice(["l2", "cos"]))
        fp16 = bool(rng.integers(0, 2))
        sb = int(rng.choice([0, 0, 0, max(K, 64), max(K, 300)]))
        base = rng.standard_normal((n, d)).astype(np.float32)
        q = rng.standard_normal((24, d)).astype(np.float32)
        what = "n %d d %d P %d deg %d K %d efS %d %s fp16 %d b %d" % (n, d, P, deg, K, efS, metric, fp16, sb)
        gix = PagIndex.build(torch.from_numpy(base).cuda(), metric=metric, max_degree=deg, num_subspaces=P,
                             ef_construction=60, seed=done + 1, flags=FLAG_FP16_VECTORS if fp16 else 0)
        ex = gix.export()
        oix = _oracle_view(orc, ex)
        gix.set_search_options(sb, 0)
        gi, gd = gix.search(torch.from_numpy(q).cuda(), K, efS)
        oi, od, _ = oix.search(q, K, efS, b=sb)
        gi, gd = gi.cpu().numpy(), gd.cpu().numpy()
        assert (gi == oi).mean() >= 0.999, what
        m = (gi == oi) & np.isfinite(od)
        assert np.all(np.abs(gd[m] - od[m]) <= 1e-5 * np.abs(od[m]) + 1e-12), what
        k = min(n, 64)
        codes, a, c, e2 = oix.recompute_edge_info(0, k)
        assert np.array_equal(codes, ex["codes"][:k]), what
        assert np.allclose(a, ex["a"][:k], rtol=3e-7, atol=0), what
        gix.close()
        done += 1


def test_online_insertion_rounds(orc):
    """Workload 5's structure at reduced size: insertion batches interleaved with query batches."""
    PagIndex = _gpu()
    w = wl.workload(5, n=4000, nq=100)
    w = dataclasses.replace(w, d=1024, P=32)
    base, q = wl.make(w, "base"), wl.make(w, "query")
    gix = PagIndex.build(torch.from_numpy(base).cuda(), metric="ip", max_degree=w.deg, num_subspaces=w.P,
                         ef_construction=100, seed=9, capacity=4000 + 3 * 500)
    allv = base
    for k in range(3):
        x = wl.make(w, "insert%d" % k, n=500)
        gix.insert(torch.from_numpy(x).cuda())
        allv = np.concatenate([allv, x])
        gt, _ = wl.brute_force(allv, q, w.K, w.metric)
        ids, _ = gix.search(torch.from_numpy(q).cuda(), w.K, 128)
        assert wl.recall_at_k(ids.cpu().numpy(), gt) >= 0.9
    ex = gix.export()
    assert ex["vectors"].shape[0] == 5500
    _parity(orc, gix, _oracle_view(orc, ex), q, w.K, 128)


def test_full_size_benchmark_workload(orc):
    """n = 1,000,000 x 768, 10,000 queries in one call (the launch configuration the benchmark times);
    the oracle searches the exported index for a sample of the queries."""
    PagIndex = _gpu()
    w = wl.workload(2)
    base, q = wl.make(w, "base"), wl.make(w, "query")
    base_d = torch.from_numpy(base).cuda()
    gix = PagIndex.build(base_d, metric="ip", max_degree=w.deg, num_subspaces=w.P, ef_construction=200, seed=2603)
    q_d = torch.from_numpy(q).cuda()
    gt, _ = wl.brute_force_torch(base_d, q_d, w.K, w.metric)
    del base_d
    ex = gix.export()
    oix = _oracle_view(orc, ex)
    # exported store = Q x for sampled rows; inference information of sampled nodes
    rows = np.arange(0, w.n, 50021)
    ref = np.stack([orc.rotate(ex["rotation"], base[i]) for i in rows])
    assert (ref == ex["vectors"][rows]).mean() >= 0.9999
    _check_edge_info(orc, oix, ex, (0, 500_000, w.n - 64))
    sample = np.arange(0, w.nq, 40)                      # 250 queries
    for efS in (64, 512, 1408):                          # 1408: the benchmark's operating point (bitmap + Bloom seen set)
        gi, gd, oi = _parity(orc, gix, oix, q, w.K, efS, sample=sample)
        assert abs(wl.recall_at_k(gi[sample], gt[sample]) - wl.recall_at_k(oi, gt[sample])) <= 0.002
        # property that holds for every query at any size: ascending keys, valid distinct ids
        assert np.all(np.diff(gd, axis=1) >= 0) and gi.min() >= 0 and gi.max() < w.n
        srt = np.sort(gi, axis=1)
        assert not np.any(srt[:, 1:] == srt[:, :-1])
    # sampled outputs checked one by one: the reported key is the true 1 - <q, x>
    ip = np.einsum("qkd,qd->qk", base[gi[sample]].astype(np.float64), q[sample].astype(np.float64))
    assert np.allclose(gd[sample], 1.0 - ip, atol=5e-6)
    # the search of an insertion at this size (efC = 200: two rounds of b = 100 over a million nodes): R_L and the
    # PES buffer H(v) of 40 vectors that are not in the index, against the oracle on the exported arrays
    fresh = q[1::250][:40].copy()
    ci, ck, cn, hi, hk, hn = gix.insertion_candidates(torch.from_numpy(fresh).cuda(), 200)
    fr, _ = oix.prepare(fresh)
    for i in range(len(fresh)):
        oi_, ok_, ohi, ohk, _ = oix.index_search(fr[i], 200)
        assert cn[i] == len(oi_) and ci[i, :cn[i]].tolist() == oi_.tolist(), i
        assert np.all(np.abs(ck[i, :cn[i]] - ok_) <= 1e-5 * ok_)
        assert hn[i] == len(ohi) and hi[i, :hn[i]].tolist() == ohi.tolist(), i


@pytest.mark.parametrize("cfg,efS", [(3, (128, 1024)), (4, (64, 640)), (5, (64, 1536))])
def test_full_size_other_workloads(orc, cfg, efS):
    """The other workloads at their full n, d, degree, subspaces, K and query-batch size (a light efC keeps
    the build short): the oracle searches the exported index for a sample of the queries, at a short and
    at a long search length."""
    PagIndex = _gpu()
    w = wl.workload(cfg)
    base, q = wl.make(w, "base"), wl.make(w, "query")
    metric = {0: "l2", 1: "ip", 2: "cos"}[w.metric]
    base_d = torch.from_numpy(base).cuda()
    gix = PagIndex.build(base_d, metric=metric, max_degree=w.deg, num_subspaces=w.P, ef_construction=100, seed=cfg)
    del base_d
    ex = gix.export()
    oix = _oracle_view(orc, ex)
    rows = np.arange(0, w.n, 250007)
    src = base[rows].astype(np.float64)
    if metric == "cos":
        src = src / np.linalg.norm(src, axis=1, keepdims=True)
    ref = src @ ex["rotation"].astype(np.float64).T
    assert np.allclose(ex["vectors"][rows], ref, rtol=0, atol=2e-6)
    _check_edge_info(orc, oix, ex, (0, w.n // 2, w.n - 64))
    sample = np.arange(0, w.nq, w.nq // 100)             # 100 queries
    for e in efS:
        gi, gd, oi = _parity(orc, gix, oix, q, w.K, e, sample=sample)
        assert np.all(np.diff(gd, axis=1) >= 0) and gi.min() >= 0 and gi.max() < w.n
        srt = np.sort(gi, axis=1)
        assert not np.any(srt[:, 1:] == srt[:, :-1])
    gix.close()
