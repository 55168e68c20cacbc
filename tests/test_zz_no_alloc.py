"""pag_search_static, the search for callers that cannot allocate device memory, against pag_search."""
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


def test_static_search_matches_pag_search(orc):
    """Two calls in a row on one index, the second with a smaller batch (the scratch array then still holds
    the first call's tables and bitmaps under another layout), short and long searches, L2 and cosine; then
    the limits.  ids and distances must equal pag_search's bit for bit, and the oracle's to the usual bar."""
    PagIndex = _gpu()
    from paper_2603_06660_amd import PagError
    w = wl.workload(1, n=6000, nq=700)
    base, q = wl.make(w, "base"), wl.make(w, "query")
    bd, qd = torch.from_numpy(base).cuda(), torch.from_numpy(q).cuda()
    for metric in ("l2", "cos"):
        gix = PagIndex.build(bd, metric=metric, max_degree=w.deg, num_subspaces=w.P, ef_construction=100, seed=9)
        for nq, K, efS in ((700, 10, 64), (300, 10, 2048), (150, 100, 300), (1, 5, 20)):
            qs = qd[:nq].contiguous()
            ref_i, ref_d = gix.search(qs, K, efS)
            out = (torch.full((nq, K), -7, dtype=torch.int64, device="cuda"),
                   torch.full((nq, K), -1.0, dtype=torch.float32, device="cuda"))
            torch.cuda.synchronize()
            free0 = torch.cuda.mem_get_info()[0]
            gix.search_static(qs, K, efS, out)
            assert torch.cuda.mem_get_info()[0] == free0      # the device's free memory did not move
            assert torch.equal(out[0], ref_i) and torch.equal(out[1], ref_d), (metric, nq, K, efS)
        # the seen set pushed into the bitmaps at once, twice: the second call starts from clean bitmaps
        gix.set_seen_capacity_log2(6)
        for nq in (500, 200):
            ref_i, ref_d = gix.search(qd[:nq].contiguous(), 10, 64)
            out = (torch.empty((nq, 10), dtype=torch.int64, device="cuda"), torch.empty((nq, 10), dtype=torch.float32, device="cuda"))
            gix.search_static(qd[:nq].contiguous(), 10, 64, out)
            assert torch.equal(out[0], ref_i) and torch.equal(out[1], ref_d)
        gix.set_seen_capacity_log2(0)
        if metric == "l2":
            ex = gix.export()
            oix = orc.OracleIndex(ex["vectors"], ex["adj"], ex["a"], ex["c"], ex["e2"], ex["codes"], ex["rotation"],
                                  ex["codebooks"], ex["entry"], metric=ex["metric"])
            out = (torch.empty((200, 10), dtype=torch.int64, device="cuda"), torch.empty((200, 10), dtype=torch.float32, device="cuda"))
            gix.search_static(qd[:200].contiguous(), 10, 64, out)
            oi, od, _ = oix.search(q[:200], 10, 64)
            assert (out[0].cpu().numpy() == oi).mean() >= 0.999
            assert np.allclose(out[1].cpu().numpy(), od, rtol=1e-5)
        # limits are errors, not allocations
        big = torch.zeros((20000, w.d), dtype=torch.float32, device="cuda")
        out = (torch.empty((20000, 10), dtype=torch.int64, device="cuda"), torch.empty((20000, 10), dtype=torch.float32, device="cuda"))
        with pytest.raises(PagError, match="4,194,304 floats"):
            gix.search_static(big, 10, 64, out)
        with pytest.raises(PagError, match="128"):
            gix.search_static(qd[:4].contiguous(), 200, 400, out)
        gix.close()
